"""Thin ctypes binding of libpackkv.so -- argument marshalling only.

Function names follow the C ABI (include/packkv.h).  PyTorch is used for
device memory and streams; every step of the path runs in the HIP kernels.
There is no CPU fallback: if the library is missing the import of the symbols
fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

from . import build as _build

KV_OK, KV_ERR_ARG, KV_ERR_UNSUPPORTED, KV_ERR_CAPACITY, KV_ERR_HIP = 0, -1, -2, -3, -4
HEAD_DIM = 128
BLOCK_TOKENS = 64
CHUNK_MAX_BYTES = 512 + 512 * 8


class kv_config_t(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_kv_heads", C.c_int32), ("n_q_heads", C.c_int32),
                ("head_dim", C.c_int32), ("block_tokens", C.c_int32), ("pack_size", C.c_int32),
                ("repack", C.c_int32), ("tail_capacity", C.c_int32),
                ("k_rel_scale", C.c_float), ("v_rel_scale", C.c_float),
                ("max_tokens", C.c_int64)]


_BUFFER_NAMES = ("k_arena", "v_arena", "k_index", "v_index", "k_token_meta", "v_token_meta",
                 "k_tail", "v_tail", "workspace", "token_order", "k_pages", "v_pages")
PAGE_BYTES = 65536
REPACK_NONE, REPACK_V_MEDIAN = 0, 1


class kv_sizes_t(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in _BUFFER_NAMES]


class kv_buffers_t(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _BUFFER_NAMES]


class kv_stats_t(C.Structure):
    _fields_ = [("tokens", C.c_int64), ("packed_tokens", C.c_int64), ("tail_tokens", C.c_int64),
                ("n_chunks", C.c_int64), ("k_bytes", C.c_int64), ("v_bytes", C.c_int64),
                ("index_bytes", C.c_int64), ("token_meta_bytes", C.c_int64),
                ("overflow", C.c_int32),
                ("k_header_bytes", C.c_int64), ("k_payload_bytes", C.c_int64), ("k_padding_bytes", C.c_int64),
                ("v_header_bytes", C.c_int64), ("v_payload_bytes", C.c_int64), ("v_padding_bytes", C.c_int64)]


EXPORTS = ("kv_query_sizes", "kv_cache_create", "kv_cache_destroy", "kv_compress_append", "kv_compress_append_bf16",
           "kv_k_matvec", "kv_v_matvec", "kv_v_matvec_noalloc", "kv_softmax", "kv_decode_attention", "kv_cache_stats", "kv_cache_restore", "kv_cache_tokens",
           "kv_strerror", "kv_fp16_k_matvec", "kv_fp16_v_matvec", "kv_fp16_v_workspace_bytes",
           "kv_stream_read", "kv_page_pool_state_bytes", "kv_page_pool_create", "kv_page_pool_destroy",
           "kv_page_pool_free_pages", "kv_query_sizes_paged", "kv_cache_create_paged", "kv_cache_release")

_lib = None


def library_path() -> str:
    return _build.LIB


def lib():
    """Load libpackkv.so; build it first only if no built library exists."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build()
        L = C.CDLL(_build.LIB)
        vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
        L.kv_query_sizes.argtypes = [C.POINTER(kv_config_t), C.c_double, C.POINTER(kv_sizes_t)]
        L.kv_cache_create.argtypes = [C.POINTER(kv_config_t), C.POINTER(kv_buffers_t),
                                      C.POINTER(kv_sizes_t), C.POINTER(vp)]
        L.kv_cache_destroy.argtypes = [vp]
        L.kv_page_pool_state_bytes.argtypes = [i64]
        L.kv_page_pool_state_bytes.restype = C.c_size_t
        L.kv_page_pool_create.argtypes = [vp, i64, vp, vp, C.POINTER(vp)]
        L.kv_page_pool_destroy.argtypes = [vp]
        L.kv_page_pool_free_pages.argtypes = [vp, C.POINTER(i64), vp]
        L.kv_query_sizes_paged.argtypes = [C.POINTER(kv_config_t), C.POINTER(kv_sizes_t)]
        L.kv_cache_create_paged.argtypes = [C.POINTER(kv_config_t), vp, C.POINTER(kv_buffers_t),
                                            C.POINTER(kv_sizes_t), C.POINTER(vp)]
        L.kv_cache_release.argtypes = [vp, vp]
        L.kv_compress_append.argtypes = [vp, vp, vp, i32, vp]
        L.kv_compress_append_bf16.argtypes = [vp, vp, vp, i32, vp]
        L.kv_k_matvec.argtypes = [vp, vp, f32, vp, i64, vp]
        L.kv_v_matvec.argtypes = [vp, vp, i64, vp, vp]
        L.kv_v_matvec_noalloc.argtypes = [vp, vp, i64, vp, vp]
        L.kv_decode_attention.argtypes = [vp, vp, f32, vp, vp]
        L.kv_softmax.argtypes = [vp, vp, i64, vp]
        L.kv_cache_stats.argtypes = [vp, C.POINTER(kv_stats_t), vp]
        L.kv_cache_restore.argtypes = [vp, i64]
        L.kv_cache_tokens.argtypes = [vp]
        L.kv_cache_tokens.restype = i64
        L.kv_strerror.argtypes = [C.c_int]
        L.kv_strerror.restype = C.c_char_p
        L.kv_fp16_k_matvec.argtypes = [vp, vp, f32, vp, i64, i32, i32, i32, i64, vp]
        L.kv_fp16_v_matvec.argtypes = [vp, vp, i64, vp, i32, i32, i32, i64, vp, vp]
        L.kv_fp16_v_workspace_bytes.argtypes = [i32, i32]
        L.kv_fp16_v_workspace_bytes.restype = C.c_size_t
        L.kv_stream_read.argtypes = [vp, C.c_size_t, vp, vp]
        for name in EXPORTS:
            if name not in ("kv_cache_tokens", "kv_strerror", "kv_fp16_v_workspace_bytes",
                            "kv_page_pool_state_bytes"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


class PackKVError(RuntimeError):
    """A library call returned an error code (kept in .code)."""

    def __init__(self, message, code=None):
        super().__init__(message)
        self.code = code


def _check(rc: int, what: str) -> None:
    if rc != KV_OK:
        raise PackKVError("%s: %s (%d)" % (what, lib().kv_strerror(rc).decode(), rc), rc)


def _stream_ptr(stream=None):
    """stream: None (torch's current stream), a torch stream, or a raw hipStream_t as int
    (looking up the current stream costs microseconds; hot loops pass the integer)."""
    if isinstance(stream, int):
        return C.c_void_p(stream)
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def make_config(batch, n_kv_heads, n_q_heads, max_tokens, k_rel_scale=0.1, v_rel_scale=0.2,
                repack=REPACK_NONE, pack_size=16):
    return kv_config_t(batch, n_kv_heads, n_q_heads, HEAD_DIM, BLOCK_TOKENS, pack_size, repack, BLOCK_TOKENS,
                       k_rel_scale, v_rel_scale, max_tokens)


def kv_query_sizes(cfg: kv_config_t, bits_per_element_budget: float = 0.0) -> kv_sizes_t:
    out = kv_sizes_t()
    _check(lib().kv_query_sizes(C.byref(cfg), bits_per_element_budget, C.byref(out)), "kv_query_sizes")
    return out


def kv_query_sizes_paged(cfg: kv_config_t) -> kv_sizes_t:
    out = kv_sizes_t()
    _check(lib().kv_query_sizes_paged(C.byref(cfg), C.byref(out)), "kv_query_sizes_paged")
    return out


class PagePool:
    """Owns the pages and the bookkeeping words (torch tensors) and the kv_page_pool_t handle."""

    def __init__(self, n_pages, device="cuda:0"):
        self.device = torch.device(device)
        self.n_pages = n_pages
        state_bytes = lib().kv_page_pool_state_bytes(n_pages)
        if state_bytes == 0:
            raise PackKVError("kv_page_pool_state_bytes: invalid argument", KV_ERR_ARG)
        with torch.cuda.device(self.device):
            self.pages = torch.empty(n_pages * PAGE_BYTES, dtype=torch.uint8, device=self.device)
            self.state = torch.empty(state_bytes, dtype=torch.uint8, device=self.device)
            torch.cuda.synchronize()
            handle = C.c_void_p()
            _check(lib().kv_page_pool_create(self.pages.data_ptr(), n_pages, self.state.data_ptr(),
                                             _stream_ptr(None), C.byref(handle)), "kv_page_pool_create")
        self.handle = handle

    def kv_page_pool_free_pages(self, stream=None) -> int:
        n = C.c_int64()
        _check(lib().kv_page_pool_free_pages(self.handle, C.byref(n), _stream_ptr(stream)),
               "kv_page_pool_free_pages")
        return int(n.value)

    def close(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.kv_page_pool_destroy(self.handle)
        self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class PackedKVCache:
    """Owns the device buffers (torch tensors) and the kv_cache_t handle.  With `pool` (a PagePool)
    the cache is paged: it has no arenas of its own and keeps its chunks in pages of the pool."""

    def __init__(self, batch, n_kv_heads, n_q_heads, max_tokens, k_rel_scale=0.1, v_rel_scale=0.2,
                 bits_per_element_budget=0.0, device="cuda:0", repack=REPACK_NONE, pack_size=16, pool=None):
        self.cfg = make_config(batch, n_kv_heads, n_q_heads, max_tokens, k_rel_scale, v_rel_scale, repack,
                               pack_size)
        self.device = torch.device(device)
        self.pool = pool
        self.sizes = (kv_query_sizes_paged(self.cfg) if pool is not None
                      else kv_query_sizes(self.cfg, bits_per_element_budget))
        self.tensors = {}
        bufs = kv_buffers_t()
        with torch.cuda.device(self.device):
            for name in _BUFFER_NAMES:
                t = torch.empty(getattr(self.sizes, name), dtype=torch.uint8, device=self.device)
                assert t.numel() == 0 or t.data_ptr() % 256 == 0
                self.tensors[name] = t
                setattr(bufs, name, t.data_ptr() if t.numel() else None)
            torch.cuda.synchronize()
            handle = C.c_void_p()
            if pool is not None:
                _check(lib().kv_cache_create_paged(C.byref(self.cfg), pool.handle, C.byref(bufs),
                                                   C.byref(self.sizes), C.byref(handle)), "kv_cache_create_paged")
            else:
                _check(lib().kv_cache_create(C.byref(self.cfg), C.byref(bufs), C.byref(self.sizes),
                                             C.byref(handle)), "kv_cache_create")
        self.handle = handle
        self.batch, self.n_kv_heads, self.n_q_heads = batch, n_kv_heads, n_q_heads

    def close(self):
        if getattr(self, "handle", None) and _lib is not None:
            # a paged cache returns its pages to the pool here: the pool must still exist
            # (if it was closed first, the handle is dropped without the call)
            if getattr(self, "pool", None) is None or self.pool.handle:
                _lib.kv_cache_destroy(self.handle)
        self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def tokens(self) -> int:
        return int(lib().kv_cache_tokens(self.handle))

    def kv_compress_append(self, k_new: torch.Tensor, v_new: torch.Tensor, stream=None):
        """k_new, v_new: fp16 (or both bf16: kv_compress_append_bf16) [B, n, H_kv, 128] contiguous device tensors."""
        assert k_new.dtype == v_new.dtype and k_new.dtype in (torch.float16, torch.bfloat16)
        assert k_new.is_contiguous() and v_new.is_contiguous() and k_new.shape == v_new.shape
        assert k_new.shape[0] == self.batch and tuple(k_new.shape[2:]) == (self.n_kv_heads, HEAD_DIM)
        if k_new.dtype == torch.bfloat16:
            _check(lib().kv_compress_append_bf16(self.handle, k_new.data_ptr(), v_new.data_ptr(),
                                                 k_new.shape[1], _stream_ptr(stream)), "kv_compress_append_bf16")
            return
        _check(lib().kv_compress_append(self.handle, k_new.data_ptr(), v_new.data_ptr(),
                                        k_new.shape[1], _stream_ptr(stream)), "kv_compress_append")

    def kv_k_matvec(self, q: torch.Tensor, sm_scale: float, scores: torch.Tensor = None, stream=None):
        """q: fp16 [B, Hq, 128] -> scores fp32 [B, Hq, ld] (ld >= tokens)."""
        assert q.dtype == torch.float16 and q.is_contiguous()
        assert tuple(q.shape) == (self.batch, self.n_q_heads, HEAD_DIM)
        if scores is None:
            scores = torch.empty(self.batch, self.n_q_heads, self.tokens, dtype=torch.float32,
                                 device=self.device)
        assert scores.dtype == torch.float32 and scores.is_contiguous()
        _check(lib().kv_k_matvec(self.handle, q.data_ptr(), sm_scale, scores.data_ptr(),
                                 scores.shape[2], _stream_ptr(stream)), "kv_k_matvec")
        return scores

    def kv_v_matvec(self, p: torch.Tensor, out: torch.Tensor = None, stream=None):
        """p: fp32 [B, Hq, ld] -> out fp32 [B, Hq, 128]."""
        assert p.dtype == torch.float32 and p.is_contiguous()
        assert tuple(p.shape[:2]) == (self.batch, self.n_q_heads)
        if out is None:
            out = torch.empty(self.batch, self.n_q_heads, HEAD_DIM, dtype=torch.float32,
                              device=self.device)
        _check(lib().kv_v_matvec(self.handle, p.data_ptr(), p.shape[2], out.data_ptr(),
                                 _stream_ptr(stream)), "kv_v_matvec")
        return out

    def kv_v_matvec_noalloc(self, p: torch.Tensor, out: torch.Tensor, stream=None):
        """As kv_v_matvec, through the entry point that allocates nothing; `out` is the caller's."""
        assert p.dtype == torch.float32 and p.is_contiguous()
        assert tuple(p.shape[:2]) == (self.batch, self.n_q_heads)
        assert out.dtype == torch.float32 and out.is_contiguous()
        assert tuple(out.shape) == (self.batch, self.n_q_heads, HEAD_DIM)
        _check(lib().kv_v_matvec_noalloc(self.handle, p.data_ptr(), p.shape[2], out.data_ptr(),
                                         _stream_ptr(stream)), "kv_v_matvec_noalloc")
        return out

    def kv_softmax(self, scores: torch.Tensor, stream=None):
        """In-place softmax over the cached tokens of scores fp32 [B, Hq, ld]; returns scores."""
        assert scores.dtype == torch.float32 and scores.is_contiguous()
        assert tuple(scores.shape[:2]) == (self.batch, self.n_q_heads)
        _check(lib().kv_softmax(self.handle, scores.data_ptr(), scores.shape[2], _stream_ptr(stream)),
               "kv_softmax")
        return scores

    def kv_decode_attention(self, q: torch.Tensor, sm_scale: float, out: torch.Tensor = None, stream=None):
        """q: fp16 [B, Hq, 128] -> out fp32 [B, Hq, 128] = softmax(sm_scale * q K^T) V over the whole cache."""
        assert q.dtype == torch.float16 and q.is_contiguous()
        assert tuple(q.shape) == (self.batch, self.n_q_heads, HEAD_DIM)
        if out is None:
            out = torch.empty(self.batch, self.n_q_heads, HEAD_DIM, dtype=torch.float32,
                              device=self.device)
        _check(lib().kv_decode_attention(self.handle, q.data_ptr(), sm_scale, out.data_ptr(),
                                         _stream_ptr(stream)), "kv_decode_attention")
        return out

    def kv_cache_stats(self, stream=None) -> kv_stats_t:
        st = kv_stats_t()
        _check(lib().kv_cache_stats(self.handle, C.byref(st), _stream_ptr(stream)), "kv_cache_stats")
        return st

    def kv_cache_release(self, stream=None):
        _check(lib().kv_cache_release(self.handle, _stream_ptr(stream)), "kv_cache_release")

    def kv_cache_restore(self, tokens: int):
        _check(lib().kv_cache_restore(self.handle, tokens), "kv_cache_restore")

    # typed views of the raw buffers, for tests and tools
    def view(self, name, dtype):
        return self.tensors[name].view(dtype)


def kv_fp16_k_matvec(k_cache, q, sm_scale, n_kv_heads, scores=None, stream=None):
    """k_cache: fp16 [B, H_kv, L, 128]; q: fp16 [B, Hq, 128] -> fp32 [B, Hq, L]."""
    B, H, L, Dd = k_cache.shape
    Hq = q.shape[1]
    if scores is None:
        scores = torch.empty(B, Hq, L, dtype=torch.float32, device=k_cache.device)
    _check(lib().kv_fp16_k_matvec(k_cache.data_ptr(), q.data_ptr(), sm_scale, scores.data_ptr(),
                                  scores.shape[2], B, H, Hq, L, _stream_ptr(stream)), "kv_fp16_k_matvec")
    return scores


def kv_fp16_v_matvec(v_cache, p, out=None, workspace=None, stream=None):
    """v_cache: fp16 [B, H_kv, L, 128]; p: fp32 [B, Hq, ld] -> fp32 [B, Hq, 128]."""
    B, H, L, Dd = v_cache.shape
    Hq = p.shape[1]
    if out is None:
        out = torch.empty(B, Hq, Dd, dtype=torch.float32, device=v_cache.device)
    if workspace is None:
        workspace = torch.empty(lib().kv_fp16_v_workspace_bytes(B, Hq), dtype=torch.uint8,
                                device=v_cache.device)
    _check(lib().kv_fp16_v_matvec(v_cache.data_ptr(), p.data_ptr(), p.shape[2], out.data_ptr(), B, H,
                                  Hq, L, workspace.data_ptr(), _stream_ptr(stream)), "kv_fp16_v_matvec")
    return out


def kv_stream_read(buf: torch.Tensor, checksum: torch.Tensor, stream=None):
    nbytes = buf.numel() * buf.element_size()
    _check(lib().kv_stream_read(buf.data_ptr(), nbytes - nbytes % 16, checksum.data_ptr(),
                                _stream_ptr(stream)), "kv_stream_read")
