"""ctypes front end of the PackKV CPU oracle (TEST INFRASTRUCTURE ONLY).

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It never imports the HIP package and
the HIP package never imports it.  All arrays are numpy, all memory is host.

The arithmetic lives in ``packkv_oracle.c`` (plain scalar C, fp64
accumulation); this file only builds it with gcc and marshals arguments.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "packkv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

D = 128          # head_dim
N = 64           # tokens per block
K = 16           # pack size
PACKS = (N // K) * D
HEADER = PACKS
CHUNK_MAX = HEADER + PACKS * 8


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no GPU, no HIP involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_h2f.restype = C.c_float
        _lib.orc_h2f.argtypes = [C.c_uint16]
        _lib.orc_f2h.restype = C.c_uint16
        _lib.orc_f2h.argtypes = [C.c_float]
        _lib.orc_qmax.restype = C.c_int
        _lib.orc_qmax.argtypes = [C.c_float]
        _lib.orc_width.restype = C.c_int
        _lib.orc_width.argtypes = [C.c_int]
        _lib.orc_xhat.restype = C.c_double
        _lib.orc_xhat.argtypes = [C.c_uint8, C.c_uint16, C.c_uint16]
        _lib.orc_pack_chunk.restype = C.c_int
        _lib.orc_pack_chunk_k.restype = C.c_int
        _lib.orc_pack_chunk_planes.restype = C.c_int
        _lib.orc_pack_chunk_wide.restype = C.c_int
        _lib.orc_compress.restype = C.c_int64
        _lib.orc_compress_k.restype = C.c_int64
        _lib.orc_threads.restype = C.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _u16(x):
    """View an fp16 / uint16 array as contiguous uint16."""
    x = np.ascontiguousarray(x)
    if x.dtype == np.float16:
        x = x.view(np.uint16)
    assert x.dtype == np.uint16
    return x


def h2f(h: int) -> float:
    return float(lib().orc_h2f(int(h)))


def f2h(f: float) -> int:
    return int(lib().orc_f2h(float(f)))


def qmax(rel: float) -> int:
    return int(lib().orc_qmax(np.float32(rel)))


def width(r: int) -> int:
    return int(lib().orc_width(int(r)))


def threads() -> int:
    return int(lib().orc_threads())


def set_threads(n: int) -> None:
    lib().orc_set_threads(C.c_int(int(n)))


def token_params(x, rel):
    """x: fp16 [B, T, H, D] -> (scale16, min16) uint16 [B, T]."""
    x = _u16(x)
    B, T, H, Dd = x.shape
    scale = np.empty((B, T), np.uint16)
    mn = np.empty((B, T), np.uint16)
    lib().orc_token_params(_p(x), B, T, H, Dd, C.c_int64(T * H * Dd), C.c_int64(H * Dd),
                           C.c_float(rel), _p(scale), _p(mn))
    return scale, mn


def quantize(x, rel, scale16, min16):
    """x: fp16 [B, T, H, D] -> codes uint8 [B, T, H, D]."""
    x = _u16(x)
    B, T, H, Dd = x.shape
    q = np.empty((B, T, H, Dd), np.uint8)
    lib().orc_quantize(_p(x), B, T, H, Dd, C.c_int64(T * H * Dd), C.c_int64(H * Dd),
                       C.c_float(rel), _p(np.ascontiguousarray(scale16)),
                       _p(np.ascontiguousarray(min16)), _p(q))
    return q


def dequant(q, scale16, min16):
    """codes uint8 [B, T, H, D] -> x_hat float64 [B, T, H, D]."""
    q = np.ascontiguousarray(q)
    B, T, H, Dd = q.shape
    out = np.empty((B, T, H, Dd), np.float64)
    lib().orc_dequant(_p(q), B, T, H, Dd, _p(np.ascontiguousarray(scale16)),
                      _p(np.ascontiguousarray(min16)), _p(out))
    return out


def pack_chunk_wide(q_chunk):
    """q_chunk: uint8 [64, 128], codes up to 255 -> (bytes, widths [1024], mins [1024]): the wide
    chunk layout (packs of 8 tokens, two metadata bytes per pack)."""
    q_chunk = np.ascontiguousarray(q_chunk, dtype=np.uint8)
    assert q_chunk.shape == (N, D)
    packs = N // 8 * D
    buf = np.zeros(2 * packs + N * D + 16, np.uint8)
    w = np.empty(packs, np.uint8)
    m = np.empty(packs, np.uint8)
    size = lib().orc_pack_chunk_wide(_p(q_chunk), C.c_int64(D), _p(buf), _p(w), _p(m))
    return buf[:size].copy(), w, m


ORDERS = {"group": 0, "channel": 1}


def pack_chunk(q_chunk, pack_size=K, order="group", contiguous=False):
    """q_chunk: uint8 [64, 128] -> (bytes uint8 [size], widths [packs], mins [packs]), packs =
    (64 / pack_size) * 128, widths and mins indexed [token_group*128 + channel].  Packs of 16 use
    the plane layout with the given pack list order ("group" or "channel"); contiguous=True
    packs them in the contiguous-pack layout instead (the layout of the packs of 8)."""
    q_chunk = np.ascontiguousarray(q_chunk, dtype=np.uint8)
    assert q_chunk.shape == (N, D) and pack_size in (8, 16)
    packs = N // pack_size * D
    buf = np.zeros(packs + N * D // 2 + 16, np.uint8)
    w = np.empty(packs, np.uint8)
    m = np.empty(packs, np.uint8)
    if pack_size == 16 and not contiguous:
        size = lib().orc_pack_chunk_planes(_p(q_chunk), C.c_int64(D), _p(buf), _p(w), _p(m), ORDERS[order])
    else:
        assert order == "group"
        size = lib().orc_pack_chunk_k(_p(q_chunk), C.c_int64(D), _p(buf), _p(w), _p(m), pack_size)
    return buf[:size].copy(), w, m


class Compressed:
    """Result of :func:`compress` -- everything the packed cache consists of."""

    def __init__(self, arena, offsets16, meta, codes, widths, mins):
        self.arena = arena          # uint8 [bytes]
        self.offsets16 = offsets16  # uint32 [nchunks + 1], 16-byte units
        self.meta = meta            # uint32 [B, T]: scale16 | min16 << 16
        self.codes = codes          # uint8 [B, T, H, D]
        self.widths = widths        # uint8 [nchunks, packs]
        self.mins = mins            # uint8 [nchunks, packs]

    @property
    def scale16(self):
        return (self.meta & 0xFFFF).astype(np.uint16)

    @property
    def min16(self):
        return (self.meta >> 16).astype(np.uint16)


def compress(x, rel, pack_size=K, order="group") -> Compressed:
    """x: fp16 [B, T, H, D] with T a multiple of 64 -> Compressed (packs of pack_size tokens).
    Scales finer than 1/15 (codes above 15) give wide chunks and need pack_size 8.  order: pack
    list of the chunks with packs of 16 tokens ("group" or "channel"; the cache keeps V
    group-major and K channel-major)."""
    x = _u16(x)
    B, T, H, Dd = x.shape
    assert Dd == D and T % N == 0 and pack_size in (8, 16)
    packs = N // pack_size * D
    nchunks = (T // N) * B * H
    cap = nchunks * (2 * packs + N * D)
    arena = np.zeros(cap, np.uint8)
    offsets = np.zeros(nchunks + 1, np.uint32)
    meta = np.empty((B, T), np.uint32)
    codes = np.empty((B, T, H, Dd), np.uint8)
    widths = np.empty((nchunks, packs), np.uint8)
    mins = np.empty((nchunks, packs), np.uint8)
    size = lib().orc_compress_k(_p(x), B, T, H, Dd, C.c_int64(T * H * Dd), C.c_int64(H * Dd),
                                C.c_float(rel), _p(arena), C.c_int64(cap), _p(offsets), _p(meta),
                                _p(codes), _p(widths), _p(mins), pack_size,
                                ORDERS[order] if pack_size == 16 else 0)
    assert size >= 0, size
    return Compressed(arena[:size].copy(), offsets, meta, codes, widths, mins)


def compress_k(x, rel, pack_size=K) -> Compressed:
    """The K cache: chunks with packs of 16 list their packs channel-major."""
    return compress(x, rel, pack_size, order="channel")


def compress_v(x, rel, pack_size=K) -> Compressed:
    """The V cache: chunks with packs of 16 list their packs group-major."""
    return compress(x, rel, pack_size, order="group")


def v_median_order(v_codes):
    """V-median repacking order: v_codes uint8 [B, T, H, D] (quantized V) -> uint8 [B, T];
    entry [b, blk*64 + s] is the in-block index of the token stored at slot s."""
    v_codes = np.ascontiguousarray(v_codes, dtype=np.uint8)
    B, T, H, Dd = v_codes.shape
    assert T % N == 0
    order = np.empty((B, T), np.uint8)
    lib().orc_v_median_order(_p(v_codes), B, T, H, Dd, _p(order))
    return order


def greedy_order(k_codes, v_codes):
    """Greedy repacking order over the joint (K | V) token vectors: uint8 [B, T], layout as
    v_median_order.  O(N^2 D) per block; oracle only."""
    k_codes = np.ascontiguousarray(k_codes, dtype=np.uint8)
    v_codes = np.ascontiguousarray(v_codes, dtype=np.uint8)
    B, T, H, Dd = v_codes.shape
    assert k_codes.shape == v_codes.shape and T % N == 0
    order = np.empty((B, T), np.uint8)
    lib().orc_greedy_order(_p(k_codes), _p(v_codes), B, T, H, Dd, _p(order))
    return order


def apply_order(x, order):
    """Reorder the tokens of x [B, T, ...] inside their 64-token blocks: out[b, blk*64+s] =
    x[b, blk*64 + order[b, blk*64+s]].  Plain indexing, no arithmetic of the method."""
    B, T = order.shape
    src = (np.arange(T) // N * N)[None, :] + order.astype(np.int64)
    return np.ascontiguousarray(np.take_along_axis(
        x[:, :T], src.reshape(B, T, *([1] * (x.ndim - 2))), axis=1))


def k_scores(codes, x, meta, n_packed, qvec, sm_scale):
    """scores float64 [B, Hq, T]; codes/x [B, T, H, D], qvec fp16 [B, Hq, D]."""
    x = _u16(x)
    B, T, H, Dd = x.shape
    qvec = _u16(qvec)
    Hq = qvec.shape[1]
    assert Hq % H == 0
    if codes is None:
        codes = np.zeros((B, T, H, Dd), np.uint8)
        meta = np.zeros((B, T), np.uint32)
        assert n_packed == 0
    out = np.empty((B, Hq, T), np.float64)
    lib().orc_k_scores(_p(np.ascontiguousarray(codes)), _p(x), _p(np.ascontiguousarray(meta)),
                       B, T, int(n_packed), H, Hq, Dd, _p(qvec), C.c_double(sm_scale), _p(out))
    return out


def v_out(codes, x, meta, n_packed, p):
    """out float64 [B, Hq, D]; p float32 [B, Hq, T]."""
    x = _u16(x)
    B, T, H, Dd = x.shape
    p = np.ascontiguousarray(p, dtype=np.float32)
    Hq = p.shape[1]
    assert Hq % H == 0 and p.shape[2] >= T
    if codes is None:
        codes = np.zeros((B, T, H, Dd), np.uint8)
        meta = np.zeros((B, T), np.uint32)
        assert n_packed == 0
    out = np.empty((B, Hq, Dd), np.float64)
    lib().orc_v_out(_p(np.ascontiguousarray(codes)), _p(x), _p(np.ascontiguousarray(meta)),
                    B, T, int(n_packed), H, Hq, Dd, _p(p), C.c_int64(p.shape[2]), _p(out))
    return out


def attention(kcodes, kx, kmeta, vcodes, vx, vmeta, n_packed, q, sm_scale):
    """Decode attention from its definition in fp64: out float64 [B, Hq, D]."""
    kx, vx, q = _u16(kx), _u16(vx), _u16(q)
    B, T, H, Dd = kx.shape
    Hq = q.shape[1]
    assert Hq % H == 0 and vx.shape == kx.shape and T >= 1
    if kcodes is None:
        kcodes = vcodes = np.zeros((B, T, H, Dd), np.uint8)
        kmeta = vmeta = np.zeros((B, T), np.uint32)
        assert n_packed == 0
    out = np.empty((B, Hq, Dd), np.float64)
    lib().orc_attention(_p(np.ascontiguousarray(kcodes)), _p(kx), _p(np.ascontiguousarray(kmeta)),
                        _p(np.ascontiguousarray(vcodes)), _p(vx), _p(np.ascontiguousarray(vmeta)),
                        B, T, int(n_packed), H, Hq, Dd, _p(q), C.c_double(sm_scale), _p(out))
    return out


def softmax(s):
    """fp64 softmax over the last axis."""
    s = np.ascontiguousarray(s, dtype=np.float64)
    T = s.shape[-1]
    rows = s.size // T
    p = np.empty_like(s)
    lib().orc_softmax(_p(s), rows, T, _p(p))
    return p
