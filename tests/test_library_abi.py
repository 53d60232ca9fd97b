"""CPU-only checks of the C-ABI boundary: the library loads, exports every
symbol the header declares, and its host-only entry points behave."""
import ctypes as C
import os
import re

import pytest

from paper_2512_24449_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "packkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kv_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    raw = C.CDLL(binding.lib()._name)
    for n in names:
        assert hasattr(raw, n), n


def test_query_sizes_and_config_checks():
    cfg = binding.make_config(1, 32, 32, 4096)
    worst = binding.kv_query_sizes(cfg)
    n_chunks = 4096 // 64 * 32
    assert worst.k_arena >= n_chunks * binding.CHUNK_MAX_BYTES
    assert worst.k_index >= (n_chunks + 1) * 4 and worst.k_token_meta >= 4096 * 4
    assert worst.k_tail >= 64 * 32 * 128 * 2
    small = binding.kv_query_sizes(cfg, 3.0)
    assert small.k_arena < worst.k_arena and small.k_arena >= n_chunks * 64 * 128 * 3 // 8
    # unsupported / invalid configurations are refused with the documented codes
    L = binding.lib()
    out = binding.kv_sizes_t()
    bad = binding.make_config(1, 32, 32, 4096)
    bad.head_dim = 64
    assert L.kv_query_sizes(C.byref(bad), 0.0, C.byref(out)) == -2
    bad = binding.make_config(1, 32, 32, 4096, k_rel_scale=0.05)   # codes above 15 need packs of 8
    assert L.kv_query_sizes(C.byref(bad), 0.0, C.byref(out)) == -2
    ok = binding.make_config(1, 32, 32, 4096, k_rel_scale=0.05, pack_size=8, repack=binding.REPACK_V_MEDIAN)
    assert L.kv_query_sizes(C.byref(ok), 0.0, C.byref(out)) == 0 and out.token_order >= 4096
    bad = binding.make_config(1, 32, 32, 4096, v_rel_scale=1 / 300, pack_size=8)   # a code is one byte
    assert L.kv_query_sizes(C.byref(bad), 0.0, C.byref(out)) == -2
    wide = binding.kv_query_sizes(binding.make_config(1, 32, 32, 4096, k_rel_scale=0.05, pack_size=8))
    assert wide.k_arena >= n_chunks * 10240 and wide.v_arena >= n_chunks * 5120 and wide.v_arena < wide.k_arena
    bad = binding.make_config(1, 3, 32, 4096)                      # query heads not a multiple of kv heads
    assert L.kv_query_sizes(C.byref(bad), 0.0, C.byref(out)) == -1
    for g in range(1, 9):                                          # every group size up to 8
        assert L.kv_query_sizes(C.byref(binding.make_config(1, 4, 4 * g, 4096)), 0.0, C.byref(out)) == 0
    for g in (9, 11, 12, 16, 24, 64):                              # split into s <= 16 groups of g / s <= 4 heads
        assert L.kv_query_sizes(C.byref(binding.make_config(1, 2, 2 * g, 4096)), 0.0, C.byref(out)) == 0
    for g in (17, 19, 65, 128):                                    # no such split
        assert L.kv_query_sizes(C.byref(binding.make_config(1, 2, 2 * g, 4096)), 0.0, C.byref(out)) == -2
    bad = binding.make_config(0, 1, 1, 64)
    assert L.kv_query_sizes(C.byref(bad), 0.0, C.byref(out)) == -1
    assert L.kv_query_sizes(None, 0.0, C.byref(out)) == -1
    bad = binding.make_config(1, 32, 32, 4096, repack=2)          # unknown repacking mode
    assert L.kv_query_sizes(C.byref(bad), 0.0, C.byref(out)) == -2
    # the token order buffer exists only with repacking
    assert worst.token_order == 0
    rp = binding.kv_query_sizes(binding.make_config(2, 32, 32, 4096, repack=binding.REPACK_V_MEDIAN))
    assert rp.token_order >= 2 * 4096 and rp.k_arena == binding.kv_query_sizes(binding.make_config(2, 32, 32, 4096)).k_arena
    # packs of 8 tokens: twice the header bytes, worst case 1024 + 4096 bytes per chunk
    p8 = binding.kv_query_sizes(binding.make_config(1, 32, 32, 4096, pack_size=8))
    assert p8.k_arena >= n_chunks * 5120 and p8.k_arena > worst.k_arena and p8.k_index == worst.k_index
    bad = binding.make_config(1, 32, 32, 4096, pack_size=4)        # only 16 and 8
    assert L.kv_query_sizes(C.byref(bad), 0.0, C.byref(out)) == -2
    assert L.kv_decode_attention(None, None, 1.0, None, None) == -1
    assert L.kv_strerror(-3) == b"cache capacity exceeded"
    assert L.kv_cache_destroy(None) == -1
    assert L.kv_k_matvec(None, None, 1.0, None, 0, None) == -1


def test_paged_sizes_and_pool_bookkeeping_bytes():
    L = binding.lib()
    cfg = binding.make_config(2, 32, 32, 4096)
    flat, paged = binding.kv_query_sizes(cfg), binding.kv_query_sizes_paged(cfg)
    max_chunks = 4096 // 64 * 2 * 32
    assert paged.k_arena == 0 and paged.v_arena == 0 and flat.k_pages == 0 and flat.v_pages == 0
    assert paged.k_index >= max_chunks * 8 and paged.v_index == paged.k_index
    # 14 largest chunks of 4608 bytes fit a page of 65536
    assert paged.k_pages >= 4 * (2 + -(-max_chunks // 14)) and paged.k_pages % 256 == 0
    for name in ("k_token_meta", "v_token_meta", "k_tail", "v_tail", "workspace", "token_order"):
        assert getattr(paged, name) == getattr(flat, name)
    wide = binding.kv_query_sizes_paged(binding.make_config(2, 32, 32, 4096, k_rel_scale=0.05, pack_size=8))
    assert wide.k_pages >= 4 * (2 + -(-max_chunks // 6)) and wide.v_pages >= 4 * (2 + -(-max_chunks // 12))
    out = binding.kv_sizes_t()
    bad = binding.make_config(2, 32, 32, 4096, pack_size=4)
    assert L.kv_query_sizes_paged(C.byref(bad), C.byref(out)) == -2
    assert L.kv_page_pool_state_bytes(1000) >= 4 * 1001 and L.kv_page_pool_state_bytes(1000) % 256 == 0
    assert L.kv_page_pool_state_bytes(0) == 0
    # argument checks that need no device
    handle = C.c_void_p()
    assert L.kv_page_pool_create(None, 4, None, None, C.byref(handle)) == -1
    assert L.kv_page_pool_destroy(None) == -1 and L.kv_cache_release(None, None) == -1
    assert L.kv_page_pool_free_pages(None, None, None) == -1


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    """No CPU fallback: a missing library with no compiler is an error."""
    from paper_2512_24449_amd import build
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(build, "LIB", str(tmp_path / "missing.so"))
    monkeypatch.setenv("HIPCC", str(tmp_path / "no-such-hipcc"))
    with pytest.raises(Exception):
        binding.lib()
