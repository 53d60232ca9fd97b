"""GPU parity tests: the HIP path, called through the C ABI, against the CPU
oracle on the same seeded inputs."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
from paper_2512_24449_amd import binding, synth
from tests import gpu_cases
from tests.gpu_cases import assert_close_vectors

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,H,Hq,L,seed", [
    (1, 1, 1, 64, 10),        # one chunk
    (1, 1, 1, 1024, 0),       # benchmark configuration 0
    (2, 3, 6, 192, 11),       # several heads and batches, G = 2
    (1, 8, 32, 512, 12),      # GQA with G = 4
    (1, 2, 16, 256, 13),      # G = 8
    (3, 5, 5, 320 + 37, 14),  # ragged: 37 tokens stay in the raw tail
    (1, 4, 4, 17, 15),        # tail only, nothing packed
    (2, 2, 8, 320 + 21, 16),  # G = 4, ragged, odd score row stride (unaligned 16-byte stores)
    (1, 3, 6, 7 * 64 + 1, 17),  # G = 2, odd number of blocks per wave
])
def test_append_then_decode_matches_oracle(B, H, Hq, L, seed):
    gpu_cases.run_case(B, H, Hq, L, seed)


@pytest.mark.parametrize("B,H,Hq,L,seed,pieces", [
    (1, 1, 1, 64, 30, None),             # one chunk
    (1, 1, 1, 1024, 31, None),           # benchmark configuration 0 with packs of 8
    (2, 3, 6, 192 + 9, 32, None),        # G = 2, ragged
    (1, 8, 32, 512, 33, None),           # G = 4
    (1, 2, 16, 256 + 63, 34, None),      # G = 8, full tail
    (3, 5, 5, 7 * 64 + 1, 35, None),     # odd number of blocks per wave
    (2, 2, 4, 64 * 3 + 5, 36, [1, 62, 1, 1, 63, 64, 5]),  # incremental appends
])
def test_packs_of_8_tokens_match_oracle(B, H, Hq, L, seed, pieces):
    """The second pack size (Sec. IV-B): packed bytes bit-exact, three-step path within the bar."""
    gpu_cases.run_case(B, H, Hq, L, seed, pieces=pieces, pack_size=8)


@pytest.mark.parametrize("B,H,Hq,L,seed,pieces,k_rel,v_rel", [
    (1, 1, 1, 64, 40, None, 0.05, 0.05),               # one chunk, codes up to 20
    (1, 1, 1, 1024, 41, None, 1 / 255, 1 / 255),        # finest scale: codes up to 255, widths up to 8
    (2, 3, 6, 192 + 9, 42, None, 0.04, 0.2),            # wide K, narrow V (packs of 8), G = 2
    (1, 8, 32, 512, 43, None, 0.1, 1 / 30),             # narrow K, wide V, G = 4
    (1, 2, 16, 256 + 63, 44, None, 1 / 60, 1 / 100),    # G = 8, full tail
    (3, 5, 5, 7 * 64 + 1, 45, [100, 64, 200, 85], 0.02, 0.03),
])
def test_wide_chunks_match_oracle(B, H, Hq, L, seed, pieces, k_rel, v_rel):
    """Relative scales below 1/15: codes above 15, wide chunk layout (packs of 8 tokens): packed
    bytes bit-exact, K, V, the three-step path and the fused attention within the bar."""
    gpu_cases.run_case(B, H, Hq, L, seed, pieces=pieces, pack_size=8, k_rel=k_rel, v_rel=v_rel)


def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        B, H, G = int(rng.integers(1, 4)), int(rng.choice([1, 2, 3, 5])), int(rng.choice([1, 2, 4, 8, 3, 5, 6, 7]))
        L = int(rng.integers(1, 900))
        cuts = sorted(set(int(c) for c in rng.integers(1, L + 1, size=int(rng.integers(0, 5))) if c < L))
        pieces = [b - a for a, b in zip([0] + cuts, cuts + [L])]
        cases.append((B, H, H * G, L, 100 + i, pieces))
    return cases


@pytest.mark.parametrize("B,H,Hq,L,seed,pieces", _random_shapes(12, 2024))
def test_random_shapes_and_append_patterns(B, H, Hq, L, seed, pieces):
    """Seeded random batch / head / group sizes, lengths and append partitions."""
    gpu_cases.run_case(B, H, Hq, L, seed, pieces=pieces)


@pytest.mark.parametrize("B,H,Hq,L,seed,pieces", _random_shapes(8, 808))
def test_random_shapes_with_packs_of_8(B, H, Hq, L, seed, pieces):
    gpu_cases.run_case(B, H, Hq, L, seed, pieces=pieces, pack_size=8)


@pytest.mark.parametrize("G,kw", [(16, dict()), (12, dict(pack_size=8)), (9, dict(repack=True)),
                                  (16, dict(pack_size=8, k_rel=0.05, v_rel=1 / 255)), (64, dict())])
def test_query_groups_above_8_heads(G, kw):
    """Groups of s * g heads (s, g <= 8) run as s groups of g heads over the same kv-head."""
    gpu_cases.run_case(2, 3, 3 * G, 64 * 9 + 17, 500 + G, pieces=[300, 293], **kw)


@pytest.mark.parametrize("B,H,Hq,L,seed,pieces", _random_shapes(8, 4711))
def test_random_shapes_with_repacking_paging_and_fine_scales(B, H, Hq, L, seed, pieces):
    """The options in combination, chosen by the seed: V-median repacking, a paged arena, packs of
    8 tokens, scales below 1/15 for either tensor."""
    rng = np.random.default_rng(seed)
    kw = dict(repack=bool(rng.integers(0, 2)))
    if rng.integers(0, 2):
        kw.update(pack_size=8, k_rel=float(rng.choice([0.1, 1 / 40])), v_rel=float(rng.choice([0.2, 1 / 255])))
    pool = binding.PagePool(128) if rng.integers(0, 2) else None
    gpu_cases.run_case(B, H, Hq, L, seed, pieces=pieces, pool=pool, **kw)
    if pool is not None:
        assert pool.kv_page_pool_free_pages() == 128
        pool.close()


def test_benchmark_configuration_1_llama2_7b_4k():
    w = synth.workload(1)
    sizes = gpu_cases.run_case(w.batch, w.n_kv_heads, w.n_q_heads, w.tokens, 1)
    assert sizes["k_bytes"] > 0


def test_incremental_appends_equal_bulk_compression():
    """Token-by-token growth with flushes every 64 tokens gives the same bytes as one call."""
    gpu_cases.run_case(2, 2, 4, 64 * 3 + 5, 20, pieces=[1, 62, 1, 1, 63, 64, 5])
    gpu_cases.run_case(1, 3, 3, 200, 21, pieces=[130, 70])
    gpu_cases.run_case(1, 1, 1, 130, 22, pieces=[1] * 130)


def test_compressor_takes_each_of_its_paths_and_writes_the_same_bytes():
    """Packs of 16, contiguous arena: a round is staged in parts (quantized once) when even its
    largest chunks fit what is left of the arena, else sized and written in two passes; the host
    skips the two-pass kernels where its own bound already says "fits" (and rounds below 1024
    chunks always take two passes).  Three appends into an arena sized for 2.85 bits per element
    meet all three cases, and the state stays the oracle's bit for bit."""
    B, H, Hq, blocks = 2, 4, 8, [150, 130, 128]   # 1200, 1040, 1024 chunks; the staging area holds 512
    L = 64 * sum(blocks)
    K, V, q = synth.make_kv(B, L, H, Hq, 77)
    cache = binding.PackedKVCache(B, H, Hq, L, k_rel_scale=0.2, v_rel_scale=0.2, bits_per_element_budget=2.85)
    n_packed, ck, cv = gpu_cases.oracle_cache(K.numpy(), V.numpy(), 0.2, 0.2)
    # which path each append takes, from the oracle's chunk sizes (288 units of 16 bytes: the largest chunk)
    seen = set()
    for c, cap16 in ((ck, cache.sizes.k_arena // 16), (cv, cache.sizes.v_arena // 16)):
        done = bound = 0
        for nb in blocks:
            n = nb * B * H
            host_sure = bound + n * 288 <= cap16
            staged = int(c.offsets16[done]) + n * 288 <= cap16
            assert int(c.offsets16[done + n]) <= cap16, "no append of this test overflows"
            seen.add((host_sure, staged))
            bound, done = bound + n * 288, done + n
    assert seen == {(True, True), (False, True), (False, False)}
    pos = 0
    for nb in blocks:
        cache.kv_compress_append(K[:, pos:pos + 64 * nb].contiguous().cuda(), V[:, pos:pos + 64 * nb].contiguous().cuda())
        pos += 64 * nb
    gpu_cases.check_packed_state(cache, n_packed, ck, cv, B, H)
    cache.close()


def test_rounding_ties_of_the_quantizer_follow_the_divide():
    """Quotients (x - min) / scale that are exactly k + 1/2 (scale 1, values on the half-integers)
    round to even, as rint of the IEEE quotient does; the compressor's reciprocal shortcut has to
    notice them.  Bit-exact bytes, both pack sizes."""
    B, H, Hq, L = 1, 2, 2, 256
    gen = torch.Generator().manual_seed(4242)
    for pack_size in (16, 8):
        halves = torch.randint(0, 21, (B, L, H, 128), generator=gen).to(torch.float32) / 2  # 0, 0.5, ..., 10
        halves[:, :, 0, 0] = 0.0
        halves[:, :, 0, 1] = 10.0      # every token: minimum 0, range 10, scale 0.1 * 10 -> 1 in fp16
        K = (halves - 3.0).to(torch.float16)   # a minimum that is not zero
        V = halves.flip(1).contiguous().to(torch.float16)
        cache = binding.PackedKVCache(B, H, Hq, L, k_rel_scale=0.1, v_rel_scale=0.1, pack_size=pack_size)
        cache.kv_compress_append(K.cuda(), V.cuda())
        n_packed, ck, cv = gpu_cases.oracle_cache(K.numpy(), V.numpy(), 0.1, 0.1, pack_size)
        assert int(ck.codes.max()) == 10 and (ck.codes[:, :, 0, 2:] % 2 == 0).mean() > 0.7, "ties went to even"
        gpu_cases.check_packed_state(cache, n_packed, ck, cv, B, H)
        cache.close()


def test_decode_kernels_on_oracle_packed_bytes():
    """Feed the fused kernels a cache written by the oracle (restore path):
    isolates the decode kernels from the GPU compressor."""
    B, H, Hq, L = 2, 4, 8, 448
    K, V, q = synth.make_kv(B, L, H, Hq, 30)
    n_packed, ck, cv = gpu_cases.oracle_cache(K.numpy(), V.numpy())
    cache = binding.PackedKVCache(B, H, Hq, L)
    for name, c in (("k", ck), ("v", cv)):
        cache.tensors[name + "_arena"][:c.arena.size].copy_(torch.from_numpy(c.arena))
        cache.view(name + "_index", torch.int32)[:c.offsets16.size].copy_(
            torch.from_numpy(c.offsets16.view(np.int32)))
        cache.view(name + "_token_meta", torch.int32).view(B, -1)[:, :L].copy_(
            torch.from_numpy(c.meta.view(np.int32)))
    cache.kv_cache_restore(L)
    qd = q.cuda()
    scores = cache.kv_k_matvec(qd, 0.125)
    p = synth.make_probs(scores)
    out = cache.kv_v_matvec(p)
    torch.cuda.synchronize()
    s_ref = oracle.k_scores(ck.codes, K.numpy(), ck.meta, L, q.numpy(), 0.125)
    o_ref = oracle.v_out(cv.codes, V.numpy(), cv.meta, L, p.cpu().numpy())
    assert_close_vectors(scores.cpu().numpy(), s_ref, "K scores on oracle bytes")
    assert_close_vectors(out.cpu().numpy(), o_ref, "V out on oracle bytes")


def _special_case(K, V, Hq, k_rel=0.1, v_rel=0.2):
    """Compress given fp16 arrays on the GPU, compare bytes and a decode step."""
    B, L, H, _ = K.shape
    q = synth.make_kv(B, 64, H, Hq, 99)[2]
    cache = binding.PackedKVCache(B, H, Hq, L, k_rel_scale=k_rel, v_rel_scale=v_rel)
    cache.kv_compress_append(torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda())
    n_packed, ck, cv = gpu_cases.oracle_cache(K, V, k_rel, v_rel)
    st = gpu_cases.check_packed_state(cache, n_packed, ck, cv, B, H)
    scores = cache.kv_k_matvec(q.cuda(), 1.0)
    p = synth.make_probs(scores)
    out = cache.kv_v_matvec(p)
    torch.cuda.synchronize()
    kc, km = gpu_cases.full_codes(ck, K.shape, n_packed)
    vc, vm = gpu_cases.full_codes(cv, V.shape, n_packed)
    assert_close_vectors(scores.cpu().numpy(), oracle.k_scores(kc, K, km, n_packed, q.numpy(), 1.0), "K")
    assert_close_vectors(out.cpu().numpy(), oracle.v_out(vc, V, vm, n_packed, p.cpu().numpy()), "V")
    return st, ck, cv


def test_degenerate_inputs():
    rng = np.random.default_rng(40)
    # constant tokens (scale 0, width 0 everywhere): chunks are headers only
    K = np.full((1, 128, 2, 128), 1.5, np.float16)
    V = np.zeros((1, 128, 2, 128), np.float16)
    V[0, 3] = -0.0
    st, ck, _ = _special_case(K, V, 2)
    assert st.k_bytes == 4 * 512 and (ck.widths == 0).all()
    # every pack at the maximum width 4 (rel 1/15, codes 0..15 on an exact grid)
    codes = rng.integers(0, 16, size=(1, 64, 1, 128))
    codes[0, 0::2] = np.where(np.arange(128) % 2 == 0, 0, 15)[None, None, :]
    codes[0, 1::2] = np.where(np.arange(128) % 2 == 0, 15, 0)[None, None, :]
    x = (codes - 7).astype(np.float16)
    st, ck, _ = _special_case(x, x.copy(), 1, k_rel=1 / 15, v_rel=1 / 15)
    assert (ck.widths == 4).all() and st.k_bytes == binding.CHUNK_MAX_BYTES
    # widths 1 and 3 mixed in, large dynamic range, subnormal and big values
    K = (rng.standard_normal((2, 64, 2, 128)) * 100).astype(np.float16)
    K[0, :, 0, :8] = 6.0e-8
    K[1, 5] = 60000.0
    K[1, 5, 0, 0] = -60000.0
    V = (rng.standard_normal((2, 64, 2, 128)) * 1e-3).astype(np.float16)
    _special_case(K, V, 4)
    # V tokens with a range around 4000 (scale above 256 at rel 0.2) under peaked attention: weights of
    # the fused path reach 2^8 * scale, far above the fp16 range
    V = (rng.standard_normal((1, 192, 2, 128)) * 3).astype(np.float16)
    V[0, 7::16] = (rng.uniform(-2000, 2000, size=(12, 2, 128))).astype(np.float16)
    K = (rng.standard_normal((1, 192, 2, 128))).astype(np.float16)
    q = synth.make_kv(1, 64, 2, 4, 98)[2]
    K[0, 7, :, :] = (q[0, ::2].numpy().astype(np.float32) * 3).astype(np.float16)   # token 7 takes most of the weight
    st, ck, cv = _special_case(K, V, 4)
    cache = binding.PackedKVCache(1, 2, 4, 192)
    cache.kv_compress_append(torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda())
    attn = cache.kv_decode_attention(q.cuda(), 1.0).cpu().numpy()
    kc, km = gpu_cases.full_codes(ck, K.shape, 192)
    vc, vm = gpu_cases.full_codes(cv, V.shape, 192)
    assert np.isfinite(attn).all()
    assert_close_vectors(attn, oracle.attention(kc, K, km, vc, V, vm, 192, q.numpy(), 1.0), "fused attention, V range 4000")
    cache.close()
    # the same tokens through packs of 8: the fp16 weight split clamps such weights, the result stays finite
    c8 = binding.PackedKVCache(1, 2, 4, 192, pack_size=8)
    c8.kv_compress_append(torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda())
    assert torch.isfinite(c8.kv_decode_attention(q.cuda(), 1.0)).all()
    c8.close()


@pytest.mark.parametrize("Hq,pack_size,k_rel", [(2, 16, 0.1), (4, 16, 0.1), (2, 8, 0.1), (8, 8, 0.1), (4, 8, 0.05)])
def test_arena_overflow_sets_sticky_flag_and_drops_the_block(Hq, pack_size, k_rel):
    B, H, L = 1, 2, 256
    K, V, q = synth.make_kv(B, L, H, Hq, 50)
    cfg = binding.make_config(B, H, Hq, L, pack_size=pack_size, k_rel_scale=k_rel)
    cache = binding.PackedKVCache(B, H, Hq, L, pack_size=pack_size, k_rel_scale=k_rel)
    # rebuild the handle over a K arena that holds about two blocks only
    sizes = binding.kv_sizes_t.from_buffer_copy(cache.sizes)
    sizes.k_arena = 2 * H * (3300 if pack_size == 16 else (3800 if k_rel == 0.1 else 5600))
    bufs = binding.kv_buffers_t()
    for name in binding._BUFFER_NAMES:
        setattr(bufs, name, cache.tensors[name].data_ptr())
    handle = C.c_void_p()
    assert binding.lib().kv_cache_create(C.byref(cfg), C.byref(bufs), C.byref(sizes), C.byref(handle)) == 0
    binding.lib().kv_cache_destroy(cache.handle)
    cache.handle = handle
    Kd, Vd = K.cuda(), V.cuda()
    for blk in range(4):
        cache.kv_compress_append(Kd[:, blk * 64:(blk + 1) * 64].contiguous(),
                                 Vd[:, blk * 64:(blk + 1) * 64].contiguous())
    st = cache.kv_cache_stats()
    assert st.overflow == 1 and st.k_bytes <= sizes.k_arena
    scores = cache.kv_k_matvec(q.cuda(), 1.0)
    torch.cuda.synchronize()
    n_packed, ck, _ = gpu_cases.oracle_cache(K.numpy(), V.numpy(), k_rel, 0.2, pack_size)
    s_ref = oracle.k_scores(ck.codes, K.numpy(), ck.meta, L, q.numpy(), 1.0)
    kept = st.k_bytes and int(np.searchsorted(ck.offsets16.astype(np.int64) * 16, st.k_bytes, "right") - 1) // (B * H)
    assert 1 <= kept < 4
    assert_close_vectors(scores[:, :, :kept * 64].cpu().numpy(), s_ref[:, :, :kept * 64], "kept blocks")
    assert torch.isinf(scores[:, :, kept * 64:]).all() and (scores[:, :, kept * 64:] < 0).all(), \
        "dropped blocks score -inf"
    # the dropped blocks carry no softmax weight, so the three-step path and the fused path agree
    # (the V arena holds every block here: only K overflowed)
    p = cache.kv_softmax(scores.clone())
    assert (p[:, :, kept * 64:] == 0).all() and torch.isfinite(p).all()
    out3 = cache.kv_v_matvec(p)
    fused = cache.kv_decode_attention(q.cuda(), 1.0)
    torch.cuda.synchronize()
    assert_close_vectors(out3.cpu().numpy(), fused.cpu().numpy().astype(np.float64), "three-step vs fused after an overflow")
    # a row of nothing but dropped blocks comes out as zeros
    none = torch.full_like(scores, float("-inf"))
    assert (cache.kv_softmax(none) == 0).all()


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("B,H,Hq,L,pieces,pack_size,k_rel,v_rel", [
    (2, 3, 6, 3 * 64 + 21, [70, 64, 1, 57, 21], 16, 0.1, 0.2),   # blocks from bulk appends and from tail flushes
    (1, 52, 52, 128, None, 16, 0.1, 0.2),                        # wide token vectors (6656 values per median)
    (2, 4, 8, 150 * 64, None, 16, 0.1, 0.2),                     # 1200 chunks in one call: the staged compressor, in three parts
    (2, 3, 6, 3 * 64 + 21, [70, 64, 1, 57, 21], 8, 0.1, 0.2),    # the same with packs of 8 tokens
    (2, 3, 6, 3 * 64 + 21, [70, 64, 1, 57, 21], 8, 0.1, 1 / 40), # medians of codes up to 40 (wide V chunks)
    (1, 52, 52, 128, None, 8, 1 / 255, 1 / 255),                 # both tensors wide, codes up to 255
])
def test_v_median_repacking_matches_oracle(B, H, Hq, L, pieces, pack_size, k_rel, v_rel, paged):
    """KV_REPACK_V_MEDIAN: order, packed bytes and token metadata bit-exact against the oracle's
    order applied before its compressor; scores in storage order; attention unchanged."""
    rng = np.random.default_rng(70 + B)
    K, V, q = synth.make_kv(B, L, H, Hq, 71)
    # give the V tokens differently leaning value distributions so that their medians differ
    lean = torch.from_numpy(rng.choice([0.3, 1.0, 3.0], size=(B, L, 1, 1))).float()
    V = (torch.rand(V.shape, generator=torch.Generator().manual_seed(72)) ** lean).to(torch.float16)
    Kn, Vn, qn = K.numpy(), V.numpy(), q.numpy()
    n_packed = L // 64 * 64
    n_pages = max(40, L // 64 * B * H * 2 * 4608 // binding.PAGE_BYTES + 8)
    pool = binding.PagePool(n_pages) if paged else None   # the same through a paged arena
    cache = binding.PackedKVCache(B, H, Hq, L, repack=binding.REPACK_V_MEDIAN, pack_size=pack_size,
                                  k_rel_scale=k_rel, v_rel_scale=v_rel, pool=pool)
    pos = 0
    for n in (pieces or [L]):
        cache.kv_compress_append(K[:, pos:pos + n].contiguous().cuda(), V[:, pos:pos + n].contiguous().cuda())
        pos += n
    cv0 = oracle.compress_v(np.ascontiguousarray(Vn[:, :n_packed]), v_rel, pack_size)
    order = oracle.v_median_order(cv0.codes)
    assert len(np.unique(order[:, :64])) == 64 and not np.array_equal(order[0, :64], np.arange(64))
    Kp = np.concatenate([oracle.apply_order(Kn, order), Kn[:, n_packed:]], axis=1)
    Vp = np.concatenate([oracle.apply_order(Vn, order), Vn[:, n_packed:]], axis=1)
    ck = oracle.compress_k(np.ascontiguousarray(Kp[:, :n_packed]), k_rel, pack_size)
    cv = oracle.compress_v(np.ascontiguousarray(Vp[:, :n_packed]), v_rel, pack_size)
    (gpu_cases.check_paged_state if paged else gpu_cases.check_packed_state)(cache, n_packed, ck, cv, B, H)
    max_tokens = cache.tensors["token_order"].numel() // B
    got_order = cache.tensors["token_order"].view(B, max_tokens)[:, :n_packed].cpu().numpy()
    assert np.array_equal(got_order, order)

    sm = 128 ** -0.5
    kc, km = gpu_cases.full_codes(ck, Kp.shape, n_packed)
    vc, vm = gpu_cases.full_codes(cv, Vp.shape, n_packed)
    scores = cache.kv_k_matvec(q.cuda(), sm)
    assert_close_vectors(scores.cpu().numpy(), oracle.k_scores(kc, Kp, km, n_packed, qn, sm), "K scores, storage order")
    p = synth.make_probs(scores)
    out = cache.kv_v_matvec(p)
    assert_close_vectors(out.cpu().numpy(), oracle.v_out(vc, Vp, vm, n_packed, p.cpu().numpy()), "V out")
    attn = cache.kv_decode_attention(q.cuda(), sm)
    a_perm = oracle.attention(kc, Kp, km, vc, Vp, vm, n_packed, qn, sm)
    assert_close_vectors(attn.cpu().numpy(), a_perm, "attention over the repacked cache")
    # and the repacked cache answers like the cache in arrival order (Att(q, PK, PV) = Att(q, K, V))
    _, ck0, cv0b = gpu_cases.oracle_cache(Kn, Vn, k_rel, v_rel, pack_size)
    kc0, km0 = gpu_cases.full_codes(ck0, Kn.shape, n_packed)
    vc0, vm0 = gpu_cases.full_codes(cv0b, Vn.shape, n_packed)
    a_orig = oracle.attention(kc0, Kn, km0, vc0, Vn, vm0, n_packed, qn, sm)
    assert_close_vectors(attn.cpu().numpy(), a_orig, "attention, arrival order")
    cache.close()
    if paged:
        assert pool.kv_page_pool_free_pages() == n_pages
        pool.close()


@pytest.mark.parametrize("B,Hq,tokens,ld", [
    (3, 1, 1, 1), (5, 1, 63, 64), (1, 4, 8192, 8192), (2, 1, 8193, 8200), (1, 1, 20000, 20003),
    (1, 2, 65536, 65536), (1, 1, 65537, 65540), (1, 1, 200001, 200001), (1, 8, 131072 + 5, 131136),
    (8, 8, 40000, 40000), (66, 8, 70000, 70000),
])
def test_softmax_matches_oracle(B, Hq, tokens, ld):
    """kv_softmax (register path, long-row path, split path) against the oracle's fp64 softmax;
    entries past the cached tokens stay untouched."""
    cache = binding.PackedKVCache(B, 1, Hq, tokens)
    x = torch.zeros(B, tokens, 1, 128, dtype=torch.float16, device="cuda")
    cache.kv_compress_append(x, x)
    assert cache.tokens == tokens
    gen = torch.Generator(device="cuda").manual_seed(B * 1000 + tokens)
    s = torch.randn(B, Hq, ld, generator=gen, device="cuda") * 6.0
    s[0, 0, tokens // 2] = 40.0                   # one dominant score
    s_host = s.cpu().numpy()
    d = s.clone()
    assert cache.kv_softmax(d) is d
    got = d.cpu().numpy()
    rows = min(B * Hq, 16)                        # the oracle on a sample of rows
    ref = oracle.softmax(s_host.reshape(B * Hq, ld)[:rows, :tokens].astype(np.float64))
    assert_close_vectors(got.reshape(B * Hq, ld)[:rows, :tokens], ref, "softmax", tol=1e-5)
    assert np.allclose(got[..., :tokens].sum(axis=-1), 1.0, atol=2e-5)
    assert np.array_equal(got[..., tokens:], s_host[..., tokens:])
    d2 = s.clone()
    cache.kv_softmax(d2)
    assert torch.equal(d, d2), "bitwise reproducible"
    assert binding.lib().kv_softmax(cache.handle, d.data_ptr(), tokens - 1, None) == -1
    cache.close()


def test_host_argument_errors():
    cache = binding.PackedKVCache(1, 2, 2, 128)
    L = binding.lib()
    x = torch.zeros(1, 64, 2, 128, dtype=torch.float16, device="cuda")
    q0 = torch.zeros(1, 2, 128, dtype=torch.float16, device="cuda")
    o0 = torch.zeros(1, 2, 128, dtype=torch.float32, device="cuda")
    assert L.kv_decode_attention(cache.handle, q0.data_ptr(), 1.0, o0.data_ptr(), None) == -1   # empty cache
    assert L.kv_compress_append(cache.handle, x.data_ptr(), None, 64, None) == -1
    assert L.kv_compress_append(cache.handle, x.data_ptr(), x.data_ptr(), -1, None) == -1
    assert L.kv_compress_append(cache.handle, x.data_ptr(), x.data_ptr(), 129, None) == -3
    cache.kv_compress_append(x, x)
    q = torch.zeros(1, 2, 128, dtype=torch.float16, device="cuda")
    s = torch.zeros(1, 2, 32, dtype=torch.float32, device="cuda")
    assert L.kv_k_matvec(cache.handle, q.data_ptr(), 1.0, s.data_ptr(), 32, None) == -1   # ld < tokens
    s64 = torch.zeros(1, 2, 64, dtype=torch.float32, device="cuda")
    assert L.kv_k_matvec(cache.handle, q.data_ptr() + 2, 1.0, s64.data_ptr(), 64, None) == -1        # q not 16-byte aligned
    assert L.kv_decode_attention(cache.handle, q.data_ptr() + 2, 1.0, o0.data_ptr(), None) == -1  # the same
    assert L.kv_v_matvec(cache.handle, s.data_ptr(), 32, s.data_ptr(), None) == -1
    with pytest.raises(binding.PackKVError):
        cache.kv_compress_append(torch.zeros(1, 65, 2, 128, dtype=torch.float16, device="cuda"),
                                 torch.zeros(1, 65, 2, 128, dtype=torch.float16, device="cuda"))


@pytest.mark.parametrize("B,H,Hq,L", [(1, 2, 2, 1000), (2, 2, 8, 333), (1, 3, 21, 500)])
def test_fp16_companion_gemv(B, H, Hq, L):
    """The uncompressed fp16 comparison kernels against numpy fp64."""
    K, V, q = synth.make_kv(B, L, H, Hq, 60)
    Kh = K.permute(0, 2, 1, 3).contiguous().cuda()     # head-major [B, H, L, D]
    Vh = V.permute(0, 2, 1, 3).contiguous().cuda()
    scores = binding.kv_fp16_k_matvec(Kh, q.cuda(), 0.25, H)
    p = synth.make_probs(scores)
    out = binding.kv_fp16_v_matvec(Vh, p)
    torch.cuda.synchronize()
    s_ref = oracle.k_scores(None, K.numpy(), None, 0, q.numpy(), 0.25)
    o_ref = oracle.v_out(None, V.numpy(), None, 0, p.cpu().numpy())
    assert_close_vectors(scores.cpu().numpy(), s_ref, "fp16 K")
    assert_close_vectors(out.cpu().numpy(), o_ref, "fp16 V")
    chk = torch.zeros(1, dtype=torch.int32, device="cuda")
    binding.kv_stream_read(Kh, chk)
    torch.cuda.synchronize()
    ref = np.bitwise_xor.reduce(Kh.cpu().numpy().view(np.uint32).ravel())
    assert int(chk.cpu().numpy().view(np.uint32)[0]) == int(ref)


@pytest.mark.parametrize("kw", [dict(), dict(pack_size=8), dict(pack_size=8, k_rel=1 / 255, v_rel=1 / 40),
                                dict(repack=binding.REPACK_V_MEDIAN)])
def test_non_finite_inputs_keep_the_format_valid(kw):
    """NaN and infinities in the input give unspecified codes, but the packed format stays valid:
    every chunk parses with the independent reader, widths and codes stay in range, sizes add up,
    and the decode entry points run."""
    from tests import chunk_reader
    B, H, Hq, L = 2, 2, 4, 64 * 3 + 5
    K, V, q = synth.make_kv(B, L, H, Hq, 66)
    rng = np.random.default_rng(66)
    for x in (K, V):
        flat = x.view(-1)
        idx = torch.from_numpy(rng.choice(flat.numel(), 400, replace=False))
        flat[idx[:150]] = float("nan")
        flat[idx[150:275]] = float("inf")
        flat[idx[275:]] = float("-inf")
    K[0, 70] = float("nan")          # a whole token of NaN
    V[1, 3] = float("inf")           # and one of infinities
    cache = binding.PackedKVCache(B, H, Hq, L, **{("k_rel_scale" if k == "k_rel" else "v_rel_scale" if k == "v_rel" else k): v
                                                  for k, v in kw.items()})
    cache.kv_compress_append(K.cuda(), V.cuda())
    st = cache.kv_cache_stats()
    assert st.overflow == 0 and st.packed_tokens == 192
    n_chunks = 3 * B * H
    pk = kw.get("pack_size", 16)
    for name, rel in (("k", kw.get("k_rel", 0.1)), ("v", kw.get("v_rel", 0.2))):
        qmax = round(1 / rel)
        index = cache.view(name + "_index", torch.int32)[:n_chunks + 1].cpu().numpy().view(np.uint32).astype(np.int64)
        assert index[0] == 0 and (np.diff(index) > 0).all() and index[-1] * 16 == (st.k_bytes if name == "k" else st.v_bytes)
        arena = cache.tensors[name + "_arena"][:index[-1] * 16].cpu().numpy()
        for c in range(n_chunks):
            buf = arena[index[c] * 16:index[c + 1] * 16]
            codes, widths, mins = chunk_reader.read_chunk_wide(buf) if qmax > 15 else chunk_reader.read_chunk(buf, pk, "channel" if name == "k" else "group")
            assert codes.min() >= 0 and codes.max() <= qmax and widths.max() <= (8 if qmax > 15 else 4)
    scores = cache.kv_k_matvec(q.cuda(), 0.1)
    cache.kv_softmax(scores)
    cache.kv_v_matvec(scores)
    cache.kv_decode_attention(q.cuda(), 0.1)
    torch.cuda.synchronize()
    cache.close()


@pytest.mark.parametrize("kw", [dict(), dict(pack_size=8, k_rel_scale=0.05, v_rel_scale=1 / 255),
                                dict(repack=binding.REPACK_V_MEDIAN), dict(big=True)])
def test_bf16_inputs_enter_as_their_fp16_roundings(kw):
    """kv_compress_append_bf16: packed bytes, index, token metadata, raw tail and every result are
    bitwise those of kv_compress_append on the inputs rounded to fp16 -- and those are compared
    with the oracle.  The values include magnitudes below fp16's normal range (rounded in its
    subnormal grid) and bf16 values that fp16 holds exactly.  big: one append of 1120 chunks per
    tensor, which takes the staged compressor."""
    kw = dict(kw)
    big = kw.pop("big", False)
    B, H, Hq, L = (2, 4, 8, 64 * 140 + 23) if big else (2, 3, 6, 64 * 5 + 23)
    g = torch.Generator().manual_seed(808)
    K = torch.randn(B, L, H, 128, generator=g)
    V = torch.randn(B, L, H, 128, generator=g) * 0.3
    K[:, ::7] *= 1e-5                      # tokens of tiny magnitudes: fp16 subnormals
    V[0, 5] = 0.0
    Kb, Vb = K.to(torch.bfloat16), V.to(torch.bfloat16)
    Kh, Vh = Kb.to(torch.float16), Vb.to(torch.float16)
    assert not torch.equal(Kh.float(), Kb.float()), "some values are meant to round"
    q = torch.randn(B, Hq, 128, generator=g).to(torch.float16)
    pieces = [64 * 140, 23] if big else [70, 64, 1, 190, 18]
    caches = []
    for Kx, Vx in ((Kb, Vb), (Kh, Vh)):
        cache = binding.PackedKVCache(B, H, Hq, L, **kw)
        pos = 0
        for n in pieces:
            cache.kv_compress_append(Kx[:, pos:pos + n].contiguous().cuda(), Vx[:, pos:pos + n].contiguous().cuda())
            pos += n
        caches.append(cache)
    a, b = caches
    sa, sb = a.kv_cache_stats(), b.kv_cache_stats()
    assert (sa.k_bytes, sa.v_bytes, sa.packed_tokens, sa.tail_tokens) == (sb.k_bytes, sb.v_bytes, sb.packed_tokens, sb.tail_tokens)
    n_chunks = sa.n_chunks
    for name, n in (("k_arena", sa.k_bytes), ("v_arena", sa.v_bytes), ("k_index", 4 * (n_chunks + 1)),
                    ("v_index", 4 * (n_chunks + 1)), ("k_token_meta", None), ("v_token_meta", None)):
        ta, tb = a.tensors[name], b.tensors[name]
        if name.endswith("token_meta"):
            mt = ta.numel() // 4 // B
            ta, tb = ta.view(torch.int32).view(B, mt)[:, :sa.packed_tokens], tb.view(torch.int32).view(B, mt)[:, :sa.packed_tokens]
        else:
            ta, tb = ta[:n], tb[:n]
        assert torch.equal(ta, tb), name
    tail_elems = sa.tail_tokens * H * 128
    for name in ("k_tail", "v_tail"):
        ta = a.tensors[name].view(torch.float16).view(B, 64 * H * 128)[:, :tail_elems]
        tb = b.tensors[name].view(torch.float16).view(B, 64 * H * 128)[:, :tail_elems]
        assert torch.equal(ta, tb), name
    qd = q.cuda()
    for fn in (lambda c: c.kv_k_matvec(qd, 0.09), lambda c: c.kv_decode_attention(qd, 0.09)):
        assert torch.equal(fn(a), fn(b))
    # and against the oracle on the rounded values
    if not kw.get("repack"):
        n_packed, ck, cv = gpu_cases.oracle_cache(Kh.numpy(), Vh.numpy(), kw.get("k_rel_scale", 0.1),
                                                  kw.get("v_rel_scale", 0.2), kw.get("pack_size", 16))
        gpu_cases.check_packed_state(a, n_packed, ck, cv, B, H)
    a.close()
    b.close()
