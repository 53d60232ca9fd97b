"""GPU parity at the full benchmark sizes, in the launch configuration bench.py
times: inputs are generated on the device, the whole cache is compressed and
decoded by the HIP library, and the oracle recomputes complete batch elements
(every chunk byte, every score, every output of that element)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_24449_amd import binding, synth
from tests.gpu_cases import assert_close_vectors

pytestmark = pytest.mark.gpu


def _check_batch_element(cache, K, V, q, scores, p, out, b, sm_scale, n_packed, attn=None, pack_size=16,
                         k_rel=0.1, v_rel=0.2):
    """Oracle over batch element b (all heads, all tokens) against the GPU state and outputs."""
    B, L, H, _ = K.shape
    Kb = K[b:b + 1].cpu().numpy()
    Vb = V[b:b + 1].cpu().numpy()
    qb = q[b:b + 1].cpu().numpy()
    st = cache.kv_cache_stats()
    assert st.overflow == 0 and st.packed_tokens == n_packed
    n_blk = n_packed // 64
    max_tokens = cache.tensors["k_token_meta"].numel() // 4 // B
    codes = {}
    for name, x, rel, nbytes in (("k", Kb, k_rel, st.k_bytes), ("v", Vb, v_rel, st.v_bytes)):
        c = (oracle.compress_k if name == "k" else oracle.compress_v)(np.ascontiguousarray(x[:, :n_packed]), rel, pack_size)
        meta = cache.view(name + "_token_meta", torch.int32).view(B, max_tokens)[b, :n_packed]
        assert np.array_equal(meta.cpu().numpy().view(np.uint32), c.meta[0]), name + " token meta"
        index = cache.view(name + "_index", torch.int32)[:st.n_chunks + 1].cpu().numpy().view(np.uint32).astype(np.int64)
        arena = cache.tensors[name + "_arena"][:nbytes].cpu().numpy()
        off = c.offsets16.astype(np.int64)
        for blk in range(n_blk):            # chunks (blk, b, 0..H-1) are contiguous on both sides
            g0, g1 = index[(blk * B + b) * H] * 16, index[(blk * B + b) * H + H] * 16
            o0, o1 = off[blk * H] * 16, off[blk * H + H] * 16
            assert g1 - g0 == o1 - o0, (name, blk)
            assert np.array_equal(arena[g0:g1], c.arena[o0:o1]), "%s arena bytes of block %d" % (name, blk)
        full = np.zeros(x.shape, np.uint8)
        full[:, :n_packed] = c.codes
        fmeta = np.zeros((1, L), np.uint32)
        fmeta[:, :n_packed] = c.meta
        codes[name] = (full, fmeta)
    s_ref = oracle.k_scores(codes["k"][0], Kb, codes["k"][1], n_packed, qb, sm_scale)
    assert_close_vectors(scores[b:b + 1, :, :L].cpu().numpy(), s_ref, "K scores, batch %d" % b)
    pb = p[b:b + 1].cpu().numpy()
    o_ref = oracle.v_out(codes["v"][0], Vb, codes["v"][1], n_packed, pb)
    assert_close_vectors(out[b:b + 1].cpu().numpy(), o_ref, "V out, batch %d" % b)
    if attn is not None:
        a_ref = oracle.attention(codes["k"][0], Kb, codes["k"][1], codes["v"][0], Vb, codes["v"][1],
                                 n_packed, qb, sm_scale)
        assert_close_vectors(attn[b:b + 1].cpu().numpy(), a_ref, "fused decode attention, batch %d" % b)


@pytest.mark.parametrize("index,batch_elements,pack_size", [(3, [7], 16), (2, [0, 3], 16), (2, [1], 8)])
def test_full_size_configuration(index, batch_elements, pack_size):
    """Benchmark configurations 3 (8 x 52 heads x 32000 tokens) and 2 (GQA, 4 x 8/32 heads x 32768),
    the latter also with packs of 8 tokens."""
    w = synth.workload(index)
    K, V, q = synth.make_workload(w, device="cuda:0")
    L = w.tokens
    cache = binding.PackedKVCache(w.batch, w.n_kv_heads, w.n_q_heads, L, pack_size=pack_size)
    cache.kv_compress_append(K, V)
    sm_scale = 128 ** -0.5
    scores = cache.kv_k_matvec(q, sm_scale)
    p = synth.make_probs(scores)
    out = cache.kv_v_matvec(p)
    attn = cache.kv_decode_attention(q, sm_scale)
    torch.cuda.synchronize()
    # properties that hold for every element, checked everywhere
    assert torch.isfinite(scores).all() and torch.isfinite(out).all() and torch.isfinite(attn).all()
    # the fused pass and the three-step path agree on every output (p here is a softmax of the scores)
    assert_close_vectors(attn.cpu().numpy(), out.cpu().numpy().astype(np.float64), "fused vs three-step")
    st = cache.kv_cache_stats()
    n_chunks = L // 64 * w.batch * w.n_kv_heads
    assert st.n_chunks == n_chunks and st.overflow == 0
    index_t = cache.view("k_index", torch.int32)[:n_chunks + 1].to(torch.int64)
    sizes = (index_t[1:] - index_t[:-1]) * 16
    header = 512 if pack_size == 16 else 1024
    assert int(sizes.min()) >= header and int(sizes.max()) <= header + 4096
    for b in batch_elements:
        _check_batch_element(cache, K, V, q, scores, p, out, b, sm_scale, L // 64 * 64, attn, pack_size)
    cache.close()


@pytest.mark.parametrize("B,H,Hq,L,k_rel,v_rel", [(1, 8, 32, 32768, 1 / 255, 1 / 255), (2, 4, 4, 16384 + 33, 0.05, 0.04)])
def test_wide_chunks_long_context(B, H, Hq, L, k_rel, v_rel):
    """Fine scales over long contexts: the softmax weights are tiny and the code sums large, so the
    V output is the difference of large terms -- the case in which a sign bias in the weight
    split showed up as 6e-3 output error.  Whole outputs against the oracle."""
    K, V, q = synth.make_kv(B, L, H, Hq, 90)
    cache = binding.PackedKVCache(B, H, Hq, L, k_rel_scale=k_rel, v_rel_scale=v_rel, pack_size=8)
    cache.kv_compress_append(K.cuda(), V.cuda())
    sm_scale = 128 ** -0.5
    scores = cache.kv_k_matvec(q.cuda(), sm_scale)
    p = synth.make_probs(scores)
    out = cache.kv_v_matvec(p)
    attn = cache.kv_decode_attention(q.cuda(), sm_scale)
    torch.cuda.synchronize()
    assert cache.kv_cache_stats().overflow == 0
    for b in range(B):
        _check_batch_element_rel(cache, K, V, q, scores, p, out, b, sm_scale, L // 64 * 64, k_rel, v_rel, attn)
    cache.close()


def _check_batch_element_rel(cache, K, V, q, scores, p, out, b, sm_scale, n_packed, k_rel, v_rel, attn):
    _check_batch_element(cache, K.cuda(), V.cuda(), q.cuda(), scores, p, out, b, sm_scale, n_packed, attn, 8,
                         k_rel, v_rel)


def test_growing_cache_decode_steps():
    """Benchmark configuration 4 (growing cache) in full: start at 131072 tokens, append one token per
    decode step for all its 1024 steps (16 tail flushes); every appended block's bytes and the outputs
    of a batch element are compared with the oracle at a step with a part-filled tail and at the end."""
    w = synth.workload(4)
    steps = w.decode_steps
    assert steps == 1024
    K, V, q = synth.make_kv(w.batch, w.tokens + steps, w.n_kv_heads, w.n_q_heads, 4, device="cuda:0")
    L0 = w.tokens
    cache = binding.PackedKVCache(w.batch, w.n_kv_heads, w.n_q_heads, L0 + steps)
    cache.kv_compress_append(K[:, :L0].contiguous(), V[:, :L0].contiguous())
    sm_scale = 128 ** -0.5
    scores = torch.empty(w.batch, w.n_q_heads, L0 + steps, dtype=torch.float32, device="cuda")
    for i in range(steps):
        cache.kv_compress_append(K[:, L0 + i:L0 + i + 1].contiguous(), V[:, L0 + i:L0 + i + 1].contiguous())
        n = L0 + i + 1
        cache.kv_k_matvec(q, sm_scale, scores)
        p = torch.softmax(scores[:, :, :n], dim=-1)
        out = cache.kv_v_matvec(p)
        if i in (36, steps - 1):
            attn = cache.kv_decode_attention(q, sm_scale)
            torch.cuda.synchronize()
            assert cache.tokens == n
            _check_batch_element(cache, K[:, :n], V[:, :n], q, scores, p, out, 0, sm_scale, n // 64 * 64,
                                 attn)
    assert cache.kv_cache_stats().tail_tokens == (L0 + steps) % 64
    cache.close()


def test_packed_arena_beyond_4_gib():
    """Maximum-size edge: more than 4 GiB of packed bytes per tensor (8 x 52 heads x 294912 tokens,
    15.7 G elements), so chunk offsets pass 2^32 bytes.  The oracle recomputes sampled blocks one by
    one: chunk bytes, token metadata, the scores of the block, and the V product restricted to the
    sampled blocks; the fused attention must agree with the three-step path everywhere."""
    B, H, Hq, L = 8, 52, 52, 294912
    K, V, q = synth.make_kv(B, L, H, Hq, 9, device="cuda:0")
    cache = binding.PackedKVCache(B, H, Hq, L, bits_per_element_budget=3.0)
    cache.kv_compress_append(K, V)
    st = cache.kv_cache_stats()
    n_blk = L // 64
    assert st.overflow == 0 and st.n_chunks == n_blk * B * H
    assert st.k_bytes > 2 ** 32 and st.v_bytes > 2 ** 32
    sm_scale = 128 ** -0.5
    scores = cache.kv_k_matvec(q, sm_scale)
    samples = [(0, 0), (n_blk // 2, 3), (n_blk - 1, B - 1), (n_blk - 1, 0)]
    p = torch.zeros_like(scores)
    for blk, b in samples:
        p[b, :, blk * 64:(blk + 1) * 64] = torch.softmax(scores[b, :, blk * 64:(blk + 1) * 64], dim=-1)
    out = cache.kv_v_matvec(p)
    del p
    torch.cuda.synchronize()
    index = {n: cache.view(n + "_index", torch.int32)[:st.n_chunks + 1] for n in ("k", "v")}
    max_tokens = cache.tensors["k_token_meta"].numel() // 4 // B
    o_ref = np.zeros((B, Hq, 128))
    for blk, b in samples:
        sl = slice(blk * 64, (blk + 1) * 64)
        Kb, Vb = K[b:b + 1, sl].cpu().numpy(), V[b:b + 1, sl].cpu().numpy()
        qb = q[b:b + 1].cpu().numpy()
        c0 = (blk * B + b) * H
        for name, x, rel in (("k", Kb, 0.1), ("v", Vb, 0.2)):
            c = (oracle.compress_k if name == "k" else oracle.compress_v)(x, rel)
            lo = int(index[name][c0].item()) & 0xFFFFFFFF
            hi = int(index[name][c0 + H].item()) & 0xFFFFFFFF
            assert (hi - lo) * 16 == c.arena.size, (name, blk, b)
            got = cache.tensors[name + "_arena"][lo * 16:hi * 16].cpu().numpy()
            assert np.array_equal(got, c.arena), "%s chunk bytes of block %d, batch %d" % (name, blk, b)
            meta = cache.view(name + "_token_meta", torch.int32).view(B, max_tokens)[b, sl]
            assert np.array_equal(meta.cpu().numpy().view(np.uint32), c.meta[0])
            if name == "k":
                s_ref = oracle.k_scores(c.codes, x, c.meta, 64, qb, sm_scale)
                assert_close_vectors(scores[b:b + 1, :, sl].cpu().numpy(), s_ref, "scores of block %d" % blk)
            else:
                pb = torch.softmax(scores[b:b + 1, :, sl], dim=-1).cpu().numpy()
                o_ref[b] += oracle.v_out(c.codes, x, c.meta, 64, pb)[0]
        if (blk, b) == samples[-2]:
            assert lo * 16 > 2 ** 32, "the sampled chunk lies beyond 4 GiB"
    touched = sorted({b for _, b in samples})
    assert_close_vectors(out[touched].cpu().numpy(), o_ref[touched], "V product over the sampled blocks")
    # whole-cache agreement of the two decode paths
    del K, V
    pfull = synth.make_probs(scores)
    out3 = cache.kv_v_matvec(pfull)
    attn = cache.kv_decode_attention(q, sm_scale)
    torch.cuda.synchronize()
    assert torch.isfinite(attn).all()
    assert_close_vectors(attn.cpu().numpy(), out3.cpu().numpy().astype(np.float64), "fused vs three-step")
    cache.close()


@pytest.mark.parametrize("B,H,Hq,L", [(8, 52, 52, 32000), (4, 8, 32, 32768 + 77), (8, 52, 52, 294912)])
def test_paged_cache_at_full_size(B, H, Hq, L):
    """The paged arena at the headline shape, at the grouped-query shape and past 4 GiB of pages per
    tensor: every result is bitwise the contiguous cache's (whose bytes the tests above compare with
    the oracle), every chunk has the contiguous chunk's size, stays inside one page and overlaps no
    other, and sampled chunks hold the same bytes."""
    K, V, q = synth.make_kv(B, L, H, Hq, 11, device="cuda:0")
    flat = binding.PackedKVCache(B, H, Hq, L, bits_per_element_budget=3.0)
    flat.kv_compress_append(K, V)
    st = flat.kv_cache_stats()
    assert st.overflow == 0
    page = binding.PAGE_BYTES
    n_pages = int((st.k_bytes + st.v_bytes) * 1.04) // page + 16
    pool = binding.PagePool(n_pages)
    paged = binding.PackedKVCache(B, H, Hq, L, pool=pool)
    paged.kv_compress_append(K, V)
    del K, V
    pst = paged.kv_cache_stats()
    assert pst.overflow == 0 and pst.n_chunks == st.n_chunks
    assert pst.k_bytes <= 1.04 * st.k_bytes + 2 * page and pst.v_bytes <= 1.04 * st.v_bytes + 2 * page
    assert pool.kv_page_pool_free_pages() == n_pages - (pst.k_bytes + pst.v_bytes) // page

    sm_scale = 128 ** -0.5
    results = []
    for cache in (flat, paged):
        scores = cache.kv_k_matvec(q, sm_scale)
        p = synth.make_probs(scores)
        results.append((scores, cache.kv_v_matvec(p), cache.kv_decode_attention(q, sm_scale)))
        del p
    torch.cuda.synchronize()
    for a, b, what in zip(results[0], results[1], ("scores", "V product", "fused attention")):
        assert torch.equal(a, b), what + ": paged and contiguous caches differ"
    del results

    n = st.n_chunks
    rng = np.random.default_rng(5)
    sample = sorted(set(rng.integers(0, n, 48).tolist()) | {0, n - 1})
    top = 0
    for name in ("k", "v"):
        pairs = (paged.view(name + "_index", torch.int32)[:2 * n].to(torch.int64) & 0xFFFFFFFF).view(n, 2)
        index = flat.view(name + "_index", torch.int32)[:n + 1].to(torch.int64) & 0xFFFFFFFF
        assert torch.equal(pairs[:, 1] - pairs[:, 0], index[1:] - index[:-1]), name + " chunk sizes"
        units = page // 16
        assert torch.equal(pairs[:, 0] // units, (pairs[:, 1] - 1) // units), name + " chunk crosses a page"
        srt = pairs[torch.argsort(pairs[:, 0])]
        assert bool((srt[1:, 0] >= srt[:-1, 1]).all()), name + " chunks overlap"
        top = max(top, int(pairs[:, 1].max().item()) * 16)
        assert top <= n_pages * page
        for c in sample:
            s, e = (int(x) * 16 for x in pairs[c].tolist())
            lo, hi = int(index[c].item()) * 16, int(index[c + 1].item()) * 16
            assert torch.equal(pool.pages[s:e], flat.tensors[name + "_arena"][lo:hi]), "%s chunk %d bytes" % (name, c)
    if L > 200000:
        assert top > 2 ** 32, "this case is meant to place chunks past 4 GiB"
    flat.close()
    paged.close()
    assert pool.kv_page_pool_free_pages() == n_pages
    pool.close()
