"""Shared machinery of the GPU parity tests: run one cache configuration
through the C-ABI library and through the CPU oracle on the same seeded inputs
and compare.

Acceptance (per output vector y, i.e. one query head's scores over the tokens,
or one query head's 128 outputs):
    packed bytes, chunk index, token metadata      bit-exact
    ||y_gpu - y_orc||_2 <= 1e-3 * ||y_orc||_2  and  max|diff| <= 1e-3 * max|y_orc|
(fp32 accumulation on the GPU against the oracle's fp64).
"""
import numpy as np
import torch

import oracle
from paper_2512_24449_amd import binding, synth

REL_TOL = 1e-3


def assert_close_vectors(got, ref, what, tol=REL_TOL):
    """got/ref: [..., n]; every vector along the last axis must meet the bar."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    if ref.size == 0:
        return
    diff = got - ref
    l2 = np.linalg.norm(diff, axis=-1)
    ref_l2 = np.linalg.norm(ref, axis=-1)
    mx = np.abs(diff).max(axis=-1)
    ref_mx = np.abs(ref).max(axis=-1)
    bad = (l2 > tol * ref_l2 + 1e-30) | (mx > tol * ref_mx + 1e-30)
    assert not bad.any(), "%s: %d vectors off; worst rel l2 %.3e, worst rel max %.3e" % (
        what, int(bad.sum()), float((l2 / np.maximum(ref_l2, 1e-300)).max()),
        float((mx / np.maximum(ref_mx, 1e-300)).max()))


def oracle_cache(K, V, k_rel=0.1, v_rel=0.2, pack_size=16):
    """Compress the packed prefix of K and V with the oracle.  K, V: numpy fp16 [B, L, H, D]."""
    L = K.shape[1]
    n_packed = L // 64 * 64
    ck = oracle.compress_k(np.ascontiguousarray(K[:, :n_packed]), k_rel, pack_size) if n_packed else None
    cv = oracle.compress_v(np.ascontiguousarray(V[:, :n_packed]), v_rel, pack_size) if n_packed else None
    return n_packed, ck, cv


def full_codes(c, shape, n_packed):
    """Codes and token meta padded out to all L tokens (tail rows unused)."""
    B, L, H, D = shape
    codes = np.zeros(shape, np.uint8)
    meta = np.zeros((B, L), np.uint32)
    if n_packed:
        codes[:, :n_packed] = c.codes
        meta[:, :n_packed] = c.meta
    return codes, meta


def check_packed_state(cache, n_packed, ck, cv, B, H):
    """Arena bytes, index and token meta of the GPU cache == the oracle's, bit for bit."""
    st = cache.kv_cache_stats()
    assert st.overflow == 0
    assert st.packed_tokens == n_packed
    if not n_packed:
        return st
    n_chunks = n_packed // 64 * B * H
    assert st.n_chunks == n_chunks
    max_tokens = cache.tensors["k_token_meta"].numel() // 4 // B
    for name, c, nbytes in (("k", ck, st.k_bytes), ("v", cv, st.v_bytes)):
        assert nbytes == c.arena.size, (name, nbytes, c.arena.size)
        index = cache.view(name + "_index", torch.int32)[:n_chunks + 1].cpu().numpy().view(np.uint32)
        assert np.array_equal(index, c.offsets16), name + " index"
        arena = cache.tensors[name + "_arena"][:nbytes].cpu().numpy()
        if not np.array_equal(arena, c.arena):
            first = int(np.nonzero(arena != c.arena)[0][0])
            raise AssertionError("%s arena differs first at byte %d of %d" % (name, first, nbytes))
        meta = cache.view(name + "_token_meta", torch.int32).view(B, max_tokens)[:, :n_packed]
        assert np.array_equal(meta.cpu().numpy().view(np.uint32), c.meta), name + " token meta"
        # the byte split of the statistics: pack metadata, exactly pack_size * width bits per pack, padding
        packs = c.widths.shape[1]
        wide = int(c.widths.max()) > 4 or int(c.mins.max()) > 15
        header = n_chunks * packs * (2 if wide else 1)
        payload = int(c.widths.astype(np.int64).sum()) * (64 * 128 // packs // 8)
        got = (getattr(st, name + "_header_bytes"), getattr(st, name + "_payload_bytes"), getattr(st, name + "_padding_bytes"))
        if not wide or packs == 1024:
            assert got == (header, payload, nbytes - header - payload), (name, got, header, payload, nbytes)
    return st


PAGE16 = binding.PAGE_BYTES // 16


class PagePlacementModel:
    """The placement rule of the paged arena as the header states it, for one pool: a chunk goes
    behind the previous one of its tensor while it fits into that tensor's newest page, else to
    the start of a fresh page; an append takes all its fresh pages or none; page 0 comes first and
    released pages are handed out again newest first."""

    def __init__(self, n_pages):
        self.free = list(range(n_pages - 1, -1, -1))  # stack, top last

    def new_tensor(self):
        return dict(pages=[], fill=PAGE16)

    def place(self, t, sizes16):
        """-> list of (start16, end16) for the chunks of one append call, or None if dropped."""
        fill, need = t["fill"], 0
        for s in sizes16:
            if fill + s > PAGE16:
                need, fill = need + 1, 0
            fill += s
        if need > len(self.free):
            return None
        out, fill = [], t["fill"]
        for s in sizes16:
            if fill + s > PAGE16:
                t["pages"].append(self.free.pop())
                fill = 0
            start = t["pages"][-1] * PAGE16 + fill
            out.append((start, start + s))
            fill += s
        t["fill"] = fill
        return out

    def release(self, *tensors):
        for t in tensors:
            self.free.extend(reversed(t["pages"]))
            t["pages"], t["fill"] = [], PAGE16


def check_paged_state(cache, n_packed, ck, cv, B, H):
    """Paged cache: every chunk's bytes (read through its index pair from the pool's pages), and the
    token metadata, equal the oracle's bit for bit; no chunk crosses a page boundary, chunks lie
    inside pages their tensor holds and do not overlap."""
    st = cache.kv_cache_stats()
    assert st.overflow == 0 and st.packed_tokens == n_packed
    if not n_packed:
        return st
    n_chunks = n_packed // 64 * B * H
    max_tokens = cache.tensors["k_token_meta"].numel() // 4 // B
    pages = cache.pool.pages.cpu().numpy()
    held_all = []
    for name, c, nbytes in (("k", ck, st.k_bytes), ("v", cv, st.v_bytes)):
        plist = cache.view(name + "_pages", torch.int32).cpu().numpy().view(np.uint32)
        held = plist[2:2 + int(plist[0])].astype(np.int64)
        assert nbytes == held.size * binding.PAGE_BYTES
        held_all.append(held)
        pairs = cache.view(name + "_index", torch.int32)[:2 * n_chunks].cpu().numpy().view(np.uint32)
        pairs = pairs.reshape(n_chunks, 2).astype(np.int64)
        assert np.array_equal(pairs[:, 1] - pairs[:, 0], np.diff(c.offsets16.astype(np.int64))), name + " chunk sizes"
        assert np.array_equal(pairs[:, 0] // PAGE16, (pairs[:, 1] - 1) // PAGE16), name + " chunk crosses a page"
        assert np.isin(pairs[:, 0] // PAGE16, held).all(), name + " chunk outside the tensor's pages"
        order = np.argsort(pairs[:, 0])
        assert (pairs[order][1:, 0] >= pairs[order][:-1, 1]).all(), name + " chunks overlap"
        for i in range(n_chunks):
            got = pages[pairs[i, 0] * 16:pairs[i, 1] * 16]
            ref = c.arena[int(c.offsets16[i]) * 16:int(c.offsets16[i + 1]) * 16]
            assert np.array_equal(got, ref), "%s chunk %d differs" % (name, i)
        meta = cache.view(name + "_token_meta", torch.int32).view(B, max_tokens)[:, :n_packed]
        assert np.array_equal(meta.cpu().numpy().view(np.uint32), c.meta), name + " token meta"
    assert not np.intersect1d(held_all[0], held_all[1]).size, "K and V share a page"
    return st


def run_case(B, H, Hq, L, seed, pieces=None, check_bytes=True, sm_scale=None, device="cuda:0",
             max_tokens=None, pack_size=16, k_rel=0.1, v_rel=0.2, pool=None, repack=False):
    """Append L tokens (in `pieces`, default one call), then one decode step; compare everything.
    pool: a binding.PagePool -> the cache is paged.  repack: V-median repacking; the oracle then
    works on the tensors permuted by its own order, and scores compare in storage order."""
    K, V, q = synth.make_kv(B, L, H, Hq, seed)
    if repack:
        # give the V tokens differently leaning value distributions so that their medians differ
        lean = torch.from_numpy(np.random.default_rng(seed).choice([0.3, 1.0, 3.0], size=(B, L, 1, 1))).float()
        V = (torch.rand(V.shape, generator=torch.Generator().manual_seed(seed)) ** lean).to(torch.float16)
    Kn, Vn, qn = K.numpy(), V.numpy(), q.numpy()
    sm_scale = sm_scale if sm_scale is not None else 128 ** -0.5
    cache = binding.PackedKVCache(B, H, Hq, max_tokens or max(L, 64), k_rel_scale=k_rel, v_rel_scale=v_rel,
                                  device=device, pack_size=pack_size, pool=pool,
                                  repack=binding.REPACK_V_MEDIAN if repack else binding.REPACK_NONE)
    Kd, Vd, qd = K.to(device), V.to(device), q.to(device)
    pos = 0
    for n in (pieces or [L]):
        cache.kv_compress_append(Kd[:, pos:pos + n].contiguous(), Vd[:, pos:pos + n].contiguous())
        pos += n
    assert pos == L and cache.tokens == L

    if repack and L >= 64:
        n_full = L // 64 * 64
        order = oracle.v_median_order(oracle.compress_v(np.ascontiguousarray(Vn[:, :n_full]), v_rel, pack_size).codes)
        Kn = np.concatenate([oracle.apply_order(Kn, order), Kn[:, n_full:]], axis=1)
        Vn = np.concatenate([oracle.apply_order(Vn, order), Vn[:, n_full:]], axis=1)
        mt = ((max_tokens or max(L, 64)) + 63) // 64 * 64
        got = cache.tensors["token_order"][:B * mt].view(B, mt)[:, :n_full].cpu().numpy()
        assert np.array_equal(got, order), "token order"
    n_packed, ck, cv = oracle_cache(Kn, Vn, k_rel, v_rel, pack_size)
    if check_bytes:
        (check_paged_state if pool is not None else check_packed_state)(cache, n_packed, ck, cv, B, H)

    scores = cache.kv_k_matvec(qd, sm_scale)
    torch.cuda.synchronize()
    kcodes, kmeta = full_codes(ck, Kn.shape, n_packed)
    s_ref = oracle.k_scores(kcodes, Kn, kmeta, n_packed, qn, sm_scale)
    assert_close_vectors(scores.cpu().numpy(), s_ref, "K scores")

    p = synth.make_probs(scores)
    out = cache.kv_v_matvec(p)
    torch.cuda.synchronize()
    vcodes, vmeta = full_codes(cv, Vn.shape, n_packed)
    o_ref = oracle.v_out(vcodes, Vn, vmeta, n_packed, p.cpu().numpy())
    assert_close_vectors(out.cpu().numpy(), o_ref, "V out")

    # end to end against an fp64 softmax of the oracle's own scores
    p64 = oracle.softmax(s_ref)
    o_e2e = oracle.v_out(vcodes, Vn, vmeta, n_packed, p64.astype(np.float32))
    assert_close_vectors(out.cpu().numpy(), o_e2e, "decode step end to end")

    # the whole three-step path inside the library: K product, softmax in place, V product
    s3 = cache.kv_k_matvec(qd, sm_scale)
    cache.kv_softmax(s3)
    out3 = cache.kv_v_matvec(s3)
    torch.cuda.synchronize()
    assert_close_vectors(out3.cpu().numpy(), o_e2e, "three-step path with the library softmax")

    # determinism: a second pass gives the same bits
    scores2 = cache.kv_k_matvec(qd, sm_scale)
    out2 = cache.kv_v_matvec(p)
    torch.cuda.synchronize()
    assert torch.equal(scores, scores2) and torch.equal(out, out2)

    # fused decode attention against the oracle's definition of Att(q, K, V)
    attn = cache.kv_decode_attention(qd, sm_scale)
    torch.cuda.synchronize()
    a_ref = oracle.attention(kcodes, Kn, kmeta, vcodes, Vn, vmeta, n_packed, qn, sm_scale)
    assert_close_vectors(attn.cpu().numpy(), a_ref, "fused decode attention")
    attn2 = cache.kv_decode_attention(qd, sm_scale)
    torch.cuda.synchronize()
    assert torch.equal(attn, attn2)
    cache.close()
    return dict(k_bytes=ck.arena.size if ck else 0, v_bytes=cv.arena.size if cv else 0,
                scores=scores.cpu(), out=out.cpu(), attn=None if attn is None else attn.cpu())
