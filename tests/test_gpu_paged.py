"""GPU tests of the paged arena: chunks of paged caches live in fixed pages taken from a shared
pool.  Chunk bytes are compared with the CPU oracle's bit for bit, results with a contiguous
cache's bit for bit, and chunk positions with the placement rule stated in include/packkv.h
(gpu_cases.PagePlacementModel, written from that text)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_24449_amd import binding, synth
from tests import gpu_cases
from tests.gpu_cases import PAGE16, assert_close_vectors

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,H,Hq,L,pieces,kw", [
    (2, 3, 3, 64 * 23 + 17, [64 * 9 + 5, 64 * 3, 1, 58, 64 * 10 + 17], dict()),
    (2, 2, 8, 64 * 40 + 3, [64 * 40 + 3], dict()),                       # one bulk append over many pages
    (1, 5, 10, 64 * 21 + 40, [30, 64 * 20, 74], dict(pack_size=8)),
    (2, 2, 4, 64 * 18 + 9, [64 * 7, 64 * 11 + 9], dict(pack_size=8, k_rel=1 / 60, v_rel=1 / 255)),
    # narrow K next to wide V at the finest scale: V takes several times the pages K takes (each
    # tensor's page list has its own capacity)
    (2, 5, 10, 64 * 64 + 31, [3081, 309, 652, 85], dict(pack_size=8, k_rel=0.1, v_rel=1 / 255)),
])
def test_paged_cache_matches_oracle_and_contiguous_cache(B, H, Hq, L, pieces, kw):
    pool = binding.PagePool(256)
    paged = gpu_cases.run_case(B, H, Hq, L, 4242, pieces=pieces, pool=pool, **kw)
    # run_case closed its cache: kv_cache_destroy of a paged cache gives the pages back
    assert pool.kv_page_pool_free_pages() == 256
    flat = gpu_cases.run_case(B, H, Hq, L, 4242, pieces=pieces, **kw)
    for name in ("scores", "out", "attn"):
        if flat[name] is not None:
            assert torch.equal(paged[name], flat[name]), name + ": paged and contiguous caches differ"
    pool.close()


def _chunk_pairs(cache, name, n_chunks):
    w = cache.view(name + "_index", torch.int32)[:2 * n_chunks].cpu().numpy().view(np.uint32)
    return [tuple(int(x) for x in row) for row in w.reshape(n_chunks, 2)]


def _page_list(cache, name):
    w = cache.view(name + "_pages", torch.int32).cpu().numpy().view(np.uint32)
    return [int(x) for x in w[2:2 + int(w[0])]], int(w[1])


def test_two_caches_share_a_pool_by_the_stated_placement_rule():
    n_pages = 48
    pool = binding.PagePool(n_pages)
    model = gpu_cases.PagePlacementModel(n_pages)
    shapes = [(2, 3, 3), (1, 4, 8)]
    caches, data, tensors, expected = [], [], [], []
    for i, (B, H, Hq) in enumerate(shapes):
        caches.append(binding.PackedKVCache(B, H, Hq, 64 * 12, pool=pool, pack_size=16 if i == 0 else 8))
        K, V, q = synth.make_kv(B, 64 * 12, H, Hq, 90 + i)
        data.append((K, V, q))
        tensors.append((model.new_tensor(), model.new_tensor()))
        expected.append(([], []))
    # interleaved appends of different lengths; the model sees the oracle's chunk sizes
    schedule = [(0, 64 * 2), (1, 64 * 5), (0, 64 * 7), (1, 64), (0, 64 * 3), (1, 64 * 6)]
    done = [0, 0]
    for who, n in schedule:
        B, H, Hq = shapes[who]
        K, V, _ = data[who]
        lo, hi = done[who], done[who] + n
        caches[who].kv_compress_append(K[:, lo:hi].contiguous().cuda(), V[:, lo:hi].contiguous().cuda())
        pk = 16 if who == 0 else 8
        for t, (x, rel) in enumerate(((K, 0.1), (V, 0.2))):
            # chunk sizes depend on the appended blocks alone: compress just those with the oracle
            c = (oracle.compress_v if t else oracle.compress_k)(np.ascontiguousarray(x.numpy()[:, lo:hi]), rel, pk)
            sizes = np.diff(c.offsets16.astype(np.int64)).tolist()
            # the library compresses at most 65536 chunks per round; these calls are far below
            placed = model.place(tensors[who][t], sizes)
            assert placed is not None
            expected[who][t].extend(placed)
        done[who] = hi
    torch.cuda.synchronize()
    seen_pages = []
    for who, (B, H, Hq) in enumerate(shapes):
        n_chunks = done[who] // 64 * B * H
        for t, name in enumerate(("k", "v")):
            assert _chunk_pairs(caches[who], name, n_chunks) == expected[who][t], (who, name)
            pages, fill = _page_list(caches[who], name)
            assert pages == tensors[who][t]["pages"] and fill == tensors[who][t]["fill"]
            seen_pages += pages
    assert len(seen_pages) == len(set(seen_pages)), "a page is held twice"
    assert pool.kv_page_pool_free_pages() == n_pages - len(seen_pages) == len(model.free)

    # both caches still decode correctly next to each other
    for who, (B, H, Hq) in enumerate(shapes):
        K, V, q = data[who]
        pk = 16 if who == 0 else 8
        n_packed, ck, cv = gpu_cases.oracle_cache(K.numpy(), V.numpy(), 0.1, 0.2, pk)
        gpu_cases.check_paged_state(caches[who], n_packed, ck, cv, B, H)
        attn = caches[who].kv_decode_attention(q.cuda(), 0.09)
        torch.cuda.synchronize()
        a_ref = oracle.attention(ck.codes, K.numpy(), ck.meta, cv.codes, V.numpy(), cv.meta, n_packed,
                                 q.numpy(), 0.09)
        assert_close_vectors(attn.cpu().numpy(), a_ref, "fused attention, cache %d" % who)

    # release the first cache: its pages are free again and the second cache is untouched
    caches[0].kv_cache_release()
    model.release(*tensors[0])
    assert pool.kv_page_pool_free_pages() == len(model.free)
    assert caches[0].tokens == 0 and caches[0].kv_cache_stats().k_bytes == 0
    B, H, Hq = shapes[1]
    K, V, q = data[1]
    n_packed, ck, cv = gpu_cases.oracle_cache(K.numpy(), V.numpy(), 0.1, 0.2, 8)
    gpu_cases.check_paged_state(caches[1], n_packed, ck, cv, B, H)
    # the released cache fills again, from the pages the model says come next
    B, H, Hq = shapes[0]
    K, V, q = data[0]
    caches[0].kv_compress_append(K[:, :64 * 5].contiguous().cuda(), V[:, :64 * 5].contiguous().cuda())
    torch.cuda.synchronize()
    for t, (name, x, rel) in enumerate((("k", K, 0.1), ("v", V, 0.2))):
        c = (oracle.compress_v if t else oracle.compress_k)(np.ascontiguousarray(x.numpy()[:, :64 * 5]), rel, 16)
        placed = model.place(tensors[0][t], np.diff(c.offsets16.astype(np.int64)).tolist())
        assert _chunk_pairs(caches[0], name, 5 * B * H) == placed, name
    n_packed, ck, cv = gpu_cases.oracle_cache(K.numpy()[:, :64 * 5], V.numpy()[:, :64 * 5])
    gpu_cases.check_paged_state(caches[0], n_packed, ck, cv, B, H)
    for c in caches:
        c.close()
    assert pool.kv_page_pool_free_pages() == n_pages
    pool.close()


def test_exhausted_pool_drops_the_call_and_keeps_its_pages():
    B, H, Hq = 1, 4, 4
    pool = binding.PagePool(3)
    model = gpu_cases.PagePlacementModel(3)
    cache = binding.PackedKVCache(B, H, Hq, 64 * 64, pool=pool)
    K, V, q = synth.make_kv(B, 64 * 64, H, Hq, 7)
    kt, vt = model.new_tensor(), model.new_tensor()
    kept = {"k": 0, "v": 0}
    dropped_at = None
    for step in range(12):  # 4 blocks per call; K needs a third page before V does
        lo, hi = 256 * step, 256 * (step + 1)
        cache.kv_compress_append(K[:, lo:hi].contiguous().cuda(), V[:, lo:hi].contiguous().cuda())
        ok = {}
        for name, t, x, rel in (("k", kt, K, 0.1), ("v", vt, V, 0.2)):
            c = (oracle.compress_k if name == "k" else oracle.compress_v)(np.ascontiguousarray(x.numpy()[:, lo:hi]), rel)
            ok[name] = model.place(t, np.diff(c.offsets16.astype(np.int64)).tolist()) is not None
            if ok[name] and dropped_at is None:
                kept[name] = hi
        if not all(ok.values()):
            dropped_at = lo
            break
    assert dropped_at is not None and dropped_at > 0, "the pool was meant to run out"
    st = cache.kv_cache_stats()
    assert st.overflow == 1
    assert pool.kv_page_pool_free_pages() == len(model.free)
    assert st.k_bytes == len(kt["pages"]) * binding.PAGE_BYTES and st.v_bytes == len(vt["pages"]) * binding.PAGE_BYTES
    # blocks of the dropped call read as zeros, earlier ones as the oracle says
    L = dropped_at + 256
    scores = cache.kv_k_matvec(q.cuda(), 1.0)
    torch.cuda.synchronize()
    n_packed, ck, cv = gpu_cases.oracle_cache(K.numpy()[:, :L], V.numpy()[:, :L])
    s_ref = oracle.k_scores(ck.codes, K.numpy()[:, :L], ck.meta, L, q.numpy(), 1.0)
    assert_close_vectors(scores[:, :, :kept["k"]].cpu().numpy(), s_ref[:, :, :kept["k"]], "kept K blocks")
    assert (scores[:, :, kept["k"]:] == 0).all()
    p = torch.softmax(scores, -1)
    out = cache.kv_v_matvec(p)
    torch.cuda.synchronize()
    pz = p.cpu().numpy().copy()
    pz[:, :, kept["v"]:] = 0
    o_ref = oracle.v_out(cv.codes, V.numpy()[:, :L], cv.meta, L, pz)
    assert_close_vectors(out.cpu().numpy(), o_ref, "V out without the dropped blocks")
    # the fused attention leaves out every block that lacks its K or its V chunk
    both = min(kept["k"], kept["v"])
    attn = cache.kv_decode_attention(q.cuda(), 0.09)
    torch.cuda.synchronize()
    a_ref = oracle.attention(ck.codes[:, :both], K.numpy()[:, :both], ck.meta[:, :both], cv.codes[:, :both],
                             V.numpy()[:, :both], cv.meta[:, :both], both, q.numpy(), 0.09)
    assert_close_vectors(attn.cpu().numpy(), a_ref, "attention over the blocks that have both chunks")
    cache.close()
    assert pool.kv_page_pool_free_pages() == 3
    pool.close()


def test_paged_host_argument_errors():
    lib = binding.lib()
    import ctypes as C
    handle = C.c_void_p()
    buf = torch.empty(4 * binding.PAGE_BYTES, dtype=torch.uint8, device="cuda:0")
    state = torch.empty(lib.kv_page_pool_state_bytes(4), dtype=torch.uint8, device="cuda:0")
    assert lib.kv_page_pool_create(None, 4, state.data_ptr(), None, C.byref(handle)) == binding.KV_ERR_ARG
    assert lib.kv_page_pool_create(buf.data_ptr(), 0, state.data_ptr(), None, C.byref(handle)) == binding.KV_ERR_ARG
    assert lib.kv_page_pool_create(buf.data_ptr(), 1 << 20, state.data_ptr(), None, C.byref(handle)) == binding.KV_ERR_ARG
    assert lib.kv_page_pool_create(buf.data_ptr() + 16, 3, state.data_ptr(), None, C.byref(handle)) == binding.KV_ERR_ARG
    cfg = binding.make_config(1, 2, 2, 256)
    sizes = binding.kv_query_sizes_paged(cfg)
    bufs = binding.kv_buffers_t()
    assert lib.kv_cache_create_paged(C.byref(cfg), None, C.byref(bufs), C.byref(sizes), C.byref(handle)) == binding.KV_ERR_ARG
    pool = binding.PagePool(4)
    # page lists missing
    assert lib.kv_cache_create_paged(C.byref(cfg), pool.handle, C.byref(bufs), C.byref(sizes),
                                     C.byref(handle)) == binding.KV_ERR_ARG
    # a contiguous cache can be emptied too
    cache = binding.PackedKVCache(1, 2, 2, 256)
    K, V, q = synth.make_kv(1, 200, 2, 2, 3)
    cache.kv_compress_append(K.cuda(), V.cuda())
    cache.kv_cache_release()
    assert cache.tokens == 0 and cache.kv_cache_stats().k_bytes == 0
    cache.kv_compress_append(K[:, :100].contiguous().cuda(), V[:, :100].contiguous().cuda())
    n_packed, ck, cv = gpu_cases.oracle_cache(K.numpy()[:, :100], V.numpy()[:, :100])
    gpu_cases.check_packed_state(cache, n_packed, ck, cv, 1, 2)
    cache.close()
    pool.close()


def test_bulk_append_placement_equals_the_rule():
    """Thousands of chunks per call (several chunks per thread of the placement kernel, many fresh
    pages per call): every chunk position equals the sequential rule's."""
    B, H, Hq = 2, 8, 8
    calls = [64 * 330, 64 * 70, 64, 64 * 99]   # 5280, 1120, 16 and 1584 chunks per tensor
    L = sum(calls)
    n_pages = 900
    pool = binding.PagePool(n_pages)
    model = gpu_cases.PagePlacementModel(n_pages)
    cache = binding.PackedKVCache(B, H, Hq, L, pool=pool)
    K, V, q = synth.make_kv(B, L, H, Hq, 31)
    tensors = (model.new_tensor(), model.new_tensor())
    expected = ([], [])
    lo = 0
    for n in calls:
        cache.kv_compress_append(K[:, lo:lo + n].contiguous().cuda(), V[:, lo:lo + n].contiguous().cuda())
        for t, (x, rel) in enumerate(((K, 0.1), (V, 0.2))):
            c = (oracle.compress_v if t else oracle.compress_k)(np.ascontiguousarray(x.numpy()[:, lo:lo + n]), rel)
            placed = model.place(tensors[t], np.diff(c.offsets16.astype(np.int64)).tolist())
            assert placed is not None
            expected[t].extend(placed)
        lo += n
    torch.cuda.synchronize()
    assert cache.kv_cache_stats().overflow == 0
    n_chunks = L // 64 * B * H
    for t, name in enumerate(("k", "v")):
        got = _chunk_pairs(cache, name, n_chunks)
        bad = [i for i in range(n_chunks) if got[i] != expected[t][i]]
        assert not bad, "%s: %d chunks misplaced, first %d: %s vs %s" % (name, len(bad), bad[0], got[bad[0]], expected[t][bad[0]])
        pages, fill = _page_list(cache, name)
        assert pages == tensors[t]["pages"] and fill == tensors[t]["fill"]
    assert pool.kv_page_pool_free_pages() == len(model.free)
    cache.close()
    pool.close()


def test_smallest_chunks_fill_pages_exactly():
    """Constant tensors give header-only chunks of 512 bytes: 128 of them fill a page to the last
    byte, the most chunks a page can hold (the placement kernel's per-page chunk count is at its
    limit) and a fill level that reaches the page size exactly."""
    B, H, Hq, L = 1, 2, 2, 64 * 200
    pool = binding.PagePool(12)
    model = gpu_cases.PagePlacementModel(12)
    cache = binding.PackedKVCache(B, H, Hq, L, pool=pool)
    K = torch.full((B, L, H, 128), 0.5, dtype=torch.float16)
    V = torch.zeros((B, L, H, 128), dtype=torch.float16)
    tensors = (model.new_tensor(), model.new_tensor())
    expected = ([], [])
    lo = 0
    for n in (64 * 70, 64 * 58, 64 * 72):   # 140, 116 and 144 chunks per tensor: page boundaries inside and at call ends
        cache.kv_compress_append(K[:, lo:lo + n].contiguous().cuda(), V[:, lo:lo + n].contiguous().cuda())
        for t in range(2):
            placed = model.place(tensors[t], [32] * (n // 64 * B * H))
            assert placed is not None
            expected[t].extend(placed)
        lo += n
    torch.cuda.synchronize()
    n_chunks = L // 64 * B * H
    for t, name in enumerate(("k", "v")):
        assert _chunk_pairs(cache, name, n_chunks) == expected[t], name
        pages, fill = _page_list(cache, name)
        assert pages == tensors[t]["pages"] and fill == tensors[t]["fill"]
    assert 128 in [len([1 for s, e in expected[0] if s // PAGE16 == p]) for p in tensors[0]["pages"]]
    n_packed, ck, cv = gpu_cases.oracle_cache(K.numpy(), V.numpy())
    gpu_cases.check_paged_state(cache, n_packed, ck, cv, B, H)
    q = torch.ones((B, Hq, 128), dtype=torch.float16)
    attn = cache.kv_decode_attention(q.cuda(), 0.1)
    torch.cuda.synchronize()
    assert_close_vectors(attn.cpu().numpy(), np.zeros((B, Hq, 128)) + V.numpy()[0, 0, 0, 0], "attention over constant V")
    cache.close()
    pool.close()
