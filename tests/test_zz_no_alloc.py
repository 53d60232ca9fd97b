"""GPU test of kv_v_matvec_noalloc, the V product for callers that cannot allocate.

Two calls in a row through the C ABI, the second on a smaller cache, each compared with
kv_v_matvec on the same inputs (bitwise: same kernels, same split count at these sizes) and
with the CPU oracle at the bar of the parity tests.  The file name sorts last on purpose.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_24449_amd import binding, synth
from tests import gpu_cases

pytestmark = pytest.mark.gpu


def _one_call(batch, n_kv, n_q, tokens, seed):
    K, V, q = synth.make_kv(batch, tokens, n_kv, n_q, seed)
    cache = binding.PackedKVCache(batch, n_kv, n_q, tokens)
    cache.kv_compress_append(K.cuda(), V.cuda())
    gen = torch.Generator().manual_seed(seed)
    p = torch.softmax(4.0 * torch.randn(batch, n_q, tokens, generator=gen), dim=-1)
    p_dev = p.cuda()
    want = cache.kv_v_matvec(p_dev)
    out = torch.full((batch, n_q, synth.HEAD_DIM), float("nan"), dtype=torch.float32, device="cuda:0")
    mem_before = torch.cuda.memory_allocated()
    cache.kv_v_matvec_noalloc(p_dev, out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == mem_before
    assert torch.equal(out, want), "no-alloc entry point differs from kv_v_matvec"
    # and against the oracle, like every other V result
    n_packed, _, cv = gpu_cases.oracle_cache(K.numpy(), V.numpy())
    codes, meta = gpu_cases.full_codes(cv, tuple(V.shape), n_packed)
    ref = oracle.v_out(codes, V.numpy(), meta, n_packed, p.numpy())
    gpu_cases.assert_close_vectors(out.cpu().numpy(), ref, "kv_v_matvec_noalloc")
    cache.close()


def test_no_alloc_two_calls_second_smaller():
    binding.lib()
    _one_call(2, 4, 8, 37 * 64 + 29, seed=901)   # several splits, grouped queries, raw tail
    _one_call(1, 2, 2, 3 * 64 + 5, seed=902)     # smaller: fewer rows, fewer splits than the array last held


def test_no_alloc_rejects_too_many_rows():
    binding.lib()
    rows = binding.lib().kv_v_matvec_noalloc  # symbol present
    assert rows is not None
    # batch * n_q_heads above the array's row count: a clear error, nothing launched
    batch, n_kv, n_q = 130, 8, 64
    assert batch * n_q > 8192
    cache = binding.PackedKVCache(batch, n_kv, n_q, 64)
    p = torch.zeros(batch, n_q, 64, dtype=torch.float32, device="cuda:0")
    out = torch.zeros(batch, n_q, synth.HEAD_DIM, dtype=torch.float32, device="cuda:0")
    with pytest.raises(binding.PackKVError) as err:
        cache.kv_v_matvec_noalloc(p, out)
    assert err.value.code == binding.KV_ERR_CAPACITY
    cache.close()
