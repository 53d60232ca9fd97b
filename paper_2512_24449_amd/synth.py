"""Seeded synthetic inputs shaped like the workloads of the PackKV evaluation.

This module holds no arithmetic of the method: it only draws random tensors.
Both the HIP tests/benchmarks and the CPU oracle tests take their inputs from
here, so the two sides always see the same bytes.

The paper measures on KV tensors collected from model inference (Sec. IV-E);
those are not available, so the stand-in is: K ~ N(0,1) with 4 fixed outlier
channels per kv-head scaled by 10 (the channel structure the paper shows for K
in Sec. III-A), V ~ N(0,1), query ~ N(0,1), all rounded to fp16.
Layout is the paper's cache layout [context_len, head_num, head_dim] with a
leading batch axis: [B, L, H_kv, D].
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

HEAD_DIM = 128
BLOCK_TOKENS = 64
SEED_BASE = 20251224


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_kv_heads: int
    n_q_heads: int
    tokens: int
    decode_steps: int = 0     # growing-cache stress only

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def elements(self) -> int:
        return self.batch * self.tokens * self.n_kv_heads * HEAD_DIM


# The five configurations of the benchmark definition, in its order.
WORKLOADS = (
    Workload("single_head_1k", 1, 1, 1, 1024),
    Workload("llama2_7b_4k", 1, 32, 32, 4096),
    Workload("llama3_8b_gqa_32k_b4", 4, 8, 32, 32768),
    Workload("llama2_30b_32k_b8", 8, 52, 52, 32000),
    Workload("llama3_8b_grow_128k", 1, 8, 32, 131072, 1024),
)


def workload(index_or_name) -> Workload:
    if isinstance(index_or_name, int):
        return WORKLOADS[index_or_name]
    for w in WORKLOADS:
        if w.name == index_or_name:
            return w
    raise KeyError(index_or_name)


def make_kv(batch, tokens, n_kv_heads, n_q_heads, seed, device="cpu", outliers=True):
    """Return (K, V, q): fp16 [B, L, H, D], fp16 [B, L, H, D], fp16 [B, Hq, D].

    Generated one batch element at a time in fp32 so that the largest
    configuration never holds more than one fp32 slice.
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(SEED_BASE + int(seed))
    cpu_gen = torch.Generator()
    cpu_gen.manual_seed(SEED_BASE + int(seed))
    # outlier channels: fixed over tokens and batch, drawn per kv-head
    idx = torch.stack([torch.randperm(HEAD_DIM, generator=cpu_gen)[:4] for _ in range(n_kv_heads)])
    gain = torch.ones(n_kv_heads, HEAD_DIM)
    if outliers:
        gain.scatter_(1, idx, 10.0)
    gain = gain.to(dev)
    K = torch.empty(batch, tokens, n_kv_heads, HEAD_DIM, dtype=torch.float16, device=dev)
    V = torch.empty_like(K)
    for b in range(batch):
        k32 = torch.randn(tokens, n_kv_heads, HEAD_DIM, generator=gen, device=dev)
        K[b] = (k32 * gain).to(torch.float16)
        del k32
        v32 = torch.randn(tokens, n_kv_heads, HEAD_DIM, generator=gen, device=dev)
        V[b] = v32.to(torch.float16)
        del v32
    q = torch.randn(batch, n_q_heads, HEAD_DIM, generator=gen, device=dev).to(torch.float16)
    return K, V, q


def make_workload(w: Workload, device="cpu", tokens=None):
    """Inputs for one of the benchmark configurations (optionally fewer tokens)."""
    return make_kv(w.batch, tokens if tokens is not None else w.tokens, w.n_kv_heads,
                   w.n_q_heads, WORKLOADS.index(w), device=device)


def make_probs(scores: torch.Tensor) -> torch.Tensor:
    """fp32 softmax weights from fp32 scores -- the p the V path is given."""
    return torch.softmax(scores.float(), dim=-1)
