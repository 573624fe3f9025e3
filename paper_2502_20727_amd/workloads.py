"""Named synthetic workloads: LLaMA2-shaped per-rank shards and their SPD masks.

Each workload fixes the shapes, the tensor-parallel degree, the per-layer SPD mask
(1 = the sync point after the attention output is dropped, Sec. 4 / Alg. 1 marks such
blocks "SPD"), the seed and the call shape (batch, q_len, context).  Nothing here
computes anything of the method; it is the recipe the input generators follow.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Tuple

F32 = 0
BF16 = 1


@dataclass(frozen=True)
class Workload:
    name: str
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    n_layers: int
    tp: int
    dtype: int            # F32 | BF16 (weights, KV cache, inter-kernel activations)
    seed: int
    batch: int
    q_len: int            # tokens per sequence in the timed / checked call
    ctx: int              # keys attended by the last query token of the call
    mask: Tuple[int, ...] = field(default=())
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    note: str = ""

    @property
    def q_per_rank(self) -> int:
        return self.n_q_heads // self.tp

    @property
    def kv_per_rank(self) -> int:
        return self.n_kv_heads // self.tp

    @property
    def ffn_per_rank(self) -> int:
        return self.ffn // self.tp

    @property
    def tokens(self) -> int:
        return self.batch * self.q_len

    def with_mask(self, mask) -> "Workload":
        return replace(self, mask=tuple(int(m) for m in mask))

    def with_layers(self, n_layers: int) -> "Workload":
        return replace(self, n_layers=n_layers, mask=tuple(self.mask[:n_layers]))


def _all(n):
    return tuple([1] * n)


TOY = Workload(
    name="toy-f32", hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn=688,
    n_layers=2, tp=2, dtype=F32, seed=0, batch=1, q_len=32, ctx=32, mask=(1, 0),
    note="prefill of 32 tokens then 8 single-token steps; all ranks emulated")

LLAMA7B_DECODE = Workload(
    name="llama2-7b-tp8-decode-b1-ctx2048", hidden=4096, n_q_heads=32, n_kv_heads=32,
    head_dim=128, ffn=11008, n_layers=32, tp=8, dtype=BF16, seed=1, batch=1, q_len=1,
    ctx=2048, mask=_all(32), note="rank 0, every layer SPD")

LLAMA13B_DECODE = Workload(
    name="llama2-13b-tp8-decode-b8-ctx4096", hidden=5120, n_q_heads=40, n_kv_heads=40,
    head_dim=128, ffn=13824, n_layers=40, tp=8, dtype=BF16, seed=2, batch=8, q_len=1,
    ctx=4096, mask=tuple(0 if l % 4 == 3 else 1 for l in range(40)),
    note="rank 0, every 4th layer keeps its attention sync point")

LLAMA70B_DECODE = Workload(
    name="llama2-70b-tp8-decode-b16-ctx4096", hidden=8192, n_q_heads=64, n_kv_heads=8,
    head_dim=128, ffn=28672, n_layers=80, tp=8, dtype=BF16, seed=3, batch=16, q_len=1,
    ctx=4096, mask=tuple(1 if 8 <= l < 72 else 0 for l in range(80)),
    note="rank 0, SPD on all but the first 8 and last 8 layers")

LLAMA70B_PREFILL = Workload(
    name="llama2-70b-tp8-prefill-b4x2048", hidden=8192, n_q_heads=64, n_kv_heads=8,
    head_dim=128, ffn=28672, n_layers=80, tp=8, dtype=BF16, seed=4, batch=4, q_len=2048,
    ctx=2048, mask=_all(80), note="rank 0, causal prefill, every layer SPD")

# the shape the paper quotes its latency breakdown on (Fig. 2: one sequence of 128 tokens), and the
# 4-way shards of the two smaller models (Sec. 5 runs them on 4 as well as 8 devices)
LLAMA70B_PREFILL_128 = Workload(
    name="llama2-70b-tp8-prefill-b1x128", hidden=8192, n_q_heads=64, n_kv_heads=8,
    head_dim=128, ffn=28672, n_layers=80, tp=8, dtype=BF16, seed=5, batch=1, q_len=128,
    ctx=128, mask=_all(80), note="rank 0, one sequence of 128 tokens, every layer SPD")

LLAMA7B_TP4_DECODE = Workload(
    name="llama2-7b-tp4-decode-b1-ctx2048", hidden=4096, n_q_heads=32, n_kv_heads=32,
    head_dim=128, ffn=11008, n_layers=32, tp=4, dtype=BF16, seed=6, batch=1, q_len=1,
    ctx=2048, mask=_all(32), note="rank 0 of 4, every layer SPD")

LLAMA13B_TP4_DECODE = Workload(
    name="llama2-13b-tp4-decode-b8-ctx4096", hidden=5120, n_q_heads=40, n_kv_heads=40,
    head_dim=128, ffn=13824, n_layers=40, tp=4, dtype=BF16, seed=7, batch=8, q_len=1,
    ctx=4096, mask=tuple(0 if l % 4 == 3 else 1 for l in range(40)),
    note="rank 0 of 4, every 4th layer keeps its attention sync point")

WORKLOADS = {w.name: w for w in
             (TOY, LLAMA7B_DECODE, LLAMA13B_DECODE, LLAMA70B_DECODE, LLAMA70B_PREFILL, LLAMA70B_PREFILL_128,
              LLAMA7B_TP4_DECODE, LLAMA13B_TP4_DECODE)}
ALIASES = {"toy": TOY, "7b-decode": LLAMA7B_DECODE, "13b-decode": LLAMA13B_DECODE,
           "70b-decode": LLAMA70B_DECODE, "70b-prefill": LLAMA70B_PREFILL, "70b-prefill-128": LLAMA70B_PREFILL_128,
           "7b-tp4-decode": LLAMA7B_TP4_DECODE, "13b-tp4-decode": LLAMA13B_TP4_DECODE}


def get(name: str) -> Workload:
    if name in WORKLOADS:
        return WORKLOADS[name]
    if name in ALIASES:
        return ALIASES[name]
    raise KeyError(f"unknown workload {name!r}; known: {sorted(ALIASES)}")
