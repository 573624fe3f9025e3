"""Shared set-up for the GPU parity tests: the same seeded inputs go to the HIP library (through
the C ABI binding) and to the CPU oracle; nothing computed by one side is fed to the other
except a layer's *input* when blocks are checked one at a time."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

from oracle import spd_oracle as O
from paper_2502_20727_amd import binding as B
from paper_2502_20727_amd import inputs
from paper_2502_20727_amd.workloads import BF16, Workload


def oracle_shapes(w: Workload) -> O.Shapes:
    return O.Shapes(w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn, w.tp, w.rms_eps, w.rope_base)


def cache_storage(w: Workload) -> str:
    """The KV cache of a bf16 workload holds bf16 values; the fp32 toy's holds what it is given."""
    return "bf16" if w.dtype == BF16 else "f64"


def tolerance(w: Workload) -> dict:
    """bf16 path: max abs error 2e-2 on fp32-stored outputs; fp32 path: 1e-3 relative to the
    largest oracle magnitude."""
    return dict(kind="abs", tol=2e-2) if w.dtype == BF16 else dict(kind="rel", tol=1e-3)


def assert_close(got: np.ndarray, want: np.ndarray, w: Workload, what: str, scale: float = 1.0):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    err = float(np.max(np.abs(got - want))) if got.size else 0.0
    t = tolerance(w)
    bound = t["tol"] * scale if t["kind"] == "abs" else t["tol"] * max(float(np.max(np.abs(want))), 1e-30)
    assert err <= bound, f"{what}: max abs err {err:.3e} > {bound:.3e} (max |oracle| {np.max(np.abs(want)):.3e})"
    return err


class Case:
    """One workload on the GPU and in the oracle, for the ranks asked for."""

    def __init__(self, w: Workload, device, ranks: Sequence[int], positions: Sequence[int],
                 layer_ids: Optional[Sequence[int]] = None, max_ctx: Optional[int] = None,
                 max_tokens: Optional[int] = None, prefill_layers: bool = True, act_split: int = 0,
                 bias_std: float = 0.0):
        import torch
        self.torch = torch
        self.w = w
        self.sh = oracle_shapes(w)
        self.ranks = list(ranks)
        self.positions = [int(p) for p in positions]
        self.layer_ids = list(layer_ids) if layer_ids is not None else list(range(w.n_layers))
        assert len(self.layer_ids) == w.n_layers
        self.dev = B.DeviceShard(w, self.ranks, device, max_ctx=max_ctx, max_tokens=max_tokens,
                                 max_batch=len(self.positions), act_split=act_split, o_bias=1 if bias_std else 0)
        mc = self.dev.cfg.max_ctx
        self.shards: List[List[dict]] = []
        self.caches: List[List[O.KVCache]] = []
        batch = len(self.positions)
        n_pre = max(self.positions) if self.positions else 0
        for li, layer in enumerate(self.layer_ids):
            sh = [inputs.layer_shard(w, layer, r) for r in self.ranks]
            if bias_std:     # block with bias: the same output-projection bias on every rank
                bo = inputs.output_bias(w, layer, bias_std)
                for d in sh:
                    d["bo"] = bo
            self.shards.append(sh)
            self.dev.load_layer(li, sh)
            caches, kvs = [], []
            for r in self.ranks:
                c = O.KVCache(batch, w.kv_per_rank, mc, w.head_dim, storage=cache_storage(w))
                if n_pre > 0 and prefill_layers:
                    k, v = inputs.kv_prefill(w, layer, r, batch, n_pre)
                    # every sequence only keeps its own prefix; the rest stays zero on both sides
                    for b, p in enumerate(self.positions):
                        k[b, :, p:, :] = 0.0
                        v[b, :, p:, :] = 0.0
                    c.fill(k, v)
                    kvs.append((k, v))
                caches.append(c)
            if kvs:
                self.dev.load_kv(li, kvs)
            self.caches.append(caches)

    def to_dev(self, a: np.ndarray):
        return self.torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.dev.device)

    def close(self):
        self.dev.close()
