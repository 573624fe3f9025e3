"""Seeded synthetic inputs shared (as data) by the CPU oracle and the HIP path.

Every tensor is a pure function of (seed, tensor id, layer, rank, element index), so a
single layer, a single rank's shard or a slice of a tensor can be regenerated on its own.
No arithmetic of the method lives here: only normal deviates, an optional rounding of the
values to bf16-representable fp32, and concatenation of per-rank shards into the dense
matrices they are slices of (Sec. 4.1: Q/K/V are split by columns, the attention output
and MLP down projections by rows).

Recipe (the paper's LLaMA2 weights and calibration text are replaced by synthetic data of
the same shapes): linear weights N(0, 0.02); norm gains 1 + N(0, 0.02); hidden states and
pre-filled KV cache N(0, 1); peer partial sums 0.05 * N(0, 1).
"""
from __future__ import annotations

import ctypes
from typing import Dict, Optional

import numpy as np

from . import build
from .workloads import BF16, Workload

# tensor ids (part of the generator key)
T_WQ, T_WK, T_WV, T_WO, T_WG, T_WU, T_WD, T_G1, T_G2 = range(1, 10)
T_X, T_KCACHE, T_VCACHE, T_SLOTS, T_MISC = range(10, 15)
T_BO = 15

_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        lib = ctypes.CDLL(build.ensure_inputs())
        lib.spd_inputs_key.restype = ctypes.c_uint64
        lib.spd_inputs_key.argtypes = [ctypes.c_uint64] * 4
        lib.spd_inputs_normal.restype = None
        lib.spd_inputs_normal.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64,
                                          ctypes.c_uint64, ctypes.c_float, ctypes.c_float,
                                          ctypes.c_int]
        _LIB = lib
    return _LIB


def normal(shape, seed: int, tensor: int, layer: int = 0, rank: int = 0, *, mean: float = 0.0,
           std: float = 1.0, bf16: bool = False, first: int = 0,
           out: Optional[np.ndarray] = None) -> np.ndarray:
    """fp32 array of `shape` filled with mean + std * N(0,1), element i drawing deviate first+i."""
    n = int(np.prod(shape))
    if out is None:
        out = np.empty(shape, dtype=np.float32)
    else:
        assert out.dtype == np.float32 and out.size == n and out.flags.c_contiguous
        out = out.reshape(shape)
    lib = _lib()
    key = lib.spd_inputs_key(seed, tensor, layer, rank)
    lib.spd_inputs_normal(out.ctypes.data, n, key, first, mean, std, 1 if bf16 else 0)
    return out


def layer_shard(w: Workload, layer: int, rank: int) -> Dict[str, np.ndarray]:
    """Rank `rank`'s slices of layer `layer` in the x @ W convention.

    wq [h, q*d], wk/wv [h, kv*d] (columns = the rank's heads), wo [q*d, h] (rows = the
    rank's heads), wg/wu [h, f] (columns = the rank's FFN slice), wd [f, h], g1/g2 [h]
    (replicated: the gains are drawn with rank 0's key for every rank).
    """
    h, d = w.hidden, w.head_dim
    q, kv, f = w.q_per_rank, w.kv_per_rank, w.ffn_per_rank
    b = w.dtype == BF16
    s = w.seed
    return {
        "wq": normal((h, q * d), s, T_WQ, layer, rank, std=0.02, bf16=b),
        "wk": normal((h, kv * d), s, T_WK, layer, rank, std=0.02, bf16=b),
        "wv": normal((h, kv * d), s, T_WV, layer, rank, std=0.02, bf16=b),
        "wo": normal((q * d, h), s, T_WO, layer, rank, std=0.02, bf16=b),
        "wg": normal((h, f), s, T_WG, layer, rank, std=0.02, bf16=b),
        "wu": normal((h, f), s, T_WU, layer, rank, std=0.02, bf16=b),
        "wd": normal((f, h), s, T_WD, layer, rank, std=0.02, bf16=b),
        "g1": normal((h,), s, T_G1, layer, 0, mean=1.0, std=0.02),
        "g2": normal((h,), s, T_G2, layer, 0, mean=1.0, std=0.02),
    }


def output_bias(w: Workload, layer: int, std: float = 0.5) -> np.ndarray:
    """[hidden] bias of the attention output projection for the block-with-bias variant (fp32, the same on every rank)."""
    return normal((w.hidden,), w.seed, T_BO, layer, 0, std=std)


def dense_layer(w: Workload, layer: int) -> Dict[str, np.ndarray]:
    """The unsharded layer whose contiguous slices are the ranks' shards."""
    shards = [layer_shard(w, layer, r) for r in range(w.tp)]
    out = {}
    for name in ("wq", "wk", "wv", "wg", "wu"):
        out[name] = np.ascontiguousarray(np.concatenate([s[name] for s in shards], axis=1))
    for name in ("wo", "wd"):
        out[name] = np.ascontiguousarray(np.concatenate([s[name] for s in shards], axis=0))
    out["g1"] = shards[0]["g1"]
    out["g2"] = shards[0]["g2"]
    return out


def hidden_states(w: Workload, n_tokens: int, first_token: int = 0) -> np.ndarray:
    """[n_tokens, hidden] N(0,1) block inputs; row t is the same whatever slice is asked for."""
    return normal((n_tokens, w.hidden), w.seed, T_X, first=first_token * w.hidden)


def kv_prefill(w: Workload, layer: int, rank: int, batch: int, n_pos: int):
    """Pre-filled cache content in natural layout: k, v of shape [batch, kv, n_pos, d].

    The keys are taken as already rotated; values are N(0,1), bf16-representable when the
    workload's dtype is bf16.
    """
    shape = (batch, w.kv_per_rank, n_pos, w.head_dim)
    b = w.dtype == BF16
    k = normal(shape, w.seed, T_KCACHE, layer, rank, bf16=b)
    v = normal(shape, w.seed, T_VCACHE, layer, rank, bf16=b)
    return k, v


def peer_slots(w: Workload, n_tokens: int) -> np.ndarray:
    """[tp, n_tokens, hidden] stand-ins for the partial sums the other ranks would deliver."""
    return normal((w.tp, n_tokens, w.hidden), w.seed, T_SLOTS, std=0.05)
