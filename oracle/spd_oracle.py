"""CPU oracle for the Sync-Point-Drop (SPD) decoder block.  TEST INFRASTRUCTURE ONLY.

Only `tests/`, the smoke check and the bench's `cpu_baseline` leg may import this module;
the product (the HIP library and its binding) never does, and this module imports nothing
from the product.  It is slow on purpose: plain NumPy in float64, one step per line, in
the order and notation of the paper, no blocking, fusion or reordering.

What it computes (arXiv 2502.20727):

* Tensor parallelism splits a decoder block over `tp` devices: query/key/value
  projections by columns (each device owns N/tp whole heads, Sec. 4.2.3 "head
  scattering": n(A_i) = N / number_of_devices), the attention output projection by rows
  (Sec. 4.1.2), the MLP likewise.  Device i therefore produces a *partial* attention
  output Y_i and a partial MLP output Z_i; a TP block all-reduces each of them (two
  sync points per block, Sec. 3, Fig. 1a) and equals single-device inference.
* An SPD block (Sec. 4.1.1, Fig. 3a, block without bias) drops the first all-reduce:
  device i feeds X + Y_i to its MLP, adds Y_i to its MLP partial *before* the remaining
  all-reduce and adds X *after* it, so the block output is X + sum_i Y_i + sum_i Z_i
  with Z_i = MLP_i(X + Y_i).
* Which blocks are SPD blocks is a per-layer boolean (the outcome of Alg. 1); here it is
  an input: mask[l] = 1 means block l drops its attention sync point.

The paper says "LLaMA2" and nothing more about the block's inside, so the standard
LLaMA block is taken: pre-norm RMSNorm (eps inside the square root), rotary embedding in
the rotate-half convention (pair (j, j + d/2), angle pos * base^(-2j/d)) applied to
queries and keys, causal softmax attention scaled by 1/sqrt(d) with grouped KV heads
(query head j uses KV head j // (q_heads / kv_heads)), SwiGLU MLP
(silu(x Wg) * (x Wu)) Wd, silu(x) = x / (1 + exp(-x)).  The second norm of an SPD block
acts on X + Y_i (that sum is "fed into MLP input").

The all-reduce is a plain sum over ranks (float64 here, so the order is immaterial).
Parity status: every function below is pinned by tests/test_oracle_pins.py (dense-block
equality with SPD off, tp = 1 identity, closed forms, an independent scalar brute force).
The paper prints no worked numeric example of a block output, and its perplexities
(Table 1) need trained weights and a text corpus: those are parity unpinned.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np

F64 = np.float64


@dataclass(frozen=True)
class Shapes:
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    tp: int = 1
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    @property
    def q(self) -> int:          # query heads per device, n(A_i) = N / number_of_devices
        assert self.n_q_heads % self.tp == 0
        return self.n_q_heads // self.tp

    @property
    def kv(self) -> int:
        assert self.n_kv_heads % self.tp == 0
        return self.n_kv_heads // self.tp

    @property
    def f(self) -> int:
        assert self.ffn % self.tp == 0
        return self.ffn // self.tp


# --------------------------------------------------------------------------- elementary steps

def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """y = x / sqrt(mean_h(x^2) + eps) * g, row by row."""
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, F64)


def rope(v: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotate-half rotary embedding.  v: [T, heads, d]; pos: [T] integer positions.

    For j < d/2 the pair (v[j], v[j + d/2]) is rotated by the angle pos * base^(-2j/d).
    """
    v = np.asarray(v, F64)
    T, H, d = v.shape
    half = d // 2
    j = np.arange(half, dtype=F64)
    theta = base ** (-2.0 * j / d)                       # [d/2]
    ang = np.asarray(pos, F64)[:, None] * theta[None, :]  # [T, d/2]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    lo, hi = v[..., :half], v[..., half:]
    out = np.empty_like(v)
    out[..., :half] = lo * c - hi * s
    out[..., half:] = hi * c + lo * s
    return out


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def token_positions(positions: Sequence[int], batch: int, q_len: int) -> np.ndarray:
    """Token b*q_len + t of the call sits at position positions[b] + t of sequence b."""
    positions = np.asarray(positions, dtype=np.int64)
    assert positions.shape == (batch,)
    return (positions[:, None] + np.arange(q_len, dtype=np.int64)[None, :]).reshape(-1)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 value (ties to even) of every element, returned as float64."""
    f = np.asarray(a, np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(F64).reshape(np.shape(a))


class KVCache:
    """One device's keys and values of one layer: [batch, kv_heads, max_ctx, d] float64.

    `storage` is the number format the cache is defined to hold.  A bf16 cache stores bf16
    values: keys and values are rounded once, when they are stored, and every later use
    reads the stored value (all arithmetic stays float64).  This is a property of the data
    structure the workload names, not of any implementation of it.
    """

    def __init__(self, batch: int, kv_heads: int, max_ctx: int, head_dim: int, storage: str = "f64"):
        assert storage in ("f64", "bf16")
        self.storage = storage
        self.k = np.zeros((batch, kv_heads, max_ctx, head_dim), F64)
        self.v = np.zeros((batch, kv_heads, max_ctx, head_dim), F64)

    def store(self, b: int, pos: int, k: np.ndarray, v: np.ndarray) -> None:
        """Append one token's keys and values [kv_heads, d] at position `pos` of sequence b."""
        if self.storage == "bf16":
            k, v = round_to_bf16(k), round_to_bf16(v)
        self.k[b, :, pos, :] = k
        self.v[b, :, pos, :] = v

    def fill(self, k: np.ndarray, v: np.ndarray) -> None:
        """Load positions [0, n) from natural-layout arrays [batch, kv, n, d]."""
        n = k.shape[2]
        self.k[:, :, :n, :] = k
        self.v[:, :, :n, :] = v

    def copy(self) -> "KVCache":
        c = KVCache.__new__(KVCache)
        c.storage = self.storage
        c.k = self.k.copy()
        c.v = self.v.copy()
        return c


# --------------------------------------------------------------------------- one device's share

def attention_partial(sh: Shapes, X: np.ndarray, W: Dict[str, np.ndarray], cache: KVCache,
                      positions: Sequence[int], batch: int, q_len: int,
                      rows: Optional[np.ndarray] = None, detail: Optional[dict] = None) -> np.ndarray:
    """Device i's partial attention output Y_i  [tokens, hidden]  (or only `rows` of it).

    W holds the device's slices: wq [h, q*d], wk/wv [h, kv*d] (column-wise split),
    wo [q*d, h] (row-wise split), g1 [h].  Keys and values of every token of the call are
    appended to `cache` at their positions before any query looks at it.
    """
    d, q, kv = sh.head_dim, sh.q, sh.kv
    group = q // kv
    T = batch * q_len
    X = np.asarray(X, F64)
    assert X.shape == (T, sh.hidden)
    pos = token_positions(positions, batch, q_len)

    n = rmsnorm(X, W["g1"], sh.rms_eps)
    K = rope((n @ np.asarray(W["wk"], F64)).reshape(T, kv, d), pos, sh.rope_base)
    V = (n @ np.asarray(W["wv"], F64)).reshape(T, kv, d)
    for t in range(T):
        b = t // q_len
        cache.store(b, int(pos[t]), K[t], V[t])

    sel = np.arange(T) if rows is None else np.asarray(rows, dtype=np.int64)
    Q = rope((n[sel] @ np.asarray(W["wq"], F64)).reshape(len(sel), q, d), pos[sel], sh.rope_base)

    A = np.zeros((len(sel), q, d), F64)
    for i, t in enumerate(sel):
        b = t // q_len
        n_keys = int(pos[t]) + 1                       # causal: key position <= query position
        for j in range(q):
            kh = j // group                            # grouped KV heads
            s = cache.k[b, kh, :n_keys, :] @ Q[i, j] / np.sqrt(d)
            p = np.exp(s - np.max(s))
            p = p / np.sum(p)
            A[i, j] = p @ cache.v[b, kh, :n_keys, :]
    if detail is not None:          # intermediates, for tests that look inside the block
        detail.update(Q=Q.reshape(len(sel), q * d), A=A.reshape(len(sel), q * d))
    return A.reshape(len(sel), q * d) @ np.asarray(W["wo"], F64)


def mlp_partial(sh: Shapes, R: np.ndarray, W: Dict[str, np.ndarray],
                detail: Optional[dict] = None) -> np.ndarray:
    """Device i's partial MLP output Z_i = (silu(m Wg_i) * (m Wu_i)) Wd_i with m = RMSNorm(R)."""
    m = rmsnorm(R, W["g2"], sh.rms_eps)
    u = silu(m @ np.asarray(W["wg"], F64)) * (m @ np.asarray(W["wu"], F64))
    if detail is not None:
        detail.update(U=u)
    return u @ np.asarray(W["wd"], F64)


# --------------------------------------------------------------------------- whole blocks

def output_bias(shard: Dict[str, np.ndarray], hidden: int) -> np.ndarray:
    """The bias b of the attention output projection, zero for a block without bias."""
    b = shard.get("bo")
    return np.zeros(hidden, F64) if b is None else np.asarray(b, F64)


def block_all_ranks(sh: Shapes, X: np.ndarray, shards: List[Dict[str, np.ndarray]],
                    caches: List[KVCache], positions: Sequence[int], batch: int, q_len: int,
                    spd: int, detail: Optional[dict] = None):
    """One decoder block with every device emulated.  Returns (X', number of sync points).

    spd = 0: TP block, two all-reduces (Sec. 3).  spd = 1: SPD block (Sec. 4.1.1): MLP input
    X + Y_i, Y_i added before the one remaining all-reduce, X after.  A shard may carry "bo", the
    bias of the output projection (replicated, it cannot be split along the rows of W_O): the
    block with bias of Sec. 4.1.2.
    """
    X = np.asarray(X, F64)
    # P_i: the device's partial weight multiplication of the output projection (no bias in it)
    Y = [attention_partial(sh, X, shards[i], caches[i], positions, batch, q_len)
         for i in range(sh.tp)]
    b = output_bias(shards[0], sh.hidden)
    if spd:
        # with bias (Sec. 4.1.2): MLP input X + P_i + b; P_i joins before the sync, b once after it
        Z = [mlp_partial(sh, X + Y[i] + b, shards[i]) for i in range(sh.tp)]
        P = [Y[i] + Z[i] for i in range(sh.tp)]          # Y_i goes in before the sync
        out = X + sum(P) + b                             # X (and the bias) after it
        syncs = 1
    else:
        R = X + sum(Y) + b                               # sync point after attention, then the bias once
        Z = [mlp_partial(sh, R, shards[i]) for i in range(sh.tp)]
        P = Z
        out = R + sum(Z)                                 # sync point after the MLP
        syncs = 2
    if detail is not None:
        detail.update(Y=Y, Z=Z, P=P)
    return out, syncs


def block_single_rank(sh: Shapes, X: np.ndarray, shard: Dict[str, np.ndarray], cache: KVCache,
                      positions: Sequence[int], batch: int, q_len: int, spd: int, rank: int,
                      slots: np.ndarray, rows: Optional[np.ndarray] = None,
                      detail: Optional[dict] = None) -> np.ndarray:
    """The same block seen from one device: the other devices' partial sums are inputs.

    `slots` [tp, tokens, hidden] float64 holds what the peers deliver at a sync point;
    slot `rank` is overwritten with this device's own partial (twice in a TP block, whose
    two sync points reuse the peers' buffers).  Returns X' (rows `rows` only if given).
    """
    X = np.asarray(X, F64)
    sel = np.arange(X.shape[0]) if rows is None else np.asarray(rows, dtype=np.int64)
    S = np.array(slots[:, sel], dtype=F64)                 # the partial sums met at a sync point
    Y = attention_partial(sh, X, shard, cache, positions, batch, q_len, rows=rows, detail=detail)
    b = output_bias(shard, sh.hidden)
    if spd:
        Z = mlp_partial(sh, X[sel] + Y + b, shard, detail)
        S[rank] = Y + Z
        out = X[sel] + np.sum(S, axis=0) + b
    else:
        S[rank] = Y
        R = X[sel] + np.sum(S, axis=0) + b
        Z = mlp_partial(sh, R, shard, detail)
        S[rank] = Z
        out = R + np.sum(S, axis=0)
    slots[rank, sel] = S[rank]
    if detail is not None:
        detail.update(Y=Y, Z=Z)
    return out


def dense_block(sh: Shapes, X: np.ndarray, dense: Dict[str, np.ndarray], cache: KVCache,
                positions: Sequence[int], batch: int, q_len: int) -> np.ndarray:
    """Single-device inference of the block: no sharding at all."""
    one = Shapes(sh.hidden, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.ffn, 1,
                 sh.rms_eps, sh.rope_base)
    X = np.asarray(X, F64)
    R = X + attention_partial(one, X, dense, cache, positions, batch, q_len) + output_bias(dense, sh.hidden)
    return R + mlp_partial(one, R, dense)


# --------------------------------------------------------------------------- whole models

def model_all_ranks(sh: Shapes, X: np.ndarray, layers: List[List[Dict[str, np.ndarray]]],
                    caches: List[List[KVCache]], positions: Sequence[int], batch: int,
                    q_len: int, mask: Sequence[int]):
    """Run the blocks in order; mask[l] = 1 makes block l an SPD block.  Returns (X', syncs)."""
    total = 0
    for l, shards in enumerate(layers):
        X, s = block_all_ranks(sh, X, shards, caches[l], positions, batch, q_len, int(mask[l]))
        total += s
    return X, total


def model_single_rank(sh: Shapes, X: np.ndarray, layers: List[Dict[str, np.ndarray]],
                      caches: List[KVCache], positions: Sequence[int], batch: int, q_len: int,
                      mask: Sequence[int], rank: int, slots: np.ndarray) -> np.ndarray:
    for l, shard in enumerate(layers):
        X = block_single_rank(sh, X, shard, caches[l], positions, batch, q_len, int(mask[l]),
                              rank, slots)
    return X


def rank_sum(base: Optional[np.ndarray], slots: np.ndarray) -> np.ndarray:
    """What a kept sync point delivers to every device: base + sum over ranks of the partials."""
    s = np.sum(np.asarray(slots, F64), axis=0)
    return s if base is None else np.asarray(base, F64) + s


# --------------------------------------------------------------------------- which blocks drop their sync point

TIER_TP, TIER_ISB, TIER_SB, TIER_ESB = 0, 1, 2, 3


def mask_from_sensitivity(S: Sequence[float], n_spd: int, tau1: float, tau2: float):
    """Sync-point drop by sensitivity (Alg. 1, Sec. 4.2).

    The blocks are ranked by ascending sync sensitivity S; the first n_spd of the ranking
    become SPD blocks.  Each of them is put in a tier by its sensitivity: in-sensitive
    (S <= tau1: SPD alone), sensitive (S <= tau2: SPD after block-to-block distillation),
    extremely sensitive (otherwise: head grouping as well).  Blocks outside the budget keep
    their sync point.  Equal sensitivities: the paper does not say; the block with the lower
    index ranks first.

    Returns (mask, tier): mask[l] = 1 iff block l drops its attention sync point."""
    L = len(S)
    if not 0 <= n_spd <= L:
        raise ValueError("n_spd out of range")
    if any(math.isnan(float(v)) for v in S) or math.isnan(tau1) or math.isnan(tau2):
        raise ValueError("NaN")
    B = sorted(range(L), key=lambda l: (float(S[l]), l))
    mask = [0] * L
    tier = [TIER_TP] * L
    for i in range(n_spd):
        blk = B[i]
        mask[blk] = 1
        if S[blk] <= tau1:
            tier[blk] = TIER_ISB
        elif S[blk] <= tau2:
            tier[blk] = TIER_SB
        else:
            tier[blk] = TIER_ESB
    return mask, tier


# --------------------------------------------------------------------------- head grouping

def grouped_shards(sh: Shapes, dense: Dict[str, np.ndarray], kv_heads: Sequence[int],
                   mlp_of_rank: Sequence[int]) -> List[Dict[str, np.ndarray]]:
    """Per-device weights after head grouping (Sec. 4.2.3, Fig. 5).

    kv_heads lists the KV heads in the order they are laid over the devices: device r holds
    kv_heads[r*kv : (r+1)*kv], each with its own query heads (for multi-head attention a KV
    head is a head); the columns of W_Q, W_K, W_V and the rows of W_O move with their head.
    mlp_of_rank[r] is the MLP partition (contiguous block of FFN columns) matched with device r.
    dense: wq [h, Hq*d], wk/wv [h, Hkv*d], wo [Hq*d, h], wg/wu [h, F], wd [F, h], g1, g2."""
    d, g = sh.head_dim, sh.n_q_heads // sh.n_kv_heads
    assert sorted(kv_heads) == list(range(sh.n_kv_heads)) and sorted(mlp_of_rank) == list(range(sh.tp))
    out = []
    for r in range(sh.tp):
        mine = [int(k) for k in kv_heads[r * sh.kv:(r + 1) * sh.kv]]
        q_cols = [c for k in mine for qh in range(k * g, (k + 1) * g) for c in range(qh * d, (qh + 1) * d)]
        kv_cols = [c for k in mine for c in range(k * d, (k + 1) * d)]
        m = int(mlp_of_rank[r])
        ffn = slice(m * sh.f, (m + 1) * sh.f)
        out.append({
            "wq": dense["wq"][:, q_cols].copy(), "wk": dense["wk"][:, kv_cols].copy(),
            "wv": dense["wv"][:, kv_cols].copy(), "wo": dense["wo"][q_cols, :].copy(),
            "wg": dense["wg"][:, ffn].copy(), "wu": dense["wu"][:, ffn].copy(), "wd": dense["wd"][ffn, :].copy(),
            "g1": dense["g1"].copy(), "g2": dense["g2"].copy(),
        })
    return out
