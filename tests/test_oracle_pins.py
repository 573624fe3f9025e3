"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these compares the oracle with itself re-typed: they use the dense single-device
block (TP equals single-device inference, Sec. 3), degenerate cases with closed forms,
algebraic consequences of the block design of Sec. 4.1.1, and an independent scalar
implementation (pure Python floats, dense matrices, devices emulated by zero-masking
instead of slicing).
"""
import math

import numpy as np
import pytest

from oracle import spd_oracle as O


def make_shards(rng, sh, std=0.3):
    h, d, q, kv, f = sh.hidden, sh.head_dim, sh.q, sh.kv, sh.f
    g1 = 1.0 + 0.1 * rng.standard_normal(h)
    g2 = 1.0 + 0.1 * rng.standard_normal(h)
    shards = []
    for _ in range(sh.tp):
        shards.append(dict(
            wq=std * rng.standard_normal((h, q * d)), wk=std * rng.standard_normal((h, kv * d)),
            wv=std * rng.standard_normal((h, kv * d)), wo=std * rng.standard_normal((q * d, h)),
            wg=std * rng.standard_normal((h, f)), wu=std * rng.standard_normal((h, f)),
            wd=std * rng.standard_normal((f, h)), g1=g1, g2=g2))
    return shards


def to_dense(shards):
    out = {}
    for n in ("wq", "wk", "wv", "wg", "wu"):
        out[n] = np.concatenate([s[n] for s in shards], axis=1)
    for n in ("wo", "wd"):
        out[n] = np.concatenate([s[n] for s in shards], axis=0)
    out["g1"], out["g2"] = shards[0]["g1"], shards[0]["g2"]
    return out


def fresh_caches(sh, batch, max_ctx, n=None):
    return [O.KVCache(batch, sh.kv, max_ctx, sh.head_dim) for _ in range(sh.tp if n is None else n)]


SHAPES = [
    O.Shapes(hidden=16, n_q_heads=4, n_kv_heads=4, head_dim=4, ffn=12, tp=2),
    O.Shapes(hidden=24, n_q_heads=8, n_kv_heads=4, head_dim=6, ffn=20, tp=4),   # grouped KV heads
    O.Shapes(hidden=16, n_q_heads=6, n_kv_heads=3, head_dim=8, ffn=9, tp=3),
]


# I1 -------------------------------------------------------------------------------------------
@pytest.mark.parametrize("sh", SHAPES)
@pytest.mark.parametrize("batch,q_len", [(1, 5), (2, 3)])
def test_tp_block_equals_single_device_block(sh, batch, q_len):
    rng = np.random.default_rng(10)
    shards = make_shards(rng, sh)
    X = rng.standard_normal((batch * q_len, sh.hidden))
    positions = [0] * batch
    out, syncs = O.block_all_ranks(sh, X, shards, fresh_caches(sh, batch, 8), positions, batch, q_len, 0)
    dense_cache = O.KVCache(batch, sh.n_kv_heads, 8, sh.head_dim)
    ref = O.dense_block(sh, X, to_dense(shards), dense_cache, positions, batch, q_len)
    assert syncs == 2
    np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-12)


# I2 -------------------------------------------------------------------------------------------
def test_tp1_spd_is_the_dense_block():
    sh = O.Shapes(hidden=16, n_q_heads=4, n_kv_heads=2, head_dim=4, ffn=12, tp=1)
    rng = np.random.default_rng(11)
    shards = make_shards(rng, sh)
    X = rng.standard_normal((4, sh.hidden))
    a, sa = O.block_all_ranks(sh, X, shards, fresh_caches(sh, 1, 8), [0], 1, 4, 1)
    b, sb = O.block_all_ranks(sh, X, shards, fresh_caches(sh, 1, 8), [0], 1, 4, 0)
    c = O.dense_block(sh, X, shards[0], O.KVCache(1, 2, 8, 4), [0], 1, 4)
    np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(a, c, rtol=1e-13, atol=1e-13)
    assert (sa, sb) == (1, 2)


# I3 -------------------------------------------------------------------------------------------
@pytest.mark.parametrize("sh", SHAPES)
def test_spd_changes_only_what_each_mlp_sees(sh):
    rng = np.random.default_rng(12)
    shards = make_shards(rng, sh)
    X = rng.standard_normal((3, sh.hidden))
    ds, dt = {}, {}
    spd, _ = O.block_all_ranks(sh, X, shards, fresh_caches(sh, 1, 8), [0], 1, 3, 1, ds)
    tp, _ = O.block_all_ranks(sh, X, shards, fresh_caches(sh, 1, 8), [0], 1, 3, 0, dt)
    for r in range(sh.tp):
        np.testing.assert_array_equal(ds["Y"][r], dt["Y"][r])     # attention part untouched
        # the MLP partial of device r is the MLP applied to X + Y_r (SPD) or X + sum Y (TP)
        np.testing.assert_allclose(ds["Z"][r], O.mlp_partial(sh, X + ds["Y"][r], shards[r]), rtol=1e-12)
        np.testing.assert_allclose(dt["Z"][r], O.mlp_partial(sh, X + sum(dt["Y"]), shards[r]), rtol=1e-12)
    # Sec. 4.1.1: the whole output of the block is X + sum Y_i + sum Z_i
    np.testing.assert_allclose(spd, X + sum(ds["Y"]) + sum(ds["Z"]), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(spd - tp, sum(ds["Z"]) - sum(dt["Z"]), rtol=1e-9, atol=1e-11)
    assert np.max(np.abs(spd - tp)) > 1e-3                          # a different function


# I4 -------------------------------------------------------------------------------------------
def test_zero_projection_special_cases():
    sh = SHAPES[1]
    rng = np.random.default_rng(13)
    shards = make_shards(rng, sh)
    X = rng.standard_normal((4, sh.hidden))
    no_o = [dict(s, wo=np.zeros_like(s["wo"])) for s in shards]
    a, _ = O.block_all_ranks(sh, X, no_o, fresh_caches(sh, 2, 4), [0, 0], 2, 2, 1)
    b, _ = O.block_all_ranks(sh, X, no_o, fresh_caches(sh, 2, 4), [0, 0], 2, 2, 0)
    np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-13)         # Y_i = 0: SPD == TP
    no_d = [dict(s, wd=np.zeros_like(s["wd"])) for s in shards]
    det = {}
    a, _ = O.block_all_ranks(sh, X, no_d, fresh_caches(sh, 2, 4), [0, 0], 2, 2, 1, det)
    b, _ = O.block_all_ranks(sh, X, no_d, fresh_caches(sh, 2, 4), [0, 0], 2, 2, 0)
    np.testing.assert_allclose(a, X + sum(det["Y"]), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(b, X + sum(det["Y"]), rtol=1e-13, atol=1e-13)


# I5 -------------------------------------------------------------------------------------------
def test_rank_local_mlp_input():
    sh = SHAPES[0]
    rng = np.random.default_rng(14)
    shards = make_shards(rng, sh)
    X = rng.standard_normal((3, sh.hidden))
    r = 1
    lone = [dict(s, wo=(s["wo"] if i == r else np.zeros_like(s["wo"]))) for i, s in enumerate(shards)]
    ds, dt = {}, {}
    O.block_all_ranks(sh, X, lone, fresh_caches(sh, 1, 4), [0], 1, 3, 1, ds)
    O.block_all_ranks(sh, X, lone, fresh_caches(sh, 1, 4), [0], 1, 3, 0, dt)
    np.testing.assert_allclose(ds["Z"][r], dt["Z"][r], rtol=1e-13, atol=1e-13)
    assert np.max(np.abs(ds["Z"][0] - dt["Z"][0])) > 1e-6            # the others do differ


# I6 -------------------------------------------------------------------------------------------
def test_every_rank_ends_with_the_same_output_and_rejected_wiring_does_not():
    sh = SHAPES[1]
    rng = np.random.default_rng(15)
    shards = make_shards(rng, sh)
    X = rng.standard_normal((2, sh.hidden))
    det = {}
    ref, _ = O.block_all_ranks(sh, X, shards, fresh_caches(sh, 1, 4), [0], 1, 2, 1, det)
    # each device's own view: the peers' slots hold their P_i, its own slot gets overwritten
    for r in range(sh.tp):
        slots = np.stack(det["P"]).copy()
        slots[r] = np.nan
        out_r = O.block_single_rank(sh, X, shards[r], fresh_caches(sh, 1, 4)[0], [0], 1, 2, 1, r, slots)
        np.testing.assert_allclose(out_r, ref, rtol=1e-12, atol=1e-12)
    # Table 1a's rejected placement adds Y_i after the MLP all-reduce: X + Y_i + sum Z
    rejected = [X + det["Y"][r] + sum(det["Z"]) for r in range(sh.tp)]
    assert np.max(np.abs(rejected[0] - rejected[1])) > 1e-3           # diverges across devices
    assert np.max(np.abs(rejected[0] - ref)) > 1e-3


def test_single_rank_view_matches_all_ranks_tp_block():
    sh = SHAPES[0]
    rng = np.random.default_rng(16)
    shards = make_shards(rng, sh)
    X = rng.standard_normal((3, sh.hidden))
    det = {}
    full, _ = O.block_all_ranks(sh, X, shards, fresh_caches(sh, 1, 4), [0], 1, 3, 0, det)

    # peers deliver Y at the first sync point and Z at the second one; a single buffer
    # cannot hold both, so check the two halves separately through the slot contract
    r = 0
    slots = np.stack(det["Y"]).copy()
    Y = O.attention_partial(sh, X, shards[r], fresh_caches(sh, 1, 4)[0], [0], 1, 3)
    slots[r] = Y
    R = O.rank_sum(X, slots)
    slots2 = np.stack(det["Z"]).copy()
    slots2[r] = O.mlp_partial(sh, R, shards[r])
    np.testing.assert_allclose(O.rank_sum(R, slots2), full, rtol=1e-12, atol=1e-12)
    # with identical peer buffers at both sync points the single-rank form is this formula
    peers = 0.05 * rng.standard_normal((sh.tp, 3, sh.hidden))
    got = O.block_single_rank(sh, X, shards[r], fresh_caches(sh, 1, 4)[0], [0], 1, 3, 0, r, peers.copy())
    others = sum(peers[i] for i in range(sh.tp) if i != r)
    R = X + Y + others
    want = R + O.mlp_partial(sh, R, shards[r]) + others
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


# I7 -------------------------------------------------------------------------------------------
def test_relabelling_and_moving_heads():
    sh = O.Shapes(hidden=16, n_q_heads=4, n_kv_heads=4, head_dim=4, ffn=12, tp=2)
    rng = np.random.default_rng(17)
    shards = make_shards(rng, sh)
    X = rng.standard_normal((3, sh.hidden))
    run = lambda s, flag: O.block_all_ranks(sh, X, s, fresh_caches(sh, 1, 4), [0], 1, 3, flag)[0]
    for flag in (0, 1):
        np.testing.assert_allclose(run(shards, flag), run(shards[::-1], flag), rtol=1e-12, atol=1e-12)
    # swap head 1 of device 0 with head 0 of device 1 (columns of Q/K/V, rows of O)
    d = sh.head_dim
    a, b = {k: v.copy() for k, v in shards[0].items()}, {k: v.copy() for k, v in shards[1].items()}
    for n in ("wq", "wk", "wv"):
        a[n][:, d:2 * d], b[n][:, 0:d] = shards[1][n][:, 0:d], shards[0][n][:, d:2 * d]
    a["wo"][d:2 * d, :], b["wo"][0:d, :] = shards[1]["wo"][0:d, :], shards[0]["wo"][d:2 * d, :]
    moved = [a, b]
    np.testing.assert_allclose(run(shards, 0), run(moved, 0), rtol=1e-11, atol=1e-12)   # TP: invariant
    assert np.max(np.abs(run(shards, 1) - run(moved, 1))) > 1e-4                        # SPD: not


# I8 -------------------------------------------------------------------------------------------
def test_prefill_then_decode_equals_longer_prefill():
    sh = SHAPES[1]
    rng = np.random.default_rng(18)
    L = 2
    layers = [make_shards(rng, sh) for _ in range(L)]
    mask = [1, 0]
    X = rng.standard_normal((10, sh.hidden))
    caches = [fresh_caches(sh, 1, 16) for _ in range(L)]
    full, _ = O.model_all_ranks(sh, X, layers, caches, [0], 1, 10, mask)
    caches = [fresh_caches(sh, 1, 16) for _ in range(L)]
    head, _ = O.model_all_ranks(sh, X[:6], layers, caches, [0], 1, 6, mask)
    np.testing.assert_allclose(head, full[:6], rtol=1e-11, atol=1e-12)
    for t in range(6, 10):
        step, _ = O.model_all_ranks(sh, X[t:t + 1], layers, caches, [t], 1, 1, mask)
        np.testing.assert_allclose(step[0], full[t], rtol=1e-10, atol=1e-11)


def test_batched_sequences_are_independent():
    sh = SHAPES[0]
    rng = np.random.default_rng(19)
    shards = make_shards(rng, sh)
    Xa, Xb = rng.standard_normal((3, sh.hidden)), rng.standard_normal((3, sh.hidden))
    both, _ = O.block_all_ranks(sh, np.concatenate([Xa, Xb]), shards, fresh_caches(sh, 2, 8), [0, 2], 2, 3, 1)
    # sequence 1 starts at position 2 with an empty cache below it: give the single run the same zeros
    a, _ = O.block_all_ranks(sh, Xa, shards, fresh_caches(sh, 1, 8), [0], 1, 3, 1)
    b, _ = O.block_all_ranks(sh, Xb, shards, fresh_caches(sh, 1, 8), [2], 1, 3, 1)
    np.testing.assert_allclose(both[:3], a, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(both[3:], b, rtol=1e-12, atol=1e-12)


# I9 -------------------------------------------------------------------------------------------
def test_textbook_reductions():
    rng = np.random.default_rng(20)
    # RoPE: identity at position 0, a plane rotation of each (j, j + d/2) pair otherwise
    v = rng.standard_normal((3, 2, 8))
    np.testing.assert_array_equal(O.rope(v, np.zeros(3, int), 10000.0), v)
    e = np.zeros((1, 1, 4)); e[0, 0, 0] = 1.0                       # pair (0, 2), theta_0 = 1
    np.testing.assert_allclose(O.rope(e, [3], 10000.0)[0, 0], [math.cos(3.0), 0, math.sin(3.0), 0], atol=1e-15)
    e = np.zeros((1, 1, 4)); e[0, 0, 1] = 1.0                       # pair (1, 3), theta_1 = 10000^(-1/2)
    np.testing.assert_allclose(O.rope(e, [7], 10000.0)[0, 0], [0, math.cos(0.07), 0, math.sin(0.07)], atol=1e-15)
    r = O.rope(v, [1, 5, 9], 10000.0)
    np.testing.assert_allclose(r[..., :4] ** 2 + r[..., 4:] ** 2, v[..., :4] ** 2 + v[..., 4:] ** 2, rtol=1e-12)
    np.testing.assert_allclose(O.rope(O.rope(v, [1, 2, 3], 100.0), [4, 4, 4], 100.0), O.rope(v, [5, 6, 7], 100.0), rtol=1e-12)
    q, k = rng.standard_normal((1, 1, 8)), rng.standard_normal((1, 1, 8))
    dot = lambda a, b: float(np.sum(O.rope(q, [a], 50.0) * O.rope(k, [b], 50.0)))
    assert abs(dot(7, 3) - dot(11, 7)) < 1e-12                      # depends on the offset only
    # RMSNorm: mean((y/g)^2) = ms / (ms + eps)
    x, g = rng.standard_normal((4, 32)), 1.0 + 0.1 * rng.standard_normal(32)
    y = O.rmsnorm(x, g, 1e-5)
    ms = np.mean(x * x, axis=1)
    np.testing.assert_allclose(np.mean((y / g) ** 2, axis=1), ms / (ms + 1e-5), rtol=1e-12)
    np.testing.assert_allclose(O.rmsnorm(3.0 * np.ones((1, 5)), np.arange(5.0), 0.0), np.arange(5.0)[None], rtol=1e-14)
    # silu
    assert O.silu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(O.silu(np.array([1.0, -2.0])), [1 / (1 + math.exp(-1)), -2 / (1 + math.exp(2))], rtol=1e-15)


def test_attention_closed_forms():
    sh = O.Shapes(hidden=8, n_q_heads=4, n_kv_heads=2, head_dim=4, ffn=8, tp=1)
    rng = np.random.default_rng(21)
    W = make_shards(rng, sh)[0]
    X = rng.standard_normal((1, 8))
    n = O.rmsnorm(X, W["g1"], sh.rms_eps)
    # one key only: softmax is 1, rotary is the identity at position 0, output = V of the KV group
    Y = O.attention_partial(sh, X, W, O.KVCache(1, 2, 4, 4), [0], 1, 1)
    V = (n @ W["wv"]).reshape(2, 4)
    A = np.concatenate([V[0], V[0], V[1], V[1]])                   # heads 0,1 -> KV 0; 2,3 -> KV 1
    np.testing.assert_allclose(Y[0], A @ W["wo"], rtol=1e-12)
    # zero queries: uniform attention = running mean of the values (causal prefix)
    W0 = dict(W, wq=np.zeros_like(W["wq"]))
    X = rng.standard_normal((5, 8))
    Y = O.attention_partial(sh, X, W0, O.KVCache(1, 2, 8, 4), [0], 1, 5)
    V = (O.rmsnorm(X, W["g1"], sh.rms_eps) @ W["wv"]).reshape(5, 2, 4)
    for t in range(5):
        m = V[:t + 1].mean(axis=0)
        A = np.concatenate([m[0], m[0], m[1], m[1]])
        np.testing.assert_allclose(Y[t], A @ W["wo"], rtol=1e-11, atol=1e-13)
    # one dominating key: attention returns that key's value (softmax saturates), scale 1/sqrt(d) irrelevant
    cache = O.KVCache(1, 2, 8, 4)
    kk = np.zeros((1, 2, 3, 4)); vv = rng.standard_normal((1, 2, 3, 4))
    cache.fill(kk, vv)
    Y = O.attention_partial(sh, X[:1], W0, cache, [3], 1, 1)      # keys 0..2 zero, key 3 = own
    Vn = (O.rmsnorm(X[:1], W["g1"], sh.rms_eps) @ W["wv"]).reshape(2, 4)
    m = (vv[0].sum(axis=1) + Vn) / 4.0
    np.testing.assert_allclose(Y[0], np.concatenate([m[0], m[0], m[1], m[1]]) @ W["wo"], rtol=1e-11)


def test_softmax_scale_is_one_over_sqrt_d():
    # two keys whose scores differ by a known amount: weights are sigmoid(delta / sqrt(d))
    sh = O.Shapes(hidden=4, n_q_heads=1, n_kv_heads=1, head_dim=4, ffn=4, tp=1)
    eye = np.eye(4)
    W = dict(wq=eye, wk=eye, wv=eye, wo=eye, wg=eye, wu=eye, wd=eye, g1=np.ones(4), g2=np.ones(4))
    cache = O.KVCache(1, 1, 4, 4)
    k0 = np.array([2.0, 0, 0, 0]); v0 = np.array([1.0, 0, 0, 0])
    cache.fill(k0.reshape(1, 1, 1, 4), v0.reshape(1, 1, 1, 4))
    x = np.array([[1.0, 1.0, 1.0, 1.0]])                           # rms 1 -> n = x (eps tiny)
    sh0 = O.Shapes(4, 1, 1, 4, 4, 1, rms_eps=0.0, rope_base=1e30)  # theta_1 ~ 0; theta_0 = 1
    Y = O.attention_partial(sh0, x, W, cache, [1], 1, 1)
    # query/key of the new token: rope at pos 1 on pair (0,2) by angle 1, pair (1,3) by ~0
    c, s = math.cos(1.0), math.sin(1.0)
    qn = np.array([c - s, 1.0, c + s, 1.0])
    s_old, s_new = float(qn @ k0) / 2.0, float(qn @ qn) / 2.0       # sqrt(d) = 2
    w_old = 1.0 / (1.0 + math.exp(s_new - s_old))
    want = w_old * v0 + (1 - w_old) * x[0]
    np.testing.assert_allclose(Y[0], want, rtol=1e-12)


# I10 ------------------------------------------------------------------------------------------
def _brute_block(h, Hq, Hkv, d, F, tp, eps, base, Wd_, X, spd):
    """Scalar re-implementation from the definitions.  Dense matrices; device i's share is
    obtained by zeroing every column/row that belongs to another device."""
    T = len(X)
    grp = Hq // Hkv
    q_per, f_per = Hq // tp, F // tp

    def norm(row, g):
        ms = sum(v * v for v in row) / h
        return [v / math.sqrt(ms + eps) * g[i] for i, v in enumerate(row)]

    def matvec(row, W, n_out):
        return [sum(row[i] * W[i][o] for i in range(len(row))) for o in range(n_out)]

    def rot(vec, pos):
        out = list(vec)
        for j in range(d // 2):
            ang = pos * base ** (-2.0 * j / d)
            a, b = vec[j], vec[j + d // 2]
            out[j] = a * math.cos(ang) - b * math.sin(ang)
            out[j + d // 2] = b * math.cos(ang) + a * math.sin(ang)
        return out

    # full attention head outputs (these do not depend on the device split)
    N = [norm(X[t], Wd_["g1"]) for t in range(T)]
    Qf = [matvec(N[t], Wd_["wq"], Hq * d) for t in range(T)]
    Kf = [matvec(N[t], Wd_["wk"], Hkv * d) for t in range(T)]
    Vf = [matvec(N[t], Wd_["wv"], Hkv * d) for t in range(T)]
    head_out = [[None] * Hq for _ in range(T)]
    for t in range(T):
        for j in range(Hq):
            qv = rot(Qf[t][j * d:(j + 1) * d], t)
            kh = j // grp
            sc = []
            for u in range(t + 1):
                kv_ = rot(Kf[u][kh * d:(kh + 1) * d], u)
                sc.append(sum(a * b for a, b in zip(qv, kv_)) / math.sqrt(d))
            mx = max(sc)
            ex = [math.exp(s - mx) for s in sc]
            den = sum(ex)
            head_out[t][j] = [sum(ex[u] / den * Vf[u][kh * d + c] for u in range(t + 1)) for c in range(d)]

    def Y_dev(i, t):     # rows of W_o that belong to other devices' heads contribute nothing
        acc = [0.0] * h
        for j in range(Hq):
            if j // q_per != i:
                continue
            for c in range(d):
                for o in range(h):
                    acc[o] += head_out[t][j][c] * Wd_["wo"][j * d + c][o]
        return acc

    def Z_dev(i, r_row):
        m = norm(r_row, Wd_["g2"])
        acc = [0.0] * h
        for c in range(F):
            if c // f_per != i:
                continue
            gte = sum(m[k] * Wd_["wg"][k][c] for k in range(h))
            up = sum(m[k] * Wd_["wu"][k][c] for k in range(h))
            act = gte / (1.0 + math.exp(-gte)) * up
            for o in range(h):
                acc[o] += act * Wd_["wd"][c][o]
        return acc

    out = []
    for t in range(T):
        Ys = [Y_dev(i, t) for i in range(tp)]
        if spd:
            Zs = [Z_dev(i, [X[t][o] + Ys[i][o] for o in range(h)]) for i in range(tp)]
            out.append([X[t][o] + sum(Ys[i][o] + Zs[i][o] for i in range(tp)) for o in range(h)])
        else:
            R = [X[t][o] + sum(Ys[i][o] for i in range(tp)) for o in range(h)]
            Zs = [Z_dev(i, R) for i in range(tp)]
            out.append([R[o] + sum(Zs[i][o] for i in range(tp)) for o in range(h)])
    return out


@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2)])
@pytest.mark.parametrize("spd", [0, 1])
def test_brute_force_tiny(Hq, Hkv, spd):
    h, d, F, tp, T = 8, 4, 8, 2, 3
    sh = O.Shapes(hidden=h, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, ffn=F, tp=tp, rms_eps=1e-5, rope_base=100.0)
    rng = np.random.default_rng(22 + Hq)
    shards = make_shards(rng, sh, std=0.5)
    dense = to_dense(shards)
    X = rng.standard_normal((T, h))
    got, _ = O.block_all_ranks(sh, X, shards, fresh_caches(sh, 1, 4), [0], 1, T, spd)
    want = _brute_block(h, Hq, Hkv, d, F, tp, 1e-5, 100.0,
                        {k: v.tolist() for k, v in dense.items()}, X.tolist(), spd)
    np.testing.assert_allclose(got, np.array(want), rtol=1e-10, atol=1e-12)


# I11 ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("mask", [[1, 0], [0, 0, 0], [1, 1, 1, 1], [0, 1, 1, 0, 1]])
def test_sync_count(mask):
    sh = SHAPES[0]
    rng = np.random.default_rng(23)
    L = len(mask)
    layers = [make_shards(rng, sh) for _ in range(L)]
    caches = [fresh_caches(sh, 1, 4) for _ in range(L)]
    X = rng.standard_normal((2, sh.hidden))
    _, syncs = O.model_all_ranks(sh, X, layers, caches, [0], 1, 2, mask)
    assert syncs == L + (L - sum(mask))                              # 2 per TP block, 1 per SPD block


def test_row_subset_matches_full_run():
    sh = SHAPES[1]
    rng = np.random.default_rng(24)
    shards = make_shards(rng, sh)
    X = rng.standard_normal((8, sh.hidden))
    peers = 0.05 * rng.standard_normal((sh.tp, 8, sh.hidden))
    for flag in (0, 1):
        full = O.block_single_rank(sh, X, shards[2], fresh_caches(sh, 2, 8)[0], [0, 1], 2, 4, flag, 2, peers.copy())
        rows = np.array([1, 6, 7])
        part = O.block_single_rank(sh, X, shards[2], fresh_caches(sh, 2, 8)[0], [0, 1], 2, 4, flag, 2, peers.copy(), rows=rows)
        np.testing.assert_allclose(part, full[rows], rtol=1e-12, atol=1e-13)


def test_bf16_cache_storage_rounds_once_at_the_store():
    # nearest-even rounding to 8 significant bits, pinned on values with known neighbours
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7, 1.0 + 3 * 2.0 ** -8, -0.3, 3.0e38, 2.0 ** -130])
    r = O.round_to_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 + 2.0 ** -7      # tie goes to the even mantissa
    assert r[3] == 1.0 + 2.0 ** -6                                       # tie, odd below: rounds up to even
    assert abs(r[4] + 0.3) <= 2.0 ** -10                                 # half an ulp of the binade [0.25, 0.5)
    assert np.float32(r[4]).view(np.uint32) & 0xFFFF == 0
    assert np.isfinite(r[5]) and r[6] == 2.0 ** -130
    sh = SHAPES[0]
    rng = np.random.default_rng(30)
    shards = make_shards(rng, sh)
    X = rng.standard_normal((3, sh.hidden))
    exact = O.KVCache(1, sh.kv, 4, sh.head_dim)
    stored = O.KVCache(1, sh.kv, 4, sh.head_dim, storage="bf16")
    ya = O.attention_partial(sh, X, shards[0], exact, [0], 1, 3)
    yb = O.attention_partial(sh, X, shards[0], stored, [0], 1, 3)
    np.testing.assert_array_equal(stored.k[:, :, :3], O.round_to_bf16(exact.k[:, :, :3]))
    np.testing.assert_array_equal(stored.v[:, :, :3], O.round_to_bf16(exact.v[:, :, :3]))
    assert 0 < np.max(np.abs(ya - yb)) < 0.05 * np.max(np.abs(ya))       # a small, real difference


# ------------------------------------------------------------------------------------------------
# Alg. 1: which blocks drop their sync point
# ------------------------------------------------------------------------------------------------
def test_mask_builder_worked_example():
    # ranking by hand: S = [0.5, 0.01, 12, 0.03, 0.04] -> blocks 1, 3, 4, 0, 2.  Budget 4 with the
    # thresholds of Sec. 5 (0.05, 10): 1, 3, 4 are in-sensitive, 0 is sensitive, 2 keeps its sync.
    mask, tier = O.mask_from_sensitivity([0.5, 0.01, 12.0, 0.03, 0.04], 4, 0.05, 10.0)
    assert mask == [1, 1, 0, 1, 1]
    assert tier == [O.TIER_SB, O.TIER_ISB, O.TIER_TP, O.TIER_ISB, O.TIER_ISB]
    # the whole model: the last block is extremely sensitive
    mask, tier = O.mask_from_sensitivity([0.5, 0.01, 12.0, 0.03, 0.04], 5, 0.05, 10.0)
    assert mask == [1] * 5 and tier[2] == O.TIER_ESB
    # thresholds are inclusive (Alg. 1 compares with <=)
    mask, tier = O.mask_from_sensitivity([0.05, 10.0, 10.000001], 3, 0.05, 10.0)
    assert tier == [O.TIER_ISB, O.TIER_SB, O.TIER_ESB]


def test_mask_builder_selection_by_repeated_minimum():
    # an independent route to the same ranking: take the least sensitive remaining block n_spd times
    rng = np.random.default_rng(5)
    for trial in range(200):
        L = int(rng.integers(1, 12))
        S = rng.choice([0.0, 0.01, 0.05, 0.3, 10.0, 11.0, 50.0], size=L).tolist() if trial % 2 else rng.random(L).tolist()
        n = int(rng.integers(0, L + 1))
        mask, tier = O.mask_from_sensitivity(S, n, 0.05, 10.0)
        left = list(range(L))
        want = [0] * L
        for _ in range(n):
            best = left[0]
            for l in left:
                if S[l] < S[best]:
                    best = l              # strict: the first (lowest index) of equal values stays
            want[best] = 1
            left.remove(best)
        assert mask == want
        assert sum(mask) == n
        # nobody outside the budget is less sensitive than somebody inside it
        if 0 < n < L:
            assert max(S[l] for l in range(L) if mask[l]) <= min(S[l] for l in range(L) if not mask[l])
        for l in range(L):
            if not mask[l]:
                assert tier[l] == O.TIER_TP
            else:
                assert tier[l] == (O.TIER_ISB if S[l] <= 0.05 else O.TIER_SB if S[l] <= 10.0 else O.TIER_ESB)


def test_mask_builder_budget_is_monotone_and_feeds_the_sync_count():
    S = [3.0, 0.2, 0.2, 7.0, 0.01, 40.0]
    prev = [0] * len(S)
    for n in range(len(S) + 1):
        mask, _ = O.mask_from_sensitivity(S, n, 0.05, 10.0)
        assert all(a <= b for a, b in zip(prev, mask))        # a larger budget only adds blocks
        prev = mask
        # every block ends with a sync point; a block outside the budget has a second one (Sec. 3)
        assert sum(1 if m else 2 for m in mask) == 2 * len(S) - n
    # equal sensitivities: the lower index first
    assert O.mask_from_sensitivity(S, 2, 0.05, 10.0)[0] == [0, 1, 0, 0, 1, 0]
    with pytest.raises(ValueError):
        O.mask_from_sensitivity(S, 7, 0.05, 10.0)
    with pytest.raises(ValueError):
        O.mask_from_sensitivity([0.1, float("nan")], 1, 0.05, 10.0)


# ------------------------------------------------------------------------------------------------
# head grouping: which heads and which MLP partition live on a device (Sec. 4.2.3, Fig. 5)
# ------------------------------------------------------------------------------------------------
def test_head_grouping_moves_weights_but_not_the_tp_result():
    sh = O.Shapes(hidden=16, n_q_heads=8, n_kv_heads=4, head_dim=4, ffn=24, tp=2)     # 2 query heads per KV head
    rng = np.random.default_rng(23)
    shards = make_shards(rng, sh)
    dense = to_dense(shards)
    X = rng.standard_normal((3, sh.hidden))
    run = lambda s, flag: O.block_all_ranks(sh, X, s, fresh_caches(sh, 1, 4), [0], 1, 3, flag)[0]
    # the identity grouping is the contiguous split
    ident = O.grouped_shards(sh, dense, [0, 1, 2, 3], [0, 1])
    for a, b in zip(ident, shards):
        for k in a:
            assert np.array_equal(a[k], b[k]), k
    # a device's query heads are those of its KV heads: KV head 3 brings query heads 6 and 7
    moved = O.grouped_shards(sh, dense, [3, 0, 2, 1], [1, 0])
    d = sh.head_dim
    assert np.array_equal(moved[0]["wq"][:, :2 * d], dense["wq"][:, 6 * d:8 * d])
    assert np.array_equal(moved[0]["wo"][2 * d:4 * d, :], dense["wo"][0:2 * d, :])
    assert np.array_equal(moved[1]["wk"][:, d:2 * d], dense["wk"][:, d:2 * d])
    assert np.array_equal(moved[0]["wd"], dense["wd"][sh.f:, :]) and np.array_equal(moved[1]["wg"], dense["wg"][:, :sh.f])
    # every dense column / row lands on exactly one device
    for name, axis in (("wq", 1), ("wk", 1), ("wv", 1), ("wg", 1), ("wu", 1), ("wo", 0), ("wd", 0)):
        got = np.sort(np.concatenate([s[name] for s in moved], axis=axis).ravel())
        assert np.array_equal(got, np.sort(dense[name].ravel())), name
    # with every sync point kept the block computes the same function wherever the heads live;
    # an SPD block does not (each MLP partition sees only its own device's heads)
    np.testing.assert_allclose(run(moved, 0), run(shards, 0), rtol=1e-11, atol=1e-12)
    assert np.max(np.abs(run(moved, 1) - run(shards, 1))) > 1e-4
    # the matching alone (same heads, MLP partitions swapped) also changes only the SPD block
    swapped = O.grouped_shards(sh, dense, [0, 1, 2, 3], [1, 0])
    np.testing.assert_allclose(run(swapped, 0), run(shards, 0), rtol=1e-11, atol=1e-12)
    assert np.max(np.abs(run(swapped, 1) - run(shards, 1))) > 1e-4


# ------------------------------------------------------------------------------------------------
# block with bias in the output projection (Sec. 4.1.2)
# ------------------------------------------------------------------------------------------------
def test_block_with_bias():
    sh = O.Shapes(hidden=16, n_q_heads=4, n_kv_heads=2, head_dim=4, ffn=24, tp=2)
    rng = np.random.default_rng(29)
    shards = make_shards(rng, sh)
    X = rng.standard_normal((5, sh.hidden))
    bo = rng.standard_normal(sh.hidden)
    with_b = [dict(s, bo=bo) for s in shards]
    zero_b = [dict(s, bo=np.zeros(sh.hidden)) for s in shards]
    run = lambda s, flag, det=None: O.block_all_ranks(sh, X, s, fresh_caches(sh, 1, 8), [0], 1, 5, flag, det)[0]
    for flag in (0, 1):
        # a zero bias is the block without bias
        np.testing.assert_array_equal(run(zero_b, flag), run(shards, flag))
        assert np.max(np.abs(run(with_b, flag) - run(shards, flag))) > 1e-3
    # TP with bias is the single-device block with bias: attention output = sum_i P_i + b, b once
    dense = to_dense(shards)
    dense["bo"] = bo
    want = O.dense_block(sh, X, dense, O.KVCache(1, sh.n_kv_heads, 8, sh.head_dim), [0], 1, 5)
    np.testing.assert_allclose(run(with_b, 0), want, rtol=1e-11, atol=1e-12)
    # SPD with bias: the output is X + sum_i P_i + b + sum_i Z_i with the bias counted once,
    # and device i's MLP saw X + P_i + b (Sec. 4.1.2)
    det = {}
    out = run(with_b, 1, det)
    np.testing.assert_allclose(out, X + sum(det["Y"]) + bo + sum(det["Z"]), rtol=1e-12, atol=1e-12)
    for i in range(sh.tp):
        np.testing.assert_allclose(det["Z"][i], O.mlp_partial(sh, X + det["Y"][i] + bo, shards[i]), rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(det["P"][i], det["Y"][i] + det["Z"][i], rtol=1e-12, atol=1e-12)     # no bias before the sync
    # the bias is counted once, not once per device: with the MLP switched off (zero down projection)
    # raising every bias entry by one raises the output by exactly one
    big = [dict(s, bo=bo + 1.0) for s in shards]
    nomlp = lambda ss: [dict(s, wd=np.zeros_like(s["wd"])) for s in ss]
    for flag in (0, 1):
        np.testing.assert_allclose(run(nomlp(big), flag) - run(nomlp(with_b), flag), np.ones_like(X), rtol=0, atol=1e-12)
    # the single-rank view agrees with the all-ranks run
    det = {}
    full = run(with_b, 1, det)
    got = O.block_single_rank(sh, X, with_b[1], O.KVCache(1, sh.kv, 8, sh.head_dim), [0], 1, 5, 1, 1,
                              np.stack(det["P"]).copy())
    np.testing.assert_allclose(got, full, rtol=1e-11, atol=1e-12)


def test_sync_points_stated_by_the_paper():
    """tests/golden/sync_points.txt: block counts and SPD shares the paper states, and the number of sync
    points they imply; the oracle's mask builder and block loop must count the same."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "sync_points.txt")
    rows = [l.split()[:3] for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 7
    sh = O.Shapes(hidden=8, n_q_heads=2, n_kv_heads=2, head_dim=4, ffn=8, tp=2)
    rng = np.random.default_rng(31)
    for n_blocks, n_spd, want in (map(int, r) for r in rows):
        S = rng.random(n_blocks).tolist()
        mask, _ = O.mask_from_sensitivity(S, n_spd, 0.05, 10.0)
        assert sum(1 if m else 2 for m in mask) == want
    # and the block loop itself reports what it did (a short model: 5 blocks, 3 of them SPD -> 7 sync points)
    shards = [make_shards(rng, sh) for _ in range(5)]
    X = rng.standard_normal((2, sh.hidden))
    _, syncs = O.model_all_ranks(sh, X, shards, [fresh_caches(sh, 1, 4) for _ in range(5)], [0], 1, 2, [1, 0, 1, 1, 0])
    assert syncs == 7
