"""CPU-only checks of the C-ABI library: it loads, exports what include/*.h declare, rejects
bad arguments before touching a device, indexes ranks and counts sync points bit-exactly,
and its packers are lossless permutations.  No compute call is made here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2502_20727_amd import binding as B
from oracle import spd_oracle as O
from paper_2502_20727_amd import inputs, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SMALL_BF16 = workloads.Workload(name="small-bf16", hidden=128, n_q_heads=8, n_kv_heads=4, head_dim=64, ffn=416,
                                n_layers=3, tp=2, dtype=workloads.BF16, seed=7, batch=2, q_len=4, ctx=64,
                                mask=(1, 0, 1))
SMALL_F32 = workloads.Workload(name="small-f32", hidden=48, n_q_heads=6, n_kv_heads=3, head_dim=8, ffn=33,
                               n_layers=2, tp=3, dtype=workloads.F32, seed=8, batch=2, q_len=3, ctx=32, mask=(1, 0))


def declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(inc, fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"\b(spd_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = declared_functions()
    assert len(names) >= 18
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names          # the binding covers the header, nothing more, nothing less


def test_static_entry_point_refuses_a_workspace_that_does_not_fit():
    """The size check of the entry point without allocations comes before any device call."""
    ctx = B.spd_create(B.make_config(workloads.LLAMA70B_PREFILL.with_layers(1)))
    assert B.spd_get_sizes(ctx).workspace_bytes > B.SPD_STATIC_WORKSPACE_BYTES
    buf = np.zeros(64, np.float32)
    with pytest.raises(B.SpdError) as e:
        B.spd_block_forward_static(ctx, 0, 1, 0, buf, buf, [0], 1, 1, buf, buf, buf, stream=0)
    assert e.value.code == B.SPD_ETOOBIG
    assert "static" in B.strerror(B.SPD_ETOOBIG)
    B.spd_destroy(ctx)


def test_mfma_probe_rejects_bad_arguments_before_any_launch():
    lib = B.lib()
    tf, mhz = C.c_double(), C.c_double()
    assert lib.spd_mfma_probe(0, 1, C.c_void_p(8), None, C.byref(tf), C.byref(mhz)) == B.SPD_EINVAL
    assert lib.spd_mfma_probe(10, 1, None, None, C.byref(tf), C.byref(mhz)) == B.SPD_EINVAL
    assert lib.spd_mfma_probe(10, 1, C.c_void_p(8), None, None, C.byref(mhz)) == B.SPD_EINVAL


def test_read_probe_rejects_bad_arguments_before_any_launch():
    lib = B.lib()
    us = C.c_double()
    ok = C.c_void_p(8)
    assert lib.spd_read_probe(None, 4 << 20, 1, 1, ok, None, C.byref(us)) == B.SPD_EINVAL
    assert lib.spd_read_probe(ok, (4 << 20) + 1024, 1, 1, ok, None, C.byref(us)) == B.SPD_EINVAL
    assert lib.spd_read_probe(ok, 4 << 20, 0, 1, ok, None, C.byref(us)) == B.SPD_EINVAL
    assert lib.spd_read_probe(ok, 4 << 20, 1, 1, None, None, C.byref(us)) == B.SPD_EINVAL
    assert lib.spd_read_probe(ok, 4 << 20, 1, 1, ok, None, None) == B.SPD_EINVAL


def test_strerror():
    assert B.strerror(0) == "ok"
    for code in (B.SPD_EINVAL, B.SPD_EUNSUPPORTED, B.SPD_EHIP, -99):
        assert B.strerror(code)


def _cfg(**over):
    base = dict(hidden=128, n_q_heads=8, n_kv_heads=4, head_dim=64, ffn=416, n_layers=2, tp_degree=2,
                dtype=B.SPD_BF16, max_batch=2, max_ctx=64, max_tokens=16, rms_eps=1e-5, rope_base=10000.0)
    base.update(over)
    return B.spd_config(**base)


@pytest.mark.parametrize("over,code", [
    (dict(hidden=0), B.SPD_EINVAL),
    (dict(tp_degree=3), B.SPD_EINVAL),                 # does not divide the heads
    (dict(ffn=417), B.SPD_EINVAL),                     # ffn not divisible by tp
    (dict(n_q_heads=6), B.SPD_EINVAL),                 # not a multiple of the KV heads
    (dict(head_dim=63), B.SPD_EINVAL),
    (dict(max_ctx=48), B.SPD_EINVAL),
    (dict(max_batch=B.SPD_MAX_BATCH + 1, max_tokens=100), B.SPD_EINVAL),
    (dict(max_tokens=1), B.SPD_EINVAL),
    (dict(n_kv_heads=1, n_q_heads=8), B.SPD_EUNSUPPORTED),   # a KV head shared by two ranks
    (dict(dtype=5), B.SPD_EUNSUPPORTED),
    (dict(hidden=120), B.SPD_EUNSUPPORTED),            # bf16 path wants multiples of 32
    (dict(ffn=408), B.SPD_EUNSUPPORTED),               # 204 per rank: not a multiple of 16
    (dict(n_q_heads=136, n_kv_heads=4, tp_degree=2), B.SPD_EUNSUPPORTED),   # 34 query heads per KV head
])
def test_create_rejects(over, code):
    with pytest.raises(B.SpdError) as e:
        B.spd_create(_cfg(**over))
    assert e.value.code == code


def test_create_null():
    out = C.c_void_p()
    assert B.lib().spd_create(None, C.byref(out)) == B.SPD_EINVAL
    assert B.lib().spd_create(C.byref(_cfg()), None) == B.SPD_EINVAL


def test_config_roundtrip_and_sizes():
    ctx = B.spd_create(_cfg())
    c = B.spd_get_config(ctx)
    assert (c.hidden, c.tp_degree, c.max_ctx) == (128, 2, 64)
    s = B.spd_get_sizes(ctx)
    # one rank: 4 query heads, 2 KV heads, 208 -> 224 padded FFN columns
    weights = 128 * (8 * 64) + (4 * 64) * 128 + 2 * 128 * 224 + 224 * 128
    assert s.weight_bytes >= 2 * weights and s.weight_bytes % 256 == 0
    assert s.kv_bytes == 2 * (2 * 2 * 64 * 64 * 2) and s.workspace_bytes % 256 == 0
    B.spd_destroy(ctx)


def test_rank_indexing_is_contiguous_equal_blocks():
    # Sec. 4.2.3: n(A_i) = N / number_of_devices heads per device
    w = workloads.LLAMA70B_DECODE
    ctx = B.spd_create(B.make_config(w))
    seen_q, seen_kv, seen_f = [], [], []
    for r in range(w.tp):
        f, n = B.spd_rank_q_heads(ctx, r); seen_q += list(range(f, f + n)); assert n == 8
        f, n = B.spd_rank_kv_heads(ctx, r); seen_kv += list(range(f, f + n)); assert n == 1
        f, n = B.spd_rank_ffn_cols(ctx, r); seen_f += list(range(f, f + n)); assert n == 3584
    assert seen_q == list(range(64)) and seen_kv == list(range(8)) and seen_f == list(range(28672))
    for bad in (-1, w.tp):
        with pytest.raises(B.SpdError):
            B.spd_rank_q_heads(ctx, bad)
    B.spd_destroy(ctx)


@pytest.mark.parametrize("w", [workloads.TOY, workloads.LLAMA13B_DECODE, workloads.LLAMA70B_DECODE,
                               workloads.LLAMA70B_PREFILL])
def test_sync_count(w):
    # two sync points per TP block, one per SPD block (Sec. 3: SPD at 100 % halves them)
    ctx = B.spd_create(B.make_config(w, max_ctx=64, max_tokens=64, max_batch=1))
    L = w.n_layers
    assert B.spd_sync_count(ctx, w.mask) == L + (L - sum(w.mask))
    assert B.spd_sync_count(ctx, [1] * L) == L
    assert B.spd_sync_count(ctx, [0] * L) == 2 * L
    with pytest.raises(B.SpdError):
        B.spd_sync_count(ctx, [2] + [0] * (L - 1))
    B.spd_destroy(ctx)


def test_mask_from_sensitivity_is_the_oracle_bit_for_bit():
    # integer logic: exact agreement with the oracle's Alg. 1 on random sensitivities with many ties,
    # infinities, every budget from 0 to L, and both threshold settings of Sec. 5
    rng = np.random.default_rng(21)
    pool = [0.0, 0.01, 0.02, 0.05, 0.0500001, 0.3, 10.0, 10.5, 50.0, float("inf"), -1.0]
    n_cases = 0
    for trial in range(300):
        L = int(rng.integers(1, 90))
        S = rng.choice(pool, size=L) if trial % 3 else rng.lognormal(-2.0, 3.0, size=L)
        for n_spd in {0, L, int(rng.integers(0, L + 1)), int(rng.integers(0, L + 1))}:
            for tau1 in (0.05, 0.02):
                want = O.mask_from_sensitivity(S.tolist(), n_spd, tau1, 10.0)
                got = B.spd_mask_from_sensitivity(S, n_spd, tau1, 10.0)
                assert got[0] == want[0] and got[1] == want[1], (S, n_spd, tau1)
                n_cases += 1
    assert n_cases > 1000
    # the mask is what spd_sync_count and spd_model_forward take
    w = workloads.LLAMA70B_DECODE
    ctx = B.spd_create(B.make_config(w))
    S = rng.random(w.n_layers)
    mask, tier = B.spd_mask_from_sensitivity(S, 64, 0.02, 10.0)
    assert B.spd_sync_count(ctx, mask) == w.n_layers + (w.n_layers - 64)
    assert tier.count(B.SPD_TIER_TP) == 16
    B.spd_destroy(ctx)


def test_sync_points_stated_by_the_paper():
    # the same golden rows as the oracle's pin, through the library's mask builder and sync counter
    path = os.path.join(os.path.dirname(__file__), "golden", "sync_points.txt")
    rng = np.random.default_rng(32)
    for n_blocks, n_spd, want in (map(int, l.split()[:3]) for l in open(path) if l.strip() and not l.startswith("#")):
        w = workloads.Workload(name="g", hidden=64, n_q_heads=2, n_kv_heads=2, head_dim=32, ffn=64, n_layers=n_blocks,
                               tp=2, dtype=workloads.BF16, seed=1, batch=1, q_len=1, ctx=32, mask=(1,) * n_blocks)
        ctx = B.spd_create(B.make_config(w))
        mask, _ = B.spd_mask_from_sensitivity(rng.random(n_blocks), n_spd, 0.05, 10.0)
        assert B.spd_sync_count(ctx, mask) == want
        B.spd_destroy(ctx)


def test_mask_from_sensitivity_rejects():
    S = [0.1, 0.2, 0.3]
    for bad in (dict(n_spd=-1), dict(n_spd=4), dict(tau1=float("nan")), dict(tau2=float("nan")),
                dict(sensitivity=[0.1, float("nan"), 0.3]), dict(sensitivity=[])):
        kw = dict(sensitivity=S, n_spd=1, tau1=0.05, tau2=10.0)
        kw.update(bad)
        with pytest.raises(B.SpdError) as e:
            B.spd_mask_from_sensitivity(**kw)
        assert e.value.code == B.SPD_EINVAL


def test_workload_masks():
    assert workloads.TOY.mask == (1, 0)
    assert sum(workloads.LLAMA7B_DECODE.mask) == 32
    m = workloads.LLAMA13B_DECODE.mask
    assert [l for l in range(40) if m[l] == 0] == list(range(3, 40, 4))
    m = workloads.LLAMA70B_DECODE.mask
    assert m[:8] == (0,) * 8 and m[72:] == (0,) * 8 and sum(m) == 64


@pytest.mark.parametrize("w", [SMALL_BF16, SMALL_F32])
def test_pack_is_a_lossless_slice(w):
    ctx = B.spd_create(B.make_config(w))
    dense = inputs.dense_layer(w, 1)
    for r in range(w.tp):
        shard = inputs.layer_shard(w, 1, r)
        a = B.spd_pack_shard(ctx, r, dense)
        b = B.spd_pack_shard_local(ctx, shard)
        assert np.array_equal(a, b)                                   # slicing by rank == the rank's shard
        back = B.spd_unpack_shard(ctx, a, {k: v.shape for k, v in shard.items()})
        for k in shard:
            assert np.array_equal(back[k], shard[k]), k               # bit-exact round trip
    # different ranks really get different columns
    assert not np.array_equal(B.spd_pack_shard(ctx, 0, dense), B.spd_pack_shard(ctx, 1, dense))
    with pytest.raises(B.SpdError):
        B.spd_pack_shard(ctx, w.tp, dense)
    B.spd_destroy(ctx)


GQA_F32 = workloads.Workload(name="gqa-f32", hidden=32, n_q_heads=8, n_kv_heads=4, head_dim=8, ffn=48, n_layers=1, tp=2,
                             dtype=workloads.F32, seed=9, batch=1, q_len=1, ctx=32, mask=(1,))
GQA_BF16 = workloads.Workload(name="gqa-bf16", hidden=64, n_q_heads=8, n_kv_heads=4, head_dim=32, ffn=96, n_layers=1,
                              tp=2, dtype=workloads.BF16, seed=9, batch=1, q_len=1, ctx=32, mask=(1,))


@pytest.mark.parametrize("w", [GQA_F32, GQA_BF16, SMALL_BF16], ids=lambda w: w.name)
def test_grouped_pack_is_the_oracle_grouping_bit_for_bit(w):
    # head grouping (Sec. 4.2.3): the packed bytes of every device equal the packing of the shard the
    # oracle cuts out of the dense layer for the same head order and MLP matching
    ctx = B.spd_create(B.make_config(w))
    dense = inputs.dense_layer(w, 0)
    sh = O.Shapes(w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn, w.tp, w.rms_eps, w.rope_base)
    rng = np.random.default_rng(4)
    for trial in range(6):
        kvh = rng.permutation(w.n_kv_heads).tolist() if trial else list(range(w.n_kv_heads))
        mlp = rng.permutation(w.tp).tolist() if trial != 1 else list(range(w.tp))
        want = O.grouped_shards(sh, dense, kvh, mlp)
        for r in range(w.tp):
            got = B.spd_pack_shard_grouped(ctx, r, dense, kvh, mlp)
            ref = B.spd_pack_shard_local(ctx, {k: np.ascontiguousarray(v, dtype=np.float32) for k, v in want[r].items()})
            assert np.array_equal(got, ref), (trial, r)
    # identity arguments (or none) are the plain contiguous split
    for r in range(w.tp):
        assert np.array_equal(B.spd_pack_shard_grouped(ctx, r, dense, None, None), B.spd_pack_shard(ctx, r, dense))
    for bad_kv, bad_mlp in (([0] * w.n_kv_heads, None), (None, [0] * w.tp), (list(range(1, w.n_kv_heads + 1)), None)):
        with pytest.raises(B.SpdError) as e:
            B.spd_pack_shard_grouped(ctx, 0, dense, bad_kv, bad_mlp)
        assert e.value.code == B.SPD_EINVAL
    with pytest.raises(B.SpdError):
        B.spd_pack_shard_grouped(ctx, w.tp, dense, None, None)
    B.spd_destroy(ctx)


def test_pack_every_value_lands_exactly_once():
    # a packed shard of the bf16 path is a permutation of the shard's values (each times its matrix's power of
    # two, as fp16) plus zero padding
    w = SMALL_BF16
    ctx = B.spd_create(B.make_config(w))
    shard = inputs.layer_shard(w, 0, 1)
    n = 0
    for k in ("wq", "wk", "wv", "wo", "wg", "wu", "wd"):
        a = shard[k]
        a[...] = (np.arange(n, n + a.size, dtype=np.int64) % 251 + 1).reshape(a.shape).astype(np.float32)
        n += a.size
    packed = B.spd_pack_shard_local(ctx, shard)
    # skip the two fp32 gain vectors and the block of four scale factors; every matrix has the largest value 251,
    # so each is stored as fp16(2^7 w)
    vals = packed[2 * 256 * 2 + 256:].view(np.float16).astype(np.float64) / 128.0
    assert np.array_equal(vals, np.round(vals))
    got = np.bincount(vals.astype(np.int64), minlength=252)
    want = np.zeros(252, dtype=np.int64)
    for k in ("wq", "wk", "wv", "wo", "wg", "wu", "wd"):
        want += np.bincount(shard[k].astype(np.int64).ravel(), minlength=252)
    assert np.array_equal(got[1:], want[1:])
    B.spd_destroy(ctx)


def test_pack_keeps_a_second_gate_up_copy_when_tiles_do_not_fill_the_chip():
    # 3200 FFN columns = 200 tiles of 16: decode reads a copy regrouped into 13-column groups, so
    # every gate/up value is stored exactly twice and everything else once
    w = workloads.Workload(name="narrow", hidden=64, n_q_heads=2, n_kv_heads=2, head_dim=32, ffn=3200, n_layers=1,
                           tp=1, dtype=workloads.BF16, seed=3, batch=1, q_len=1, ctx=32, mask=(1,))
    ctx = B.spd_create(B.make_config(w))
    shard = inputs.layer_shard(w, 0, 0)
    n = 0
    for k in ("wq", "wk", "wv", "wo", "wg", "wu", "wd"):
        a = shard[k]
        a[...] = (np.arange(n, n + a.size, dtype=np.int64) % 251 + 1).reshape(a.shape).astype(np.float32)
        n += a.size
    packed = B.spd_pack_shard_local(ctx, shard)
    assert packed.size == B.spd_get_sizes(ctx).weight_bytes
    # skip the two fp32 gain vectors (64 floats, padded) and the block of scale factors; stored as fp16(2^7 w)
    vals = packed[2 * 256 + 256:].view(np.float16).astype(np.float64) / 128.0
    assert np.array_equal(vals, np.round(vals))
    got = np.bincount(vals.astype(np.int64), minlength=252)
    want = np.zeros(252, dtype=np.int64)
    for k in ("wq", "wk", "wv", "wo", "wg", "wu", "wd"):
        want += np.bincount(shard[k].astype(np.int64).ravel(), minlength=252) * (2 if k in ("wg", "wu") else 1)
    assert np.array_equal(got[1:], want[1:])
    back = B.spd_unpack_shard(ctx, packed, {k: v.shape for k, v in shard.items()})
    for k in ("wg", "wu", "wd"):
        assert np.array_equal(back[k], shard[k]), k
    B.spd_destroy(ctx)


@pytest.mark.parametrize("w", [SMALL_BF16, SMALL_F32])
def test_pack_with_output_bias(w):
    # block with bias (Sec. 4.1.2): the bias travels with the packed shard, in fp32, and must be given
    # exactly when the configuration says the block has one
    ctx_b, ctx = B.spd_create(B.make_config(w, o_bias=1)), B.spd_create(B.make_config(w))
    shard = inputs.layer_shard(w, 0, 1)
    bo = (inputs.output_bias(w, 0) * (1.0 + 2.0 ** -20)).astype(np.float32)       # not bf16 values: kept as fp32
    with pytest.raises(B.SpdError):
        B.spd_pack_shard_local(ctx_b, shard)                 # bias missing
    with pytest.raises(B.SpdError):
        B.spd_pack_shard_local(ctx, dict(shard, bo=bo))      # bias not expected
    packed = B.spd_pack_shard_local(ctx_b, dict(shard, bo=bo))
    assert packed.size == B.spd_get_sizes(ctx_b).weight_bytes > B.spd_get_sizes(ctx).weight_bytes
    shapes = {k: v.shape for k, v in shard.items()}
    shapes["bo"] = bo.shape
    back = B.spd_unpack_shard(ctx_b, packed, shapes)
    assert np.array_equal(back["bo"], bo)
    for k in shard:
        assert np.array_equal(back[k], shard[k]), k
    bad = B.make_config(w)
    bad.o_bias = 2
    with pytest.raises(B.SpdError) as e:
        B.spd_create(bad)
    assert e.value.code == B.SPD_EINVAL
    B.spd_destroy(ctx_b)
    B.spd_destroy(ctx)


def test_fp16_encoding_of_the_weights_reproduces_them():
    """The packed shard holds every weight as round_fp16(2^k w), one power of two per matrix.  bf16 values fit:
    every weight within 2^-29 of its matrix's largest comes back bit for bit; whatever is smaller lands on
    fp16's subnormal grid, at most 2^-25 / 2^k < 2^-39 max|w| away."""
    w = SMALL_BF16
    ctx = B.spd_create(B.make_config(w))
    shard = inputs.layer_shard(w, 0, 1)
    shapes = {k: v.shape for k, v in shard.items()}
    # a wide dynamic range inside one matrix, far beyond trained or synthetic weights
    for k in ("wq", "wd"):
        a = shard[k]
        a.flat[0] = np.float32(64.0)
        a.flat[1] = np.float32(2.0 ** -20)            # 26 binades below the largest: still exact
        a.flat[2] = np.float32(1.5 * 2.0 ** -22)
    back = B.spd_unpack_shard(ctx, B.spd_pack_shard_local(ctx, shard), shapes)
    for k in shapes:
        assert np.array_equal(back[k], shard[k]), k
    # beyond fp16's reach: the large entries stay exact, the tiny ones move by less than 2^-39 of the largest
    for k in ("wq", "wd"):
        a = shard[k]
        a.flat[1] = np.float32(2.0 ** -40)            # 46 binades below the largest
        a.flat[2] = np.float32(1.5 * 2.0 ** -60)
    back = B.spd_unpack_shard(ctx, B.spd_pack_shard_local(ctx, shard), shapes)
    for k in shapes:
        diff = np.abs(back[k].astype(np.float64) - shard[k].astype(np.float64))
        if k in ("wq", "wd"):
            assert 0.0 < diff.max() <= 2.0 ** -39 * 64.0 and np.count_nonzero(diff) <= 2
            assert back[k].flat[0] == 64.0
        else:
            assert diff.max() == 0.0
    B.spd_destroy(ctx)


def test_pack_rejects_values_that_are_not_bf16():
    w = SMALL_BF16
    ctx = B.spd_create(B.make_config(w))
    shard = inputs.layer_shard(w, 0, 0)
    shard["wd"][3, 5] = np.float32(1.0 + 2.0 ** -12)
    with pytest.raises(B.SpdError) as e:
        B.spd_pack_shard_local(ctx, shard)
    assert e.value.code == B.SPD_EINVAL
    B.spd_destroy(ctx)


@pytest.mark.parametrize("w", [SMALL_BF16, SMALL_F32])
def test_kv_pack_roundtrip(w):
    ctx = B.spd_create(B.make_config(w))
    sizes = B.spd_get_sizes(ctx)
    k, v = inputs.kv_prefill(w, 0, 1, w.batch, 37 if w.dtype == workloads.BF16 else 20)
    cache = np.zeros(sizes.kv_bytes, dtype=np.uint8)
    B.spd_kv_pack(ctx, k, v, cache)
    k2, v2 = B.spd_kv_unpack(ctx, cache, w.batch, k.shape[2], w.kv_per_rank, w.head_dim)
    assert np.array_equal(k, k2) and np.array_equal(v, v2)
    # positions beyond n_pos stay zero
    k3, v3 = B.spd_kv_unpack(ctx, cache, w.batch, k.shape[2] + 5, w.kv_per_rank, w.head_dim)
    assert not k3[:, :, k.shape[2]:].any() and not v3[:, :, k.shape[2]:].any()
    B.spd_destroy(ctx)


def test_forward_calls_reject_bad_arguments_before_any_launch():
    # fake, suitably aligned addresses: every one of these calls must fail on the host
    w = SMALL_BF16
    ctx = B.spd_create(B.make_config(w))
    P = 0x10000
    ok = dict(ctx=ctx, layer=0, spd_flag=1, rank=0, packed_weights=P, kv_cache=P, positions=[0, 0], batch=2,
              q_len=4, x_in=P, slots=P, x_out=P, workspace=P, stream=0)

    def call(**over):
        a = dict(ok); a.update(over)
        with pytest.raises(B.SpdError) as e:
            B.spd_block_forward(**a)
        return e.value.code

    assert call(rank=2) == B.SPD_EINVAL
    assert call(rank=-2) == B.SPD_EINVAL
    assert call(spd_flag=2) == B.SPD_EINVAL
    assert call(layer=3) == B.SPD_EINVAL
    assert call(batch=3, positions=[0, 0, 0]) == B.SPD_EINVAL          # > max_batch
    assert call(q_len=5) == B.SPD_EINVAL                               # > max_tokens
    assert call(positions=[0, 61]) == B.SPD_EINVAL                     # 61 + 4 > max_ctx
    assert call(positions=[-1, 0]) == B.SPD_EINVAL
    assert call(x_in=P + 4) == B.SPD_EINVAL                            # misaligned
    for name in ("packed_weights", "kv_cache", "x_in", "slots", "x_out", "workspace"):
        assert call(**{name: None}) == B.SPD_EINVAL, name

    okm = dict(ctx=ctx, spd_mask=[1, 0, 1], rank=0, layer_weights=[P] * 3, layer_kv=[P] * 3, positions=[0, 0],
               batch=2, q_len=4, x_in=P, slots=P, x_out=P, workspace=P, stream=0)

    def callm(**over):
        a = dict(okm); a.update(over)
        with pytest.raises(B.SpdError) as e:
            B.spd_model_forward(**a)
        return e.value.code

    assert callm(spd_mask=[1, 2, 0]) == B.SPD_EINVAL
    assert callm(rank=5) == B.SPD_EINVAL
    assert callm(layer_weights=[P, None, P]) == B.SPD_EINVAL
    assert callm(positions=[0, 62]) == B.SPD_EINVAL
    # empty calls are valid no-ops
    B.spd_block_forward(**dict(ok, batch=0, positions=[]))
    assert B.spd_model_forward(**dict(okm, q_len=0)) == 0
    with pytest.raises(B.SpdError):
        B.spd_rank_sum(ctx, None, None, 2, 16, P, stream=0)
    B.spd_rank_sum(ctx, None, None, 0, 0, P, stream=0)                 # zero elements: nothing to do
    B.spd_destroy(ctx)


def test_inputs_are_counter_based():
    w = SMALL_BF16
    a = inputs.hidden_states(w, 6)
    b = inputs.hidden_states(w, 2, first_token=3)
    assert np.array_equal(a[3:5], b)
    s0, s1 = inputs.layer_shard(w, 0, 0), inputs.layer_shard(w, 0, 1)
    assert not np.array_equal(s0["wq"], s1["wq"]) and np.array_equal(s0["g1"], s1["g1"])
    bits = s0["wq"].view(np.uint32)
    assert not (bits & 0xFFFF).any()                                   # bf16-representable
    x = inputs.normal((200000,), 1, inputs.T_MISC)
    assert abs(float(x.mean())) < 0.01 and abs(float(x.std()) - 1.0) < 0.01


# ------------------------------------------------------------------------------------------------
# launch order of the GEMM tiles: every tile exactly once, for whole and ragged grids, for the launch
# pair that finishes a ragged last round with half tiles, and runs of neighbours per XCD
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("TN,TM,rn,rm", [(28, 32, 256, 256), (32, 32, 256, 256), (1, 3, 256, 256), (5, 9, 256, 256),
                                         (10, 22, 128, 384), (7, 33, 256, 256), (56, 3, 128, 384), (3, 2, 128, 384),
                                         (40, 40, 256, 256), (1, 1, 256, 256), (9, 29, 256, 128)])
def test_gemm_tile_order_covers_every_tile_once(TN, TM, rn, rm):
    total = TN * TM
    # the launch plan of the library: one launch, or whole rounds + a second launch over the rest (that one
    # walks its tiles one after the other in the library; any dealing of the same set covers the same tiles)
    rem = total % 256
    plans = [[(0, total)]]
    if total > 256 and 0 < rem <= 128:
        plans.append([(0, total - rem), (total - rem, rem)])
    for plan in plans:
        seen = {}
        for li, (tile0, n_tiles) in enumerate(plan):
            n_wgs = B.spd_gemm_launch_size(n_tiles)
            assert n_wgs % 8 == 0 and n_tiles <= n_wgs < n_tiles + 64
            spare = 0
            for b in range(n_wgs):
                t = B.spd_gemm_tile_of(TN, TM, rn, rm, tile0, n_tiles, b)
                if t is None:
                    spare += 1
                    continue
                assert 0 <= t[0] < TN and 0 <= t[1] < TM
                assert t not in seen, (t, b, seen[t])
                seen[t] = (li, b)
            assert spare == n_wgs - n_tiles
        assert len(seen) == total


def test_gemm_tile_order_keeps_an_xcd_on_neighbours():
    """Gate/up of the 70B shard (28 x 32 tiles of 256 x 256): the 32 tiles an XCD has in flight in a round
    form one block of 4 x 8, i.e. 12 operand panels, and the eight blocks of a round are consecutive."""
    TN, TM, n = 28, 32, 768
    for rnd in range(3):
        blocks = []
        for x in range(8):
            tiles = [B.spd_gemm_tile_of(TN, TM, 256, 256, 0, n, rnd * 256 + 8 * q + x) for q in range(32)]
            ns, ms = {t[0] for t in tiles}, {t[1] for t in tiles}
            assert len(ns) == 4 and len(ms) == 8 and len(set(tiles)) == 32
            blocks.append((min(ms) // 8, min(ns) // 4))
        order = [bm * 7 + bn for bm, bn in blocks]
        assert order == list(range(order[0], order[0] + 8))


def test_gemm_tile_order_rejects():
    assert B.lib().spd_gemm_launch_size(-1) == B.SPD_EINVAL
    import ctypes as C
    tn, tm = C.c_int32(), C.c_int32()
    f = B.lib().spd_gemm_tile_of
    assert f(4, 4, 256, 256, 0, 16, 16, C.byref(tn), C.byref(tm)) == B.SPD_EINVAL      # workgroup past the launch
    assert f(4, 4, 256, 256, 8, 16, 0, C.byref(tn), C.byref(tm)) == B.SPD_EINVAL       # more tiles than the matrix has
    assert f(0, 4, 256, 256, 0, 0, 0, C.byref(tn), C.byref(tm)) == B.SPD_EINVAL
    assert f(4, 4, 256, 256, 0, 16, 0, None, C.byref(tm)) == B.SPD_EINVAL
