"""GPU parity: the HIP library, called through the C ABI, against the CPU oracle on the same
seeded inputs.  bf16 path: max abs error 2e-2 on the fp32-stored block outputs; fp32 path:
1e-3 relative; integer logic (sync counts, rank indexing) bit-exact."""
import numpy as np
import pytest

from oracle import spd_oracle as O
from paper_2502_20727_amd import binding as B
from paper_2502_20727_amd import inputs, workloads
from paper_2502_20727_amd.workloads import BF16, F32, Workload

from helpers import Case, assert_close, cache_storage, oracle_shapes

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------------------------------------
# rank-sum: the kept sync point
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n_slots,n,with_base", [(0, 64, True), (1, 7, True), (2, 1024, False), (8, 4099, True),
                                                 (8, 16 * 8192, True), (3, 1, False)])
def test_rank_sum(gpu, n_slots, n, with_base):
    import torch
    ctx = B.spd_create(B.make_config(workloads.TOY, max_ctx=64))
    rng = np.random.default_rng(n_slots * 1000 + n)
    slots = rng.standard_normal((max(n_slots, 1), n)).astype(np.float32)
    base = rng.standard_normal(n).astype(np.float32) if with_base else None
    d_slots = torch.from_numpy(slots).to(gpu)
    d_base = torch.from_numpy(base).to(gpu) if with_base else None
    out = torch.full((n,), 7.0, dtype=torch.float32, device=gpu)
    B.spd_rank_sum(ctx, d_base, d_slots, n_slots, n, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    # contract: partials in ascending slot order, base last, all in fp32 -> bit-exact
    acc = np.zeros(n, np.float32)
    if n_slots:
        acc = slots[0].copy()
        for s in range(1, n_slots):
            acc = acc + slots[s]
    want32 = (base + acc) if with_base else acc
    assert np.array_equal(got, want32.astype(np.float32))
    want64 = O.rank_sum(base, slots[:n_slots]) if n_slots else (np.asarray(base, np.float64) if with_base else np.zeros(n))
    assert np.max(np.abs(got - want64)) <= 1e-5 * max(1.0, float(np.max(np.abs(want64))))
    B.spd_destroy(ctx)


# ------------------------------------------------------------------------------------------------
# configuration 0: the fp32 toy model, all ranks emulated, prefill 32 + 8 single-token steps
# ------------------------------------------------------------------------------------------------
def test_toy_fp32_prefill_then_decode(gpu):
    import torch
    w = workloads.TOY
    case = Case(w, gpu, ranks=range(w.tp), positions=[0], max_ctx=64, max_tokens=32)
    X = inputs.hidden_states(w, 40)
    slots = torch.zeros((w.tp, 32, w.hidden), dtype=torch.float32, device=gpu)
    out = torch.empty((32, w.hidden), dtype=torch.float32, device=gpu)
    syncs = B.spd_model_forward(case.dev.ctx, w.mask, B.SPD_ALL_RANKS, case.dev.weights, case.dev.kv, [0], 1, 32,
                                case.to_dev(X[:32]), slots, out, case.dev.workspace)
    torch.cuda.synchronize()
    want, osyncs = O.model_all_ranks(case.sh, X[:32], case.shards, case.caches, [0], 1, 32, w.mask)
    assert syncs == osyncs == 3                        # mask [1, 0]: 1 + 2 sync points
    err = assert_close(out.cpu().numpy(), want, w, "toy prefill")
    say(f"toy prefill: max err {err:.2e}, max |oracle| {np.max(np.abs(want)):.2f}")
    for t in range(32, 40):                            # teacher-forced single-token steps
        o1 = torch.empty((1, w.hidden), dtype=torch.float32, device=gpu)
        B.spd_model_forward(case.dev.ctx, w.mask, B.SPD_ALL_RANKS, case.dev.weights, case.dev.kv, [t], 1, 1,
                            case.to_dev(X[t:t + 1]), slots, o1, case.dev.workspace)
        torch.cuda.synchronize()
        want, _ = O.model_all_ranks(case.sh, X[t:t + 1], case.shards, case.caches, [t], 1, 1, w.mask)
        assert_close(o1.cpu().numpy(), want, w, f"toy decode step {t}")
    case.close()


def _block_with_taps(case, li, flag, rank_arg, x_dev, slots, batch, q_len, positions):
    import torch
    w = case.w
    M = batch * q_len
    qd = w.q_per_rank * w.head_dim
    taps = dict(q=torch.zeros((M, qd), dtype=torch.float32, device=x_dev.device),
                attn=torch.zeros((M, qd), dtype=torch.float32, device=x_dev.device),
                y=torch.zeros((M, w.hidden), dtype=torch.float32, device=x_dev.device),
                u=torch.zeros((M, w.ffn_per_rank), dtype=torch.float32, device=x_dev.device))
    out = torch.empty((M, w.hidden), dtype=torch.float32, device=x_dev.device)
    B.spd_block_forward(case.dev.ctx, li, flag, rank_arg, case.dev.weights[li], case.dev.kv[li], positions, batch,
                        q_len, x_dev, slots, out, case.dev.workspace, taps=taps)
    torch.cuda.synchronize()
    return out, {k: v.cpu().numpy() for k, v in taps.items()}


def _check_taps(taps, det, w, what):
    # bf16-stored intermediates carry one rounding of their own: half an ulp (2^-9 relative) on top
    for name, key in (("q", "Q"), ("attn", "A"), ("y", "Y"), ("u", "U")):
        want = det[key]
        scale = 1.0 + float(np.max(np.abs(want))) * (2.0 ** -8) / 2e-2 if w.dtype == BF16 else 1.0
        assert_close(taps[name], want, w, f"{what} tap {name}", scale=scale)


def test_toy_fp32_block_intermediates(gpu):
    import torch
    w = workloads.TOY
    for flag in (1, 0):
        case = Case(w, gpu, ranks=range(w.tp), positions=[0], max_ctx=64, max_tokens=32)
        X = inputs.hidden_states(w, 32)
        slots = torch.zeros((w.tp, 32, w.hidden), dtype=torch.float32, device=gpu)
        out, taps = _block_with_taps(case, 0, flag, B.SPD_ALL_RANKS, case.to_dev(X), slots, 1, 32, [0])
        det = {}
        want, _ = O.block_all_ranks(case.sh, X, case.shards[0], case.caches[0], [0], 1, 32, flag, det)
        assert_close(out.cpu().numpy(), want, w, f"toy block flag={flag}")
        # the taps belong to the last rank run
        d2 = {}
        c2 = O.KVCache(1, w.kv_per_rank, 64, w.head_dim)
        r = w.tp - 1
        Y = O.attention_partial(case.sh, X, case.shards[0][r], c2, [0], 1, 32, detail=d2)
        R = X + (Y if flag else sum(det["Y"]))
        O.mlp_partial(case.sh, R, case.shards[0][r], d2)
        d2["Y"] = Y
        _check_taps(taps, d2, w, f"toy flag={flag}")
        # slots hold what meets at the final sync point
        got_slots = slots.cpu().numpy()
        for i in range(w.tp):
            assert_close(got_slots[i], det["P"][i], w, f"toy slot {i} flag={flag}")
        case.close()


# ------------------------------------------------------------------------------------------------
# bf16 path, small shapes, all ranks: several tiles, ragged tails, ragged positions
# ------------------------------------------------------------------------------------------------
SMALL = Workload(name="small-bf16", hidden=256, n_q_heads=8, n_kv_heads=4, head_dim=64, ffn=832, n_layers=2,
                 tp=4, dtype=BF16, seed=11, batch=3, q_len=1, ctx=64, mask=(1, 0))
SMALL_MHA = Workload(name="small-bf16-mha", hidden=128, n_q_heads=4, n_kv_heads=4, head_dim=128, ffn=256,
                     n_layers=1, tp=2, dtype=BF16, seed=12, batch=2, q_len=1, ctx=64, mask=(1,))


# 3200 FFN columns per rank: 200 tiles of 16 do not fill the chip evenly, so decode-sized calls read the
# copy of the gate/up weights with 13-column groups (247 groups, the last one with 2 real columns)
NARROW_GU = Workload(name="narrow-gate-up", hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=6400, n_layers=1,
                     tp=2, dtype=BF16, seed=14, batch=3, q_len=1, ctx=64, mask=(1,))


# 2080 FFN columns per rank (130 pairs of gate/up tiles: 17 groups of 8, the last with 2) and 37 k-tiles
# (19 stages of two, the last with one, in 4 slices of 4 or 5): a call of 17 .. 128 tokens takes the
# gate/up kernel that shares the activations through LDS and cuts K into slices
WIDE_MID = Workload(name="wide-ffn-mid", hidden=1184, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=4160, n_layers=1,
                    tp=2, dtype=BF16, seed=17, batch=2, q_len=1, ctx=64, mask=(1,))


# head sizes other than LLaMA2's 128 and the small shapes' 64: 96 (six 16-wide slices per head, three rotary tile
# pairs) and 32 (two slices), with grouped KV heads
SMALL_D96 = Workload(name="small-bf16-d96", hidden=256, n_q_heads=8, n_kv_heads=4, head_dim=96, ffn=512, n_layers=1,
                     tp=2, dtype=BF16, seed=21, batch=3, q_len=1, ctx=64, mask=(1,))
SMALL_D32 = Workload(name="small-bf16-d32", hidden=128, n_q_heads=8, n_kv_heads=2, head_dim=32, ffn=256, n_layers=1,
                     tp=2, dtype=BF16, seed=22, batch=3, q_len=1, ctx=64, mask=(1,))


@pytest.mark.parametrize("w", [SMALL, SMALL_MHA, NARROW_GU, WIDE_MID, SMALL_D96, SMALL_D32], ids=lambda w: w.name)
@pytest.mark.parametrize("batch,q_len,positions", [
    (3, 1, [0, 17, 40]),          # decode, ragged contexts, one sequence with a single key
    (2, 7, [0, 5]),               # 14 tokens: a partial m-tile
    (2, 10, [0, 4]),              # 20 tokens: two m-tiles
    (3, 11, [3, 0, 20]),          # 33 tokens: three m-tiles with a ragged tail
    (1, 40, [8]),                 # one long chunk crossing several key blocks
    (2, 50, [0, 5]),              # 100 tokens: seven m-tiles, the last one ragged
    (3, 50, [0, 5, 14]),          # 150 tokens: two groups of 8 m-tiles per projection, the second one partly empty
], ids=["decode", "chunk14", "chunk20", "chunk33", "chunk40", "chunk100", "chunk150"])
@pytest.mark.parametrize("flag", [1, 0], ids=["spd", "tp"])
def test_bf16_small_all_ranks(gpu, w, batch, q_len, positions, flag):
    import torch
    M = batch * q_len
    case = Case(w, gpu, ranks=range(w.tp), positions=positions, max_ctx=64, max_tokens=max(48, M))
    X = inputs.hidden_states(w, M)
    slots = torch.zeros((w.tp, M, w.hidden), dtype=torch.float32, device=gpu)
    say(f"case {w.name} batch={batch} q_len={q_len} pos={positions} flag={flag}")
    out, taps = _block_with_taps(case, 0, flag, B.SPD_ALL_RANKS, case.to_dev(X), slots, batch, q_len, positions)
    det = {}
    want, _ = O.block_all_ranks(case.sh, X, case.shards[0], case.caches[0], positions, batch, q_len, flag, det)
    r = w.tp - 1
    d2 = {}
    c2 = O.KVCache(batch, w.kv_per_rank, 64, w.head_dim, storage=cache_storage(w))
    c2.k[...] = 0
    # the last rank's intermediates: recompute them with a cache holding the same prefill
    if max(positions) > 0:
        k, v = inputs.kv_prefill(w, 0, r, batch, max(positions))
        for b, p in enumerate(positions):
            k[b, :, p:, :] = 0.0
            v[b, :, p:, :] = 0.0
        c2.fill(k, v)
    Y = O.attention_partial(case.sh, X, case.shards[0][r], c2, positions, batch, q_len, detail=d2)
    O.mlp_partial(case.sh, X + (Y if flag else sum(det["Y"])), case.shards[0][r], d2)
    d2["Y"] = Y
    _check_taps(taps, d2, w, "small")
    err = assert_close(out.cpu().numpy(), want, w, "small block output")
    say(f"  block output max err {err:.2e} (max |oracle| {np.max(np.abs(want)):.2f})")
    # the appended keys / values: bf16 copies of the oracle's
    for i, rr in enumerate(case.ranks):
        n_pos = max(positions) + q_len
        k, v = case.dev.read_kv(0, i, batch, n_pos)
        for b, p in enumerate(positions):
            ko, vo = case.caches[0][i].k[b, :, p:p + q_len], case.caches[0][i].v[b, :, p:p + q_len]
            # both sides hold bf16 values; a last-bit disagreement is one ulp (2^-7 relative at most)
            assert np.max(np.abs(k[b, :, p:p + q_len] - ko)) <= 2.0 ** -7 * np.max(np.abs(ko)) + 1e-3
            assert np.max(np.abs(v[b, :, p:p + q_len] - vo)) <= 2.0 ** -7 * np.max(np.abs(vo)) + 1e-3
    case.close()


SMALL_H512 = Workload(name="small-bf16-h512", hidden=512, n_q_heads=8, n_kv_heads=4, head_dim=64, ffn=832, n_layers=1,
                      tp=4, dtype=BF16, seed=18, batch=3, q_len=1, ctx=64, mask=(1,))


@pytest.mark.parametrize("w", [SMALL, SMALL_H512, SMALL_MHA, SMALL_D96, SMALL_D32], ids=lambda w: w.name)
@pytest.mark.parametrize("flag", [1, 0], ids=["spd", "tp"])
@pytest.mark.parametrize("split", [B.SPD_SPLIT_AUTO, B.SPD_SPLIT_ALWAYS, B.SPD_SPLIT_NEVER], ids=["default", "all-split", "no-split"])
def test_bf16_long_call_small_shape(gpu, w, flag, split):
    """More than 512 tokens in one call on a small shape, all ranks: the launch shapes of the long
    prefill (LDS-tiled GEMM, key-split attention, row-wise norm preparation) with a ragged last
    m-tile, every output element checked (hidden size 256 and 512: one and two pieces of 256 features per
    workgroup of the row-wise preparation; the 128-wide shape takes the 256 x 256 tiles with their block-wise
    numbering, most of whose blocks stick out of so small a matrix)."""
    import torch
    batch, q_len, positions = 3, 181, [0, 0, 0]          # 543 tokens = 33 m-tiles + 15 rows
    M = batch * q_len
    case = Case(w, gpu, ranks=range(w.tp), positions=positions, max_ctx=192, max_tokens=M, act_split=split)
    X = inputs.hidden_states(w, M)
    slots = torch.zeros((w.tp, M, w.hidden), dtype=torch.float32, device=gpu)
    say(f"long call on the small shape: {M} tokens flag={flag} split={split}")
    out = torch.empty((M, w.hidden), dtype=torch.float32, device=gpu)
    B.spd_block_forward(case.dev.ctx, 0, flag, B.SPD_ALL_RANKS, case.dev.weights[0], case.dev.kv[0], positions, batch,
                        q_len, case.to_dev(X), slots, out, case.dev.workspace)
    torch.cuda.synchronize()
    want, _ = O.block_all_ranks(case.sh, X, case.shards[0], case.caches[0], positions, batch, q_len, flag, {})
    err = assert_close(out.cpu().numpy(), want, w, "long call block output")
    say(f"  block output max err {err:.2e} (max |oracle| {np.max(np.abs(want)):.2f})")
    case.close()


# ------------------------------------------------------------------------------------------------
# block with bias in the output projection (Sec. 4.1.2): both paths, both block kinds
# ------------------------------------------------------------------------------------------------
TOY_BIAS = Workload(name="toy-f32-bias", hidden=128, n_q_heads=4, n_kv_heads=2, head_dim=32, ffn=344, n_layers=3, tp=2,
                    dtype=F32, seed=15, batch=2, q_len=1, ctx=32, mask=(1, 0, 1))
SMALL_BIAS = Workload(name="small-bf16-bias", hidden=256, n_q_heads=8, n_kv_heads=4, head_dim=64, ffn=832, n_layers=3,
                      tp=4, dtype=BF16, seed=16, batch=3, q_len=1, ctx=64, mask=(1, 0, 1))


SMALL_BIAS8 = Workload(name="small-bf16-bias-tp8", hidden=256, n_q_heads=16, n_kv_heads=8, head_dim=32, ffn=1024, n_layers=3,
                       tp=8, dtype=BF16, seed=17, batch=3, q_len=1, ctx=64, mask=(1, 0, 1))


@pytest.mark.parametrize("w", [TOY_BIAS, SMALL_BIAS, SMALL_BIAS8], ids=lambda w: w.name)
@pytest.mark.parametrize("batch,q_len,positions",
                         [(3, 1, [0, 9, 30]), (2, 10, [0, 4]), (2, 40, [0, 8]), (3, 181, [0, 3, 0]), (2, 1030, [0, 8])],
                         ids=["decode", "chunk20", "chunk80", "chunk543", "chunk2060"])
@pytest.mark.parametrize("mode", ["all-ranks", "one-rank"])
def test_block_with_bias(gpu, w, batch, q_len, positions, mode):
    """Three blocks (SPD, TP, SPD) with a bias of the size of the activations on the output projection:
    model forward against the oracle, with every rank emulated and from one rank's point of view (whose bf16 call
    of 2 x 1030 tokens runs as two chains, the bias joining the rank-sums of their preparation kernel: four slots in
    the 4-way shard, eight in the 8-way one)."""
    import torch
    M = batch * q_len
    ranks = list(range(w.tp)) if mode == "all-ranks" else [1]
    case = Case(w, gpu, ranks=ranks, positions=positions, max_ctx=max(64, (max(positions) + q_len + 31) // 32 * 32), max_tokens=max(48, M),
                bias_std=1.0)
    X = inputs.hidden_states(w, M)
    say(f"case {w.name} {mode} batch={batch} q_len={q_len}")
    peers = inputs.peer_slots(w, M) if mode == "one-rank" else np.zeros((w.tp, M, w.hidden), np.float32)
    slots = case.to_dev(peers).reshape(w.tp, M, w.hidden)
    out = torch.empty((M, w.hidden), dtype=torch.float32, device=gpu)
    taps = torch.zeros((w.n_layers, M, w.hidden), dtype=torch.float32, device=gpu)
    syncs = B.spd_model_forward_staged(case.dev.ctx, w.mask, case.dev.rank_arg(), case.dev.weights, case.dev.kv,
                                       positions, batch, q_len, case.to_dev(X), slots, out, case.dev.workspace,
                                       layer_out=taps)
    torch.cuda.synchronize()
    assert syncs == 4
    got = taps.cpu().numpy()
    assert np.array_equal(got[-1], out.cpu().numpy())
    # block by block, the oracle's block fed the same input as the library's: the bound as it stands
    worst = 0.0
    o_slots = peers.astype(np.float64)
    for l in range(w.n_layers):
        x_in = X if l == 0 else got[l - 1]
        if mode == "all-ranks":
            want, _ = O.block_all_ranks(case.sh, x_in, case.shards[l], case.caches[l], positions, batch, q_len, w.mask[l])
        else:
            want = O.block_single_rank(case.sh, x_in, case.shards[l][0], case.caches[l][0], positions, batch, q_len,
                                       w.mask[l], 1, o_slots)
        worst = max(worst, assert_close(got[l], want, w, f"{w.name} {mode} block {l}"))
    say(f"  worst block max err {worst:.2e}")
    case.close()


# ------------------------------------------------------------------------------------------------
# bf16 path, one rank of eight with peer slots as inputs, several layers, mixed mask
# ------------------------------------------------------------------------------------------------
MID = Workload(name="mid-bf16", hidden=1024, n_q_heads=32, n_kv_heads=8, head_dim=128, ffn=11008, n_layers=4,
               tp=8, dtype=BF16, seed=13, batch=5, q_len=1, ctx=256, mask=(1, 0, 1, 1))


@pytest.mark.parametrize("batch,q_len,positions", [(5, 1, [255, 100, 0, 31, 64]), (2, 24, [0, 100])],
                         ids=["decode", "chunk"])
def test_bf16_single_rank_model(gpu, batch, q_len, positions):
    import torch
    w, rank = MID, 3
    M = batch * q_len
    case = Case(w, gpu, ranks=[rank], positions=positions, max_ctx=256, max_tokens=48)
    X = inputs.hidden_states(w, M)
    peers = inputs.peer_slots(w, M)
    # per layer: oracle fed the GPU's layer input
    x = case.to_dev(X)
    slots = case.to_dev(peers)
    worst = 0.0
    for l in range(w.n_layers):
        x_host = x.cpu().numpy()
        out = torch.empty_like(x)
        B.spd_block_forward(case.dev.ctx, l, w.mask[l], rank, case.dev.weights[l], case.dev.kv[l], positions, batch,
                            q_len, x, slots, out, case.dev.workspace)
        torch.cuda.synchronize()
        o_slots = peers.astype(np.float64)
        want = O.block_single_rank(case.sh, x_host, case.shards[l][0], case.caches[l][0], positions, batch, q_len,
                                   w.mask[l], rank, o_slots)
        worst = max(worst, assert_close(out.cpu().numpy(), want, w, f"mid layer {l}"))
        # the slot this rank wrote must be what the oracle's rank contributes to the last sync point
        assert_close(slots[rank].cpu().numpy(), o_slots[rank], w, f"mid slot layer {l}")
        # peers untouched, bit for bit
        for i in range(w.tp):
            if i != rank:
                assert np.array_equal(slots[i].cpu().numpy(), peers[i])
        x = out
    say(f"mid {q_len=}: worst per-layer err {worst:.2e}")
    chain = x.cpu().numpy()

    # end to end through spd_model_forward on fresh caches.  It fuses each block's closing rank-sum
    # into the down projection, so the norm statistics are added in another (fixed) order than in
    # the block-by-block chain: equal up to rounding, not bit for bit
    case2 = Case(w, gpu, ranks=[rank], positions=positions, max_ctx=256, max_tokens=48)
    slots2 = case2.to_dev(peers)
    out2 = torch.empty((M, w.hidden), dtype=torch.float32, device=gpu)
    syncs = B.spd_model_forward(case2.dev.ctx, w.mask, rank, case2.dev.weights, case2.dev.kv, positions, batch, q_len,
                                case2.to_dev(X), slots2, out2, case2.dev.workspace)
    torch.cuda.synchronize()
    assert syncs == B.spd_sync_count(case2.dev.ctx, w.mask) == 5
    assert np.max(np.abs(out2.cpu().numpy() - chain)) <= 2e-3
    chain = out2.cpu().numpy()
    want = O.model_single_rank(case2.sh, X, [s[0] for s in case2.shards], [c[0] for c in case2.caches], positions,
                               batch, q_len, w.mask, rank, peers.astype(np.float64))
    err = float(np.max(np.abs(chain - want)))
    rms = float(np.sqrt(np.mean(want ** 2)))
    say(f"mid end-to-end over {w.n_layers} layers: max err {err:.2e}, output rms {rms:.2f}")
    assert err <= 2e-2 * w.n_layers * max(1.0, rms)
    # run twice: bit-identical (fixed summation orders, no float atomics)
    case3 = Case(w, gpu, ranks=[rank], positions=positions, max_ctx=256, max_tokens=48)
    out3 = torch.empty_like(out2)
    B.spd_model_forward(case3.dev.ctx, w.mask, rank, case3.dev.weights, case3.dev.kv, positions, batch, q_len,
                        case3.to_dev(X), case3.to_dev(peers), out3, case3.dev.workspace)
    torch.cuda.synchronize()
    assert np.array_equal(out3.cpu().numpy(), chain)
    for c in (case, case2, case3):
        c.close()


def test_bf16_prefill_then_decode_matches_longer_prefill(gpu):
    """KV-cache consistency on the device: 20 tokens at once == 12 at once + 8 one by one."""
    import torch
    w = SMALL
    X = inputs.hidden_states(w, 20)
    full = Case(w, gpu, ranks=range(w.tp), positions=[0], max_ctx=64, max_tokens=32)
    slots = torch.zeros((w.tp, 20, w.hidden), dtype=torch.float32, device=gpu)
    o_full = torch.empty((20, w.hidden), dtype=torch.float32, device=gpu)
    B.spd_model_forward(full.dev.ctx, w.mask, B.SPD_ALL_RANKS, full.dev.weights, full.dev.kv, [0], 1, 20,
                        full.to_dev(X), slots, o_full, full.dev.workspace)
    step = Case(w, gpu, ranks=range(w.tp), positions=[0], max_ctx=64, max_tokens=32)
    o_head = torch.empty((12, w.hidden), dtype=torch.float32, device=gpu)
    B.spd_model_forward(step.dev.ctx, w.mask, B.SPD_ALL_RANKS, step.dev.weights, step.dev.kv, [0], 1, 12,
                        step.to_dev(X[:12]), slots, o_head, step.dev.workspace)
    torch.cuda.synchronize()
    want, _ = O.model_all_ranks(full.sh, X, full.shards, full.caches, [0], 1, 20, w.mask)
    assert_close(o_full.cpu().numpy(), want, w, "20-token chunk")
    assert_close(o_head.cpu().numpy(), want[:12], w, "12-token chunk")
    for t in range(12, 20):
        o1 = torch.empty((1, w.hidden), dtype=torch.float32, device=gpu)
        B.spd_model_forward(step.dev.ctx, w.mask, B.SPD_ALL_RANKS, step.dev.weights, step.dev.kv, [t], 1, 1,
                            step.to_dev(X[t:t + 1]), slots, o1, step.dev.workspace)
        torch.cuda.synchronize()
        assert_close(o1.cpu().numpy()[0], want[t], w, f"step {t}")
    full.close()
    step.close()


def test_edge_cases(gpu):
    import torch
    w = SMALL
    # maximum position: the last slot of the cache; and maximum batch
    case = Case(w, gpu, ranks=[1], positions=[63, 0, 63], max_ctx=64, max_tokens=16)
    X = inputs.hidden_states(w, 3)
    peers = inputs.peer_slots(w, 3)
    slots = case.to_dev(peers)
    out = torch.empty((3, w.hidden), dtype=torch.float32, device=gpu)
    B.spd_block_forward(case.dev.ctx, 0, 1, 1, case.dev.weights[0], case.dev.kv[0], [63, 0, 63], 3, 1,
                        case.to_dev(X), slots, out, case.dev.workspace)
    torch.cuda.synchronize()
    want = O.block_single_rank(case.sh, X, case.shards[0][0], case.caches[0][0], [63, 0, 63], 3, 1, 1, 1,
                               peers.astype(np.float64))
    assert_close(out.cpu().numpy(), want, w, "max position")
    # empty call: nothing is launched, the output buffer is left alone
    out.fill_(5.0)
    B.spd_block_forward(case.dev.ctx, 0, 1, 1, case.dev.weights[0], case.dev.kv[0], [], 0, 1,
                        case.to_dev(X), slots, out, case.dev.workspace)
    torch.cuda.synchronize()
    assert float(out.min()) == 5.0
    # x_out may alias x_in
    x = case.to_dev(X)
    case_b = Case(w, gpu, ranks=[1], positions=[63, 0, 63], max_ctx=64, max_tokens=16)
    B.spd_block_forward(case_b.dev.ctx, 0, 0, 1, case_b.dev.weights[0], case_b.dev.kv[0], [63, 0, 63], 3, 1,
                        x, case_b.to_dev(peers), x, case_b.dev.workspace)
    torch.cuda.synchronize()
    want = O.block_single_rank(case_b.sh, X, case_b.shards[0][0], case_b.caches[0][0], [63, 0, 63], 3, 1, 0, 1,
                               peers.astype(np.float64))
    assert_close(x.cpu().numpy(), want, w, "aliased output")
    case.close()
    case_b.close()
    # 64 sequences in one call
    w64 = Workload(name="b64", hidden=128, n_q_heads=4, n_kv_heads=2, head_dim=32, ffn=128, n_layers=1, tp=2,
                   dtype=BF16, seed=14, batch=64, q_len=1, ctx=32, mask=(1,))
    pos = [(7 * i) % 32 for i in range(64)]
    c64 = Case(w64, gpu, ranks=range(2), positions=pos, max_ctx=32, max_tokens=64)
    X = inputs.hidden_states(w64, 64)
    slots = torch.zeros((2, 64, 128), dtype=torch.float32, device=gpu)
    out = torch.empty((64, 128), dtype=torch.float32, device=gpu)
    B.spd_block_forward(c64.dev.ctx, 0, 1, B.SPD_ALL_RANKS, c64.dev.weights[0], c64.dev.kv[0], pos, 64, 1,
                        c64.to_dev(X), slots, out, c64.dev.workspace)
    torch.cuda.synchronize()
    want, _ = O.block_all_ranks(c64.sh, X, c64.shards[0], c64.caches[0], pos, 64, 1, 1)
    assert_close(out.cpu().numpy(), want, w64, "64 sequences")
    c64.close()


def test_long_context_decode(gpu):
    """Decode steps against caches of 16383, 9000 and 31 positions in one call (capacity 16384): the attention
    kernel cuts the context into as many splits as it may and merges them; one rank of four."""
    import torch
    w, rank = SMALL, 2
    positions = [16383, 9000, 31]
    case = Case(w, gpu, ranks=[rank], positions=positions, max_ctx=16384, max_tokens=16)
    X = inputs.hidden_states(w, 3)
    peers = inputs.peer_slots(w, 3)
    slots = case.to_dev(peers)
    out = torch.empty((3, w.hidden), dtype=torch.float32, device=gpu)
    say("long-context decode, positions", positions)
    for l, flag in enumerate(w.mask):
        x_in = X if l == 0 else out.cpu().numpy()
        B.spd_block_forward(case.dev.ctx, l, flag, rank, case.dev.weights[l], case.dev.kv[l], positions, 3, 1,
                            case.to_dev(x_in), slots, out, case.dev.workspace)
        torch.cuda.synchronize()
        want = O.block_single_rank(case.sh, x_in, case.shards[l][0], case.caches[l][0], positions, 3, 1, flag, rank,
                                   peers.astype(np.float64))
        err = assert_close(out.cpu().numpy(), want, w, f"long context block {l}")
        say(f"  block {l}: max err {err:.2e}")
    case.close()


# ------------------------------------------------------------------------------------------------
# full-size shapes through spd_block_forward (2 layers each: the first as an SPD block, the last as a TP block);
# the call the bench makes, spd_model_forward at full depth, is checked at the end of this file
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["7b-decode", "13b-decode", "70b-decode", "7b-tp4-decode", "13b-tp4-decode"])
def test_full_size_decode_shapes(gpu, name):
    import torch
    full = workloads.get(name)
    w = full.with_layers(2).with_mask((1, 0))
    layer_ids = [0, full.n_layers - 1]
    positions = [full.ctx - 1] * full.batch
    say(f"full-size {name}: batch {full.batch}, ctx {full.ctx}")
    case = Case(w, gpu, ranks=[0], positions=positions, layer_ids=layer_ids)
    M = full.batch
    X = inputs.hidden_states(w, M)
    peers = inputs.peer_slots(w, M)
    x = case.to_dev(X)
    slots = case.to_dev(peers)
    for l in range(2):
        x_host = x.cpu().numpy()
        out = torch.empty_like(x)
        B.spd_block_forward(case.dev.ctx, l, w.mask[l], 0, case.dev.weights[l], case.dev.kv[l], positions, M, 1, x,
                            slots, out, case.dev.workspace)
        torch.cuda.synchronize()
        want = O.block_single_rank(case.sh, x_host, case.shards[l][0], case.caches[l][0], positions, M, 1, w.mask[l],
                                   0, peers.astype(np.float64))
        err = assert_close(out.cpu().numpy(), want, w, f"{name} layer {layer_ids[l]} flag {w.mask[l]}")
        say(f"  layer {layer_ids[l]} flag {w.mask[l]}: max err {err:.2e}, max |oracle| {np.max(np.abs(want)):.2f}")
        x = out
    case.close()


@pytest.mark.parametrize("batch", [24, 48, 64])
def test_full_size_large_batch_decode(gpu, batch):
    """LLaMA2-70B shard, one decode step of 24 / 48 / 64 sequences at ragged positions of a 1024-position cache: the
    projections take the kernels for 17 to 512 tokens, the QKV one on a single activation plane (a decode step
    attends to one new key per sequence).  An SPD block and a TP block, every row at the 2e-2 bound."""
    import torch
    from dataclasses import replace
    full = replace(workloads.get("70b-decode"), batch=batch, ctx=1024)
    w = full.with_layers(2).with_mask((1, 0))
    positions = [int(p) for p in np.random.default_rng(batch).integers(0, full.ctx, size=batch)]
    positions[0], positions[-1] = full.ctx - 1, 0
    say(f"full-size decode, batch {batch}")
    case = Case(w, gpu, ranks=[0], positions=positions, layer_ids=[0, workloads.get("70b-decode").n_layers - 1])
    X = inputs.hidden_states(w, batch)
    peers = inputs.peer_slots(w, batch)
    x, slots = case.to_dev(X), case.to_dev(peers)
    for l in range(2):
        x_host = x.cpu().numpy()
        out = torch.empty_like(x)
        B.spd_block_forward(case.dev.ctx, l, w.mask[l], 0, case.dev.weights[l], case.dev.kv[l], positions, batch, 1, x,
                            slots, out, case.dev.workspace)
        torch.cuda.synchronize()
        want = O.block_single_rank(case.sh, x_host, case.shards[l][0], case.caches[l][0], positions, batch, 1, w.mask[l],
                                   0, peers.astype(np.float64))
        err = assert_close(out.cpu().numpy(), want, w, f"decode batch {batch} flag {w.mask[l]}")
        say(f"  flag {w.mask[l]}: max err {err:.2e}, max |oracle| {np.max(np.abs(want)):.2f}")
        x = out
    case.close()
    torch.cuda.empty_cache()


@pytest.mark.parametrize("q_len", [128, 200, 500])
def test_full_size_short_prefill(gpu, q_len):
    """LLaMA2-70B shard, one sequence of 128 tokens (the shape of the paper's latency breakdown,
    Fig. 2), an SPD block then a TP block, every output row checked at the 2e-2 bound as it
    stands, in the default configuration (the one the bench times).  200 and 500 tokens: from 145
    tokens on the QKV and down projections take the kernel that shares the activations through LDS
    (the QKV one on its hi + lo input pair), with ragged last m-tiles."""
    import torch
    from dataclasses import replace
    full = workloads.get("70b-prefill-128")
    full = replace(full, q_len=q_len, ctx=(q_len + 31) // 32 * 32)
    w = full.with_layers(2).with_mask((1, 0))
    M = full.q_len
    case = Case(w, gpu, ranks=[0], positions=[0], layer_ids=[0, full.n_layers - 1])
    X = inputs.hidden_states(w, M)
    peers = inputs.peer_slots(w, M)
    x, slots = case.to_dev(X), case.to_dev(peers)
    say(f"full-size short prefill: 1 x {M} tokens")
    for l in range(2):
        x_host = x.cpu().numpy()
        out = torch.empty_like(x)
        B.spd_block_forward(case.dev.ctx, l, w.mask[l], 0, case.dev.weights[l], case.dev.kv[l], [0], 1, M, x, slots, out,
                            case.dev.workspace)
        torch.cuda.synchronize()
        want = O.block_single_rank(case.sh, x_host, case.shards[l][0], case.caches[l][0], [0], 1, M, w.mask[l], 0,
                                   peers.astype(np.float64))
        err = assert_close(out.cpu().numpy(), want, w, f"short prefill layer {l}")
        say(f"  flag {w.mask[l]}: max err {err:.2e}, max |oracle| {np.max(np.abs(want)):.2f}")
        x = out
    # the same two blocks through spd_model_forward (the call the bench makes: the down projection's epilogue then
    # carries the closing sync point and the next block's norm preparation), block by block against the oracle
    case2 = Case(w, gpu, ranks=[0], positions=[0], layer_ids=[0, full.n_layers - 1])
    taps = torch.zeros((2, M, w.hidden), dtype=torch.float32, device=gpu)
    out2 = torch.empty((M, w.hidden), dtype=torch.float32, device=gpu)
    syncs = B.spd_model_forward_staged(case2.dev.ctx, w.mask, 0, case2.dev.weights, case2.dev.kv, [0], 1, M, case2.to_dev(X),
                                       case2.to_dev(peers), out2, case2.dev.workspace, layer_out=taps)
    torch.cuda.synchronize()
    assert syncs == 3
    got = taps.cpu().numpy()
    for l in range(2):
        x_in = X if l == 0 else got[l - 1]
        want = O.block_single_rank(case2.sh, x_in, case2.shards[l][0], case2.caches[l][0], [0], 1, M, w.mask[l], 0,
                                   peers.astype(np.float64))
        err = assert_close(got[l], want, w, f"short prefill, model forward, layer {l}")
        say(f"  model forward, flag {w.mask[l]}: max err {err:.2e}")
    case2.close()
    case.close()


@pytest.mark.parametrize("q_len", [700, 1100, 2048])
def test_full_size_single_sequence_prefill(gpu, q_len):
    """LLaMA2-70B shard, one sequence of 700 / 1100 / 2048 tokens: a single chain, whose QKV GEMM (24, 40 or 64 tiles
    for 256 compute units) runs in 8 or 4 K slices side by side, the slices' partial rows added by the gather kernel;
    at 700 tokens the other projections run as 256 x 128 half tiles throughout (a ragged last one).  An SPD
    block and a TP block, sampled output rows against the oracle at 2e-2."""
    import torch
    from dataclasses import replace
    full = replace(workloads.LLAMA70B_PREFILL, batch=1, q_len=q_len, ctx=(q_len + 31) // 32 * 32)
    w = full.with_layers(2).with_mask((1, 0))
    M = q_len
    rows = np.unique(np.concatenate([np.array([0, 1, 15, 16, 255, 256, 511, 512, 640, M - 17, M - 1]),
                                     np.random.default_rng(5).choice(M, size=54, replace=False)]))
    X = inputs.hidden_states(w, M)
    peers = inputs.peer_slots(w, M)
    say(f"full-size single-sequence prefill: 1 x {M} tokens")
    case = Case(w, gpu, ranks=[0], positions=[0], layer_ids=[0, workloads.LLAMA70B_PREFILL.n_layers - 1])
    x, slots = case.to_dev(X), case.to_dev(peers)
    sel = torch.from_numpy(rows).to(gpu)
    for l in range(2):
        x_host = x.cpu().numpy()
        out = torch.empty_like(x)
        B.spd_block_forward(case.dev.ctx, l, w.mask[l], 0, case.dev.weights[l], case.dev.kv[l], [0], 1, M, x, slots, out,
                            case.dev.workspace)
        torch.cuda.synchronize()
        want = O.block_single_rank(case.sh, x_host, case.shards[l][0], case.caches[l][0], [0], 1, M, w.mask[l], 0,
                                   peers.astype(np.float64), rows=rows)
        err = assert_close(out[sel].cpu().numpy(), want, w, f"single-sequence prefill layer {l}")
        say(f"  flag {w.mask[l]}: max err {err:.2e} on {len(rows)} sampled rows")
        assert bool(torch.isfinite(out).all())
        x = out
    # the appended keys and values of the first block, all positions: bf16 copies of the oracle's
    k, v = case.dev.read_kv(0, 0, 1, M)
    ko, vo = case.caches[0][0].k[0, :, :M], case.caches[0][0].v[0, :, :M]
    assert np.max(np.abs(k[0] - ko)) <= 2.0 ** -7 * np.max(np.abs(ko)) + 1e-3
    assert np.max(np.abs(v[0] - vo)) <= 2.0 ** -7 * np.max(np.abs(vo)) + 1e-3
    case.close()
    torch.cuda.empty_cache()


@pytest.mark.parametrize("flag", [1, 0], ids=["spd", "tp"])
@pytest.mark.parametrize("split", [B.SPD_SPLIT_AUTO, B.SPD_SPLIT_ALWAYS], ids=["default", "all-split"])
def test_full_size_prefill_shape_sampled_rows(gpu, flag, split):
    """LLaMA2-70B shard, 4 x 2048 tokens, the launch configuration the bench times (and, beside
    it, the one with every projection input split): the oracle computes sampled output rows one
    by one; the 2e-2 bound as it stands."""
    import torch
    full = workloads.LLAMA70B_PREFILL
    w = full.with_layers(1).with_mask((flag,))
    M = full.batch * full.q_len
    rows = np.unique(np.concatenate([
        np.array([0, 1, 15, 16, 17, 255, 256, 2047, 2048, 2049, 3000, 4095, 4096, 5555, 6143, 6144, 8000, 8191]),
        np.random.default_rng(7).choice(M, size=110, replace=False)]))
    X = inputs.hidden_states(w, M)
    peers = inputs.peer_slots(w, M)
    say(f"full-size prefill flag={flag} split={split}")
    case = Case(w, gpu, ranks=[0], positions=[0] * full.batch, act_split=split)
    x = case.to_dev(X)
    slots = case.to_dev(peers)
    out = torch.empty_like(x)
    B.spd_block_forward(case.dev.ctx, 0, flag, 0, case.dev.weights[0], case.dev.kv[0], [0] * full.batch,
                        full.batch, full.q_len, x, slots, out, case.dev.workspace)
    torch.cuda.synchronize()
    got = out[torch.from_numpy(rows).to(gpu)].cpu().numpy()
    del x, out
    want = O.block_single_rank(case.sh, X, case.shards[0][0], case.caches[0][0], [0] * full.batch, full.batch,
                               full.q_len, flag, 0, peers, rows=rows)
    rms = float(np.sqrt(np.mean(want ** 2)))
    worst = np.max(np.abs(got - want), axis=1)
    say("  largest per-row max err:", " ".join(f"{rows[i]}:{worst[i]:.1e}" for i in np.argsort(worst)[-6:]))
    err = assert_close(got, want, w, f"prefill rows flag={flag} split={split}")
    say(f"  {len(rows)} sampled rows: max err {err:.2e}, max |oracle| {np.max(np.abs(want)):.2f}, rms {rms:.2f}")
    if split == B.SPD_SPLIT_AUTO:
        # what the bench launches: spd_model_forward (two chains of 2 x 2048 tokens on two streams) replayed from a
        # HIP graph; the same sampled rows against the same oracle rows
        x = case.to_dev(X)
        slots_g = case.to_dev(peers)
        out_g = torch.empty_like(x)
        graph = _capture(torch, lambda: B.spd_model_forward(case.dev.ctx, w.mask, 0, case.dev.weights, case.dev.kv,
                                                            [0] * full.batch, full.batch, full.q_len, x, slots_g, out_g,
                                                            case.dev.workspace))
        out_g.fill_(-1.0)
        graph.replay()
        torch.cuda.synchronize()
        got_g = out_g[torch.from_numpy(rows).to(gpu)].cpu().numpy()
        err_g = assert_close(got_g, want, w, f"prefill rows, two chains under a graph, flag={flag}")
        say(f"  two chains replayed from a graph: max err {err_g:.2e}; against the one-chain block call {np.max(np.abs(got_g - got)):.2e}")
        assert bool(torch.isfinite(out_g).all())
        del graph, x, out_g, slots_g
    # properties that hold at any size: peers' slots untouched; finite everywhere
    assert np.array_equal(slots[5][:64].cpu().numpy(), peers[5][:64])
    assert bool(torch.isfinite(slots[0]).all())
    del slots
    case.close()
    torch.cuda.empty_cache()


# ------------------------------------------------------------------------------------------------
# the prefill call the bench makes, several blocks deep: two chains, each block's closing sync point
# preparing the next block's first norm
# ------------------------------------------------------------------------------------------------
def test_full_size_prefill_model_forward_three_blocks(gpu):
    """LLaMA2-70B shard, 4 x 2048 tokens through spd_model_forward (two chains of 2 x 2048 on two streams) over
    three blocks with mask (1, 0, 1): every block's output on sampled rows against the oracle's block fed the
    input the library's block had (all rows of it: the keys and values of every token matter), 2e-2 each."""
    import torch
    full = workloads.LLAMA70B_PREFILL
    w = full.with_layers(3).with_mask((1, 0, 1))
    batch, q_len = full.batch, full.q_len
    M = batch * q_len
    positions = [0] * batch
    rows = np.unique(np.concatenate([np.array([0, 15, 16, 2047, 2048, 4095, 4096, 6144, 8191]),
                                     np.random.default_rng(11).choice(M, size=40, replace=False)]))
    X = inputs.hidden_states(w, M)
    peers = inputs.peer_slots(w, M)
    say(f"full-size prefill, model forward over {w.n_layers} blocks, mask {w.mask}")
    case = Case(w, gpu, ranks=[0], positions=positions)
    x, slots = case.to_dev(X), case.to_dev(peers)
    out = torch.empty_like(x)
    taps = torch.zeros((w.n_layers, M, w.hidden), dtype=torch.float32, device=gpu)
    syncs = B.spd_model_forward_staged(case.dev.ctx, w.mask, 0, case.dev.weights, case.dev.kv, positions, batch, q_len, x,
                                       slots, out, case.dev.workspace, layer_out=taps)
    torch.cuda.synchronize()
    assert syncs == B.spd_sync_count(case.dev.ctx, w.mask) == 4
    assert bool(torch.equal(taps[-1], out))
    sel = torch.from_numpy(rows).to(gpu)
    worst = 0.0
    for l in range(w.n_layers):
        x_in = X if l == 0 else taps[l - 1].cpu().numpy()
        want = O.block_single_rank(case.sh, x_in, case.shards[l][0], case.caches[l][0], positions, batch, q_len,
                                   int(w.mask[l]), 0, peers.astype(np.float64), rows=rows)
        err = assert_close(taps[l][sel].cpu().numpy(), want, w, f"prefill model forward block {l} (mask {w.mask[l]})")
        say(f"  block {l}: max err {err:.2e} on {len(rows)} sampled rows")
        worst = max(worst, err)
    del taps, x, out, slots
    case.close()
    torch.cuda.empty_cache()


# ------------------------------------------------------------------------------------------------
# the call the bench makes: spd_model_forward at full depth with the workload's own mask
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name,n_syncs", [("7b-decode", 32), ("13b-decode", 50), ("70b-decode", 96)])
def test_full_depth_model_forward(gpu, name, n_syncs):
    """Rank 0's share of the whole model (32 / 40 / 80 blocks, the workload's mask: all SPD, every 4th
    block synced, SPD on blocks 8..71) through spd_model_forward, the call the bench times, where each
    block's closing sync point also prepares the next block's first norm.  Every block's output is
    compared with the oracle's block fed the same input (2e-2 as it stands); the whole chain is compared
    with the oracle's own chain relative to the output's rms."""
    import torch
    w = workloads.get(name)
    M, positions = w.batch, [w.ctx - 1] * w.batch
    say(f"full depth {name}: {w.n_layers} blocks, mask sum {sum(w.mask)}, batch {w.batch}, ctx {w.ctx}")
    dev = B.DeviceShard(w, [0], gpu)
    n_pre = w.ctx - 1
    for l in range(w.n_layers):
        dev.load_layer(l, [inputs.layer_shard(w, l, 0)])
        dev.load_kv(l, [inputs.kv_prefill(w, l, 0, w.batch, n_pre)])
    X = inputs.hidden_states(w, M)
    peers = inputs.peer_slots(w, M)
    x, slots = torch.from_numpy(X).to(gpu), torch.from_numpy(peers).to(gpu)
    out = torch.empty_like(x)
    taps = torch.zeros((w.n_layers, M, w.hidden), dtype=torch.float32, device=gpu)
    syncs = B.spd_model_forward_staged(dev.ctx, w.mask, 0, dev.weights, dev.kv, positions, w.batch, 1, x, slots, out,
                                       dev.workspace, layer_out=taps)
    torch.cuda.synchronize()
    assert syncs == B.spd_sync_count(dev.ctx, w.mask) == n_syncs
    got = taps.cpu().numpy()
    assert np.array_equal(got[-1], out.cpu().numpy())
    # the launch configuration the bench times: the same call replayed from a HIP graph (twice, into another
    # output buffer) gives the eager result bit for bit
    out_g = torch.empty_like(x)
    slots_g = torch.from_numpy(peers).to(gpu)
    graph = _capture(torch, lambda: B.spd_model_forward(dev.ctx, w.mask, 0, dev.weights, dev.kv, positions, w.batch, 1, x,
                                                        slots_g, out_g, dev.workspace))
    for rep in range(2):
        out_g.fill_(-1.0)
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(out_g.cpu().numpy(), got[-1]), f"graph replay {rep} differs from the eager forward"
    del graph
    dev.close()
    del dev, taps
    torch.cuda.empty_cache()

    sh = oracle_shapes(w)
    mc = (w.ctx + 31) // 32 * 32
    o_slots = peers.astype(np.float64)
    chain = X.astype(np.float64)
    worst, worst_l = 0.0, -1
    for l in range(w.n_layers):
        shard = inputs.layer_shard(w, l, 0)
        k, v = inputs.kv_prefill(w, l, 0, w.batch, n_pre)
        cache = O.KVCache(w.batch, w.kv_per_rank, mc, w.head_dim, storage=cache_storage(w))
        cache.fill(k, v)
        x_in = X if l == 0 else got[l - 1]
        want = O.block_single_rank(sh, x_in, shard, cache.copy(), positions, w.batch, 1, int(w.mask[l]), 0, o_slots)
        err = assert_close(got[l], want, w, f"{name} block {l} (mask {w.mask[l]})")
        if err > worst:
            worst, worst_l = err, l
        chain = O.block_single_rank(sh, chain, shard, cache, positions, w.batch, 1, int(w.mask[l]), 0, o_slots)
    rms = float(np.sqrt(np.mean(chain ** 2)))
    e2e = float(np.max(np.abs(got[-1] - chain)))
    say(f"  worst block {worst_l}: max err {worst:.2e}; end to end: max err {e2e:.2e}, output rms {rms:.2f}, "
        f"relative {e2e / rms:.2e}")
    # errors of the blocks add up along the chain (each at most 2e-2, amplified or damped by what follows):
    # the end-to-end figure is reported relative to the output's rms and bounded by the sum of the per-block bounds
    assert e2e <= 2e-2 * w.n_layers * max(1.0, rms)


# ------------------------------------------------------------------------------------------------
# a long prefill of several sequences: spd_model_forward runs it as two chains on two streams
# ------------------------------------------------------------------------------------------------
TWO_CHAIN = Workload(name="two-chain-bf16", hidden=256, n_q_heads=8, n_kv_heads=4, head_dim=64, ffn=832, n_layers=3,
                     tp=4, dtype=BF16, seed=19, batch=3, q_len=1100, ctx=1120, mask=(1, 0, 1))


def test_bf16_two_chain_prefill(gpu):
    """Three sequences of 1100 tokens (the second one continuing after 5 cached positions): the model
    forward cuts the call into a chain of two sequences and a chain of one and runs them on two streams.
    Every block's output is checked against the oracle's block fed the same input, and the result against
    what the blocks give one after the other on one stream (spd_block_forward)."""
    import torch
    w, rank = TWO_CHAIN, 1
    batch, q_len, positions = w.batch, w.q_len, [0, 5, 0]
    M = batch * q_len
    X = inputs.hidden_states(w, M)
    peers = inputs.peer_slots(w, M)
    case = Case(w, gpu, ranks=[rank], positions=positions, max_ctx=w.ctx, max_tokens=M)
    x, slots = case.to_dev(X), case.to_dev(peers)
    out = torch.empty_like(x)
    taps = torch.zeros((w.n_layers, M, w.hidden), dtype=torch.float32, device=gpu)
    say(f"two-chain prefill: {batch} x {q_len} tokens")
    syncs = B.spd_model_forward_staged(case.dev.ctx, w.mask, rank, case.dev.weights, case.dev.kv, positions, batch, q_len,
                                       x, slots, out, case.dev.workspace, layer_out=taps)
    torch.cuda.synchronize()
    assert syncs == B.spd_sync_count(case.dev.ctx, w.mask) == 4
    got = taps.cpu().numpy()
    assert np.array_equal(got[-1], out.cpu().numpy())
    # the same blocks one after the other, one chain
    ref = Case(w, gpu, ranks=[rank], positions=positions, max_ctx=w.ctx, max_tokens=M)
    xr, sr = ref.to_dev(X), ref.to_dev(peers)
    for l in range(w.n_layers):
        o = torch.empty_like(xr)
        B.spd_block_forward(ref.dev.ctx, l, w.mask[l], rank, ref.dev.weights[l], ref.dev.kv[l], positions, batch, q_len, xr,
                            sr, o, ref.dev.workspace)
        xr = o
    torch.cuda.synchronize()
    # (not bit for bit: which kernel runs a projection depends on the number of tokens of the call or chain, and
    # the kernels add up K in different orders)
    d = float(np.max(np.abs(xr.cpu().numpy() - got[-1])))
    say(f"  two chains vs one chain of blocks: max difference {d:.2e}")
    assert d <= 2e-3
    assert float(np.max(np.abs(sr.cpu().numpy() - slots.cpu().numpy()))) <= 2e-3
    for l in (0, w.n_layers - 1):
        k0, v0 = case.dev.read_kv(l, 0, batch, max(positions) + q_len)
        k1, v1 = ref.dev.read_kv(l, 0, batch, max(positions) + q_len)
        # bf16 values on both sides; a last-bit disagreement is one unit in the last place
        assert np.max(np.abs(k0 - k1)) <= 2.0 ** -7 * np.max(np.abs(k1)) and np.max(np.abs(v0 - v1)) <= 2.0 ** -7 * np.max(np.abs(v1))
    ref.close()
    # block by block against the oracle
    o_slots = peers.astype(np.float64)
    worst = 0.0
    for l in range(w.n_layers):
        x_in = X if l == 0 else got[l - 1]
        want = O.block_single_rank(case.sh, x_in, case.shards[l][0], case.caches[l][0], positions, batch, q_len, w.mask[l],
                                   rank, o_slots)
        worst = max(worst, assert_close(got[l], want, w, f"two-chain block {l}"))
    say(f"  worst block max err {worst:.2e}")
    case.close()


# ------------------------------------------------------------------------------------------------
# the launch configuration bench.py times: the whole-model forward replayed from a HIP graph
# ------------------------------------------------------------------------------------------------
def _capture(torch, fn):
    """fn() captured into a graph on a side stream, the way bench.py does it."""
    stream = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    side.wait_stream(stream)
    with torch.cuda.stream(side):
        fn()
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            fn()
    stream.wait_stream(side)
    torch.cuda.synchronize()
    return graph


@pytest.mark.parametrize("kind", ["decode", "two-chain-prefill"])
def test_graph_replays_equal_the_eager_forward(gpu, kind):
    """spd_model_forward captured into a HIP graph and replayed three times, each time on new hidden states written
    into the same buffers, with the library's own eager forward between the replays: every replay must equal the
    eager result on the same inputs bit for bit (the path is deterministic).  The two-chain prefill records
    its second chain on the library's helper stream into the same graph."""
    import torch
    if kind == "decode":
        w, rank, batch, q_len = MID, 3, 2, 1
        positions = [100, 37]
        case = Case(w, gpu, ranks=[rank], positions=positions, max_ctx=256, max_tokens=48)
    else:
        w, rank, batch, q_len = TWO_CHAIN, 1, TWO_CHAIN.batch, TWO_CHAIN.q_len
        positions = [0, 5, 0]
        case = Case(w, gpu, ranks=[rank], positions=positions, max_ctx=w.ctx, max_tokens=batch * q_len)
    M = batch * q_len
    X = inputs.hidden_states(w, M)
    peers = inputs.peer_slots(w, M)
    x = case.to_dev(X)
    slots, slots_e = case.to_dev(peers), case.to_dev(peers)
    out, out_e = torch.empty_like(x), torch.empty_like(x)

    def run(o, sl):
        return B.spd_model_forward(case.dev.ctx, w.mask, rank, case.dev.weights, case.dev.kv, positions, batch, q_len, x, sl, o,
                                   case.dev.workspace)

    graph = _capture(torch, lambda: run(out, slots))
    for rep in range(3):
        say(f"graph replay {rep} ({kind})")
        x.copy_(torch.from_numpy(X * (1.0 + 0.25 * rep)).to(gpu))         # new inputs in the captured buffers
        out.fill_(-1.0)
        graph.replay()
        torch.cuda.synchronize()
        got, got_slot = out.cpu().numpy().copy(), slots[rank].cpu().numpy().copy()
        out_e.fill_(-2.0)
        run(out_e, slots_e)                                                # eager, same inputs, other output buffers
        torch.cuda.synchronize()
        assert np.isfinite(got).all()
        assert np.array_equal(got, out_e.cpu().numpy()), f"replay {rep} differs from the eager forward"
        assert np.array_equal(got_slot, slots_e[rank].cpu().numpy())
    case.close()


@pytest.mark.gpu
def test_mfma_probe_reports_a_plausible_rate():
    """The benchmark aid runs and lands between a tenth of and the whole nominal fp16 MFMA peak, at a clock the chip has."""
    import torch
    scratch = torch.empty(B.SPD_MFMA_PROBE_SCRATCH_BYTES, dtype=torch.uint8, device="cuda:0")
    for random_data in (True, False):
        tf, mhz = B.spd_mfma_probe(2000, random_data, scratch)
        assert 250.0 < tf < 2600.0, (random_data, tf)
        assert 500.0 < mhz < 2600.0, (random_data, mhz)


def test_read_probe_reports_a_plausible_rate(gpu):
    """The benchmark aid runs: 64 MiB per launch from 8 distinct buffers, between 1 and 8 TB/s."""
    import torch
    chunk = 64 << 20
    buf = torch.zeros(8 * chunk, dtype=torch.uint8, device=gpu)
    sink = torch.zeros(4, dtype=torch.float32, device=gpu)
    us = B.spd_read_probe(buf, chunk, 8, 16, sink)
    rate = chunk / (us * 1e-6) / 1e12
    say(f"read probe: {us:.2f} us per 64 MiB = {rate:.2f} TB/s")
    assert 1.0 < rate < 8.0
    assert float(sink.sum()) == 0.0
