"""The entry point that allocates nothing (spd_block_forward_static) against spd_block_forward on
the same seeded inputs: two calls in a row through the C ABI, the second one smaller, so that the
second runs on whatever the first left in the library's static scratch."""
import numpy as np
import pytest

from paper_2502_20727_amd import binding as B
from paper_2502_20727_amd import inputs, workloads
from paper_2502_20727_amd.workloads import BF16, F32, Workload

from helpers import Case, assert_close

pytestmark = pytest.mark.gpu

BF = Workload(name="static-bf16", hidden=256, n_q_heads=8, n_kv_heads=4, head_dim=64, ffn=832, n_layers=1,
              tp=4, dtype=BF16, seed=21, batch=3, q_len=1, ctx=64, mask=(1,))
FP = Workload(name="static-f32", hidden=128, n_q_heads=4, n_kv_heads=2, head_dim=32, ffn=344, n_layers=1, tp=2,
              dtype=F32, seed=22, batch=2, q_len=1, ctx=64, mask=(1,))


def _run(gpu, w, rank, flag, static, calls):
    """The calls in a row on one context and one KV cache, through one of the two entry points."""
    import torch
    case = Case(w, gpu, ranks=[rank], positions=calls[0][2], max_ctx=64, max_tokens=48)
    res = []
    for batch, q_len, positions in calls:
        M = batch * q_len
        x, slots = case.to_dev(inputs.hidden_states(w, M)), case.to_dev(inputs.peer_slots(w, M))
        out = torch.empty_like(x)
        if static:
            B.spd_block_forward_static(case.dev.ctx, 0, flag, rank, case.dev.weights[0], case.dev.kv[0], positions,
                                       batch, q_len, x, slots, out)
        else:
            B.spd_block_forward(case.dev.ctx, 0, flag, rank, case.dev.weights[0], case.dev.kv[0], positions, batch,
                                q_len, x, slots, out, case.dev.workspace)
        torch.cuda.synchronize()
        res.append((out.cpu().numpy(), slots.cpu().numpy(), case.dev.read_kv(0, 0, batch, max(positions) + q_len)))
    case.close()
    return res


@pytest.mark.parametrize("w", [BF, FP], ids=lambda w: w.name)
@pytest.mark.parametrize("flag", [1, 0], ids=["spd", "tp"])
def test_static_entry_point_matches_the_ordinary_one(gpu, w, flag):
    rank = 1
    # 33 tokens in one call, then a smaller call (the next token of each sequence) on what the first left in
    # the scratch; same context, same cache.  The parametrisations alternate contexts of different shapes,
    # so the array changes owner between them.
    calls = [(3, 11, [3, 0, 20]), (3, 1, [14, 11, 31])]
    ref = _run(gpu, w, rank, flag, False, calls)
    got = _run(gpu, w, rank, flag, True, calls)
    for (batch, q_len, _), (o_ref, s_ref, kv_ref), (o_st, s_st, kv_st) in zip(calls, ref, got):
        err = assert_close(o_st, o_ref, w, f"static vs ordinary, {batch}x{q_len}")
        assert_close(s_st[rank], s_ref[rank], w, "own slot")
        for i in range(w.tp):
            if i != rank:
                assert np.array_equal(s_st[i], s_ref[i])         # peers untouched by both
        assert_close(kv_st[0], kv_ref[0], w, "appended keys")
        assert_close(kv_st[1], kv_ref[1], w, "appended values")
        print(f"static entry point {w.name} flag={flag} {batch}x{q_len}: max |static - ordinary| {err:.2e}, "
              f"bit-identical: {np.array_equal(o_st, o_ref)}", flush=True)


def test_static_entry_point_rejects_what_does_not_fit(gpu):
    """A configuration whose workspace exceeds the static scratch is refused before anything is launched."""
    import torch
    w = workloads.LLAMA70B_PREFILL.with_layers(1)
    ctx = B.spd_create(B.make_config(w))
    assert B.spd_get_sizes(ctx).workspace_bytes > B.SPD_STATIC_WORKSPACE_BYTES
    dummy = torch.zeros(64, dtype=torch.float32, device=gpu)
    with pytest.raises(B.SpdError) as e:
        B.spd_block_forward_static(ctx, 0, 1, 0, dummy, dummy, [0], 1, 1, dummy, dummy, dummy)
    assert e.value.code == B.SPD_ETOOBIG
    B.spd_destroy(ctx)
