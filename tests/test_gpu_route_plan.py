"""moin_route_plan through the C ABI: routing and grouping in one call must leave the ids and the plan
that the two separate calls leave -- ids exact, and the planned linear layer's output bit for bit that of a
plan built on its own, and within the oracle's bars."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_09687_amd import moin
from paper_2410_09687_amd import workloads as wl
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu


def _batch(N, K, D, E, lens, d_in, d_out, r, seed):
    rin = wl.make_route_inputs(wl.RouteWorkload("rp", N, K, D, "bf16", True, seed), "cuda")
    slots = torch.from_numpy(wl.retained_slot_table(K, E, seed=seed + 1)).cuda()
    lin = wl.make_linear_inputs(wl.LinearWorkload("rp", d_in, d_out, r, E, lens, "uniform", seed=seed + 2), "cuda")
    return rin, slots, lin


# request-sized prefill (one launch), decode-sized (one launch, tokens grouped), an empty sequence in the mix,
# more queries than ride in the routing launch (two launches), D not a multiple of 64 (generic router)
@pytest.mark.parametrize("N,K,D,E,lens,dims", [
    (24, 700, 128, 600, None, (128, 192, 16)),
    (64, 300, 64, 280, "decode", (256, 128, 16)),
    (7, 1000, 192, 900, "ragged", (64, 64, 8)),
    (512, 260, 64, 200, "decode", (128, 64, 8)),
    (600, 260, 64, 200, "decode", (128, 64, 8)),
    (33, 90, 40, 90, None, (64, 128, 8)),
])
def test_one_call_equals_route_then_plan(N, K, D, E, lens, dims):
    rng = np.random.default_rng(N + K)
    if lens == "decode":
        lens = [1] * N
    elif lens == "ragged":
        lens = [0, 300, 1, 0, 129, 64, 5][:N]
    else:
        lens = rng.integers(1, 200, size=N).tolist()
    d_in, d_out, r = dims
    rin, slots, lin = _batch(N, K, D, E, lens, d_in, d_out, r, seed=N * 3 + K)
    ctx = gc.ctx()
    T = lin.wl.T
    print(f"[gpu] route+plan N={N} K={K} D={D} E={E} T={T}", flush=True)
    ranks = torch.from_numpy(np.where(np.arange(E) % 3 == 0, r // 2 // 8 * 8, r).astype(np.int32)).cuda()
    for rank_of_expert in (None, ranks):
        e_ref, c_ref, cnt_ref = moin.moin_route(ctx, rin.emb, rin.centroids, slot_of_centroid=slots, want_counts=True)
        plan_ref = moin.Plan(ctx).build(lin.seq_offsets, e_ref, T, E, rank_of_expert=rank_of_expert)
        y_ref = moin.moin_lora_linear_planned(ctx, plan_ref, lin.x, lin.W, lin.A_stack, lin.B_stack, 2.0)
        ctx.check()
        plan = moin.Plan(ctx)
        for rep in range(2):     # the second call on scratch the first one left
            e, c, cnt = moin.moin_route_plan(ctx, plan, rin.emb, rin.centroids, lin.seq_offsets, T, E,
                                             slot_of_centroid=slots, rank_of_expert=rank_of_expert,
                                             want_centroid_ids=True, want_counts=True, same_centroids=(rep > 0))
            y = moin.moin_lora_linear_planned(ctx, plan, lin.x, lin.W, lin.A_stack, lin.B_stack, 2.0)
            ctx.check()
            assert torch.equal(e, e_ref) and torch.equal(c, c_ref) and torch.equal(cnt, cnt_ref)
            assert torch.equal(y, y_ref)
        plan.close()
        plan_ref.close()
    gc.check_route(rin.emb, rin.centroids, c_ref)
    assert np.array_equal(e_ref.cpu().numpy(), oracle.slot_map(c_ref.cpu().numpy(), slots.cpu().numpy()))
    # (ranked plans are covered against the oracle elsewhere; here the full-rank result)
    y_full = moin.moin_lora_linear(ctx, lin.x, lin.seq_offsets, e_ref, lin.W, lin.A_stack, lin.B_stack, 2.0)
    ctx.check()
    lin.expert_ids = e_ref
    gc.compare_linear(y_full, gc.oracle_rows(lin), what="route+plan")


def test_centroid_indices_as_ids_and_argument_errors():
    # no slot map: the ids are centroid indices, so the stacks must have K entries
    N, K, D = 16, 40, 64
    rin = wl.make_route_inputs(wl.RouteWorkload("rp", N, K, D, "bf16", True, 5), "cuda")
    lin = wl.make_linear_inputs(wl.LinearWorkload("rp", 64, 64, 8, K, [3] * N, "uniform", seed=6), "cuda")
    ctx = gc.ctx()
    plan = moin.Plan(ctx)
    e, _, _ = moin.moin_route_plan(ctx, plan, rin.emb, rin.centroids, lin.seq_offsets, lin.wl.T, K)
    y = moin.moin_lora_linear_planned(ctx, plan, lin.x, lin.W, lin.A_stack, lin.B_stack, 2.0)
    ctx.check()
    gc.check_route(rin.emb, rin.centroids, e)
    assert torch.equal(y, moin.moin_lora_linear(ctx, lin.x, lin.seq_offsets, e, lin.W, lin.A_stack, lin.B_stack, 2.0))
    with pytest.raises(moin.MoinError):      # E smaller than K with ids that are centroid indices
        moin.moin_route_plan(ctx, plan, rin.emb, rin.centroids, lin.seq_offsets, lin.wl.T, K - 1)
    with pytest.raises(ValueError):          # one offset per query, plus one
        moin.moin_route_plan(ctx, plan, rin.emb, rin.centroids, lin.seq_offsets[:-1].contiguous(), lin.wl.T, K)
    # an empty batch builds an empty plan
    e, _, _ = moin.moin_route_plan(ctx, plan, rin.emb[:0], rin.centroids, lin.seq_offsets[:1].contiguous(), 0, K)
    assert e.numel() == 0
    ctx.check()
    plan.close()
