"""Projections of a layer that read the same input (q, k, v; gate, up) through one call: the bits of the single
planned calls, whichever path the batch takes."""
import numpy as np
import pytest
import torch

from paper_2410_09687_amd import moin
from paper_2410_09687_amd import workloads as wl
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu


def _projections(d_in, d_outs, r, E, lens, ids, seed):
    inps = []
    for i, d_out in enumerate(d_outs):
        w = wl.LinearWorkload(f"shared{i}", d_in, d_out, r, E, lens, "uniform", scale=2.0, seed=seed + i)
        inps.append(wl.make_linear_inputs(w, "cuda", expert_ids=np.asarray(ids, np.int32)))
    return inps


@pytest.mark.parametrize("d_in,r,d_outs", [(256, 128, (264, 136, 136)), (256, 64, (520, 72)), (384, 192, (136, 264, 72, 8)),
                                           (328, 24, (264, 136))])
def test_shared_input_equals_single_calls(d_in, r, d_outs):
    lens = [300, 1, 0, 257, 255, 512, 77, 256, 3, 640]
    ids = [3, 0, 5, -1, 3, 6, 2, 2, -1, 1]
    inps = _projections(d_in, d_outs, r, 7, lens, ids, seed=600 + r)
    x = inps[0].x
    ctx = gc.ctx()
    plan = moin.Plan(ctx).build(inps[0].seq_offsets, inps[0].expert_ids, inps[0].wl.T, 7)
    for dt in (torch.bfloat16, torch.float32):
        print(f"[gpu] shared input d_in={d_in} r={r} n={len(d_outs)} y={dt}", flush=True)
        single = [moin.moin_lora_linear_planned(ctx, plan, x, i.W, i.A_stack, i.B_stack, 2.0, y_dtype=dt) for i in inps]
        ys = moin.moin_lora_linear_planned_shared(ctx, plan, x, [i.W for i in inps], [i.A_stack for i in inps],
                                                  [i.B_stack for i in inps], 2.0, y_dtype=dt)
        ctx.check()
        for a, b in zip(single, ys):
            assert torch.equal(a, b)
    # the first projection against the oracle as well
    inp0 = wl.LinearInputs(inps[0].wl, x, inps[0].W, inps[0].A_stack, inps[0].B_stack, inps[0].seq_offsets,
                           inps[0].expert_ids)
    gc.compare_linear(ys[0], gc.oracle_rows(inp0), what="shared/first")
    plan.close()


@pytest.mark.parametrize("d_in,r,d_outs,T", [
    (256, 64, (136, 264), 100),            # two projections, one base part each
    (2048, 128, (264, 264), 256),          # gate / up shaped: two base parts, full-rank fast path
    (2048, 128, (520, 72, 72), 77),        # q / k / v shaped: widths that differ
    (512, 40, (264, 136, 72, 8), 300),     # four projections, a rank that is no multiple of 32, groups of several tokens
    (328, 24, (264, 136), 50),             # contraction length the shared launches do not take: one after the other
])
def test_decode_sized_batches_share_their_two_launches(d_in, r, d_outs, T):
    # Decode-sized batches: the projections' base tiles and shrink slabs side by side in one launch, their
    # expand blocks in another.  The bits of the single calls, in both output types; the ranked plan too.
    E = 9
    rng = np.random.default_rng(T + r)
    ids = (rng.integers(0, E + 1, size=T) - 1).tolist()
    inps = _projections(d_in, d_outs, r, E, [1] * T, ids, seed=800 + r)
    x = inps[0].x
    ctx = gc.ctx()
    ranks = torch.from_numpy(np.asarray([r, r // 2 // 8 * 8, 8, r, 0, r, r, 16 if r >= 16 else 8, r], np.int32)).cuda()
    for rank_of_expert in (None, ranks):
        plan = moin.Plan(ctx).build(inps[0].seq_offsets, inps[0].expert_ids, T, E, rank_of_expert=rank_of_expert)
        for dt in (torch.bfloat16, torch.float32):
            print(f"[gpu] shared decode d_in={d_in} r={r} n={len(d_outs)} T={T} y={dt} ranks={rank_of_expert is not None}",
                  flush=True)
            single = [moin.moin_lora_linear_planned(ctx, plan, x, i.W, i.A_stack, i.B_stack, 2.0, y_dtype=dt)
                      for i in inps]
            outs = [torch.full((T, d), float("nan"), dtype=dt, device="cuda") for d in d_outs]
            ys = moin.moin_lora_linear_planned_shared(ctx, plan, x, [i.W for i in inps], [i.A_stack for i in inps],
                                                      [i.B_stack for i in inps], 2.0, y_dtype=dt, outs=outs)
            ctx.check()
            for a, b in zip(single, ys):
                assert torch.equal(a, b)
        plan.close()
    # every projection of the full-rank call against the oracle as well
    plan = moin.Plan(ctx).build(inps[0].seq_offsets, inps[0].expert_ids, T, E)
    ys = moin.moin_lora_linear_planned_shared(ctx, plan, x, [i.W for i in inps], [i.A_stack for i in inps],
                                              [i.B_stack for i in inps], 2.0)
    ctx.check()
    for i, y in zip(inps, ys):
        inp = wl.LinearInputs(i.wl, x, i.W, i.A_stack, i.B_stack, i.seq_offsets, i.expert_ids)
        gc.compare_linear(y, gc.oracle_rows(inp), what="shared decode")
    plan.close()


def test_shared_input_on_the_other_paths_and_argument_errors():
    ctx = gc.ctx()
    # decode-sized batch, and no adapters at all
    inps = _projections(256, (136, 264), 64, 5, [1] * 100, (np.arange(100) % 6 - 1).tolist(), seed=700)
    x = inps[0].x
    plan = moin.Plan(ctx).build(inps[0].seq_offsets, inps[0].expert_ids, 100, 5)
    single = [moin.moin_lora_linear_planned(ctx, plan, x, i.W, i.A_stack, i.B_stack, 2.0) for i in inps]
    ys = moin.moin_lora_linear_planned_shared(ctx, plan, x, [i.W for i in inps], [i.A_stack for i in inps],
                                              [i.B_stack for i in inps], 2.0)
    base = moin.moin_lora_linear_planned_shared(ctx, plan, x, [i.W for i in inps], None, None, 2.0)
    base1 = [moin.moin_lora_linear_planned(ctx, plan, x, i.W, None, None, 2.0) for i in inps]
    ctx.check()
    for a, b in zip(single + base1, ys + base):
        assert torch.equal(a, b)
    with pytest.raises(ValueError):
        moin.moin_lora_linear_planned_shared(ctx, plan, x, [i.W for i in inps] * 3, None, None, 2.0)
    with pytest.raises(ValueError):
        moin.moin_lora_linear_planned_shared(ctx, plan, x, [inps[0].W], [inps[0].A_stack], None, 2.0)
    plan.close()
