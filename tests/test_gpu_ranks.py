"""GPU parity of the per-expert adapter rank ("Future Works": adaptive rank per
topic) against the oracle, on the prefill paths (streaming and tiled kernels)
and the decode path.  The stacks keep the full rank r; what lies beyond an
expert's own rank is filled with NaN wherever the kernels promise not to touch
it, and with finite noise where they multiply it by zeros (columns of B_e from
the rank to the next multiple of 64, prefill only)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_09687_amd import moin
from paper_2410_09687_amd import workloads as wl
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu


def _poison(inp, ranks, decode):
    """Overwrites everything beyond each expert's rank: NaN where it must never be read."""
    A, B = inp.A_stack.clone(), inp.B_stack.clone()
    r = A.shape[1]
    nan = float("nan")
    for e, k in enumerate(ranks):
        A[e, k:] = nan
        lim = k if decode else min(r, (k + 63) // 64 * 64)
        B[e][:, lim:] = nan
    return A, B


def _check(inp, ranks, what, decode=False, dtypes=(torch.bfloat16, torch.float32)):
    ranks = np.asarray(ranks, np.int32)
    A, B = _poison(inp, ranks, decode)
    ranks_dev = torch.from_numpy(ranks).cuda()
    ref = oracle.lora_linear(wl.bf16_bits(inp.x), inp.seq_offsets.cpu().numpy(), inp.expert_ids.cpu().numpy(),
                             wl.bf16_bits(inp.W), wl.bf16_bits(inp.A_stack), wl.bf16_bits(inp.B_stack),
                             inp.wl.scale, rank_of_expert=ranks)
    out = {}
    for dt in dtypes:
        print(f"[gpu] ranked {what} y={dt}", flush=True)
        y = moin.moin_lora_linear(gc.ctx(), inp.x, inp.seq_offsets, inp.expert_ids, inp.W, A, B, inp.wl.scale,
                                  y_dtype=dt, rank_of_expert=ranks_dev)
        gc.ctx().check()
        gc.compare_linear(y, ref, what=f"{what}/{dt}")
        out[dt] = y
    return out


def _case(name, d_in, d_out, r, E, lens, ids, seed):
    w = wl.LinearWorkload(name, d_in, d_out, r, E, lens, "uniform", scale=2.0, seed=seed)
    return wl.make_linear_inputs(w, "cuda", expert_ids=np.asarray(ids, np.int32))


def test_prefill_streaming_kernel_with_ranks():
    lens = [300, 1, 0, 257, 255, 512, 77, 256, 3, 640]
    ids = [3, 0, 5, -1, 3, 6, 2, 2, -1, 1]
    inp = _case("ranked_stream", 192, 520, 128, 7, lens, ids, 31)
    _check(inp, [128, 64, 0, 8, 72, 40, 128], "stream")


def test_prefill_tiled_kernel_with_ranks():
    # d_in and r leave tails: the tiled kernels, rank tiles of the 64 x 64 shrink
    lens = [700, 400, 33]
    inp = _case("ranked_tiled", 328, 264, 136, 4, lens, [2, 0, 1], 32)
    _check(inp, [136, 16, 96, 0], "tiled")


def test_decode_with_ranks_reads_nothing_beyond_them():
    rng = np.random.default_rng(7)
    S = 200
    ids = rng.integers(-1, 12, size=S)
    lens = rng.integers(1, 4, size=S).tolist()
    inp = _case("ranked_decode", 256, 328, 64, 12, lens, ids, 33)
    assert inp.wl.T <= 1024
    ranks = [64, 8, 0, 32, 40, 64, 16, 24, 56, 48, 8, 64]
    _check(inp, ranks, "decode", decode=True)


def test_full_and_zero_ranks_are_the_plain_and_the_base_layer():
    lens = [300, 200, 600]
    inp = _case("ranked_limits", 128, 128, 64, 3, lens, [0, 2, 1], 34)
    full = torch.full((3,), 64, dtype=torch.int32, device="cuda")
    zero = torch.zeros(3, dtype=torch.int32, device="cuda")
    args = (inp.x, inp.seq_offsets, inp.expert_ids, inp.W, inp.A_stack, inp.B_stack, 2.0)
    plain = moin.moin_lora_linear(gc.ctx(), *args)
    assert torch.equal(plain, moin.moin_lora_linear(gc.ctx(), *args, rank_of_expert=full))
    # a rank above r counts as r
    assert torch.equal(plain, moin.moin_lora_linear(gc.ctx(), *args, rank_of_expert=full * 4))
    base = moin.moin_lora_linear(gc.ctx(), inp.x, inp.seq_offsets, torch.full_like(inp.expert_ids, -1), inp.W,
                                 inp.A_stack, inp.B_stack, 2.0)
    assert torch.equal(base, moin.moin_lora_linear(gc.ctx(), *args, rank_of_expert=zero))
    gc.ctx().check()


def test_bad_ranks_are_rounded_down_and_reported():
    lens = [300, 200, 600]
    inp = _case("ranked_bad", 128, 128, 64, 3, lens, [0, 2, 1], 35)
    args = (inp.x, inp.seq_offsets, inp.expert_ids, inp.W, inp.A_stack, inp.B_stack, 2.0)
    bad = torch.tensor([21, -3, 40], dtype=torch.int32, device="cuda")
    y = moin.moin_lora_linear(gc.ctx(), *args, rank_of_expert=bad)
    with pytest.raises(moin.MoinError) as e:
        gc.ctx().check()
    assert e.value.code == -4
    good = torch.tensor([16, 64, 40], dtype=torch.int32, device="cuda")   # 21 -> 16, negative -> full
    assert torch.equal(y, moin.moin_lora_linear(gc.ctx(), *args, rank_of_expert=good))
    gc.ctx().check()


def test_planned_projections_share_the_ranks():
    lens = [260, 90, 700]
    ids = np.array([1, 0, 1], np.int32)
    ranks = np.array([24, 64], np.int32)
    a = _case("ranked_plan_a", 128, 192, 64, 2, lens, ids, 36)
    b = _case("ranked_plan_b", 128, 64, 64, 2, lens, ids, 37)
    plan = moin.Plan(gc.ctx()).build(a.seq_offsets, a.expert_ids, a.wl.T, 2,
                                     rank_of_expert=torch.from_numpy(ranks).cuda())
    for inp in (a, b):
        y = moin.moin_lora_linear_planned(gc.ctx(), plan, inp.x, inp.W, inp.A_stack, inp.B_stack, 2.0,
                                          y_dtype=torch.float32)
        gc.ctx().check()
        ref = oracle.lora_linear(wl.bf16_bits(inp.x), inp.seq_offsets.cpu().numpy(), ids, wl.bf16_bits(inp.W),
                                 wl.bf16_bits(inp.A_stack), wl.bf16_bits(inp.B_stack), 2.0, rank_of_expert=ranks)
        gc.compare_linear(y, ref, what=inp.wl.name)
    plan.close()
