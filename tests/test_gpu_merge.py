"""moin_merge_adapters against the oracle, bit for bit, and in its place in the path: the k nearest topics of a
query, weights from their distances, the merged adapter in a slot of wider stacks, the layer with that slot."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_09687_amd import moin
from paper_2410_09687_amd import workloads as wl
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu


def _stacks(E, r, d_in, d_out, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    A = (torch.randn((E, r, d_in), device="cuda", generator=g) / d_in ** 0.5).bfloat16()
    B = (torch.randn((E, d_out, r), device="cuda", generator=g) / r ** 0.5).bfloat16()
    return A, B


def test_bits_of_the_oracle():
    ctx = gc.ctx()
    A, B = _stacks(9, 24, 136, 72, 91)
    g = torch.Generator(device="cuda").manual_seed(92)
    for ids, r_out in (([4], 24), ([8, 0, 3], 72), ([2, -1, 7, 7], 128), ([], 8)):
        print(f"[gpu] merge ids={ids} r_out={r_out}", flush=True)
        n = len(ids)
        ids_t = torch.tensor(ids, dtype=torch.int32, device="cuda")
        w = torch.randn(n, device="cuda", generator=g) if n else torch.zeros(0, device="cuda")
        A_out = torch.full((r_out, 136), float("nan"), dtype=torch.bfloat16, device="cuda")
        B_out = torch.full((72, r_out), float("nan"), dtype=torch.bfloat16, device="cuda")
        moin.moin_merge_adapters(ctx, A, B, ids_t, w, A_out, B_out)
        ctx.check()
        ra, rb = oracle.merge_adapters(wl.bf16_bits(A), wl.bf16_bits(B), ids, w.cpu().numpy(), r_out)
        assert np.array_equal(wl.bf16_bits(A_out), ra) and np.array_equal(wl.bf16_bits(B_out), rb)


def test_nearest_topics_merged_into_a_slot_and_used_by_the_layer():
    ctx = gc.ctx()
    E, r, d_in, d_out, k = 12, 64, 256, 264, 3
    A, B = _stacks(E, r, d_in, d_out, 93)
    g = torch.Generator(device="cuda").manual_seed(94)
    cent = torch.randn((E, 128), device="cuda", generator=g)
    query = (cent[5] + cent[9] + 0.3 * torch.randn(128, device="cuda", generator=g))[None]
    _, cids, d2 = moin.moin_route_topk(ctx, query, cent, k)
    w = torch.softmax(-d2[0] / d2[0].mean(), dim=0).float().contiguous()
    # stacks of rank k r whose last slot receives the merged adapter; the others hold plain adapters at rank r
    A_wide = torch.zeros((E + 1, k * r, d_in), dtype=torch.bfloat16, device="cuda")
    B_wide = torch.zeros((E + 1, d_out, k * r), dtype=torch.bfloat16, device="cuda")
    A_wide[:E, :r] = A
    B_wide[:E, :, :r] = B
    moin.moin_merge_adapters(ctx, A, B, cids[0].contiguous(), w, A_wide[E], B_wide[E])
    ranks = torch.tensor([r] * E + [k * r], dtype=torch.int32, device="cuda")
    lens = [300, 700, 1, 260]
    seq_ids = [E, 2, E, -1]
    wk = wl.LinearWorkload("merged", d_in, d_out, k * r, E + 1, lens, "uniform", scale=2.0, seed=95)
    inp = wl.make_linear_inputs(wk, "cuda", expert_ids=np.asarray(seq_ids, np.int32), stacks=(A_wide, B_wide))
    print("[gpu] layer with a merged adapter", flush=True)
    y = moin.moin_lora_linear(ctx, inp.x, inp.seq_offsets, inp.expert_ids, inp.W, A_wide, B_wide, 2.0,
                              y_dtype=torch.float32, rank_of_expert=ranks)
    ctx.check()
    # the oracle end to end from the GPU's ids and weights: its own merge, its own layer
    ra, rb = oracle.merge_adapters(wl.bf16_bits(A), wl.bf16_bits(B), cids[0].cpu().numpy(), w.cpu().numpy(), k * r)
    Ah, Bh = wl.bf16_bits(A_wide), wl.bf16_bits(B_wide)
    assert np.array_equal(Ah[E], ra) and np.array_equal(Bh[E], rb)
    ref = oracle.lora_linear(wl.bf16_bits(inp.x), inp.seq_offsets.cpu().numpy(), np.asarray(seq_ids, np.int32),
                             wl.bf16_bits(inp.W), Ah, Bh, 2.0, rank_of_expert=ranks.cpu().numpy())
    gc.compare_linear(y, ref, what="merged adapter")
    assert set(cids[0].tolist()) >= {5, 9}


def test_bad_ids_are_reported_and_argument_errors():
    ctx = gc.ctx()
    A, B = _stacks(4, 8, 64, 16, 96)
    A_out = torch.zeros((16, 64), dtype=torch.bfloat16, device="cuda")
    B_out = torch.zeros((16, 16), dtype=torch.bfloat16, device="cuda")
    ids = torch.tensor([1, 4], dtype=torch.int32, device="cuda")
    moin.moin_merge_adapters(ctx, A, B, ids, torch.ones(2, device="cuda"), A_out, B_out)
    with pytest.raises(moin.MoinError):
        ctx.check()
    assert torch.equal(A_out[:8], A[1]) and not A_out[8:].any() and not B_out[:, 8:].any()
    with pytest.raises(moin.MoinError):     # three adapters of rank 8 do not fit rank 16
        moin.moin_merge_adapters(ctx, A, B, torch.tensor([0, 1, 2], dtype=torch.int32, device="cuda"),
                                 torch.ones(3, device="cuda"), A_out, B_out)
