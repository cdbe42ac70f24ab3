"""GPU parity of the adapter with an activation between its two linear layers ("Future Works", better
adapters) against the oracle: prefill (streaming and tiled kernels), decode, per-expert ranks, the
quantised base."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_09687_amd import moin
from paper_2410_09687_amd import workloads as wl
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu
ACTS = ("relu", "silu", "gelu")


@pytest.fixture
def ctx():
    c = gc.ctx()
    yield c
    c.set_adapter_activation(None)   # the context is shared with the other tests


def _case(name, d_in, d_out, r, E, lens, ids=None, seed=1234, dist="uniform"):
    w = wl.LinearWorkload(name, d_in, d_out, r, E, lens, dist, scale=2.0, seed=seed)
    inp = wl.make_linear_inputs(w, "cuda", expert_ids=None if ids is None else np.asarray(ids, np.int32))
    # W_a x of unit size, so that the activations work on their curved part
    inp.A_stack.mul_(float(np.sqrt(d_in)) / 4)
    return inp


def _check(ctx, inp, what, ranks=None):
    A, B, ids = wl.compact_stacks(inp)
    ranks_c, ranks_t = None, None
    if ranks is not None:
        ranks_t = torch.from_numpy(np.asarray(ranks, np.int32)).cuda()
        used = np.unique(inp.expert_ids.cpu().numpy())
        ranks_c = np.asarray(ranks, np.int32)[used[used >= 0]]
    lin = None
    for act in (None,) + ACTS:
        ref = oracle.lora_linear(wl.bf16_bits(inp.x), inp.seq_offsets.cpu().numpy(), ids, wl.bf16_bits(inp.W), A, B,
                                 inp.wl.scale, rank_of_expert=ranks_c, activation=act)
        ctx.set_adapter_activation(act)
        for dt in (torch.float32, torch.bfloat16):
            print(f"[gpu] activation {what} act={act} y={dt}", flush=True)
            y = moin.moin_lora_linear(ctx, inp.x, inp.seq_offsets, inp.expert_ids, inp.W, inp.A_stack,
                                      inp.B_stack, inp.wl.scale, y_dtype=dt, rank_of_expert=ranks_t)
            ctx.check()
            gc.compare_linear(y, ref, what=f"{what}/{act}/{dt}")
        if act is None:
            lin = ref
        else:
            assert np.abs(ref - lin).max() > 0.1, f"{what}/{act}: the case does not exercise the activation"


def test_prefill_streaming_kernel(ctx):
    lens = [300, 1, 0, 257, 255, 512, 77, 256, 3, 640]
    ids = [3, 0, 5, -1, 3, 6, 2, 2, -1, 1]
    _check(ctx, _case("act_stream", 256, 264, 64, 7, lens, ids, seed=61), "stream_r64")
    _check(ctx, _case("act_stream128", 384, 136, 128, 7, lens, ids, seed=62), "stream_r128")


def test_prefill_tiled_kernel_and_rank_tail(ctx):
    lens = [300, 1, 0, 257, 255, 512, 77]
    ids = [3, 0, 5, -1, 3, 6, 2]
    _check(ctx, _case("act_tiled", 328, 264, 24, 7, lens, ids, seed=63), "tiled_r24")


def test_decode(ctx):
    w = wl.LinearWorkload("act_dec", 384, 520, 40, 50, [1] * 256, "zipf", 1.1, 2.0, seed=64)
    inp = wl.make_linear_inputs(w, "cuda")
    inp.A_stack.mul_(float(np.sqrt(384)) / 4)
    _check(ctx, inp, "decode_256x1")
    lens = [20, 0, 1, 3, 17, 1, 1, 40, 2, 0, 5]
    ids = [4, 1, -1, 4, 4, 0, 2, 2, -1, 3, 0]
    _check(ctx, _case("act_dec_mixed", 264, 136, 16, 5, lens, ids, seed=65), "decode_mixed")


def test_per_expert_ranks(ctx):
    lens = [300, 200, 257, 100, 280]
    ids = [0, 1, 2, -1, 3]
    inp = _case("act_ranks", 256, 264, 128, 4, lens, ids, seed=66)
    ranks = [128, 64, 8, 0]
    for e, k in enumerate(ranks):
        inp.A_stack[e, k:] = float("nan")
        inp.B_stack[e, :, (k + 63) // 64 * 64:] = float("nan")
        inp.B_stack[e, :, k:(k + 63) // 64 * 64] = 0
    _check(ctx, inp, "ranks", ranks=ranks)


def test_quantised_base(ctx):
    lens = [300, 200, 257, 100, 280, 1, 700]
    ids = [0, 1, 2, -1, 3, -1, 1]
    inp = _case("act_mx", 256, 264, 64, 4, lens, ids, seed=67)
    Wq, Ws = moin.moin_mx_quantize(ctx, inp.W, blocked=True)
    Ws_rows = Ws.permute(1, 0, 2).reshape(Ws.shape[1], -1).contiguous().cpu().numpy()   # [d_out, d_in / 32]
    A, B, cid = wl.compact_stacks(inp)
    for act in ACTS:
        ref = oracle.lora_linear_mx(wl.bf16_bits(inp.x), inp.seq_offsets.cpu().numpy(), cid, Wq.cpu().numpy(), Ws_rows,
                                    A, B, inp.wl.scale, activation=act)
        ctx.set_adapter_activation(act)
        print(f"[gpu] activation mx act={act}", flush=True)
        y = moin.moin_lora_linear_mx(ctx, inp.x, inp.seq_offsets, inp.expert_ids, Wq, Ws, inp.A_stack, inp.B_stack,
                                     inp.wl.scale, y_dtype=torch.float32)
        ctx.check()
        gc.compare_linear(y, ref, what=f"mx/{act}")


def test_setter_rejects_unknown_codes_and_keeps_the_setting(ctx):
    with pytest.raises(ValueError):
        ctx.set_adapter_activation("tanh")
    assert moin.load().moin_set_adapter_activation(ctx._h, 7) != 0
    assert moin.load().moin_set_adapter_activation(ctx._h, -1) != 0
