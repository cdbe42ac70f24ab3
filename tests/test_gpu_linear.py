"""GPU parity of moin_lora_linear (through the C ABI) against the CPU oracle,
element by element on small and ragged cases."""
import numpy as np
import pytest
import torch

from paper_2410_09687_amd import moin
from paper_2410_09687_amd import workloads as wl
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu


def _case(name, d_in, d_out, r, E, lens, ids=None, seed=1234, dist="uniform"):
    w = wl.LinearWorkload(name, d_in, d_out, r, E, lens, dist, scale=2.0, seed=seed)
    return wl.make_linear_inputs(w, "cuda", expert_ids=None if ids is None else np.asarray(ids, np.int32))


def _full_check(inp, what):
    ref = gc.oracle_rows(inp)
    out = {}
    for dt in (torch.bfloat16, torch.float32):
        print(f"[gpu] {what} y={dt}", flush=True)
        y = gc.run_linear(inp, dt)
        out[dt] = gc.compare_linear(y, ref, what=f"{what}/{dt}")
        out[("y", dt)] = y
    # both outputs come from the same fp32 accumulators (runs repeat bit for bit),
    # so the bf16 one must be the round-to-nearest-even image of the fp32 one
    y16, y32 = out.pop(("y", torch.bfloat16)), out.pop(("y", torch.float32))
    assert torch.equal(y16.view(torch.int16), y32.to(torch.bfloat16).view(torch.int16)), \
        f"{what}: bf16 output is not RNE(fp32 output)"
    return out


def test_tiny_config_route_feeds_linear():
    rw, lw = wl.config_tiny()
    rin = wl.make_route_inputs(rw, "cuda")
    print("[gpu] c0 route", flush=True)
    eids, cids, counts = moin.moin_route(gc.ctx(), rin.emb, rin.centroids, want_counts=True)
    gc.ctx().check()
    assert gc.check_route(rin.emb, rin.centroids, cids) == 0
    assert torch.equal(eids, cids)
    assert counts.sum().item() == rw.N
    inp = wl.make_linear_inputs(lw, "cuda", expert_ids=eids.cpu().numpy())
    _full_check(inp, "c0")


def test_prefill_ragged_tiles_and_tails():
    # T > 1024 -> prefill path.  d_in, d_out, r leave K-, N- and rank-tails; lengths
    # cover empty, 1-token, tile-exact, tile+1 and multi-tile sequences.
    lens = [300, 1, 0, 257, 255, 512, 77, 256, 3, 640]
    ids = [3, 0, 5, -1, 3, 6, 2, 2, -1, 1]
    inp = _case("ragged_prefill", 328, 264, 24, 7, lens, ids)
    assert inp.wl.T > 1024
    _full_check(inp, "ragged_prefill")


def test_prefill_streaming_kernel_ragged_tiles_mixed_adapters():
    # shapes the persistent streaming kernel takes (d_in, r multiples of 64): ragged
    # token tiles, an output tail of 8 columns, base-only sequences between adapter
    # ones, rank spanning two k blocks
    lens = [300, 1, 0, 257, 255, 512, 77, 256, 3, 640]
    ids = [3, 0, 5, -1, 3, 6, 2, 2, -1, 1]
    inp = _case("stream_ragged", 192, 520, 128, 7, lens, ids, seed=11)
    assert inp.wl.T > 1024
    _full_check(inp, "stream_ragged")
    # a single tile (fewer work items than workgroups), d_in at the two-block minimum
    inp = _case("stream_one_tile", 128, 64, 64, 2, [1030], [1], seed=12)
    _full_check(inp, "stream_one_tile")


def test_prefill_streaming_kernel_many_tiles_per_workgroup():
    # > 256 * 8 work items: every workgroup walks several tiles, adapter and
    # base-only tiles alternating in its stream
    rng = np.random.default_rng(5)
    lens = rng.integers(1, 300, size=700).tolist()
    ids = rng.integers(-1, 4, size=700).tolist()
    inp = _case("stream_many", 128, 1024, 64, 4, lens, ids, seed=13)
    _full_check(inp, "stream_many")


def test_prefill_rank_multiple_tiles():
    # r = 136 spans several rank tiles of the shrink and three K blocks of the expand
    inp = _case("rank136", 192, 520, 136, 3, [700, 400], [2, 0], seed=77)
    _full_check(inp, "rank136")


def test_prefill_all_one_expert_and_all_distinct():
    inp = _case("one_expert", 256, 256, 16, 4, [200] * 6, [2] * 6, seed=5)
    _full_check(inp, "one_expert")
    inp = _case("distinct", 256, 256, 16, 12, [100] * 12, list(range(12)), seed=6)
    _full_check(inp, "distinct")


def test_prefill_base_only_and_no_stacks():
    inp = _case("base_only", 128, 136, 8, 2, [600, 500], [-1, -1], seed=8)
    st = _full_check(inp, "base_only")
    y = moin.moin_lora_linear(gc.ctx(), inp.x, inp.seq_offsets, inp.expert_ids, inp.W, None, None, 2.0)
    gc.ctx().check()
    assert torch.equal(y, gc.run_linear(inp))
    assert st[torch.float32]["max_abs"] < 1e-4   # plain fp32-accumulated GEMM


def test_decode_single_token_sequences():
    # T <= 1024 -> decode path; Zipf ids so several tokens share an expert
    w = wl.LinearWorkload("dec", 384, 520, 40, 50, [1] * 256, "zipf", 1.1, 2.0, seed=99)
    inp = wl.make_linear_inputs(w, "cuda")
    _full_check(inp, "decode_256x1")


def test_decode_mixed_lengths_and_big_groups():
    # one expert owns > 16 tokens (several token blocks), empty sequences, base-only ones
    lens = [20, 0, 1, 3, 17, 1, 1, 40, 2, 0, 5]
    ids = [4, 1, -1, 4, 4, 0, 2, 2, -1, 3, 0]
    inp = _case("decode_mixed", 264, 136, 16, 5, lens, ids, seed=31)
    assert inp.wl.T <= 1024
    _full_check(inp, "decode_mixed")


def test_many_short_sequences_use_the_global_sort_scratch():
    # more sequences than the plan kernel sorts in LDS; every tile is 1..3 rows
    rng = np.random.default_rng(3)
    lens = rng.integers(0, 4, size=2500).tolist()
    ids = rng.integers(-1, 6, size=2500).tolist()
    inp = _case("many_seqs", 64, 64, 8, 6, lens, ids, seed=91)
    assert inp.wl.T > 1024
    _full_check(inp, "many_seqs")


def test_planned_calls_share_one_plan():
    lens = [400, 300, 500]
    ids = [1, -1, 0]
    a = _case("pA", 128, 256, 16, 2, lens, ids, seed=41)
    b = _case("pB", 128, 64, 16, 2, lens, ids, seed=42)
    plan = moin.Plan(gc.ctx()).build(a.seq_offsets, a.expert_ids, a.wl.T, 2)
    for inp in (a, b):
        y = moin.moin_lora_linear_planned(gc.ctx(), plan, inp.x, inp.W, inp.A_stack, inp.B_stack, 2.0)
        gc.ctx().check()
        assert torch.equal(y, gc.run_linear(inp))
    plan.close()


def test_runs_are_bitwise_repeatable():
    inp = _case("repeat", 256, 256, 16, 4, [300, 300, 300, 300], [0, 1, 2, 3], seed=51)
    assert torch.equal(gc.run_linear(inp), gc.run_linear(inp))
    w = wl.LinearWorkload("repeat_dec", 256, 256, 16, 9, [1] * 64, "zipf", 1.1, 2.0, seed=52)
    inp = wl.make_linear_inputs(w, "cuda")
    assert torch.equal(gc.run_linear(inp), gc.run_linear(inp))


def test_empty_batches_and_argument_errors():
    c = gc.ctx()
    inp = _case("args", 64, 64, 8, 2, [5, 5], [0, 1], seed=61)
    empty_x = inp.x[:0]
    y = moin.moin_lora_linear(c, empty_x, torch.zeros(1, dtype=torch.int32, device="cuda"),
                              torch.zeros(0, dtype=torch.int32, device="cuda"), inp.W, inp.A_stack,
                              inp.B_stack, 2.0)
    assert y.shape == (0, 64)
    # host-checkable faults -> MOIN_EINVAL, nothing launched
    bad_w = torch.zeros((64, 60), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(moin.MoinError) as ei:
        moin.moin_lora_linear(c, torch.zeros((10, 60), dtype=torch.bfloat16, device="cuda"),
                              inp.seq_offsets, inp.expert_ids, bad_w, None, None, 2.0)
    assert ei.value.code == -1
    with pytest.raises(moin.MoinError):
        moin.moin_lora_linear(c, inp.x, inp.seq_offsets, inp.expert_ids, inp.W, inp.A_stack,
                              inp.B_stack, float("nan"))
    c.check()


def test_device_side_data_faults_are_sticky_and_fall_back_to_base():
    c = gc.ctx()
    for lens in ([600, 600], [3, 4]):          # prefill and decode paths
        inp = _case("fault", 64, 64, 8, 2, lens, [0, 1], seed=71)
        bad = inp.expert_ids.clone()
        bad[1] = 2                              # >= E
        y = moin.moin_lora_linear(c, inp.x, inp.seq_offsets, bad, inp.W, inp.A_stack, inp.B_stack, 2.0)
        with pytest.raises(moin.MoinError) as ei:
            c.check()
        assert ei.value.code == -4
        c.check()                               # the word was cleared
        ok = inp.expert_ids.clone()
        ok[1] = -1
        y2 = moin.moin_lora_linear(c, inp.x, inp.seq_offsets, ok, inp.W, inp.A_stack, inp.B_stack, 2.0)
        c.check()
        assert torch.equal(y, y2)


def test_offsets_that_do_not_tile_the_batch_give_base_only_rows_everywhere():
    c = gc.ctx()
    for lens in ([600, 600, 300], [3, 4, 5]):          # prefill and decode paths
        inp = _case("badoff", 64, 64, 8, 2, lens, [0, 1, 0], seed=73)
        bad = inp.seq_offsets.clone()
        bad[1], bad[2] = inp.seq_offsets[2].item(), inp.seq_offsets[1].item()   # runs backwards
        y = moin.moin_lora_linear(c, inp.x, bad, inp.expert_ids, inp.W, inp.A_stack, inp.B_stack, 2.0)
        with pytest.raises(moin.MoinError) as ei:
            c.check()
        assert ei.value.code == -4
        none = torch.full_like(inp.expert_ids, -1)
        y2 = moin.moin_lora_linear(c, inp.x, inp.seq_offsets, none, inp.W, inp.A_stack, inp.B_stack, 2.0)
        c.check()
        assert torch.equal(y, y2)
