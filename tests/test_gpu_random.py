"""Seeded random sweep of the routed LoRA linear over shapes, length mixes, expert assignments, per-expert
ranks, activations and output types, through whichever kernels the library picks (streaming or tiled prefill,
decode, gathered batches of short sequences), each case against the oracle on the same bytes."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_09687_amd import moin
from paper_2410_09687_amd import workloads as wl
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu


def _draw_case(rng):
    kind = rng.choice(["stream", "tiled", "decode", "gather", "gather_tiled"])
    if kind in ("stream", "gather"):
        d_in = int(rng.choice([128, 192, 256, 384]))
        r = int(rng.choice([64, 128]))
    else:
        d_in = int(rng.choice([72, 136, 264, 328]))
        r = int(rng.choice([8, 16, 24, 40, 72]))
    d_out = int(rng.choice([8, 72, 136, 264, 520]))
    E = int(rng.integers(1, 9))
    if kind in ("stream", "tiled"):
        S = int(rng.integers(1, 8))
        lens = rng.choice([0, 1, 3, 255, 256, 257, 300, 511, 700], size=S).tolist()
        if sum(lens) <= 1024:
            lens.append(1100)
    elif kind == "decode":
        S = int(rng.integers(1, 200))
        lens = rng.integers(0, 5, size=S).tolist()
        while sum(lens) > 1024:
            lens.pop()
        if sum(lens) == 0:
            lens.append(1)
    else:
        S = int(rng.integers(300, 1500))
        lens = rng.integers(0, 6, size=S).tolist()
        lens[int(rng.integers(0, S))] = int(rng.integers(1, 600))
        if sum(lens) <= 1024:
            lens += [1] * 1100
    S = len(lens)
    ids = rng.integers(-1, E, size=S)
    ranks = None
    if rng.random() < 0.4:
        ranks = (rng.integers(0, r // 8 + 1, size=E) * 8).astype(np.int32)
    act = rng.choice([None, None, "relu", "silu", "gelu"])
    dt = torch.float32 if rng.random() < 0.5 else torch.bfloat16
    return kind, d_in, d_out, r, E, lens, ids, ranks, act, dt


@pytest.mark.parametrize("block", range(6))
def test_random_cases(block):
    ctx = gc.ctx()
    rng = np.random.default_rng(9000 + block)
    try:
        for i in range(12):
            kind, d_in, d_out, r, E, lens, ids, ranks, act, dt = _draw_case(rng)
            what = f"block {block} case {i}: {kind} d_in={d_in} d_out={d_out} r={r} E={E} S={len(lens)} " \
                   f"T={sum(lens)} ranks={'yes' if ranks is not None else 'no'} act={act} y={dt}"
            print("[gpu] random " + what, flush=True)
            w = wl.LinearWorkload("rnd", d_in, d_out, r, E, lens, "uniform", scale=2.0, seed=int(rng.integers(1 << 30)))
            inp = wl.make_linear_inputs(w, "cuda", expert_ids=ids.astype(np.int32))
            if act is not None:
                inp.A_stack.mul_(float(np.sqrt(d_in)) / 4)
            ref = oracle.lora_linear(wl.bf16_bits(inp.x), inp.seq_offsets.cpu().numpy(), ids.astype(np.int32),
                                     wl.bf16_bits(inp.W), wl.bf16_bits(inp.A_stack), wl.bf16_bits(inp.B_stack), 2.0,
                                     rank_of_expert=ranks, activation=act)
            ctx.set_adapter_activation(act)
            y = moin.moin_lora_linear(ctx, inp.x, inp.seq_offsets, inp.expert_ids, inp.W, inp.A_stack, inp.B_stack,
                                      2.0, y_dtype=dt,
                                      rank_of_expert=None if ranks is None else torch.from_numpy(ranks).cuda())
            ctx.check()
            gc.compare_linear(y, ref, what=what)
    finally:
        ctx.set_adapter_activation(None)


@pytest.mark.parametrize("block", range(3))
def test_random_cases_quantised_base(block):
    ctx = gc.ctx()
    rng = np.random.default_rng(9500 + block)
    try:
        for i in range(6):
            kind, _, d_out, _, E, lens, ids, ranks, act, dt = _draw_case(rng)
            d_in = int(rng.choice([256, 384, 512]))
            r = int(rng.choice([64, 128]))
            if ranks is not None:
                ranks = (rng.integers(0, r // 8 + 1, size=E) * 8).astype(np.int32)
            what = f"mx block {block} case {i}: {kind} d_in={d_in} d_out={d_out} r={r} E={E} S={len(lens)} " \
                   f"T={sum(lens)} ranks={'yes' if ranks is not None else 'no'} act={act} y={dt}"
            print("[gpu] random " + what, flush=True)
            w = wl.LinearWorkload("rnd_mx", d_in, d_out, r, E, lens, "uniform", scale=2.0, seed=int(rng.integers(1 << 30)))
            inp = wl.make_linear_inputs(w, "cuda", expert_ids=ids.astype(np.int32))
            if act is not None:
                inp.A_stack.mul_(float(np.sqrt(d_in)) / 4)
            Wq, Ws = moin.moin_mx_quantize(ctx, inp.W, blocked=True)
            Ws_rows = Ws.permute(1, 0, 2).reshape(Ws.shape[1], -1).contiguous().cpu().numpy()
            ref = oracle.lora_linear_mx(wl.bf16_bits(inp.x), inp.seq_offsets.cpu().numpy(), ids.astype(np.int32),
                                        Wq.cpu().numpy(), Ws_rows, wl.bf16_bits(inp.A_stack),
                                        wl.bf16_bits(inp.B_stack), 2.0, rank_of_expert=ranks, activation=act)
            ctx.set_adapter_activation(act)
            y = moin.moin_lora_linear_mx(ctx, inp.x, inp.seq_offsets, inp.expert_ids, Wq, Ws, inp.A_stack, inp.B_stack,
                                         2.0, y_dtype=dt,
                                         rank_of_expert=None if ranks is None else torch.from_numpy(ranks).cuda())
            ctx.check()
            gc.compare_linear(y, ref, what=what)
    finally:
        ctx.set_adapter_activation(None)


@pytest.mark.parametrize("block", range(3))
def test_random_router_cases(block):
    """moin_route over random sizes, both storage types, slot maps and retained-only searches: ids against the
    oracle (a different id only inside the near-tie band), the histogram = the tally of the ids returned."""
    ctx = gc.ctx()
    rng = np.random.default_rng(9700 + block)
    for i in range(10):
        bf16 = bool(rng.random() < 0.6)
        N = int(rng.choice([1, 7, 64, 65, 300, 1025, 4097, 9000]))
        K = int(rng.choice([1, 2, 63, 64, 65, 257, 500, 1030]))
        D = int(rng.choice([8, 64, 72, 128, 264, 768]) if bf16 else rng.choice([4, 36, 64, 260]))
        normalise = bool(rng.random() < 0.5)
        use_slot = rng.random() < 0.5
        retained = bool(use_slot and rng.random() < 0.5)
        what = f"router block {block} case {i}: N={N} K={K} D={D} {'bf16' if bf16 else 'f32'} slot={use_slot} retained_only={retained}"
        print("[gpu] random " + what, flush=True)
        rw = wl.RouteWorkload("rnd_route", N=N, K=K, D=D, dtype="bf16" if bf16 else "f32", normalise=normalise,
                              seed=int(rng.integers(1 << 30)))
        rin = wl.make_route_inputs(rw, "cuda")
        slot = None
        eligible = None
        if use_slot:
            sl = rng.integers(-1, 5, size=K).astype(np.int32)
            if retained and (sl < 0).all():
                sl[int(rng.integers(0, K))] = 3
            slot = torch.from_numpy(sl).cuda()
            eligible = (sl >= 0) if retained else None
        eids, cids, counts = moin.moin_route(ctx, rin.emb, rin.centroids, slot_of_centroid=slot,
                                             retained_only=retained, want_counts=True)
        ctx.check()
        gc.check_route(rin.emb, rin.centroids, cids, eligible=eligible)
        c = cids.cpu().numpy()
        assert np.array_equal(counts.cpu().numpy(), np.bincount(c, minlength=K))
        want_e = c if slot is None else slot.cpu().numpy()[c]
        assert np.array_equal(eids.cpu().numpy(), want_e)


@pytest.mark.parametrize("block", range(2))
def test_random_kmeans_update_cases(block):
    from tests.test_gpu_kmeans import _check_update, _inputs
    rng = np.random.default_rng(9800 + block)
    for i in range(8):
        bf16 = bool(rng.random() < 0.5)
        N = int(rng.choice([1, 50, 1000, 5000, 70000]))
        K = int(rng.choice([1, 3, 64, 500, 2000]))
        D = int(rng.choice([8, 64, 136, 768]) if bf16 else rng.choice([4, 36, 64, 260]))
        # skewed assignment with empty clusters: ids drawn from a few of the centres only
        pool = rng.choice(K, size=max(1, K // int(rng.choice([1, 2, 10]))), replace=False)
        ids = pool[rng.integers(0, len(pool), size=N)]
        what = f"kmeans block {block} case {i}: N={N} K={K} D={D} {'bf16' if bf16 else 'f32'}"
        print("[gpu] random " + what, flush=True)
        emb, ids_t, cent = _inputs(N, K, D, torch.bfloat16 if bf16 else torch.float32, int(rng.integers(1 << 30)), ids)
        _check_update(emb, ids_t, cent, what)
