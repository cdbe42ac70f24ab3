#!/usr/bin/env python3
"""Benchmark of the MoIN hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch of the q_proj
prefill workload (64 sequences x 512 tokens, 2048 -> 2048, rank 64, 500
experts): route the 64 sequence embeddings to their nearest topic (with
histogram and slot map), group the batch by expert, then the routed LoRA
linear layer.  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line: whole-path TFLOP/s (`value`), the roofline of the
dominant kernel measured with HIP events on the launch stream, what the box
itself sustains (an MFMA-only loop and a streaming read, beside the datasheet
peaks), and the CPU oracle timed on a bounded sample of the same workload.
`--also` adds further workloads as extra objects: decode (GB/s), router
(queries/s, and the four nearest topics of a request-sized batch), the full
layer, the K-means update, the quantised base (step, layer, decode), an
activation inside the adapters, and one expert per token.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2410_09687_amd import moin  # noqa: E402
from paper_2410_09687_amd import workloads as wl  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_FP8_TFLOPS = 5000.0    # MI355X dense FP8 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_all_workloads.md")


def measured_traffic(kernel, workload):
    """HBM-side bytes per launch of `kernel` on `workload`, from the committed summary of the two
    rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE; KiB per dispatch, each scaled by what the same counter
    reads for a plain copy of known size).  The summary carries one line per kernel of the form
    `traffic: kernel=<name> workload=<name> bytes=<n>`; None when it has none for this pair (the
    counters cannot be read from inside a timed run)."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                if line.startswith("traffic:"):
                    kv = dict(tok.split("=", 1) for tok in line.split()[1:] if "=" in tok)
                    if kv.get("kernel") == kernel and kv.get("workload") == workload:
                        return int(float(kv["bytes"]))
    except OSError:
        pass
    return None


def decode_traffic(workload):
    """HBM-side bytes of a decode call: its two launches together (None when the summary lacks either)."""
    parts = [measured_traffic(k, workload) for k in ("decode_base_shrink_kernel", "decode_expand_kernel")]
    return None if None in parts else sum(parts)


PREWARM_STEPS = 150   # untimed steps of the headline workload before its warm-up (clock ramp from idle)


def timed_region(fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(steps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return start.elapsed_time(stop) / steps, wall * 1e3 / steps


def step_stats(fn, steps):
    """Median and minimum of the single steps: a second pass over the same steps with an event between
    every two of them (the mean that `value` is computed from comes from the undisturbed loop above)."""
    n = max(int(steps), 50)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    torch.cuda.synchronize()
    ev[0].record()
    for i in range(n):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    t = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(n)])
    return {"median_ms": float(np.median(t)), "min_ms": float(t.min()), "steps": n}


def kernel_times(ctx, fn, steps):
    """Average launch duration per kernel id, from HIP events the library records
    around each launch on the launch stream."""
    ctx.timing_reset()
    ctx.timing_enable(True)
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    out = {}
    for kid, name in enumerate(moin.KERNEL_NAMES):
        ms, n = ctx.timing_read(kid)
        if n:
            out[name] = {"avg_ms": ms / n, "launches": n}
    ctx.timing_enable(False)
    ctx.timing_reset()
    return out


def parity_stats(y_gpu, ref, rows=None):
    """rel-Frobenius and max-abs error of the GPU output against oracle rows (fp64)."""
    y = y_gpu if rows is None else y_gpu[torch.as_tensor(np.asarray(rows), device=y_gpu.device)]
    y = y.float().cpu().double().numpy()
    err = np.abs(y - ref)
    return {"rel_fro": float(np.linalg.norm(y - ref) / max(np.linalg.norm(ref), 1e-30)),
            "max_abs": float(err.max()) if err.size else 0.0, "rows": int(ref.shape[0])}


def cpu_baseline_prefill(inp, y=None, target_s=12.0):
    """Times the oracle, as it stands, on a bounded sample of the batch's rows; with y, the GPU's output for
    the same batch, also reports its error against those oracle rows."""
    import oracle
    A, B, ids = wl.compact_stacks(inp)
    x, W = wl.bf16_bits(inp.x), wl.bf16_bits(inp.W)
    off = inp.seq_offsets.cpu().numpy()
    w = inp.wl
    threads = min(oracle.max_threads(), os.cpu_count() or 1)
    per_row = 2.0 * w.d_in * w.d_out + 2.0 * w.r * (w.d_in + w.d_out)
    rng = np.random.default_rng(0)
    probe = np.sort(rng.choice(w.T, size=min(w.T, 4 * threads), replace=False))
    t0 = time.perf_counter()
    oracle.lora_linear(x, off, ids, W, A, B, w.scale, rows=probe, threads=threads)
    dt = time.perf_counter() - t0
    n = int(min(w.T, max(len(probe), target_s / max(dt / len(probe), 1e-9))))
    rows = np.sort(rng.choice(w.T, size=n, replace=False))
    t0 = time.perf_counter()
    ref = oracle.lora_linear(x, off, ids, W, A, B, w.scale, rows=rows, threads=threads)
    dt = time.perf_counter() - t0
    out = {"value": per_row * n / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
           "sample": f"{n} of {w.T} token rows of the same batch (all {w.d_out} outputs each), "
                     f"fp64 oracle, {dt:.1f} s"}
    if y is not None:
        out["gpu_vs_oracle"] = parity_stats(y, ref, rows)
    return out


def oracle_on_rows(inp, rows, y):
    """Oracle seconds and GPU-vs-oracle error for the given token rows of a batch."""
    import oracle
    A, B, ids = wl.compact_stacks(inp)
    threads = min(oracle.max_threads(), os.cpu_count() or 1)
    t0 = time.perf_counter()
    ref = oracle.lora_linear(wl.bf16_bits(inp.x), inp.seq_offsets.cpu().numpy(), ids, wl.bf16_bits(inp.W), A, B,
                             inp.wl.scale, rows=rows, threads=threads)
    dt = time.perf_counter() - t0
    return dt, threads, parity_stats(y, ref, rows)


def bench_ceilings(ctx):
    """What this very box sustains, beside the datasheet peaks: a loop of bf16 MFMAs alone on N(0,1)
    operands (the matrix cores reach their power limit on random data well below the datasheet figure) and a
    plain streaming read of 1 GiB.  About 40 ms of GPU time."""
    g = torch.Generator(device="cuda").manual_seed(20241013)
    ops = torch.randn((1 << 20,), device="cuda", generator=g).to(torch.bfloat16)
    buf = torch.empty(1 << 28, dtype=torch.int32, device="cuda").fill_(1)
    iters = 20000
    flops = [0.0]

    def run():
        flops[0] = moin.moin_probe_mfma_bf16(ctx, ops, iters)[1]
        moin.moin_probe_read(ctx, buf)

    run()
    kt = kernel_times(ctx, run, 3)
    ctx.check()
    # the block-scaled FP8 instruction on the codes of the same N(0,1) values
    codes, _ = moin.moin_mx_quantize(ctx, ops.view(-1, 128))
    fl8 = [0.0]

    def run8():
        fl8[0] = moin.moin_probe_mfma_mxfp8(ctx, codes.view(-1), iters)[1]

    run8()
    kt8 = kernel_times(ctx, run8, 3)
    ctx.check()
    return {"mfma_bf16_TFLOPs": flops[0] / (kt["probe_mfma"]["avg_ms"] * 1e-3) / 1e12,
            "mfma_mxfp8_TFLOPs": fl8[0] / (kt8["probe_mfma"]["avg_ms"] * 1e-3) / 1e12,
            "read_GBps": buf.numel() * 4.0 / (kt["probe_read"]["avg_ms"] * 1e-3) / 1e9,
            "what": "MFMA-only loops (v_mfma_f32_16x16x32_bf16, the instruction of the prefill and router kernels, on N(0,1) operands; "
                    "v_mfma_scale_f32_32x32x64_f8f6f4 on their MXFP8 codes; 2 workgroups of 8 waves per "
                    "compute unit); streaming read of 1 GiB (two workgroups per compute unit take 32 KB chunks in turn, "
                    "non-temporal 16-byte loads, 8 in flight per thread: the fastest of the shapes swept)"}


def bench_prefill(ctx, steps, warmup, with_cpu):
    w = wl.config_prefill()
    inp = wl.make_linear_inputs(w, "cuda")
    # the batch's 64 sequence embeddings, one topic per resident expert
    rw = wl.RouteWorkload("c1_route", N=w.S, K=w.E, D=768, dtype="bf16", normalise=True, seed=w.seed)
    rin = wl.make_route_inputs(rw, "cuda")
    slots = torch.arange(w.E, dtype=torch.int32, device="cuda")
    y = torch.empty((w.T, w.d_out), dtype=torch.bfloat16, device="cuda")

    # a serving loop: every batch is routed against the same topic table, and says so
    route_out = (torch.empty(w.S, dtype=torch.int32, device="cuda"), None,
                 torch.empty(w.E, dtype=torch.int32, device="cuda"))

    plan = moin.Plan(ctx)

    def step():
        # routing, histogram, slot map and grouping: one launch for a request-sized batch
        moin.moin_route_plan(ctx, plan, rin.emb, rin.centroids, inp.seq_offsets, w.T, w.E,
                             slot_of_centroid=slots, out=route_out, same_centroids=True)
        moin.moin_lora_linear_planned(ctx, plan, inp.x, inp.W, inp.A_stack, inp.B_stack, w.scale, out=y)

    # The chip takes tens of milliseconds of load to leave its idle clocks: bring it to its working state
    # first (untimed, like the set-up above), so that the W warm-up steps and the K timed ones measure the
    # steady state whatever W is.
    for _ in range(PREWARM_STEPS):
        step()
    torch.cuda.synchronize()
    ms, wall_ms = timed_region(step, steps, warmup)
    ctx.check()
    stats = step_stats(step, steps)
    flops = w.flops() + rw.flops()
    kt = kernel_times(ctx, step, steps)
    lin = kt.get("linear", {"avg_ms": float("nan")})
    lin_flops = 2.0 * w.T * w.d_in * w.d_out + 2.0 * w.T * w.r * w.d_out
    achieved = lin_flops / (lin["avg_ms"] * 1e-3) / 1e12
    res = {
        "metric": "routed-LoRA linear TFLOP/s & decode GB/s (% of MI355X roofline); route qps",
        "value": flops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1]: q_proj prefill 2048->2048, r=64, E=500, 64 seq x 512 tok, "
                               "uniform expert ids; step = route(64x768 vs 500 centroids)+histogram+"
                               "slot map+group-by-expert+routed LoRA linear.  `value` is this workload's (the "
                               "one the metric's prefill figure is quoted on); the largest single-GPU "
                               "configuration, configs[4], is reported under `layer`, decode (configs[2], per "
                               "projection, the batch's plan built once outside the timed call as one plan "
                               "serves every projection of every layer) under `decode`, configs[3] under `router`",
                   "ms_per_step_median": stats["median_ms"], "ms_per_step_min": stats["min_ms"],
                   "tokens_per_step": w.T, "tokens_per_s": w.T / (ms * 1e-3),
                   "frac_of_bf16_peak": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                   "wall_ms_per_step": wall_ms, "prewarm_steps": PREWARM_STEPS},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                     "traffic": measured_traffic("linear_stream_kernel", "c1"),
                     "kernel": "linear_stream_kernel (base GEMM + fused expand)",
                     "avg_launch_ms": lin["avg_ms"]},
        "kernels": kt,
    }
    if with_cpu:
        # the routed ids of the step are inp.expert_ids' topics only if the route says so: take them from it
        eids = route_out[0].clone()
        chk = wl.LinearInputs(inp.wl, inp.x, inp.W, inp.A_stack, inp.B_stack, inp.seq_offsets, eids)
        res["cpu_baseline"] = cpu_baseline_prefill(chk, y)
    return res


def bench_decode(ctx, steps, warmup, n_draws=8, with_cpu=False):
    """configs[2]: three MLP projections, 256 single-token sequences, Zipf(1.1)
    ids over 5000 experts.  Rotates through independent id draws so the adapter
    working set (>= 2 GB) exceeds the 256 MB last-level cache."""
    out = {}
    for w in wl.config_decode():
        inp = wl.make_linear_inputs(w, "cuda")
        draws, plans, bytes_alg = [], [], []
        for k in range(n_draws):
            ids = wl.draw_expert_ids(w.S, w.E, "zipf", w.zipf_s, w.seed * 8 + 100 + k)
            t = torch.from_numpy(ids).cuda()
            draws.append(t)
            plans.append(moin.Plan(ctx).build(inp.seq_offsets, t, w.T, w.E))
            distinct = len(np.unique(ids))
            bytes_alg.append(2.0 * w.d_in * w.d_out + distinct * 2.0 * w.r * (w.d_in + w.d_out)
                             + 2.0 * w.T * (w.d_in + w.d_out))
        y = torch.empty((w.T, w.d_out), dtype=torch.bfloat16, device="cuda")
        state = {"i": 0}

        def step():
            k = state["i"] % n_draws
            state["i"] += 1
            moin.moin_lora_linear_planned(ctx, plans[k], inp.x, inp.W, inp.A_stack, inp.B_stack,
                                          w.scale, out=y)

        n = max(steps, n_draws) // n_draws * n_draws
        state["i"] = 0
        ms, _ = timed_region(step, n, max(warmup, n_draws))
        ctx.check()
        state["i"] = 0
        stats = step_stats(step, n)
        state["i"] = 0
        kt = kernel_times(ctx, step, n)
        avg_bytes = float(np.mean(bytes_alg))
        cpu = None
        if with_cpu:
            # the whole batch of draw 0 through the oracle: its time, and the GPU's error against it
            state["i"] = 0
            step()
            torch.cuda.synchronize()
            chk = wl.LinearInputs(inp.wl, inp.x, inp.W, inp.A_stack, inp.B_stack, inp.seq_offsets, draws[0])
            dt, threads, par = oracle_on_rows(chk, None, y)
            cpu = {"value": w.flops() / dt / 1e12, "unit": "TFLOP/s", "seconds": dt, "cores": threads,
                   "kind": "oracle", "sample": f"all {w.T} rows of one batch", "gpu_vs_oracle": par}
        out[w.name] = {"ms_per_call": ms, "ms_per_call_median": stats["median_ms"], "ms_per_call_min": stats["min_ms"],
                       "plan": "built once per batch outside the timed call", "cpu_baseline": cpu,
                       "algorithmic_bytes": avg_bytes,
                       "GBps": avg_bytes / (ms * 1e-3) / 1e9,
                       "frac_of_hbm_peak": avg_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                       "roofline": {"bound": "hbm", "achieved": avg_bytes / (ms * 1e-3) / 1e9,
                                    "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                    "frac": avg_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                    "traffic": decode_traffic("c2_down" if "down" in w.name else "c2_gate_up")},
                       "kernels": kt}
        for p in plans:
            p.close()
        del inp, draws, plans
        torch.cuda.empty_cache()

    # gate and up read the same x: one call for both (their base tiles and shrink slabs in one launch,
    # their expand blocks in another), the way a serving loop would issue them
    ws = {w.name: w for w in wl.config_decode()}
    g, u = ws["c2_gate_decode"], ws["c2_up_decode"]
    ig = wl.make_linear_inputs(g, "cuda")
    iu = wl.make_linear_inputs(u, "cuda", x=ig.x)
    plans, bytes_alg = [], []
    for k in range(n_draws):
        ids = wl.draw_expert_ids(g.S, g.E, "zipf", g.zipf_s, g.seed * 8 + 100 + k)
        plans.append(moin.Plan(ctx).build(ig.seq_offsets, torch.from_numpy(ids).cuda(), g.T, g.E))
        distinct = len(np.unique(ids))
        bytes_alg.append(sum(2.0 * w.d_in * w.d_out + distinct * 2.0 * w.r * (w.d_in + w.d_out)
                             + 2.0 * w.T * (w.d_in + w.d_out) for w in (g, u)))
    ys = [torch.empty((g.T, w.d_out), dtype=torch.bfloat16, device="cuda") for w in (g, u)]
    state = {"i": 0}

    def step2():
        k = state["i"] % n_draws
        state["i"] += 1
        moin.moin_lora_linear_planned_shared(ctx, plans[k], ig.x, [ig.W, iu.W], [ig.A_stack, iu.A_stack],
                                             [ig.B_stack, iu.B_stack], g.scale, outs=ys)

    n = max(steps, n_draws) // n_draws * n_draws
    ms, _ = timed_region(step2, n, max(warmup, n_draws))
    ctx.check()
    state["i"] = 0
    stats = step_stats(step2, n)
    state["i"] = 0
    kt = kernel_times(ctx, step2, n)
    avg_bytes = float(np.mean(bytes_alg))
    out["c2_gate_and_up_one_call"] = {
        "ms_per_call": ms, "ms_per_call_median": stats["median_ms"], "ms_per_call_min": stats["min_ms"],
        "projections": 2, "ms_per_projection": ms / 2, "plan": "built once per batch outside the timed call",
        "algorithmic_bytes": avg_bytes, "GBps": avg_bytes / (ms * 1e-3) / 1e9,
        "frac_of_hbm_peak": avg_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "roofline": {"bound": "hbm", "achieved": avg_bytes / (ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": avg_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                     "traffic": decode_traffic("c2_gate_and_up_one_call")},
        "kernels": kt}
    for p in plans:
        p.close()
    del ig, iu, plans, ys
    torch.cuda.empty_cache()
    return out


def cpu_baseline_router(rin, rw, cids):
    """The oracle on every 16th query (all K centroids each), its time extrapolated linearly to the whole
    batch; the GPU's ids on those queries against it (a different id counts as a mismatch unless its
    squared distance, in fp64, is within 1e-4 relative of the minimum)."""
    import oracle
    sel = np.arange(0, rw.N, 16)
    q = wl.bf16_bits(rin.emb[::16].contiguous())
    c = wl.bf16_bits(rin.centroids)
    t0 = time.perf_counter()
    ref, best, _ = oracle.route(q, c, want_gaps=True)
    dt = time.perf_counter() - t0
    got = cids.cpu().numpy()[sel]
    bad = np.flatnonzero(got != ref)
    outside = 0
    if bad.size:
        d = oracle.dist2(q, c, bad, got[bad])
        outside = int((d > np.where(best[bad] > 0, best[bad] * (1 + 1e-4), 1e-30)).sum())
    return {"value": 2.0 * sel.size * rw.K * rw.D / dt / 1e12, "unit": "TFLOP/s", "seconds_on_sample": dt,
            "seconds_whole_batch_extrapolated": dt * rw.N / sel.size, "cores": oracle.max_threads(),
            "kind": "oracle", "sample": f"every 16th query ({sel.size} of {rw.N}), all {rw.K} centroids",
            "gpu_vs_oracle": {"queries": int(sel.size), "ids_differing_inside_the_near_tie_band": int(bad.size) - outside,
                              "ids_differing_outside_it": outside}}


def bench_router(ctx, steps, warmup, with_cpu=False):
    rw = wl.config_router()
    rin = wl.make_route_inputs(rw, "cuda")
    outs = (torch.empty(rw.N, dtype=torch.int32, device="cuda"), torch.empty(rw.N, dtype=torch.int32, device="cuda"),
            torch.empty(rw.K, dtype=torch.int32, device="cuda"))

    def step():
        moin.moin_route(ctx, rin.emb, rin.centroids, want_counts=True, out=outs)

    ms, _ = timed_region(step, steps, warmup)
    ctx.check()
    stats = step_stats(step, steps)
    kt = kernel_times(ctx, step, steps)
    tf = rw.flops() / (ms * 1e-3) / 1e12
    # request-time batch: the four nearest topics of 4096 queries ("Future Works", creating new experts on the fly)
    q = rin.emb[:4096]

    def topk():
        moin.moin_route_topk(ctx, q, rin.centroids, 4)

    tms, _ = timed_region(topk, 10, 2)
    ctx.check()
    cpu = cpu_baseline_router(rin, rw, outs[1]) if with_cpu else None
    return {"ms_per_call": ms, "ms_per_call_median": stats["median_ms"], "ms_per_call_min": stats["min_ms"],
            "queries_per_s": rw.N / (ms * 1e-3), "TFLOPs": tf,
            "frac_of_bf16_peak": tf / PEAK_BF16_TFLOPS, "cpu_baseline": cpu,
            "traffic": measured_traffic("route_stream4_kernel", "c3"),
            "top4_of_4096_queries": {"ms_per_call": tms, "queries_per_s": 4096 / (tms * 1e-3)}, "kernels": kt}


def bench_kmeans(ctx, steps, warmup):
    """One Lloyd iteration on the router workload (configs[3] shapes): assignment =
    moin_route, then the centre update, which reads every embedding once."""
    rw = wl.config_router()
    rin = wl.make_route_inputs(rw, "cuda")
    ids, _, _ = moin.moin_route(ctx, rin.emb, rin.centroids, want_counts=False)
    new = torch.empty_like(rin.centroids)

    def step():
        moin.moin_kmeans_update(ctx, rin.emb, ids, rin.centroids, out=new)

    ms, _ = timed_region(step, steps, warmup)
    ctx.check()
    kt = kernel_times(ctx, step, steps)
    # what the update must move: every embedding and id once, old and new centres
    bytes_alg = rw.N * rw.D * 2.0 + rw.N * 4.0 + 2 * rw.K * rw.D * 2.0
    seg = kt.get("kmeans_sum", {"avg_ms": float("nan")})
    gbs = bytes_alg / (seg["avg_ms"] * 1e-3) / 1e9
    return {"ms_per_update": ms, "points_per_s": rw.N / (ms * 1e-3), "algorithmic_bytes": bytes_alg,
            "GBps_whole_update": bytes_alg / (ms * 1e-3) / 1e9,
            "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": gbs / PEAK_HBM_GBS, "kernel": "km_segsum", "avg_launch_ms": seg["avg_ms"]},
            "kernels": kt}


def bench_ranks(ctx, steps, warmup, n_draws=8):
    """configs[2] gate projection with a rank per expert ("Future Works": larger adapters
    for bigger topics): the 10 % most popular experts keep rank 128, the next 30 % get 64,
    the rest 32.  The decode kernels read only rank_e rows / columns of each distinct
    adapter; algorithmic bytes shrink accordingly."""
    w = wl.config_decode()[0]
    inp = wl.make_linear_inputs(w, "cuda")
    perm = np.random.default_rng(777).permutation(w.E)          # popularity order of this stream
    ranks = np.full(w.E, 32, np.int32)
    ranks[perm[: w.E * 4 // 10]] = 64
    ranks[perm[: w.E // 10]] = 128
    ranks_dev = torch.from_numpy(ranks).cuda()
    out = {}
    for label, rk in (("full_rank", None), ("adaptive_rank", ranks_dev)):
        plans, bytes_alg = [], []
        for k in range(n_draws):
            ids = wl.draw_expert_ids(w.S, w.E, "zipf", w.zipf_s, 9000 + k, perm_seed=777)
            plans.append(moin.Plan(ctx).build(inp.seq_offsets, torch.from_numpy(ids).cuda(), w.T, w.E,
                                              rank_of_expert=rk))
            per = np.array([w.r if rk is None else ranks[e] for e in np.unique(ids)], np.float64)
            bytes_alg.append(2.0 * w.d_in * w.d_out + per.sum() * 2.0 * (w.d_in + w.d_out)
                             + 2.0 * w.T * (w.d_in + w.d_out))
        y = torch.empty((w.T, w.d_out), dtype=torch.bfloat16, device="cuda")
        state = {"i": 0}

        def step():
            k = state["i"] % n_draws
            state["i"] += 1
            moin.moin_lora_linear_planned(ctx, plans[k], inp.x, inp.W, inp.A_stack, inp.B_stack, w.scale, out=y)

        n = max(steps, n_draws) // n_draws * n_draws
        ms, _ = timed_region(step, n, max(warmup, n_draws))
        ctx.check()
        avg = float(np.mean(bytes_alg))
        out[label] = {"ms_per_call": ms, "algorithmic_bytes": avg, "GBps": avg / (ms * 1e-3) / 1e9}
        for p in plans:
            p.close()
    return out


def bench_mx(ctx, steps, warmup):
    """configs[1] projection on a quantised base ("Future Works", quantising the base model):
    W held as MXFP8 codes + scales, x quantised per call, base product on the block-scaled FP8
    matrix cores, adapter term in bf16.  Same step as the headline (route + plan + layer);
    the roofline is that of the main kernel against the dense FP8 peak."""
    w = wl.config_prefill()
    inp = wl.make_linear_inputs(w, "cuda")
    rw = wl.RouteWorkload("c1_route", N=w.S, K=w.E, D=768, dtype="bf16", normalise=True, seed=w.seed)
    rin = wl.make_route_inputs(rw, "cuda")
    slots = torch.arange(w.E, dtype=torch.int32, device="cuda")
    y = torch.empty((w.T, w.d_out), dtype=torch.bfloat16, device="cuda")
    Wq, Ws = moin.moin_mx_quantize(ctx, inp.W, blocked=True)

    def step():
        eids, _, _ = moin.moin_route(ctx, rin.emb, rin.centroids, slot_of_centroid=slots,
                                     want_centroid_ids=False, want_counts=True)
        moin.moin_lora_linear_mx(ctx, inp.x, inp.seq_offsets, eids, Wq, Ws, inp.A_stack, inp.B_stack,
                                 w.scale, out=y)

    ms, _ = timed_region(step, steps, warmup)
    ctx.check()
    kt = kernel_times(ctx, step, steps)
    lin = kt.get("mx_linear", {"avg_ms": float("nan")})
    qt = kt.get("shrink", {"avg_ms": float("nan")})
    base_flops = 2.0 * w.T * w.d_in * w.d_out
    lora_flops = 2.0 * w.T * w.r * w.d_out
    # the kernel mixes FP8 (base) and bf16 (adapter) MFMA work: time at peak = sum of both
    t_peak = base_flops / (PEAK_FP8_TFLOPS * 1e12) + 2.0 * lora_flops / (PEAK_BF16_TFLOPS * 1e12)
    achieved = (base_flops + lora_flops) / (lin["avg_ms"] * 1e-3) / 1e12
    # the shrink's pass over x also writes x's codes and scales: x once, A_e of the distinct experts,
    # u as a bf16 pair, codes, scale bytes
    n_distinct = int(torch.unique(inp.expert_ids[inp.expert_ids >= 0]).numel())
    q_bytes = w.T * w.d_in * (2.0 + 1.0 + 1.0 / 32) + n_distinct * w.r * w.d_in * 2.0 + w.T * w.r * 4.0
    return {"ms_per_step": ms, "TFLOPs_whole_step": (w.flops() + rw.flops()) / (ms * 1e-3) / 1e12,
            "tokens_per_s": w.T / (ms * 1e-3),
            "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP8_TFLOPS, "unit": "TFLOP/s",
                         "frac": achieved / PEAK_FP8_TFLOPS,
                         "frac_of_mixed_peak": t_peak / (lin["avg_ms"] * 1e-3),
                         "traffic": measured_traffic("linear_stream4_kernel", "c1_mx"),
                         "kernel": "linear_mx_stream_kernel (MXFP8 base + bf16 adapter term)",
                         "avg_launch_ms": lin["avg_ms"]},
            "shrink_and_quantise_x": {"avg_launch_ms": qt["avg_ms"], "algorithmic_bytes": q_bytes,
                                      "GBps": q_bytes / (qt["avg_ms"] * 1e-3) / 1e9},
            "kernels": kt}


def bench_activation(ctx, steps, warmup):
    """configs[1] projection with an activation between the adapter's two layers ("Future Works", better
    adapters): SiLU on W_a x in the shrink's epilogue; same kernels and bytes as the headline step."""
    w = wl.config_prefill()
    inp = wl.make_linear_inputs(w, "cuda")
    y = torch.empty((w.T, w.d_out), dtype=torch.bfloat16, device="cuda")
    plan = moin.Plan(ctx).build(inp.seq_offsets, inp.expert_ids, w.T, w.E)
    out = {}
    try:
        for act in (None, "silu"):
            ctx.set_adapter_activation(act)

            def step():
                moin.moin_lora_linear_planned(ctx, plan, inp.x, inp.W, inp.A_stack, inp.B_stack, w.scale, out=y)

            ms, _ = timed_region(step, steps, warmup)
            ctx.check()
            kt = kernel_times(ctx, step, steps)
            out[act or "none"] = {"ms_per_call": ms, "shrink_us": kt["shrink"]["avg_ms"] * 1e3,
                                  "linear_us": kt["linear"]["avg_ms"] * 1e3}
    finally:
        ctx.set_adapter_activation(None)
        plan.close()
    return out


def bench_per_token(ctx, steps, warmup):
    """One expert per token ("Future Works", per token adapters) at serving size: 8192 single-token sequences
    through the gate projection of configs[2] (2048 -> 5632, r = 128, 5000 experts, Zipf(1.1) ids).  The
    batch takes the path that gathers tokens by expert; bound by the adapters' bytes."""
    w0 = wl.config_decode()[0]
    T = 8192
    w = wl.LinearWorkload("per_token_gate", w0.d_in, w0.d_out, w0.r, w0.E, [1] * T, "zipf", 1.1, w0.scale,
                          seed=w0.seed + 77)
    inp = wl.make_linear_inputs(w, "cuda")
    y = torch.empty((T, w.d_out), dtype=torch.bfloat16, device="cuda")
    plan = moin.Plan(ctx)

    def build():
        plan.build(inp.seq_offsets, inp.expert_ids, T, w.E)

    build()
    plan_ms, _ = timed_region(build, 5, 1)

    def step():
        moin.moin_lora_linear_planned(ctx, plan, inp.x, inp.W, inp.A_stack, inp.B_stack, w.scale, out=y)

    ms, _ = timed_region(step, max(5, steps // 5), 2)
    ctx.check()
    kt = kernel_times(ctx, step, 5)
    distinct = int(torch.unique(inp.expert_ids).numel())
    nbytes = 2.0 * w.d_in * w.d_out + distinct * 2.0 * w.r * (w.d_in + w.d_out) + 2.0 * T * (w.d_in + w.d_out)
    flops = 2.0 * T * w.d_in * w.d_out + 2.0 * T * w.r * (w.d_in + w.d_out)
    plan.close()
    return {"tokens": T, "distinct_experts": distinct, "ms_per_call": ms, "plan_ms": plan_ms,
            "tokens_per_s": T / (ms * 1e-3), "TFLOPs": flops / (ms * 1e-3) / 1e12,
            "roofline": {"bound": "hbm", "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
            "algorithmic_bytes": nbytes, "kernels": kt}


def bench_cache(ctx, n_batches=48, n_slots=256, n_experts=1000):
    """Decode batches of the gate projection (configs[2] shapes) served through the adapter
    residency cache: `n_experts` experts in pinned host memory (2 MB each), `n_slots` resident, one
    request stream with a fixed Zipf(1.1) popularity order, the cache in overlap mode (batch k+1 admitted
    right after batch k's kernels were enqueued: its adapters cross PCIe under them).  Reports the hit
    rate, the host-to-device rate of the misses and the time per batch against the all-resident case."""
    import dataclasses
    w = dataclasses.replace(wl.config_decode()[0], E=n_experts)
    per_a, per_b = w.r * w.d_in, w.d_out * w.r
    blk = wl._randn_bf16((1 << 24,), 0.02, torch.device("cpu"), 99)      # 32 MB of values, repeated
    def host_stack(per):
        t = torch.empty((w.E, per), dtype=torch.bfloat16, pin_memory=True)
        flat = t.view(-1)
        for lo in range(0, flat.numel(), blk.numel()):
            n = min(blk.numel(), flat.numel() - lo)
            flat[lo:lo + n] = blk[:n]
        return t
    A_host = host_stack(per_a).view(w.E, w.r, w.d_in)
    B_host = host_stack(per_b).view(w.E, w.d_out, w.r)
    A_slots = torch.zeros((n_slots, w.r, w.d_in), dtype=torch.bfloat16, device="cuda")
    B_slots = torch.zeros((n_slots, w.d_out, w.r), dtype=torch.bfloat16, device="cuda")
    W = wl._randn_bf16((w.d_out, w.d_in), w.d_in ** -0.5, torch.device("cuda"), 5)
    x = wl._randn_bf16((w.T, w.d_in), 1.0, torch.device("cuda"), 6)
    off = torch.from_numpy(wl.seq_offsets_of(w.seq_lens)).cuda()
    y = torch.empty((w.T, w.d_out), dtype=torch.bfloat16, device="cuda")
    cache = moin.Cache(w.E, n_slots, overlap=True)
    cache.add_stack(A_host, B_host, A_slots, B_slots)
    batches = [wl.draw_expert_ids(w.S, w.E, "zipf", w.zipf_s, 5000 + k, perm_seed=4242) for k in range(2 * n_batches)]

    def serve(seq):
        # look-ahead pipeline: kernels of batch k, then the admission of batch k+1
        slots = cache.admit(seq[0])
        for k in range(len(seq)):
            moin.moin_lora_linear(ctx, x, off, slots.cuda(), W, A_slots, B_slots, w.scale, out=y)
            if k + 1 < len(seq):
                slots = cache.admit(seq[k + 1])

    serve(batches[:n_batches])       # warm the cache
    torch.cuda.synchronize()
    s0 = cache.stats()
    t0 = time.perf_counter()
    serve(batches[n_batches:])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    s1 = cache.stats()
    ctx.check()
    d = {k: s1[k] - s0[k] for k in s1}
    # all-resident reference: the same batches, slot ids = what the warm cache holds (no copies)
    slots_dev = [cache.admit(ids).cuda() for ids in batches[n_batches:n_batches + 8]]
    torch.cuda.synchronize()
    ms_res, _ = timed_region(lambda: [moin.moin_lora_linear(ctx, x, off, sd, W, A_slots, B_slots, w.scale, out=y)
                                      for sd in slots_dev], 4, 1)
    cache.close()
    return {"experts": w.E, "slots": n_slots, "bytes_per_expert": 2 * (per_a + per_b),
            "hit_rate": d["seq_hits"] / max(1, d["seq_hits"] + d["seq_misses"]),
            "loads_per_batch": d["loads"] / n_batches, "h2d_GB_per_batch": d["bytes"] / n_batches / 1e9,
            "ms_per_batch": dt * 1e3 / n_batches, "h2d_GBps_over_the_batch_time": d["bytes"] / dt / 1e9,
            "ms_per_batch_all_resident": ms_res / len(slots_dev), "overflows": d["overflows"]}


def rows_per_sequence(off, seed, n_edge=16, n_random=32):
    """The first and last n_edge rows of every sequence and n_random seeded rows from its middle."""
    rng = np.random.default_rng(seed)
    picks = []
    for s in range(len(off) - 1):
        lo, hi = int(off[s]), int(off[s + 1])
        if hi - lo <= 2 * n_edge + n_random:
            picks.append(np.arange(lo, hi))
            continue
        picks += [np.arange(lo, lo + n_edge), np.arange(hi - n_edge, hi),
                  rng.choice(np.arange(lo + n_edge, hi - n_edge), size=n_random, replace=False)]
    return np.unique(np.concatenate(picks)).astype(np.int64)


def bench_layer(ctx, steps, warmup, with_cpu=False):
    """configs[4]: seven chained projections, r=128, E=5000, 32 x 2048 tokens, Zipf(1.5)."""
    wls = wl.config_layer()
    T = wls[0].T
    ids = wl.draw_expert_ids(wls[0].S, wls[0].E, "zipf", 1.5, wls[0].seed * 8 + 4)
    off = torch.from_numpy(wl.seq_offsets_of(wls[0].seq_lens)).cuda()
    eids = torch.from_numpy(ids).cuda()
    h0 = wl._randn_bf16((T, 2048), 1.0, torch.device("cuda"), 4242)
    inputs = {w.name.split("_", 1)[1]: wl.make_linear_inputs(w, "cuda", expert_ids=ids, x=h0[:1])
              for w in wls}
    outs = {n: torch.empty((T, i.wl.d_out), dtype=torch.bfloat16, device="cuda") for n, i in inputs.items()}
    src = {"q": None, "k": None, "v": None, "o": "q", "gate": "o", "up": "o", "down": "gate"}
    plan = moin.Plan(ctx)

    # projections that read the same input go through one call (their adapters' first products come out of
    # one pass over it): q, k, v; o; gate, up; down
    calls = [("q", "k", "v"), ("o",), ("gate", "up"), ("down",)]

    def step():
        plan.build(off, eids, T, wls[0].E)
        for names in calls:
            x = h0 if src[names[0]] is None else outs[src[names[0]]]
            ins = [inputs[n] for n in names]
            moin.moin_lora_linear_planned_shared(ctx, plan, x, [i.W for i in ins], [i.A_stack for i in ins],
                                                 [i.B_stack for i in ins], ins[0].wl.scale,
                                                 outs=[outs[n] for n in names])

    def step_single():
        plan.build(off, eids, T, wls[0].E)
        for n, i in inputs.items():
            x = h0 if src[n] is None else outs[src[n]]
            moin.moin_lora_linear_planned(ctx, plan, x, i.W, i.A_stack, i.B_stack, i.wl.scale, out=outs[n])

    ms, _ = timed_region(step, steps, warmup)
    ctx.check()
    stats = step_stats(step, steps)
    kt = kernel_times(ctx, step, steps)
    # every projection on its own: launch durations by projection (the layer's breakdown)
    per_proj = {}
    plan.build(off, eids, T, wls[0].E)
    for n, i in inputs.items():
        x = h0 if src[n] is None else outs[src[n]]

        def one():
            moin.moin_lora_linear_planned(ctx, plan, x, i.W, i.A_stack, i.B_stack, i.wl.scale, out=outs[n])

        one()
        k1 = kernel_times(ctx, one, 5)
        fl = i.wl.flops()
        t_ms = sum(v["avg_ms"] for v in k1.values())
        per_proj[n] = {"shape": f"{i.wl.d_in}->{i.wl.d_out}", "shrink_us": k1.get("shrink", {"avg_ms": 0})["avg_ms"] * 1e3,
                       "linear_us": k1.get("linear", {"avg_ms": 0})["avg_ms"] * 1e3,
                       "TFLOPs": fl / (t_ms * 1e-3) / 1e12, "frac_of_bf16_peak": fl / (t_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
    ms_single, _ = timed_region(step_single, steps, warmup)
    ctx.check()
    flops = sum(w.flops() for w in wls)
    tf = flops / (ms * 1e-3) / 1e12
    cpu = None
    if with_cpu:
        # 64 rows of every sequence through the oracle, projection by projection on the GPU's actual input
        step()
        torch.cuda.synchronize()
        rows = rows_per_sequence(off.cpu().numpy(), seed=2)
        secs, par, threads = 0.0, {}, 0
        for n, i in inputs.items():
            x = h0 if src[n] is None else outs[src[n]]
            chk = wl.LinearInputs(i.wl, x, i.W, i.A_stack, i.B_stack, off, eids)
            dt, threads, p1 = oracle_on_rows(chk, rows, outs[n])
            secs += dt
            par[n] = p1
        sample_flops = flops * rows.size / T
        cpu = {"value": sample_flops / secs / 1e12, "unit": "TFLOP/s", "seconds_on_sample": secs,
               "seconds_whole_layer_extrapolated": secs * T / rows.size, "cores": threads, "kind": "oracle",
               "sample": f"64 rows of each of the {wls[0].S} sequences (first 16, last 16, 32 seeded), all outputs, "
                         f"all 7 projections ({rows.size} of {T} rows)", "gpu_vs_oracle": par}
    plan.close()
    return {"ms_per_layer": ms, "ms_per_layer_median": stats["median_ms"], "ms_per_layer_min": stats["min_ms"],
            "TFLOPs": tf, "frac_of_bf16_peak": tf / PEAK_BF16_TFLOPS,
            "tokens_per_s": T / (ms * 1e-3), "ms_per_layer_seven_single_calls": ms_single, "per_projection": per_proj,
            "cpu_baseline": cpu, "kernels": kt}


def bench_decode_mx(ctx, steps, warmup, n_draws=8):
    """configs[2] gate projection on the quantised base: activations' quantiser, base product for all
    256 tokens on the FP8 matrix cores (contraction range in parts), then the decode kernels' adapter
    term.  Same request stream and byte count convention as the bf16 decode figure (W counted at
    one byte per element plus its scales)."""
    w = wl.config_decode()[0]
    inp = wl.make_linear_inputs(w, "cuda")
    Wq, Ws = moin.moin_mx_quantize(ctx, inp.W, blocked=True)
    plans, bytes_alg = [], []
    for k in range(n_draws):
        ids = wl.draw_expert_ids(w.S, w.E, "zipf", w.zipf_s, 9000 + k, perm_seed=777)
        plans.append(moin.Plan(ctx).build(inp.seq_offsets, torch.from_numpy(ids).cuda(), w.T, w.E))
        distinct = len(np.unique(ids))
        bytes_alg.append(w.d_in * w.d_out * (1.0 + 1.0 / 32) + distinct * 2.0 * w.r * (w.d_in + w.d_out)
                         + 2.0 * w.T * (w.d_in + w.d_out))
    y = torch.empty((w.T, w.d_out), dtype=torch.bfloat16, device="cuda")
    state = {"i": 0}

    def step():
        k = state["i"] % n_draws
        state["i"] += 1
        moin.moin_lora_linear_mx_planned(ctx, plans[k], inp.x, Wq, Ws, inp.A_stack, inp.B_stack, w.scale, out=y)

    n = max(steps, n_draws) // n_draws * n_draws
    ms, _ = timed_region(step, n, max(warmup, n_draws))
    ctx.check()
    kt = kernel_times(ctx, step, n)
    for p in plans:
        p.close()
    avg = float(np.mean(bytes_alg))
    return {"ms_per_call": ms, "algorithmic_bytes": avg, "GBps": avg / (ms * 1e-3) / 1e9, "kernels": kt}


def bench_layer_mx(ctx, steps, warmup):
    """configs[4] on a quantised base: the seven projections' weights in MXFP8 (quantised once, outside
    the step); activations quantised once per distinct input (q, k, v share theirs, gate and up theirs), by the
    first projection that reads it."""
    wls = wl.config_layer()
    T = wls[0].T
    ids = wl.draw_expert_ids(wls[0].S, wls[0].E, "zipf", 1.5, wls[0].seed * 8 + 4)
    off = torch.from_numpy(wl.seq_offsets_of(wls[0].seq_lens)).cuda()
    eids = torch.from_numpy(ids).cuda()
    h0 = wl._randn_bf16((T, 2048), 1.0, torch.device("cuda"), 4242)
    inputs = {w.name.split("_", 1)[1]: wl.make_linear_inputs(w, "cuda", expert_ids=ids, x=h0[:1])
              for w in wls}
    outs = {n: torch.empty((T, i.wl.d_out), dtype=torch.bfloat16, device="cuda") for n, i in inputs.items()}
    src = {"q": None, "k": None, "v": None, "o": "q", "gate": "o", "up": "o", "down": "gate"}
    wq = {n: moin.moin_mx_quantize(ctx, i.W, blocked=True) for n, i in inputs.items()}
    plan = moin.Plan(ctx)

    codes = {}
    for n, i in inputs.items():
        if src[n] not in codes:
            codes[src[n]] = (torch.empty((T, i.wl.d_in), dtype=torch.uint8, device="cuda"),
                             torch.empty((i.wl.d_in // 128, T, 4), dtype=torch.uint8, device="cuda"))

    def step():
        plan.build(off, eids, T, wls[0].E)
        quantised = set()
        for n, i in inputs.items():
            x = h0 if src[n] is None else outs[src[n]]
            xq, xs = codes[src[n]]
            # the first projection of each distinct input quantises it (in its shrink's pass over x)
            moin.moin_lora_linear_mx_planned(ctx, plan, x, wq[n][0], wq[n][1], i.A_stack, i.B_stack, i.wl.scale,
                                             xq=xq, xs=xs, emit=src[n] not in quantised, out=outs[n])
            quantised.add(src[n])

    ms, _ = timed_region(step, steps, warmup)
    ctx.check()
    kt = kernel_times(ctx, step, steps)
    flops = sum(w.flops() for w in wls)
    tf = flops / (ms * 1e-3) / 1e12
    plan.close()
    return {"ms_per_layer": ms, "TFLOPs": tf, "frac_of_fp8_peak": tf / PEAK_FP8_TFLOPS,
            "tokens_per_s": T / (ms * 1e-3), "kernels": kt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the on-box ceilings (MFMA-only loop, streaming read) reported beside the datasheet peaks")
    ap.add_argument("--copy-mib", type=int, default=0,
                    help="first run a plain device copy of this many MiB (3 times): the known-size "
                         "kernel that calibrates rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--also", default="decode,router,layer,kmeans,cache,mx,act,pertoken",
                    help="comma list of extra workloads to report: decode,router,layer,kmeans,cache,ranks,mx,mx-step,act,pertoken "
                         "(or 'none'); cache pins 2 GB of host memory; ranks is not in the default list; "
                         "mx-step is the headline step on the quantised base alone, mx adds its layer and decode")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (no multi-GPU figure exists)",
              file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.copy_mib > 0:
        src = torch.empty(args.copy_mib << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    ctx = moin.Context(0)
    res = bench_prefill(ctx, args.steps, args.warmup, not args.no_cpu_baseline)
    if not args.no_ceilings:
        # after the headline, so that the probes do not warm or cool the chip ahead of it
        res["measured_ceilings"] = c = bench_ceilings(ctx)
        res["roofline"]["frac_of_measured_mfma_ceiling"] = res["roofline"]["achieved"] / c["mfma_bf16_TFLOPs"]
    extra = [s for s in args.also.split(",") if s and s != "none"]
    if "decode" in extra:
        res["decode"] = bench_decode(ctx, args.steps, args.warmup, with_cpu=not args.no_cpu_baseline)
        if "measured_ceilings" in res:
            for d in res["decode"].values():
                d["roofline"]["frac_of_measured_read_ceiling"] = d["roofline"]["achieved"] / c["read_GBps"]
    if "router" in extra:
        res["router"] = bench_router(ctx, max(5, args.steps // 5), 2, with_cpu=not args.no_cpu_baseline)
    if "layer" in extra:
        res["layer"] = bench_layer(ctx, max(5, args.steps // 5), 2, with_cpu=not args.no_cpu_baseline)
    if "kmeans" in extra:
        res["kmeans"] = bench_kmeans(ctx, max(5, args.steps // 5), 2)
    if "measured_ceilings" in res:
        for k in ("router", "layer"):
            if k in res:
                res[k]["frac_of_measured_mfma_ceiling"] = res[k]["TFLOPs"] / c["mfma_bf16_TFLOPs"]
        if "kmeans" in res:
            res["kmeans"]["roofline"]["frac_of_measured_read_ceiling"] = \
                res["kmeans"]["roofline"]["achieved"] / c["read_GBps"]
    if "act" in extra:
        res["activation"] = bench_activation(ctx, args.steps, args.warmup)
    if "pertoken" in extra:
        res["per_token"] = bench_per_token(ctx, args.steps, args.warmup)
    if "cache" in extra:
        res["cache"] = bench_cache(ctx)
    if "ranks" in extra:
        res["ranks"] = bench_ranks(ctx, args.steps, args.warmup)
    if "mx" in extra or "mx-step" in extra:
        res["mx"] = bench_mx(ctx, args.steps, args.warmup)
        if "measured_ceilings" in res:
            res["mx"]["roofline"]["frac_of_measured_mfma_ceiling"] = \
                res["mx"]["roofline"]["achieved"] / c["mfma_mxfp8_TFLOPs"]
    if "mx" in extra:
        res["mx"]["layer"] = bench_layer_mx(ctx, max(5, args.steps // 5), 2)
        res["mx"]["decode_gate"] = bench_decode_mx(ctx, args.steps, args.warmup)
    ctx.close()
    print(json.dumps(res))


if __name__ == "__main__":
    main()
