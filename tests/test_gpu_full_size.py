"""Parity at the full benchmark sizes, in the launch configuration bench.py
times: sampled outputs the oracle computes one by one, plus properties that
hold at any size."""
import numpy as np
import pytest
import torch

from paper_2410_09687_amd import moin
from paper_2410_09687_amd import workloads as wl
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu


def _sample_rows(T, seq_offsets, n_random, seed):
    """First and last rows of the batch and of a few sequences, plus random rows."""
    rng = np.random.default_rng(seed)
    off = seq_offsets.cpu().numpy()
    picks = {0, T - 1}
    for s in rng.choice(len(off) - 1, size=min(8, len(off) - 1), replace=False):
        if off[s + 1] > off[s]:
            picks.update({int(off[s]), int(off[s + 1] - 1)})
    picks.update(int(v) for v in rng.integers(0, T, size=n_random))
    return np.array(sorted(picks), dtype=np.int64)


def _rows_per_sequence(seq_offsets, seed, n_edge=16, n_random=32):
    """The first and last `n_edge` rows of every sequence plus `n_random` seeded rows from its middle."""
    rng = np.random.default_rng(seed)
    off = seq_offsets.cpu().numpy()
    picks = []
    for s in range(len(off) - 1):
        lo, hi = int(off[s]), int(off[s + 1])
        if hi - lo <= 2 * n_edge + n_random:
            picks.append(np.arange(lo, hi))
            continue
        picks.append(np.arange(lo, lo + n_edge))
        picks.append(np.arange(hi - n_edge, hi))
        picks.append(rng.choice(np.arange(lo + n_edge, hi - n_edge), size=n_random, replace=False))
    return np.unique(np.concatenate(picks)).astype(np.int64)


def test_prefill_q_proj_full_size():
    # every row of the batch: the oracle takes a few seconds on it
    w = wl.config_prefill()
    inp = wl.make_linear_inputs(w, "cuda")
    rows = None
    ref = gc.oracle_rows(inp, rows)
    for dt in (torch.bfloat16, torch.float32):
        print(f"[gpu] c1 full size y={dt}", flush=True)
        y = gc.run_linear(inp, dt)
        print(gc.compare_linear(y, ref, rows, what=f"c1/{dt}"), flush=True)
        assert torch.isfinite(y.float()).all()


def test_prefill_q_proj_quantised_base_full_size():
    # the same batch on the MXFP8 base ("Future Works", quantising the base model), in the launch
    # shape `bench.py --also mx` times: the activations' codes and scale bytes bit for bit on sampled
    # rows, the layer on the same rows, and the weight's codes / scales in full
    import oracle
    w = wl.config_prefill()
    inp = wl.make_linear_inputs(w, "cuda")
    ctx = gc.ctx()
    Wq, Ws = moin.moin_mx_quantize(ctx, inp.W, blocked=True)
    ctx.check()
    Ws_rows = Ws.permute(1, 0, 2).reshape(w.d_out, w.d_in // 32).cpu().numpy()
    rc, rs = oracle.mx_quantize(wl.bf16_bits(inp.W))
    assert np.array_equal(Wq.cpu().numpy(), rc) and np.array_equal(Ws_rows, rs)
    rows = _sample_rows(w.T, inp.seq_offsets, 200, seed=3)
    xq, xs = moin.moin_mx_quantize(ctx, inp.x)
    xc, xsc = oracle.mx_quantize(wl.bf16_bits(inp.x[torch.from_numpy(rows).cuda()]))
    assert np.array_equal(xq.cpu().numpy()[rows], xc) and np.array_equal(xs.cpu().numpy()[rows], xsc)
    A, B, ids = wl.compact_stacks(inp)
    ref = oracle.lora_linear_mx(wl.bf16_bits(inp.x), inp.seq_offsets.cpu().numpy(), ids, rc, rs, A, B,
                                w.scale, rows=rows)
    for dt in (torch.bfloat16, torch.float32):
        print(f"[gpu] c1 quantised base full size y={dt}", flush=True)
        y = moin.moin_lora_linear_mx(ctx, inp.x, inp.seq_offsets, inp.expert_ids, Wq, Ws, inp.A_stack,
                                     inp.B_stack, w.scale, y_dtype=dt)
        ctx.check()
        print(gc.compare_linear(y, ref, rows, what=f"c1 mx/{dt}"), flush=True)
        assert torch.isfinite(y.float()).all()


def test_decode_mlp_full_size():
    for w in wl.config_decode():
        inp = wl.make_linear_inputs(w, "cuda")
        ref = gc.oracle_rows(inp)
        for dt in (torch.bfloat16, torch.float32):
            print(f"[gpu] {w.name} y={dt}", flush=True)
            y = gc.run_linear(inp, dt)
            print(gc.compare_linear(y, ref, what=f"{w.name}/{dt}"), flush=True)
        del inp
        torch.cuda.empty_cache()


def test_router_full_size():
    rw = wl.config_router()
    rin = wl.make_route_inputs(rw, "cuda")
    print("[gpu] c3 router full size", flush=True)
    eids, cids, counts = moin.moin_route(gc.ctx(), rin.emb, rin.centroids, want_counts=True)
    gc.ctx().check()
    # properties at full size: histogram is the exact tally of the ids returned
    assert counts.sum().item() == rw.N
    assert torch.equal(counts.long(), torch.bincount(cids.long(), minlength=rw.K))
    # sampled queries against the oracle: every 16th (a stride that walks through every lane and
    # wave position of the kernel's 256-query tiles) plus one whole tile at each end
    sample = np.unique(np.concatenate([np.arange(0, rw.N, 16), np.arange(256), np.arange(rw.N - 256, rw.N)]))
    n_band = gc.check_route(rin.emb, rin.centroids, cids, sample=sample)
    print(f"[gpu] c3: {sample.size} sampled queries, {n_band} differ inside the near-tie band", flush=True)


def test_layer_chain_full_size():
    """Seven projections of one layer chained through their bf16 outputs; each
    projection is checked against the oracle run on the GPU's actual input."""
    wls = wl.config_layer()
    T = wls[0].T
    ids = wl.draw_expert_ids(wls[0].S, wls[0].E, "zipf", 1.5, wls[0].seed * 8 + 4)
    c = gc.ctx()
    off = torch.from_numpy(wl.seq_offsets_of(wls[0].seq_lens)).cuda()
    eids = torch.from_numpy(ids).cuda()
    plan = moin.Plan(c).build(off, eids, T, wls[0].E)
    h0 = wl._randn_bf16((T, 2048), 1.0, torch.device("cuda"), 4242)
    outs = {}
    src = {"q": "h0", "k": "h0", "v": "h0", "o": "q", "gate": "o", "up": "o", "down": "gate"}
    outs["h0"] = h0
    rows = _rows_per_sequence(off, seed=2)      # 64 rows of each of the 32 sequences
    assert rows.size == 64 * wls[0].S
    for w in wls:
        name = w.name.split("_", 1)[1]
        x = outs[src[name]]
        inp = wl.make_linear_inputs(w, "cuda", expert_ids=ids, x=x)
        print(f"[gpu] c4 {name} {w.d_in}->{w.d_out}", flush=True)
        y = moin.moin_lora_linear_planned(c, plan, inp.x, inp.W, inp.A_stack, inp.B_stack, w.scale)
        c.check()
        ref = gc.oracle_rows(inp, rows)
        print(name, gc.compare_linear(y, ref, rows, what=f"c4/{name}"), flush=True)
        if name in ("q", "o", "gate"):
            outs[name] = y
        del inp
        torch.cuda.empty_cache()
    plan.close()


def test_layer_chain_on_a_quantised_base_full_size():
    """The same chain with every projection's weight in MXFP8, as `bench.py --also mx` runs it: the first
    projection that reads an input quantises it into the caller's buffers (inside its shrink's pass), the
    others read those codes; each projection against the oracle on the GPU's actual input, and the shared-input
    call for q, k, v on the bf16 base against its single calls."""
    import oracle
    wls = wl.config_layer()
    T = wls[0].T
    ids = wl.draw_expert_ids(wls[0].S, wls[0].E, "zipf", 1.5, wls[0].seed * 8 + 4)
    c = gc.ctx()
    off = torch.from_numpy(wl.seq_offsets_of(wls[0].seq_lens)).cuda()
    eids = torch.from_numpy(ids).cuda()
    plan = moin.Plan(c).build(off, eids, T, wls[0].E)
    h0 = wl._randn_bf16((T, 2048), 1.0, torch.device("cuda"), 4242)
    outs = {"h0": h0}
    src = {"q": "h0", "k": "h0", "v": "h0", "o": "q", "gate": "o", "up": "o", "down": "gate"}
    codes = {}
    rows = _sample_rows(T, off, 24, seed=9)
    qkv = {}
    for w in wls:
        name = w.name.split("_", 1)[1]
        x = outs[src[name]]
        inp = wl.make_linear_inputs(w, "cuda", expert_ids=ids, x=x)
        Wq, Ws = moin.moin_mx_quantize(c, inp.W, blocked=True)
        first = src[name] not in codes
        if first:
            codes[src[name]] = (torch.empty((T, w.d_in), dtype=torch.uint8, device="cuda"),
                                torch.empty((w.d_in // 128, T, 4), dtype=torch.uint8, device="cuda"))
        xq, xs = codes[src[name]]
        print(f"[gpu] c4 mx {name} {w.d_in}->{w.d_out} emit={first}", flush=True)
        y = moin.moin_lora_linear_mx_planned(c, plan, x, Wq, Ws, inp.A_stack, inp.B_stack, w.scale, xq=xq, xs=xs,
                                             emit=first)
        c.check()
        A, B, cid = wl.compact_stacks(inp)
        Ws_rows = Ws.permute(1, 0, 2).reshape(w.d_out, w.d_in // 32).cpu().numpy()
        ref = oracle.lora_linear_mx(wl.bf16_bits(x), off.cpu().numpy(), cid, Wq.cpu().numpy(), Ws_rows, A, B, w.scale,
                                    rows=rows)
        print(name, gc.compare_linear(y, ref, rows, what=f"c4 mx/{name}"), flush=True)
        if first:
            # the codes the shrink's pass wrote are the quantiser's, bit for bit, on the sampled rows
            oc, osc = oracle.mx_quantize(wl.bf16_bits(x[torch.from_numpy(rows).cuda()]))
            xs_rows = xs.permute(1, 0, 2).reshape(T, w.d_in // 32)
            assert np.array_equal(xq.cpu().numpy()[rows], oc) and np.array_equal(xs_rows.cpu().numpy()[rows], osc)
        if name in ("q", "o", "gate"):
            outs[name] = y
        if name in ("q", "k", "v"):
            qkv[name] = inp
        else:
            del inp
        torch.cuda.empty_cache()
    print("[gpu] c4 q, k, v through the shared-input call", flush=True)
    ins = [qkv[n] for n in ("q", "k", "v")]
    single = [moin.moin_lora_linear_planned(c, plan, h0, i.W, i.A_stack, i.B_stack, i.wl.scale) for i in ins]
    shared = moin.moin_lora_linear_planned_shared(c, plan, h0, [i.W for i in ins], [i.A_stack for i in ins],
                                                  [i.B_stack for i in ins], ins[0].wl.scale)
    c.check()
    for a, b in zip(single, shared):
        assert torch.equal(a, b)
    plan.close()


def test_kmeans_update_full_size():
    """One centre update at the router workload's size (1 048 576 x 768 bf16,
    5000 centres), ids from the GPU router: every centre against the oracle,
    which reads the same bytes (about 1 s of host time per Gflop of sums)."""
    import oracle
    rw = wl.config_router()
    rin = wl.make_route_inputs(rw, "cuda")
    print("[gpu] c3 kmeans update full size: route", flush=True)
    _, cids, rcounts = moin.moin_route(gc.ctx(), rin.emb, rin.centroids, want_counts=True)
    print("[gpu] c3 kmeans update full size: update", flush=True)
    new, counts, inertia = moin.moin_kmeans_update(gc.ctx(), rin.emb, cids, rin.centroids, out_dtype=torch.float32)
    gc.ctx().check()
    assert torch.equal(counts, rcounts)
    emb_h, ids_h = wl.bf16_bits(rin.emb), cids.cpu().numpy()
    print("[gpu] c3 kmeans update full size: oracle", flush=True)
    ref_new, ref_counts, ref_inertia = oracle.kmeans_update(emb_h, ids_h, wl.bf16_bits(rin.centroids))
    assert np.array_equal(counts.cpu().numpy(), ref_counts)
    assert abs(inertia.item() - ref_inertia) <= 2e-6 * ref_inertia
    got = new.double().cpu().numpy()
    # bound of tests/test_gpu_kmeans.py with mean|x| replaced by its upper bound
    # max|x| over the table (unit vectors in 768 dimensions: entries are small)
    xmax = float(rin.emb.abs().max().item())
    tol = 520 * 2.0 ** -24 * xmax + 2 * 2.0 ** -24 * np.abs(ref_new)
    err = np.abs(got - ref_new)
    assert not (err > tol).any(), f"{int((err > tol).sum())} entries beyond the bound, worst {err.max():.3e}"
    print(f"[gpu] c3 kmeans: worst centre error {err.max():.3e} (bound {tol.min():.3e}), "
          f"{int((ref_counts == 0).sum())} empty clusters", flush=True)


def test_prefill_addresses_beyond_4_gib():
    # maximum sizes: x holds 4.8 GB, so the byte offsets of the rows from 1 048 576 on do not fit 32 bits;
    # rows on both sides of that line, the first and the last ones against the oracle
    lens = [4096] * 285 + [2929, 1, 0, 300]
    w = wl.LinearWorkload("beyond_4gib", 2048, 264, 64, 6, lens, "uniform", scale=2.0, seed=4242)
    T = w.T
    assert T * 2048 * 2 > (1 << 32) + (1 << 28)
    inp = wl.make_linear_inputs(w, "cuda")
    line = (1 << 32) // (2048 * 2)
    rows = np.unique(np.concatenate([np.arange(0, 4), np.arange(line - 4, line + 4), np.arange(T - 304, T - 296),
                                     np.arange(T - 4, T), _sample_rows(T, inp.seq_offsets, 24, seed=5)]))
    x_rows = wl.bf16_bits(inp.x[torch.from_numpy(rows).cuda()])
    # the oracle on a batch made of just those rows, one sequence each, with the expert of the row's sequence
    off = inp.seq_offsets.cpu().numpy()
    seq_of = np.searchsorted(off, rows, side="right") - 1
    A, B, ids = wl.compact_stacks(inp)
    import oracle
    ref = oracle.lora_linear(x_rows, np.arange(len(rows) + 1, dtype=np.int32), ids[seq_of], wl.bf16_bits(inp.W), A, B,
                             w.scale)
    for dt in (torch.bfloat16, torch.float32):
        print(f"[gpu] rows beyond 4 GiB y={dt}", flush=True)
        y = gc.run_linear(inp, dt)
        print(gc.compare_linear(y[torch.from_numpy(rows).cuda()], ref, what=f"beyond_4gib/{dt}"), flush=True)
        del y
    del inp
    torch.cuda.empty_cache()


def test_router_addresses_beyond_4_gib():
    # 3.2 M queries of 768 bf16 values: 4.9 GB, query rows from 2 796 203 on start beyond 32-bit byte offsets
    rw = wl.RouteWorkload("route_beyond_4gib", N=3_200_000, K=500, D=768, dtype="bf16", normalise=True, seed=777)
    rin = wl.make_route_inputs(rw, "cuda")
    assert rin.emb.numel() * 2 > (1 << 32) + (1 << 28)
    print("[gpu] router beyond 4 GiB", flush=True)
    eids, cids, counts = moin.moin_route(gc.ctx(), rin.emb, rin.centroids, want_counts=True)
    gc.ctx().check()
    assert counts.sum().item() == rw.N
    assert torch.equal(counts.long(), torch.bincount(cids.long(), minlength=rw.K))
    line = (1 << 32) // (768 * 2)
    sample = np.unique(np.concatenate([np.arange(0, 64), np.arange(line - 64, line + 64),
                                       np.arange(rw.N - 300, rw.N), np.arange(0, rw.N, 4099)]))
    n_band = gc.check_route(rin.emb, rin.centroids, cids, sample=sample)
    print(f"[gpu] {sample.size} sampled queries, {n_band} differ inside the near-tie band", flush=True)
    # the centre update over the same table (its rows are gathered by index: 64-bit row addresses)
    import oracle
    print("[gpu] kmeans update beyond 4 GiB", flush=True)
    new, kcounts, inertia = moin.moin_kmeans_update(gc.ctx(), rin.emb, cids, rin.centroids, out_dtype=torch.float32)
    gc.ctx().check()
    assert torch.equal(kcounts, counts)
    ref_new, ref_counts, ref_inertia = oracle.kmeans_update(wl.bf16_bits(rin.emb), cids.cpu().numpy(),
                                                            wl.bf16_bits(rin.centroids))
    assert np.array_equal(kcounts.cpu().numpy(), ref_counts)
    assert abs(inertia.item() - ref_inertia) <= 2e-6 * ref_inertia
    xmax = float(rin.emb.abs().max().item())
    tol = 520 * 2.0 ** -24 * xmax + 2 * 2.0 ** -24 * np.abs(ref_new)
    err = np.abs(new.double().cpu().numpy() - ref_new)
    assert not (err > tol).any(), f"{int((err > tol).sum())} entries beyond the bound, worst {err.max():.3e}"
    del rin
    torch.cuda.empty_cache()


def test_per_token_adapters_full_size():
    # the workload `bench.py --also pertoken` times: 8192 single-token sequences through the 2048 -> 5632
    # projection, r = 128, 5000 experts, Zipf(1.1); sampled tokens against the oracle
    w0 = wl.config_decode()[0]
    T = 8192
    w = wl.LinearWorkload("per_token_gate", w0.d_in, w0.d_out, w0.r, w0.E, [1] * T, "zipf", 1.1, w0.scale,
                          seed=w0.seed + 77)
    inp = wl.make_linear_inputs(w, "cuda")
    rows = _sample_rows(T, inp.seq_offsets, 150, seed=7)
    # the oracle on a batch of just those tokens (one sequence each) with the experts they use
    sel = torch.from_numpy(rows).cuda()
    sub = wl.LinearInputs(wl.LinearWorkload("sub", w.d_in, w.d_out, w.r, w.E, [1] * len(rows), "zipf", 1.1, w.scale),
                          inp.x[sel].contiguous(), inp.W, inp.A_stack, inp.B_stack,
                          torch.arange(len(rows) + 1, dtype=torch.int32, device="cuda"),
                          inp.expert_ids[sel].contiguous())
    ref = gc.oracle_rows(sub)
    for dt in (torch.bfloat16, torch.float32):
        print(f"[gpu] per-token full size y={dt}", flush=True)
        y = gc.run_linear(inp, dt)
        print(gc.compare_linear(y[sel], ref, what=f"per-token/{dt}"), flush=True)
        assert torch.isfinite(y.float()).all()
    del inp, sub
    torch.cuda.empty_cache()


def test_nearest_topics_at_request_size():
    # what bench.py reports beside the router: the four nearest of 5000 topics for 4096 queries (D = 768, bf16);
    # every 16th query against the oracle, place by place
    import oracle
    rw = wl.RouteWorkload("topk_request", N=4096, K=5000, D=768, dtype="bf16", normalise=True, seed=4321)
    rin = wl.make_route_inputs(rw, "cuda")
    print("[gpu] top-4 of 5000 topics, 4096 queries", flush=True)
    _, cids, d2 = moin.moin_route_topk(gc.ctx(), rin.emb, rin.centroids, 4)
    gc.ctx().check()
    sample = np.arange(0, rw.N, 16)
    emb_h, cent_h = wl.bf16_bits(rin.emb[torch.from_numpy(sample).cuda()]), wl.bf16_bits(rin.centroids)
    ref_ids, ref_d2 = oracle.route_topk(emb_h, cent_h, 4)
    got = cids.cpu().numpy()[sample]
    n_band = 0
    for i, m in zip(*np.nonzero(got != ref_ids)):
        true_d = oracle.dist2(emb_h, cent_h, np.array([i]), np.array([got[i, m]]))[0]
        assert true_d <= ref_d2[i, m] * (1 + 1e-4), (i, m, got[i], ref_ids[i])
        n_band += 1
    assert np.allclose(d2.double().cpu().numpy()[sample], oracle.dist2(
        emb_h, cent_h, np.repeat(np.arange(len(sample)), 4), got.ravel()).reshape(-1, 4), rtol=2e-5)
    print(f"[gpu] {len(sample)} sampled queries, {n_band} places inside the near-tie band", flush=True)
