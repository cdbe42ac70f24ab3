"""GPU parity of the K-means centre update, the cluster pruning and the Lloyd
loop (through the C ABI) against the CPU oracle.

Tolerances (derived from the kernel's arithmetic, u = 2^-24):
  * a column sum adds at most 512 values in fp32 one after the other, then at
    most 256 partial sums, everything later is fp64, the mean is rounded to fp32
    once: |error| <= (512 + 8) u mean|x| + 2 u |mean|;
  * a bf16 centre adds half a bf16 ulp: 2^-8 |mean|;
  * the objective sums 8 (bf16) or 4 (fp32) squared differences of a row in
    fp32 and everything else in fp64: relative error of a few u, bar 2e-6.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_09687_amd import moin
from paper_2410_09687_amd import workloads as wl
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu

U = 2.0 ** -24


def _host(t):
    return wl.bf16_bits(t) if t.dtype == torch.bfloat16 else t.cpu().numpy()


def _f64(t):
    return t.detach().float().cpu().double().numpy()


def _check_update(emb, ids, cent, what, out_dtypes=(torch.float32, torch.bfloat16)):
    ids_h = ids.cpu().numpy()
    ref_new, ref_counts, ref_inertia = oracle.kmeans_update(_host(emb), ids_h, _host(cent))
    K, D = cent.shape
    x = _f64(emb)
    sum_abs = np.zeros((K, D))
    np.add.at(sum_abs, ids_h, np.abs(x))
    mean_abs = sum_abs / np.maximum(ref_counts, 1)[:, None]
    res = {}
    for odt in out_dtypes:
        print(f"[gpu] kmeans_update {what} out={odt}", flush=True)
        new, counts, inertia = moin.moin_kmeans_update(gc.ctx(), emb, ids, cent, out_dtype=odt)
        gc.ctx().check()
        assert np.array_equal(counts.cpu().numpy(), ref_counts), what
        got = _f64(new)
        tol = 520 * U * mean_abs + 2 * U * np.abs(ref_new)
        if odt == torch.bfloat16:
            tol = tol + 2.0 ** -8 * np.abs(ref_new)
        empty = ref_counts == 0
        # (kept as it was, in the output type: an fp32 centre written as bf16 is rounded once)
        assert np.array_equal(got[empty], _f64(cent.to(odt))[empty]), f"{what}: an empty cluster moved"
        over = np.abs(got - ref_new) > tol
        assert not over.any(), f"{what}/{odt}: {int(over.sum())} centre entries beyond the bound, worst {np.abs(got - ref_new).max():.3e}"
        gi = float(inertia.item())
        assert abs(gi - ref_inertia) <= 2e-6 * max(ref_inertia, 1e-300), (what, gi, ref_inertia)
        res[odt] = new
    return res


def _inputs(N, K, D, dtype, seed, ids=None):
    g = torch.Generator(device="cuda").manual_seed(seed)
    emb = torch.randn((N, D), generator=g, device="cuda", dtype=torch.float32).to(dtype)
    cent = torch.randn((K, D), generator=g, device="cuda", dtype=torch.float32).to(dtype)
    if ids is None:
        ids = torch.randint(0, K, (N,), generator=g, device="cuda", dtype=torch.int32)
    else:
        ids = torch.as_tensor(np.asarray(ids, np.int32), device="cuda")
    return emb, ids, cent


def test_small_fp32_and_bf16_with_empty_clusters():
    emb, ids, cent = _inputs(1000, 7, 12, torch.float32, 1)
    _check_update(emb, ids, cent, "fp32 small", out_dtypes=(torch.float32,))
    rng = np.random.default_rng(2)
    ids_h = rng.choice([0, 2, 3, 7, 11, 36], size=5003)   # 31 of 37 clusters stay empty
    emb, ids, cent = _inputs(5003, 37, 24, torch.bfloat16, 3, ids_h)
    _check_update(emb, ids, cent, "bf16 ragged")


def test_heavy_cluster_spans_many_pieces_and_chunks():
    # 60 % of 20 000 points in one cluster (24 pieces), five chunks of points
    rng = np.random.default_rng(4)
    ids_h = np.where(rng.random(20000) < 0.6, 3, rng.integers(0, 50, size=20000))
    emb, ids, cent = _inputs(20000, 50, 768, torch.bfloat16, 5, ids_h)
    a = _check_update(emb, ids, cent, "heavy")
    # fixed summation order: a second run repeats bit for bit
    b, _, _ = moin.moin_kmeans_update(gc.ctx(), emb, ids, cent, out_dtype=torch.float32)
    assert torch.equal(a[torch.float32], b)


def test_wide_rows_use_column_blocks():
    emb, ids, cent = _inputs(600, 5, 4096, torch.float32, 6)          # 1024 chunks per row: 4 column blocks
    _check_update(emb, ids, cent, "fp32 wide", out_dtypes=(torch.float32,))
    emb, ids, cent = _inputs(700, 9, 2056, torch.bfloat16, 7)         # 257 chunks: a second block of one chunk
    _check_update(emb, ids, cent, "bf16 257 chunks")


def test_no_points_and_in_place_update():
    emb, ids, cent = _inputs(0, 6, 16, torch.bfloat16, 8)
    new, counts, inertia = moin.moin_kmeans_update(gc.ctx(), emb, ids, cent)
    gc.ctx().check()
    assert torch.equal(new, cent) and counts.sum().item() == 0 and inertia.item() == 0.0
    emb, ids, cent = _inputs(3000, 11, 64, torch.bfloat16, 9)
    want, _, _ = moin.moin_kmeans_update(gc.ctx(), emb, ids, cent)
    buf = cent.clone()
    got, _, _ = moin.moin_kmeans_update(gc.ctx(), emb, ids, buf, out=buf)
    gc.ctx().check()
    assert got.data_ptr() == buf.data_ptr() and torch.equal(buf, want)
    # objective and counts alone
    none, counts, inertia = moin.moin_kmeans_update(gc.ctx(), emb, ids, cent, want_centroids=False)
    assert none is None
    ref = oracle.kmeans_update(_host(emb), ids.cpu().numpy(), _host(cent))
    assert np.array_equal(counts.cpu().numpy(), ref[1])
    assert abs(inertia.item() - ref[2]) <= 2e-6 * ref[2]


def test_bad_ids_are_skipped_and_reported():
    emb, ids, cent = _inputs(900, 5, 16, torch.float32, 10)
    ids_h = ids.cpu().numpy().copy()
    ids_h[[3, 500, 899]] = [-1, 5, 1 << 20]
    new, counts, inertia = moin.moin_kmeans_update(gc.ctx(), emb, torch.as_tensor(ids_h, device="cuda"), cent)
    with pytest.raises(moin.MoinError) as e:
        gc.ctx().check()
    assert e.value.code == -4
    keep = np.ones(900, bool)
    keep[[3, 500, 899]] = False
    ref = oracle.kmeans_update(_host(emb)[keep], ids_h[keep], _host(cent))
    assert np.array_equal(counts.cpu().numpy(), ref[1])
    assert np.allclose(_f64(new), ref[0], rtol=1e-5, atol=1e-6)
    assert abs(inertia.item() - ref[2]) <= 2e-6 * ref[2]
    gc.ctx().check()   # the word was cleared


def test_argument_errors():
    emb, ids, cent = _inputs(10, 3, 16, torch.bfloat16, 11)
    with pytest.raises(moin.MoinError):   # D not a multiple of 8 for bf16
        moin.moin_kmeans_update(gc.ctx(), emb[:, :12].contiguous(), ids, cent[:, :12].contiguous())
    big = torch.zeros((32769, 8), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(moin.MoinError):   # K beyond the LDS cursor table
        moin.moin_kmeans_update(gc.ctx(), emb[:, :8].contiguous(), ids, big)
    # in place with a different output type
    rc = moin.load().moin_kmeans_update(gc.ctx()._h, emb.data_ptr(), ids.data_ptr(), 10, cent.data_ptr(), 3, 16,
                                        moin.MOIN_BF16, cent.data_ptr(), moin.MOIN_F32, None, None, None)
    assert rc == -1


def test_retain_clusters_matches_the_oracle():
    rng = np.random.default_rng(12)
    for K, t in ((6, 3), (5000, 40), (1, 1), (1025, 0)):
        counts_h = rng.integers(0, 100, size=K)
        slot, n = moin.moin_retain_clusters(gc.ctx(), torch.as_tensor(counts_h.astype(np.int32), device="cuda"), t)
        gc.ctx().check()
        ref_slot, ref_n = oracle.retain_clusters(counts_h, t)
        assert np.array_equal(slot.cpu().numpy(), ref_slot) and n.item() == ref_n


def test_lloyd_loop_matches_the_oracle_on_separated_blobs():
    # fp32, well separated blobs: no near-ties, so the GPU loop and an oracle loop
    # make the same assignments and the centres agree to rounding
    rng = np.random.default_rng(13)
    K, D, N, iters = 8, 16, 3000, 3
    true_c = rng.standard_normal((K, D)) * 3
    lab = rng.integers(0, K, size=N)
    x = (true_c[lab] + 0.1 * rng.standard_normal((N, D))).astype(np.float32)
    c0 = (true_c + 0.3 * rng.standard_normal((K, D))).astype(np.float32)
    emb = torch.as_tensor(x, device="cuda")
    cent = torch.as_tensor(c0, device="cuda").clone()
    print("[gpu] kmeans_fit fp32 blobs", flush=True)
    ids, counts, inertia = moin.moin_kmeans_fit(gc.ctx(), emb, cent, iters)
    gc.ctx().check()
    c = c0.copy()
    ref_in = []
    for _ in range(iters):
        rid = oracle.route(x, c)
        new, _, inert = oracle.kmeans_update(x, rid, c)
        ref_in.append(inert)
        c = new.astype(np.float32)
    rid, best, _ = oracle.route(x, c, want_gaps=True)
    ref_in.append(best.sum())
    assert np.array_equal(ids.cpu().numpy(), rid)
    assert np.array_equal(counts.cpu().numpy(), np.bincount(rid, minlength=K))
    assert np.allclose(cent.cpu().numpy(), c, rtol=1e-5, atol=1e-6)
    gi = inertia.cpu().numpy()
    assert np.allclose(gi, ref_in, rtol=1e-5)
    assert (np.diff(gi) <= 1e-9 * gi[:-1]).all()


def test_lloyd_loop_bf16_descends_and_is_consistent():
    # bf16 through the streaming router (N > 4096): properties only -- the
    # objective never rises by more than the rounding of the centres to bf16
    # explains, ids are the nearest centres of the returned table, counts tally
    g = torch.Generator(device="cuda").manual_seed(14)
    N, K, D, iters = 8192, 20, 64, 4
    emb = torch.randn((N, D), generator=g, device="cuda").to(torch.bfloat16)
    cent = emb[torch.randperm(N, generator=g, device="cuda")[:K]].clone()
    print("[gpu] kmeans_fit bf16", flush=True)
    ids, counts, inertia = moin.moin_kmeans_fit(gc.ctx(), emb, cent, iters)
    gc.ctx().check()
    gi = inertia.cpu().numpy()
    assert (gi[1:] <= gi[:-1] * (1 + 2e-3)).all(), gi
    assert gi[-1] < gi[0]
    gc.check_route(emb, cent, ids)
    assert np.array_equal(counts.cpu().numpy(), np.bincount(ids.cpu().numpy(), minlength=K))
    ref = oracle.kmeans_update(_host(emb), ids.cpu().numpy(), _host(cent))
    assert abs(gi[-1] - ref[2]) <= 2e-6 * ref[2]


def test_launch_shape_limits():
    # K = 1 (no id bits to match), fewer points than one batch of 64
    emb, ids, cent = _inputs(37, 1, 8, torch.bfloat16, 20)
    _check_update(emb, ids, cent, "K=1", out_dtypes=(torch.float32,))
    # the largest K the cursor table in LDS holds (128 KB), most clusters empty
    emb, ids, cent = _inputs(3000, 32768, 8, torch.bfloat16, 21)
    _check_update(emb, ids, cent, "K=32768", out_dtypes=(torch.float32,))
    # more than 1024 chunks of 4096 points: the chunk grows instead (4 400 000 points -> chunks of 4352)
    emb, ids, cent = _inputs(4_400_000, 300, 8, torch.bfloat16, 22)
    _check_update(emb, ids, cent, "many chunks", out_dtypes=(torch.float32,))
