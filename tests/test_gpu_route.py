"""GPU parity of moin_route / moin_histogram (through the C ABI) against the
CPU oracle: ids exact outside the 1e-4 near-tie band, histograms exact."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_09687_amd import moin
from paper_2410_09687_amd import workloads as wl
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu


def _route_case(N, K, D, dtype, normalise, seed):
    return wl.make_route_inputs(wl.RouteWorkload("t", N, K, D, dtype, normalise, seed), "cuda")


@pytest.mark.parametrize("N,K,D", [(700, 300, 96), (256, 256, 64), (1, 1, 8), (513, 1000, 200)])
def test_bf16_router_small(N, K, D):
    rin = _route_case(N, K, D, "bf16", True, seed=N + K)
    print(f"[gpu] route bf16 N={N} K={K} D={D}", flush=True)
    eids, cids, counts = moin.moin_route(gc.ctx(), rin.emb, rin.centroids, want_counts=True)
    gc.ctx().check()
    gc.check_route(rin.emb, rin.centroids, cids)
    assert torch.equal(eids, cids)
    assert torch.equal(counts.long(), torch.bincount(cids.long(), minlength=K))


@pytest.mark.parametrize("N,K,D", [(5000, 700, 128), (4100, 300, 64), (4097, 256, 192), (4500, 100, 64)])
def test_bf16_router_streaming_kernel_edges(N, K, D):
    # more than 4096 queries and D a multiple of 64: the large-batch kernel, with a
    # ragged last centroid tile, a ragged last query tile, one or two k blocks per tile
    rin = _route_case(N, K, D, "bf16", True, seed=N + K + D)
    print(f"[gpu] route bf16 stream N={N} K={K} D={D}", flush=True)
    eids, cids, counts = moin.moin_route(gc.ctx(), rin.emb, rin.centroids, want_counts=True)
    gc.ctx().check()
    gc.check_route(rin.emb, rin.centroids, cids)
    assert torch.equal(counts.long(), torch.bincount(cids.long(), minlength=K))


@pytest.mark.parametrize("N,K,D", [(40000, 520, 64), (70000, 200, 64), (66000, 1100, 128)])
def test_bf16_router_streaming_kernel_several_items_per_workgroup(N, K, D):
    # more query tiles than the persistent launch has workgroups: a workgroup streams through several
    # (query tile, group member) items, the last of them ragged; groups of 3, 1 and 5 workgroups per tile
    rin = _route_case(N, K, D, "bf16", True, seed=N + K + D)
    print(f"[gpu] route bf16 stream, several items N={N} K={K} D={D}", flush=True)
    eids, cids, counts = moin.moin_route(gc.ctx(), rin.emb, rin.centroids, want_counts=True)
    gc.ctx().check()
    gc.check_route(rin.emb, rin.centroids, cids)
    assert torch.equal(counts.long(), torch.bincount(cids.long(), minlength=K))


@pytest.mark.parametrize("N,K,D", [(30000, 600, 64), (50000, 257, 64), (45000, 1281, 192), (100000, 64, 64),
                                   (4097, 5000, 64), (33333, 2049, 128)])
def test_bf16_router_streaming_kernel_shape_sweep(N, K, D):
    # one block per centroid tile (D = 64) with several items per workgroup, a last centroid tile of one row,
    # fewer centroids than a tile holds, group sizes 1 to 5, ragged last query tiles
    rin = _route_case(N, K, D, "bf16", True, seed=3 * N + K + D)
    print(f"[gpu] route bf16 stream sweep N={N} K={K} D={D}", flush=True)
    eids, cids, counts = moin.moin_route(gc.ctx(), rin.emb, rin.centroids, want_counts=True)
    gc.ctx().check()
    gc.check_route(rin.emb, rin.centroids, cids)
    assert torch.equal(counts.long(), torch.bincount(cids.long(), minlength=K))


def test_f32_router_small():
    rin = _route_case(300, 77, 100, "f32", False, seed=3)
    eids, cids, counts = moin.moin_route(gc.ctx(), rin.emb, rin.centroids, want_counts=True)
    gc.ctx().check()
    gc.check_route(rin.emb, rin.centroids, cids)
    assert counts.sum().item() == 300


def test_queries_equal_centroids_and_duplicates():
    rin = _route_case(8, 600, 128, "bf16", True, seed=9)
    cent = rin.centroids.clone()
    cent[400] = cent[17]                       # duplicate: lowest index must win
    eids, cids, counts = moin.moin_route(gc.ctx(), cent, cent, want_counts=True)
    gc.ctx().check()
    expect = torch.arange(600, device="cuda", dtype=torch.int32)
    expect[400] = 17
    assert torch.equal(cids, expect)
    assert counts[17].item() == 2 and counts[400].item() == 0 and counts.sum().item() == 600


# (the last case has more query tiles than workgroups in the launch: several items per workgroup, the last one ragged)
@pytest.mark.parametrize("K,D,N", [(1280, 768, 8192), (1030, 64, 12000), (5000, 768, 10000), (1030, 64, 90001)])
def test_lowest_index_wins_ties_in_the_large_batch_kernel(K, D, N):
    # More than 4096 queries: the streaming kernel, whose workgroups share a query tile and merge
    # their winners with a packed atomic minimum.  Every query IS a centroid and a third of the
    # centroids are copies of an earlier one (some in the same 256-centroid tile, some in another
    # tile, i.e. held by another workgroup of the group), so each query has two or three exact
    # minima at distance 0 and only the lowest index is right.  Ids are compared exactly.
    rin = _route_case(8, K, D, "bf16", True, seed=K + D)
    cent = rin.centroids.clone()
    rng = np.random.default_rng(K)
    src = np.arange(K)
    third = K // 3
    src[K - third:] = rng.integers(0, K - third, size=third)      # copies of earlier centroids, far away
    near = rng.choice(K - third - 8, size=third // 4, replace=False)
    src[near + 5] = src[near]                                     # copies five places further on
    cent = cent[torch.from_numpy(src).cuda()].contiguous()
    qsel = rng.integers(0, K, size=N)
    qsel[:K] = np.arange(K)
    emb = cent[torch.from_numpy(qsel).cuda()].contiguous()
    print(f"[gpu] route ties stream N={N} K={K} D={D}", flush=True)
    eids, cids, counts = moin.moin_route(gc.ctx(), emb, cent, want_counts=True)
    gc.ctx().check()
    ref = oracle.route(wl.bf16_bits(emb), wl.bf16_bits(cent))
    # the oracle's answer is the first holder of the query's vector
    first = np.full(K, -1)
    seen = {}
    cb = wl.bf16_bits(cent)
    for k in range(K):
        first[k] = seen.setdefault(cb[k].tobytes(), k)
    assert np.array_equal(ref, first[qsel])
    assert (first != np.arange(K)).sum() >= third
    assert torch.equal(cids.cpu(), torch.from_numpy(ref.astype(np.int32)))
    assert torch.equal(counts.long(), torch.bincount(cids.long(), minlength=K))


def test_slot_map_and_retained_only_search():
    rin = _route_case(900, 260, 64, "bf16", True, seed=21)
    table = wl.retained_slot_table(260, 231, seed=4)
    slots = torch.from_numpy(table).cuda()
    eids, cids, _ = moin.moin_route(gc.ctx(), rin.emb, rin.centroids, slot_of_centroid=slots)
    gc.ctx().check()
    gc.check_route(rin.emb, rin.centroids, cids)
    assert np.array_equal(eids.cpu().numpy(), oracle.slot_map(cids.cpu().numpy(), table))
    assert (eids == -1).any()
    eids2, cids2, counts2 = moin.moin_route(gc.ctx(), rin.emb, rin.centroids, slot_of_centroid=slots,
                                            retained_only=True, want_counts=True)
    gc.ctx().check()
    gc.check_route(rin.emb, rin.centroids, cids2, eligible=table >= 0)
    assert (eids2 >= 0).all()
    assert counts2[torch.from_numpy(table < 0).cuda()].sum().item() == 0


def test_histogram_alone_and_bad_ids():
    ids = torch.randint(0, 5000, (200_000,), device="cuda", dtype=torch.int32)
    counts = moin.moin_histogram(gc.ctx(), ids, 5000)
    gc.ctx().check()
    assert np.array_equal(counts.cpu().numpy(), oracle.histogram(ids.cpu().numpy(), 5000))
    big = moin.moin_histogram(gc.ctx(), ids, 40_000)      # more bins than the LDS tally holds
    assert torch.equal(big[:5000], counts) and big[5000:].sum().item() == 0
    ids[5] = 7000
    moin.moin_histogram(gc.ctx(), ids, 5000)
    with pytest.raises(moin.MoinError):
        gc.ctx().check()
    assert moin.moin_histogram(gc.ctx(), ids[:0], 16).sum().item() == 0
    gc.ctx().check()


def test_route_argument_errors():
    rin = _route_case(16, 16, 64, "bf16", True, seed=2)
    with pytest.raises(moin.MoinError):
        moin.moin_route(gc.ctx(), rin.emb[:, :12].contiguous(), rin.centroids[:, :12].contiguous())
    with pytest.raises(moin.MoinError):
        moin.moin_route(gc.ctx(), rin.emb, rin.centroids, retained_only=True)
    e, c, _ = moin.moin_route(gc.ctx(), rin.emb[:0], rin.centroids)
    assert e.numel() == 0


def test_request_sized_batches_reuse_the_norms_and_keep_their_scratch_clean():
    # Request-sized batches take one self-cleaning launch.  A serving loop: the same table over and over
    # (norms reused when the caller says so), batches of different sizes, a linear call in between (it
    # overwrites the shared workspace), then ANOTHER table at the same address claimed unchanged only
    # after one honest call -- every result against the oracle and against a fresh context.
    ctx = gc.ctx()
    K, D = 700, 128
    rin = _route_case(900, K, D, "bf16", True, seed=77)
    cent = rin.centroids.clone()
    slots = torch.from_numpy(wl.retained_slot_table(K, K - 50, seed=6)).cuda()
    fresh = moin.Context(0)
    try:
        for i, n in enumerate([900, 64, 1, 333, 900]):
            q = rin.emb[:n].contiguous()
            e, c, cnt = moin.moin_route(ctx, q, cent, slot_of_centroid=slots, want_counts=True,
                                        same_centroids=(i > 0))
            ctx.check()
            e2, c2, cnt2 = moin.moin_route(fresh, q, cent, slot_of_centroid=slots, want_counts=True)
            fresh.check()
            assert torch.equal(c, c2) and torch.equal(e, e2) and torch.equal(cnt, cnt2)
            gc.check_route(q, cent, c)
            assert torch.equal(cnt.long(), torch.bincount(c.long(), minlength=K))
            if i == 1:   # a linear call between two routing calls
                lin = wl.make_linear_inputs(wl.LinearWorkload("t", 128, 136, 16, 4, [3, 5, 2], "uniform", seed=5), "cuda")
                gc.run_linear(lin)
        # new contents at the same address: one call without the flag picks them up ...
        cent.copy_(_route_case(8, K, D, "bf16", True, seed=78).centroids)
        q = rin.emb[:500].contiguous()
        _, c, _ = moin.moin_route(ctx, q, cent)
        ctx.check()
        gc.check_route(q, cent, c)
        # ... and from then on the flag is honest again; retained-only changes what the norms mean
        _, c, _ = moin.moin_route(ctx, q, cent, same_centroids=True)
        ctx.check()
        gc.check_route(q, cent, c)
        _, c, _ = moin.moin_route(ctx, q, cent, slot_of_centroid=slots, retained_only=True, same_centroids=True)
        ctx.check()
        gc.check_route(q, cent, c, eligible=(slots >= 0).cpu().numpy())
    finally:
        fresh.close()
