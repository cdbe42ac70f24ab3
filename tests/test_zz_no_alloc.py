"""moin_route_static -- the routing call for callers that cannot allocate device memory -- against
moin_route on the same inputs: ids, slot ids and counts must be the same bits.  Two calls in a row on
the library's fixed scratch array, the second one smaller, so that whatever the first left there must
not leak into the second; then the size limits."""
import numpy as np
import pytest
import torch

from paper_2410_09687_amd import moin
from paper_2410_09687_amd import workloads as wl
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu


def _case(N, K, D, dtype, seed):
    return wl.make_route_inputs(wl.RouteWorkload("t", N, K, D, dtype, dtype == "bf16", seed), "cuda")


def _both(rin, K, **kw):
    ctx = gc.ctx()
    N = rin.emb.shape[0]
    out = (torch.full((N,), -7, dtype=torch.int32, device="cuda"),
           torch.full((N,), -7, dtype=torch.int32, device="cuda") if kw.pop("cids", True) else None,
           torch.full((K,), -7, dtype=torch.int32, device="cuda"))
    got = moin.moin_route(ctx, rin.emb, rin.centroids, out=out, static=True, **kw)
    ctx.check()
    ref = moin.moin_route(ctx, rin.emb, rin.centroids, want_centroid_ids=out[1] is not None,
                          want_counts=True, **kw)
    ctx.check()
    for g, r in zip(got, ref):
        assert (g is None) == (r is None)
        if g is not None:
            assert torch.equal(g, r)
    return got


@pytest.mark.parametrize("dtype,D", [("bf16", 768), ("bf16", 72), ("f32", 100)])
def test_static_route_equals_route_twice_in_a_row(dtype, D):
    # first call: more than 4096 queries (the large-batch kernel with workgroups sharing a query tile,
    # per-query packed minima in the scratch array); second call: a small batch (centroid range split
    # across workgroups, arrival counter, in-kernel tally), and only counts + slot ids asked for
    K = 1300
    big = _case(6000 if dtype == "bf16" else 700, K, D, dtype, seed=31)
    small = _case(333, K, D, dtype, seed=32)
    table = torch.from_numpy(wl.retained_slot_table(K, K - 100, seed=5)).cuda()
    print(f"[gpu] static route {dtype} D={D}: large batch", flush=True)
    e1, c1, n1 = _both(big, K)
    assert n1.sum().item() == big.emb.shape[0]
    gc.check_route(big.emb, big.centroids, c1, sample=np.arange(0, big.emb.shape[0], 7))
    print(f"[gpu] static route {dtype} D={D}: small batch after it", flush=True)
    e2, c2, n2 = _both(small, K, slot_of_centroid=table, retained_only=True, cids=False)
    assert c2 is None and n2.sum().item() == 333 and (e2 >= 0).all()
    # and the large one again after the small one
    _both(big, K, slot_of_centroid=table)


def test_static_route_limits_and_empty_batch():
    ctx = gc.ctx()
    rin = _case(16, 64, 64, "bf16", seed=33)
    e, c, n = moin.moin_route(ctx, rin.emb[:0], rin.centroids, want_counts=True, static=True)
    ctx.check()
    assert e.numel() == 0 and n.sum().item() == 0
    too_many_q = torch.zeros((65537, 8), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(moin.MoinError) as ei:
        moin.moin_route(ctx, too_many_q, rin.centroids[:, :8].contiguous(), static=True)
    assert ei.value.code == -5
    too_many_c = torch.zeros((16385, 8), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(moin.MoinError) as ei:
        moin.moin_route(ctx, rin.emb[:, :8].contiguous(), too_many_c, static=True)
    assert ei.value.code == -5
    # at the limits it runs: 65536 queries against 16384 centroids of 8 dimensions
    g = torch.Generator(device="cuda").manual_seed(3)
    q = torch.randn((65536, 8), device="cuda", generator=g).to(torch.bfloat16)
    cen = torch.randn((16384, 8), device="cuda", generator=g).to(torch.bfloat16)
    print("[gpu] static route at its size limits", flush=True)
    got = moin.moin_route(ctx, q, cen, want_counts=True, static=True)
    ctx.check()
    ref = moin.moin_route(ctx, q, cen, want_counts=True)
    ctx.check()
    for a, b in zip(got, ref):
        assert torch.equal(a, b)
