"""GPU parity of moin_route_topk against the oracle: ids in order, ties by index, the near-tie band of the
router's reading for distances that fp32 rounding can swap."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_09687_amd import moin
from paper_2410_09687_amd import workloads as wl
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu


def _host(t):
    return wl.bf16_bits(t) if t.dtype == torch.bfloat16 else t.cpu().numpy()


def _check(emb, cent, k, slot=None, retained_only=False, what=""):
    ctx = gc.ctx()
    print(f"[gpu] route_topk {what} N={emb.shape[0]} K={cent.shape[0]} D={emb.shape[1]} k={k} {emb.dtype}", flush=True)
    eids, cids, d2 = moin.moin_route_topk(ctx, emb, cent, k, slot_of_centroid=slot, retained_only=retained_only)
    ctx.check()
    el = None
    if retained_only:
        el = (slot.cpu().numpy() >= 0)
    ref_ids, ref_d2 = oracle.route_topk(_host(emb), _host(cent), k, eligible=el)
    got = cids.cpu().numpy()
    gd = d2.double().cpu().numpy()
    # unfilled places agree exactly
    assert np.array_equal(got < 0, ref_ids < 0) and np.array_equal(np.isinf(gd), np.isinf(ref_d2))
    n_band = 0
    for i, m in zip(*np.nonzero(got != ref_ids)):
        # a different centroid in a place is accepted only inside the near-tie band (relative 1e-4 on the
        # squared distance, in fp64) of the distance that belongs there
        true_d = oracle.dist2(_host(emb), _host(cent), np.array([i]), np.array([got[i, m]]))[0]
        assert true_d <= ref_d2[i, m] * (1 + 1e-4) + 1e-30, (i, m, got[i], ref_ids[i], true_d, ref_d2[i, m])
        n_band += 1
    filled = got >= 0
    rows = np.nonzero(filled)
    true = oracle.dist2(_host(emb), _host(cent), rows[0], got[filled])
    assert np.allclose(gd[filled], true, rtol=2e-5, atol=1e-30)
    for r in got.tolist():
        f = [v for v in r if v >= 0]
        assert len(set(f)) == len(f)
    want_e = got if slot is None else np.where(got >= 0, slot.cpu().numpy()[np.maximum(got, 0)], -1)
    assert np.array_equal(eids.cpu().numpy(), want_e)
    return n_band


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_random_embeddings(dtype):
    g = torch.Generator(device="cuda").manual_seed(11)
    emb = torch.randn((300, 768), device="cuda", generator=g).to(dtype)
    cent = torch.randn((517, 768), device="cuda", generator=g).to(dtype)
    total = 0
    for k in (1, 3, 8):
        total += _check(emb, cent, k, what="random")
    print(f"[gpu] {total} places inside the near-tie band", flush=True)
    # column 0 is the router's answer
    _, cids, _ = moin.moin_route_topk(gc.ctx(), emb, cent, 1)
    _, rc, _ = moin.moin_route(gc.ctx(), emb, cent)
    gc.ctx().check()
    assert (cids[:, 0] != rc).sum().item() <= 1


def test_exact_ties_keep_index_order_and_small_shapes():
    D = 64
    cent = torch.eye(D, device="cuda")[:40]
    cent = torch.cat([cent, cent[5:6], cent[5:6]])      # 40 and 41 duplicate 5
    emb = torch.eye(D, device="cuda")[[5, 0, 39, 50]]    # the last query is equally far from everything
    for dt in (torch.float32, torch.bfloat16):
        n = _check(emb.to(dt), cent.to(dt), 4, what="one-hot")
        assert n == 0
        _, cids, d2 = moin.moin_route_topk(gc.ctx(), emb.to(dt), cent.to(dt), 4)
        assert cids.tolist() == [[5, 40, 41, 0], [0, 1, 2, 3], [39, 0, 1, 2], [0, 1, 2, 3]]
        assert d2.tolist() == [[0, 0, 0, 2], [0, 2, 2, 2], [0, 2, 2, 2], [2, 2, 2, 2]]
    # D with a ragged last round of lanes, fewer centroids than k
    g = torch.Generator(device="cuda").manual_seed(12)
    _check(torch.randn((9, 200), device="cuda", generator=g), torch.randn((3, 200), device="cuda", generator=g), 8,
           what="K<k")
    _check(torch.randn((1, 8), device="cuda", generator=g).bfloat16(),
           torch.randn((11, 8), device="cuda", generator=g).bfloat16(), 2, what="tiny")


def test_slot_map_retained_only_and_argument_errors():
    g = torch.Generator(device="cuda").manual_seed(13)
    emb = torch.randn((50, 128), device="cuda", generator=g)
    cent = torch.randn((30, 128), device="cuda", generator=g)
    slot = torch.full((30,), -1, dtype=torch.int32, device="cuda")
    slot[[2, 9, 17, 28]] = torch.tensor([7, 3, 0, 5], dtype=torch.int32, device="cuda")
    _check(emb, cent, 6, slot=slot, what="slot map")
    _check(emb, cent, 6, slot=slot, retained_only=True, what="retained only")
    with pytest.raises(ValueError):
        moin.moin_route_topk(gc.ctx(), emb, cent, 9)
    with pytest.raises(moin.MoinError):
        moin.moin_route_topk(gc.ctx(), emb, cent, 2, retained_only=True)
    e, c, d = moin.moin_route_topk(gc.ctx(), emb[:0], cent, 2)
    assert e.shape == (0, 2)
