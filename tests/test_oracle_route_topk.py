"""Pins for the oracle's k nearest centroids ("Future Works", creating new experts on the fly: queries on the
boundary of several clusters).  CPU only."""
import numpy as np
import pytest

import oracle
from tests.helpers import bits_to_f64, to_bf16_bits


def _brute(q, c, k, eligible=None):
    """numpy: all distances by broadcasting, then a lexicographic sort by (distance, index)."""
    d = ((q[:, None, :].astype(np.float64) - c[None, :, :].astype(np.float64)) ** 2).sum(axis=2)
    if eligible is not None:
        d = np.where(np.asarray(eligible, bool)[None, :], d, np.inf)
    K = c.shape[0]
    ids = np.zeros((q.shape[0], k), np.int32)
    dd = np.zeros((q.shape[0], k))
    for i in range(q.shape[0]):
        order = np.lexsort((np.arange(K), d[i]))[:k]
        for m in range(k):
            if m < len(order) and np.isfinite(d[i, order[m]]):
                ids[i, m], dd[i, m] = order[m], d[i, order[m]]
            else:
                ids[i, m], dd[i, m] = -1, np.inf
    return ids, dd


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_against_numpy_sort_and_first_column_is_the_router(dtype):
    rng = np.random.default_rng(3)
    q = rng.standard_normal((37, 24)).astype(np.float32)
    c = rng.standard_normal((19, 24)).astype(np.float32)
    if dtype == "bf16":
        qa, ca = to_bf16_bits(q), to_bf16_bits(c)
        qf, cf = bits_to_f64(qa), bits_to_f64(ca)
    else:
        qa, ca, qf, cf = q, c, q, c
    for k in (1, 3, 19, 25):
        ids, d2 = oracle.route_topk(qa, ca, k)
        bi, bd = _brute(qf, cf, k)
        assert np.array_equal(ids, bi)
        assert np.allclose(d2[np.isfinite(bd)], bd[np.isfinite(bd)], rtol=1e-13) and np.array_equal(np.isinf(d2), np.isinf(bd))
        assert np.array_equal(ids[:, 0], oracle.route(qa, ca))


def test_hand_cases_ties_and_duplicates():
    # one-hot vectors: a query e_j is at distance 0 from centroid e_j and sqrt(2) from every other one,
    # so the list is (j, then the remaining indices in increasing order); duplicated centroids tie as well
    D = 6
    c = np.eye(D, dtype=np.float32)
    c = np.concatenate([c, c[2:3]])           # centroid 6 duplicates centroid 2
    q = np.eye(D, dtype=np.float32)[[4, 2, 0]]
    ids, d2 = oracle.route_topk(q, c, 4)
    assert ids.tolist() == [[4, 0, 1, 2], [2, 6, 0, 1], [0, 1, 2, 3]]
    assert d2.tolist() == [[0, 2, 2, 2], [0, 0, 2, 2], [0, 2, 2, 2]]


def test_nested_lists_ascending_distances_and_eligibility():
    rng = np.random.default_rng(4)
    q = rng.standard_normal((20, 8)).astype(np.float32)
    c = rng.standard_normal((30, 8)).astype(np.float32)
    i8, d8 = oracle.route_topk(q, c, 8)
    i3, d3 = oracle.route_topk(q, c, 3)
    assert np.array_equal(i8[:, :3], i3) and np.array_equal(d8[:, :3], d3)
    assert (np.diff(d8, axis=1) >= 0).all()
    assert all(len(set(r)) == 8 for r in i8.tolist())
    el = np.zeros(30, bool)
    el[[3, 11, 29]] = True
    ie, de = oracle.route_topk(q, c, 5, eligible=el)
    assert set(ie[:, :3].ravel().tolist()) <= {3, 11, 29} and (ie[:, 3:] == -1).all() and np.isinf(de[:, 3:]).all()
    bi, _ = _brute(q, c, 5, el)
    assert np.array_equal(ie, bi)
    # a centroid full of NaN never enters a list
    c2 = c.copy()
    c2[7] = np.nan
    assert 7 not in oracle.route_topk(q, c2, 30)[0][:, :29]
    with pytest.raises(ValueError):
        oracle.route_topk(q, c, 0)
