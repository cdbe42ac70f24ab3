"""Pins of the oracle's K-means centre update (Section 3.1: plain K-means in the
embedding space, its centres are the topic embeddings): a hand-worked example,
closed forms, conservation laws and the descent property of Lloyd's iteration.
None of them re-uses the oracle's own formula."""
import os

import numpy as np
import pytest

import oracle
from tests.helpers import bits_to_f64, read_golden, to_bf16_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "kmeans_hand_example.txt")


def test_hand_worked_example():
    g = read_golden(GOLDEN)
    pts = np.array(g["points"], dtype=np.float32).reshape(5, 2)
    ids = np.array(g["ids"], dtype=np.int32)
    old = np.array(g["old"], dtype=np.float32).reshape(3, 2)
    new, counts, inertia = oracle.kmeans_update(pts, ids, old)
    assert np.allclose(new.ravel(), g["new"], rtol=0, atol=1e-15)
    assert counts.tolist() == [int(v) for v in g["counts"]]
    assert inertia == g["inertia"][0]


def test_points_on_a_line_closed_form():
    # points 0..9 on a line (padded to D = 4 with zeros), ids 0 for < 5 else 1:
    # means 2 and 7; inertia against old centres 0 and 9: sum k^2 (k<5) + sum (9-k)^2 (k>=5)
    x = np.zeros((10, 4), dtype=np.float32)
    x[:, 0] = np.arange(10)
    ids = (np.arange(10) >= 5).astype(np.int32)
    old = np.array([[0, 0, 0, 0], [9, 0, 0, 0]], dtype=np.float32)
    new, counts, inertia = oracle.kmeans_update(x, ids, old)
    assert np.array_equal(new, [[2, 0, 0, 0], [7, 0, 0, 0]])
    assert counts.tolist() == [5, 5]
    assert inertia == 2 * (0 + 1 + 4 + 9 + 16)


def test_points_equal_to_their_centres_are_a_fixed_point():
    rng = np.random.default_rng(1)
    cent = to_bf16_bits(rng.standard_normal((7, 16)))
    ids = rng.integers(0, 7, size=50).astype(np.int32)
    ids[:7] = np.arange(7)                       # every centre used
    new, counts, inertia = oracle.kmeans_update(cent[ids], ids, cent)
    assert np.array_equal(new, bits_to_f64(cent))
    assert inertia == 0.0 and counts.sum() == 50


def test_empty_clusters_keep_their_old_centre_and_mass_is_conserved():
    rng = np.random.default_rng(2)
    x = to_bf16_bits(rng.standard_normal((200, 24)))
    old = to_bf16_bits(rng.standard_normal((9, 24)))
    ids = rng.choice([0, 2, 3, 7], size=200).astype(np.int32)
    new, counts, _ = oracle.kmeans_update(x, ids, old)
    for k in (1, 4, 5, 6, 8):
        assert counts[k] == 0 and np.array_equal(new[k], bits_to_f64(old[k]))
    # sum_k count_k * mean_k = sum_i x_i, checked with an independent exact sum
    total = (counts[:, None] * new)[counts > 0].sum(axis=0)
    xs = bits_to_f64(x)
    exact = np.array([float(np.sum(xs[:, j], dtype=np.longdouble)) for j in range(24)])
    assert np.allclose(total, exact, rtol=1e-12, atol=1e-12)
    assert np.array_equal(counts, np.bincount(ids, minlength=9))


def test_mean_minimises_the_within_cluster_sum_of_squares():
    # the update must return the minimiser of sum ||x - c||^2 per cluster: any
    # perturbed centre is worse (fp64, independent evaluation with numpy)
    rng = np.random.default_rng(3)
    x = rng.standard_normal((300, 8)).astype(np.float32)
    ids = rng.integers(0, 5, size=300).astype(np.int32)
    old = rng.standard_normal((5, 8)).astype(np.float32)
    new, _, _ = oracle.kmeans_update(x, ids, old)
    xs = x.astype(np.float64)
    for k in range(5):
        pts = xs[ids == k]
        best = ((pts - new[k]) ** 2).sum()
        for _ in range(5):
            other = new[k] + 1e-3 * rng.standard_normal(8)
            assert ((pts - other) ** 2).sum() > best


def test_lloyd_iterations_never_increase_the_objective():
    # assignment (oracle.route) + update: the inertia sequence is non-increasing
    # and the assignment-step inertia equals the sum of the routed minimum distances
    rng = np.random.default_rng(4)
    x = rng.standard_normal((400, 12)).astype(np.float32)
    cent = x[rng.choice(400, size=10, replace=False)].copy()
    prev = np.inf
    for _ in range(6):
        ids, best, _ = oracle.route(x, cent, want_gaps=True)
        new, counts, inertia = oracle.kmeans_update(x, ids, cent)
        assert np.isclose(inertia, best.sum(), rtol=1e-12)
        assert inertia <= prev * (1 + 1e-12)
        prev = inertia
        cent = new.astype(np.float32)


def test_bad_ids_are_rejected_and_dtypes_agree():
    x = np.zeros((3, 4), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.kmeans_update(x, np.array([0, 5, 0], np.int32), np.zeros((2, 4), np.float32))
    # bf16 storage widens exactly: same result as the fp32 copy of the same values
    rng = np.random.default_rng(5)
    xb = to_bf16_bits(rng.standard_normal((40, 8)))
    cb = to_bf16_bits(rng.standard_normal((3, 8)))
    ids = rng.integers(0, 3, size=40).astype(np.int32)
    a = oracle.kmeans_update(xb, ids, cb)
    b = oracle.kmeans_update(bits_to_f64(xb).astype(np.float32), ids, bits_to_f64(cb).astype(np.float32))
    assert np.array_equal(a[0], b[0]) and a[2] == b[2]


def test_retained_clusters_are_numbered_in_order():
    # hand example: threshold 3 keeps clusters 0, 2 and 5
    slot, kept = oracle.retain_clusters([3, 2, 10, 0, 1, 3], 3)
    assert slot.tolist() == [0, -1, 1, -1, -1, 2] and kept == 3
    # threshold 0 keeps everything (identity map), a threshold above the maximum nothing
    slot, kept = oracle.retain_clusters([0, 5, 1], 0)
    assert slot.tolist() == [0, 1, 2] and kept == 3
    slot, kept = oracle.retain_clusters([0, 5, 1], 6)
    assert slot.tolist() == [-1, -1, -1] and kept == 0
    # invariants on random counts: kept == #(counts >= t); kept slots are 0..kept-1 ascending
    rng = np.random.default_rng(6)
    counts = rng.integers(0, 50, size=200)
    slot, kept = oracle.retain_clusters(counts, 20)
    assert kept == int((counts >= 20).sum())
    assert np.array_equal(slot[slot >= 0], np.arange(kept))
    assert np.array_equal(slot >= 0, counts >= 20)
    # composing with the slot map sends members of dropped clusters to the base model (-1)
    ids = rng.integers(0, 200, size=1000).astype(np.int32)
    mapped = oracle.slot_map(ids, slot)
    assert np.array_equal(mapped < 0, counts[ids] < 20)
