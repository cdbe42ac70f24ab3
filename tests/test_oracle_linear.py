"""Pins for the oracle's routed LoRA linear (Section 3.2: y = W x + W_b (W_a x)).

Each test is chosen so that one plausible mistake -- a dropped term, a
transposed operand, a wrong gather index, a misplaced scale -- fails it.
CPU only.
"""
import os

import numpy as np
import pytest

import oracle
from tests.helpers import bits_to_f64, read_golden, to_bf16_bits


def _rand_case(rng, T_lens, d_in, d_out, r, E):
    T = int(sum(T_lens))
    x = to_bf16_bits(rng.standard_normal((T, d_in)))
    W = to_bf16_bits(rng.standard_normal((d_out, d_in)) / np.sqrt(d_in))
    A = to_bf16_bits(rng.standard_normal((E, r, d_in)) / np.sqrt(d_in))
    B = to_bf16_bits(rng.standard_normal((E, d_out, r)) / np.sqrt(r))
    off = np.concatenate([[0], np.cumsum(T_lens)]).astype(np.int32)
    ids = rng.integers(0, E, size=len(T_lens)).astype(np.int32)
    return x, W, A, B, off, ids


def test_hand_worked_example(golden_dir):
    g = read_golden(os.path.join(golden_dir, "lora_hand_example.txt"))
    d_in, d_out, r = int(g["d_in"][0]), int(g["d_out"][0]), int(g["r"][0])
    W = to_bf16_bits(np.array(g["W"]).reshape(d_out, d_in))
    A = to_bf16_bits(np.array(g["A"]).reshape(-1, r, d_in))
    # fixture lists W_b per expert as a column: [E, d_out, r]
    B = to_bf16_bits(np.array(g["B"]).reshape(-1, d_out, r))
    x = to_bf16_bits(np.array(g["x"]).reshape(-1, d_in))
    y = oracle.lora_linear(x, np.array(g["seq_offsets"], dtype=np.int32),
                           np.array(g["expert_ids"], dtype=np.int32), W, A, B, g["scale"][0])
    assert np.array_equal(y, np.array(g["y"]).reshape(-1, d_out))


def test_zero_B_reproduces_base_layer():
    """Invariant: W_b = 0 gives the frozen layer, a textbook GEMM (numpy fp64)."""
    rng = np.random.default_rng(1)
    x, W, A, B, off, ids = _rand_case(rng, [5, 9, 3], 48, 40, 8, 4)
    B[:] = 0
    y = oracle.lora_linear(x, off, ids, W, A, B, 2.0)
    ref = bits_to_f64(x) @ bits_to_f64(W).T
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)
    # and the same through the explicit fallback id and through absent stacks
    y2 = oracle.lora_linear(x, off, np.full_like(ids, -1), W, A, B, 2.0)
    y3 = oracle.lora_linear(x, off, np.full_like(ids, -1), W, None, None, 2.0)
    assert np.array_equal(y2, y) and np.array_equal(y3, y)


def test_uniform_assignment_equals_merged_weight():
    """Invariant: one expert for every sequence == the merged W + s W_b W_a."""
    rng = np.random.default_rng(2)
    x, W, A, B, off, _ = _rand_case(rng, [7, 1, 12], 64, 24, 16, 5)
    e, s = 3, 2.0
    ids = np.full(3, e, dtype=np.int32)
    y = oracle.lora_linear(x, off, ids, W, A, B, s)
    merged = bits_to_f64(W) + s * (bits_to_f64(B[e]) @ bits_to_f64(A[e]))
    ref = bits_to_f64(x) @ merged.T
    assert np.allclose(y, ref, rtol=1e-11, atol=1e-11)
    # a different expert must give a different answer (the gather is live)
    y_other = oracle.lora_linear(x, off, np.full(3, 1, dtype=np.int32), W, A, B, s)
    assert np.abs(y_other - y).max() > 1e-2


def test_identity_closed_form():
    """W = I, W_a = first r rows of I, W_b = first r columns of I, s = 2:
    y = x + 2 * (x_0..x_{r-1}, 0, ...), exact."""
    rng = np.random.default_rng(3)
    d, r, T = 32, 8, 6
    x = to_bf16_bits(rng.integers(-8, 9, size=(T, d)))
    eye = np.eye(d)
    W = to_bf16_bits(eye)
    A = to_bf16_bits(eye[:r][None])
    B = to_bf16_bits(eye[:, :r][None])
    y = oracle.lora_linear(x, np.array([0, T], dtype=np.int32), np.array([0], dtype=np.int32),
                           W, A, B, 2.0)
    xf = bits_to_f64(x)
    ref = xf.copy()
    ref[:, :r] += 2.0 * xf[:, :r]
    assert np.array_equal(y, ref)


def test_selection_matrices_catch_transposes():
    """Non-square selection matrices with a closed form: W picks input column
    pw[o] for output o; W_a picks input column pa[j]; W_b adds u_j to output
    pb[j] only.  Any transposed or mis-strided operand changes the answer."""
    rng = np.random.default_rng(4)
    d_in, d_out, r, T, s = 12, 7, 3, 5, 0.5
    pw = rng.integers(0, d_in, size=d_out)
    pa = np.array([2, 9, 11])
    pb = np.array([6, 0, 3])
    Wm = np.zeros((d_out, d_in)); Wm[np.arange(d_out), pw] = 1
    Am = np.zeros((1, r, d_in)); Am[0, np.arange(r), pa] = 1
    Bm = np.zeros((1, d_out, r)); Bm[0, pb, np.arange(r)] = 1
    xv = rng.integers(-5, 6, size=(T, d_in)).astype(np.float64)
    y = oracle.lora_linear(to_bf16_bits(xv), np.array([0, T], dtype=np.int32),
                           np.array([0], dtype=np.int32), to_bf16_bits(Wm), to_bf16_bits(Am),
                           to_bf16_bits(Bm), s)
    ref = xv[:, pw].copy()
    for j in range(r):
        ref[:, pb[j]] += s * xv[:, pa[j]]
    assert np.array_equal(y, ref)


def test_mixed_experts_match_per_sequence_numpy():
    rng = np.random.default_rng(5)
    lens = [4, 0, 11, 1, 6]
    x, W, A, B, off, ids = _rand_case(rng, lens, 40, 56, 8, 6)
    ids[3] = -1
    s = 2.0
    y = oracle.lora_linear(x, off, ids, W, A, B, s)
    xf, Wf = bits_to_f64(x), bits_to_f64(W)
    for q in range(len(lens)):
        lo, hi = off[q], off[q + 1]
        ref = xf[lo:hi] @ Wf.T
        if ids[q] >= 0:
            ref = ref + s * (xf[lo:hi] @ bits_to_f64(A[ids[q]]).T) @ bits_to_f64(B[ids[q]]).T
        assert np.allclose(y[lo:hi], ref, rtol=1e-11, atol=1e-11)


def test_adapter_term_is_linear_in_scale():
    rng = np.random.default_rng(6)
    x, W, A, B, off, ids = _rand_case(rng, [3, 5], 32, 16, 4, 3)
    y0 = oracle.lora_linear(x, off, ids, W, A, B, 0.0)
    y1 = oracle.lora_linear(x, off, ids, W, A, B, 1.0)
    y3 = oracle.lora_linear(x, off, ids, W, A, B, 3.0)
    assert np.allclose(y0, bits_to_f64(x) @ bits_to_f64(W).T, rtol=1e-12, atol=1e-12)
    assert np.allclose(y3 - y0, 3.0 * (y1 - y0), rtol=1e-10, atol=1e-12)
    assert np.abs(y1 - y0).max() > 1e-2


def test_metamorphic_relations():
    rng = np.random.default_rng(7)
    lens = [6, 2, 9, 4]
    x, W, A, B, off, ids = _rand_case(rng, lens, 24, 20, 4, 5)
    ids[:] = [4, 0, 2, 0]
    s = 2.0
    y = oracle.lora_linear(x, off, ids, W, A, B, s)

    # permuting whole sequences permutes the output rows
    order = [2, 0, 3, 1]
    xs = np.concatenate([x[off[q]:off[q + 1]] for q in order])
    offp = np.concatenate([[0], np.cumsum([lens[q] for q in order])]).astype(np.int32)
    yp = oracle.lora_linear(xs, offp, ids[order], W, A, B, s)
    assert np.array_equal(yp, np.concatenate([y[off[q]:off[q + 1]] for q in order]))

    # splitting a sequence in two with the same expert changes nothing
    off_split = np.array([0, 6, 8, 12, 17, 21], dtype=np.int32)
    ids_split = np.array([4, 0, 2, 2, 0], dtype=np.int32)
    assert np.array_equal(oracle.lora_linear(x, off_split, ids_split, W, A, B, s), y)

    # relabelling experts (permute stacks and ids together) changes nothing
    perm = rng.permutation(5)               # new slot p holds old expert perm[p]
    inv = np.argsort(perm)
    assert np.array_equal(oracle.lora_linear(x, off, inv[ids].astype(np.int32), W, A[perm],
                                             B[perm], s), y)

    # an expert no sequence uses may hold NaNs without effect
    A2, B2 = A.copy(), B.copy()
    A2[1] = 0x7FC0
    B2[3] = 0x7FC0
    assert np.array_equal(oracle.lora_linear(x, off, ids, W, A2, B2, s), y)


def test_row_subset_equals_full():
    rng = np.random.default_rng(8)
    x, W, A, B, off, ids = _rand_case(rng, [5, 5, 5], 16, 12, 4, 3)
    y = oracle.lora_linear(x, off, ids, W, A, B, 2.0)
    rows = np.array([14, 0, 7, 7, 5])
    assert np.array_equal(oracle.lora_linear(x, off, ids, W, A, B, 2.0, rows=rows), y[rows])
    assert np.array_equal(oracle.lora_linear(x, off, ids, W, A, B, 2.0, threads=1), y)


def test_empty_and_invalid_inputs():
    rng = np.random.default_rng(9)
    x, W, A, B, off, ids = _rand_case(rng, [2, 2], 8, 8, 2, 2)
    y = oracle.lora_linear(x[:0], np.array([0], dtype=np.int32), np.zeros(0, np.int32), W, A, B, 2.0)
    assert y.shape == (0, 8)
    with pytest.raises(ValueError):
        oracle.lora_linear(x, off, np.array([0, 2], dtype=np.int32), W, A, B, 2.0)   # id >= E
    with pytest.raises(ValueError):
        oracle.lora_linear(x, np.array([0, 3, 2], dtype=np.int32), ids, W, A, B, 2.0)  # not monotone / end != T
    with pytest.raises(ValueError):
        oracle.lora_linear(x, off, np.array([0, -2], dtype=np.int32), W, A, B, 2.0)


def test_adaptive_rank_per_expert():
    """"Future Works" (adaptive rank per topic): expert e uses its first rank_e rows of
    A_e and columns of B_e.  Pinned against numpy fp64 on truncated copies, against the
    padded-with-zeros equivalence, and against the limits rank = r and rank = 0."""
    rng = np.random.default_rng(21)
    d_in, d_out, r, E = 24, 16, 8, 4
    lens = [3, 2, 4, 1, 2]
    ids = np.array([2, 0, 3, 1, 2], np.int32)
    ranks = np.array([8, 0, 3, 5], np.int32)
    T = sum(lens)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    x = to_bf16_bits(rng.standard_normal((T, d_in)))
    W = to_bf16_bits(rng.standard_normal((d_out, d_in)) * 0.2)
    A = to_bf16_bits(rng.standard_normal((E, r, d_in)) * 0.2)
    B = to_bf16_bits(rng.standard_normal((E, d_out, r)) * 0.3)
    got = oracle.lora_linear(x, off, ids, W, A, B, 2.0, rank_of_expert=ranks)
    # numpy fp64 on explicitly truncated factors, token by token
    xs, Ws, As, Bs = bits_to_f64(x), bits_to_f64(W), bits_to_f64(A), bits_to_f64(B)
    want = np.zeros((T, d_out))
    for s, e in enumerate(ids):
        k = ranks[e]
        for t in range(off[s], off[s + 1]):
            want[t] = Ws @ xs[t] + 2.0 * (Bs[e][:, :k] @ (As[e][:k] @ xs[t]))
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    # same as full rank on stacks whose tail is zeroed; what lies in the tail is never read
    Az, Bz = A.copy(), B.copy()
    An, Bn = A.copy(), B.copy()
    for e in range(E):
        Az[e, ranks[e]:] = 0
        Bz[e][:, ranks[e]:] = 0
        An[e, ranks[e]:] = 0x7FC0          # bf16 NaN
        Bn[e][:, ranks[e]:] = 0x7FC0
    assert np.array_equal(got, oracle.lora_linear(x, off, ids, W, Az, Bz, 2.0))
    assert np.array_equal(got, oracle.lora_linear(x, off, ids, W, An, Bn, 2.0, rank_of_expert=ranks))
    # limits: all ranks = r is the plain layer; all ranks = 0 is the base layer
    full = oracle.lora_linear(x, off, ids, W, A, B, 2.0)
    assert np.array_equal(full, oracle.lora_linear(x, off, ids, W, A, B, 2.0, rank_of_expert=np.full(E, r)))
    base = oracle.lora_linear(x, off, np.full(len(ids), -1, np.int32), W, A, B, 2.0)
    assert np.array_equal(base, oracle.lora_linear(x, off, ids, W, A, B, 2.0, rank_of_expert=np.zeros(E, np.int32)))
    with pytest.raises(ValueError):
        oracle.lora_linear(x, off, ids, W, A, B, 2.0, rank_of_expert=np.array([9, 0, 0, 0]))


def test_general_case_against_numpy_matrices():
    """Several experts, base-only and empty sequences, per-expert ranks, a row subset: the layer written
    sequence by sequence with numpy fp64 matrix products."""
    rng = np.random.default_rng(77)
    lens = [5, 0, 9, 3, 1, 7]
    x, W, A, B, off, _ = _rand_case(rng, lens, 40, 24, 16, 4)
    ids = np.array([2, 1, -1, 0, 3, 2], dtype=np.int32)
    ranks = np.array([16, 8, 0, 5], dtype=np.int32)
    s = 2.0
    xd, Wd, Ad, Bd = bits_to_f64(x), bits_to_f64(W), bits_to_f64(A), bits_to_f64(B)
    for rk in (None, ranks):
        ref = xd @ Wd.T
        for q, e in enumerate(ids):
            if e < 0:
                continue
            k = 16 if rk is None else int(rk[e])
            rows = slice(off[q], off[q + 1])
            ref[rows] += s * (xd[rows] @ Ad[e, :k].T) @ Bd[e][:, :k].T
        y = oracle.lora_linear(x, off, ids, W, A, B, s, rank_of_expert=rk)
        assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)
        sub = np.array([24, 0, 13, 14, 5], dtype=np.int64)
        assert np.array_equal(oracle.lora_linear(x, off, ids, W, A, B, s, rank_of_expert=rk, rows=sub), y[sub])
