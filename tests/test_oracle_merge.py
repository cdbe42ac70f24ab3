"""Pins for the oracle's merged adapter ("Future Works", creating new experts on the fly): one adapter of rank
n r that stands for a weighted sum of n existing ones.  CPU only."""
import numpy as np
import pytest

import oracle
from tests.helpers import bits_to_f64, to_bf16_bits


def _stacks(rng, E, r, d_in, d_out):
    A = to_bf16_bits(rng.standard_normal((E, r, d_in)) / np.sqrt(d_in))
    B = to_bf16_bits(rng.standard_normal((E, d_out, r)) / np.sqrt(r))
    return A, B


def test_the_merged_adapter_is_the_weighted_sum_of_its_parts():
    """With weights that are powers of two the scaled W_b is exact, so the layer with the merged adapter equals
    base + sum_m w_m (layer with adapter e_m - base), to fp64 rounding."""
    rng = np.random.default_rng(21)
    E, r, d_in, d_out, T = 5, 8, 32, 24, 7
    A, B = _stacks(rng, E, r, d_in, d_out)
    x = to_bf16_bits(rng.standard_normal((T, d_in)))
    W = to_bf16_bits(rng.standard_normal((d_out, d_in)) / np.sqrt(d_in))
    ids, w = np.array([3, 0, 4], np.int32), np.array([0.5, 2.0, -0.25], np.float32)
    Am, Bm = oracle.merge_adapters(A, B, ids, w, 32)
    assert Am.shape == (32, d_in) and Bm.shape == (d_out, 32)
    off = np.array([0, T], np.int32)
    merged = oracle.lora_linear(x, off, np.array([0], np.int32), W, Am[None], Bm[None], 2.0)
    base = oracle.lora_linear(x, off, np.array([-1], np.int32), W, A, B, 2.0)
    want = base.copy()
    for e, wm in zip(ids, w):
        want += float(wm) * (oracle.lora_linear(x, off, np.array([e], np.int32), W, A, B, 2.0) - base)
    assert np.allclose(merged, want, rtol=1e-12, atol=1e-12)
    # and against the definition with numpy matrices
    Af, Bf = bits_to_f64(A), bits_to_f64(B)
    delta = sum(float(wm) * Bf[e] @ Af[e] for e, wm in zip(ids, w))
    assert np.allclose(bits_to_f64(Bm) @ bits_to_f64(Am), delta, rtol=1e-12, atol=1e-14)


def test_layout_padding_missing_ids_and_rounding():
    rng = np.random.default_rng(22)
    E, r, d_in, d_out = 4, 8, 16, 8
    A, B = _stacks(rng, E, r, d_in, d_out)
    # weight 1, one adapter: a copy, zero padded
    Am, Bm = oracle.merge_adapters(A, B, [2], [1.0], 24)
    assert np.array_equal(Am[:8], A[2]) and not Am[8:].any()
    assert np.array_equal(Bm[:, :8], B[2]) and not Bm[:, 8:].any()
    # an id of -1 leaves its block zero; blocks lie in the order of the list
    Am, Bm = oracle.merge_adapters(A, B, [1, -1, 3], [1.0, 5.0, 1.0], 24)
    assert np.array_equal(Am[:8], A[1]) and not Am[8:16].any() and np.array_equal(Am[16:], A[3])
    assert np.array_equal(Bm[:, :8], B[1]) and not Bm[:, 8:16].any() and np.array_equal(Bm[:, 16:], B[3])
    # the scaled W_b is rounded to nearest even from the fp32 product
    w = np.float32(1.0 + 2.0 ** -7)     # exact in fp32; b * w has up to 16 significant bits
    Am, Bm = oracle.merge_adapters(A, B, [0], [w], 8)
    prod = (bits_to_f64(B[0]).astype(np.float32) * w).astype(np.float32)
    assert np.array_equal(Bm, to_bf16_bits(prod))
    # a hand case: 1.5 * (1 + 2^-7) = 1.51171875 = 1 + 65.5 * 2^-7 -> tie between 65 and 66 -> even -> 66
    one = to_bf16_bits(np.array([[[1.5]]]))
    _, Bh = oracle.merge_adapters(to_bf16_bits(np.array([[[1.0]]])), one, [0], [w], 1)
    assert bits_to_f64(Bh)[0, 0] == 1.0 + 66 * 2.0 ** -7
    # and a tie whose even neighbour lies below: 1 * (1 + 66.5 * 2^-7) -> 66, not 67
    _, Bh = oracle.merge_adapters(to_bf16_bits(np.array([[[1.0]]])), to_bf16_bits(np.array([[[1.0]]])), [0],
                                  [np.float32(1.0 + 66.5 * 2.0 ** -7)], 1)
    assert bits_to_f64(Bh)[0, 0] == 1.0 + 66 * 2.0 ** -7
    with pytest.raises(ValueError):
        oracle.merge_adapters(A, B, [0, 1, 2, 3], [1, 1, 1, 1], 24)      # 32 > 24
    with pytest.raises(ValueError):
        oracle.merge_adapters(A, B, [4], [1.0], 8)
