"""Pins for the oracle's adapter with an activation between its two linear layers ("Future Works",
better adapters): y = W x + s W_b act(W_a x).  CPU only."""
import os

import numpy as np
import pytest
import torch

import oracle
from tests.helpers import bits_to_f64, read_golden, to_bf16_bits

ACTS = ("relu", "silu", "gelu")


def _rand_case(rng, T_lens, d_in, d_out, r, E):
    T = int(sum(T_lens))
    x = to_bf16_bits(rng.standard_normal((T, d_in)))
    W = to_bf16_bits(rng.standard_normal((d_out, d_in)) / np.sqrt(d_in))
    A = to_bf16_bits(rng.standard_normal((E, r, d_in)) / np.sqrt(d_in))
    B = to_bf16_bits(rng.standard_normal((E, d_out, r)) / np.sqrt(r))
    off = np.concatenate([[0], np.cumsum(T_lens)]).astype(np.int32)
    ids = rng.integers(-1, E, size=len(T_lens)).astype(np.int32)
    return x, W, A, B, off, ids


def test_hand_worked_example(golden_dir):
    g = read_golden(os.path.join(golden_dir, "activation_hand_example.txt"))
    d_in, d_out, r = int(g["d_in"][0]), int(g["d_out"][0]), int(g["r"][0])
    W = to_bf16_bits(np.array(g["W"]).reshape(d_out, d_in))
    A = to_bf16_bits(np.array(g["A"]).reshape(1, r, d_in))
    B = to_bf16_bits(np.array(g["B"]).reshape(1, d_out, r))
    x = to_bf16_bits(np.array(g["x"]).reshape(1, d_in))
    off, ids = np.array([0, 1], np.int32), np.array([0], np.int32)
    for act in (None, "none") + ACTS:
        y = oracle.lora_linear(x, off, ids, W, A, B, g["scale"][0], activation=act)
        want = g["y_" + (act or "none")][0]
        assert abs(y[0, 0] - want) <= 4e-16 * max(1.0, abs(want)), (act, y[0, 0], want)


@pytest.mark.parametrize("act", ACTS)
def test_against_the_library_activation_in_fp64(act):
    """The layer written with torch's own activation routines (fp64, CPU)."""
    rng = np.random.default_rng(11)
    x, W, A, B, off, ids = _rand_case(rng, [4, 7, 1, 5], 40, 24, 16, 3)
    s = 2.0
    y = oracle.lora_linear(x, off, ids, W, A, B, s, activation=act)
    f = {"relu": torch.relu, "silu": torch.nn.functional.silu, "gelu": torch.nn.functional.gelu}[act]
    xd, Wd = torch.from_numpy(bits_to_f64(x)), torch.from_numpy(bits_to_f64(W))
    ref = xd @ Wd.T
    for q in range(len(ids)):
        e = ids[q]
        if e < 0:
            continue
        rows = slice(off[q], off[q + 1])
        Ad, Bd = torch.from_numpy(bits_to_f64(A[e])), torch.from_numpy(bits_to_f64(B[e]))
        ref[rows] += s * (f(xd[rows] @ Ad.T) @ Bd.T)
    assert np.allclose(y, ref.numpy(), rtol=1e-12, atol=1e-12)
    # and it is not the linear adapter
    assert np.abs(y - oracle.lora_linear(x, off, ids, W, A, B, s)).max() > 1e-2


@pytest.mark.parametrize("act", ACTS)
def test_odd_part_of_the_activation_is_the_linear_adapter(act):
    """act(v) - act(-v) = v for all three, so the layer with W_a minus the layer with -W_a is the plain
    adapter term s W_b W_a x: the activation sits on W_a x, before W_b and before the scale."""
    rng = np.random.default_rng(12)
    x, W, A, B, off, ids = _rand_case(rng, [6, 2, 9], 32, 20, 8, 4)
    ids = np.abs(ids)
    s = 2.0
    y_pos = oracle.lora_linear(x, off, ids, W, A, B, s, activation=act)
    y_neg = oracle.lora_linear(x, off, ids, W, A ^ np.uint16(0x8000), B, s, activation=act)
    lin = oracle.lora_linear(x, off, ids, W, A, B, s) - oracle.lora_linear(x, off, np.full_like(ids, -1), W, A, B, s)
    assert np.allclose(y_pos - y_neg, lin, rtol=1e-11, atol=1e-11)


def test_none_is_the_paper_adapter_bit_for_bit_and_ranks_compose():
    rng = np.random.default_rng(13)
    x, W, A, B, off, ids = _rand_case(rng, [3, 8, 2], 24, 16, 8, 3)
    y0 = oracle.lora_linear(x, off, ids, W, A, B, 2.0)
    assert np.array_equal(y0, oracle.lora_linear(x, off, ids, W, A, B, 2.0, activation="none"))
    # an expert's rank cuts rows of W_a / columns of W_b: the same as zeroing them (act(0) = 0)
    ranks = np.array([8, 3, 0], np.int32)
    A0, B0 = A.copy(), B.copy()
    for e, k in enumerate(ranks):
        A0[e, k:] = 0
        B0[e, :, k:] = 0
    for act in ACTS:
        y_r = oracle.lora_linear(x, off, ids, W, A, B, 2.0, activation=act, rank_of_expert=ranks)
        assert np.array_equal(y_r, oracle.lora_linear(x, off, ids, W, A0, B0, 2.0, activation=act))
    with pytest.raises(ValueError):
        oracle.lora_linear(x, off, ids, W, A, B, 2.0, activation="tanh")


def test_quantised_base_takes_the_same_activation():
    """On the MXFP8 base only the base term differs: (y_mx - y_mx_base_only) = (y - y_base_only)."""
    rng = np.random.default_rng(14)
    x, W, A, B, off, ids = _rand_case(rng, [5, 4], 64, 16, 8, 2)
    ids = np.abs(ids)
    Wq, Ws = oracle.mx_quantize(W)
    none = np.full_like(ids, -1)
    for act in ACTS:
        d_mx = oracle.lora_linear_mx(x, off, ids, Wq, Ws, A, B, 2.0, activation=act) - \
            oracle.lora_linear_mx(x, off, none, Wq, Ws, A, B, 2.0, activation=act)
        d = oracle.lora_linear(x, off, ids, W, A, B, 2.0, activation=act) - \
            oracle.lora_linear(x, off, none, W, A, B, 2.0, activation=act)
        assert np.allclose(d_mx, d, rtol=1e-11, atol=1e-11)
