"""Pins of the oracle's MXFP8 quantiser and of the routed LoRA linear layer on a
quantised base ("Future Works", quantising the base model; the block format is
the OCP Microscaling v1.0 MXFP8 one with FP8 E4M3 elements).  The value table
and the rounding are pinned against torch's float8_e4m3fn conversion (a library
routine the oracle does not use), a hand-worked block, closed forms and
invariants; the layer against numpy fp64 products of independently dequantised
operands and against the unquantised layer on exactly representable inputs.
CPU only."""
import os

import numpy as np
import pytest
import torch

import oracle
from tests.helpers import bits_to_f64, read_golden, to_bf16_bits


def _torch_e4m3_values(codes):
    t = torch.from_numpy(np.asarray(codes, dtype=np.uint8).copy()).view(torch.float8_e4m3fn)
    return t.to(torch.float32).numpy().astype(np.float64)


def _torch_e4m3_codes(values):
    t = torch.from_numpy(np.asarray(values, dtype=np.float32).copy()).to(torch.float8_e4m3fn)
    return t.view(torch.uint8).numpy()


def test_e4m3_value_table():
    codes = np.arange(256, dtype=np.uint8).reshape(1, 256)
    vals = oracle.mx_dequantize(codes, np.full((1, 8), 127, np.uint8))[0]
    ref = _torch_e4m3_values(codes[0])
    finite = ~np.isnan(ref)
    assert finite.sum() == 254 and np.isnan(vals[0x7F]) and np.isnan(vals[0xFF])
    assert np.array_equal(vals[finite], ref[finite])
    # anchors of the format: 1, the largest finite value, the smallest normal and subnormal
    assert vals[0x38] == 1.0 and vals[0x7E] == 448.0 and vals[0x08] == 2.0 ** -6 and vals[0x01] == 2.0 ** -9
    assert vals[0x80] == 0.0 and np.signbit(vals[0x80]) and vals[0xFE] == -448.0
    # the scale byte is a biased power-of-two exponent
    for E in (0, 1, 120, 127, 135, 254):
        v = oracle.mx_dequantize(codes, np.full((1, 8), E, np.uint8))[0]
        assert np.array_equal(v[finite], ref[finite] * 2.0 ** (E - 127))


def test_hand_worked_blocks(golden_dir):
    g = read_golden(os.path.join(golden_dir, "mx_hand_example.txt"))
    row = np.zeros(128)
    for b in range(4):
        row[32 * b:32 * b + len(g[f"block{b}"])] = g[f"block{b}"]
    bits = to_bf16_bits(row.reshape(1, 128))
    assert np.array_equal(bits_to_f64(bits)[0], row)          # the example is exact in bf16
    codes, scales = oracle.mx_quantize(bits)
    assert scales[0].tolist() == [int(v) for v in g["scales"]]
    back = oracle.mx_dequantize(codes, scales)[0]
    for b in range(4):
        n = len(g[f"codes{b}"])
        assert codes[0, 32 * b:32 * b + n].tolist() == [int(v) for v in g[f"codes{b}"]]
        assert not codes[0, 32 * b + n:32 * (b + 1)].any()
        assert back[32 * b:32 * b + n].tolist() == g[f"back{b}"]


def test_element_rounding_matches_the_library_conversion_on_every_bf16_value():
    # blocks led by 448 take scale 1, so the other 31 slots see the bare element rounding;
    # every finite bf16 value of magnitude <= 448 goes through one of them
    allb = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    v = bits_to_f64(allb)
    keep = np.isfinite(v) & (np.abs(v) <= 448)
    cand = allb[keep]
    pad = (-cand.size) % 31
    cand = np.concatenate([cand, np.zeros(pad, np.uint16)]).reshape(-1, 31)
    lead = np.full((cand.shape[0], 1), to_bf16_bits([448.0])[0], np.uint16)
    blocks = np.concatenate([lead, cand], axis=1)              # [n, 32]
    codes, scales = oracle.mx_quantize(blocks)
    assert (scales == 127).all()
    ref = _torch_e4m3_codes(bits_to_f64(blocks))
    assert np.array_equal(codes, ref)
    # ties go to the even mantissa: midpoints of neighbouring codes (exact in bf16)
    grid = _torch_e4m3_values(np.arange(0x08, 0x7E, dtype=np.uint8))
    mid = (grid[:-1] + grid[1:]) / 2
    mb = to_bf16_bits(mid)
    assert np.array_equal(bits_to_f64(mb), mid)
    blk = np.zeros((mid.size, 32), np.uint16)
    blk[:, 0] = lead[0, 0]
    blk[:, 1] = mb
    c, _ = oracle.mx_quantize(blk)
    assert (c[:, 1] % 2 == 0).all()
    lo = np.arange(0x08, 0x7D, dtype=np.uint8)
    assert np.array_equal(c[:, 1], np.where(lo % 2 == 0, lo, lo + 1))


def test_saturation_and_scale_choice():
    # amax in [256, 512) * 2^k: scale byte 127 + k; quotients above 448 clamp to the top code
    for k in (-30, -3, 0, 5, 40):
        vals = np.array([257.0, 448.0, 449.0, 464.0, 480.0, 510.0, -500.0, 300.0]) * 2.0 ** k
        blk = np.zeros((1, 32))
        blk[0, :8] = vals
        codes, scales = oracle.mx_quantize(to_bf16_bits(blk))
        assert scales[0, 0] == 127 + k
        assert codes[0, :8].tolist() == [0x78, 0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0xFE, 0x79]
    # powers of two: 2^m alone in a block is stored as 256 * 2^(m-8), exactly
    for m in (-100, -1, 0, 1, 100):
        blk = np.zeros((1, 32))
        blk[0, 7] = -2.0 ** m
        codes, scales = oracle.mx_quantize(to_bf16_bits(blk))
        assert scales[0, 0] == 127 + m - 8 and codes[0, 7] == 0xF8
        assert oracle.mx_dequantize(codes, scales)[0, 7] == -2.0 ** m
    # the scale byte stays inside 0..254: tiny blocks clamp at 0 and still round correctly
    blk = np.zeros((1, 32))
    blk[0, 0] = 2.0 ** -126                    # wants byte -7
    blk[0, 1] = 2.0 ** -133                    # smallest bf16 subnormal
    codes, scales = oracle.mx_quantize(to_bf16_bits(blk))
    assert scales[0, 0] == 0
    assert codes[0, 0] == 0x40 and codes[0, 1] == 0x08     # 2^-126 / 2^-127 = 2 ; 2^-6
    big = np.zeros((1, 32))
    big[0, 0] = 2.0 ** 127 * 1.5
    codes, scales = oracle.mx_quantize(to_bf16_bits(big))
    assert scales[0, 0] == 246 and codes[0, 0] == 0x7C


def test_quantiser_invariants():
    rng = np.random.default_rng(11)
    x = rng.standard_normal((64, 256)) * np.exp2(rng.integers(-6, 6, size=(64, 1)))
    x[3, 32:64] = 0.0
    bits = to_bf16_bits(x)
    v = bits_to_f64(bits)
    codes, scales = oracle.mx_quantize(bits)
    back = oracle.mx_dequantize(codes, scales)
    X = np.exp2(scales.astype(np.float64) - 127)
    amax = np.abs(v).reshape(64, 8, 32).max(axis=2)
    nz = amax > 0
    # scale = 2^(floor(log2 amax) - 8): amax / scale lies in [256, 512)
    assert ((amax[nz] / X[nz] >= 256) & (amax[nz] / X[nz] < 512)).all()
    assert (scales[~nz] == 127).all()
    # every block's largest element lands in the top binade; no NaN code is ever produced
    top = (codes & 0x7F).reshape(64, 8, 32).max(axis=2)
    assert (top[nz] >= 0x78).all() and ((codes & 0x7F) != 0x7F).all()
    # error bound: half a step of the top binade (16 scales) unless clamped, then below 64 scales;
    # relative to the element itself at most 2^-4 for elements that stay normal (>= 2^-6 scales)
    err = np.abs(back - v).reshape(64, 8, 32)
    q = np.abs(v).reshape(64, 8, 32) / X[:, :, None]
    assert (err[q <= 448] <= 16 * np.broadcast_to(X[:, :, None], err.shape)[q <= 448]).all()
    assert (err[q > 448] < 64 * np.broadcast_to(X[:, :, None], err.shape)[q > 448]).all()
    normal = (q >= 2.0 ** -6) & (q <= 448)
    assert (err[normal] <= np.abs(v).reshape(64, 8, 32)[normal] * 2.0 ** -4).all()
    # signs survive, zeros stay zero
    assert np.array_equal(np.signbit(back), np.signbit(v))
    assert (back[v == 0] == 0).all()
    # power-of-two rescaling moves only the scale byte; negation only the sign bit
    c2, s2 = oracle.mx_quantize(to_bf16_bits(v * 8.0))
    assert np.array_equal(c2, codes) and np.array_equal(s2[nz], scales[nz] + 3)
    c3, s3 = oracle.mx_quantize(to_bf16_bits(-v))
    assert np.array_equal(c3, codes ^ 0x80) and np.array_equal(s3, scales)
    # quantising the dequantised values changes nothing (they are exact in bf16)
    bb = to_bf16_bits(back)
    assert np.array_equal(bits_to_f64(bb), back)
    c4, s4 = oracle.mx_quantize(bb)
    assert np.array_equal(c4, codes) and np.array_equal(s4, scales)
    # blocks are independent: permuting whole blocks permutes the outputs
    perm = rng.permutation(8)
    c5, s5 = oracle.mx_quantize(bits.reshape(64, 8, 32)[:, perm].reshape(64, 256))
    assert np.array_equal(c5.reshape(64, 8, 32), codes.reshape(64, 8, 32)[:, perm])
    assert np.array_equal(s5, scales[:, perm])


def test_bad_inputs_are_rejected():
    with pytest.raises(ValueError):
        oracle.mx_quantize(np.zeros((2, 48), np.uint16))
    nan = np.zeros((1, 32), np.uint16)
    nan[0, 5] = 0x7FC0
    with pytest.raises(ValueError):
        oracle.mx_quantize(nan)
    inf = np.zeros((1, 32), np.uint16)
    inf[0, 5] = 0xFF80
    with pytest.raises(ValueError):
        oracle.mx_quantize(inf)
    with pytest.raises(ValueError):
        oracle.mx_dequantize(np.zeros((2, 64), np.uint8), np.zeros((2, 3), np.uint8))


def _case(rng, lens, d_in, d_out, r, E):
    T = int(sum(lens))
    x = to_bf16_bits(rng.standard_normal((T, d_in)))
    W = to_bf16_bits(rng.standard_normal((d_out, d_in)) / np.sqrt(d_in))
    A = to_bf16_bits(rng.standard_normal((E, r, d_in)) / np.sqrt(d_in))
    B = to_bf16_bits(rng.standard_normal((E, d_out, r)) / np.sqrt(r))
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ids = rng.integers(-1, E, size=len(lens)).astype(np.int32)
    return x, W, A, B, off, ids


def test_layer_against_numpy_on_independently_dequantised_operands():
    rng = np.random.default_rng(12)
    lens = [5, 0, 9, 1, 7]
    x, W, A, B, off, ids = _case(rng, lens, 96, 40, 16, 4)
    ids[0], ids[2] = 2, -1
    Wq, Ws = oracle.mx_quantize(W)
    y = oracle.lora_linear_mx(x, off, ids, Wq, Ws, A, B, 1.75)
    # dequantise with torch's value table and numpy powers of two
    def deq(c, s):
        return _torch_e4m3_values(c.ravel()).reshape(c.shape) * np.repeat(np.exp2(s.astype(np.float64) - 127), 32, axis=1)
    xq, xs = oracle.mx_quantize(x)
    base = deq(xq, xs) @ deq(Wq, Ws).T
    xf, Af, Bf = bits_to_f64(x), bits_to_f64(A), bits_to_f64(B)
    want = base.copy()
    for s, e in enumerate(ids):
        if e >= 0:
            rows = slice(off[s], off[s + 1])
            want[rows] += 1.75 * (xf[rows] @ Af[e].T) @ Bf[e].T
    assert np.allclose(y, want, rtol=1e-12, atol=1e-12)
    # the base really is the quantised one: it differs from the bf16 product by the
    # quantisation error, which is of relative size 2^-4 per operand at most
    plain = oracle.lora_linear(x, off, ids, W, A, B, 1.75)
    diff = np.abs(y - plain)
    assert diff.max() > 1e-3
    bound = 2 * 2.0 ** -4 * (np.abs(xf) @ np.abs(bits_to_f64(W)).T) * (1 + 2.0 ** -4)
    assert (diff <= bound + 1e-9).all()
    # rows= and rank_of_expert= select as in the unquantised layer
    sel = np.array([21, 0, 13], dtype=np.int64)
    assert np.array_equal(oracle.lora_linear_mx(x, off, ids, Wq, Ws, A, B, 1.75, rows=sel), y[sel])
    ranks = np.array([8, 0, 16, 8], dtype=np.int32)
    yr = oracle.lora_linear_mx(x, off, ids, Wq, Ws, A, B, 1.75, rank_of_expert=ranks)
    want_r = base.copy()
    for s, e in enumerate(ids):
        if e >= 0:
            rows = slice(off[s], off[s + 1])
            k = ranks[e]
            want_r[rows] += 1.75 * (xf[rows] @ Af[e, :k].T) @ Bf[e][:, :k].T
    assert np.allclose(yr, want_r, rtol=1e-12, atol=1e-12)


def test_layer_equals_the_unquantised_one_on_representable_operands():
    # small integers times one power of two per block survive the quantiser exactly, so the
    # quantised layer must return the bf16 layer's result
    rng = np.random.default_rng(13)
    lens = [4, 6]
    T, d_in, d_out, r, E = 10, 64, 24, 8, 3
    x = rng.integers(-7, 8, size=(T, d_in)).astype(np.float64)
    x[:, ::32] = 8                                            # every block has amax 8: 4-bit integers fit
    x *= np.exp2(rng.integers(-3, 4, size=(T, 1)))
    W = rng.integers(-7, 8, size=(d_out, d_in)).astype(np.float64)
    W[:, 5::32] = -8
    W *= 0.125
    xb, Wb = to_bf16_bits(x), to_bf16_bits(W)
    A = to_bf16_bits(rng.standard_normal((E, r, d_in)))
    B = to_bf16_bits(rng.standard_normal((E, d_out, r)))
    off = np.array([0, 4, 10], np.int32)
    ids = np.array([1, 2], np.int32)
    Wq, Ws = oracle.mx_quantize(Wb)
    assert np.array_equal(oracle.mx_dequantize(Wq, Ws), W)
    y = oracle.lora_linear_mx(xb, off, ids, Wq, Ws, A, B, 0.5)
    assert np.array_equal(y, oracle.lora_linear(xb, off, ids, Wb, A, B, 0.5))
