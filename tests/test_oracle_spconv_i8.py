"""Pins for the oracle's quantised sparse convolution.  The paper names model quantisation (Sec. 3.6 (2)) without
a scheme; the scheme is this build's own and is stated in the oracle: int8 operands, exact integer accumulation,
v = fl(fl(acc * mul) + add) per output channel in fp32 (unfused), optional ReLU, q = clamp(rint(v / s), +-127).

Expected values come from torch's dense conv3d in fp64 on the integer-valued grid (exact there), from numpy
float32 arithmetic for the epilogue, from exact rational arithmetic for the roundings, and from hand cases."""
from fractions import Fraction

import numpy as np
import torch

import oracle
from paper_2507_04123_amd import gen
from test_oracle_kmap import _random_coords
from test_oracle_spconv import _dense_conv


def _rand_i8(seed, shape, lim=127):
    b = gen.Stream(seed, 21).bits(int(np.prod(shape)))
    return ((b % np.uint64(2 * lim + 1)).astype(np.int64) - lim).astype(np.int8).reshape(shape)


def test_quantize_hand_cases_and_numpy():
    x = np.array([0.0, 0.49, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5, 127.4, 127.5, 1e9, -1e9, np.inf, -np.inf, np.nan], np.float32)
    assert oracle.quantize_i8(x, 1.0).tolist() == [0, 0, 0, 2, 2, 0, -2, -2, 126, 127, 127, 127, -127, 127, -127, 0]
    assert oracle.quantize_i8(np.array([1.0, -3.0, 0.26], np.float32), 4.0).tolist() == [4, -12, 1]      # x * inv_scale
    v = gen.Stream(3, 3).normal(20000, 2.0).astype(np.float32)
    inv = np.float32(1.0 / 0.037)
    exp = np.clip(np.rint(v * inv), -127, 127).astype(np.int8)          # float32 product, ties to even
    assert np.array_equal(oracle.quantize_i8(v, inv), exp)
    assert (np.abs(exp) == 127).any() and (exp == 0).any()


def test_integer_accumulation_equals_dense_conv():
    """With mul = 1, add = 0 the float result is the integer accumulator converted to fp32: torch's fp64 dense
    convolution of the same integer-valued grid is exact, so equality is exact."""
    grid, nb, cin, cout = (9, 8, 6), 2, 8, 6
    coords = _random_coords(1, grid, nb, 260)
    xq = _rand_i8(2, (len(coords), cin))
    wq = _rand_i8(3, (27, cin, cout))
    one, zero = np.ones(cout, np.float32), np.zeros(cout, np.float32)
    for kind, stride in ((0, 1), (1, 2)):
        out_c, nbr, gout = oracle.build_kmap(kind, coords, grid, nb)
        v = oracle.spconv_i8(xq, wq, one, zero, False, nbr)
        dense = _dense_conv(coords, xq.astype(np.float32), wq.astype(np.float32), grid, nb, stride)
        c = out_c.astype(np.int64)
        exp = dense[c[:, 0], :, c[:, 1], c[:, 2], c[:, 3]].numpy()
        assert np.abs(exp).max() > 1e5 and np.abs(exp).max() < 2 ** 24      # large, still exactly representable in fp32
        assert np.array_equal(v.astype(np.float64), exp)
        # the same through the fp64 oracle conv (pinned on its own against conv3d)
        assert np.array_equal(v, oracle.spconv(xq.astype(np.float32), wq.astype(np.float32), None, None, 0, nbr))
    # an asymmetric single tap, by hand: out[o] = x[nbr[k0][o]] @ w[k0]
    _, nbr, _ = oracle.build_kmap(0, coords, grid, nb)
    k0 = 2 * 9 + 0 * 3 + 1
    w1 = np.zeros_like(wq); w1[k0] = wq[k0]
    v1 = oracle.spconv_i8(xq, w1, one, zero, False, nbr)
    for o in range(0, len(coords), 7):
        j = nbr[k0, o]
        want = xq[j].astype(np.int64) @ wq[k0].astype(np.int64) if j >= 0 else np.zeros(cout, np.int64)
        assert np.array_equal(v1[o].astype(np.int64), want)


def test_epilogue_is_unfused_fp32_and_requantises():
    grid, nb, cin, cout = (8, 8, 5), 1, 16, 12
    coords = _random_coords(5, grid, nb, 200)
    xq = _rand_i8(6, (len(coords), cin))
    wq = _rand_i8(7, (27, cin, cout), 40)
    _, nbr, _ = oracle.build_kmap(0, coords, grid, nb)
    st = gen.Stream(8, 8)
    mul = (st.uniform(cout, 0.5, 1.5) * 1e-4).astype(np.float32)
    add = st.uniform(cout, -1.0, 1.0).astype(np.float32)
    acc = oracle.spconv_i8(xq, wq, np.ones(cout, np.float32), np.zeros(cout, np.float32), False, nbr).astype(np.float32)
    assert np.abs(acc).max() < 2 ** 24
    inv_s = np.float32(1.0 / 0.05)
    for relu in (False, True):
        v, q = oracle.spconv_i8(xq, wq, mul, add, relu, nbr, inv_out_scale=inv_s)
        exp = acc * mul + add                                          # numpy float32: product and sum rounded separately
        if relu:
            exp = np.maximum(exp, np.float32(0))
        assert exp.dtype == np.float32 and np.array_equal(v, exp)
        assert np.array_equal(q, np.clip(np.rint(v * inv_s), -127, 127).astype(np.int8))
        assert (np.abs(q) == 127).any() and (q == 0).any() and (relu == bool((q >= 0).all()))
    # exact rational check of the two roundings on a sample, and proof that the fused form would differ somewhere
    v = oracle.spconv_i8(xq, wq, mul, add, False, nbr)
    fused_differs = 0
    for o in range(0, len(coords), 3):
        for c in range(cout):
            a, m, b = Fraction(float(acc[o, c])), Fraction(float(mul[c])), Fraction(float(add[c]))
            p = np.float32(float(a * m))                                # Fraction -> double is exact enough to round once more:
            assert Fraction(float(p)) == Fraction(float(np.float32(np.float64(acc[o, c]) * np.float64(mul[c]))))
            unfused = np.float32(np.float64(p) + np.float64(add[c]))    # |p|, |add| < 2^12 and 24-bit: the fp64 sum is exact
            assert v[o, c] == unfused
            fused = np.float32(float(a * m + b))
            fused_differs += int(fused != unfused)
    assert fused_differs > 0


def test_relu_and_empty_and_errors():
    nbr = -np.ones((27, 3), np.int32)
    nbr[13, 0] = 0; nbr[13, 1] = 1
    xq = np.array([[1, -2], [3, 4]], np.int8)
    wq = np.zeros((27, 2, 2), np.int8); wq[13] = [[1, 2], [3, -4]]
    v, q = oracle.spconv_i8(xq, wq, np.array([0.5, 0.25], np.float32), np.array([1.0, -1.0], np.float32), True, nbr, inv_out_scale=2.0)
    # acc = [[1-6, 2+8], [3+12, 6-16], [0, 0]] = [[-5, 10], [15, -10], [0, 0]] -> v = relu(acc * mul + add)
    assert v.tolist() == [[0.0, 1.5], [8.5, 0.0], [1.0, 0.0]]
    assert q.tolist() == [[0, 3], [17, 0], [2, 0]]
    import pytest
    bad = nbr.copy(); bad[0, 0] = 5
    with pytest.raises(RuntimeError):
        oracle.spconv_i8(xq, wq, np.ones(2, np.float32), np.zeros(2, np.float32), False, bad)
    v0 = oracle.spconv_i8(xq, wq, np.ones(2, np.float32), np.zeros(2, np.float32), False, np.zeros((27, 0), np.int32))
    assert v0.shape == (0, 2)
