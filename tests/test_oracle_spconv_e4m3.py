"""Pins for the oracle's 8-bit floating-point (E4M3) sparse convolution.  The paper names model quantisation
(Sec. 3.6 (2)) without a scheme; the scheme is this build's own and is stated in the oracle: E4M3 operands (no
infinities, bias 7, largest value 448), exact accumulation of the exact products, one rounding to fp32, then
v = fl(fl(acc * mul) + add) per output channel (unfused), optional ReLU.

Expected values come from the format's definition written out by hand, from torch's float8_e4m3fn storage type as a
library decoder / in-range encoder, from exact rational arithmetic for the roundings, and from torch's dense conv3d
in fp64 on the decoded grid (exact there)."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2507_04123_amd import gen
from test_oracle_kmap import _random_coords
from test_oracle_spconv import _dense_conv


def test_code_values_by_hand_and_against_the_library_type():
    v = oracle.e4m3_value
    assert v(0x00) == 0.0 and v(0x80) == 0.0
    assert v(0x38) == 1.0 and v(0xB8) == -1.0 and v(0x3C) == 1.5 and v(0x40) == 2.0
    assert v(0x01) == 2.0 ** -9 and v(0x07) == 7 * 2.0 ** -9 and v(0x08) == 2.0 ** -6      # subnormals, then the first normal
    assert v(0x7E) == 448.0 and v(0xFE) == -448.0
    assert np.isnan(v(0x7F)) and np.isnan(v(0xFF))
    # the format's formula for every code
    for c in range(256):
        s, e, m = c >> 7, (c >> 3) & 15, c & 7
        if e == 15 and m == 7:
            continue
        want = Fraction(2) ** (e - 7) * (1 + Fraction(m, 8)) if e else Fraction(2) ** -6 * Fraction(m, 8)
        assert Fraction(v(c)) == (-want if s else want)
    # torch's storage type decodes the same bytes to the same numbers
    codes = torch.arange(256, dtype=torch.uint8)
    lib = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    mine = np.array([v(c) for c in range(256)])
    ok = ~np.isnan(mine)
    assert np.array_equal(np.isnan(lib), ~ok) and np.array_equal(lib[ok], mine[ok])


def _nearest_even_rational(t: Fraction) -> int:
    """Nearest finite code to the rational t, ties to the even code, by exact comparison of distances."""
    vals = [Fraction(oracle.e4m3_value(c)) for c in range(0x7F)]
    a = abs(t)
    best = min(range(0x7F), key=lambda c: (abs(a - vals[c]), c & 1))
    return 0 if best == 0 else best | (0x80 if t < 0 else 0)


def test_quantizer_roundings_saturation_and_library_agreement():
    q = lambda xs, inv=1.0: oracle.quantize_e4m3(np.array(xs, np.float32), inv).tolist()
    assert q([0.0, -0.0, 1.0, -1.0, 448.0, 449.0, 1e9, -1e9, np.inf, -np.inf, np.nan]) == \
        [0x00, 0x00, 0x38, 0xB8, 0x7E, 0x7E, 0x7E, 0xFE, 0x7E, 0xFE, 0x00]
    # ties: halfway between 1.0 (0x38, even) and 1.125 (0x39) goes down; between 1.125 and 1.25 (0x3A, even) goes up
    assert q([1.0625, 1.1875, -1.0625]) == [0x38, 0x3A, 0xB8]
    # halfway between 0 and the smallest subnormal goes to 0 (even); just above goes up; the scale multiplies first
    assert q([2.0 ** -10, 2.0 ** -10 * 1.0001, 2.0 ** -12], 1.0) == [0x00, 0x01, 0x00]
    assert q([0.25], 4.0) == [0x38]
    # between 448 and the next value the format would have (480): everything saturates, nothing becomes a non-number
    assert q([464.0, 479.0, 480.0]) == [0x7E, 0x7E, 0x7E]
    # exact rational check on seeded values, incl. the fp32 rounding of the product
    st = gen.Stream(8, 8)
    xs = (st.normal(400, 30.0)).astype(np.float32)
    inv = np.float32(0.37)
    got = oracle.quantize_e4m3(xs, inv)
    for x, g in zip(xs, got):
        t = Fraction(float(np.float32(x) * inv))          # numpy float32 product: one rounding
        assert g == _nearest_even_rational(t), (x, g)
    # the library's cast agrees wherever the scaled value is inside the finite range
    big = (st.normal(20000, 60.0)).astype(np.float32)
    inside = np.abs(big) <= 448.0
    lib = torch.from_numpy(big[inside]).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    mine = oracle.quantize_e4m3(big[inside], 1.0)
    lib = np.where(lib == 0x80, 0, lib)                  # the library keeps the sign of a value that rounds to zero
    assert np.array_equal(lib, mine)


def _rand_codes(seed, shape, top=0x5F):
    """Random finite codes of both signs with magnitudes up to the code `top` (0x5F = 30)."""
    b = gen.Stream(seed, 23).bits(2 * int(np.prod(shape))).reshape(2, -1)
    mag = (b[0] % np.uint64(top + 1)).astype(np.uint8)
    sign = ((b[1] & np.uint64(1)) << np.uint64(7)).astype(np.uint8)
    c = (mag | sign).reshape(shape)
    return np.where(c == 0x80, 0, c).astype(np.uint8)


def _decode(codes):
    return np.vectorize(oracle.e4m3_value)(codes).astype(np.float64)


def test_exact_accumulation_equals_dense_conv():
    """With mul = 1, add = 0 the result is the exact sum of products rounded once to fp32: torch's fp64 dense
    convolution of the decoded grid is exact for these magnitudes, so the comparison is exact."""
    grid, nb, cin, cout = (9, 8, 6), 2, 8, 6
    coords = _random_coords(1, grid, nb, 260)
    xq = _rand_codes(2, (len(coords), cin))
    wq = _rand_codes(3, (27, cin, cout))
    x, w = _decode(xq), _decode(wq)
    one, zero = np.ones(cout, np.float32), np.zeros(cout, np.float32)
    for kind, stride in ((0, 1), (1, 2)):
        out_c, nbr, _ = oracle.build_kmap(kind, coords, grid, nb)
        v = oracle.spconv_e4m3(xq, wq, one, zero, False, nbr)
        dense = _dense_conv(coords, x, w, grid, nb, stride)
        c = out_c.astype(np.int64)
        exp = dense[c[:, 0], :, c[:, 1], c[:, 2], c[:, 3]].numpy()
        assert np.abs(exp).max() > 100
        assert np.array_equal(v, exp.astype(np.float32))
        # the same through the fp64 oracle conv on the decoded values (pinned on its own against conv3d)
        assert np.array_equal(v, oracle.spconv(x.astype(np.float32), w.astype(np.float32), None, None, 0, nbr))
    # an asymmetric single tap, by hand, in exact rationals
    _, nbr, _ = oracle.build_kmap(0, coords, grid, nb)
    k0 = 2 * 9 + 0 * 3 + 1
    w1 = np.zeros_like(wq); w1[k0] = wq[k0]
    v1 = oracle.spconv_e4m3(xq, w1, one, zero, False, nbr)
    for o in range(0, len(coords), 11):
        j = nbr[k0, o]
        for d in range(cout):
            want = sum(Fraction(x[j, ch]) * Fraction(w[k0, ch, d]) for ch in range(cin)) if j >= 0 else Fraction(0)
            assert float(want) == want                          # a dyadic rational well inside fp64: float() is exact
            assert v1[o, d] == np.float32(float(want))          # so this is the exact sum rounded once to fp32


def test_epilogue_is_unfused_fp32_and_relu():
    grid, nb, cin, cout = (7, 7, 5), 1, 16, 8
    coords = _random_coords(5, grid, nb, 150)
    xq, wq = _rand_codes(6, (len(coords), cin)), _rand_codes(7, (27, cin, cout))
    _, nbr, _ = oracle.build_kmap(0, coords, grid, nb)
    st = gen.Stream(9, 9)
    mul = st.uniform(cout, 1e-3, 3e-3).astype(np.float32)
    add = st.uniform(cout, -0.5, 0.5).astype(np.float32)
    acc = oracle.spconv_e4m3(xq, wq, np.ones(cout, np.float32), np.zeros(cout, np.float32), False, nbr)
    v = oracle.spconv_e4m3(xq, wq, mul, add, False, nbr)
    exp = (acc * mul[None, :]).astype(np.float32) + add[None, :]          # numpy float32: product and sum rounded separately
    assert np.array_equal(v, exp.astype(np.float32))
    fused = (acc.astype(np.float64) * mul[None, :].astype(np.float64) + add[None, :]).astype(np.float32)
    assert (fused != v).any()                                              # the fused form differs somewhere on this data
    r = oracle.spconv_e4m3(xq, wq, mul, add, True, nbr)
    assert np.array_equal(r, np.maximum(v, 0.0)) and (v < 0).any()
    # codes that are not numbers are refused
    bad = xq.copy(); bad[3, 2] = 0x7F
    with pytest.raises(RuntimeError):
        oracle.spconv_e4m3(bad, wq, mul, add, False, nbr)
