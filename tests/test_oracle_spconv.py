"""Pins for the oracle's sparse convolution and epilogue (paper Sec. 3.5: conv over the N non-empty
voxels only, cost O(N x C_v); Sec. 3.6 graph fusion -> fused affine + ReLU).  The library special
case is torch's dense conv3d (CPU, fp64) on the densified grid."""
import numpy as np
import torch

import oracle
from paper_2507_04123_amd import gen
from test_oracle_kmap import _random_coords


def _dense_conv(coords, feats, w, grid, nb, stride):
    """Scatter into a dense zero grid and run torch conv3d (cross-correlation, padding 1)."""
    gx, gy, gz = grid
    cin, cout = w.shape[1], w.shape[2]
    dense = torch.zeros((nb, cin, gz, gy, gx), dtype=torch.float64)
    c = torch.from_numpy(coords.astype(np.int64))
    dense[c[:, 0], :, c[:, 1], c[:, 2], c[:, 3]] = torch.from_numpy(feats.astype(np.float64))
    # W[(kz*3+ky)*3+kx][c][d] -> weight[d][c][kz][ky][kx]
    wt = torch.from_numpy(w.astype(np.float64)).reshape(3, 3, 3, cin, cout).permute(4, 3, 0, 1, 2).contiguous()
    return torch.nn.functional.conv3d(dense, wt, bias=None, stride=stride, padding=1)


def _rand(seed, shape, sigma=1.0):
    return gen.Stream(seed, 11).normal(int(np.prod(shape)), sigma).astype(np.float32).reshape(shape)


def test_subm_equals_dense_conv_masked_to_active_sites():
    grid, nb, cin, cout = (9, 8, 6), 2, 5, 7
    coords = _random_coords(1, grid, nb, 260)
    x = _rand(2, (len(coords), cin))
    w = _rand(3, (27, cin, cout), 0.1)
    _, nbr, _ = oracle.build_kmap(0, coords, grid, nb)
    y, macs = oracle.spconv(x, w, None, None, 0, nbr, return_macs=True)
    dense = _dense_conv(coords, x, w, grid, nb, 1)
    c = coords.astype(np.int64)
    exp = dense[c[:, 0], :, c[:, 1], c[:, 2], c[:, 3]].numpy()
    np.testing.assert_allclose(y, exp, rtol=1e-6, atol=1e-7)
    assert macs == int((nbr >= 0).sum()) * cin * cout                  # work ~ non-empty voxels only


def test_strided_equals_dense_conv_and_is_zero_elsewhere():
    for grid in [(9, 8, 6), (10, 7, 5)]:
        nb, cin, cout = 2, 4, 6
        coords = _random_coords(4, grid, nb, 90)
        x = _rand(5, (len(coords), cin))
        w = _rand(6, (27, cin, cout), 0.1)
        out, nbr, gout = oracle.build_kmap(1, coords, grid, nb)
        y = oracle.spconv(x, w, None, None, 0, nbr)
        dense = _dense_conv(coords, x, w, grid, nb, 2)
        assert tuple(dense.shape[2:]) == (gout[2], gout[1], gout[0])
        c = out.astype(np.int64)
        exp = dense[c[:, 0], :, c[:, 1], c[:, 2], c[:, 3]].numpy()
        np.testing.assert_allclose(y, exp, rtol=1e-6, atol=1e-7)
        mask = torch.ones((nb, gout[2], gout[1], gout[0]), dtype=torch.bool)
        mask[c[:, 0], c[:, 1], c[:, 2], c[:, 3]] = False
        assert float(dense.permute(0, 2, 3, 4, 1)[mask].abs().max()) == 0.0   # inactive outputs are exactly 0


def test_fully_active_grid_equals_dense_everywhere_and_mac_count():
    g, cin, cout = 4, 3, 2
    coords = np.array([(0, z, y, x) for z in range(g) for y in range(g) for x in range(g)], np.int32)
    x = _rand(7, (len(coords), cin))
    w = _rand(8, (27, cin, cout))
    _, nbr, _ = oracle.build_kmap(0, coords, (g, g, g), 1)
    y, macs = oracle.spconv(x, w, None, None, 0, nbr, return_macs=True)
    dense = _dense_conv(coords, x, w, (g, g, g), 1, 1)[0].permute(1, 2, 3, 0).reshape(-1, cout).numpy()
    np.testing.assert_allclose(y, dense, rtol=1e-6, atol=1e-7)
    # dense MAC count: per axis sum over sites of in-range taps = 3g - 2
    assert macs == (3 * g - 2) ** 3 * cin * cout


def test_single_voxel_centre_tap_and_asymmetric_tap():
    cin, cout = 3, 4
    x = _rand(9, (1, cin))
    w = np.zeros((27, cin, cout), np.float32)
    w[13] = _rand(10, (cin, cout))
    nbr = -np.ones((27, 1), np.int32); nbr[13, 0] = 0
    y = oracle.spconv(x, w, None, None, 0, nbr)
    np.testing.assert_allclose(y[0], x[0].astype(np.float64) @ w[13].astype(np.float64), rtol=1e-6)
    # two sites along +x: tap kx=2 (k=14) of site 0 must read site 1, not the other way round
    coords = np.array([(0, 2, 2, 2), (0, 2, 2, 3)], np.int32)
    _, nbr2, _ = oracle.build_kmap(0, coords, (6, 6, 6), 1)
    w2 = np.zeros((27, 1, 1), np.float32); w2[14, 0, 0] = 1.0
    y2 = oracle.spconv(np.array([[10.0], [20.0]], np.float32), w2, None, None, 0, nbr2)
    assert y2[:, 0].tolist() == [20.0, 0.0]


def test_linearity_and_epilogues():
    grid, nb, cin, cout = (8, 8, 4), 1, 4, 5
    coords = _random_coords(11, grid, nb, 120)
    _, nbr, _ = oracle.build_kmap(0, coords, grid, nb)
    xa, xb = _rand(12, (len(coords), cin)), _rand(13, (len(coords), cin))
    w = _rand(14, (27, cin, cout), 0.1)
    ya = oracle.spconv(xa, w, None, None, 0, nbr).astype(np.float64)
    yb = oracle.spconv(xb, w, None, None, 0, nbr).astype(np.float64)
    yab = oracle.spconv((2 * xa + xb).astype(np.float32), w, None, None, 0, nbr)
    np.testing.assert_allclose(yab, 2 * ya + yb, rtol=1e-5, atol=1e-5)
    one, zero = np.ones(cout, np.float32), np.zeros(cout, np.float32)
    assert np.array_equal(oracle.spconv(xa, w, one, zero, 1, nbr), ya.astype(np.float32))
    assert np.array_equal(oracle.spconv(xa, w, one, zero, 2, nbr), np.maximum(ya, 0).astype(np.float32))
    sc = gen.Stream(15).uniform(cout, 0.5, 2.0).astype(np.float32)
    sh = gen.Stream(16).uniform(cout, -1.0, 1.0).astype(np.float32)
    y1 = oracle.spconv(xa, w, sc, sh, 1, nbr)
    np.testing.assert_allclose(y1, ya * sc + sh, rtol=1e-6, atol=1e-6)
    y2 = oracle.spconv(xa, w, sc, sh, 2, nbr)
    np.testing.assert_allclose(y2, np.maximum(ya * sc + sh, 0), rtol=1e-6, atol=1e-6)
    assert (y2 == 0).any() and (y2 > 0).any()


def test_empty_conv():
    y = oracle.spconv(np.zeros((0, 4), np.float32), np.zeros((27, 4, 8), np.float32), None, None, 0,
                      np.zeros((27, 0), np.int32))
    assert y.shape == (0, 8)
