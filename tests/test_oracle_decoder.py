"""Pins for the oracle's decoder-side pieces: the inverse (transposed) kernel map of a stride-2 layer
(paper Sec. 3.1: the LiDAR branch is a UNet plus a sparse CNN, so features come back up the levels) and
the bird's-eye-view flattening (Sec. 3.3: the latency-prioritised expert works on BEV projections).

Expected values come from coordinate arithmetic on the sites themselves (independent of the stride-2
map the oracle inverts), from torch's dense transposed convolution in fp64, and from closed forms."""
import numpy as np
import pytest
import torch

import oracle
from paper_2507_04123_amd import gen

TAPS = [(kx, ky, kz) for kz in range(3) for ky in range(3) for kx in range(3)]   # k = (kz*3+ky)*3+kx


def _random_coords(seed, grid, n_batch, n):
    gx, gy, gz = grid
    total = gx * gy * gz * n_batch
    st = gen.Stream(seed, 3)
    keys = np.unique((st.bits(3 * n) % np.uint64(total)).astype(np.int64))[:n]
    keys.sort()
    x = keys % gx; y = (keys // gx) % gy; z = (keys // (gx * gy)) % gz; b = keys // (gx * gy * gz)
    return np.stack([b, z, y, x], axis=1).astype(np.int32)


def _inverse_by_geometry(fine, coarse):
    """Fine site i is read by coarse site j at tap k iff i = 2j - 1 + k on every axis, i.e. j = (i + 1 - k)/2
    with an even numerator: looked up in a dictionary of coarse coordinates, never touching the down map."""
    lut = {tuple(c): j for j, c in enumerate(coarse.tolist())}
    inv = -np.ones((27, len(fine)), np.int32)
    for i, (b, z, y, x) in enumerate(fine.tolist()):
        for k, (kx, ky, kz) in enumerate(TAPS):
            tx, ty, tz = x + 1 - kx, y + 1 - ky, z + 1 - kz
            if tx % 2 or ty % 2 or tz % 2 or tx < 0 or ty < 0 or tz < 0:
                continue
            inv[k, i] = lut.get((b, tz // 2, ty // 2, tx // 2), -1)
    return inv


@pytest.mark.parametrize("grid,nb,n", [((12, 9, 7), 2, 400), ((8, 8, 8), 1, 300), ((5, 4, 3), 3, 60), ((16, 3, 1), 1, 20)])
def test_inverse_map_matches_coordinate_arithmetic(grid, nb, n):
    fine = _random_coords(11 + n, grid, nb, n)
    coarse, down, gout = oracle.build_kmap(1, fine, grid, nb)
    inv = oracle.invert_kmap(down, len(fine))
    assert np.array_equal(inv, _inverse_by_geometry(fine, coarse))
    # the same pairs, seen from the other side: count and round trip
    assert int((inv >= 0).sum()) == int((down >= 0).sum())
    ks, js = np.nonzero(down >= 0)
    assert np.array_equal(inv[ks, down[ks, js]], js.astype(np.int32))
    ks, is_ = np.nonzero(inv >= 0)
    assert np.array_equal(down[ks, inv[ks, is_]], is_.astype(np.int32))
    # every fine site is covered by at least one tap (the coarse level exists because of it) and by at most 8
    per_site = (inv >= 0).sum(axis=0)
    assert per_site.min() >= 1 and per_site.max() <= 8
    # closed form by parity: i + 1 - k is even on an axis iff k = 1 (i even) or k in {0, 2} (i odd)
    odd = np.all(fine[:, 1:] % 2 == 1, axis=1)
    even = np.all(fine[:, 1:] % 2 == 0, axis=1)
    centre = (1 * 3 + 1) * 3 + 1
    # even coordinates: i + 1 - k even only for k = 1 on every axis -> exactly the centre tap
    assert np.all(per_site[even] == 1) and np.all(inv[centre, even] >= 0)
    # odd coordinates: k in {0, 2} per axis -> never the centre tap
    assert np.all(inv[centre, odd] == -1)


def test_inverse_map_rejects_inconsistent_tables():
    down = -np.ones((27, 3), np.int32)
    down[4, 0] = 1
    down[4, 2] = 1                          # two coarse sites claim fine site 1 at the same tap
    with pytest.raises(RuntimeError):
        oracle.invert_kmap(down, 5)
    down[4, 2] = 7                          # names a fine site that does not exist
    with pytest.raises(RuntimeError):
        oracle.invert_kmap(down, 5)
    assert oracle.invert_kmap(-np.ones((27, 0), np.int32), 4).shape == (27, 4)


@pytest.mark.parametrize("grid", [(9, 7, 5), (8, 6, 4), (7, 8, 5)])
def test_transposed_conv_matches_torch_conv_transpose3d(grid):
    """conv over the inverse map == dense transposed convolution (stride 2, padding 1, output padding chosen to
    land on the fine grid) of the coarse features, read at the fine sites.  Inactive coarse sites hold zeros, so
    they contribute nothing either way."""
    gx, gy, gz = grid
    cin, cout = 3, 5
    fine = _random_coords(77, grid, 1, 150)
    coarse, down, gout = oracle.build_kmap(1, fine, grid, 1)
    inv = oracle.invert_kmap(down, len(fine))
    st = gen.Stream(5, 5)
    xc = st.normal(len(coarse) * cin).astype(np.float32).reshape(-1, cin)
    w = st.normal(27 * cin * cout, 0.3).astype(np.float32).reshape(27, cin, cout)
    y = oracle.spconv(xc, w, None, None, 0, inv)
    dense = torch.zeros((1, cin, gout[2], gout[1], gout[0]), dtype=torch.float64)
    for j, (b, z, yy, x) in enumerate(coarse.tolist()):
        dense[0, :, z, yy, x] = torch.from_numpy(xc[j].astype(np.float64))
    wt = torch.from_numpy(w.astype(np.float64)).reshape(3, 3, 3, cin, cout).permute(3, 4, 0, 1, 2).contiguous()
    op = tuple(g - (2 * go - 1) for g, go in zip((gz, gy, gx), (gout[2], gout[1], gout[0])))
    assert all(o in (0, 1) for o in op)
    up = torch.nn.functional.conv_transpose3d(dense, wt, stride=2, padding=1, output_padding=op)
    assert tuple(up.shape[2:]) == (gz, gy, gx)
    exp = np.stack([up[0, :, z, yy, x].numpy() for (b, z, yy, x) in fine.tolist()])
    assert np.allclose(y, exp, rtol=1e-6, atol=1e-6)
    # an asymmetric single tap: only W[k0] non-zero -> each fine site receives exactly its parent's row times W[k0]
    k0 = 2 * 9 + 0 * 3 + 1
    w1 = np.zeros_like(w); w1[k0] = w[k0]
    y1 = oracle.spconv(xc, w1, None, None, 0, inv)
    for i in range(len(fine)):
        j = inv[k0, i]
        want = xc[j].astype(np.float64) @ w[k0].astype(np.float64) if j >= 0 else np.zeros(cout)
        assert np.allclose(y1[i], want, rtol=1e-6, atol=1e-7)


def test_bev_flatten_against_indexing_and_closed_forms():
    grid, nb, c = (7, 5, 3), 2, 4
    coords = _random_coords(3, grid, nb, 90)
    st = gen.Stream(8, 1)
    feats = st.normal(len(coords) * c).astype(np.float32).reshape(-1, c)
    out = oracle.bev_flatten(coords, feats, grid, nb)
    assert out.shape == (nb, grid[1], grid[0], grid[2] * c) and out.dtype == np.float32
    # numpy advanced indexing: an independent scatter
    exp = np.zeros((nb, grid[1], grid[0], grid[2], c), np.float32)
    exp[coords[:, 0], coords[:, 2], coords[:, 3], coords[:, 1]] = feats
    assert np.array_equal(out, exp.reshape(out.shape))
    # nothing invented, nothing lost
    assert int((out != 0).sum()) == int((feats != 0).sum())
    assert np.isclose(out.astype(np.float64).sum(), feats.astype(np.float64).sum())
    # one hand-placed voxel: (b, z, y, x) = (1, 2, 3, 4), channel 1 -> out[1][3][4][2*C + 1]
    one = oracle.bev_flatten(np.array([[1, 2, 3, 4]], np.int32), np.array([[10., 11., 12., 13.]], np.float32), grid, nb)
    assert one[1, 3, 4, 2 * c + 1] == 11.0 and float(np.abs(one).sum()) == 46.0
    # z is the slow index of the collapsed channel axis: the same column, two heights
    two = oracle.bev_flatten(np.array([[0, 0, 1, 1], [0, 2, 1, 1]], np.int32), np.array([[1, 2, 3, 4], [5, 6, 7, 8]], np.float32), grid, 1)
    assert np.array_equal(two[0, 1, 1], np.array([1, 2, 3, 4, 0, 0, 0, 0, 5, 6, 7, 8], np.float32))
    # empty set -> all zeros
    assert not oracle.bev_flatten(np.zeros((0, 4), np.int32), np.zeros((0, c), np.float32), grid, nb).any()


def test_bev_flatten_rejects_bad_input():
    grid = (4, 4, 2)
    f = np.ones((2, 3), np.float32)
    with pytest.raises(RuntimeError):
        oracle.bev_flatten(np.array([[0, 0, 1, 1], [0, 0, 1, 1]], np.int32), f, grid, 1)      # two voxels in one cell
    with pytest.raises(RuntimeError):
        oracle.bev_flatten(np.array([[0, 2, 1, 1], [0, 0, 0, 0]], np.int32), f, grid, 1)      # z outside the grid
    with pytest.raises(RuntimeError):
        oracle.bev_flatten(np.array([[1, 0, 1, 1], [0, 0, 0, 0]], np.int32), f, grid, 1)      # frame id outside
