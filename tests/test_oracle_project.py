"""Pins for the oracle's point -> image projection with bilinear gather (paper Sec. 3.1: image
features are aligned with 3D positions; Fig. 5 caption: unmatched sites get zero-filled features).
Expectations are closed forms: integer-pixel hits, an affine feature map, an identity camera."""
import numpy as np

import oracle
from paper_2507_04123_amd import gen


def test_identity_camera_closed_form_and_integer_pixel_hits():
    h, w, c = 7, 9, 3
    img = gen.Stream(1).normal(h * w * c).astype(np.float16).reshape(h, w, c)
    pm = np.array([1, 0, 0, 0, 0, 1, 0, 0, 0, 0, 1, 0], np.float32)       # u = x/z, v = y/z
    pts = np.array([[6.0, 4.0, 2.0, 0], [8.0, 6.0, 1.0, 0], [0.0, 0.0, 5.0, 0], [4.0, 12.0, 2.0, 0]], np.float32)
    g, valid, uv = oracle.project_gather(pts, pm, img, want_uv=True)
    assert valid.tolist() == [1, 1, 1, 1]
    assert uv.tolist() == [[3.0, 2.0], [8.0, 6.0], [0.0, 0.0], [2.0, 6.0]]
    for i, (col, row) in enumerate([(3, 2), (8, 6), (0, 0), (2, 6)]):     # includes last row / last col
        assert np.array_equal(g[i], img[row, col].astype(np.float32))


def test_affine_feature_map_is_reproduced():
    h, w = 11, 13
    jj, ii = np.meshgrid(np.arange(h), np.arange(w), indexing="ij")
    img = np.stack([0.5 * ii + 0.25 * jj + 1.0, -0.125 * ii + 2.0 * jj, np.full_like(ii, 3.0, dtype=float)],
                   axis=2).astype(np.float16)                                # exact in fp16
    # general pinhole with a translation: u = 6 - 20 y / (x + 0.1), v = 5 - 20 z / (x + 0.1)
    pm2 = np.array([6.0, -20.0, 0.0, 0.6, 5.0, 0.0, -20.0, 0.5, 1.0, 0.0, 0.0, 0.1], np.float32)
    st = gen.Stream(4)
    pts = np.stack([st.uniform(400, 2, 30), st.uniform(400, -3, 3), st.uniform(400, -2, 2),
                    st.uniform(400)], axis=1).astype(np.float32)
    g, valid, uv = oracle.project_gather(pts, pm2, img, want_uv=True)
    assert (valid == 0).sum() > 20
    assert valid.sum() > 50
    u, v = uv[valid == 1, 0], uv[valid == 1, 1]
    exp = np.stack([0.5 * u + 0.25 * v + 1.0, -0.125 * u + 2.0 * v, np.full_like(u, 3.0)], axis=1)
    np.testing.assert_allclose(g[valid == 1], exp, rtol=1e-6, atol=1e-6)


def test_uv_matches_exact_projection_and_row_col_are_not_swapped():
    pm = gen.make_camera(5)
    pts = np.array([[10.0, 1.0, -0.5, 0.3]], np.float32)
    h, w, c = 375, 1242, 2
    img = np.zeros((h, w, c), np.float16)
    _, valid, uv = oracle.project_gather(pts, pm, img, want_uv=True)
    p = pm.astype(np.float64).reshape(3, 4) @ np.array([10.0, 1.0, -0.5, 1.0])
    np.testing.assert_allclose(uv[0], [p[0] / p[2], p[1] / p[2]], rtol=1e-14)
    assert valid[0] == 1 and 0 <= uv[0, 0] <= w - 1 and 0 <= uv[0, 1] <= h - 1
    # a single hot pixel: only points whose (u, v) is within one pixel of (col, row) see it
    col, row = int(np.floor(uv[0, 0])), int(np.floor(uv[0, 1]))
    assert col != row
    img[row, col, 0] = 1.0
    g, _ = oracle.project_gather(pts, pm, img)
    a, b = uv[0, 0] - col, uv[0, 1] - row
    np.testing.assert_allclose(g[0, 0], (1 - a) * (1 - b), rtol=1e-6)
    assert g[0, 1] == 0.0


def test_behind_camera_and_off_image_are_zero_filled():
    h, w, c = 5, 6, 4
    img = np.ones((h, w, c), np.float16)
    pm = np.array([1, 0, 0, 0, 0, 1, 0, 0, 0, 0, 1, 0], np.float32)
    pts = np.array([
        [1.0, 1.0, -1.0, 0],      # behind the camera (w < 0)
        [1.0, 1.0, 0.0, 0],       # w == 0
        [6.0, 1.0, 1.0, 0],       # u = 6 > W-1 = 5
        [5.0, 4.0, 1.0, 0],       # exactly on the last pixel: valid
        [-0.001, 1.0, 1.0, 0],    # u < 0
        [1.0, 4.001, 1.0, 0],     # v > H-1
        [float("nan"), 1.0, 1.0, 0],
        [2.5, 1.5, 1.0, 0],       # interior
    ], np.float32)
    g, valid = oracle.project_gather(pts, pm, img)
    assert valid.tolist() == [0, 0, 0, 1, 0, 0, 0, 1]
    assert np.all(g[valid == 0] == 0.0)
    np.testing.assert_allclose(g[valid == 1], 1.0, rtol=1e-7)              # weights sum to one
