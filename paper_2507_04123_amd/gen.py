"""Seeded synthetic inputs: point clouds, conv weights, folded-BN parameters, camera, image features.

These stand in for KITTI front-view frames and nuScenes 10-sweep frames (the datasets of the paper's
Sec. 4.1), which are not available here; only shapes, ranges and density laws are modelled, no
dataset record is reproduced.  The module serves both the HIP path and the tests' oracle side and
therefore holds none of the method's arithmetic (no voxel index, no hashing, no convolution, no
projection of points): it only draws numbers.

Random numbers come from a self-contained counter-based generator (splitmix64 finaliser over
seed + counter), so streams do not depend on the numpy version.
"""
from __future__ import annotations

import math
from typing import Dict, List, Tuple

import numpy as np

from .configs import Config, Layer, F16, BF16, F32

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


class Stream:
    """Counter-based stream: value i is mix(seed' + (i+1)*GOLDEN); draws advance the counter."""

    def __init__(self, seed: int, stream_id: int = 0):
        s = np.array([seed & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64)
        t = np.array([(stream_id + 1) & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64)
        with np.errstate(over="ignore"):
            self._seed = _mix(s + _mix(t * _GOLDEN))[0]
        self._ctr = 0

    def bits(self, n: int) -> np.ndarray:
        idx = np.arange(self._ctr + 1, self._ctr + n + 1, dtype=np.uint64)
        self._ctr += n
        with np.errstate(over="ignore"):
            return _mix(self._seed + idx * _GOLDEN)

    def uniform(self, n: int, lo: float = 0.0, hi: float = 1.0) -> np.ndarray:
        """24-bit uniforms in [lo, hi) as float64 (u24 / 2^24 is exact in fp32 too)."""
        u = (self.bits(n) >> np.uint64(40)).astype(np.float64) * (1.0 / 16777216.0)
        return lo + (hi - lo) * u

    def normal(self, n: int, sigma: float = 1.0) -> np.ndarray:
        """Box-Muller on two 24-bit uniforms per pair of outputs (float64)."""
        m = (n + 1) // 2
        b = self.bits(m)
        u1 = ((b >> np.uint64(40)).astype(np.float64) + 1.0) * (1.0 / 16777216.0)   # (0, 1]
        u2 = ((b >> np.uint64(16)) & np.uint64(0xFFFFFF)).astype(np.float64) * (1.0 / 16777216.0)
        r = np.sqrt(-2.0 * np.log(u1))
        out = np.empty(2 * m, dtype=np.float64)
        out[0::2] = r * np.cos(2.0 * math.pi * u2)
        out[1::2] = r * np.sin(2.0 * math.pi * u2)
        return sigma * out[:n]

    def permutation(self, n: int) -> np.ndarray:
        """Permutation by sorting random 64-bit tags (ties are astronomically unlikely; stable)."""
        return np.argsort(self.bits(n), kind="stable")


def frame_seed(cfg_index: int, frame: int) -> int:
    return 0xE3C20000 + 256 * cfg_index + frame


# ----------------------------------------------------------------------------------------------
# clouds
# ----------------------------------------------------------------------------------------------

def _ground(st: Stream, n: int, r_lo: float, r_hi: float, az_lo: float, az_hi: float,
            xb: Tuple[float, float], yb: Tuple[float, float], z_lo: float, z_hi: float) -> np.ndarray:
    """Range r ~ U[r_lo, r_hi] with uniform azimuth gives areal density ~ 1/r; reject into the box."""
    xs: List[np.ndarray] = []
    ys: List[np.ndarray] = []
    have = 0
    while have < n:
        m = max(4096, 2 * (n - have))
        r = st.uniform(m, r_lo, r_hi)
        a = st.uniform(m, az_lo, az_hi)
        x = r * np.cos(a)
        y = r * np.sin(a)
        keep = (x >= xb[0]) & (x < xb[1]) & (y >= yb[0]) & (y < yb[1])
        xs.append(x[keep])
        ys.append(y[keep])
        have += int(keep.sum())
    x = np.concatenate(xs)[:n]
    y = np.concatenate(ys)[:n]
    z = st.uniform(n, z_lo, z_hi)
    return np.stack([x, y, z], axis=1)


def _boxes(st: Stream, n_boxes: int, per_box: int, cx: Tuple[float, float], cy: Tuple[float, float],
           z_floor: float) -> np.ndarray:
    """Points uniform in the volume of 4 x 1.8 x 1.6 m boxes with random centre and yaw."""
    c_x = st.uniform(n_boxes, *cx)
    c_y = st.uniform(n_boxes, *cy)
    yaw = st.uniform(n_boxes, -math.pi, math.pi)
    out = np.empty((n_boxes * per_box, 3), dtype=np.float64)
    for b in range(n_boxes):
        lx = st.uniform(per_box, -2.0, 2.0)
        ly = st.uniform(per_box, -0.9, 0.9)
        lz = st.uniform(per_box, 0.0, 1.6)
        c, s = math.cos(yaw[b]), math.sin(yaw[b])
        sl = slice(b * per_box, (b + 1) * per_box)
        out[sl, 0] = c_x[b] + c * lx - s * ly
        out[sl, 1] = c_y[b] + s * lx + c * ly
        out[sl, 2] = z_floor + lz
    return out


def make_cloud(recipe: str, n_points: int, seed: int) -> np.ndarray:
    """Return points[P][4] float32 (x, y, z, intensity), shuffled.

    Points that leave the voxel bounds (rotated boxes near the border) stay in the cloud on
    purpose: dropping them is the voxelizer's job.
    """
    st = Stream(seed, 0)
    if recipe == "uniform_tiny":
        xyz = np.stack([st.uniform(n_points, 0.0, 20.0), st.uniform(n_points, -10.0, 10.0),
                        st.uniform(n_points, -3.0, 1.0)], axis=1)
    elif recipe == "front":
        n_box_pts = (n_points * 3) // 10
        n_boxes = 20
        per_box = n_box_pts // n_boxes
        n_box_pts = per_box * n_boxes
        g = _ground(st, n_points - n_box_pts, 2.0, 70.4, -math.pi / 2, math.pi / 2,
                    (0.0, 70.4), (-40.0, 40.0), -1.65, -1.55)
        b = _boxes(st, n_boxes, per_box, (5.0, 65.4), (-35.0, 35.0), -1.6)
        xyz = np.concatenate([g, b], axis=0)
    elif recipe == "surround":
        n_box_pts = (n_points * 3) // 10
        n_boxes = 60
        per_box = n_box_pts // n_boxes
        n_box_pts = per_box * n_boxes
        g = _ground(st, n_points - n_box_pts, 1.0, 76.4, -math.pi, math.pi,
                    (-54.0, 54.0), (-54.0, 54.0), -1.85, -1.75)
        b = _boxes(st, n_boxes, per_box, (-50.0, 50.0), (-50.0, 50.0), -1.8)
        xyz = np.concatenate([g, b], axis=0)
    else:
        raise ValueError(f"unknown cloud recipe {recipe!r}")
    inten = st.uniform(xyz.shape[0], 0.0, 1.0)
    pts = np.concatenate([xyz, inten[:, None]], axis=1).astype(np.float32)
    perm = st.permutation(pts.shape[0])
    return np.ascontiguousarray(pts[perm])


def make_frames(cfg: Config, first_frame: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """points[P_total][4] float32 and batch[P_total] int32 for cfg.n_frames consecutive frames."""
    pts, bat = [], []
    for f in range(cfg.n_frames):
        p = make_cloud(cfg.cloud, cfg.n_points, frame_seed(cfg.index, first_frame + f))
        pts.append(p)
        bat.append(np.full(p.shape[0], f, dtype=np.int32))
    return np.ascontiguousarray(np.concatenate(pts, axis=0)), np.concatenate(bat)


# ----------------------------------------------------------------------------------------------
# dtype helpers (plain storage conversions, round-to-nearest-even)
# ----------------------------------------------------------------------------------------------

def round_to_dtype(a32: np.ndarray, dtype: int) -> np.ndarray:
    """Round fp32 values to the storage dtype and return them as fp32 again (exact up-cast)."""
    a32 = np.asarray(a32, dtype=np.float32)
    if dtype == F32:
        return a32.copy()
    if dtype == F16:
        return a32.astype(np.float16).astype(np.float32)
    if dtype == BF16:
        return bf16_bits_to_f32(f32_to_bf16_bits(a32))
    raise ValueError(dtype)


def f32_to_bf16_bits(a32: np.ndarray) -> np.ndarray:
    u = np.asarray(a32, dtype=np.float32).view(np.uint32).astype(np.uint64)
    rounded = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)
    nan = np.isnan(a32)
    out = rounded.astype(np.uint16)
    out[nan] = 0x7FC0
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------------------------
# weights, folded BN, camera, image
# ----------------------------------------------------------------------------------------------

def make_layer_params(layer: Layer, seed: int, layer_id: int) -> Dict[str, np.ndarray]:
    """W[27][Cin][Cout] ~ N(0, 0.1) in fp32; folded-BN scale/shift[Cout] in fp32.

    scale ~ U[0.8, 1.2] / (0.1 * sqrt(9 * Cin)) keeps activations O(1) through a deep fp16 stack.
    """
    st = Stream(seed, 1000 + layer_id)
    w = st.normal(27 * layer.cin * layer.cout, 0.1).astype(np.float32).reshape(27, layer.cin, layer.cout)
    scale = (st.uniform(layer.cout, 0.8, 1.2) / (0.1 * math.sqrt(9.0 * layer.cin))).astype(np.float32)
    shift = st.uniform(layer.cout, -0.1, 0.1).astype(np.float32)
    return {"w": w, "scale": scale, "shift": shift}


def make_camera(seed: int) -> np.ndarray:
    """Seeded 3x4 pinhole matrix P = K [R | t], row-major float32[12].

    R maps LiDAR axes (x forward, y left, z up) to camera axes (x right, y down, z forward).
    """
    st = Stream(seed, 2000)
    u = st.uniform(4, 0.0, 1.0)
    f = 720.0 * (1.0 + 0.02 * u[0])
    cx, cy = 620.5, 187.0
    t = -0.3 + 0.6 * u[1:4]
    k = np.array([[f, 0.0, cx], [0.0, f, cy], [0.0, 0.0, 1.0]])
    r = np.array([[0.0, -1.0, 0.0], [0.0, 0.0, -1.0], [1.0, 0.0, 0.0]])
    rt = np.concatenate([r, t[:, None]], axis=1)
    return np.ascontiguousarray((k @ rt).astype(np.float32).reshape(12))


def make_image(height: int, width: int, channels: int, seed: int) -> np.ndarray:
    """img[H][W][C] float16 ~ N(0, 1) (stand-in for an image-branch feature map)."""
    st = Stream(seed, 3000)
    return st.normal(height * width * channels, 1.0).astype(np.float16).reshape(height, width, channels)


def make_unprojection(pmat: np.ndarray) -> np.ndarray:
    """Inverse of the pinhole matrix as an input of the pooling step: Q float32[12] with
    X_lidar = Q (d*u, d*v, d, 1) for the pixel (u, v) at depth d.  With P = [M | p4], Q = [M^-1 | -M^-1 p4],
    inverted in float64 and rounded once."""
    p = np.asarray(pmat, np.float64).reshape(3, 4)
    mi = np.linalg.inv(p[:, :3])
    return np.ascontiguousarray(np.concatenate([mi, -(mi @ p[:, 3:4])], axis=1).astype(np.float32).reshape(12))


def make_depth(height: int, width: int, seed: int, proposals_only: bool = False, n_objects: int = 40) -> np.ndarray:
    """depth[H][W] float32 of a road scene seen by the camera of make_camera: 0 = no depth (sky, or outside
    every proposal region when `proposals_only`).

    Rows below the horizon (row 187) see a ground plane 1.6 m under the camera, depth 720*1.6/(row - 187)
    capped at 70 m; `n_objects` upright rectangles (1.8 x 1.6 m at depths 6..60 m, standing on the ground
    row of their depth) occlude what lies behind them; +-1 % multiplicative noise.  With `proposals_only`
    only the pixels inside the rectangles grown by half their size keep a depth: the image regions of the
    3D proposals."""
    st = Stream(seed, 4000)
    f, cy, h_cam = 720.0, 187.0, 1.6
    rows = np.arange(height, dtype=np.float64)[:, None]
    cols = np.arange(width, dtype=np.float64)[None, :]
    depth = np.zeros((height, width), np.float64)
    below = rows > cy + 1.0
    ground = f * h_cam / np.maximum(rows - cy, 1e-9)
    depth = np.where(below & (ground <= 70.0), ground, 0.0) * np.ones((1, width))
    d_obj = np.sort(st.uniform(n_objects, 6.0, 60.0))[::-1]          # far to near: nearer ones overwrite
    c_col = st.uniform(n_objects, 0.0, float(width))
    mask = np.zeros((height, width), bool)
    for d, cc in zip(d_obj, c_col):
        half_w = 0.9 * f / d
        top = cy + f * (h_cam - 1.6) / d
        bot = cy + f * h_cam / d
        inside = (np.abs(cols - cc) <= half_w) & (rows >= top) & (rows <= bot)
        depth = np.where(inside, d, depth)
        grown = (np.abs(cols - cc) <= 1.5 * half_w) & (rows >= top - 0.25 * (bot - top)) & (rows <= bot + 0.25 * (bot - top))
        mask |= grown
    noise = 1.0 + 0.01 * (2.0 * st.uniform(height * width, 0.0, 1.0).reshape(height, width) - 1.0)
    depth = depth * noise
    if proposals_only:
        depth = np.where(mask, depth, 0.0)
    return np.ascontiguousarray(depth.astype(np.float32))


def make_proposals(n_scenes: int, seed: int, dist: float = 23.5, conf: float = 0.5,
                   max_per_scene: int = 300) -> Tuple[np.ndarray, np.ndarray]:
    """Proposal regions of `n_scenes` driving scenes: props[N][4] float32 (x, y, z, confidence) and scene[N] int32,
    shuffled.  A third of the scenes hold only near, confidently detected objects, a third add a few that are
    near but unclear or far but clear, a third also some that are far and unclear (confidence falls with range,
    as sparse returns make distant objects hard); a few scenes are empty.  About one proposal in fifty sits on a
    threshold: at range exactly `dist`, one float below it, or at `dist` in a slanted direction (where the
    squared range is decided by how the two products round), and with confidence exactly `conf` or one float
    beside it -- always on the side that keeps the scene in its third, so the mix of experts stays balanced
    while every comparison is exercised at its edge."""
    st = Stream(seed, 5000)
    kinds = (st.bits(n_scenes) % np.uint64(3)).astype(np.int64)
    sizes = (st.bits(n_scenes) % np.uint64(max_per_scene + 1)).astype(np.int64)
    sizes[(st.bits(n_scenes) % np.uint64(16)) == 0] = 0
    props, scenes = [], []
    for s in range(n_scenes):
        k = int(sizes[s])
        if k == 0:
            continue
        r = st.uniform(k, 2.0, 0.97 * dist)
        a = st.uniform(k, -math.pi / 2, math.pi / 2)
        c = st.uniform(k, min(1.0, conf + 0.05), 1.0)
        odd = st.uniform(k, 0.0, 1.0) < 0.05                      # the few objects that change the scene's class
        far = st.uniform(k, 0.0, 1.0) < 0.5
        if kinds[s] >= 1:
            r = np.where(odd & far, st.uniform(k, 1.02 * dist, 3.0 * dist), r)           # far but clear
            c = np.where(odd & ~far, st.uniform(k, 0.0, max(conf - 0.05, 0.0)), c)       # near but unclear
        if kinds[s] == 2:
            both = st.uniform(k, 0.0, 1.0) < 0.03
            r = np.where(both, st.uniform(k, 1.02 * dist, 3.0 * dist), r)
            c = np.where(both, st.uniform(k, 0.0, max(conf - 0.05, 0.0)), c)
        z = st.uniform(k, -1.6, 0.4)
        rows = np.stack([r * np.cos(a), r * np.sin(a), z, c], axis=1).astype(np.float32)
        # threshold cases (float32 values placed after the rounding above)
        d32, c32 = np.float32(dist), np.float32(conf)
        d_below, c_above, c_below = np.nextafter(d32, np.float32(0)), np.nextafter(c32, np.float32(2)), np.nextafter(c32, np.float32(-1))
        n_edge = max(1, k // 50)
        which = (st.bits(n_edge) % np.uint64(4)).astype(np.int64)
        axis = (st.bits(n_edge) % np.uint64(4)).astype(np.int64)      # +x, -x, +y, -y
        slant = st.uniform(n_edge, -1.5, 1.5)
        for e in range(n_edge):
            if kinds[s] == 0:        # stays near and clear: one float inside the distance, at or just above the confidence
                rr, cc = d_below, (c32 if which[e] % 2 == 0 else c_above)
            elif kinds[s] == 1:      # far but clear (range exactly on the threshold), or near but just unclear
                rr, cc = (d32, c_above) if which[e] % 2 == 0 else (d_below, c_below)
            else:                    # far and just unclear
                rr, cc = d32, c_below
            if kinds[s] >= 1 and which[e] >= 2 and rr == d32:
                # slanted direction: x^2 + y^2 lands within a few floats of dist^2, on either side; the scene is in
                # the versatile or accuracy third either way, and both sides must decide it by the same roundings
                xy = (np.float32(dist * math.cos(slant[e])), np.float32(dist * math.sin(slant[e])))
            else:
                xy = [(rr, 0.0), (-rr, 0.0), (0.0, rr), (0.0, -rr)][axis[e]]
            rows[e] = (xy[0], xy[1], rows[e, 2], cc)
        props.append(rows)
        scenes.append(np.full(k, s, np.int64))
    if not props:
        return np.zeros((0, 4), np.float32), np.zeros((0,), np.int32)
    p = np.concatenate(props).astype(np.float32)
    sc = np.concatenate(scenes).astype(np.int32)
    perm = st.permutation(len(p))
    return np.ascontiguousarray(p[perm]), np.ascontiguousarray(sc[perm])
