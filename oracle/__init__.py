"""ctypes front end of the CPU oracle (``emc2o.c``).

TEST INFRASTRUCTURE ONLY.  Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline``
leg of ``bench.py`` may import this package; the product (``paper_2507_04123_amd``) never does and
this package never imports the product's HIP binding.

Every function takes and returns numpy arrays on the host.  Floating point: fp64 accumulation with
one final rounding to fp32, except the voxel cell index, which is defined in IEEE fp32.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "emc2o.c")
_LIB = os.path.join(_HERE, "libemc2o.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared",
               "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    c_i64, c_i32, c_f, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_void_p
    lib.emc2o_set_threads.argtypes = [ctypes.c_int]
    lib.emc2o_get_threads.restype = ctypes.c_int
    lib.emc2o_max_threads.restype = ctypes.c_int
    lib.emc2o_voxelize.restype = c_i64
    lib.emc2o_voxelize.argtypes = [vp, vp, c_i64, c_i32, vp, vp, vp, c_i32, c_f, c_f, c_i64, vp, vp, vp]
    lib.emc2o_build_kmap.restype = c_i64
    lib.emc2o_build_kmap.argtypes = [c_i32, vp, c_i64, vp, c_i32, c_i64, vp, vp, vp]
    lib.emc2o_spconv.restype = c_i64
    lib.emc2o_spconv.argtypes = [vp, c_i64, vp, vp, vp, c_i32, vp, c_i64, c_i64, c_i32, c_i32, vp]
    lib.emc2o_invert_kmap.restype = c_i64
    lib.emc2o_invert_kmap.argtypes = [vp, c_i64, c_i64, c_i64, c_i64, vp]
    lib.emc2o_bev_flatten.restype = c_i64
    lib.emc2o_bev_flatten.argtypes = [vp, vp, c_i64, vp, c_i32, c_i32, vp]
    lib.emc2o_pool_image.restype = c_i64
    lib.emc2o_pool_image.argtypes = [vp, vp, c_i32, c_i32, c_i32, vp, vp, vp, vp, c_i32, c_i32, c_i32, c_i64, vp, vp,
                                     vp, vp]
    lib.emc2o_fuse.restype = c_i64
    lib.emc2o_fuse.argtypes = [vp, vp, c_i64, c_i32, vp, vp, c_i64, c_i32, vp, c_i32, c_i64, vp, vp, vp, vp]
    lib.emc2o_e4m3_value.restype = ctypes.c_double
    lib.emc2o_e4m3_value.argtypes = [ctypes.c_uint8]
    lib.emc2o_quantize_e4m3.restype = c_i32
    lib.emc2o_quantize_e4m3.argtypes = [vp, c_i64, c_f, vp]
    lib.emc2o_spconv_e4m3.restype = c_i64
    lib.emc2o_spconv_e4m3.argtypes = [vp, c_i64, vp, vp, vp, c_i32, vp, c_i64, c_i64, c_i32, c_i32, vp]
    lib.emc2o_group_points.restype = c_i32
    lib.emc2o_group_points.argtypes = [vp, c_i64, vp, vp, vp, c_i32, c_i32, vp, vp]
    lib.emc2o_quantize_i8.restype = c_i32
    lib.emc2o_quantize_i8.argtypes = [vp, c_i64, c_f, vp]
    lib.emc2o_spconv_i8.restype = c_i64
    lib.emc2o_spconv_i8.argtypes = [vp, c_i64, vp, vp, vp, c_i32, c_f, vp, c_i64, c_i64, c_i32, c_i32, vp, vp]
    lib.emc2o_dispatch.restype = c_i32
    lib.emc2o_dispatch.argtypes = [vp, vp, c_i64, c_i32, c_f, c_f, vp, vp, vp]
    lib.emc2o_project_gather.restype = c_i32
    lib.emc2o_project_gather.argtypes = [vp, c_i32, c_i64, vp, vp, c_i32, c_i32, c_i32, vp, vp, vp]
    _lib = lib
    return lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(rc: int, what: str) -> int:
    if rc < 0:
        raise RuntimeError(f"oracle {what} failed: code {rc}")
    return rc


def set_threads(n: int) -> None:
    _load().emc2o_set_threads(int(n))


def max_threads() -> int:
    return int(_load().emc2o_max_threads())


def voxelize(points: np.ndarray, batch: Optional[np.ndarray], lo: Sequence[float], vs: Sequence[float],
             grid: Sequence[int], n_batch: int = 1, r2_min: float = 0.0, r2_max: float = float("inf"),
             capacity: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """points[P][F>=4] fp32 -> (coords[V][4] i32 (b,z,y,x) ascending key, means[V][4] f32, counts[V] i32)."""
    lib = _load()
    points = np.ascontiguousarray(points, dtype=np.float32)
    n, stride = points.shape if points.ndim == 2 else (0, 4)
    if batch is not None:
        batch = np.ascontiguousarray(batch, dtype=np.int32)
        assert batch.shape == (n,)
    cap = int(capacity if capacity is not None else max(n, 1))
    coords = np.empty((cap, 4), np.int32)
    feats = np.empty((cap, 4), np.float32)
    counts = np.empty((cap,), np.int32)
    lo_a = np.asarray(lo, np.float32)
    vs_a = np.asarray(vs, np.float32)
    g_a = np.asarray(grid, np.int32)
    v = _chk(lib.emc2o_voxelize(_p(points), _p(batch), n, stride, _p(lo_a), _p(vs_a), _p(g_a), int(n_batch),
                                float(np.float32(r2_min)), float(np.float32(r2_max)), cap, _p(coords),
                                _p(feats), _p(counts)), "voxelize")
    return coords[:v].copy(), feats[:v].copy(), counts[:v].copy()


def build_kmap(kind: int, in_coords: np.ndarray, grid_in: Sequence[int], n_batch: int = 1,
               capacity_out: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray, Tuple[int, int, int]]:
    """-> (out_coords[Vout][4], nbr[27][Vout] i32 with -1 = absent, grid_out)."""
    lib = _load()
    in_coords = np.ascontiguousarray(in_coords, dtype=np.int32).reshape(-1, 4)
    n_in = in_coords.shape[0]
    g_in = np.asarray(grid_in, np.int32)
    if capacity_out is None:
        gout = g_in if kind == 0 else (g_in - 1) // 2 + 1
        capacity_out = n_in if kind == 0 else int(min(8 * n_in, int(np.prod(gout.astype(np.int64))) * n_batch))
    cap = max(int(capacity_out), 1)
    out_coords = np.empty((cap, 4), np.int32)
    nbr = np.empty((27, cap), np.int32)
    g_out = np.zeros(3, np.int32)
    n_out = _chk(lib.emc2o_build_kmap(int(kind), _p(in_coords), n_in, _p(g_in), int(n_batch), cap,
                                      _p(out_coords), _p(nbr), _p(g_out)), "build_kmap")
    return out_coords[:n_out].copy(), np.ascontiguousarray(nbr[:, :n_out]), tuple(int(g) for g in g_out)


def invert_kmap(down: np.ndarray, n_fine: int) -> np.ndarray:
    """down[27][Vcoarse] (a stride-2 map over n_fine inputs) -> inv[27][n_fine]: the same pairs, read from the fine side."""
    lib = _load()
    down = np.ascontiguousarray(down, dtype=np.int32)
    assert down.ndim == 2 and down.shape[0] == 27
    n_coarse = down.shape[1]
    cap_f = max(int(n_fine), 1)
    inv = np.empty((27, cap_f), np.int32)
    _chk(lib.emc2o_invert_kmap(_p(down), n_coarse, max(n_coarse, 0), int(n_fine), cap_f, _p(inv)), "invert_kmap")
    return np.ascontiguousarray(inv[:, :n_fine])


def bev_flatten(coords: np.ndarray, feats: np.ndarray, grid: Sequence[int], n_batch: int = 1) -> np.ndarray:
    """coords[V][4] (b,z,y,x), feats[V][C] -> dense out[B][Gy][Gx][Gz*C] f32, zero where no voxel sits."""
    lib = _load()
    coords = np.ascontiguousarray(coords, dtype=np.int32).reshape(-1, 4)
    feats = np.ascontiguousarray(feats, dtype=np.float32)
    n, c = feats.shape
    assert coords.shape[0] == n
    g = np.asarray(grid, np.int32)
    out = np.empty((n_batch, int(g[1]), int(g[0]), int(g[2]) * c), np.float32)
    _chk(lib.emc2o_bev_flatten(_p(coords), _p(feats), n, _p(g), int(n_batch), c, _p(out)), "bev_flatten")
    return out


POOL_MEAN, POOL_MAX = 0, 1


def pool_image(img: np.ndarray, depth: np.ndarray, qmat: np.ndarray, lo: Sequence[float], vs: Sequence[float],
               grid: Sequence[int], mode: int = POOL_MEAN, n_batch: int = 1, batch_index: int = 0,
               capacity: Optional[int] = None, want_xyz: bool = False):
    """img[H][W][C] (any float; up-cast to f32), depth[H][W] f32, qmat[12] f32 (pixel*depth -> LiDAR frame)
    -> (coords[N][4], feats[N][C] f32, counts[N][, xyz[H][W][3] f32]), cells in ascending key order."""
    lib = _load()
    img32 = np.ascontiguousarray(img.astype(np.float32))
    h, wd, c = img32.shape
    depth = np.ascontiguousarray(depth, dtype=np.float32)
    assert depth.shape == (h, wd)
    qmat = np.ascontiguousarray(qmat, dtype=np.float32).reshape(12)
    lo_a, vs_a, g = np.asarray(lo, np.float32), np.asarray(vs, np.float32), np.asarray(grid, np.int32)
    cap = int(capacity) if capacity is not None else max(h * wd, 1)
    coords = np.empty((cap, 4), np.int32)
    feats = np.empty((cap, c), np.float32)
    counts = np.empty((cap,), np.int32)
    xyz = np.empty((h, wd, 3), np.float32) if want_xyz else None
    n = _chk(lib.emc2o_pool_image(_p(img32), _p(depth), h, wd, c, _p(qmat), _p(lo_a), _p(vs_a), _p(g), int(n_batch),
                                  int(batch_index), int(mode), cap, _p(coords), _p(feats), _p(counts), _p(xyz)),
             "pool_image")
    res = (coords[:n].copy(), feats[:n].copy(), counts[:n].copy())
    return res + (xyz,) if want_xyz else res


def fuse(coords_l: np.ndarray, feats_l: np.ndarray, coords_i: np.ndarray, feats_i: np.ndarray, grid: Sequence[int],
         n_batch: int = 1, capacity: Optional[int] = None, want_src: bool = False):
    """Union of two key-sorted sparse sets with concatenated features [LiDAR | image], zero-filled halves.
    -> (coords[N][4], feats[N][Cl+Ci] f32[, src_l[N], src_i[N]])."""
    lib = _load()
    coords_l = np.ascontiguousarray(coords_l, dtype=np.int32).reshape(-1, 4)
    coords_i = np.ascontiguousarray(coords_i, dtype=np.int32).reshape(-1, 4)
    feats_l = np.ascontiguousarray(feats_l, dtype=np.float32)
    feats_i = np.ascontiguousarray(feats_i, dtype=np.float32)
    n_l, cl = feats_l.shape
    n_i, ci = feats_i.shape
    assert coords_l.shape[0] == n_l and coords_i.shape[0] == n_i
    g = np.asarray(grid, np.int32)
    cap = int(capacity) if capacity is not None else max(n_l + n_i, 1)
    coords = np.empty((cap, 4), np.int32)
    feats = np.empty((cap, cl + ci), np.float32)
    src_l = np.empty((cap,), np.int32) if want_src else None
    src_i = np.empty((cap,), np.int32) if want_src else None
    n = _chk(lib.emc2o_fuse(_p(coords_l), _p(feats_l), n_l, cl, _p(coords_i), _p(feats_i), n_i, ci, _p(g),
                            int(n_batch), cap, _p(coords), _p(feats), _p(src_l), _p(src_i)), "fuse")
    res = (coords[:n].copy(), feats[:n].copy())
    return res + (src_l[:n].copy(), src_i[:n].copy()) if want_src else res


def quantize_i8(x: np.ndarray, inv_scale: float) -> np.ndarray:
    """q = clamp(rint(fl32(x * inv_scale)), -127, 127), ties to even."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.empty(x.shape, np.int8)
    _chk(lib.emc2o_quantize_i8(_p(x), x.size, float(np.float32(inv_scale)), _p(q)), "quantize_i8")
    return q


def spconv_i8(xq: np.ndarray, wq: np.ndarray, mul: np.ndarray, add: np.ndarray, relu: bool, nbr: np.ndarray,
              inv_out_scale: Optional[float] = None):
    """int8 x[n][Cin], int8 w[27][Cin][Cout], fp32 mul/add[Cout], nbr[27][V] -> v[V][Cout] f32 (and int8 q if
    inv_out_scale is given): exact integer accumulation, v = fl(fl(acc * mul) + add), optional ReLU, re-quantisation."""
    lib = _load()
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    mul = np.ascontiguousarray(mul, dtype=np.float32)
    add = np.ascontiguousarray(add, dtype=np.float32)
    nbr = np.ascontiguousarray(nbr, dtype=np.int32)
    n_in, cin = xq.shape
    assert wq.shape[0] == 27 and wq.shape[1] == cin and nbr.shape[0] == 27
    cout = wq.shape[2]
    n_out = nbr.shape[1]
    v = np.empty((n_out, cout), np.float32)
    q = np.empty((n_out, cout), np.int8) if inv_out_scale is not None else None
    _chk(lib.emc2o_spconv_i8(_p(xq), n_in, _p(wq), _p(mul), _p(add), int(bool(relu)),
                             float(np.float32(inv_out_scale if inv_out_scale is not None else 0.0)), _p(nbr),
                             max(n_out, 0), n_out, cin, cout, _p(v), _p(q)), "spconv_i8")
    return (v, q) if inv_out_scale is not None else v


def e4m3_value(code: int) -> float:
    """Value of one E4M3 code (NaN for the two codes that are not numbers)."""
    return float(_load().emc2o_e4m3_value(int(code) & 0xFF))


def quantize_e4m3(x: np.ndarray, inv_scale: float) -> np.ndarray:
    """fp32 -> E4M3 codes (uint8): nearest finite value of fl(x * inv_scale), ties to even, saturating, NaN -> 0."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.empty(x.shape, np.uint8)
    _chk(lib.emc2o_quantize_e4m3(_p(x), x.size, float(np.float32(inv_scale)), _p(q)), "quantize_e4m3")
    return q


def spconv_e4m3(xq: np.ndarray, wq: np.ndarray, mul: np.ndarray, add: np.ndarray, relu: bool, nbr: np.ndarray) -> np.ndarray:
    """uint8 E4M3 codes x[n][Cin], w[27][Cin][Cout], fp32 mul/add[Cout], nbr[27][V] -> v[V][Cout] f32: exact accumulation
    of the exact products, one rounding to fp32, v = fl(fl(acc * mul) + add), optional ReLU."""
    lib = _load()
    xq = np.ascontiguousarray(xq, dtype=np.uint8)
    wq = np.ascontiguousarray(wq, dtype=np.uint8)
    mul = np.ascontiguousarray(mul, dtype=np.float32)
    add = np.ascontiguousarray(add, dtype=np.float32)
    nbr = np.ascontiguousarray(nbr, dtype=np.int32)
    n_in, cin = xq.shape
    assert wq.shape[0] == 27 and wq.shape[1] == cin and nbr.shape[0] == 27
    cout = wq.shape[2]
    n_out = nbr.shape[1]
    v = np.empty((n_out, cout), np.float32)
    _chk(lib.emc2o_spconv_e4m3(_p(xq), n_in, _p(wq), _p(mul), _p(add), int(bool(relu)), _p(nbr), max(n_out, 0), n_out, cin, cout,
                               _p(v)), "spconv_e4m3")
    return v


LPE, VEE, APE = 0, 1, 2


def dispatch(props: np.ndarray, scene: Optional[np.ndarray], n_scenes: int, dist: float, conf: float):
    """props[N][4] f32 (x, y, z, confidence), scene[N] i32 -> (expert[S], counts[3], order[S]): the expert of
    every scene and the scenes grouped by expert."""
    lib = _load()
    props = np.ascontiguousarray(props, dtype=np.float32).reshape(-1, 4)
    n = props.shape[0]
    if scene is not None:
        scene = np.ascontiguousarray(scene, dtype=np.int32)
        assert scene.shape == (n,)
    expert = np.empty((max(n_scenes, 1),), np.int32)
    counts = np.empty((3,), np.int32)
    order = np.empty((max(n_scenes, 1),), np.int32)
    _chk(lib.emc2o_dispatch(_p(props), _p(scene), n, int(n_scenes), float(np.float32(dist)), float(np.float32(conf)),
                            _p(expert), _p(counts), _p(order)), "dispatch")
    return expert[:n_scenes].copy(), counts, order[:n_scenes].copy()


def group_points(scene: Optional[np.ndarray], n_points: int, expert: np.ndarray, order: np.ndarray, counts: np.ndarray,
                 e: int):
    """Dispatcher outputs -> (slot[S], group_batch[P]): every scene's position inside its expert's group, and the batch
    ids of the points for expert e's group (-1 for points of other experts' scenes)."""
    lib = _load()
    expert = np.ascontiguousarray(expert, dtype=np.int32)
    order = np.ascontiguousarray(order, dtype=np.int32)
    counts = np.ascontiguousarray(counts, dtype=np.int32)
    n_scenes = len(expert)
    if scene is not None:
        scene = np.ascontiguousarray(scene, dtype=np.int32)
        assert len(scene) == n_points
    slot = np.empty((n_scenes,), np.int32)
    gb = np.empty((n_points,), np.int32)
    _chk(lib.emc2o_group_points(_p(scene), int(n_points), _p(expert), _p(order), _p(counts), n_scenes, int(e), _p(slot), _p(gb)),
         "group_points")
    return slot, gb


def spconv(x: np.ndarray, w: np.ndarray, scale: Optional[np.ndarray], shift: Optional[np.ndarray],
           epilogue: int, nbr: np.ndarray, return_macs: bool = False):
    """x[Vin][Cin] f32, w[27][Cin][Cout] f32, nbr[27][Vout] -> y[Vout][Cout] f32 (fp64 accumulation)."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    nbr = np.ascontiguousarray(nbr, dtype=np.int32)
    assert w.ndim == 3 and w.shape[0] == 27 and nbr.ndim == 2 and nbr.shape[0] == 27
    n_in, cin = x.shape
    cout = w.shape[2]
    assert w.shape[1] == cin
    n_out = nbr.shape[1]
    if scale is not None:
        scale = np.ascontiguousarray(scale, dtype=np.float32)
        shift = np.ascontiguousarray(shift, dtype=np.float32)
    y = np.empty((n_out, cout), np.float32)
    macs = _chk(lib.emc2o_spconv(_p(x), n_in, _p(w), _p(scale), _p(shift), int(epilogue), _p(nbr),
                                 max(n_out, 0), n_out, cin, cout, _p(y)), "spconv")
    return (y, macs) if return_macs else y


def project_gather(points: np.ndarray, pmat: np.ndarray, img: np.ndarray, want_uv: bool = False):
    """points[P][F>=3] f32, pmat[12] f32, img[H][W][C] (any float; up-cast to f32) -> (g[P][C] f32, valid[P] u8[, uv f64])."""
    lib = _load()
    points = np.ascontiguousarray(points, dtype=np.float32)
    pmat = np.ascontiguousarray(pmat, dtype=np.float32).reshape(12)
    img32 = np.ascontiguousarray(img.astype(np.float32))
    h, wd, c = img32.shape
    n, stride = points.shape
    out = np.empty((n, c), np.float32)
    valid = np.empty((n,), np.uint8)
    uv = np.empty((n, 2), np.float64) if want_uv else None
    _chk(lib.emc2o_project_gather(_p(points), stride, n, _p(pmat), _p(img32), h, wd, c, _p(out), _p(valid),
                                  _p(uv)), "project_gather")
    return (out, valid, uv) if want_uv else (out, valid)
