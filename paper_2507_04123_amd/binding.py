"""ctypes binding over libemc2.so: argument marshalling only, every step runs in the HIP kernels.

Tensors are torch CUDA(=HIP) tensors used purely as device buffers; the current torch stream is
passed as the HIP stream.  There is no CPU fallback: if the library is missing or no GPU is present
the calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

from .configs import VoxelSpec

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libemc2.so")

OK, ERR_INVALID_ARG, ERR_CAPACITY, ERR_UNSUPPORTED, ERR_DEVICE, ERR_MAP = 0, 1, 2, 3, 4, 5
F32, F16, BF16, I8 = 0, 1, 2, 3
SUBM, STRIDED = 0, 1
EPI_NONE, EPI_AFFINE, EPI_AFFINE_RELU = 0, 1, 2
W_PLAIN, W_PACKED = 0, 1
POOL_MEAN, POOL_MAX = 0, 1
MAP_ANY = -1   # emc2_spconv map_hint: SUBM / STRIDED as passed to build_kmap, or unknown

_TORCH_DTYPE = {F32: torch.float32, F16: torch.float16, BF16: torch.bfloat16}

EXPORTS = ["emc2_create", "emc2_destroy", "emc2_status_sync", "emc2_last_error", "emc2_voxelize",
           "emc2_build_kmap", "emc2_spconv", "emc2_project_gather", "emc2_pack_weights", "emc2_spconv_uses_mfma",
           "emc2_spconv_kernel", "emc2_build_inverse_kmap", "emc2_bev_flatten", "emc2_pool_image", "emc2_fuse", "emc2_dispatch", "emc2_spconv_i8_supported",
           "emc2_quantize_i8", "emc2_pack_weights_i8", "emc2_spconv_i8", "emc2_build_kmap_static", "emc2_group_points", "emc2_quantize_e4m3", "emc2_spconv_e4m3"]


class Emc2Error(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"emc2 status {status}: {msg}")
        self.status = status


class _VoxelSpecC(ctypes.Structure):
    _fields_ = [("lo", ctypes.c_float * 3), ("vs", ctypes.c_float * 3), ("grid", ctypes.c_int32 * 3),
                ("n_batch", ctypes.c_int32), ("r2_min", ctypes.c_float), ("r2_max", ctypes.c_float),
                ("stride_f", ctypes.c_int32)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libemc2.so (build it first with ``python -m paper_2507_04123_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is not built; run __graft_entry__.build() or paper_2507_04123_amd/build.py")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    lib.emc2_create.restype = ctypes.c_int
    lib.emc2_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64, i64, i64, i32]
    lib.emc2_destroy.restype = None
    lib.emc2_destroy.argtypes = [vp]
    lib.emc2_status_sync.restype = ctypes.c_int
    lib.emc2_status_sync.argtypes = [vp, vp]
    lib.emc2_last_error.restype = ctypes.c_char_p
    lib.emc2_last_error.argtypes = [vp]
    lib.emc2_voxelize.restype = ctypes.c_int
    lib.emc2_voxelize.argtypes = [vp, vp, vp, i64, ctypes.POINTER(_VoxelSpecC), i64, vp, vp, vp, vp, ctypes.c_int, vp,
                                  ctypes.POINTER(i32), i32, vp]
    lib.emc2_build_kmap.restype = ctypes.c_int
    lib.emc2_build_kmap.argtypes = [vp, ctypes.c_int, vp, vp, i64, ctypes.POINTER(i32), i32, i32, i32, i64, vp, vp, vp,
                                    ctypes.POINTER(i32), ctypes.POINTER(i32), vp]
    lib.emc2_build_kmap_static.restype = ctypes.c_int
    lib.emc2_build_kmap_static.argtypes = [ctypes.c_int, vp, vp, i64, ctypes.POINTER(i32), i32, i64, vp, vp, vp,
                                           ctypes.POINTER(i32), vp, vp]
    lib.emc2_spconv.restype = ctypes.c_int
    lib.emc2_spconv.argtypes = [vp, ctypes.c_int, vp, vp, ctypes.c_int, vp, vp, ctypes.c_int, vp, i32, vp, i64, i64, i32, i32, vp, vp]
    lib.emc2_pack_weights.restype = ctypes.c_int
    lib.emc2_pack_weights.argtypes = [vp, ctypes.c_int, vp, i32, i32, vp, vp]
    lib.emc2_spconv_kernel.restype = ctypes.c_char_p
    lib.emc2_spconv_kernel.argtypes = [ctypes.c_int, i32, i32, i32]
    lib.emc2_spconv_uses_mfma.restype = i32
    lib.emc2_spconv_uses_mfma.argtypes = [ctypes.c_int, i32, i32]
    lib.emc2_pool_image.restype = ctypes.c_int
    lib.emc2_pool_image.argtypes = [vp, vp, vp, i32, i32, i32, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(_VoxelSpecC),
                                    i32, ctypes.c_int, i64, vp, vp, vp, vp, ctypes.POINTER(i32), i32, vp]
    lib.emc2_fuse.restype = ctypes.c_int
    lib.emc2_fuse.argtypes = [vp, ctypes.c_int, vp, vp, vp, i64, i32, vp, vp, vp, i64, i32, ctypes.POINTER(i32), i32, i32,
                              i64, i32, vp, vp, vp, vp, vp, ctypes.POINTER(i32), vp]
    lib.emc2_spconv_i8_supported.restype = i32
    lib.emc2_spconv_i8_supported.argtypes = [i32, i32]
    lib.emc2_quantize_i8.restype = ctypes.c_int
    lib.emc2_quantize_i8.argtypes = [vp, ctypes.c_int, vp, i64, ctypes.c_float, vp, vp]
    lib.emc2_pack_weights_i8.restype = ctypes.c_int
    lib.emc2_pack_weights_i8.argtypes = [vp, vp, i32, i32, vp, vp]
    lib.emc2_spconv_i8.restype = ctypes.c_int
    lib.emc2_spconv_i8.argtypes = [vp, vp, vp, vp, vp, i32, ctypes.c_int, ctypes.c_float, vp, vp, i64, i64, i32, i32, vp, vp]
    lib.emc2_quantize_e4m3.restype = ctypes.c_int
    lib.emc2_quantize_e4m3.argtypes = [vp, ctypes.c_int, vp, i64, ctypes.c_float, vp, vp]
    lib.emc2_spconv_e4m3.restype = ctypes.c_int
    lib.emc2_spconv_e4m3.argtypes = [vp, vp, vp, vp, vp, i32, ctypes.c_int, vp, vp, i64, i64, i32, i32, vp, vp]
    lib.emc2_dispatch.restype = ctypes.c_int
    lib.emc2_dispatch.argtypes = [vp, vp, vp, i64, i32, ctypes.c_float, ctypes.c_float, vp, vp, vp, vp]
    lib.emc2_group_points.restype = ctypes.c_int
    lib.emc2_group_points.argtypes = [vp, vp, i64, vp, vp, vp, i32, i32, vp, vp, vp]
    lib.emc2_project_gather.restype = ctypes.c_int
    lib.emc2_project_gather.argtypes = [vp, vp, i32, i64, ctypes.POINTER(ctypes.c_float), vp, i32, i32, i32, vp, vp, vp, vp]
    lib.emc2_build_inverse_kmap.restype = ctypes.c_int
    lib.emc2_build_inverse_kmap.argtypes = [vp, vp, vp, i64, ctypes.POINTER(i32), i32, i32, vp, vp, vp]
    lib.emc2_bev_flatten.restype = ctypes.c_int
    lib.emc2_bev_flatten.argtypes = [vp, ctypes.c_int, vp, vp, vp, i64, ctypes.POINTER(i32), i32, i32, vp, vp]
    _lib = lib
    return lib


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_check(t: torch.Tensor, dtype: torch.dtype, name: str) -> None:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name}: need a contiguous {dtype} device tensor, got {t.dtype} on {t.device}")


STATIC_KMAP_MAX_CELLS = 1 << 24


def build_kmap_static(kind: int, in_coords: torch.Tensor, n_in: torch.Tensor, capacity_in: int, grid_in: Sequence[int],
                      n_batch: int, capacity_out: int, nbr: torch.Tensor, n_out: torch.Tensor,
                      out_coords: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None) -> Tuple[int, int, int]:
    """emc2_build_kmap_static: the kernel map without a context (static device scratch, nothing allocated), on the
    current device and torch's current stream.  Returns the output grid."""
    if not torch.cuda.is_available():
        raise RuntimeError("emc2 needs a GPU: there is no CPU path")
    lib = load_library()
    _dev_check(in_coords, torch.int32, "in_coords")
    _dev_check(n_in, torch.int32, "n_in")
    _dev_check(nbr, torch.int32, "nbr")
    _dev_check(n_out, torch.int32, "n_out")
    if in_coords.numel() < 4 * capacity_in or nbr.numel() < 27 * capacity_out:
        raise ValueError("buffers smaller than capacity")
    if out_coords is not None:
        _dev_check(out_coords, torch.int32, "out_coords")
        if out_coords.numel() < 4 * capacity_out:
            raise ValueError("out_coords smaller than capacity_out")
    if status is not None:
        _dev_check(status, torch.int32, "status")
    g_in = (ctypes.c_int32 * 3)(*grid_in)
    g_out = (ctypes.c_int32 * 3)()
    st = lib.emc2_build_kmap_static(kind, _ptr(in_coords), _ptr(n_in), capacity_in, g_in, n_batch, capacity_out,
                                    _ptr(out_coords), _ptr(n_out), _ptr(nbr), g_out, _ptr(status), _stream())
    if st != OK:
        raise Emc2Error(st, lib.emc2_last_error(None).decode())
    return g_out[0], g_out[1], g_out[2]


class Context:
    """Owns the library's scratch on one GPU (see emc2_create)."""

    def __init__(self, max_points: int, max_voxels: int, max_cells: int, n_slots: int = 4, device: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("emc2 needs a GPU: there is no CPU path")
        self.lib = load_library()
        self.device = device
        h = ctypes.c_void_p()
        st = self.lib.emc2_create(ctypes.byref(h), device, max_points, max_voxels, max_cells, n_slots)
        if st != OK:
            raise Emc2Error(st, "emc2_create failed")
        self.h = h
        self.max_voxels = max_voxels

    def close(self) -> None:
        if getattr(self, "h", None):
            self.lib.emc2_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _chk(self, st: int) -> None:
        if st != OK:
            raise Emc2Error(st, self.lib.emc2_last_error(self.h).decode())

    def status_sync(self) -> None:
        self._chk(self.lib.emc2_status_sync(self.h, _stream()))

    # ------------------------------------------------------------------------------------------
    def voxelize(self, points: torch.Tensor, batch: Optional[torch.Tensor], spec: VoxelSpec, capacity: int,
                 coords: torch.Tensor, feats: torch.Tensor, counts: torch.Tensor, n_voxels: torch.Tensor,
                 feats_lp: Optional[torch.Tensor] = None, index_slot: int = 0, sync_count: bool = False) -> Optional[int]:
        _dev_check(points, torch.float32, "points")
        _dev_check(coords, torch.int32, "coords")
        _dev_check(feats, torch.float32, "feats")
        _dev_check(counts, torch.int32, "counts")
        _dev_check(n_voxels, torch.int32, "n_voxels")
        n, stride = (points.shape[0], points.shape[1]) if points.dim() == 2 else (0, 4)
        if coords.numel() < 4 * capacity or feats.numel() < 4 * capacity or counts.numel() < capacity:
            raise ValueError("output buffers smaller than capacity")
        if batch is not None:
            _dev_check(batch, torch.int32, "batch")
            if batch.numel() != n:
                raise ValueError("batch length != number of points")
        lp_dtype = F16
        if feats_lp is not None:
            lp_dtype = {torch.float16: F16, torch.bfloat16: BF16}[feats_lp.dtype]
            if feats_lp.numel() < 4 * capacity or not feats_lp.is_cuda:
                raise ValueError("feats_lp smaller than capacity")
        cs = _VoxelSpecC((ctypes.c_float * 3)(*spec.lo), (ctypes.c_float * 3)(*spec.vs), (ctypes.c_int32 * 3)(*spec.grid),
                         spec.n_batch, spec.r2_min, spec.r2_max, stride)
        h_n = ctypes.c_int32(0)
        self._chk(self.lib.emc2_voxelize(self.h, _ptr(points), _ptr(batch), n, ctypes.byref(cs), capacity, _ptr(coords),
                                         _ptr(feats), _ptr(counts), _ptr(feats_lp), lp_dtype, _ptr(n_voxels),
                                         ctypes.byref(h_n) if sync_count else None, index_slot, _stream()))
        return int(h_n.value) if sync_count else None

    def build_kmap(self, kind: int, in_coords: torch.Tensor, n_in: torch.Tensor, capacity_in: int, grid_in: Sequence[int],
                   n_batch: int, capacity_out: int, nbr: torch.Tensor, n_out: torch.Tensor,
                   out_coords: Optional[torch.Tensor] = None, in_slot: int = -1, out_slot: int = -1,
                   sync_count: bool = False) -> Tuple[Tuple[int, int, int], Optional[int]]:
        _dev_check(in_coords, torch.int32, "in_coords")
        _dev_check(n_in, torch.int32, "n_in")
        _dev_check(nbr, torch.int32, "nbr")
        _dev_check(n_out, torch.int32, "n_out")
        if in_coords.numel() < 4 * capacity_in or nbr.numel() < 27 * capacity_out:
            raise ValueError("buffers smaller than capacity")
        if out_coords is not None:
            _dev_check(out_coords, torch.int32, "out_coords")
            if out_coords.numel() < 4 * capacity_out:
                raise ValueError("out_coords smaller than capacity_out")
        g_in = (ctypes.c_int32 * 3)(*grid_in)
        g_out = (ctypes.c_int32 * 3)()
        h_n = ctypes.c_int32(0)
        self._chk(self.lib.emc2_build_kmap(self.h, kind, _ptr(in_coords), _ptr(n_in), capacity_in, g_in, n_batch, in_slot,
                                           out_slot, capacity_out, _ptr(out_coords), _ptr(n_out), _ptr(nbr), g_out,
                                           ctypes.byref(h_n) if sync_count else None, _stream()))
        return (g_out[0], g_out[1], g_out[2]), (int(h_n.value) if sync_count else None)

    def build_inverse_kmap(self, fine_coords: torch.Tensor, n_fine: torch.Tensor, capacity_fine: int,
                           grid_coarse: Sequence[int], n_batch: int, coarse_slot: int, n_coarse: torch.Tensor,
                           nbr: torch.Tensor) -> None:
        """Gather table of the transposed stride-2 conv: nbr[27][capacity_fine] over the fine sites."""
        _dev_check(fine_coords, torch.int32, "fine_coords")
        _dev_check(n_fine, torch.int32, "n_fine")
        _dev_check(n_coarse, torch.int32, "n_coarse")
        _dev_check(nbr, torch.int32, "nbr")
        if fine_coords.numel() < 4 * capacity_fine or nbr.numel() < 27 * capacity_fine:
            raise ValueError("buffers smaller than capacity_fine")
        g = (ctypes.c_int32 * 3)(*grid_coarse)
        self._chk(self.lib.emc2_build_inverse_kmap(self.h, _ptr(fine_coords), _ptr(n_fine), capacity_fine, g, n_batch,
                                                   coarse_slot, _ptr(n_coarse), _ptr(nbr), _stream()))

    def bev_flatten(self, dtype: int, coords: torch.Tensor, feats: torch.Tensor, n: torch.Tensor, capacity: int,
                    grid: Sequence[int], n_batch: int, out: torch.Tensor) -> None:
        """out[B][Gy][Gx][Gz*C] <- feats[v][C] at (b, z, y, x) = coords[v], zero elsewhere."""
        td = _TORCH_DTYPE[dtype]
        _dev_check(coords, torch.int32, "coords")
        _dev_check(feats, td, "feats")
        _dev_check(out, td, "out")
        _dev_check(n, torch.int32, "n")
        c = int(feats.shape[1])
        if coords.numel() < 4 * capacity or feats.numel() < capacity * c:
            raise ValueError("coords / feats smaller than capacity")
        if out.numel() != n_batch * grid[0] * grid[1] * grid[2] * c:
            raise ValueError("out must be [n_batch][Gy][Gx][Gz*C]")
        g = (ctypes.c_int32 * 3)(*grid)
        self._chk(self.lib.emc2_bev_flatten(self.h, dtype, _ptr(coords), _ptr(feats), _ptr(n), capacity, g, n_batch, c,
                                            _ptr(out), _stream()))

    def pool_image(self, img: torch.Tensor, depth: torch.Tensor, qmat: Sequence[float], spec: VoxelSpec, mode: int,
                   capacity: int, coords: torch.Tensor, feats: torch.Tensor, counts: torch.Tensor, n_cells: torch.Tensor,
                   batch_index: int = 0, index_slot: int = 0, sync_count: bool = False) -> Optional[int]:
        """img[H][W][C] f16 + depth[H][W] f32 -> pooled cells (coords, feats[cap][C] f16, counts) on spec's grid."""
        _dev_check(img, torch.float16, "img")
        _dev_check(depth, torch.float32, "depth")
        _dev_check(coords, torch.int32, "coords")
        _dev_check(feats, torch.float16, "feats")
        _dev_check(counts, torch.int32, "counts")
        _dev_check(n_cells, torch.int32, "n_cells")
        if img.dim() != 3 or tuple(depth.shape) != tuple(img.shape[:2]):
            raise ValueError("img must be [H][W][C] and depth [H][W]")
        h, w, c = (int(v) for v in img.shape)
        if coords.numel() < 4 * capacity or feats.numel() < capacity * c or counts.numel() < capacity:
            raise ValueError("output buffers smaller than capacity")
        q = (ctypes.c_float * 12)(*[float(v) for v in qmat])
        cs = _VoxelSpecC((ctypes.c_float * 3)(*spec.lo), (ctypes.c_float * 3)(*spec.vs), (ctypes.c_int32 * 3)(*spec.grid),
                         spec.n_batch, 0.0, float("inf"), 4)
        h_n = ctypes.c_int32(0)
        self._chk(self.lib.emc2_pool_image(self.h, _ptr(img), _ptr(depth), h, w, c, q, ctypes.byref(cs), batch_index, mode,
                                           capacity, _ptr(coords), _ptr(feats), _ptr(counts), _ptr(n_cells),
                                           ctypes.byref(h_n) if sync_count else None, index_slot, _stream()))
        return int(h_n.value) if sync_count else None

    def fuse(self, dtype: int, coords_l: torch.Tensor, feats_l: torch.Tensor, n_l: torch.Tensor, capacity_l: int,
             coords_i: torch.Tensor, feats_i: torch.Tensor, n_i: torch.Tensor, capacity_i: int, grid: Sequence[int],
             n_batch: int, capacity_out: int, coords_out: torch.Tensor, feats_out: torch.Tensor, n_out: torch.Tensor,
             src_l: Optional[torch.Tensor] = None, src_i: Optional[torch.Tensor] = None, out_slot: int = 0,
             sync_count: bool = False) -> Optional[int]:
        """Union of the LiDAR voxels and the image cells, rows [LiDAR | image | zero padding up to feats_out's width]."""
        td = _TORCH_DTYPE[dtype]
        for t, nm in ((coords_l, "coords_l"), (coords_i, "coords_i"), (coords_out, "coords_out"), (n_l, "n_l"), (n_i, "n_i"),
                      (n_out, "n_out")):
            _dev_check(t, torch.int32, nm)
        for t, nm in ((feats_l, "feats_l"), (feats_i, "feats_i"), (feats_out, "feats_out")):
            _dev_check(t, td, nm)
        c_l, c_i, c_out = int(feats_l.shape[1]), int(feats_i.shape[1]), int(feats_out.shape[1])
        if coords_l.numel() < 4 * capacity_l or feats_l.numel() < capacity_l * c_l:
            raise ValueError("LiDAR buffers smaller than capacity_l")
        if coords_i.numel() < 4 * capacity_i or feats_i.numel() < capacity_i * c_i:
            raise ValueError("image buffers smaller than capacity_i")
        if coords_out.numel() < 4 * capacity_out or feats_out.numel() < capacity_out * c_out:
            raise ValueError("output buffers smaller than capacity_out")
        for t, nm in ((src_l, "src_l"), (src_i, "src_i")):
            if t is not None:
                _dev_check(t, torch.int32, nm)
                if t.numel() < capacity_out:
                    raise ValueError(f"{nm} smaller than capacity_out")
        g = (ctypes.c_int32 * 3)(*grid)
        h_n = ctypes.c_int32(0)
        self._chk(self.lib.emc2_fuse(self.h, dtype, _ptr(coords_l), _ptr(feats_l), _ptr(n_l), capacity_l, c_l, _ptr(coords_i),
                                     _ptr(feats_i), _ptr(n_i), capacity_i, c_i, g, n_batch, out_slot, capacity_out, c_out,
                                     _ptr(coords_out), _ptr(feats_out), _ptr(src_l), _ptr(src_i), _ptr(n_out),
                                     ctypes.byref(h_n) if sync_count else None, _stream()))
        return int(h_n.value) if sync_count else None

    def dispatch(self, props: torch.Tensor, scene: Optional[torch.Tensor], n_scenes: int, dist: float, conf: float,
                 expert: torch.Tensor, counts: torch.Tensor, order: torch.Tensor) -> None:
        """props[N][4] f32 (x, y, z, confidence), scene[N] i32 -> expert[S], counts[3], order[S] (scenes grouped by expert)."""
        _dev_check(props, torch.float32, "props")
        for t, nm in ((expert, "expert"), (counts, "counts"), (order, "order")):
            _dev_check(t, torch.int32, nm)
        n = int(props.shape[0]) if props.dim() == 2 else 0
        if props.dim() != 2 or props.shape[1] != 4:
            raise ValueError("props must be [N][4]")
        if scene is not None:
            _dev_check(scene, torch.int32, "scene")
            if scene.numel() != n:
                raise ValueError("scene length != number of proposals")
        if expert.numel() < n_scenes or order.numel() < n_scenes or counts.numel() < 3:
            raise ValueError("output buffers too small")
        self._chk(self.lib.emc2_dispatch(self.h, _ptr(props), _ptr(scene), n, n_scenes, dist, conf, _ptr(expert),
                                         _ptr(counts), _ptr(order), _stream()))

    def spconv_i8_supported(self, cin: int, cout: int) -> bool:
        return bool(self.lib.emc2_spconv_i8_supported(cin, cout))

    def quantize_i8(self, x: torch.Tensor, inv_scale: float, q: torch.Tensor) -> None:
        """q = clamp(rint(x * inv_scale), -127, 127) for an F32 or F16 tensor x."""
        dt = {torch.float32: F32, torch.float16: F16}[x.dtype]
        _dev_check(x, x.dtype, "x")
        _dev_check(q, torch.int8, "q")
        if q.numel() < x.numel():
            raise ValueError("q smaller than x")
        self._chk(self.lib.emc2_quantize_i8(self.h, dt, _ptr(x), x.numel(), inv_scale, _ptr(q), _stream()))

    def pack_weights_i8(self, w: torch.Tensor, packed: torch.Tensor) -> None:
        """w [27][Cin][Cout] int8 -> packed (same size) in the int8 matrix-core fragment order."""
        _dev_check(w, torch.int8, "w")
        _dev_check(packed, torch.int8, "packed")
        if w.dim() != 3 or w.shape[0] != 27 or packed.numel() != w.numel():
            raise ValueError("w must be [27][Cin][Cout] and packed the same size")
        self._chk(self.lib.emc2_pack_weights_i8(self.h, _ptr(w), int(w.shape[1]), int(w.shape[2]), _ptr(packed), _stream()))

    def spconv_i8(self, x: torch.Tensor, w_packed: torch.Tensor, cin: int, cout: int, mul: torch.Tensor, add: torch.Tensor,
                  relu: bool, nbr: torch.Tensor, n_out: torch.Tensor, capacity_out: int, out: torch.Tensor,
                  inv_out_scale: float = 0.0, n_in_rows: Optional[int] = None) -> None:
        """Quantised conv: x [n][Cin] int8, packed int8 weights, out [cap][Cout] int8 (re-quantised) or float16.
        n_in_rows: rows of x a map entry may name (default: all rows of the tensor)."""
        _dev_check(x, torch.int8, "x")
        _dev_check(w_packed, torch.int8, "w_packed")
        _dev_check(mul, torch.float32, "mul")
        _dev_check(add, torch.float32, "add")
        _dev_check(nbr, torch.int32, "nbr")
        _dev_check(n_out, torch.int32, "n_out")
        if out.dtype not in (torch.int8, torch.float16) or not out.is_cuda or not out.is_contiguous():
            raise ValueError("out must be a contiguous int8 or float16 device tensor")
        if x.dim() != 2 or x.shape[1] != cin or w_packed.numel() != 27 * cin * cout or mul.numel() != cout or add.numel() != cout:
            raise ValueError("shape mismatch")
        if out.numel() < capacity_out * cout or nbr.numel() < 27 * capacity_out:
            raise ValueError("out / nbr smaller than capacity_out")
        self._chk(self.lib.emc2_spconv_i8(self.h, _ptr(x), _ptr(w_packed), _ptr(mul), _ptr(add), int(bool(relu)),
                                          I8 if out.dtype == torch.int8 else F16, inv_out_scale, _ptr(nbr), _ptr(n_out),
                                          capacity_out, int(x.shape[0]) if n_in_rows is None else n_in_rows, cin, cout,
                                          _ptr(out), _stream()))

    def quantize_e4m3(self, x: torch.Tensor, inv_scale: float, q: torch.Tensor) -> None:
        """q[i] = E4M3 code (uint8) nearest to x[i] * inv_scale; x float32 or float16."""
        if x.dtype not in (torch.float32, torch.float16) or not x.is_cuda or not x.is_contiguous():
            raise ValueError("x must be a contiguous float32 or float16 device tensor")
        _dev_check(q, torch.uint8, "q")
        if q.numel() != x.numel():
            raise ValueError("q and x differ in size")
        self._chk(self.lib.emc2_quantize_e4m3(self.h, F32 if x.dtype == torch.float32 else F16, _ptr(x), x.numel(),
                                              inv_scale, _ptr(q), _stream()))

    def spconv_e4m3(self, x: torch.Tensor, w_packed: torch.Tensor, cin: int, cout: int, mul: torch.Tensor, add: torch.Tensor,
                    relu: bool, nbr: torch.Tensor, n_out: torch.Tensor, capacity_out: int, out: torch.Tensor,
                    n_in_rows: Optional[int] = None) -> None:
        """E4M3 conv: x [n][Cin] uint8 codes, weights packed by pack_weights_i8 (as bytes), out float32 or float16."""
        _dev_check(x, torch.uint8, "x")
        _dev_check(mul, torch.float32, "mul")
        _dev_check(add, torch.float32, "add")
        _dev_check(nbr, torch.int32, "nbr")
        _dev_check(n_out, torch.int32, "n_out")
        if w_packed.dtype not in (torch.uint8, torch.int8) or not w_packed.is_cuda or not w_packed.is_contiguous():
            raise ValueError("w_packed must be a contiguous 8-bit device tensor")
        if out.dtype not in (torch.float32, torch.float16) or not out.is_cuda or not out.is_contiguous():
            raise ValueError("out must be a contiguous float32 or float16 device tensor")
        if x.dim() != 2 or x.shape[1] != cin or w_packed.numel() != 27 * cin * cout or mul.numel() != cout or add.numel() != cout:
            raise ValueError("shape mismatch")
        if out.numel() < capacity_out * cout or nbr.numel() < 27 * capacity_out:
            raise ValueError("out / nbr smaller than capacity_out")
        self._chk(self.lib.emc2_spconv_e4m3(self.h, _ptr(x), _ptr(w_packed), _ptr(mul), _ptr(add), int(bool(relu)),
                                            F32 if out.dtype == torch.float32 else F16, _ptr(nbr), _ptr(n_out), capacity_out,
                                            int(x.shape[0]) if n_in_rows is None else n_in_rows, cin, cout, _ptr(out), _stream()))

    def uses_mfma(self, dtype: int, cin: int, cout: int) -> bool:
        return bool(self.lib.emc2_spconv_uses_mfma(dtype, cin, cout))

    def pack_weights(self, dtype: int, w: torch.Tensor, packed: torch.Tensor) -> None:
        """w [27][Cin][Cout] -> packed (same shape/dtype buffer) in MFMA fragment order."""
        td = _TORCH_DTYPE[dtype]
        _dev_check(w, td, "w")
        _dev_check(packed, td, "packed")
        if w.dim() != 3 or w.shape[0] != 27 or packed.numel() != w.numel():
            raise ValueError("w must be [27][Cin][Cout] and packed the same size")
        self._chk(self.lib.emc2_pack_weights(self.h, dtype, _ptr(w), int(w.shape[1]), int(w.shape[2]), _ptr(packed),
                                             _stream()))

    def spconv_kernel(self, dtype: int, cin: int, cout: int, map_hint: int = MAP_ANY) -> str:
        """Name of the device kernel `spconv` launches for these arguments (for matching profiles to layers)."""
        return self.lib.emc2_spconv_kernel(dtype, cin, cout, map_hint).decode()

    def spconv(self, dtype: int, x: torch.Tensor, w: torch.Tensor, scale: Optional[torch.Tensor],
               shift: Optional[torch.Tensor], epilogue: int, nbr: torch.Tensor, n_out: torch.Tensor, capacity_out: int,
               out: torch.Tensor, w_layout: int = W_PLAIN, map_hint: int = MAP_ANY, n_in_rows: Optional[int] = None) -> None:
        """n_in_rows: rows of x a map entry may name (default: all rows of the tensor)."""
        td = _TORCH_DTYPE[dtype]
        _dev_check(x, td, "x")
        _dev_check(w, td, "w")
        _dev_check(out, td, "out")
        _dev_check(nbr, torch.int32, "nbr")
        _dev_check(n_out, torch.int32, "n_out")
        if w.dim() != 3 or w.shape[0] != 27 or x.dim() != 2 or x.shape[1] != w.shape[1]:
            raise ValueError("w must be [27][Cin][Cout] and x [n][Cin]")
        cin, cout = int(w.shape[1]), int(w.shape[2])
        if out.numel() < capacity_out * cout or nbr.numel() < 27 * capacity_out:
            raise ValueError("out / nbr smaller than capacity_out")
        if scale is not None:
            _dev_check(scale, torch.float32, "scale")
            _dev_check(shift, torch.float32, "shift")
            if scale.numel() != cout or shift.numel() != cout:
                raise ValueError("scale/shift must have Cout entries")
        self._chk(self.lib.emc2_spconv(self.h, dtype, _ptr(x), _ptr(w), w_layout, _ptr(scale), _ptr(shift), epilogue, _ptr(nbr),
                                       map_hint, _ptr(n_out), capacity_out,
                                       int(x.shape[0]) if n_in_rows is None else n_in_rows, cin, cout, _ptr(out), _stream()))

    def group_points(self, scene: Optional[torch.Tensor], n_points: int, expert: torch.Tensor, order: torch.Tensor,
                     counts: torch.Tensor, n_scenes: int, e: int, slot: torch.Tensor, group_batch: torch.Tensor) -> None:
        """Dispatcher outputs -> slot[n_scenes] and, for expert e, group_batch[n_points] (-1 for other experts' points)."""
        for t, nm in ((expert, "expert"), (order, "order"), (counts, "counts"), (slot, "slot"), (group_batch, "group_batch")):
            _dev_check(t, torch.int32, nm)
        if scene is not None:
            _dev_check(scene, torch.int32, "scene")
            if scene.numel() != n_points:
                raise ValueError("scene length != n_points")
        if expert.numel() < n_scenes or order.numel() < n_scenes or counts.numel() < 3 or slot.numel() < n_scenes or \
                group_batch.numel() < n_points:
            raise ValueError("buffers smaller than n_scenes / n_points")
        self._chk(self.lib.emc2_group_points(self.h, _ptr(scene), n_points, _ptr(expert), _ptr(order), _ptr(counts), n_scenes,
                                             e, _ptr(slot), _ptr(group_batch), _stream()))

    def project_gather(self, points: torch.Tensor, pmat: Sequence[float], img: torch.Tensor, out: torch.Tensor,
                       valid: torch.Tensor, uv: Optional[torch.Tensor] = None) -> None:
        _dev_check(points, torch.float32, "points")
        _dev_check(img, torch.float16, "img")
        _dev_check(out, torch.float16, "out")
        _dev_check(valid, torch.uint8, "valid")
        n, stride = points.shape
        h, w, c = img.shape
        if out.numel() < n * c or valid.numel() < n:
            raise ValueError("out / valid too small")
        if uv is not None:
            _dev_check(uv, torch.float32, "uv")
            if uv.numel() < 2 * n:
                raise ValueError("uv too small")
        pm = (ctypes.c_float * 12)(*[float(v) for v in pmat])
        self._chk(self.lib.emc2_project_gather(self.h, _ptr(points), stride, n, pm, _ptr(img), h, w, c, _ptr(out),
                                               _ptr(valid), _ptr(uv), _stream()))
