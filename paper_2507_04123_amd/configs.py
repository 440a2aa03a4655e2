"""Workload table: the five synthetic driving-scene configurations.

Each entry fixes the cloud recipe, the voxel grids ("pool sizes" are user-configurable in the
paper's Sec. 3.5, so every grid is an explicit runtime parameter), and the sparse-conv layer stack
that stands in for the LiDAR experts' 3D CNN backbone (paper Sec. 3.1 / 3.3).  Nothing here does
any of the method's arithmetic: this is data about shapes only, shared by the HIP path, the
oracle-side tests and the bench.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

SUBM = 0      # submanifold 3x3x3, stride 1: output sites == input sites
STRIDED = 1   # regular sparse 3x3x3, stride 2, padding 1

EPI_NONE = 0
EPI_AFFINE = 1
EPI_AFFINE_RELU = 2

F32, F16, BF16 = 0, 1, 2


@dataclass(frozen=True)
class VoxelSpec:
    lo: Tuple[float, float, float]
    vs: Tuple[float, float, float]
    grid: Tuple[int, int, int]            # (Gx, Gy, Gz) -- given, never derived from (hi-lo)/vs
    n_batch: int = 1
    r2_min: float = 0.0                   # keep iff r2_min <= x^2+y^2 < r2_max
    r2_max: float = float("inf")


@dataclass(frozen=True)
class Layer:
    kind: int          # SUBM or STRIDED
    cin: int
    cout: int
    epilogue: int = EPI_AFFINE_RELU


@dataclass(frozen=True)
class Branch:
    """One voxelization followed by a stack of sparse-conv layers."""
    name: str
    spec: VoxelSpec
    layers: Tuple[Layer, ...]


@dataclass(frozen=True)
class Camera:
    height: int
    width: int
    channels: int


@dataclass(frozen=True)
class Config:
    index: int                 # 1..5
    name: str
    cloud: str                 # generator recipe id
    n_points: int              # per frame
    n_frames: int
    dtype: int                 # conv feature/weight dtype
    branches: Tuple[Branch, ...]
    camera: Optional[Camera] = None


def _stage(cin: int, cout: int) -> Tuple[Layer, ...]:
    """Stride-2 conv cin->cout followed by two submanifold convs at cout."""
    return (Layer(STRIDED, cin, cout), Layer(SUBM, cout, cout), Layer(SUBM, cout, cout))


_FRONT_LO = (0.0, -40.0, -3.0)


def _front_spec(mult: int, n_batch: int = 1, r2_min: float = 0.0,
                r2_max: float = float("inf")) -> VoxelSpec:
    """Front-view grid at `mult` times the base voxel (0.05, 0.05, 0.1) m."""
    assert mult in (1, 2, 4)
    vs = {1: (0.05, 0.05, 0.1), 2: (0.1, 0.1, 0.2), 4: (0.2, 0.2, 0.4)}[mult]
    return VoxelSpec(_FRONT_LO, vs, (1408 // mult, 1600 // mult, 40 // mult), n_batch, r2_min, r2_max)


def make_configs() -> List[Config]:
    c1 = Config(
        1, "tiny", "uniform_tiny", 2000, 1, F32,
        (Branch("l0", VoxelSpec((0.0, -10.0, -3.0), (0.2, 0.2, 0.2), (100, 100, 20)),
                (Layer(SUBM, 4, 16, EPI_NONE),)),))
    c2 = Config(
        2, "front64", "front", 120_000, 1, F16,
        (Branch("backbone", _front_spec(1),
                (Layer(SUBM, 4, 16),) + _stage(16, 32) + _stage(32, 64) + _stage(64, 64)),))
    c3 = Config(
        3, "bridge", "front", 120_000, 1, F16,
        tuple(Branch(f"scale{m}", _front_spec(m), (Layer(SUBM, 4, 16), Layer(SUBM, 16, 32)))
              for m in (1, 2, 4)),
        camera=Camera(375, 1242, 64))
    c4 = Config(
        4, "surround", "surround", 300_000, 1, F16,
        (Branch("backbone",
                VoxelSpec((-54.0, -54.0, -5.0), (0.075, 0.075, 0.2), (1440, 1440, 41)),
                (Layer(SUBM, 4, 16), Layer(SUBM, 16, 16), Layer(SUBM, 16, 16))
                + _stage(16, 32) + _stage(32, 64) + _stage(64, 128)),))
    c5 = Config(
        5, "routed8", "front", 120_000, 8, F16,
        (Branch("near", _front_spec(1, n_batch=8, r2_min=0.0, r2_max=900.0),
                (Layer(SUBM, 4, 16),) + _stage(16, 32) + _stage(32, 64)),
         Branch("far", _front_spec(2, n_batch=8, r2_min=900.0, r2_max=float("inf")),
                (Layer(SUBM, 4, 32),) + _stage(32, 64))))
    return [c1, c2, c3, c4, c5]


def expert_branches(n_scenes: int) -> Tuple[Branch, Branch, Branch]:
    """Stand-ins for the LiDAR stacks of the three experts a scene can be routed to (paper Sec. 3.2 / 3.3), indexed
    by expert id: the latency-prioritised expert works on coarse voxels with a short stack, the versatile one on
    fine voxels with two stages, the accuracy-prioritised one on fine voxels with the full three-stage backbone.
    Each runs on a batch of up to n_scenes scenes (the scenes the dispatcher routes to it)."""
    lpe = Branch("lpe", _front_spec(2, n_batch=n_scenes), (Layer(SUBM, 4, 32),) + _stage(32, 64))
    vee = Branch("vee", _front_spec(1, n_batch=n_scenes), (Layer(SUBM, 4, 16),) + _stage(16, 32) + _stage(32, 64))
    ape = Branch("ape", _front_spec(1, n_batch=n_scenes),
                 (Layer(SUBM, 4, 16),) + _stage(16, 32) + _stage(32, 64) + _stage(64, 64))
    return (lpe, vee, ape)


CONFIGS = make_configs()


def get_config(index: int) -> Config:
    return CONFIGS[index - 1]


def out_grid(grid: Tuple[int, int, int]) -> Tuple[int, int, int]:
    """Output grid of the k3 s2 p1 conv: floor((G + 2 - 3) / 2) + 1 per axis."""
    return tuple((g - 1) // 2 + 1 for g in grid)
