"""Shared test helpers: the oracle-side chain of a workload branch and the feature tolerance."""
from __future__ import annotations

import os
from typing import Dict, List, Tuple

import numpy as np

import oracle
from paper_2507_04123_amd import gen
from paper_2507_04123_amd.configs import Branch, SUBM, STRIDED, EPI_NONE, F32


def assert_features_close(got: np.ndarray, exp: np.ndarray, rtol: float, what: str = "") -> None:
    """|g - o| <= rtol * (|o| + rms(o)) for every element (scale-aware relative tolerance)."""
    got = np.asarray(got, dtype=np.float64)
    exp = np.asarray(exp, dtype=np.float64)
    assert got.shape == exp.shape, f"{what}: shape {got.shape} vs {exp.shape}"
    if exp.size == 0:
        return
    assert np.all(np.isfinite(got)), f"{what}: non-finite values in the GPU result"
    rms = float(np.sqrt(np.mean(exp * exp)))
    err = np.abs(got - exp)
    bound = rtol * (np.abs(exp) + rms)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())}/{exp.size} elements outside rtol={rtol}; worst at {i}: "
                             f"got {got[i]!r} exp {exp[i]!r} rms {rms:.4g}")


_PROGRESS_LOG = os.environ.get("EMC2_PROGRESS_LOG", "")


def progress(msg: str) -> None:
    """A progress line of a long test: printed, and appended to the file EMC2_PROGRESS_LOG names, if any, for a job
    monitor to watch (pytest holds back what a passing test prints)."""
    print(msg, flush=True)
    if not _PROGRESS_LOG:
        return
    try:
        with open(_PROGRESS_LOG, "a") as f:
            f.write(msg + "\n")
    except OSError:
        pass


def worst_feature_ratio(got: np.ndarray, exp: np.ndarray) -> float:
    """max |g - o| / (|o| + rms(o)): the smallest rtol at which assert_features_close would pass."""
    got = np.asarray(got, dtype=np.float64)
    exp = np.asarray(exp, dtype=np.float64)
    if exp.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(exp * exp)))
    return float(np.max(np.abs(got - exp) / (np.abs(exp) + rms)))


def layer_params_host(branch: Branch, seed: int, dtype: int) -> List[Dict[str, np.ndarray]]:
    """Same seeded parameters as the device side, weights rounded to `dtype` and up-cast to fp32."""
    out = []
    for li, layer in enumerate(branch.layers):
        p = gen.make_layer_params(layer, seed, li)
        out.append({"w": gen.round_to_dtype(p["w"], dtype), "scale": p["scale"], "shift": p["shift"]})
    return out


def oracle_branch(points: np.ndarray, batch, branch: Branch, dtype: int, params) -> Dict[str, list]:
    """Oracle chain: voxelize -> maps -> convs with fp32 activations between layers (the first
    layer's input is the mean feature rounded to `dtype`, as the 16-bit path consumes it)."""
    sp = branch.spec
    coords, means, counts = oracle.voxelize(points, batch, sp.lo, sp.vs, sp.grid, sp.n_batch, sp.r2_min, sp.r2_max)
    levels = [{"coords": coords, "grid": tuple(sp.grid), "subm": None}]
    x = gen.round_to_dtype(means, dtype)
    acts, maps = [], []
    for li, layer in enumerate(branch.layers):
        p = params[li]
        cur = levels[-1]
        if layer.kind == STRIDED:
            out_coords, nbr, gout = oracle.build_kmap(1, cur["coords"], cur["grid"], sp.n_batch)
            levels.append({"coords": out_coords, "grid": gout, "subm": None, "down": nbr})
        else:
            if cur["subm"] is None:
                _, cur["subm"], _ = oracle.build_kmap(0, cur["coords"], cur["grid"], sp.n_batch)
            nbr = cur["subm"]
        epi = layer.epilogue
        x = oracle.spconv(x, p["w"], p["scale"] if epi != EPI_NONE else None, p["shift"] if epi != EPI_NONE else None,
                          epi, nbr)
        acts.append(x)
        maps.append(nbr)
    return {"levels": levels, "means": means, "counts": counts, "acts": acts, "maps": maps}


def make_scene(seed, h=60, w=200, c=6, proposals=False):
    """A crop of the camera scene around the principal point: (pmat, qmat, depth[h][w] f32, img[h][w][c] f16)."""
    pm = gen.make_camera(seed).astype(np.float64).reshape(3, 4).copy()
    pm[0] += pm[2] * (w / 2 - 620.5)          # move the principal point to the crop's centre column
    pm[1] += pm[2] * (h / 3 - 187.0)          # and to a third of its height (the horizon)
    pm = pm.astype(np.float32).reshape(12)
    full = gen.make_depth(375, 1242, seed, proposals)
    r0, c0 = 187 - h // 3, 620 - w // 2
    depth = np.ascontiguousarray(full[r0:r0 + h, c0:c0 + w])
    img = gen.make_image(h, w, c, seed)
    return pm, gen.make_unprojection(pm), depth, img
