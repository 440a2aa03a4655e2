"""Host-side sequencing of the C-ABI calls for one workload branch: voxelize -> kernel maps -> convs.

Only call ordering and buffer ownership live here; all arithmetic is in the HIP library.  Buffers
are allocated once in ``__init__`` (sized by capacity), ``run`` allocates nothing and never syncs
with the host: voxel counts stay in device memory between calls.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

from . import binding as B
from .configs import Branch, Config, Layer, SUBM, STRIDED, F32, F16, BF16, EPI_NONE, out_grid
from . import gen

_TD = {F32: torch.float32, F16: torch.float16, BF16: torch.bfloat16}


def cells_of(grid: Sequence[int], n_batch: int) -> int:
    return int(grid[0]) * int(grid[1]) * int(grid[2]) * int(n_batch)


def default_capacities(branch: Branch, n_points: int) -> List[int]:
    """Safe per-level voxel capacities: L0 <= points; a stride-2 level holds at most 8x its input
    and at most every cell of its grid."""
    caps = [min(n_points, cells_of(branch.spec.grid, branch.spec.n_batch))]
    grid = branch.spec.grid
    for layer in branch.layers:
        if layer.kind == STRIDED:
            grid = out_grid(grid)
            caps.append(min(8 * caps[-1], cells_of(grid, branch.spec.n_batch)))
    return caps


def device_params(layers: Sequence[Layer], seed: int, dtype: int, device: str = "cuda") -> List[Dict[str, torch.Tensor]]:
    """Seeded weights / folded-BN parameters of a layer stack, rounded to `dtype`, on the device."""
    out = []
    for li, layer in enumerate(layers):
        p = gen.make_layer_params(layer, seed, li)
        out.append({
            "w": torch.from_numpy(p["w"]).to(device).to(_TD[dtype]).contiguous(),
            "scale": torch.from_numpy(p["scale"]).to(device),
            "shift": torch.from_numpy(p["shift"]).to(device),
        })
    return out


class _NoTimer:
    def __enter__(self):
        return self

    def __exit__(self, *a):
        return False


_NO_TIMER = _NoTimer()


def _no_timer(tag):
    return _NO_TIMER


@dataclass
class Level:
    grid: Tuple[int, int, int]
    cap: int
    slot: int
    coords: torch.Tensor          # [cap][4] i32
    n: torch.Tensor               # [1] i32 (device count)
    subm_nbr: Optional[torch.Tensor] = None   # [27][cap] i32, built lazily once per run
    down_nbr: Optional[torch.Tensor] = None   # map from the previous level into this one


def capture_stream(device) -> "torch.cuda.Stream":
    """A stream to record one graph capture on: a stream of its own for every capture.  Graphs recorded on one shared
    stream were measured 8-17 % slower when several of them are replayed side by side on different streams."""
    return torch.cuda.Stream(device=device)


class BranchRunner:
    """Runs one Branch (one voxelization + its conv stack) through the library."""

    def __init__(self, ctx: B.Context, branch: Branch, dtype: int, n_points: int, params: List[Dict[str, torch.Tensor]],
                 capacities: Optional[Sequence[int]] = None, slot_base: int = 0, device: str = "cuda"):
        self.ctx, self.branch, self.dtype = ctx, branch, dtype
        self.params = params
        # static weights: re-order once for the MFMA path (model-load time, not part of a frame)
        self.wdev: List[Tuple[torch.Tensor, int]] = []
        for layer, p in zip(branch.layers, params):
            if ctx.uses_mfma(dtype, layer.cin, layer.cout):
                packed = torch.empty_like(p["w"])
                ctx.pack_weights(dtype, p["w"], packed)
                self.wdev.append((packed, B.W_PACKED))
            else:
                self.wdev.append((p["w"], B.W_PLAIN))
        caps = list(capacities) if capacities is not None else default_capacities(branch, n_points)
        self.levels: List[Level] = []
        grid = tuple(branch.spec.grid)
        i32 = dict(dtype=torch.int32, device=device)
        lvl = 0
        self.levels.append(Level(grid, caps[0], slot_base, torch.empty((caps[0], 4), **i32), torch.zeros(1, **i32)))
        need_subm = [False]
        for layer in branch.layers:
            if layer.kind == STRIDED:
                lvl += 1
                grid = out_grid(grid)
                self.levels.append(Level(grid, caps[lvl], slot_base + lvl, torch.empty((caps[lvl], 4), **i32),
                                         torch.zeros(1, **i32)))
                self.levels[lvl].down_nbr = torch.empty((27, caps[lvl]), **i32)
                need_subm.append(False)
            else:
                need_subm[lvl] = True
        for lv, need in zip(self.levels, need_subm):
            if need:
                lv.subm_nbr = torch.empty((27, lv.cap), **i32)
        self.n_slots = len(self.levels)
        c0 = caps[0]
        self.feats32 = torch.empty((c0, 4), dtype=torch.float32, device=device)
        self.counts = torch.empty((c0,), dtype=torch.int32, device=device)
        self.feats_lp = torch.empty((c0, 4), dtype=_TD[dtype], device=device) if dtype != F32 else None
        # one activation buffer per layer output
        self.acts: List[torch.Tensor] = []
        lvl = 0
        for layer in branch.layers:
            if layer.kind == STRIDED:
                lvl += 1
            self.acts.append(torch.empty((self.levels[lvl].cap, layer.cout), dtype=_TD[dtype], device=device))
        # Second stream for voxelization and kernel maps.  They share the context's scratch and stay ordered
        # among themselves; the convolutions (packed weights: no context scratch) run on the caller's stream
        # and wait, per layer, only for the map they read.  Both streams keep the default priority.
        self._map_stream = None       # created on first use: torch hands streams out of a small round-robin pool
        self._device = device
        self.ev_feats = torch.cuda.Event()
        self.ev_done = None           # recorded on the caller's stream at the end of the previous overlapped run
        self.ev_subm = [torch.cuda.Event() for _ in self.levels]
        self.ev_down = [torch.cuda.Event() for _ in self.levels]
        self.can_overlap = all(lay == B.W_PACKED or not ctx.uses_mfma(dtype, l.cin, l.cout)
                               for (_, lay), l in zip(self.wdev, branch.layers))

    @property
    def map_stream(self) -> "torch.cuda.Stream":
        if self._map_stream is None:
            self._map_stream = torch.cuda.Stream(device=self._device)
        return self._map_stream

    def run_overlapped(self, points: torch.Tensor, batch: Optional[torch.Tensor], timer=None,
                       inputs_ready: Optional["torch.cuda.Event"] = None, _capturing: bool = False) -> torch.Tensor:
        """Same results as run(); map building is issued on a second stream and overlaps the convolutions.
        `timer` brackets the conv calls only (they are the ones on the caller's stream).

        The second stream waits for `inputs_ready` if given, else for everything issued so far on the caller's
        stream.  Passing an event lets two runners (two contexts) alternate frames: the maps of frame f+1 are
        then built while the convolutions of frame f still run."""
        if not self.can_overlap:
            return self.run(points, batch, timer)
        ctx, br = self.ctx, self.branch
        tm = timer if timer is not None else _no_timer
        main = torch.cuda.current_stream()
        ms = self.map_stream
        nb = br.spec.n_batch
        if inputs_ready is None:
            ms.wait_stream(main)      # inputs, and the previous frame's readers of the buffers rewritten below
        else:
            ms.wait_event(inputs_ready)
            if self.ev_done is not None:
                ms.wait_event(self.ev_done)   # this runner's previous frame: its convs read what is rewritten below
        with torch.cuda.stream(ms):
            l0 = self.levels[0]
            ctx.voxelize(points, batch, br.spec, l0.cap, l0.coords, self.feats32, self.counts, l0.n,
                         feats_lp=self.feats_lp, index_slot=l0.slot)
            self.ev_feats.record(ms)
            lvl = 0
            built = [False] * len(self.levels)
            for layer in br.layers:
                if layer.kind == STRIDED:
                    src, dst = self.levels[lvl], self.levels[lvl + 1]
                    ctx.build_kmap(B.STRIDED, src.coords, src.n, src.cap, src.grid, nb, dst.cap, dst.down_nbr, dst.n,
                                   out_coords=dst.coords, in_slot=src.slot, out_slot=dst.slot)
                    lvl += 1
                    self.ev_down[lvl].record(ms)
                elif not built[lvl]:
                    lv = self.levels[lvl]
                    ctx.build_kmap(B.SUBM, lv.coords, lv.n, lv.cap, lv.grid, nb, lv.cap, lv.subm_nbr, lv.n, in_slot=lv.slot)
                    built[lvl] = True
                    self.ev_subm[lvl].record(ms)
        main.wait_event(self.ev_feats)
        x = self.feats32 if self.dtype == F32 else self.feats_lp
        lvl = 0
        for li, layer in enumerate(br.layers):
            p = self.params[li]
            has_epi = layer.epilogue != EPI_NONE
            if layer.kind == STRIDED:
                lvl += 1
                lv = self.levels[lvl]
                main.wait_event(self.ev_down[lvl])
                nbr = lv.down_nbr
            else:
                lv = self.levels[lvl]
                main.wait_event(self.ev_subm[lvl])
                nbr = lv.subm_nbr
            y = self.acts[li]
            with tm(("conv", li)):
                ctx.spconv(self.dtype, x, self.wdev[li][0], p["scale"] if has_epi else None,
                           p["shift"] if has_epi else None, layer.epilogue, nbr, lv.n, lv.cap, y,
                           w_layout=self.wdev[li][1], map_hint=layer.kind)
            x = y
        main.wait_stream(ms)          # everything of this frame is now ordered before later work on the caller's stream
        if _capturing:
            return x
        if self.ev_done is None:
            self.ev_done = torch.cuda.Event()
        self.ev_done.record(main)
        return x

    def capture(self, points: torch.Tensor, batch: Optional[torch.Tensor], overlapped: bool = True) -> "torch.cuda.CUDAGraph":
        """Record one whole frame (both streams, with their event dependencies) into a HIP graph: a frame is
        ~50 small launches, and issuing them from the host one by one costs about as long as the GPU needs to run
        them.  The graph reads `points` / `batch` and writes this runner's buffers, as run() does; replay it with
        graph.replay() on any stream.  The library records no memset node (every clear is a kernel)."""
        side = capture_stream(points.device)
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            out = self.run_overlapped(points, batch, _capturing=True) if (overlapped and self.can_overlap) else self.run(points, batch)
        torch.cuda.current_stream().wait_stream(side)
        self.graph, self.graph_out = graph, out
        return graph

    def run(self, points: torch.Tensor, batch: Optional[torch.Tensor], timer=None) -> torch.Tensor:
        """One pass of the branch.  `timer`, if given, is called as timer(tag) and must return a context
        manager; it brackets each library call (used by the bench to time kernels with stream events)."""
        ctx, br = self.ctx, self.branch
        tm = timer if timer is not None else _no_timer
        l0 = self.levels[0]
        with tm("voxelize"):
            ctx.voxelize(points, batch, br.spec, l0.cap, l0.coords, self.feats32, self.counts, l0.n,
                         feats_lp=self.feats_lp, index_slot=l0.slot)
        x = self.feats32 if self.dtype == F32 else self.feats_lp
        lvl = 0
        built = [False] * len(self.levels)
        nb = br.spec.n_batch
        for li, layer in enumerate(br.layers):
            p = self.params[li]
            has_epi = layer.epilogue != EPI_NONE
            if layer.kind == STRIDED:
                src, dst = self.levels[lvl], self.levels[lvl + 1]
                with tm("kmap_strided"):
                    ctx.build_kmap(B.STRIDED, src.coords, src.n, src.cap, src.grid, nb, dst.cap, dst.down_nbr, dst.n,
                                   out_coords=dst.coords, in_slot=src.slot, out_slot=dst.slot)
                lvl += 1
                nbr, lv = dst.down_nbr, dst
            else:
                lv = self.levels[lvl]
                if not built[lvl]:
                    with tm("kmap_subm"):
                        ctx.build_kmap(B.SUBM, lv.coords, lv.n, lv.cap, lv.grid, nb, lv.cap, lv.subm_nbr, lv.n,
                                       in_slot=lv.slot)
                    built[lvl] = True
                nbr = lv.subm_nbr
            y = self.acts[li]
            with tm(("conv", li)):
                ctx.spconv(self.dtype, x, self.wdev[li][0], p["scale"] if has_epi else None,
                           p["shift"] if has_epi else None, layer.epilogue, nbr, lv.n, lv.cap, y,
                           w_layout=self.wdev[li][1], map_hint=layer.kind)
            x = y
        return x

    def run_maps(self, points: torch.Tensor, batch: Optional[torch.Tensor], timer=None) -> None:
        """First stage of a pass, on the current stream: voxelization and every kernel map of the branch (all the
        work that uses the context's scratch).  run_convs() is the second stage; together they do what run() does,
        with every map built before the first convolution."""
        ctx, br = self.ctx, self.branch
        tm = timer if timer is not None else _no_timer
        l0 = self.levels[0]
        with tm("voxelize"):
            ctx.voxelize(points, batch, br.spec, l0.cap, l0.coords, self.feats32, self.counts, l0.n,
                         feats_lp=self.feats_lp, index_slot=l0.slot)
        lvl = 0
        built = [False] * len(self.levels)
        nb = br.spec.n_batch
        for layer in br.layers:
            if layer.kind == STRIDED:
                src, dst = self.levels[lvl], self.levels[lvl + 1]
                with tm("kmap_strided"):
                    ctx.build_kmap(B.STRIDED, src.coords, src.n, src.cap, src.grid, nb, dst.cap, dst.down_nbr, dst.n,
                                   out_coords=dst.coords, in_slot=src.slot, out_slot=dst.slot)
                lvl += 1
            elif not built[lvl]:
                lv = self.levels[lvl]
                with tm("kmap_subm"):
                    ctx.build_kmap(B.SUBM, lv.coords, lv.n, lv.cap, lv.grid, nb, lv.cap, lv.subm_nbr, lv.n, in_slot=lv.slot)
                built[lvl] = True

    def run_convs(self, timer=None) -> torch.Tensor:
        """Second stage of a pass, on the current stream: every convolution of the branch over the voxels and kernel
        maps run_maps() left in this runner's buffers.  Uses no context scratch when the weights are packed, so it
        may overlap the first stage of another runner."""
        ctx, br = self.ctx, self.branch
        tm = timer if timer is not None else _no_timer
        x = self.feats32 if self.dtype == F32 else self.feats_lp
        lvl = 0
        for li, layer in enumerate(br.layers):
            p = self.params[li]
            has_epi = layer.epilogue != EPI_NONE
            if layer.kind == STRIDED:
                lvl += 1
                lv = self.levels[lvl]
                nbr = lv.down_nbr
            else:
                lv = self.levels[lvl]
                nbr = lv.subm_nbr
            y = self.acts[li]
            with tm(("conv", li)):
                ctx.spconv(self.dtype, x, self.wdev[li][0], p["scale"] if has_epi else None,
                           p["shift"] if has_epi else None, layer.epilogue, nbr, lv.n, lv.cap, y,
                           w_layout=self.wdev[li][1], map_hint=layer.kind)
            x = y
        return x

    def layer_map(self, li: int) -> Tuple[torch.Tensor, "Level"]:
        """Kernel map and output level used by layer `li` (valid after a run)."""
        lvl = 0
        for j, layer in enumerate(self.branch.layers[: li + 1]):
            if layer.kind == STRIDED:
                lvl += 1
        lv = self.levels[lvl]
        return (lv.down_nbr if self.branch.layers[li].kind == STRIDED else lv.subm_nbr), lv


def make_context_for(cfg: Config, capacities: Optional[Dict[str, Sequence[int]]] = None) -> Tuple[B.Context, int]:
    """Context sized for every branch of a config: returns (ctx, total points)."""
    n_points = cfg.n_points * cfg.n_frames
    max_cells = max(cells_of(b.spec.grid, b.spec.n_batch) for b in cfg.branches)
    max_vox = 1
    n_slots = 1
    for b in cfg.branches:
        caps = capacities[b.name] if capacities and b.name in capacities else default_capacities(b, n_points)
        max_vox = max(max_vox, max(caps))
        n_slots = max(n_slots, len(caps))
    return B.Context(n_points, max_vox, max_cells, n_slots=n_slots), n_points


class ConfigRunner:
    """Every branch of one workload configuration (config 3: three scales plus the point-to-image gather; config 5:
    the near and the far expert), each on a context of its own so that the branches of one frame can share the GPU.
    Only sequencing: one pass = every branch's voxelization, kernel maps and convolutions over the same points."""

    def __init__(self, cfg: Config, n_points: int, capacities: Optional[Dict[str, Sequence[int]]] = None,
                 device: str = "cuda"):
        self.cfg = cfg
        self.n_points = n_points
        self.branches: List[Tuple[B.Context, BranchRunner]] = []
        for br in cfg.branches:
            caps = list(capacities[br.name]) if capacities and br.name in capacities else default_capacities(br, n_points)
            ctx = B.Context(n_points, max(caps), cells_of(br.spec.grid, br.spec.n_batch), n_slots=len(caps))
            seed = gen.frame_seed(cfg.index, 0) + len(br.name)
            self.branches.append((ctx, BranchRunner(ctx, br, cfg.dtype, n_points, device_params(br.layers, seed, cfg.dtype),
                                                    capacities=caps, device=device)))
        self._side: List["torch.cuda.Stream"] = []
        self._device = device
        self.camera = None
        if cfg.camera is not None:
            cam, seed = cfg.camera, gen.frame_seed(cfg.index, 0)
            self.camera = {
                "P": gen.make_camera(seed),
                "img": torch.from_numpy(gen.make_image(cam.height, cam.width, cam.channels, seed)).to(device),
                "out": torch.empty((n_points, cam.channels), dtype=torch.float16, device=device),
                "valid": torch.empty((n_points,), dtype=torch.uint8, device=device),
            }
        self.graph = None
        self.flat_graph = None
        self.ev_maps = torch.cuda.Event()
        self.ev_convs = [torch.cuda.Event() for _ in self.branches]
        self.stages_in_flight = False

    def close(self) -> None:
        for ctx, _ in self.branches:
            ctx.close()

    def status_sync(self) -> None:
        for ctx, _ in self.branches:
            ctx.status_sync()

    @property
    def side(self) -> List["torch.cuda.Stream"]:
        """Streams of the branches after the first when branches run side by side (created on first use)."""
        if not self._side:
            self._side = [torch.cuda.Stream(device=self._device) for _ in self.branches[1:]]
        return self._side

    def _gather(self, points: torch.Tensor, tm) -> None:
        if self.camera is not None:
            c = self.camera
            with tm("project_gather"):
                self.branches[0][0].project_gather(points, c["P"], c["img"], c["out"], c["valid"])

    def run(self, points: torch.Tensor, batch: Optional[torch.Tensor], timer=None) -> List[torch.Tensor]:
        """Everything on the current stream, one call after the other."""
        tm = timer if timer is not None else _no_timer
        outs = []
        for bi, (_, r) in enumerate(self.branches):
            outs.append(r.run(points, batch, (lambda tag, bi=bi: tm((bi, tag))) if timer is not None else None))
        self._gather(points, tm)
        return outs

    def run_overlapped(self, points: torch.Tensor, batch: Optional[torch.Tensor], timer=None) -> List[torch.Tensor]:
        """Branches side by side: the first on the current stream, the others on streams of their own that fork
        from it and join it again; inside a branch, map building overlaps the convolutions as in BranchRunner."""
        tm = timer if timer is not None else _no_timer
        main = torch.cuda.current_stream()
        outs: List[Optional[torch.Tensor]] = [None] * len(self.branches)
        for bi, (_, r) in enumerate(self.branches[1:], start=1):
            s = self.side[bi - 1]
            s.wait_stream(main)
            with torch.cuda.stream(s):
                outs[bi] = r.run_overlapped(points, batch, (lambda tag, bi=bi: tm((bi, tag))) if timer is not None else None,
                                            _capturing=True)
        outs[0] = self.branches[0][1].run_overlapped(points, batch, (lambda tag: tm((0, tag))) if timer is not None else None,
                                                     _capturing=True)
        self._gather(points, tm)
        for s in self.side:
            main.wait_stream(s)
        return outs

    def capture(self, points: torch.Tensor, batch: Optional[torch.Tensor], overlapped: bool = True) -> None:
        """Record one HIP graph per branch (BranchRunner.capture: the branch's two streams with their events, no
        memset nodes); replay() then launches them side by side.  One graph per branch, not one for the whole
        configuration: a capture in which a forked stream forks again (branch stream -> its map stream) ended in a
        crash inside the runtime's end-of-capture on this ROCm, whereas a single level of forking is what the
        per-branch graphs have always used."""
        self.graph_points = points
        if not overlapped:
            # the whole pass in launch order on one stream: a graph without forks
            side = capture_stream(points.device)
            side.wait_stream(torch.cuda.current_stream())
            self.flat_graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(self.flat_graph, stream=side):
                self.graph_out = self.run(points, batch)
            torch.cuda.current_stream().wait_stream(side)
            self.graph = True
            return
        self.flat_graph = None
        for _, r in self.branches:
            r.capture(points, batch, overlapped=True)
        self.graph_out = [r.graph_out for _, r in self.branches]
        self.graph = True

    def capture_stages(self, points: torch.Tensor, batch: Optional[torch.Tensor]) -> None:
        """The pass as two stages, for pipelining across batches: one fork-free graph with every branch's
        voxelization and kernel maps (and the point-to-image gather), and one fork-free graph per branch with its
        convolutions.  replay_stages() launches them on a map stream and on one conv stream per branch, so that the
        first stage of the next batch (another runner, another context) runs under the convolutions of this one."""
        assert all(r.can_overlap for _, r in self.branches), "the conv stage must not use context scratch"
        cur = torch.cuda.current_stream()

        def grab(fn):
            side = capture_stream(points.device)
            side.wait_stream(cur)
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                out = fn()
            cur.wait_stream(side)
            return g, out

        def maps():
            for _, r in self.branches:
                r.run_maps(points, batch)
            self._gather(points, _no_timer)

        self.stage_maps, _ = grab(maps)
        self.stage_convs, self.graph_out = [], []
        for _, r in self.branches:
            g, out = grab(r.run_convs)
            self.stage_convs.append(g)
            self.graph_out.append(out)
        self.graph_points = points

    def replay_stages(self, map_stream: "torch.cuda.Stream", conv_streams: Sequence["torch.cuda.Stream"]) -> List[torch.Tensor]:
        """One pass from the staged graphs.  The maps wait for this runner's previous convolutions (they rewrite what
        those read); each branch's convolutions wait for the maps."""
        if self.stages_in_flight:
            for ev in self.ev_convs:
                map_stream.wait_event(ev)
        with torch.cuda.stream(map_stream):
            self.stage_maps.replay()
            self.ev_maps.record(map_stream)
        for bi, g in enumerate(self.stage_convs):
            cs = conv_streams[bi % len(conv_streams)]
            cs.wait_event(self.ev_maps)
            with torch.cuda.stream(cs):
                g.replay()
                self.ev_convs[bi].record(cs)
        self.stages_in_flight = True
        return self.graph_out

    def run_stages(self, points: torch.Tensor, batch: Optional[torch.Tensor], map_stream: "torch.cuda.Stream",
                   conv_streams: Sequence["torch.cuda.Stream"], timer=None) -> List[torch.Tensor]:
        """replay_stages() issued from the host, call by call (same streams, same events; `timer` brackets the calls)."""
        tm = timer if timer is not None else _no_timer
        if self.stages_in_flight:
            for ev in self.ev_convs:
                map_stream.wait_event(ev)
        with torch.cuda.stream(map_stream):
            for bi, (_, r) in enumerate(self.branches):
                r.run_maps(points, batch, (lambda tag, bi=bi: tm((bi, tag))) if timer is not None else None)
            self._gather(points, tm)
            self.ev_maps.record(map_stream)
        outs = []
        for bi, (_, r) in enumerate(self.branches):
            cs = conv_streams[bi % len(conv_streams)]
            cs.wait_event(self.ev_maps)
            with torch.cuda.stream(cs):
                outs.append(r.run_convs((lambda tag, bi=bi: tm((bi, tag))) if timer is not None else None))
                self.ev_convs[bi].record(cs)
        self.stages_in_flight = True
        return outs

    def replay(self) -> List[torch.Tensor]:
        """Replay the captured graphs: the first branch on the current stream, the others on streams of their own
        that fork from it and join it again (ordinary stream and event calls, outside any capture)."""
        if self.flat_graph is not None:
            self.flat_graph.replay()
            return self.graph_out
        main = torch.cuda.current_stream()
        for bi, (_, r) in enumerate(self.branches[1:], start=1):
            s = self.side[bi - 1]
            s.wait_stream(main)
            with torch.cuda.stream(s):
                r.graph.replay()
        self.branches[0][1].graph.replay()
        self._gather(self.graph_points, _no_timer)
        for s in self.side:
            main.wait_stream(s)
        return self.graph_out


class RoutedRunner:
    """Scene-level routing (paper Sec. 3.2): the dispatcher picks an expert per scene from the scene's proposal
    regions, the scenes are grouped by expert, and each expert's stack runs on its own group only.  Sequencing
    only: emc2_dispatch -> per expert emc2_group_points -> that expert's BranchRunner with the group's batch ids
    (points of other experts' scenes carry -1 and are dropped by the voxelizer).  Group sizes stay on the device:
    every expert's buffers are sized for all n_scenes, and nothing here waits for the host."""

    def __init__(self, experts: Sequence[Branch], dtype: int, n_points: int, n_scenes: int, seed: int, device: str = "cuda"):
        self.n_points, self.n_scenes = n_points, n_scenes
        i32 = dict(dtype=torch.int32, device=device)
        self.expert = torch.zeros((n_scenes,), **i32)
        self.counts = torch.zeros((3,), **i32)
        self.order = torch.zeros((n_scenes,), **i32)
        self.slot = torch.zeros((n_scenes,), **i32)
        self.runners: List[Tuple[B.Context, BranchRunner]] = []
        self.group_batch: List[torch.Tensor] = []
        for e, br in enumerate(experts):
            assert br.spec.n_batch == n_scenes
            caps = default_capacities(br, n_points)
            ctx = B.Context(n_points, max(caps), cells_of(br.spec.grid, n_scenes), n_slots=len(caps))
            self.runners.append((ctx, BranchRunner(ctx, br, dtype, n_points, device_params(br.layers, seed + e, dtype),
                                                   capacities=caps, device=device)))
            self.group_batch.append(torch.empty((n_points,), **i32))

    def close(self) -> None:
        for ctx, _ in self.runners:
            ctx.close()

    def status_sync(self) -> None:
        for ctx, _ in self.runners:
            ctx.status_sync()

    def capture(self, points: torch.Tensor, scene: torch.Tensor, props: torch.Tensor, prop_scene: Optional[torch.Tensor],
                dist: float, conf: float) -> None:
        """Record one routed pass (dispatch, grouping, every expert's stack) as one fork-free HIP graph.  The graph reads
        the four input tensors in place: new proposals, scene ids and points are written into them before replay();
        their sizes (number of proposals included) and the two thresholds are those of the capture."""
        cur = torch.cuda.current_stream()
        side = capture_stream(points.device)
        side.wait_stream(cur)
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph, stream=side):
            self.graph_out = self.run(points, scene, props, prop_scene, dist, conf)
        cur.wait_stream(side)

    def replay(self) -> List[torch.Tensor]:
        self.graph.replay()
        return self.graph_out

    def run(self, points: torch.Tensor, scene: torch.Tensor, props: torch.Tensor, prop_scene: Optional[torch.Tensor],
            dist: float, conf: float) -> List[torch.Tensor]:
        ctx0 = self.runners[0][0]
        ctx0.dispatch(props, prop_scene, self.n_scenes, dist, conf, self.expert, self.counts, self.order)
        outs = []
        for e, (ctx, r) in enumerate(self.runners):
            ctx.group_points(scene, self.n_points, self.expert, self.order, self.counts, self.n_scenes, e, self.slot,
                             self.group_batch[e])
            outs.append(r.run(points, self.group_batch[e]))
        return outs
