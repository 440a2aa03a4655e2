#!/usr/bin/env python3
"""Bench: frames/s through voxelize + kernel maps + sparse-conv backbone on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input, already resident in HBM.  The
headline workload is the largest single-GPU configuration, config 5 (eight front-view frames in one batch,
960 k points, routed by range to a near and a far expert: 2 voxelizations, 8 kernel maps, 11 convs per step);
`value` = 8 frames / step time.  The other four configurations are measured the same way and listed under
`per_config`.  Prints ONE JSON line with the throughput, a `roofline` object for the dominant kernel (its own
launch duration, event-bracketed with the GPU to itself; the figure under sharing, bracketed inside the timed
steps, beside it) and a `cpu_baseline` object (the CPU oracle on this machine's host cores).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F16_TFLOPS = 2500.0      # MI355X dense fp16/bf16 MFMA, published
PEAK_HBM_GBS = 8000.0              # MI355X HBM3E, published
PEAK_VALU_F32_TFLOPS = 157.3       # MI355X fp32 vector ALU, published (256 CUs x 128 lanes x 2 flop x 2.4 GHz)
DTYPE_NAME = {0: "f32", 1: "f16", 2: "bf16"}   # the arithmetic type of the conv operands (accumulation is fp32)


# ----------------------------------------------------------------------------------------------------------
# timing helpers
# ----------------------------------------------------------------------------------------------------------

class EventTimer:
    """Brackets library calls with events on the stream they are launched on (torch's current stream)."""

    def __init__(self, torch):
        self.torch = torch
        self.records = []           # (tag, start_event, stop_event)
        self.enabled = False
        self.only = None            # None = bracket every call; else the set of tags to bracket

    def __call__(self, tag):
        if not self.enabled or (self.only is not None and tag not in self.only):
            return _NULL_SPAN
        return _Span(self, tag)

    def reset(self):
        self.records = []


class _NullSpan:
    def __enter__(self):
        return self

    def __exit__(self, *a):
        return False


_NULL_SPAN = _NullSpan()


class _Span:
    def __init__(self, timer, tag):
        self.t, self.tag = timer, tag

    def __enter__(self):
        self.e0 = self.t.torch.cuda.Event(enable_timing=True)
        self.e1 = self.t.torch.cuda.Event(enable_timing=True)
        self.e0.record()
        return self

    def __exit__(self, *a):
        self.e1.record()
        self.t.records.append((self.tag, self.e0, self.e1))
        return False


def percentiles(xs):
    import numpy as np
    a = np.sort(np.asarray(xs, dtype=np.float64))
    if a.size == 0:
        return None
    return {"median": float(np.median(a)), "p10": float(np.percentile(a, 10)), "p90": float(np.percentile(a, 90)),
            "min": float(a[0]), "max": float(a[-1]), "n": int(a.size)}


def timed_loop(torch, fn, reps=20, warm=3):
    """Mean ms per call of `fn` over `reps` back-to-back calls on the current stream."""
    for _ in range(warm):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def profiled_traffic(kernel, config_index):
    """HBM bytes per launch of `kernel` from the committed counter summary (rocprofv3 --pmc FETCH_SIZE and
    WRITE_SIZE runs of this same bench, scaled by a known-size copy); None if no summary covers it."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_config{config_index}_pmc_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


# ----------------------------------------------------------------------------------------------------------
# measured ceilings of the part (probe kernels of libemc2probe.so)
# ----------------------------------------------------------------------------------------------------------

def measure_probes(torch):
    """Empty-launch floor (eager and inside a HIP graph), plain-copy bandwidth and a dense fp16 MFMA loop."""
    path = os.path.join(ROOT, "paper_2507_04123_amd", "libemc2probe.so")
    lib = ctypes.CDLL(path)
    vp = ctypes.c_void_p
    lib.emc2_probe_empty.argtypes = [ctypes.c_int32, vp]
    lib.emc2_probe_copy.argtypes = [vp, vp, ctypes.c_int64, vp]
    lib.emc2_probe_mfma_f16.argtypes = [ctypes.c_int64, ctypes.c_int32, vp, vp]
    lib.emc2_probe_fill.argtypes = [vp, ctypes.c_int64, vp]
    lib.emc2_probe_atomic.argtypes = [vp, ctypes.c_int32, ctypes.c_int64, vp]
    out = {}
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        sp = vp(s.cuda_stream)
        # eager: host issue + device dispatch of back-to-back empty kernels
        lib.emc2_probe_empty(200, sp)
        s.synchronize()
        t0 = time.perf_counter()
        lib.emc2_probe_empty(2000, sp)
        t_issue = time.perf_counter() - t0
        s.synchronize()
        t_all = time.perf_counter() - t0
        out["empty_launch_eager_us"] = {"host_issue": t_issue / 2000 * 1e6, "issue_to_drain": t_all / 2000 * 1e6}
        # inside a HIP graph: what a dependent chain of launches costs on the device alone
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            lib.emc2_probe_empty(500, vp(torch.cuda.current_stream().cuda_stream))
        g.replay()
        s.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(s)
        for _ in range(4):
            g.replay()
        e1.record(s)
        s.synchronize()
        out["empty_launch_in_graph_us"] = e0.elapsed_time(e1) * 1e3 / 2000
        # plain copy, 1 GiB each way
        nbytes = 1 << 30
        src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        ms = timed_loop(torch, lambda: lib.emc2_probe_copy(vp(dst.data_ptr()), vp(src.data_ptr()), nbytes, sp), reps=10)
        out["copy_GBs"] = 2.0 * nbytes / (ms * 1e-3) / 1e9
        out["copy_frac_of_hbm_peak"] = out["copy_GBs"] / PEAK_HBM_GBS
        ms = timed_loop(torch, lambda: lib.emc2_probe_fill(vp(dst.data_ptr()), nbytes, sp), reps=10)
        out["fill_GBs"] = nbytes / (ms * 1e-3) / 1e9
        # scattered atomics: 4 M of them on a 64 MiB table (the rate does not depend on the table's size)
        n_at = 4 << 20
        ms = timed_loop(torch, lambda: lib.emc2_probe_atomic(vp(dst.data_ptr()), 24, n_at, sp), reps=10)
        out["random_atomics_G_per_s"] = n_at / (ms * 1e-3) / 1e9
        del src, dst
        # dense MFMA loop: 2 blocks of 4 waves per CU (2 waves per SIMD)
        blocks, iters = 512, 20000
        sink = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
        ms = timed_loop(torch, lambda: lib.emc2_probe_mfma_f16(iters, blocks, vp(sink.data_ptr()), sp), reps=5, warm=1)
        flops = blocks * 4 * iters * 8 * 2.0 * 32 * 32 * 16
        out["mfma_f16_dense_TFLOPs"] = flops / (ms * 1e-3) / 1e12
        out["mfma_frac_of_published_peak"] = out["mfma_f16_dense_TFLOPs"] / PEAK_MFMA_F16_TFLOPS
    torch.cuda.synchronize()
    return out


# ----------------------------------------------------------------------------------------------------------
# the CPU oracle as it stands, on the same workload
# ----------------------------------------------------------------------------------------------------------

def cpu_baseline(cfg, pts_np, batch_np, threads, single_thread_sample=True):
    """Whole batch on `threads` host threads (voxelize + kernel maps + convs of every branch, + the image gather
    of config 3), and one frame of it single-threaded (the configuration the parity tests pin)."""
    import numpy as np
    import oracle
    from paper_2507_04123_amd import gen
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import layer_params_host, oracle_branch

    def one_pass(p, b):
        t0 = time.perf_counter()
        for br in cfg.branches:
            hp = layer_params_host(br, gen.frame_seed(cfg.index, 0) + len(br.name), cfg.dtype)
            oracle_branch(p, b, br, cfg.dtype, hp)
        if cfg.camera is not None:
            cam, seed = cfg.camera, gen.frame_seed(cfg.index, 0)
            oracle.project_gather(p, gen.make_camera(seed), gen.make_image(cam.height, cam.width, cam.channels, seed))
        return time.perf_counter() - t0

    oracle.set_threads(threads)
    b_all = batch_np if cfg.n_frames > 1 else None
    dt = one_pass(pts_np, b_all)
    out = {"value": cfg.n_frames / dt, "unit": "frames/s", "cores": threads, "kind": "oracle",
           "sample": f"the whole batch of config {cfg.index} ({cfg.n_frames} frame(s), {len(pts_np)} points, every branch), "
                     f"{dt:.2f} s on {threads} threads", "ms_per_frame": dt * 1e3 / cfg.n_frames}
    if single_thread_sample:
        oracle.set_threads(1)
        if cfg.n_frames > 1:
            sel = batch_np == 0
            p1, b1 = np.ascontiguousarray(pts_np[sel]), np.ascontiguousarray(batch_np[sel])
        else:
            p1, b1 = pts_np, None
        dt1 = one_pass(p1, b1)
        out["single_thread"] = {"value": 1.0 / dt1, "unit": "frames/s", "cores": 1,
                                "sample": f"frame 0 of the batch ({len(p1)} points, every branch), {dt1:.2f} s"}
        oracle.set_threads(threads)
    return out


# ----------------------------------------------------------------------------------------------------------
# one configuration: throughput, calibration, roofline of its dominant kernel
# ----------------------------------------------------------------------------------------------------------

_REPLAY_STREAMS = []


def replay_stream(torch, k):
    """The k-th of the streams the batches in flight are replayed on: created once, first, and shared by every
    configuration measured in this process.  The runtime spreads streams over a handful of hardware queues as they
    appear; two replay streams that land on one queue serialise their batches, which a later configuration's fresh
    streams did more often than the first one's."""
    while len(_REPLAY_STREAMS) <= k:
        _REPLAY_STREAMS.append(torch.cuda.Stream())
    return _REPLAY_STREAMS[k]


def measure_config(cfg_index, args, steps, warmup, full):
    """`full`: also the step-time distribution, the cold-cache pass and the repeated regions (headline only)."""
    import numpy as np
    import torch
    from paper_2507_04123_amd import gen
    from paper_2507_04123_amd.configs import get_config, STRIDED
    from paper_2507_04123_amd.pipeline import ConfigRunner

    cfg = get_config(cfg_index)
    pts_np, batch_np = gen.make_frames(cfg)
    n_points = len(pts_np)
    pts = torch.from_numpy(pts_np).cuda()
    batch = torch.from_numpy(batch_np).cuda() if cfg.n_frames > 1 else None

    depth = 1 if args.serial else args.frames_in_flight
    ring = []                        # one set of contexts, buffers and streams per batch in flight
    for _ in range(depth):
        r = ConfigRunner(cfg, n_points)
        r.in_pts = pts.clone()       # the buffers this runner's graph reads (refilled in the cold-cache pass)
        r.in_batch = batch.clone() if batch is not None else None
        r.run(r.in_pts, r.in_batch)
        r.status_sync()
        r.stream = replay_stream(torch, len(ring))
        ring.append(r)
    torch.cuda.synchronize()
    runner = ring[0]

    # flop / byte accounting from the kernel maps of this batch (outside the timed region)
    layers = []                      # (branch index, layer index, Layer, pairs, flops)
    layer_bytes = {}                 # ideal-reuse HBM bytes of a layer: features in and out, kernel map, weights
    vox = []
    for bi, (ctx, br) in enumerate(runner.branches):
        vox.append([int(lv.n.item()) for lv in br.levels])
        lvl = 0
        for li, layer in enumerate(br.branch.layers):
            nbr, lv = br.layer_map(li)
            n = int(lv.n.item())
            n_in_rows = vox[bi][lvl]
            if layer.kind == STRIDED:
                lvl += 1
            pairs = int((nbr[:, :n] >= 0).sum().item())
            layers.append((bi, li, layer, pairs, 2.0 * pairs * layer.cin * layer.cout))
            esz = 4 if cfg.dtype == 0 else 2
            layer_bytes[(bi, li)] = n_in_rows * layer.cin * esz + n * layer.cout * esz + 27.0 * n * 4 + 27.0 * layer.cin * layer.cout * esz
    total_flops = sum(l[4] for l in layers)
    ctx0 = runner.branches[0][0]

    use_graphs = not args.no_graphs
    # two-stage pipeline across batches: maps of the next batch under the convolutions of this one
    can_stage = use_graphs and not args.serial and not args.branch_graphs and depth >= 2 and \
        all(br.can_overlap for r in ring for _, br in r.branches)
    want = args.launch_shape if can_stage else "batches"
    if want == "auto":
        # The staged form costs ~0.2 ms more host time per step (three graph launches and their events instead of
        # one) and runs two or three streams instead of `depth`: it pays where a step is long and has several
        # branches (config 5: +2 %), and loses on short steps (config 3: half the throughput).
        want = "stages" if len(runner.branches) >= 2 and n_points >= 500_000 else "batches"
    map_stream = replay_stream(torch, 0)
    nb_ = len(runner.branches)
    # every batch in flight has conv streams of its own (one per branch); the maps of all batches share one stream
    # (two map streams were measured slower: 4 240 against 4 760 frames/s on config 5)
    conv_sets = [[replay_stream(torch, 1 + k * nb_ + bi) for bi in range(nb_)] for k in range(depth)]
    if use_graphs:
        for r in ring:
            with torch.cuda.stream(r.stream):
                if want == "stages":
                    r.capture_stages(r.in_pts, r.in_batch)
                else:
                    r.capture(r.in_pts, r.in_batch, overlapped=args.branch_graphs and not args.serial)
        torch.cuda.synchronize()
    staged = want == "stages"

    step_no = [0]

    def step(tm=None):
        """One pass over one batch on the next runner of the ring; bracketed (eager) when `tm` is enabled."""
        r = ring[step_no[0] % depth]
        step_no[0] += 1
        if staged:
            k_ = (step_no[0] - 1) % depth
            if use_graphs and (tm is None or not tm.enabled):
                r.replay_stages(map_stream, conv_sets[k_])
            else:
                r.run_stages(r.in_pts, r.in_batch, map_stream, conv_sets[k_], tm)
            return
        with torch.cuda.stream(r.stream):
            if use_graphs and (tm is None or not tm.enabled):
                r.replay()
            elif args.serial or (use_graphs and not args.branch_graphs):
                r.run(r.in_pts, r.in_batch, tm)          # the launch order the graph holds, issued from the host
            else:
                r.run_overlapped(r.in_pts, r.in_batch, tm)

    timer = EventTimer(torch)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    if args.config_result_only:
        # a child process measuring one of the small configurations starts on an idle GPU and its whole timed region
        # lasts a millisecond or two: keep stepping (untimed) until the clocks have come up
        t_w = time.perf_counter()
        while time.perf_counter() - t_w < 0.05:
            for _ in range(depth):
                step()
            torch.cuda.synchronize()

    # Calibration pass (outside the timed region): one stream, one batch at a time, every library call bracketed.
    # Finds the dominant conv kernel, gives its launch duration with the GPU to itself, and the per-stage breakdown.
    cal_reps = 3
    timer.enabled, timer.only = True, None
    for _ in range(cal_reps):
        runner.run(runner.in_pts, runner.in_batch, timer)
    torch.cuda.synchronize()
    stage_ms, conv_ms = {}, {}
    for tag, e0, e1 in timer.records:
        ms = e0.elapsed_time(e1) / cal_reps
        if isinstance(tag, tuple) and isinstance(tag[1], tuple):          # (branch, ("conv", li))
            conv_ms[(tag[0], tag[1][1])] = conv_ms.get((tag[0], tag[1][1]), 0.0) + ms
            stage_ms["conv"] = stage_ms.get("conv", 0.0) + ms
        else:
            name = tag[1] if isinstance(tag, tuple) else tag
            stage_ms[name] = stage_ms.get(name, 0.0) + ms
    groups = {}
    for bi, li, layer, pairs, fl in layers:
        kname = ctx0.spconv_kernel(cfg.dtype, layer.cin, layer.cout, layer.kind)
        g = groups.setdefault((kname, layer.cin, layer.cout), {"ms": 0.0, "flops": 0.0, "tags": []})
        g["ms"] += conv_ms.get((bi, li), 0.0)
        g["flops"] += fl
        g["tags"].append((bi, ("conv", li)))
    dom_key = max(groups, key=lambda k: groups[k]["ms"])
    dom = groups[dom_key]
    dom_on_mfma = bool(ctx0.uses_mfma(cfg.dtype, dom_key[1], dom_key[2]))
    dom_peak = PEAK_MFMA_F16_TFLOPS if dom_on_mfma else PEAK_VALU_F32_TFLOPS
    dom_name = f"{dom_key[0]}<{DTYPE_NAME[cfg.dtype]}, Cin={dom_key[1]}, Cout={dom_key[2]}>"

    # timed region: `steps` passes, graph replays with `depth` batches in flight; every N-th step is issued eagerly
    # with event brackets around the dominant kernel's launches (its duration while it shares the GPU)
    timer.reset()
    timer.only = set(dom["tags"])

    def region(n_steps, bracket_every):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n_steps):
            timer.enabled = bracket_every > 0 and (i % bracket_every == 0)
            step(timer)
        t_issued = time.perf_counter()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        timer.enabled = False
        return t1 - t0, t_issued - t0

    wall, issue = region(steps, args.bracket_every)
    runner_status = [r.status_sync() for r in ring]
    del runner_status
    ms_per_step = wall * 1e3 / steps
    frames_per_s = cfg.n_frames * steps / wall

    shared_ms, shared_flops, shared_n = 0.0, 0.0, 0
    flops_of = {(bi, ("conv", li)): fl for bi, li, _, _, fl in layers}
    for tag, e0, e1 in timer.records:
        shared_ms += e0.elapsed_time(e1)
        shared_flops += flops_of[tag]
        shared_n += 1
    excl_tflops = dom["flops"] / (dom["ms"] * 1e-3) / 1e12 if dom["ms"] > 0 else 0.0
    roofline = {
        "kernel": dom_name, "bound": "mfma" if dom_on_mfma else "alu",
        "achieved": excl_tflops, "peak": dom_peak, "unit": "TFLOP/s", "frac": excl_tflops / dom_peak,
        "flops_per_launch": dom["flops"] / max(len(dom["tags"]), 1), "launches_per_step": len(dom["tags"]),
        "avg_launch_ms": dom["ms"] / max(len(dom["tags"]), 1),
        "measured": "event brackets on the launch stream, one batch at a time (the kernel has the GPU to itself, as "
                    "under rocprofv3 kernel tracing)",
        "traffic": profiled_traffic(dom_key[0], cfg.index),
    }
    if shared_n:
        sh_tflops = shared_flops / (shared_ms * 1e-3) / 1e12
        roofline["under_sharing"] = {"achieved": sh_tflops, "frac": sh_tflops / dom_peak, "avg_launch_ms": shared_ms / shared_n,
                                     "launches_timed": shared_n,
                                     "note": f"bracketed inside the timed steps, {depth} batches in flight"}

    # memory-bound stages against the HBM peak: bytes over the calibration pass's stage time, counted two ways.
    # "algorithmic": what this design must move at the least -- voxelize: 16 B (+ 4 B batch id) per point read, 36 B
    # per voxel written; kernel maps: 16 B of coordinates read and 27 x 4 B of map written per output (+ 16 B of
    # coordinates written per stride-2 output, 16 B per input read); the index words are shared by 32 cells.
    # "per_unit_of_the_method": the per-unit figures of a hash-based formulation of the same steps -- 44 B per point
    # (16 read, a key slot, five accumulator updates) + 36 B per voxel; 340 B per submanifold output (coordinates, 27
    # probes of 8 B, 27 entries); 360 B per stride-2 output + 80 B per input.
    per_pt = 16.0 + (4.0 if batch is not None else 0.0)
    stage_bytes = {"voxelize": 0.0, "kmap_subm": 0.0, "kmap_strided": 0.0}
    unit_bytes = {"voxelize": 0.0, "kmap_subm": 0.0, "kmap_strided": 0.0}
    for bi, (_, br) in enumerate(runner.branches):
        nv = vox[bi]
        stage_bytes["voxelize"] += n_points * per_pt + nv[0] * 36.0
        unit_bytes["voxelize"] += n_points * 44.0 + nv[0] * 36.0
        lvl, seen = 0, set()
        for layer in br.branch.layers:
            if layer.kind == STRIDED:
                stage_bytes["kmap_strided"] += nv[lvl] * 16.0 + nv[lvl + 1] * (16.0 + 16.0 + 108.0)
                unit_bytes["kmap_strided"] += nv[lvl] * 80.0 + nv[lvl + 1] * 360.0
                lvl += 1
            elif lvl not in seen:
                seen.add(lvl)
                stage_bytes["kmap_subm"] += nv[lvl] * (16.0 + 108.0)
                unit_bytes["kmap_subm"] += nv[lvl] * 340.0
    if cfg.camera is not None:
        stage_bytes["project_gather"] = n_points * (16.0 + 5 * 2.0 * cfg.camera.channels + 1.0)
    stage_hbm = {}
    for k_, b_ in stage_bytes.items():
        if stage_ms.get(k_) and b_ > 0:
            gbs = b_ / (stage_ms[k_] * 1e-3) / 1e9
            stage_hbm[k_] = {"algorithmic_MB": b_ / 1e6, "ms": stage_ms[k_], "GB/s": gbs, "frac_of_hbm_peak": gbs / PEAK_HBM_GBS}
            if unit_bytes.get(k_):
                stage_hbm[k_]["per_unit_of_the_method_MB"] = unit_bytes[k_] / 1e6
                stage_hbm[k_]["per_unit_frac_of_hbm_peak"] = unit_bytes[k_] / (stage_ms[k_] * 1e-3) / 1e9 / PEAK_HBM_GBS

    res = {
        "config": cfg.index, "name": cfg.name,
        "workload": f"config {cfg.index} ({cfg.name}): {cfg.n_points} points x {cfg.n_frames} frame(s), "
                    + "; ".join(f"{br.branch.name} grid {tuple(br.branch.spec.grid)} {len(br.branch.layers)} convs"
                                for _, br in runner.branches)
                    + (f"; image gather {cfg.camera.height}x{cfg.camera.width}x{cfg.camera.channels}" if cfg.camera else ""),
        "value": frames_per_s, "unit": "frames/s", "ms_per_step": ms_per_step, "steps": steps,
        "host_issue_ms_per_step": issue * 1e3 / steps, "dtype": DTYPE_NAME[cfg.dtype],
        "launch_shape": ("two-stage pipeline across batches: maps of the next batch under the convs of this one"
                         if staged else "one batch at a time" if depth == 1 else "independent batches, one stream each"),

        "voxels_per_level": {br.branch.name: vox[bi] for bi, (_, br) in enumerate(runner.branches)},
        "roofline": roofline,
        "stages_ms_calibration_pass": stage_ms,
        "step_ms_one_batch_at_a_time_one_stream": sum(stage_ms.values()),
        "voxelize_mpts_per_s": (len(runner.branches) * n_points / (stage_ms["voxelize"] * 1e-3) / 1e6) if stage_ms.get("voxelize") else None,
        "conv_useful_gflop_per_step": total_flops / 1e9,
        "conv_useful_tflops": total_flops / (stage_ms["conv"] * 1e-3) / 1e12 if stage_ms.get("conv") else None,
        "memory_bound_stages": stage_hbm,
        "conv_layers": [{"branch": runner.branches[bi][1].branch.name, "cin": l.cin, "cout": l.cout, "strided": l.kind == STRIDED,
                         "pairs": p, "ms": conv_ms.get((bi, li), 0.0), "kernel": ctx0.spconv_kernel(cfg.dtype, l.cin, l.cout, l.kind),
                         "frac_of_mfma_peak": (f / (conv_ms[(bi, li)] * 1e-3) / 1e12 / PEAK_MFMA_F16_TFLOPS)
                         if conv_ms.get((bi, li)) and ctx0.uses_mfma(cfg.dtype, l.cin, l.cout) else None,
                         "ideal_reuse_MB": layer_bytes[(bi, li)] / 1e6,
                         "frac_of_hbm_peak": (layer_bytes[(bi, li)] / (conv_ms[(bi, li)] * 1e-3) / 1e9 / PEAK_HBM_GBS)
                         if conv_ms.get((bi, li)) else None}
                        for bi, li, l, p, f in layers],
    }

    if full:
        # repeated regions (no brackets): spread of the throughput figure
        reps = [cfg.n_frames * steps / region(steps, 0)[0] for _ in range(args.region_repeats)]
        res["value_over_repeated_regions"] = percentiles(reps)
        # one batch at a time: latency of a step, start to end, over many single steps
        lat = []
        r0 = ring[0]
        if staged:
            # one step alone in the staged form: from the first map kernel to the last branch's last convolution
            for _ in range(args.dist_reps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(map_stream)
                r0.replay_stages(map_stream, conv_sets[0])
                for ev in r0.ev_convs:
                    map_stream.wait_event(ev)
                e1.record(map_stream)
                e1.synchronize()
                lat.append(e0.elapsed_time(e1))
        else:
            with torch.cuda.stream(r0.stream):
                for _ in range(args.dist_reps):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    if use_graphs:
                        r0.replay()
                    else:
                        r0.run_overlapped(r0.in_pts, r0.in_batch)
                    e1.record()
                    e1.synchronize()
                    lat.append(e0.elapsed_time(e1))
        res["step_latency_ms"] = percentiles(lat)
        # cold inputs: every step reads another of `cold_frames` distinct seeded frames (copied into the runner's
        # input buffer on its stream right before the pass), so no step finds its own input or intermediate data
        # of the same scene in the caches
        n_cold = max(args.cold_frames // cfg.n_frames, 2)
        cold = []
        for i in range(n_cold):
            p_, b_ = gen.make_frames(cfg, first_frame=(i + 1) * cfg.n_frames)
            cold.append(torch.from_numpy(p_).cuda())
        for i in range(depth + 2):
            r = ring[i % depth]
            with torch.cuda.stream(map_stream if staged else r.stream):
                r.in_pts.copy_(cold[i % n_cold], non_blocking=True)
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps * 2):
            r = ring[step_no[0] % depth]
            with torch.cuda.stream(map_stream if staged else r.stream):
                r.in_pts.copy_(cold[i % n_cold], non_blocking=True)
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        for r in ring:
            r.status_sync()
        res["cold_inputs"] = {"value": cfg.n_frames * steps * 2 / dt, "unit": "frames/s", "ms_per_step": dt * 1e3 / (steps * 2),
                              "distinct_frames": n_cold * cfg.n_frames, "steps": steps * 2}
        for r in ring:
            r.in_pts.copy_(pts)
        torch.cuda.synchronize()
        del cold
    return res, ring, (cfg, pts_np, batch_np)


# ----------------------------------------------------------------------------------------------------------
# side measurements on the other calls of the boundary (outside every timed region)
# ----------------------------------------------------------------------------------------------------------

def side_project_gather(torch):
    from paper_2507_04123_amd import binding as B
    from paper_2507_04123_amd import gen
    from paper_2507_04123_amd.configs import get_config
    cfg3 = get_config(3)
    cam = cfg3.camera
    pts3_np, _ = gen.make_frames(cfg3)
    pts3 = torch.from_numpy(pts3_np).cuda()
    img = torch.from_numpy(gen.make_image(cam.height, cam.width, cam.channels, gen.frame_seed(3, 0))).cuda()
    pm = gen.make_camera(gen.frame_seed(3, 0))
    g_out = torch.empty((len(pts3_np), cam.channels), dtype=torch.float16, device="cuda")
    g_valid = torch.empty((len(pts3_np),), dtype=torch.uint8, device="cuda")
    ctx = B.Context(16, 16, 64, n_slots=1)
    ms = timed_loop(torch, lambda: ctx.project_gather(pts3, pm, img, g_out, g_valid))
    nbytes = len(pts3_np) * (16.0 + 4 * 2.0 * cam.channels + 2.0 * cam.channels + 1.0)
    out = {"workload": f"config 3: {len(pts3_np)} points, image {cam.height}x{cam.width}x{cam.channels} f16",
           "ms": ms, "algorithmic_MB": nbytes / 1e6, "GB/s": nbytes / (ms * 1e-3) / 1e9,
           "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "valid_points": int(g_valid.sum().item())}
    ctx.close()
    return out


def side_decoder(torch):
    """Inverse map of the last stride-2 layer of config 2, the transposed 64->64 conv over it, BEV flattening."""
    from paper_2507_04123_amd import binding as B
    from paper_2507_04123_amd import gen
    from paper_2507_04123_amd.configs import get_config
    from paper_2507_04123_amd.pipeline import ConfigRunner
    cfg = get_config(2)
    pts_np, _ = gen.make_frames(cfg)
    cr = ConfigRunner(cfg, len(pts_np))
    ctx, runner = cr.branches[0]
    runner.run(torch.from_numpy(pts_np).cuda(), None)
    torch.cuda.synchronize()
    fine, coarse = runner.levels[-2], runner.levels[-1]
    nf, nc = int(fine.n.item()), int(coarse.n.item())
    inv = torch.empty((27, fine.cap), dtype=torch.int32, device="cuda")
    x_c = runner.acts[-1]
    cch = int(x_c.shape[1])
    w_t = torch.randn((27, cch, cch), device="cuda").mul_(0.1).to(x_c.dtype)
    sc = torch.full((cch,), 0.1, dtype=torch.float32, device="cuda")
    sh = torch.zeros((cch,), dtype=torch.float32, device="cuda")
    w_p = torch.empty_like(w_t)
    ctx.pack_weights(cfg.dtype, w_t, w_p)
    y_f = torch.empty((fine.cap, cch), dtype=x_c.dtype, device="cuda")
    nb = runner.branch.spec.n_batch
    bev = torch.empty((nb, coarse.grid[1], coarse.grid[0], coarse.grid[2] * cch), dtype=x_c.dtype, device="cuda")
    ms_inv = timed_loop(torch, lambda: ctx.build_inverse_kmap(fine.coords, fine.n, fine.cap, coarse.grid, nb, coarse.slot, coarse.n, inv))
    pairs_t = int((inv[:, :nf] >= 0).sum().item())
    ms_tc = timed_loop(torch, lambda: ctx.spconv(cfg.dtype, x_c, w_p, sc, sh, 2, inv, fine.n, fine.cap, y_f, w_layout=B.W_PACKED))
    ms_bev = timed_loop(torch, lambda: ctx.bev_flatten(cfg.dtype, coarse.coords, x_c, coarse.n, coarse.cap, coarse.grid, nb, bev))
    esz = x_c.element_size()
    inv_bytes = nf * (16.0 + 108.0)
    bev_bytes = bev.numel() * esz + nc * (16.0 + 2.0 * cch * esz)
    fl_t = 2.0 * pairs_t * cch * cch
    out = {"inverse_kmap": {"fine": nf, "coarse": nc, "ms": ms_inv, "algorithmic_MB": inv_bytes / 1e6,
                            "GB/s": inv_bytes / (ms_inv * 1e-3) / 1e9, "frac_of_hbm_peak": inv_bytes / (ms_inv * 1e-3) / 1e9 / PEAK_HBM_GBS},
           "transposed_conv": {"cin": cch, "cout": cch, "pairs": pairs_t, "ms": ms_tc, "kernel": ctx.spconv_kernel(cfg.dtype, cch, cch),
                               "useful_tflops": fl_t / (ms_tc * 1e-3) / 1e12, "frac_of_mfma_peak": fl_t / (ms_tc * 1e-3) / 1e12 / PEAK_MFMA_F16_TFLOPS},
           "bev_flatten": {"voxels": nc, "dense_MB": bev.numel() * esz / 1e6, "ms": ms_bev, "algorithmic_MB": bev_bytes / 1e6,
                           "GB/s": bev_bytes / (ms_bev * 1e-3) / 1e9, "frac_of_hbm_peak": bev_bytes / (ms_bev * 1e-3) / 1e9 / PEAK_HBM_GBS}}
    # quantised conv on the two 64 -> 64 maps of the same frame, beside the fp16 kernels
    quant = []
    lvl = 0
    from paper_2507_04123_amd.configs import STRIDED
    seen = set()
    for li, layer in enumerate(runner.branch.layers):
        if layer.kind == STRIDED:
            lvl += 1
        if not (layer.cin == 64 and layer.cout == 64) or layer.kind in seen:
            continue
        seen.add(layer.kind)
        lv_o = runner.levels[lvl]
        nbr_t = lv_o.down_nbr if layer.kind == STRIDED else lv_o.subm_nbr
        n_in = int(runner.levels[lvl - 1].n.item()) if layer.kind == STRIDED else int(lv_o.n.item())
        n_o = int(lv_o.n.item())
        pairs = int((nbr_t[:, :n_o] >= 0).sum().item())
        xq = torch.randint(-127, 128, (max(n_in, 1), 64), dtype=torch.int8, device="cuda")
        wq = torch.randint(-60, 61, (27, 64, 64), dtype=torch.int8, device="cuda")
        wpk = torch.empty((27 * 64 * 64,), dtype=torch.int8, device="cuda")
        ctx.pack_weights_i8(wq, wpk)
        ml = torch.full((64,), 1e-5, dtype=torch.float32, device="cuda")
        ad = torch.zeros((64,), dtype=torch.float32, device="cuda")
        yq = torch.empty((lv_o.cap, 64), dtype=torch.int8, device="cuda")
        ms_q = timed_loop(torch, lambda: ctx.spconv_i8(xq, wpk, 64, 64, ml, ad, True, nbr_t, lv_o.n, lv_o.cap, yq, inv_out_scale=30.0))
        x16 = runner.acts[li - 1]
        p = runner.params[li]
        ms_h = timed_loop(torch, lambda: ctx.spconv(cfg.dtype, x16, runner.wdev[li][0], p["scale"], p["shift"], 2, nbr_t, lv_o.n, lv_o.cap,
                                                    runner.acts[li], w_layout=runner.wdev[li][1], map_hint=layer.kind))
        # the same layer in 8-bit floating point (E4M3 codes, fp32 accumulation on the fp8 matrix cores)
        x8 = torch.empty((max(n_in, 1), 64), dtype=torch.uint8, device="cuda")
        ctx.quantize_e4m3(torch.randn((max(n_in, 1), 64), device="cuda"), 1.0, x8)
        w8 = torch.empty((27, 64, 64), dtype=torch.uint8, device="cuda")
        ctx.quantize_e4m3(torch.randn((27, 64, 64), device="cuda").mul_(0.1), 8.0, w8)
        w8p = torch.empty((27 * 64 * 64,), dtype=torch.int8, device="cuda")
        ctx.pack_weights_i8(w8.view(torch.int8), w8p)
        y8 = torch.empty((lv_o.cap, 64), dtype=torch.float16, device="cuda")
        ms_8 = timed_loop(torch, lambda: ctx.spconv_e4m3(x8, w8p, 64, 64, ml, ad, True, nbr_t, lv_o.n, lv_o.cap, y8))
        ops = 2.0 * pairs * 64 * 64
        quant.append({"cin": 64, "cout": 64, "strided": layer.kind == STRIDED, "pairs": pairs, "ms_int8": ms_q, "ms_e4m3": ms_8,
                      "ms_fp16_same_map": ms_h,
                      "useful_TOPS": ops / (ms_q * 1e-3) / 1e12, "frac_of_int8_peak": ops / (ms_q * 1e-3) / 1e12 / 5000.0,
                      "e4m3_useful_TFLOPs": ops / (ms_8 * 1e-3) / 1e12, "frac_of_fp8_peak": ops / (ms_8 * 1e-3) / 1e12 / 5000.0})
    # Cross-layer fusion of the two submanifold layers of a stage (paper Sec. 3.6, graph optimisation (3)): a block
    # that owns T consecutive output rows of the second layer needs the first layer's outputs on every row its map
    # names (the halo H), so a fused block recomputes |H| / |T| times the first layer's work.  Measured on this
    # frame's maps for the block size the conv kernels use (512 rows) and for a whole 4096-row super-block.
    halo = []
    lvl = 0
    for li, layer in enumerate(runner.branch.layers):
        if layer.kind == STRIDED:
            lvl += 1
            continue
        lv_o = runner.levels[lvl]
        if lv_o.subm_nbr is None or any(h["level"] == lvl for h in halo):
            continue
        n_o = int(lv_o.n.item())
        row = {"level": lvl, "voxels": n_o}
        for tile in (512, 4096):
            n_t = n_o // tile
            if n_t == 0:
                continue
            m = lv_o.subm_nbr[:, :n_t * tile].reshape(27, n_t, tile).permute(1, 0, 2).reshape(n_t, 27 * tile)
            srt, _ = torch.sort(m, dim=1)
            distinct = ((srt[:, 1:] != srt[:, :-1]) & (srt[:, 1:] >= 0)).sum(dim=1) + (srt[:, 0] >= 0).to(torch.int64)
            row[f"rows_needed_per_row_owned_tile{tile}"] = float(distinct.double().mean().item()) / tile
        halo.append(row)
    out["two_layer_fusion_halo"] = halo
    cr.close()
    return out, quant


def side_bridge(torch):
    """Multiscale Pooling and fusion on config 3's image and clouds, on each of its three scales."""
    from paper_2507_04123_amd import binding as B
    from paper_2507_04123_amd import gen
    from paper_2507_04123_amd.configs import get_config
    from paper_2507_04123_amd.pipeline import cells_of
    cfg3 = get_config(3)
    cam = cfg3.camera
    npix = cam.height * cam.width
    seed3 = gen.frame_seed(3, 0)
    pts3_np, _ = gen.make_frames(cfg3)
    sp0 = cfg3.branches[0].spec
    ctx_b = B.Context(max(npix, len(pts3_np)), npix + len(pts3_np), cells_of(sp0.grid, sp0.n_batch), n_slots=3)
    fmap = torch.from_numpy(gen.make_image(cam.height, cam.width, cam.channels, seed3)).cuda()
    dmap = torch.from_numpy(gen.make_depth(cam.height, cam.width, seed3)).cuda()
    qm = gen.make_unprojection(gen.make_camera(seed3))
    pts3 = torch.from_numpy(pts3_np).cuda()
    cap_b = npix + len(pts3_np)
    i32 = dict(dtype=torch.int32, device="cuda")
    ic, icnt, n_i = torch.empty((cap_b, 4), **i32), torch.empty((cap_b,), **i32), torch.zeros(1, **i32)
    if_ = torch.empty((cap_b, cam.channels), dtype=torch.float16, device="cuda")
    lc, lcnt, n_l = torch.empty((cap_b, 4), **i32), torch.empty((cap_b,), **i32), torch.zeros(1, **i32)
    lm = torch.empty((cap_b, 4), dtype=torch.float32, device="cuda")
    lf = torch.randn((cap_b, 32), device="cuda").to(torch.float16)
    fc, n_f = torch.empty((cap_b, 4), **i32), torch.zeros(1, **i32)
    ff = torch.empty((cap_b, 96), dtype=torch.float16, device="cuda")
    scales = []
    for br3 in cfg3.branches:
        sp3 = br3.spec
        row = {"scale": br3.name, "cell_m": list(sp3.vs)}
        for mode, nm in ((B.POOL_MEAN, "mean"), (B.POOL_MAX, "max")):
            ms_p = timed_loop(torch, lambda: ctx_b.pool_image(fmap, dmap, qm, sp3, mode, cap_b, ic, if_, icnt, n_i, index_slot=1))
            ni = int(n_i.item())
            pooled = int(icnt[:ni].sum().item())
            pb = npix * 4.0 + pooled * 2.0 * cam.channels + ni * (20.0 + 2.0 * cam.channels)
            row["pool_" + nm] = {"ms": ms_p, "cells": ni, "pixels_pooled": pooled, "algorithmic_MB": pb / 1e6,
                                 "GB/s": pb / (ms_p * 1e-3) / 1e9, "frac_of_hbm_peak": pb / (ms_p * 1e-3) / 1e9 / PEAK_HBM_GBS}
        nl = ctx_b.voxelize(pts3, None, sp3, cap_b, lc, lm, lcnt, n_l, index_slot=0, sync_count=True)
        ms_f = timed_loop(torch, lambda: ctx_b.fuse(cfg3.dtype, lc, lf, n_l, cap_b, ic, if_, n_i, cap_b, sp3.grid, sp3.n_batch, cap_b,
                                                    fc, ff, n_f, out_slot=2))
        nf_ = int(n_f.item())
        fb = nl * (16.0 + 64.0) + ni * (16.0 + 2.0 * cam.channels) + nf_ * (16.0 + 192.0)
        row["fuse"] = {"ms": ms_f, "voxels": nl, "image_cells": ni, "fused": nf_, "shared": nl + ni - nf_,
                       "algorithmic_MB": fb / 1e6, "GB/s": fb / (ms_f * 1e-3) / 1e9,
                       "frac_of_hbm_peak": fb / (ms_f * 1e-3) / 1e9 / PEAK_HBM_GBS}
        scales.append(row)
    ctx_b.status_sync()
    out = {"workload": f"config 3: image {cam.height}x{cam.width}x{cam.channels} f16 with depth ({int((dmap > 0).sum().item())} "
                       f"relevant pixels), {len(pts3_np)} points", "scales": scales}
    ctx_b.close()
    return out


def side_dispatcher(torch):
    from paper_2507_04123_amd import binding as B
    from paper_2507_04123_amd import gen
    ctx = B.Context(16, 16, 64, n_slots=1)
    out = []
    for n_sc in (8, 1024):
        pr_np, sc_np = gen.make_proposals(n_sc, gen.frame_seed(5, 0))
        pr, sc_t = torch.from_numpy(pr_np).cuda(), torch.from_numpy(sc_np).cuda()
        ex = torch.empty((n_sc,), dtype=torch.int32, device="cuda")
        cn = torch.empty((3,), dtype=torch.int32, device="cuda")
        od = torch.empty((n_sc,), dtype=torch.int32, device="cuda")
        ms_d = timed_loop(torch, lambda: ctx.dispatch(pr, sc_t, n_sc, 23.5, 0.5, ex, cn, od))
        db = len(pr_np) * 20.0 + n_sc * 8.0
        out.append({"scenes": n_sc, "proposals": len(pr_np), "ms": ms_d, "scenes_per_expert": cn.tolist(),
                    "algorithmic_MB": db / 1e6, "GB/s": db / (ms_d * 1e-3) / 1e9})
    ctx.close()
    # scene-level routing end to end: dispatch -> group the points by expert -> every expert's stack on its group
    from paper_2507_04123_amd.configs import expert_branches, get_config
    from paper_2507_04123_amd.pipeline import RoutedRunner
    cfg5 = get_config(5)
    pts_np, batch_np = gen.make_frames(cfg5)
    n_sc = cfg5.n_frames
    rr = RoutedRunner(expert_branches(n_sc), cfg5.dtype, len(pts_np), n_sc, seed=7)
    pr_np, sc_np = gen.make_proposals(n_sc, gen.frame_seed(5, 0))
    pts, scene = torch.from_numpy(pts_np).cuda(), torch.from_numpy(batch_np).cuda()
    pr, sc_t = torch.from_numpy(pr_np).cuda(), torch.from_numpy(sc_np).cuda()
    ms_r = timed_loop(torch, lambda: rr.run(pts, scene, pr, sc_t, 23.5, 0.5), reps=10)
    rr.status_sync()
    rr.capture(pts, scene, pr, sc_t, 23.5, 0.5)
    ms_g = timed_loop(torch, rr.replay, reps=10)
    rr.status_sync()
    out.append({"routed_run": f"{n_sc} scenes of config 5's cloud through dispatch, grouping and the three expert stacks (one stream)",
                "ms": ms_r, "ms_graph_replay": ms_g, "scenes_per_expert": rr.counts.tolist(), "frames/s": n_sc / (ms_g * 1e-3)})
    rr.close()
    return out


def side_voxelize_scaling(torch, batches):
    """The voxelizer alone on config 2's cloud repeated B times with batch ids (one frame is ~6 MB of algorithmic
    traffic, too little to be anything but launch- and latency-bound; many frames per launch show what the kernels
    sustain).  Bytes: 16 B point + 4 B batch id read per point, 36 B written per voxel."""
    from paper_2507_04123_amd import binding as B
    from paper_2507_04123_amd import gen
    from paper_2507_04123_amd.configs import get_config, VoxelSpec
    from paper_2507_04123_amd.pipeline import cells_of
    cfg = get_config(2)
    sp = cfg.branches[0].spec
    pts_np, _ = gen.make_frames(cfg)
    pts = torch.from_numpy(pts_np).cuda()
    n_points = len(pts_np)
    out = []
    for nb_ in batches:
        pts_b = pts.repeat(nb_, 1).contiguous()
        bid = torch.arange(nb_, dtype=torch.int32, device="cuda").repeat_interleave(n_points).contiguous()
        sp_ = VoxelSpec(sp.lo, sp.vs, sp.grid, n_batch=nb_)
        cap_ = n_points * nb_
        cx_ = B.Context(cap_, cap_, cells_of(sp_.grid, nb_), n_slots=1)
        co_ = torch.empty((cap_, 4), dtype=torch.int32, device="cuda")
        fe_ = torch.empty((cap_, 4), dtype=torch.float32, device="cuda")
        cn_ = torch.empty((cap_,), dtype=torch.int32, device="cuda")
        nn_ = torch.zeros(1, dtype=torch.int32, device="cuda")
        ms_ = timed_loop(torch, lambda: cx_.voxelize(pts_b, bid, sp_, cap_, co_, fe_, cn_, nn_, index_slot=0), reps=5, warm=2)
        cx_.status_sync()
        nv_ = int(nn_.item())
        by_ = cap_ * 20.0 + nv_ * 36.0
        out.append({"frames": nb_, "points": cap_, "voxels": nv_, "ms": ms_, "Mpts/s": cap_ / (ms_ * 1e-3) / 1e6,
                    "GB/s": by_ / (ms_ * 1e-3) / 1e9, "frac_of_hbm_peak": by_ / (ms_ * 1e-3) / 1e9 / PEAK_HBM_GBS})
        cx_.close()
        del pts_b, bid, co_, fe_, cn_, nn_, cx_
        torch.cuda.empty_cache()
    return out


def guarded(fn, *a):
    """A side measurement must never take the headline number down with it."""
    try:
        return fn(*a)
    except Exception as exc:  # noqa: BLE001
        return {"error": repr(exc)}


def measure_other_configs(args):
    """The `per_config` list: each of the other configurations measured by a child process of its own (`bench.py
    --config N`, run to its end before the next starts, and before this process touches the GPU), so that its figures
    do not depend on what the headline measurement created before it: torch hands streams out of a small round-robin
    pool, streams share a few hardware queues, and a second process with work on the GPU slows a launch-bound one."""
    per = []
    for idx in [int(x) for x in args.per_config.split(",") if x.strip()]:
        if idx == args.config:
            continue
        cmd = [sys.executable, os.path.abspath(__file__), "--config", str(idx), "--config-result-only",
               "--steps", str(min(args.steps, 20)), "--warmup", str(args.warmup),
               "--frames-in-flight", str(args.frames_in_flight), "--bracket-every", str(args.bracket_every),
               "--launch-shape", args.launch_shape]
        for flag, on in (("--no-cpu-baseline", args.no_cpu_baseline), ("--no-graphs", args.no_graphs),
                         ("--branch-graphs", args.branch_graphs), ("--serial", args.serial)):
            if on:
                cmd.append(flag)
        try:
            cp = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, timeout=600, check=False)
            line = cp.stdout.decode().strip().splitlines()[-1] if cp.stdout.strip() else ""
            if cp.returncode != 0 or not line.startswith("{"):
                raise RuntimeError(f"exit {cp.returncode}: {cp.stderr.decode()[-400:]}")
            per.append(json.loads(line))
        except Exception as exc:  # noqa: BLE001
            per.append({"config": idx, "error": repr(exc)})
    return per


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5, help="headline workload (5 = the largest single-GPU configuration)")
    ap.add_argument("--per-config", type=str, default="1,2,3,4", help="other configurations to list (comma separated; '' = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--serial", action="store_true", help="one batch at a time, every call on one stream")
    ap.add_argument("--frames-in-flight", type=int, default=4, choices=[1, 2, 3, 4, 5, 6, 8],
                    help="batches in flight: each has its own contexts, buffers and stream, so the small index / map kernels "
                         "of one batch fill the CUs that another batch's convs leave idle (a step is still one whole batch)")
    ap.add_argument("--bracket-every", type=int, default=10,
                    help="the dominant kernel's launches carry event brackets on every N-th timed step (0 = never)")
    ap.add_argument("--no-graphs", action="store_true", help="issue every launch from the host instead of replaying HIP graphs")
    ap.add_argument("--branch-graphs", action="store_true",
                    help="one two-stream graph per branch (map building forked from the convs inside the graph) instead of one "
                         "graph without forks per batch; measured slower: the batches in flight supply the overlap")
    ap.add_argument("--launch-shape", choices=["auto", "batches", "stages"], default="auto",
                    help="batches: every batch in flight replays its whole pass (one graph) on a stream of its own; "
                         "stages: a two-stage pipeline, voxelization and kernel maps of the next batch on a map stream "
                         "under the convolutions of this batch on one conv stream per branch; auto: stages for a "
                         "workload with several branches and at least 500 000 points per step, else batches")
    ap.add_argument("--config-result-only", action="store_true", help=argparse.SUPPRESS)
    ap.add_argument("--headline-only", action="store_true",
                    help="only the headline configuration's timed region and calibration: for profiler and counter runs")
    ap.add_argument("--dist-reps", type=int, default=200, help="single steps timed for the step-latency distribution")
    ap.add_argument("--region-repeats", type=int, default=10, help="repetitions of the timed region for the throughput spread")
    ap.add_argument("--cold-frames", type=int, default=64, help="distinct seeded frames the cold-input pass rotates through")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also launch one plain device copy of this many MiB (a known-size reference for scaling "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (frames shard across GPUs with no "
              "exchange, so several GPUs would each run this same program on their share). Run with --gpus 1.", file=sys.stderr)
        return 2

    per = measure_other_configs(args) if not (args.headline_only or args.config_result_only) else None

    import faulthandler
    faulthandler.enable()            # a fatal signal in native code still names the Python line it came from
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    replay_stream(torch, 3 * args.frames_in_flight)      # the replay streams come first (staged form: 1 + branches per batch)

    if args.copy_probe_mib > 0:
        src = torch.empty(args.copy_probe_mib << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.config_result_only:
        # child of a full run: one configuration's entry of `per_config`, as one JSON line
        r_, ring_, (cfg_, p_, b_) = measure_config(args.config, args, args.steps, args.warmup, full=False)
        for x in ring_:
            x.close()
        if not args.no_cpu_baseline:
            import oracle
            r_["cpu_baseline"] = cpu_baseline(cfg_, p_, b_, min(oracle.max_threads(), 16), single_thread_sample=False)
        print(json.dumps(r_))
        return 0

    head, ring, (cfg, pts_np, batch_np) = measure_config(args.config, args, args.steps, args.warmup, full=not args.headline_only)
    for r in ring:
        r.close()
    del ring
    torch.cuda.empty_cache()

    out = {
        "metric": "frames/s through voxelize+spconv backbone",
        "value": head["value"], "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": head["workload"], "frames_per_step": cfg.n_frames, "batches_in_flight": 1 if args.serial else args.frames_in_flight, "launch_shape": head["launch_shape"],
                   "hip_graphs": not args.no_graphs, "voxels_per_level": head["voxels_per_level"]},
        "roofline": head["roofline"],
    }
    for k in ("host_issue_ms_per_step", "value_over_repeated_regions", "step_latency_ms", "cold_inputs", "stages_ms_calibration_pass",
              "step_ms_one_batch_at_a_time_one_stream", "voxelize_mpts_per_s", "conv_useful_gflop_per_step", "conv_useful_tflops",
              "memory_bound_stages", "conv_layers"):
        if k in head:
            out[k] = head[k]

    if not args.headline_only:
        out["measured_ceilings"] = guarded(measure_probes, torch)
        out["per_config"] = per
        out["project_gather"] = guarded(side_project_gather, torch)
        dq = guarded(side_decoder, torch)
        out["decoder_side"], out["quantised_conv"] = dq if isinstance(dq, tuple) else (dq, dq)
        out["multimodal_bridge"] = guarded(side_bridge, torch)
        out["dispatcher"] = guarded(side_dispatcher, torch)
        out["voxelize_scaling"] = guarded(side_voxelize_scaling, torch, (1, 8, 64, 256))
    if not args.no_cpu_baseline:
        import oracle
        threads = min(oracle.max_threads(), 16)
        out["cpu_baseline"] = cpu_baseline(cfg, pts_np, batch_np, threads)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
