#!/usr/bin/env python3
"""Bench: frames/s through voxelize + kernel maps + sparse-conv backbone on one MI355X.

A step is one pass of the whole hot path over one synthetic frame of the front-view 64-beam
workload (120k points, fp16 SECOND-style backbone: 1 voxelization, 7 kernel maps, 10 convs), with
the points already resident in HBM.  Prints ONE JSON line with the throughput, a `roofline` object
for the dominant kernel (timed live with stream events inside the timed steps) and a `cpu_baseline`
object (the CPU oracle timed on this machine's host cores on one frame).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F16_TFLOPS = 2500.0      # MI355X dense fp16/bf16 MFMA, published
PEAK_HBM_GBS = 8000.0              # MI355X HBM3E, published
PEAK_VALU_F32_TFLOPS = 157.3       # MI355X fp32 vector ALU, published (256 CUs x 128 lanes x 2 flop x 2.4 GHz)
DTYPE_NAME = {0: "f32", 1: "f16", 2: "bf16"}   # the arithmetic type of the conv operands (accumulation is fp32)


class EventTimer:
    """Brackets library calls with events on the stream they are launched on (torch's current stream)."""

    def __init__(self, torch):
        self.torch = torch
        self.records = []           # (tag, start_event, stop_event)
        self.enabled = False
        self.only = None            # None = bracket every call; else the set of tags to bracket

    def __call__(self, tag):
        if self.only is not None and tag not in self.only:
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
        if self.t.enabled:
            self.e0 = self.t.torch.cuda.Event(enable_timing=True)
            self.e1 = self.t.torch.cuda.Event(enable_timing=True)
            self.e0.record()
        return self

    def __exit__(self, *a):
        if self.t.enabled:
            self.e1.record()
            self.t.records.append((self.tag, self.e0, self.e1))
        return False


def cpu_baseline(cfg, pts, seed, threads):
    """The oracle as it stands, on one full frame of the same workload, all stages."""
    import oracle
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import layer_params_host, oracle_branch
    oracle.set_threads(threads)
    br = cfg.branches[0]
    hp = layer_params_host(br, seed, cfg.dtype)
    t0 = time.perf_counter()
    oracle_branch(pts, None, br, cfg.dtype, hp)
    dt = time.perf_counter() - t0
    return {"value": 1.0 / dt, "unit": "frames/s", "cores": threads, "kind": "oracle",
            "sample": f"1 full frame of {cfg.name} (voxelize + 7 kernel maps + 10 convs), {dt:.2f} s",
            "ms_per_frame": dt * 1e3}


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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="workload index (2 = the metric's configuration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tight-capacity", action="store_true",
                    help="size per-level capacities from a calibration pass (x1.25) instead of the safe bounds")
    ap.add_argument("--serial", action="store_true",
                    help="issue every call on one stream (default: map building on a second stream, overlapping the convs)")
    ap.add_argument("--conv-streams", type=int, default=2, choices=[1, 2],
                    help="with several frames in flight: 2 gives each context its own conv stream as well")
    ap.add_argument("--frames-in-flight", type=int, default=3, choices=[1, 2, 3, 4],
                    help="2: two contexts alternate frames, so the maps of frame f+1 are built while the convs of "
                         "frame f run (throughput mode; each step is still one whole frame); 1: one frame at a time")
    ap.add_argument("--bracket-every", type=int, default=4,
                    help="the dominant kernel's launches carry event brackets on every N-th timed step")
    ap.add_argument("--no-graphs", action="store_true",
                    help="issue every launch from the host (default: each context's frame is recorded once into a HIP "
                         "graph and replayed; the steps that carry the dominant kernel's event brackets stay eager)")
    ap.add_argument("--no-scaling-sweep", action="store_true", help="skip the voxelizer batch-size sweep")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip every side measurement outside the timed region (projection, decoder side, pooling and "
                         "fusion, dispatcher, voxelizer sweep): for counter runs, where every kernel is serialised")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also launch one plain device copy of this many MiB (a known-size reference for scaling "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (frames shard across GPUs with no "
              "exchange, so several GPUs would each run this same program on their share). Run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2507_04123_amd import binding as B
    from paper_2507_04123_amd import gen
    from paper_2507_04123_amd.configs import get_config, STRIDED
    from paper_2507_04123_amd.pipeline import BranchRunner, cells_of, default_capacities, device_params

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = get_config(args.config)
    assert len(cfg.branches) == 1, "bench covers single-branch backbones"
    br = cfg.branches[0]
    pts_np, batch_np = gen.make_frames(cfg)
    seed = gen.frame_seed(cfg.index, 0)
    pts = torch.from_numpy(pts_np).cuda()
    batch = torch.from_numpy(batch_np).cuda() if cfg.n_frames > 1 else None
    n_points = len(pts_np)

    caps = default_capacities(br, n_points)

    def make(caps_):
        ctx_ = B.Context(n_points, max(caps_), cells_of(br.spec.grid, br.spec.n_batch), n_slots=len(caps_))
        return ctx_, BranchRunner(ctx_, br, cfg.dtype, n_points, device_params(br.layers, seed, cfg.dtype), capacities=caps_)

    ctx, runner = make(caps)
    runner.run(pts, batch)
    ctx.status_sync()
    if args.tight_capacity:
        counts = [int(lv.n.item()) for lv in runner.levels]
        caps = [min(c, int(v * 1.25) + 256) for c, v in zip(caps, counts)]
        ctx.close()
        ctx, runner = make(caps)
        runner.run(pts, batch)
        ctx.status_sync()

    # flop / byte accounting from the kernel maps of this frame (outside the timed region)
    n_vox = [int(lv.n.item()) for lv in runner.levels]
    layer_pairs, layer_flops = [], []
    for li, layer in enumerate(br.layers):
        nbr, lv = runner.layer_map(li)
        n = int(lv.n.item())
        pairs = int((nbr[:, :n] >= 0).sum().item())
        layer_pairs.append(pairs)
        layer_flops.append(2.0 * pairs * layer.cin * layer.cout)

    if args.copy_probe_mib > 0:
        src = torch.empty(args.copy_probe_mib << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    depth = 1 if args.serial else args.frames_in_flight
    ring = [(ctx, runner)]            # one context (scratch, buffers, streams) per frame in flight
    for _ in range(depth - 1):
        c_, r_ = make(caps)
        r_.run(pts, batch)
        c_.status_sync()
        ring.append((c_, r_))
    torch.cuda.synchronize()
    inputs_ready = torch.cuda.Event()
    inputs_ready.record()             # the points are resident and complete from here on
    torch.cuda.synchronize()
    step_no = [0]
    conv_streams = [torch.cuda.Stream() for _ in ring] if (depth >= 2 and args.conv_streams == 2) else None

    use_graphs = not args.no_graphs
    graphs = None

    def step(p, b, tm=None):
        if graphs is not None and (tm is None or not tm.enabled):
            k = step_no[0] % depth
            step_no[0] += 1
            if conv_streams is not None:
                with torch.cuda.stream(conv_streams[k]):
                    graphs[k].replay()
            else:
                graphs[k].replay()
            return ring[k][1].graph_out
        if graphs is not None:
            # an eager, bracketed step between replays: order its map stream after everything this context's
            # stream holds (the previous replay included) rather than after the shared input event only
            k = step_no[0] % depth
            step_no[0] += 1
            if conv_streams is not None:
                with torch.cuda.stream(conv_streams[k]):
                    return (ring[k][1].run(p, b, tm) if args.serial else ring[k][1].run_overlapped(p, b, tm))
            return (ring[k][1].run(p, b, tm) if args.serial else ring[k][1].run_overlapped(p, b, tm))
        if args.serial:
            return runner.run(p, b, tm)
        if depth == 1:
            return runner.run_overlapped(p, b, tm)
        k = step_no[0] % depth
        step_no[0] += 1
        if conv_streams is not None:
            # each context also gets a conv stream of its own: the convs of consecutive frames share the machine
            with torch.cuda.stream(conv_streams[k]):
                return ring[k][1].run_overlapped(p, b, tm, inputs_ready=inputs_ready)
        return ring[k][1].run_overlapped(p, b, tm, inputs_ready=inputs_ready)

    timer = EventTimer(torch)
    if use_graphs:
        torch.cuda.synchronize()
        graphs = [r_.capture(pts, batch, overlapped=not args.serial) for _, r_ in ring]
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step(pts, batch)
    torch.cuda.synchronize()

    # Calibration pass (outside the timed region): every library call bracketed by events, to find the
    # dominant conv kernel and to report a per-stage breakdown.  Event records cost ~10 us of stream
    # idle each, so the timed region below brackets only the dominant kernel, and only on every 4th step.
    timer.enabled = True
    timer.only = None
    for _ in range(3):
        runner.run(pts, batch, timer)
    torch.cuda.synchronize()
    stage_ms = {}
    conv_ms = [0.0] * len(br.layers)
    for tag, e0, e1 in timer.records:
        ms = e0.elapsed_time(e1) / 3.0
        if isinstance(tag, tuple):
            conv_ms[tag[1]] += ms
            stage_ms["conv"] = stage_ms.get("conv", 0.0) + ms
        else:
            stage_ms[tag] = stage_ms.get(tag, 0.0) + ms
    groups = {}
    for li, layer in enumerate(br.layers):
        kname = ctx.spconv_kernel(cfg.dtype, layer.cin, layer.cout, layer.kind)
        g = groups.setdefault((kname, layer.cin, layer.cout), {"ms": 0.0, "layers": []})
        g["ms"] += conv_ms[li]
        g["layers"].append(li)
    dom_key = max(groups, key=lambda k: groups[k]["ms"])
    dom_layers = groups[dom_key]["layers"]

    # timed region
    timer.reset()
    timer.only = set(("conv", li) for li in dom_layers)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        timer.enabled = (i % args.bracket_every == 0)
        step(pts, batch, timer)
    t_issued = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for c_, _ in ring:
        c_.status_sync()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    frames_per_s = cfg.n_frames * args.steps / (t1 - t0)

    # dominant kernel: durations of its launches, from the events recorded inside the timed steps
    dom_ms_total, dom_flops_total, dom_launches = 0.0, 0.0, 0
    for tag, e0, e1 in timer.records:
        dom_ms_total += e0.elapsed_time(e1)
        dom_flops_total += layer_flops[tag[1]]
        dom_launches += 1
    achieved_tflops = dom_flops_total / (dom_ms_total * 1e-3) / 1e12 if dom_ms_total > 0 else 0.0
    # a conv that runs on the matrix cores is priced against their dense 16-bit peak, one on the vector ALU
    # (fp32, or channel counts no MFMA kernel covers) against the fp32 vector peak
    dom_on_mfma = bool(ctx.uses_mfma(cfg.dtype, dom_key[1], dom_key[2]))
    dom_peak = PEAK_MFMA_F16_TFLOPS if dom_on_mfma else PEAK_VALU_F32_TFLOPS
    roofline = {
        "kernel": f"{dom_key[0]}<{DTYPE_NAME[cfg.dtype]}, Cin={dom_key[1]}, Cout={dom_key[2]}>",
        "bound": "mfma" if dom_on_mfma else "alu", "achieved": achieved_tflops, "peak": dom_peak, "unit": "TFLOP/s",
        "frac": achieved_tflops / dom_peak,
        "flops_per_launch": dom_flops_total / max(dom_launches, 1), "launches_per_step": len(dom_layers),
        "avg_launch_ms": dom_ms_total / max(dom_launches, 1), "launches_timed": dom_launches,
        "traffic": profiled_traffic(dom_key[0], cfg.index),
    }

    # the same kernel with the GPU to itself (calibration pass: one stream, one frame at a time).  In the timed
    # region above two frames share the machine, which raises throughput and lengthens every single launch.
    excl_ms = sum(conv_ms[li] for li in dom_layers)
    excl_flops = sum(layer_flops[li] for li in dom_layers)
    excl_tflops = excl_flops / (excl_ms * 1e-3) / 1e12 if excl_ms > 0 else 0.0
    roofline_exclusive = {"kernel": roofline["kernel"], "achieved": excl_tflops, "peak": dom_peak,
                          "unit": "TFLOP/s", "frac": excl_tflops / dom_peak,
                          "avg_launch_ms": excl_ms / max(len(dom_layers), 1),
                          "note": "calibration pass outside the timed region, kernel alone on the GPU"}

    # Memory-bound stages: algorithmic bytes (what the method itself must move) over the calibration pass's
    # stage time, against the published HBM peak.  voxelize: 16 B per point read, 36 B per voxel written;
    # kernel maps: 16 B of coordinates read and 27 x 4 B of map written per output voxel (+ 16 B of coordinates
    # written per stride-2 output, 16 B read per stride-2 input).
    stage_bytes = {"voxelize": n_points * 16.0 + n_vox[0] * 36.0, "kmap_subm": 0.0, "kmap_strided": 0.0}
    lvl_ = 0
    seen_subm = set()
    for layer in br.layers:
        if layer.kind == STRIDED:
            stage_bytes["kmap_strided"] += n_vox[lvl_] * 16.0 + n_vox[lvl_ + 1] * (16.0 + 16.0 + 108.0)
            lvl_ += 1
        elif lvl_ not in seen_subm:
            seen_subm.add(lvl_)
            stage_bytes["kmap_subm"] += n_vox[lvl_] * (16.0 + 108.0)
    stage_hbm = {}
    for k_, b_ in stage_bytes.items():
        if stage_ms.get(k_):
            gbs = b_ / (stage_ms[k_] * 1e-3) / 1e9
            stage_hbm[k_] = {"algorithmic_MB": b_ / 1e6, "ms": stage_ms[k_], "GB/s": gbs, "frac_of_hbm_peak": gbs / PEAK_HBM_GBS}

    # the fifth call of the boundary, on its own workload (config 3: every point of the frame samples a
    # 375 x 1242 x 64 fp16 feature map): 16 B + 4 corners x 128 B + 128 B + 1 B per point
    pg = None
    try:
        if args.headline_only:
            raise RuntimeError("skipped (--headline-only)")
        cfg3 = get_config(3)
        cam = cfg3.camera
        pts3_np, _ = gen.make_frames(cfg3)
        pts3 = torch.from_numpy(pts3_np).cuda()
        img = torch.from_numpy(gen.make_image(cam.height, cam.width, cam.channels, gen.frame_seed(3, 0))).cuda()
        pm = gen.make_camera(gen.frame_seed(3, 0))
        g_out = torch.empty((len(pts3_np), cam.channels), dtype=torch.float16, device="cuda")
        g_valid = torch.empty((len(pts3_np),), dtype=torch.uint8, device="cuda")
        for _ in range(3):
            ctx.project_gather(pts3, pm, img, g_out, g_valid)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(20):
            ctx.project_gather(pts3, pm, img, g_out, g_valid)
        e1.record()
        torch.cuda.synchronize()
        pg_ms = e0.elapsed_time(e1) / 20.0
        pg_bytes = len(pts3_np) * (16.0 + 4 * 2.0 * cam.channels + 2.0 * cam.channels + 1.0)
        pg = {"workload": f"config 3: {len(pts3_np)} points, image {cam.height}x{cam.width}x{cam.channels} f16",
              "ms": pg_ms, "algorithmic_MB": pg_bytes / 1e6, "GB/s": pg_bytes / (pg_ms * 1e-3) / 1e9,
              "frac_of_hbm_peak": pg_bytes / (pg_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
              "valid_points": int(g_valid.sum().item())}
        del img, g_out, g_valid, pts3
    except Exception as exc:  # the side measurement must never take the headline number down with it
        pg = {"error": repr(exc)}

    # Decoder-side calls on this frame's levels (outside the timed region): the inverse map of the last stride-2
    # layer, the transposed 64->64 conv over it, and the bird's-eye-view flattening of the coarsest level.
    dec = None
    try:
        if args.headline_only:
            raise RuntimeError("skipped (--headline-only)")
        runner.run(pts, batch)
        torch.cuda.synchronize()
        fine, coarse = runner.levels[-2], runner.levels[-1]
        nf, nc = int(fine.n.item()), int(coarse.n.item())
        inv = torch.empty((27, fine.cap), dtype=torch.int32, device="cuda")
        x_c = runner.acts[-1]
        cch = int(x_c.shape[1])
        w_t = torch.randn((27, cch, cch), device="cuda").mul_(0.1).to(x_c.dtype)
        sc = torch.full((cch,), 0.1, dtype=torch.float32, device="cuda")
        sh = torch.zeros((cch,), dtype=torch.float32, device="cuda")
        lay = B.W_PLAIN
        if ctx.uses_mfma(cfg.dtype, cch, cch):
            w_p = torch.empty_like(w_t)
            ctx.pack_weights(cfg.dtype, w_t, w_p)
            w_t, lay = w_p, B.W_PACKED
        y_f = torch.empty((fine.cap, cch), dtype=x_c.dtype, device="cuda")
        bev = torch.empty((br.spec.n_batch, coarse.grid[1], coarse.grid[0], coarse.grid[2] * cch), dtype=x_c.dtype, device="cuda")

        def timed(fn, reps=20):
            for _ in range(3):
                fn()
            e0_, e1_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0_.record()
            for _ in range(reps):
                fn()
            e1_.record()
            torch.cuda.synchronize()
            return e0_.elapsed_time(e1_) / reps

        ms_inv = timed(lambda: ctx.build_inverse_kmap(fine.coords, fine.n, fine.cap, coarse.grid, br.spec.n_batch, coarse.slot, coarse.n, inv))
        pairs_t = int((inv[:, :nf] >= 0).sum().item())
        ms_tc = timed(lambda: ctx.spconv(cfg.dtype, x_c, w_t, sc, sh, 2, inv, fine.n, fine.cap, y_f, w_layout=lay))
        ms_bev = timed(lambda: ctx.bev_flatten(cfg.dtype, coarse.coords, x_c, coarse.n, coarse.cap, coarse.grid, br.spec.n_batch, bev))
        esz = x_c.element_size()
        inv_bytes = nf * (16.0 + 108.0)
        bev_bytes = bev.numel() * esz + nc * (16.0 + 2.0 * cch * esz)
        fl_t = 2.0 * pairs_t * cch * cch
        dec = {"inverse_kmap": {"fine": nf, "coarse": nc, "ms": ms_inv, "algorithmic_MB": inv_bytes / 1e6,
                                "GB/s": inv_bytes / (ms_inv * 1e-3) / 1e9, "frac_of_hbm_peak": inv_bytes / (ms_inv * 1e-3) / 1e9 / PEAK_HBM_GBS},
               "transposed_conv": {"cin": cch, "cout": cch, "pairs": pairs_t, "ms": ms_tc, "kernel": ctx.spconv_kernel(cfg.dtype, cch, cch),
                                   "useful_tflops": fl_t / (ms_tc * 1e-3) / 1e12, "frac_of_mfma_peak": fl_t / (ms_tc * 1e-3) / 1e12 / PEAK_MFMA_F16_TFLOPS},
               "bev_flatten": {"voxels": nc, "dense_MB": bev.numel() * esz / 1e6, "ms": ms_bev, "algorithmic_MB": bev_bytes / 1e6,
                               "GB/s": bev_bytes / (ms_bev * 1e-3) / 1e9, "frac_of_hbm_peak": bev_bytes / (ms_bev * 1e-3) / 1e9 / PEAK_HBM_GBS}}
        del inv, y_f, bev, w_t
    except Exception as exc:
        dec = {"error": repr(exc)}

    # Multimodal leg of the data bridge on config 3 (outside the timed region): the 375 x 1242 x 64 feature map
    # pooled on each of the three scales, then fused with that scale's LiDAR voxels (32 channels) into 96-channel
    # rows.  Algorithmic bytes: pooling reads 4 B of depth per pixel and one 2C-byte row per pixel that lands in
    # the grid, writes 20 + 2C B per cell; fusion reads 16 B + a row per input site and writes 16 B + a row per
    # fused site.
    bridge = None
    try:
        if args.headline_only:
            raise RuntimeError("skipped (--headline-only)")
        cfg3 = get_config(3)
        cam = cfg3.camera
        npix = cam.height * cam.width
        seed3 = gen.frame_seed(3, 0)
        pts3_np, _ = gen.make_frames(cfg3)
        ctx_b = B.Context(max(npix, len(pts3_np)), npix + len(pts3_np), cells_of(cfg3.branches[0].spec.grid, cfg3.branches[0].spec.n_batch), n_slots=3)
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

        def timed_b(fn, reps=20):
            for _ in range(3):
                fn()
            e0_, e1_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0_.record()
            for _ in range(reps):
                fn()
            e1_.record()
            torch.cuda.synchronize()
            return e0_.elapsed_time(e1_) / reps

        scales = []
        for br3 in cfg3.branches:
            sp3 = br3.spec
            row = {"scale": br3.name, "cell_m": list(sp3.vs)}
            for mode, nm in ((B.POOL_MEAN, "mean"), (B.POOL_MAX, "max")):
                ms_p = timed_b(lambda: ctx_b.pool_image(fmap, dmap, qm, sp3, mode, cap_b, ic, if_, icnt, n_i, index_slot=1))
                ni = int(n_i.item())
                pooled = int(icnt[:ni].sum().item())
                pb = npix * 4.0 + pooled * 2.0 * cam.channels + ni * (20.0 + 2.0 * cam.channels)
                row["pool_" + nm] = {"ms": ms_p, "cells": ni, "pixels_pooled": pooled, "algorithmic_MB": pb / 1e6,
                                     "GB/s": pb / (ms_p * 1e-3) / 1e9, "frac_of_hbm_peak": pb / (ms_p * 1e-3) / 1e9 / PEAK_HBM_GBS}
            nl = ctx_b.voxelize(pts3, None, sp3, cap_b, lc, lm, lcnt, n_l, index_slot=0, sync_count=True)
            ms_f = timed_b(lambda: ctx_b.fuse(cfg3.dtype, lc, lf, n_l, cap_b, ic, if_, n_i, cap_b, sp3.grid, sp3.n_batch, cap_b,
                                              fc, ff, n_f, out_slot=2))
            nf_ = int(n_f.item())
            fb = nl * (16.0 + 64.0) + ni * (16.0 + 2.0 * cam.channels) + nf_ * (16.0 + 192.0)
            row["fuse"] = {"ms": ms_f, "voxels": nl, "image_cells": ni, "fused": nf_, "shared": nl + ni - nf_,
                           "algorithmic_MB": fb / 1e6, "GB/s": fb / (ms_f * 1e-3) / 1e9,
                           "frac_of_hbm_peak": fb / (ms_f * 1e-3) / 1e9 / PEAK_HBM_GBS}
            scales.append(row)
        ctx_b.status_sync()
        bridge = {"workload": f"config 3: image {cam.height}x{cam.width}x{cam.channels} f16 with depth ({int((dmap > 0).sum().item())} "
                              f"relevant pixels), {len(pts3_np)} points", "scales": scales}
        ctx_b.close()
        del fmap, dmap, ic, if_, lc, lf, fc, ff, pts3
    except Exception as exc:
        bridge = {"error": repr(exc)}

    # Scenario-Adaptive Dispatcher (outside the timed region): one batch of 8 scenes as in config 5, and a large
    # batch of 1024 scenes; 20 B per proposal read, 8 B per scene written.
    disp = None
    try:
        if args.headline_only:
            raise RuntimeError("skipped (--headline-only)")
        disp = []
        for n_sc in (8, 1024):
            pr_np, sc_np = gen.make_proposals(n_sc, seed)
            pr, sc_t = torch.from_numpy(pr_np).cuda(), torch.from_numpy(sc_np).cuda()
            ex = torch.empty((n_sc,), dtype=torch.int32, device="cuda")
            cn = torch.empty((3,), dtype=torch.int32, device="cuda")
            od = torch.empty((n_sc,), dtype=torch.int32, device="cuda")
            for _ in range(3):
                ctx.dispatch(pr, sc_t, n_sc, 23.5, 0.5, ex, cn, od)
            e0_, e1_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0_.record()
            for _ in range(20):
                ctx.dispatch(pr, sc_t, n_sc, 23.5, 0.5, ex, cn, od)
            e1_.record()
            torch.cuda.synchronize()
            ms_d = e0_.elapsed_time(e1_) / 20.0
            db = len(pr_np) * 20.0 + n_sc * 8.0
            disp.append({"scenes": n_sc, "proposals": len(pr_np), "ms": ms_d, "scenes_per_expert": cn.tolist(),
                         "algorithmic_MB": db / 1e6, "GB/s": db / (ms_d * 1e-3) / 1e9})
    except Exception as exc:
        disp = {"error": repr(exc)}

    # Quantised conv (outside the timed region): the int8 kernel on the two 64 -> 64 maps of this frame (level-2
    # submanifold, the shape of the dominant kernel, and the stride-2 map into level 3), beside the fp16 kernel
    # on the same maps.  Useful operations = 2 x pairs x 64 x 64 against the published dense int8 peak.
    quant = None
    try:
        if args.headline_only:
            raise RuntimeError("skipped (--headline-only)")
        runner.run(pts, batch)
        torch.cuda.synchronize()
        quant = []
        for li, layer in enumerate(br.layers):
            if not (layer.cin == 64 and layer.cout == 64) or any(q_["strided"] == (layer.kind == STRIDED) for q_ in quant):
                continue
            lvl_out = sum(1 for l_ in br.layers[:li + 1] if l_.kind == STRIDED)
            lv_o = runner.levels[lvl_out]
            nbr_t = lv_o.down_nbr if layer.kind == STRIDED else lv_o.subm_nbr
            n_in = int(runner.levels[lvl_out - 1].n.item()) if layer.kind == STRIDED else int(lv_o.n.item())
            xq = torch.randint(-127, 128, (max(n_in, 1), 64), dtype=torch.int8, device="cuda")
            wq = torch.randint(-60, 61, (27, 64, 64), dtype=torch.int8, device="cuda")
            wpk = torch.empty((27 * 64 * 64,), dtype=torch.int8, device="cuda")
            ctx.pack_weights_i8(wq, wpk)
            ml = torch.full((64,), 1e-5, dtype=torch.float32, device="cuda")
            ad = torch.zeros((64,), dtype=torch.float32, device="cuda")
            yq = torch.empty((lv_o.cap, 64), dtype=torch.int8, device="cuda")
            for _ in range(3):
                ctx.spconv_i8(xq, wpk, 64, 64, ml, ad, True, nbr_t, lv_o.n, lv_o.cap, yq, inv_out_scale=30.0)
            e0_, e1_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0_.record()
            for _ in range(20):
                ctx.spconv_i8(xq, wpk, 64, 64, ml, ad, True, nbr_t, lv_o.n, lv_o.cap, yq, inv_out_scale=30.0)
            e1_.record()
            torch.cuda.synchronize()
            ms_q = e0_.elapsed_time(e1_) / 20.0
            ops = 2.0 * layer_pairs[li] * 64 * 64
            quant.append({"cin": 64, "cout": 64, "strided": layer.kind == STRIDED, "pairs": layer_pairs[li], "ms_int8": ms_q,
                          "ms_fp16_same_map": conv_ms[li], "useful_TOPS": ops / (ms_q * 1e-3) / 1e12,
                          "frac_of_int8_peak": ops / (ms_q * 1e-3) / 1e12 / 5000.0})
            del xq, yq
    except Exception as exc:
        quant = {"error": repr(exc)}

    # Voxelizer alone at growing batch (the bandwidth claim: one frame is ~6 MB of algorithmic traffic, far too
    # little to be anything but launch- and latency-bound; many frames per launch show what the kernels sustain)
    vox_scaling = []
    if args.config == 2 and not args.no_scaling_sweep and not args.headline_only:
        try:
            from paper_2507_04123_amd.configs import VoxelSpec
            for nb_ in (1, 8, 32):
                pts_b = pts.repeat(nb_, 1).contiguous()
                bid = torch.arange(nb_, dtype=torch.int32, device="cuda").repeat_interleave(n_points).contiguous()
                sp_ = VoxelSpec(br.spec.lo, br.spec.vs, br.spec.grid, n_batch=nb_)
                cap_ = n_points * nb_
                cx_ = B.Context(cap_, cap_, cells_of(sp_.grid, nb_), n_slots=1)
                co_ = torch.empty((cap_, 4), dtype=torch.int32, device="cuda")
                fe_ = torch.empty((cap_, 4), dtype=torch.float32, device="cuda")
                cn_ = torch.empty((cap_,), dtype=torch.int32, device="cuda")
                nn_ = torch.zeros(1, dtype=torch.int32, device="cuda")
                for _ in range(2):
                    cx_.voxelize(pts_b, bid, sp_, cap_, co_, fe_, cn_, nn_, index_slot=0)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for _ in range(5):
                    cx_.voxelize(pts_b, bid, sp_, cap_, co_, fe_, cn_, nn_, index_slot=0)
                e1.record()
                torch.cuda.synchronize()
                cx_.status_sync()
                ms_ = e0.elapsed_time(e1) / 5.0
                nv_ = int(nn_.item())
                by_ = cap_ * 20.0 + nv_ * 36.0   # 16 B point + 4 B batch id read; 36 B per voxel written
                vox_scaling.append({"frames": nb_, "points": cap_, "voxels": nv_, "ms": ms_,
                                    "Mpts/s": cap_ / (ms_ * 1e-3) / 1e6, "GB/s": by_ / (ms_ * 1e-3) / 1e9,
                                    "frac_of_hbm_peak": by_ / (ms_ * 1e-3) / 1e9 / PEAK_HBM_GBS})
                cx_.close()
                del pts_b, bid, co_, fe_, cn_, nn_
        except Exception as exc:
            vox_scaling.append({"error": repr(exc)})

    total_flops = sum(layer_flops)
    vox_ms = stage_ms.get("voxelize", 0.0)
    out = {
        "metric": "frames/s through voxelize+spconv backbone",
        "value": frames_per_s, "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "host_issue_ms_per_step": (t_issued - t0) * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE_NAME[cfg.dtype], "data": "synthetic",
        "streams": 1 if args.serial else 2, "frames_in_flight": depth, "hip_graphs": bool(use_graphs),
        "config": {"workload": f"config {cfg.index} ({cfg.name}): {cfg.n_points} points x {cfg.n_frames} frame(s), "
                               f"grid {br.spec.grid}, {len(br.layers)} sparse convs", "capacities": caps,
                   "voxels_per_level": n_vox},
        "roofline": roofline,
        "roofline_exclusive": roofline_exclusive,
        "stages_ms_calibration_pass": stage_ms,
        "voxelize_mpts_per_s": (n_points / (vox_ms * 1e-3) / 1e6) if vox_ms > 0 else None,
        "conv_useful_gflop_per_frame": total_flops / 1e9,
        "conv_useful_tflops": total_flops / (stage_ms.get("conv", 0.0) * 1e-3) / 1e12 if stage_ms.get("conv") else None,
        "memory_bound_stages": stage_hbm,
        "project_gather": pg,
        "decoder_side": dec,
        "multimodal_bridge": bridge,
        "dispatcher": disp,
        "quantised_conv": quant,
        "voxelize_scaling": vox_scaling,
        "conv_layers": [{"cin": l.cin, "cout": l.cout, "strided": l.kind == STRIDED, "pairs": p, "ms": m,
                         "kernel": ctx.spconv_kernel(cfg.dtype, l.cin, l.cout, l.kind),
                         "useful_tflops": (f / (m * 1e-3) / 1e12) if m > 0 else None,
                         "frac_of_mfma_peak": (f / (m * 1e-3) / 1e12 / PEAK_MFMA_F16_TFLOPS) if m > 0 else None}
                        for l, p, m, f in zip(br.layers, layer_pairs, conv_ms, layer_flops)],
    }
    for c_, _ in ring:
        c_.close()
    if not args.no_cpu_baseline:
        import oracle
        threads = min(oracle.max_threads(), 16)
        out["cpu_baseline"] = cpu_baseline(cfg, pts_np, seed, threads)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
