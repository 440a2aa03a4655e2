"""GPU tests of ConfigRunner (every branch of a configuration on contexts of their own, side by side, and as one HIP
graph): whatever the way of running, each branch produces what its BranchRunner produces alone -- coordinates,
counts and kernel maps bit for bit, activations up to the voxel means' summation order -- and BranchRunner itself
is held to the oracle in test_gpu_parity.py."""
import numpy as np
import pytest
import torch

from helpers import assert_features_close, progress
from paper_2507_04123_amd import binding as B
from paper_2507_04123_amd import gen
from paper_2507_04123_amd.configs import get_config
from paper_2507_04123_amd.pipeline import BranchRunner, ConfigRunner, cells_of, default_capacities, device_params

pytestmark = pytest.mark.gpu


def _snapshot(runner, out):
    ns = [int(lv.n.item()) for lv in runner.levels]
    maps = []
    for li in range(len(runner.branch.layers)):
        nbr, lv = runner.layer_map(li)
        maps.append(nbr[:, :int(lv.n.item())].clone())
    return ns, [lv.coords[:n].clone() for lv, n in zip(runner.levels, ns)], maps, out[:ns[-1]].float().clone()


def _same(a, b, what):
    assert a[0] == b[0], what
    for x, y in zip(a[1], b[1]):
        assert torch.equal(x, y), what
    for x, y in zip(a[2], b[2]):
        assert torch.equal(x, y), what
    assert_features_close(a[3].cpu().numpy(), b[3].cpu().numpy(), 2e-2, what)


def _reference(cfg, pts, batch):
    """Each branch alone, one call after the other, on a context of its own that is closed before the next."""
    refs = []
    for br in cfg.branches:
        caps = default_capacities(br, len(pts))
        ctx = B.Context(len(pts), max(caps), cells_of(br.spec.grid, br.spec.n_batch), n_slots=len(caps))
        seed = gen.frame_seed(cfg.index, 0) + len(br.name)
        runner = BranchRunner(ctx, br, cfg.dtype, len(pts), device_params(br.layers, seed, cfg.dtype), capacities=caps)
        out = runner.run(pts, batch)
        torch.cuda.synchronize()
        ctx.status_sync()
        refs.append(_snapshot(runner, out))
        ctx.close()
        del runner
    return refs


@pytest.mark.parametrize("cfg_index", [3, 5])
def test_config_runner_every_way_of_running_matches_the_branches_alone(cfg_index):
    cfg = get_config(cfg_index)
    pts_np, batch_np = gen.make_frames(cfg)
    pts = torch.from_numpy(pts_np).cuda()
    batch = torch.from_numpy(batch_np).cuda() if cfg.n_frames > 1 else None
    refs = _reference(cfg, pts, batch)
    progress(f"config runner cfg{cfg_index}: references done")
    cr = ConfigRunner(cfg, len(pts_np))

    def check(outs, what):
        torch.cuda.synchronize()
        cr.status_sync()
        for (ctx, r), out, ref in zip(cr.branches, outs, refs):
            _same(_snapshot(r, out), ref, f"cfg{cfg_index} {r.branch.name} {what}")

    progress("  serial run")
    check(cr.run(pts, batch), "serial")
    progress("  branches side by side")
    check(cr.run_overlapped(pts, batch), "side by side")
    check(cr.run_overlapped(pts, batch), "side by side, again")
    if cfg.camera is not None:
        exp_valid = int(cr.camera["valid"].sum().item())
        assert exp_valid > len(pts_np) // 20
    progress("  capture (one graph per branch)")
    frame = pts.clone()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        cr.capture(frame, batch)
    torch.cuda.synchronize()
    for it in range(3):
        progress(f"  replay {it}")
        with torch.cuda.stream(side):
            outs = cr.replay()
        check(outs, f"replay {it}")
        check(cr.run_overlapped(frame, batch), f"eager after replay {it}")
    progress("  capture (the whole pass as one graph without forks)")
    with torch.cuda.stream(side):
        cr.capture(frame, batch, overlapped=False)
    torch.cuda.synchronize()
    for it in range(3):
        progress(f"  flat replay {it}")
        with torch.cuda.stream(side):
            outs = cr.replay()
        check(outs, f"flat replay {it}")
        check(cr.run(frame, batch), f"eager after flat replay {it}")
    progress("  capture (two stages: maps on one stream, each branch's convolutions on another)")
    with torch.cuda.stream(side):
        cr.capture_stages(frame, batch)
    torch.cuda.synchronize()
    map_stream = torch.cuda.Stream()
    conv_streams = [torch.cuda.Stream() for _ in cr.branches]
    for it in range(3):
        progress(f"  staged replay {it}")
        outs = cr.replay_stages(map_stream, conv_streams)
        outs = cr.replay_stages(map_stream, conv_streams)     # back to back: the maps wait for the previous convolutions
        check(outs, f"staged replay {it}")
        check(cr.run_stages(frame, batch, map_stream, conv_streams), f"staged eager issue after replay {it}")
        check(cr.run(frame, batch), f"eager after staged replay {it}")
    cr.close()
