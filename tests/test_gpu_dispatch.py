"""GPU parity of the Scenario-Adaptive Dispatcher (through the C-ABI) against the CPU oracle: integer results,
bit-exact, on both launch paths (one block for small batches, three launches for large ones)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2507_04123_amd import binding as B
from paper_2507_04123_amd import gen

pytestmark = pytest.mark.gpu


def gpu_dispatch(ctx, props, scene, n_scenes, d, c):
    dp = torch.from_numpy(np.ascontiguousarray(props)).cuda() if len(props) else torch.zeros((0, 4), device="cuda")
    ds = None if scene is None else torch.from_numpy(np.ascontiguousarray(scene)).cuda()
    expert = torch.full((n_scenes + 3,), -7, dtype=torch.int32, device="cuda")
    counts = torch.full((3,), -7, dtype=torch.int32, device="cuda")
    order = torch.full((n_scenes + 3,), -7, dtype=torch.int32, device="cuda")
    ctx.dispatch(dp, ds, n_scenes, d, c, expert, counts, order)
    torch.cuda.synchronize()
    assert expert[n_scenes:].tolist() == [-7] * 3 and order[n_scenes:].tolist() == [-7] * 3
    return expert[:n_scenes].cpu().numpy(), counts.cpu().numpy(), order[:n_scenes].cpu().numpy()


@pytest.mark.parametrize("n_scenes,d,c,seed,per", [(1, 23.5, 0.5, 1, 300), (8, 23.5, 0.5, 2, 300), (8, 35.0, 0.3, 3, 300),
                                                   (200, 35.0, 0.3, 4, 100),       # one block, many scenes
                                                   (1000, 23.5, 0.7, 5, 300),      # large: three launches
                                                   (9000, 23.5, 0.5, 6, 3),        # more scenes than the block keeps in LDS
                                                   (3000, 35.0, 0.5, 7, 40)])
def test_dispatch_matches_oracle(n_scenes, d, c, seed, per):
    ctx = B.Context(16, 16, 64, n_slots=1)
    props, scene = gen.make_proposals(n_scenes, seed, d, c, max_per_scene=per)
    if len(props) > 10:
        scene[::97] = n_scenes + 3          # ids outside the batch
        scene[5] = -1
        props[7, 3] = np.nan                # unreadable values
        props[9, 0] = np.inf
    print(f"dispatch scenes={n_scenes} proposals={len(props)} D={d} C={c}", flush=True)
    e, counts, order = gpu_dispatch(ctx, props, scene, n_scenes, d, c)
    oe, oc, oo = oracle.dispatch(props, scene, n_scenes, d, c)
    assert np.array_equal(e, oe) and np.array_equal(counts, oc) and np.array_equal(order, oo)
    ctx.close()


def test_dispatch_edge_cases():
    ctx = B.Context(16, 16, 64, n_slots=1)
    # no proposal at all: every scene is a latency-prioritised one
    e, counts, order = gpu_dispatch(ctx, np.zeros((0, 4), np.float32), None, 5, 23.5, 0.5)
    assert e.tolist() == [0] * 5 and counts.tolist() == [5, 0, 0] and order.tolist() == [0, 1, 2, 3, 4]
    # no scene array: everything belongs to scene 0; thresholds are ">= D is far", ">= C is clear"
    rows = np.array([[23.5, 0, 0, 0.9]], np.float32)
    assert gpu_dispatch(ctx, rows, None, 1, 23.5, 0.5)[0].tolist() == [1]
    rows = np.array([[np.nextafter(np.float32(23.5), np.float32(0)), 0, 0, 0.5]], np.float32)
    assert gpu_dispatch(ctx, rows, None, 1, 23.5, 0.5)[0].tolist() == [0]
    rows = np.array([[3, 4, 50, 0.9], [30, 40, 0, 0.1]], np.float32)
    e, counts, order = gpu_dispatch(ctx, rows, np.array([1, 0], np.int32), 3, 5.001, 0.5)
    assert e.tolist() == [2, 0, 0] and counts.tolist() == [2, 0, 1] and order.tolist() == [1, 2, 0]
    # arguments the entry point must refuse
    z = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(B.Emc2Error):
        ctx.dispatch(torch.zeros((1, 4), device="cuda"), None, 1, -1.0, 0.5, z, z, z)
    with pytest.raises(B.Emc2Error):
        ctx.dispatch(torch.zeros((1, 4), device="cuda"), None, 1, 23.5, float("nan"), z, z, z)
    ctx.close()
