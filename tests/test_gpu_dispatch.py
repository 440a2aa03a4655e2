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


# ------------------------------------------------------------------------------------------------
# expert-grouped batching: emc2_group_points and the routed runner
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("n_scenes,seed", [(1, 1), (8, 2), (300, 3)])
def test_group_points_matches_oracle(n_scenes, seed):
    ctx = B.Context(16, 16, 64, n_slots=1)
    props, pscene = gen.make_proposals(n_scenes, seed, max_per_scene=40)
    e_np, c_np, o_np = oracle.dispatch(props, pscene, n_scenes, 23.5, 0.5)
    st = gen.Stream(seed, 31)
    n_pts = 7013
    scene = (st.bits(n_pts) % np.uint64(n_scenes + 2)).astype(np.int32) - 1            # ids -1 .. n_scenes: two invalid
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    for e in (0, 1, 2):
        slot = torch.full((n_scenes + 2,), -7, dtype=torch.int32, device="cuda")
        gb = torch.full((n_pts + 2,), -7, dtype=torch.int32, device="cuda")
        ctx.group_points(dev(scene), n_pts, dev(e_np), dev(o_np), dev(c_np), n_scenes, e, slot, gb)
        torch.cuda.synchronize()
        oslot, ogb = oracle.group_points(scene, n_pts, e_np, o_np, c_np, e)
        assert np.array_equal(slot[:n_scenes].cpu().numpy(), oslot) and slot[n_scenes:].tolist() == [-7, -7]
        assert np.array_equal(gb[:n_pts].cpu().numpy(), ogb) and gb[n_pts:].tolist() == [-7, -7]
    # no scene array: every point is in scene 0
    gb = torch.empty((5,), dtype=torch.int32, device="cuda")
    slot = torch.empty((n_scenes,), dtype=torch.int32, device="cuda")
    ctx.group_points(None, 5, dev(e_np), dev(o_np), dev(c_np), n_scenes, int(e_np[0]), slot, gb)
    assert gb.tolist() == [0] * 5
    with pytest.raises(B.Emc2Error):
        ctx.group_points(None, 5, dev(e_np), dev(o_np), dev(c_np), n_scenes, 3, slot, gb)
    ctx.close()


def test_routed_runner_matches_the_ungrouped_run_scene_by_scene():
    """Eight scenes (config 5's batch), routed by seeded proposals: every expert's stack runs on its group only, and
    for each scene the voxels and kernel maps of every level equal, bit for bit, those of the same stack run on the
    whole batch (frame index and voxel indices shifted), the features up to the voxel means' summation order."""
    from helpers import assert_features_close, progress
    from paper_2507_04123_amd.configs import get_config, expert_branches, STRIDED
    from paper_2507_04123_amd.pipeline import BranchRunner, RoutedRunner, cells_of, default_capacities, device_params
    cfg = get_config(5)
    n_scenes = cfg.n_frames
    pts_np, scene_np = gen.make_frames(cfg)
    props_np, pscene_np = gen.make_proposals(n_scenes, 11)
    pts, scene = torch.from_numpy(pts_np).cuda(), torch.from_numpy(scene_np).cuda()
    props, pscene = torch.from_numpy(props_np).cuda(), torch.from_numpy(pscene_np).cuda()
    experts = expert_branches(n_scenes)
    seed = gen.frame_seed(5, 0)
    rr = RoutedRunner(experts, cfg.dtype, len(pts_np), n_scenes, seed)
    outs = rr.run(pts, scene, props, pscene, 23.5, 0.5)
    torch.cuda.synchronize()
    rr.status_sync()
    e_np, c_np, o_np = oracle.dispatch(props_np, pscene_np, n_scenes, 23.5, 0.5)
    assert np.array_equal(rr.expert.cpu().numpy(), e_np) and np.array_equal(rr.counts.cpu().numpy(), c_np)
    assert np.array_equal(rr.order.cpu().numpy(), o_np)
    progress(f"routed runner: experts {e_np.tolist()} counts {c_np.tolist()}")
    assert len(set(e_np.tolist())) >= 2, "the seeded proposals should exercise more than one expert"

    def scene_ranges(coords, n, nb):
        b = coords[:n, 0]
        starts = np.searchsorted(b, np.arange(nb), side="left")
        ends = np.searchsorted(b, np.arange(nb), side="right")
        return starts, ends

    for e, br in enumerate(experts):
        if c_np[e] == 0:
            continue
        # the same stack on the whole batch, original frame indices
        caps = default_capacities(br, len(pts_np))
        ctx = B.Context(len(pts_np), max(caps), cells_of(br.spec.grid, n_scenes), n_slots=len(caps))
        ref = BranchRunner(ctx, br, cfg.dtype, len(pts_np), device_params(br.layers, seed + e, cfg.dtype), capacities=caps)
        ref_out = ref.run(pts, scene)
        torch.cuda.synchronize()
        ctx.status_sync()
        grp = rr.runners[e][1]
        slot_of = {int(s): int(np.flatnonzero(o_np[int(c_np[:e].sum()):int(c_np[:e + 1].sum())] == s)[0]) for s in np.flatnonzero(e_np == e)}
        progress(f"  expert {e} ({br.name}): scenes -> slots {slot_of}")
        for lvl in range(len(ref.levels)):
            ng, nr = int(grp.levels[lvl].n.item()), int(ref.levels[lvl].n.item())
            cg, cr = grp.levels[lvl].coords[:ng].cpu().numpy(), ref.levels[lvl].coords[:nr].cpu().numpy()
            sg, eg = scene_ranges(cg, ng, n_scenes)
            sr, er = scene_ranges(cr, nr, n_scenes)
            assert ng == sum(er[s] - sr[s] for s in slot_of), "the group holds exactly its scenes' voxels"
            for s, k in slot_of.items():
                assert eg[k] - sg[k] == er[s] - sr[s]
                assert np.array_equal(cg[sg[k]:eg[k], 1:], cr[sr[s]:er[s], 1:]), f"expert {e} level {lvl} scene {s}: coordinates"
        lvl = 0
        for li, layer in enumerate(br.layers):
            if layer.kind == STRIDED:
                lvl += 1
            mg, lg = grp.layer_map(li)
            mr, lr = ref.layer_map(li)
            ng, nr = int(lg.n.item()), int(lr.n.item())
            cg, cr = lg.coords[:ng].cpu().numpy(), lr.coords[:nr].cpu().numpy()
            sg, eg = scene_ranges(cg, ng, n_scenes)
            sr, er = scene_ranges(cr, nr, n_scenes)
            # the rows a map entry names belong to the input level of the layer
            lin_g = grp.levels[lvl - 1] if layer.kind == STRIDED else lg
            lin_r = ref.levels[lvl - 1] if layer.kind == STRIDED else lr
            nig, nir = int(lin_g.n.item()), int(lin_r.n.item())
            isg, _ = scene_ranges(lin_g.coords[:nig].cpu().numpy(), nig, n_scenes)
            isr, _ = scene_ranges(lin_r.coords[:nir].cpu().numpy(), nir, n_scenes)
            mg_np, mr_np = mg[:, :ng].cpu().numpy(), mr[:, :nr].cpu().numpy()
            fg, fr = grp.acts[li][:ng].float().cpu().numpy(), ref.acts[li][:nr].float().cpu().numpy()
            for s, k in slot_of.items():
                a, b_ = mg_np[:, sg[k]:eg[k]], mr_np[:, sr[s]:er[s]]
                assert np.array_equal(a >= 0, b_ >= 0)
                assert np.array_equal(np.where(a >= 0, a - isg[k], -1), np.where(b_ >= 0, b_ - isr[s], -1)), (
                    f"expert {e} layer {li} scene {s}: kernel map")
                assert_features_close(fg[sg[k]:eg[k]], fr[sr[s]:er[s]], 2e-2, f"expert {e} layer {li} scene {s}: features")
        ctx.close()
    rr.close()


def test_routed_runner_graph_replays_follow_their_inputs():
    """One routed pass recorded as a HIP graph and replayed on changing proposals and points (written into the captured
    tensors in place): every replay routes the scenes as the oracle does for the inputs of that replay and leaves the
    same voxels, maps and features as the same pass issued from the host, with eager work between the replays."""
    from helpers import assert_features_close, progress
    from paper_2507_04123_amd.configs import get_config, expert_branches
    from paper_2507_04123_amd.pipeline import RoutedRunner
    cfg = get_config(5)
    n_scenes = cfg.n_frames
    n_props = 600
    frames = [gen.make_frames(cfg, first_frame=8 * k) for k in range(3)]
    prop_sets = []
    for k in range(3):
        p_np, s_np = gen.make_proposals(n_scenes, 21 + k)
        idx = np.resize(np.arange(len(p_np)), n_props)          # the captured proposal count is fixed: repeat to fill
        prop_sets.append((p_np[idx].copy(), s_np[idx].copy()))
    pts = torch.from_numpy(frames[0][0]).cuda()
    scene = torch.from_numpy(frames[0][1]).cuda()
    props = torch.from_numpy(prop_sets[0][0]).cuda()
    pscene = torch.from_numpy(prop_sets[0][1]).cuda()
    experts = expert_branches(n_scenes)
    seed = gen.frame_seed(5, 0)
    rr = RoutedRunner(experts, cfg.dtype, pts.shape[0], n_scenes, seed)
    ref = RoutedRunner(experts, cfg.dtype, pts.shape[0], n_scenes, seed)
    rr.run(pts, scene, props, pscene, 23.5, 0.5)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        rr.capture(pts, scene, props, pscene, 23.5, 0.5)
    torch.cuda.synchronize()
    seen = set()
    for it in range(5):
        k = it % 3
        pts.copy_(torch.from_numpy(frames[k][0]))
        scene.copy_(torch.from_numpy(frames[k][1]))
        props.copy_(torch.from_numpy(prop_sets[k][0]))
        pscene.copy_(torch.from_numpy(prop_sets[k][1]))
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            outs = rr.replay()
        torch.cuda.synchronize()
        rr.status_sync()
        e_np, c_np, o_np = oracle.dispatch(prop_sets[k][0], prop_sets[k][1], n_scenes, 23.5, 0.5)
        assert np.array_equal(rr.expert.cpu().numpy(), e_np) and np.array_equal(rr.counts.cpu().numpy(), c_np)
        assert np.array_equal(rr.order.cpu().numpy(), o_np)
        seen.add(tuple(c_np.tolist()))
        progress(f"routed replay {it}: scenes per expert {c_np.tolist()}")
        exp_outs = ref.run(pts, scene, props, pscene, 23.5, 0.5)      # the same pass issued from the host (eager work between replays)
        torch.cuda.synchronize()
        ref.status_sync()
        for e, ((_, g), (_, h)) in enumerate(zip(rr.runners, ref.runners)):
            for lg, lh in zip(g.levels, h.levels):
                n = int(lh.n.item())
                assert int(lg.n.item()) == n
                assert torch.equal(lg.coords[:n], lh.coords[:n])
            for li in range(len(g.branch.layers)):
                mg, lvg = g.layer_map(li)
                mh, lvh = h.layer_map(li)
                n = int(lvh.n.item())
                assert torch.equal(mg[:, :n], mh[:, :n]), f"replay {it} expert {e} layer {li}: kernel map"
            n = int(h.levels[-1].n.item())
            if n:
                assert_features_close(outs[e][:n].float().cpu().numpy(), exp_outs[e][:n].float().cpu().numpy(), 2e-2,
                                      f"replay {it} expert {e} features")
    assert len(seen) >= 2, "the proposal sets should route the scenes differently"
    rr.close()
    ref.close()
