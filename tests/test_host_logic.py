"""Host-side logic that needs no GPU: the workload table, the seeded generators, the bench's argument handling and
the profile summaries it reads."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

from paper_2507_04123_amd import gen  # noqa: E402
from paper_2507_04123_amd.configs import CONFIGS, STRIDED, SUBM, expert_branches, get_config, out_grid  # noqa: E402


def test_workload_table_shapes():
    assert [c.index for c in CONFIGS] == [1, 2, 3, 4, 5]
    c2, c3, c4, c5 = get_config(2), get_config(3), get_config(4), get_config(5)
    assert tuple(c2.branches[0].spec.grid) == (1408, 1600, 40) and len(c2.branches[0].layers) == 10
    assert [tuple(b.spec.grid) for b in c3.branches] == [(1408, 1600, 40), (704, 800, 20), (352, 400, 10)]
    assert c3.camera is not None and (c3.camera.height, c3.camera.width, c3.camera.channels) == (375, 1242, 64)
    assert tuple(c4.branches[0].spec.grid) == (1440, 1440, 41) and len(c4.branches[0].layers) == 12
    assert c5.n_frames == 8 and [b.name for b in c5.branches] == ["near", "far"]
    assert c5.branches[0].spec.r2_max == 900.0 and c5.branches[1].spec.r2_min == 900.0
    # channel counts chain through every stack, and a stage is one stride-2 layer followed by submanifold layers
    for cfg in CONFIGS:
        for br in cfg.branches:
            cin = 4
            for layer in br.layers:
                assert layer.cin == cin and layer.kind in (SUBM, STRIDED)
                cin = layer.cout
    assert out_grid((1408, 1600, 40)) == (704, 800, 20) and out_grid((1440, 1440, 41)) == (720, 720, 21)
    assert out_grid((5, 4, 1)) == (3, 2, 1)


def test_expert_stacks_share_the_batch_size():
    lpe, vee, ape = expert_branches(8)
    assert all(b.spec.n_batch == 8 for b in (lpe, vee, ape))
    assert len(lpe.layers) < len(vee.layers) < len(ape.layers)
    assert lpe.spec.vs[0] > vee.spec.vs[0] == ape.spec.vs[0]      # the latency expert works on coarser voxels


def test_generators_are_seeded_and_frames_differ():
    cfg = get_config(1)
    a, _ = gen.make_frames(cfg)
    b, _ = gen.make_frames(cfg)
    c, _ = gen.make_frames(cfg, first_frame=1)
    assert a.dtype == np.float32 and a.shape == (2000, 4)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    assert gen.frame_seed(2, 0) != gen.frame_seed(2, 1) != gen.frame_seed(3, 1)
    cfg5 = get_config(5)
    p, bt = gen.make_frames(cfg5)
    assert p.shape == (8 * 120000, 4) and bt.dtype == np.int32
    assert np.array_equal(np.unique(bt), np.arange(8)) and np.all(np.bincount(bt) == 120000)


def test_proposals_cover_every_expert_and_sit_on_thresholds():
    props, scene = gen.make_proposals(64, 11)
    assert props.dtype == np.float32 and props.shape[1] == 4 and scene.shape == (len(props),)
    assert scene.min() >= 0 and scene.max() < 64
    r2 = props[:, 0] * props[:, 0] + props[:, 1] * props[:, 1]
    d2 = np.float32(23.5) * np.float32(23.5)
    assert (r2 < d2).any() and (r2 >= d2).any()
    assert (props[:, 3] == np.float32(0.5)).any(), "some confidences lie exactly on the threshold"


def test_bench_refuses_more_than_one_gpu():
    cp = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                        stderr=subprocess.PIPE, timeout=120, check=False)
    assert cp.returncode == 2 and cp.stdout == b""
    assert b"one GPU" in cp.stderr


def test_bench_reads_the_committed_traffic_summaries():
    sys.path.insert(0, ROOT)
    import bench
    for kernel, cfg in (("k_spconv_span", 5), ("k_spconv_span", 2), ("k_spconv_direct", 4)):
        t = bench.profiled_traffic(kernel, cfg)
        assert t is not None and 1e7 < t < 1e9, (kernel, cfg, t)
    assert bench.profiled_traffic("k_no_such_kernel", 5) is None
    # every summary names the command that produced it, and that command runs committed files only
    pdir = os.path.join(ROOT, "profiles")
    for name in os.listdir(pdir):
        text = open(os.path.join(pdir, name)).read()
        assert "rocprofv3" in text and "bench.py" in text, name
        assert "_work" not in text, name
