"""GPU parity of Multiscale Pooling and multimodal fusion (through the C-ABI) against the CPU oracle.

Bar: cell coordinates, pixel counts, set sizes and every copied feature bit-exact; pooled maxima bit-exact; pooled
means within 2e-3 of the fp64 mean (one rounding to fp16, 2^-11, on top of fp32 sums in no fixed order), measured
as |g - o| <= rtol * (|o| + rms(o))."""
import numpy as np
import pytest
import torch

import oracle
from helpers import assert_features_close, make_scene
from paper_2507_04123_amd import binding as B
from paper_2507_04123_amd import gen
from paper_2507_04123_amd.configs import get_config, VoxelSpec, F32, F16, BF16, SUBM, EPI_NONE

pytestmark = pytest.mark.gpu

TD = {F32: torch.float32, F16: torch.float16, BF16: torch.bfloat16}
LO = (0.0, -40.0, -3.0)
MEAN_RTOL = 2e-3


@pytest.fixture(scope="module", autouse=True)
def _threads():
    oracle.set_threads(min(16, oracle.max_threads()))
    yield


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


def gpu_pool(ctx, img, depth, q, spec, mode, cap, slot=0, batch_index=0):
    c = img.shape[2]
    coords = torch.full((cap, 4), -7, dtype=torch.int32, device="cuda")
    feats = torch.full((cap, c), 77.0, dtype=torch.float16, device="cuda")
    counts = torch.full((cap,), -3, dtype=torch.int32, device="cuda")
    n = torch.zeros(1, dtype=torch.int32, device="cuda")
    nv = ctx.pool_image(dev(img), dev(depth), q, spec, mode, cap, coords, feats, counts, n, batch_index=batch_index,
                        index_slot=slot, sync_count=True)
    assert nv == int(n.item())
    return coords, feats, counts, n, nv


def check_pool(ctx, img, depth, q, spec, mode, cap, batch_index=0):
    print(f"pool_image HxWxC={img.shape} grid={spec.grid} vs={spec.vs} mode={mode} cap={cap}", flush=True)
    coords, feats, counts, n, nv = gpu_pool(ctx, img, depth, q, spec, mode, cap, batch_index=batch_index)
    ctx.status_sync()
    oc, of, on = oracle.pool_image(img, depth, q, spec.lo, spec.vs, spec.grid, mode, spec.n_batch, batch_index)
    assert nv == len(oc)
    assert np.array_equal(coords[:nv].cpu().numpy(), oc)
    assert np.array_equal(counts[:nv].cpu().numpy(), on)
    got = feats[:nv].float().cpu().numpy()
    if mode == B.POOL_MAX:
        assert np.array_equal(got, of)                      # a maximum of fp16 values is one of them
    else:
        assert_features_close(got, of, MEAN_RTOL, "pooled means")
    if nv < cap:                                            # rows past the count: features untouched, counts untouched or 0
        assert float(feats[nv:].float().min().item()) == 77.0 and int(coords[nv:].max().item()) == -7
        assert set(np.unique(counts[nv:].cpu().numpy()).tolist()) <= {0, -3}
    return coords, feats, counts, n, nv, (oc, of, on)


@pytest.mark.parametrize("mode", [B.POOL_MEAN, B.POOL_MAX])
@pytest.mark.parametrize("c", [8, 24, 64, 128, 200, 256])
def test_pool_image_small_scenes(mode, c):
    ctx = B.Context(60 * 200, 60 * 200, 1408 * 1600 * 40, n_slots=1)
    pm, q, depth, img = make_scene(5 + c, c=c)
    for vs, grid, lo in (((0.05, 0.05, 0.1), (1408, 1600, 40), LO),          # a pixel or two per cell
                         ((0.4, 0.4, 0.4), (176, 200, 10), LO),            # tens of pixels per cell
                         ((3.2, 3.2, 4.0), (22, 25, 1), LO),               # hundreds: lists crossing many blocks
                         ((200.0, 200.0, 200.0), (1, 1, 1), (-100.0, -100.0, -100.0)),   # one cell takes everything
                         ((0.4, 0.4, 0.4), (100, 120, 4), LO)):            # most pixels fall outside the grid
        spec = VoxelSpec(lo, vs, grid)
        check_pool(ctx, img, depth, q, spec, mode, 60 * 200)
    # the proposal-masked depth map, and no relevant pixel at all
    pm, q, depth_p, _ = make_scene(5 + c, c=c, proposals=True)
    check_pool(ctx, img, depth_p, q, VoxelSpec(LO, (0.2, 0.2, 0.4), (352, 400, 10)), mode, 60 * 200)
    *_, nv, _ = check_pool(ctx, img, np.zeros_like(depth), q, VoxelSpec(LO, (0.2, 0.2, 0.4), (352, 400, 10)), mode, 100)
    assert nv == 0
    # depth values that are not depths
    weird = depth.copy()
    weird[0, :] = np.nan; weird[1, :] = np.inf; weird[2, :] = -1.0; weird[3, :] = -np.inf
    check_pool(ctx, img, weird, q, VoxelSpec(LO, (0.4, 0.4, 0.4), (176, 200, 10)), mode, 60 * 200)
    # a frame tag other than 0
    check_pool(ctx, img, depth, q, VoxelSpec(LO, (0.8, 0.8, 0.8), (88, 100, 5), n_batch=3), mode, 60 * 200, batch_index=2)
    ctx.close()


def test_pool_image_ragged_image_sizes():
    """Pixel counts that are not multiples of the block sizes, down to a single pixel."""
    ctx = B.Context(4096, 4096, 176 * 200 * 10, n_slots=1)
    for h, w in ((1, 1), (1, 37), (3, 5), (17, 129), (33, 64)):
        pm, q, depth, img = make_scene(h * w, h=60, w=200, c=16)
        depth, img = np.ascontiguousarray(depth[40:40 + h, 10:10 + w]), np.ascontiguousarray(img[40:40 + h, 10:10 + w])
        depth[depth <= 0] = 20.0                                     # every pixel relevant
        for mode in (B.POOL_MEAN, B.POOL_MAX):
            check_pool(ctx, img, depth, q, VoxelSpec(LO, (0.4, 0.4, 0.4), (176, 200, 10)), mode, 4096)
    ctx.close()


def test_pool_image_capacity_overflow_is_reported():
    ctx = B.Context(60 * 200, 60 * 200, 176 * 200 * 10, n_slots=1)
    pm, q, depth, img = make_scene(3, c=8)
    spec = VoxelSpec(LO, (0.4, 0.4, 0.4), (176, 200, 10))
    oc, of, on = oracle.pool_image(img, depth, q, spec.lo, spec.vs, spec.grid, oracle.POOL_MAX)
    cap = len(oc) // 2
    coords, feats, counts, n, nv = gpu_pool(ctx, img, depth, q, spec, B.POOL_MAX, cap)
    assert nv == cap
    with pytest.raises(B.Emc2Error) as e:
        ctx.status_sync()
    assert e.value.status == B.ERR_CAPACITY
    # the first `cap` cells in key order are still right
    assert np.array_equal(coords.cpu().numpy(), oc[:cap]) and np.array_equal(counts.cpu().numpy(), on[:cap])
    assert np.array_equal(feats.float().cpu().numpy(), of[:cap])
    ctx.status_sync()
    # arguments the entry point must refuse
    z = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(B.Emc2Error):        # more pixels than the context was sized for
        big = torch.zeros((200, 200, 8), dtype=torch.float16, device="cuda")
        ctx.pool_image(big, torch.zeros((200, 200), device="cuda"), q, spec, 0, 10, torch.zeros((10, 4), dtype=torch.int32, device="cuda"),
                       torch.zeros((10, 8), dtype=torch.float16, device="cuda"), torch.zeros(10, dtype=torch.int32, device="cuda"), z)
    with pytest.raises(B.Emc2Error):        # channel count not a multiple of 8
        im = torch.zeros((4, 4, 6), dtype=torch.float16, device="cuda")
        ctx.pool_image(im, torch.zeros((4, 4), device="cuda"), q, spec, 0, 10, torch.zeros((10, 4), dtype=torch.int32, device="cuda"),
                       torch.zeros((10, 6), dtype=torch.float16, device="cuda"), torch.zeros(10, dtype=torch.int32, device="cuda"), z)
    ctx.close()


@pytest.mark.parametrize("mode", [B.POOL_MEAN, B.POOL_MAX])
def test_pool_image_config3_full_size(mode):
    """The camera of the bridge workload (375 x 1242 x 64) pooled on each of its three scales, every element compared."""
    cfg = get_config(3)
    cam = cfg.camera
    npix = cam.height * cam.width
    ctx = B.Context(npix, npix, 1408 * 1600 * 40, n_slots=1)
    pm = gen.make_camera(gen.frame_seed(3, 0))
    q = gen.make_unprojection(pm)
    depth = gen.make_depth(cam.height, cam.width, gen.frame_seed(3, 0))
    img = gen.make_image(cam.height, cam.width, cam.channels, gen.frame_seed(3, 0))
    for br in cfg.branches:
        *_, nv, _ = check_pool(ctx, img, depth, q, br.spec, mode, npix)
        assert nv > 5000
    ctx.close()


# ------------------------------------------------------------------------------------------------------------
# fusion
# ------------------------------------------------------------------------------------------------------------

def _rand_set(seed, grid, nb, n, c, dtype):
    gx, gy, gz = grid
    total = gx * gy * gz * nb
    st = gen.Stream(seed, 7)
    if n == 0:
        return np.zeros((0, 4), np.int32), np.zeros((0, c), np.float32)
    keys = np.unique((st.bits(3 * n) % np.uint64(total)).astype(np.int64))[:n]
    keys.sort()
    coords = np.stack([keys // (gx * gy * gz), (keys // (gx * gy)) % gz, (keys // gx) % gy, keys % gx], axis=1).astype(np.int32)
    feats = gen.round_to_dtype(st.normal(len(coords) * c).astype(np.float32).reshape(-1, c), dtype)
    return coords, feats


def gpu_fuse(ctx, dtype, lc, lf, ic, if_, grid, nb, cap_out, c_out, want_src=True, slot=0, shuffle=None):
    def put(coords, feats, extra):
        cap = len(coords) + extra
        c = feats.shape[1]
        d_c = torch.full((cap, 4), 1 << 20, dtype=torch.int32, device="cuda")        # rows past n: never read
        d_f = torch.full((cap, c), 5.0, dtype=TD[dtype], device="cuda")
        if len(coords):
            order = np.arange(len(coords)) if shuffle is None else gen.Stream(shuffle, len(coords)).permutation(len(coords))
            d_c[:len(coords)] = dev(coords[order])
            d_f[:len(coords)] = dev(feats[order], TD[dtype])
        else:
            order = np.zeros(0, np.int64)
        return d_c, d_f, torch.tensor([len(coords)], dtype=torch.int32, device="cuda"), cap, order
    d_lc, d_lf, n_l, cap_l, ord_l = put(lc, lf, 5)
    d_ic, d_if, n_i, cap_i, ord_i = put(ic, if_, 3)
    co = torch.full((cap_out, 4), -7, dtype=torch.int32, device="cuda")
    fo = torch.full((cap_out, c_out), 9.0, dtype=TD[dtype], device="cuda")
    n_out = torch.zeros(1, dtype=torch.int32, device="cuda")
    sl = torch.full((cap_out,), -9, dtype=torch.int32, device="cuda") if want_src else None
    si = torch.full((cap_out,), -9, dtype=torch.int32, device="cuda") if want_src else None
    nv = ctx.fuse(dtype, d_lc, d_lf, n_l, cap_l, d_ic, d_if, n_i, cap_i, grid, nb, cap_out, co, fo, n_out, sl, si,
                  out_slot=slot, sync_count=True)
    assert nv == int(n_out.item())
    return co, fo, sl, si, n_out, nv, ord_l, ord_i


@pytest.mark.parametrize("dtype,cl,ci,pad", [(F16, 32, 64, 0), (F16, 32, 64, 32), (F32, 4, 4, 0), (BF16, 6, 10, 2), (F16, 2, 6, 0),
                                             (F32, 3, 5, 1)])
def test_fuse_matches_oracle(dtype, cl, ci, pad):
    ctx = B.Context(16, 40000, 176 * 200 * 10 * 2, n_slots=2)
    for grid, nb, nl, ni, shuffle in (((9, 7, 5), 2, 200, 150, None), ((6, 6, 6), 1, 150, 150, None), ((176, 200, 10), 2, 9000, 15000, None),
                                      ((5, 5, 2), 3, 0, 40, None), ((5, 5, 2), 3, 40, 0, None), ((4, 4, 4), 1, 0, 0, None),
                                      ((40, 30, 8), 1, 3000, 2500, 11)):
        lc, lf = _rand_set(1 + cl, grid, nb, nl, cl, dtype)
        ic, if_ = _rand_set(2 + ci, grid, nb, ni, ci, dtype)
        print(f"fuse dtype={dtype} cl={cl} ci={ci} pad={pad} grid={grid} B={nb} nl={len(lc)} ni={len(ic)} shuffle={shuffle}", flush=True)
        oc, of, osl, osi = oracle.fuse(lc, lf, ic, if_, grid, nb, want_src=True)
        cap_out = len(oc) + 7
        for want_src in (True, False):
            co, fo, sl, si, n_out, nv, ord_l, ord_i = gpu_fuse(ctx, dtype, lc, lf, ic, if_, grid, nb, cap_out, cl + ci + pad,
                                                               want_src, slot=1, shuffle=shuffle)
            ctx.status_sync()
            assert nv == len(oc)
            assert np.array_equal(co[:nv].cpu().numpy(), oc)
            got = fo[:nv].float().cpu().numpy()
            assert np.array_equal(got[:, :cl + ci], of)                 # a copy: bit-exact
            assert not got[:, cl + ci:].any()                            # padding is zero
            assert float(fo[nv:].float().min().item()) == 9.0            # rows past the count are not written
            if want_src:
                gsl, gsi = sl[:nv].cpu().numpy(), si[:nv].cpu().numpy()
                assert np.array_equal(gsl >= 0, osl >= 0) and np.array_equal(gsi >= 0, osi >= 0)
                # the inputs went in permuted by ord_*: row s of the device array is row ord[s] of the sorted set
                assert np.array_equal(ord_l[gsl[gsl >= 0]], osl[osl >= 0]) and np.array_equal(ord_i[gsi[gsi >= 0]], osi[osi >= 0])
    ctx.close()


def test_fuse_capacity_and_bad_arguments():
    ctx = B.Context(16, 1000, 20 * 20 * 20, n_slots=1)
    grid = (20, 20, 20)
    lc, lf = _rand_set(1, grid, 1, 300, 4, F32)
    ic, if_ = _rand_set(2, grid, 1, 300, 4, F32)
    oc, of = oracle.fuse(lc, lf, ic, if_, grid, 1)
    cap = len(oc) - 50
    co, fo, sl, si, n_out, nv, _, _ = gpu_fuse(ctx, F32, lc, lf, ic, if_, grid, 1, cap, 8)
    assert nv == cap
    with pytest.raises(B.Emc2Error) as e:
        ctx.status_sync()
    assert e.value.status == B.ERR_CAPACITY
    assert np.array_equal(co.cpu().numpy(), oc[:cap]) and np.array_equal(fo.cpu().numpy(), of[:cap])
    ctx.status_sync()
    with pytest.raises(B.Emc2Error):                                     # output rows narrower than the two halves
        gpu_fuse(ctx, F32, lc, lf, ic, if_, grid, 1, len(oc), 7)
    with pytest.raises(B.Emc2Error):                                     # a half that is not a multiple of 4 bytes
        l3, f3 = _rand_set(1, grid, 1, 30, 3, F16)
        gpu_fuse(ctx, F16, l3, f3, l3, f3, grid, 1, 100, 6)
    # malformed coordinates are ignored, not written out of bounds
    bad = np.array([[0, 0, 0, 0], [0, 25, 0, 0], [3, 0, 0, 0], [0, 0, -1, 0]], np.int32)
    co, fo, sl, si, n_out, nv, _, _ = gpu_fuse(ctx, F32, bad, np.ones((4, 4), np.float32), ic[:0], if_[:0], grid, 1, 10, 8)
    assert nv == 1 and co[0].tolist() == [0, 0, 0, 0]
    ctx.close()


def test_pool_fuse_conv_chain():
    """The data bridge's multimodal leg end to end on a crop: voxelize the cloud, pool the image on the same grid, fuse
    (rows padded to 128 channels), build a submanifold map from the index the fusion left behind, convolve."""
    vs, grid = (0.4, 0.4, 0.4), (176, 200, 10)
    spec = VoxelSpec(LO, vs, grid)
    h, w, c = 90, 300, 64
    ctx = B.Context(max(h * w, 20000), 40000, 176 * 200 * 10, n_slots=3)
    pm, q, depth, img = make_scene(4, h=h, w=w, c=c)
    pts = gen.make_cloud("front", 20000, 4)
    cap = 40000
    # LiDAR side: mean features rounded to fp16, padded to 8 channels so that the half is 16 bytes
    coords = torch.zeros((cap, 4), dtype=torch.int32, device="cuda")
    means = torch.zeros((cap, 4), dtype=torch.float32, device="cuda")
    counts = torch.zeros((cap,), dtype=torch.int32, device="cuda")
    n_l = torch.zeros(1, dtype=torch.int32, device="cuda")
    lp = torch.zeros((cap, 4), dtype=torch.float16, device="cuda")
    nl = ctx.voxelize(dev(pts), None, spec, cap, coords, means, counts, n_l, feats_lp=lp, index_slot=0, sync_count=True)
    ic, if_, _, n_i, ni = gpu_pool(ctx, img, depth, q, spec, B.POOL_MAX, cap, slot=1)
    co = torch.zeros((cap, 4), dtype=torch.int32, device="cuda")
    fo = torch.zeros((cap, 128), dtype=torch.float16, device="cuda")
    n_f = torch.zeros(1, dtype=torch.int32, device="cuda")
    print(f"chain: {nl} voxels, {ni} image cells", flush=True)
    nf = ctx.fuse(F16, coords, lp, n_l, cap, ic, if_, n_i, cap, grid, 1, cap, co, fo, n_f, out_slot=2, sync_count=True)
    nbr = torch.full((27, cap), -5, dtype=torch.int32, device="cuda")
    n_o = torch.zeros(1, dtype=torch.int32, device="cuda")
    ctx.build_kmap(SUBM, co, n_f, cap, grid, 1, cap, nbr, n_o, in_slot=2)
    st = gen.Stream(12, 1)
    wgt = gen.round_to_dtype(st.normal(27 * 128 * 32, 0.05).astype(np.float32).reshape(27, 128, 32), F16)
    y = torch.zeros((cap, 32), dtype=torch.float16, device="cuda")
    ctx.spconv(F16, fo, dev(wgt, torch.float16), None, None, EPI_NONE, nbr, n_f, cap, y, map_hint=SUBM)
    ctx.status_sync()
    # oracle chain
    olc, olm, _ = oracle.voxelize(pts, None, LO, vs, grid)
    oic, oif, _ = oracle.pool_image(img, depth, q, LO, vs, grid, oracle.POOL_MAX)
    ofc, off = oracle.fuse(olc, gen.round_to_dtype(olm, F16), oic, oif, grid)
    assert (nl, ni, nf) == (len(olc), len(oic), len(ofc)) and nf > max(nl, ni)
    assert np.array_equal(co[:nf].cpu().numpy(), ofc)
    got = fo[:nf].float().cpu().numpy()
    assert not got[:, 68:].any()
    assert_features_close(got[:, :4], off[:, :4], 2e-3, "LiDAR half")          # fp32 means in no fixed order, then fp16
    assert np.array_equal(got[:, 4:68], off[:, 4:])
    _, onbr, _ = oracle.build_kmap(0, ofc, grid, 1)
    assert np.array_equal(nbr[:, :nf].cpu().numpy(), onbr)
    x = np.zeros((nf, 128), np.float32); x[:, :68] = got[:, :68]                # the conv is checked on the GPU's own input rows
    oy = oracle.spconv(x, wgt, None, None, EPI_NONE, onbr)
    assert_features_close(y[:nf].float().cpu().numpy(), oy, 2e-2, "conv over the fused set")
    ctx.close()


def test_bridge_and_dispatcher_replay_in_a_hip_graph():
    """Pooling, fusion and the dispatcher recorded into one HIP graph (serving loops replay them): every replay,
    with eager work and synchronisations in between and after the input buffers were refilled, gives the oracle's
    result for the inputs it saw.  None of the three calls may depend on a host round trip or on a memset node."""
    vs, grid = (0.4, 0.4, 0.4), (176, 200, 10)
    spec = VoxelSpec(LO, vs, grid)
    h, w, c = 60, 200, 64
    scenes = []
    for seed in (4, 9):
        pm, q, depth, img = make_scene(seed, h=h, w=w, c=c)
        lc, lf = _rand_set(seed, grid, 1, 3000, 32, F16)
        props, scene = gen.make_proposals(8, seed)
        scenes.append((q, depth, img, lc, lf, props, scene))
    q = scenes[0][0]
    # the second scene is lifted with the first scene's camera: only device buffers change between replays
    cap = h * w + 4000
    n_prop_cap = max(len(s[5]) for s in scenes)
    ctx = B.Context(h * w, cap, 176 * 200 * 10, n_slots=2)
    d_img = torch.zeros((h, w, c), dtype=torch.float16, device="cuda")
    d_depth = torch.zeros((h, w), dtype=torch.float32, device="cuda")
    d_lc = torch.zeros((4000, 4), dtype=torch.int32, device="cuda")
    d_lf = torch.zeros((4000, 32), dtype=torch.float16, device="cuda")
    n_l = torch.zeros(1, dtype=torch.int32, device="cuda")
    d_props = torch.zeros((n_prop_cap, 4), dtype=torch.float32, device="cuda")
    d_scene = torch.full((n_prop_cap,), -1, dtype=torch.int32, device="cuda")     # -1: ignored by the dispatcher
    ic = torch.zeros((cap, 4), dtype=torch.int32, device="cuda")
    if_ = torch.zeros((cap, c), dtype=torch.float16, device="cuda")
    icnt = torch.zeros((cap,), dtype=torch.int32, device="cuda")
    n_i = torch.zeros(1, dtype=torch.int32, device="cuda")
    fc = torch.zeros((cap, 4), dtype=torch.int32, device="cuda")
    ff = torch.zeros((cap, 96), dtype=torch.float16, device="cuda")
    n_f = torch.zeros(1, dtype=torch.int32, device="cuda")
    expert = torch.zeros(8, dtype=torch.int32, device="cuda")
    counts = torch.zeros(3, dtype=torch.int32, device="cuda")
    order = torch.zeros(8, dtype=torch.int32, device="cuda")

    def fill(s):
        _, depth, img, lc, lf, props, scene = s
        d_img.copy_(dev(img)); d_depth.copy_(dev(depth))
        d_lc.zero_(); d_lc[:len(lc)] = dev(lc); d_lf.zero_(); d_lf[:len(lc)] = dev(lf, torch.float16)
        n_l.fill_(len(lc))
        d_props.zero_(); d_props[:len(props)] = dev(props)
        d_scene.fill_(-1); d_scene[:len(props)] = dev(scene)

    def calls():
        ctx.pool_image(d_img, d_depth, q, spec, B.POOL_MAX, cap, ic, if_, icnt, n_i, index_slot=0)
        ctx.fuse(F16, d_lc, d_lf, n_l, 4000, ic, if_, n_i, cap, grid, 1, cap, fc, ff, n_f, out_slot=1)
        ctx.dispatch(d_props, d_scene, 8, 23.5, 0.5, expert, counts, order)

    def expected(s):
        _, depth, img, lc, lf, props, scene = s
        oic, oif, _ = oracle.pool_image(img, depth, q, LO, vs, grid, oracle.POOL_MAX)
        ofc, off = oracle.fuse(lc, lf, oic, oif, grid)
        return ofc, off, oracle.dispatch(props, scene, 8, 23.5, 0.5)

    def check(s, what):
        torch.cuda.synchronize()
        ctx.status_sync()
        ofc, off, (oe, ocn, oo) = expected(s)
        nf = int(n_f.item())
        assert nf == len(ofc), what
        assert np.array_equal(fc[:nf].cpu().numpy(), ofc), what
        assert np.array_equal(ff[:nf].float().cpu().numpy(), off), what
        assert np.array_equal(expert.cpu().numpy(), oe) and np.array_equal(counts.cpu().numpy(), ocn), what
        assert np.array_equal(order.cpu().numpy(), oo), what

    fill(scenes[0])
    calls()
    check(scenes[0], "eager")
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        calls()                                   # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            calls()
    torch.cuda.synchronize()
    for it in range(5):
        s = scenes[it % 2]
        print(f"bridge graph replay {it}", flush=True)
        fill(s)
        torch.cuda.synchronize()
        graph.replay()
        check(s, f"replay {it}")
        if it == 2:
            calls()                               # eager work between replays
            check(s, "eager between replays")
    ctx.close()
