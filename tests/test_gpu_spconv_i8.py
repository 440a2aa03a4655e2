"""GPU parity of the quantised sparse convolution (through the C-ABI) against the CPU oracle.  Integer
accumulation is exact and the epilogue a fixed sequence of individually rounded fp32 operations, so every output
(int8 and fp16) must match bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2507_04123_amd import binding as B
from paper_2507_04123_amd import gen
from paper_2507_04123_amd.configs import get_config, SUBM, STRIDED

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _threads():
    oracle.set_threads(min(16, oracle.max_threads()))
    yield


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _rand_i8(seed, shape, lim=127):
    b = gen.Stream(seed, 21).bits(int(np.prod(shape)))
    return ((b % np.uint64(2 * lim + 1)).astype(np.int64) - lim).astype(np.int8).reshape(shape)


def _rand_sites(seed, grid, nb, n):
    gx, gy, gz = grid
    total = gx * gy * gz * nb
    keys = np.unique((gen.Stream(seed, 3).bits(3 * n) % np.uint64(total)).astype(np.int64))[:n]
    keys.sort()
    x = keys % gx; y = (keys // gx) % gy; z = (keys // (gx * gy)) % gz; b = keys // (gx * gy * gz)
    return np.stack([b, z, y, x], axis=1).astype(np.int32)


def check_conv(ctx, xq, wq, mul, add, relu, nbr_np, cap, inv_s):
    n_out = nbr_np.shape[1]
    cin, cout = wq.shape[1], wq.shape[2]
    nbr = torch.full((27, cap), -1, dtype=torch.int32, device="cuda")
    nbr[:, :n_out] = dev(nbr_np)
    n_t = torch.tensor([n_out], dtype=torch.int32, device="cuda")
    wp = torch.empty((27 * cin * cout,), dtype=torch.int8, device="cuda")
    ctx.pack_weights_i8(dev(wq), wp)
    ov, oq = oracle.spconv_i8(xq, wq, mul, add, relu, nbr_np, inv_out_scale=inv_s)
    d_x = dev(xq) if len(xq) else torch.zeros((1, cin), dtype=torch.int8, device="cuda")
    for out_dtype in (torch.int8, torch.float16):
        out = torch.full((cap, cout), 55, dtype=out_dtype, device="cuda")
        print(f"spconv_i8 {cin}->{cout} n_out={n_out} cap={cap} relu={relu} out={out_dtype}", flush=True)
        ctx.spconv_i8(d_x, wp, cin, cout, dev(mul), dev(add), relu, nbr, n_t, cap, out, inv_out_scale=inv_s)
        torch.cuda.synchronize()
        got = out[:n_out].cpu().numpy()
        if out_dtype == torch.int8:
            assert np.array_equal(got, oq)
        else:
            with np.errstate(over="ignore"):
                assert np.array_equal(got, ov.astype(np.float16))
        if n_out < cap:
            assert int((out[n_out:] != 55).sum().item()) == 0           # rows past the count are not written
    return ov, oq


@pytest.mark.parametrize("cin,cout", [(64, 64), (64, 32), (128, 64), (128, 32)])
def test_spconv_i8_random_maps_bit_exact(cin, cout):
    ctx = B.Context(16, 4096, 64 * 64 * 8, n_slots=1)
    assert ctx.spconv_i8_supported(cin, cout)
    st = gen.Stream(cin + cout, 9)
    for seed, grid, nb, n, relu in ((1, (24, 20, 6), 2, 2500, True), (2, (9, 8, 5), 1, 300, False), (3, (40, 3, 1), 1, 70, True),
                                    (4, (5, 5, 5), 1, 1, False)):
        coords = _rand_sites(seed, grid, nb, n)
        xq = _rand_i8(seed + 10, (len(coords), cin))
        wq = _rand_i8(seed + 20, (27, cin, cout), 60)
        mul = (st.uniform(cout, 0.5, 1.5) * 2e-5).astype(np.float32)
        add = st.uniform(cout, -2.0, 2.0).astype(np.float32)
        for kind in (0, 1):
            out_c, nbr_np, _ = oracle.build_kmap(kind, coords, grid, nb)
            ov, oq = check_conv(ctx, xq, wq, mul, add, relu, nbr_np, nbr_np.shape[1] + 37, np.float32(1.0 / 0.04))
            if len(coords) > 100:
                assert (np.abs(oq) == 127).any() and (oq == 0).any()    # saturation and the zero bin are both exercised
    # an arbitrary (non-geometric) table, and an empty output set
    xq = _rand_i8(7, (500, cin)); wq = _rand_i8(8, (27, cin, cout))
    tb = (gen.Stream(5, 5).bits(27 * 333) % np.uint64(700)).astype(np.int64).reshape(27, 333) - 200
    tb = np.where((tb >= 0) & (tb < 500), tb, -1).astype(np.int32)
    check_conv(ctx, xq, wq, np.full(cout, 1e-5, np.float32), np.zeros(cout, np.float32), False, tb, 400, np.float32(8.0))
    check_conv(ctx, xq, wq, np.ones(cout, np.float32), np.zeros(cout, np.float32), False, np.zeros((27, 0), np.int32), 64, np.float32(1.0))
    ctx.close()


def test_quantize_i8_bit_exact():
    ctx = B.Context(16, 16, 64, n_slots=1)
    x = gen.Stream(3, 3).normal(100003, 2.0).astype(np.float32)
    x[:16] = [0.0, 0.49, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5, 127.4, 127.5, 1e9, -1e9, np.inf, -np.inf, np.nan]
    for inv in (1.0, 1.0 / 0.037, 4.0):
        for dt in (np.float32, np.float16):
            with np.errstate(over="ignore"):
                xs = x.astype(dt)
            q = torch.full((len(x) + 5,), 99, dtype=torch.int8, device="cuda")
            ctx.quantize_i8(dev(xs), float(np.float32(inv)), q)
            torch.cuda.synchronize()
            assert np.array_equal(q[:len(x)].cpu().numpy(), oracle.quantize_i8(xs.astype(np.float32), np.float32(inv)))
            assert q[len(x):].tolist() == [99] * 5
    ctx.close()


def test_spconv_i8_config2_level2_full_size():
    """The heaviest layer shape of config 2 (submanifold 64 -> 64 on the level-2 voxel set, 222 k sites) and the
    stride-2 64 -> 64 layer after it, at full size, every output compared."""
    cfg = get_config(2)
    br = cfg.branches[0]
    sp = br.spec
    pts, _ = gen.make_frames(cfg)
    coords, _, _ = oracle.voxelize(pts, None, sp.lo, sp.vs, sp.grid)
    grid = tuple(sp.grid)
    for _ in range(2):
        coords, _, grid = oracle.build_kmap(1, coords, grid, 1)
    _, sub, _ = oracle.build_kmap(0, coords, grid, 1)
    c3, down, _ = oracle.build_kmap(1, coords, grid, 1)
    n = len(coords)
    assert n > 200000
    ctx = B.Context(16, n + 100, 64, n_slots=1)
    xq = _rand_i8(1, (n, 64)); wq = _rand_i8(2, (27, 64, 64), 50)
    st = gen.Stream(4, 4)
    mul = (st.uniform(64, 0.5, 1.5) * 1e-5).astype(np.float32)
    add = st.uniform(64, -1.0, 1.0).astype(np.float32)
    check_conv(ctx, xq, wq, mul, add, True, sub, n + 100, np.float32(1.0 / 0.03))
    check_conv(ctx, xq, wq, mul, add, True, down, len(c3) + 11, np.float32(1.0 / 0.03))
    ctx.close()


def test_spconv_i8_rejects_unsupported():
    ctx = B.Context(16, 64, 64, n_slots=1)
    assert not ctx.spconv_i8_supported(32, 64) and not ctx.spconv_i8_supported(64, 16)
    z = torch.zeros(1, dtype=torch.int32, device="cuda")
    nbr = torch.full((27, 64), -1, dtype=torch.int32, device="cuda")
    with pytest.raises(B.Emc2Error):
        ctx.spconv_i8(torch.zeros((4, 32), dtype=torch.int8, device="cuda"), torch.zeros(27 * 32 * 64, dtype=torch.int8, device="cuda"),
                      32, 64, torch.ones(64, device="cuda"), torch.zeros(64, device="cuda"), False, nbr, z, 64,
                      torch.zeros((64, 64), dtype=torch.int8, device="cuda"))
    with pytest.raises(B.Emc2Error):
        ctx.pack_weights_i8(torch.zeros((27, 48, 64), dtype=torch.int8, device="cuda"), torch.zeros(27 * 48 * 64, dtype=torch.int8, device="cuda"))
    ctx.close()


def test_spconv_i8_entries_beyond_the_input_are_refused():
    """As for the 16-bit conv: an entry at or beyond n_in_rows reads nothing and is reported through the status word."""
    ctx = B.Context(16, 4096, 64 * 64 * 8, n_slots=1)
    cin, cout, n_in, n_out, slack = 64, 64, 200, 333, 30
    st = gen.Stream(515, 2)
    xq = (st.bits((n_in + slack) * cin) % np.uint64(255)).astype(np.int64).astype(np.int32) - 127
    xq = xq.astype(np.int8).reshape(-1, cin)
    wq = ((st.bits(27 * cin * cout) % np.uint64(121)).astype(np.int32) - 60).astype(np.int8).reshape(27, cin, cout)
    mul = st.uniform(cout, 1e-5, 3e-5).astype(np.float32)
    add = st.uniform(cout, -0.1, 0.1).astype(np.float32)
    bad = (st.bits(27 * n_out) % np.uint64(n_in + slack)).astype(np.int32).reshape(27, n_out)
    bad[st.uniform(27 * n_out, 0.0, 1.0).reshape(27, n_out) < 0.5] = -1
    bad[5, 64] = n_in
    cleaned = np.where(bad >= n_in, -1, bad).astype(np.int32)
    ov, oq = oracle.spconv_i8(xq[:n_in], wq, mul, add, True, cleaned, inv_out_scale=25.0)
    wp = torch.empty((27 * cin * cout,), dtype=torch.int8, device="cuda")
    ctx.pack_weights_i8(dev(wq), wp)
    out = torch.zeros((n_out, cout), dtype=torch.int8, device="cuda")
    n_t = torch.tensor([n_out], dtype=torch.int32, device="cuda")
    print("spconv_i8 refused entries", flush=True)
    ctx.spconv_i8(dev(xq), wp, cin, cout, dev(mul), dev(add), True, dev(bad), n_t, n_out, out, inv_out_scale=25.0, n_in_rows=n_in)
    with pytest.raises(B.Emc2Error) as ei:
        ctx.status_sync()
    assert ei.value.status == B.ERR_MAP
    assert np.array_equal(out.cpu().numpy(), oq)
    ctx.spconv_i8(dev(xq), wp, cin, cout, dev(mul), dev(add), True, dev(cleaned), n_t, n_out, out, inv_out_scale=25.0, n_in_rows=n_in)
    ctx.status_sync()
    ctx.close()
