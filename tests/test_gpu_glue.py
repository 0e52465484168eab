"""GPU parity of the U-Net glue entry points (max-pool, transposed convolution, 1x1x1 convolution,
concat / split) against the numpy fp64 oracle on the unpartitioned volume."""
import numpy as np
import pytest
import torch

from oracle import unet_ops as U
from paper_1909_03108_amd import sp3d, synth
from gpu_util import DT, TOL, bits, f64, guard_alloc, guards_intact, rel_err, to_dev, widen

pytestmark = pytest.mark.gpu


def padded(g, V, c, dt):
    """host volume (storage array) -> padded tiles on the device (margins zero)"""
    P = sp3d.alloc_padded(g, c, dt)
    sp3d.sp_partition(to_dev(V), P, g, c, dt)
    return P


def volume(g, P, c, dt):
    V = torch.empty((g.n, g.d, g.h, g.w, c), dtype=P.dtype, device="cuda")
    sp3d.sp_unpartition(P, V, g, c, dt)
    return V


def draw(dtype, shape, seed):
    return synth.normal_volume(shape, seed, dtype)


CASES = [  # n, fine dhw, grid, dtype
    (1, (8, 8, 16), (4, 4, 1), "bf16"),      # coarse tiles 1x1x8
    (2, (4, 12, 8), (2, 3, 2), "f32"),
    (1, (16, 8, 64), (2, 2, 1), "bf16"),
    (1, (4, 8, 80), (1, 2, 1), "bf16"),      # coarse rows of 40 voxels: one whole and one ragged 32-voxel segment
]


@pytest.mark.parametrize("n,dhw,grid,dtype", CASES)
@pytest.mark.parametrize("c", [3, 32])
def test_maxpool_forward_and_backward_bit_exact(n, dhw, grid, dtype, c):
    gf = sp3d.Geom(n, dhw, grid)
    gc = sp3d.coarse_geom(gf)
    dt = DT[dtype]
    x = draw(dtype, (n,) + dhw + (c,), 1)
    # plant ties: ReLU-like zeros are the common case after an activation
    xv = widen(x)
    x = np.where(xv < 0, np.zeros_like(x), x)
    dy = draw(dtype, (n, dhw[0] // 2, dhw[1] // 2, dhw[2] // 2, c), 2)
    Px = padded(gf, x, c, dt)
    Py = torch.full(gc.padded_shape + (c,), 9.0, dtype=Px.dtype, device="cuda")
    sp3d.sp_maxpool2_fwd(Px, Py, gf, c, dt)
    assert np.array_equal(f64(volume(gc, Py, c, dt)), U.maxpool2_fwd(widen(x)))
    got = f64(Py)
    mask = np.ones(got.shape, dtype=bool)
    mask[(slice(None),) * 4 + (slice(1, -1),) * 3] = False
    assert np.all(got[mask] == 9.0)                       # margins untouched
    Pdx = sp3d.alloc_padded(gf, c, dt)
    Pdy = padded(gc, dy, c, dt)
    sp3d.sp_maxpool2_bwd(Px, Pdy, Pdx, gf, c, dt)
    assert np.array_equal(f64(volume(gf, Pdx, c, dt)), U.maxpool2_bwd(widen(x), widen(dy)))
    # the encoder level's whole backward join, [x > 0] * (pool backward + skip gradient): the oracle's three
    # steps composed (exact selects and one rounded sum), and bit for bit the three separate calls; in place too
    skip = draw(dtype, (n,) + dhw + (c,), 3)
    Ps = padded(gf, skip, c, dt)
    Pj = torch.full(gf.padded_shape + (c,), 9.0, dtype=Px.dtype, device="cuda")
    sp3d.sp_maxpool2_bwd_join(Px, Pdy, Ps, Pj, gf, c, dt)
    ref = np.where(widen(x) > 0, U.maxpool2_bwd(widen(x), widen(dy)) + widen(skip), 0.0)
    assert rel_err(f64(volume(gf, Pj, c, dt)), ref) <= (2.0 ** -8 if dtype == "bf16" else 1e-6)
    got = f64(Pj)
    maskf = np.ones(got.shape, dtype=bool)
    maskf[(slice(None),) * 4 + (slice(1, -1),) * 3] = False
    assert np.all(got[maskf] == 9.0)                      # margins untouched
    sp3d.sp_add(Pdx, Ps, Pdx, gf, c, dt)
    sp3d.sp_relu_bwd(Pdx, Px, Pdx, gf, c, dt)
    assert torch.equal(volume(gf, Pdx, c, dt), volume(gf, Pj, c, dt))
    sp3d.sp_maxpool2_bwd_join(Px, Pdy, Ps, Ps, gf, c, dt)
    assert torch.equal(volume(gf, Ps, c, dt), volume(gf, Pj, c, dt))


@pytest.mark.parametrize("n,dhw,grid,dtype", CASES)
@pytest.mark.parametrize("cin,cout", [(8, 4), (64, 32), (5, 3), (128, 64), (32, 96), (256, 128), (288, 320), (512, 64)])
def test_upconv_fwd_dgrad_wgrad(n, dhw, grid, dtype, cin, cout):
    gf = sp3d.Geom(n, dhw, grid)
    gc = sp3d.coarse_geom(gf)
    dt, tol = DT[dtype], TOL[dtype]
    cshape = (n, dhw[0] // 2, dhw[1] // 2, dhw[2] // 2)
    x = draw(dtype, cshape + (cin,), 3)
    dy = draw(dtype, (n,) + dhw + (cout,), 4)
    u = synth.weights(cin, cout, 5, dtype, taps=(2, 2, 2))
    bias = np.linspace(-1, 1, cout).astype(np.float32)
    Px, Pdy = padded(gc, x, cin, dt), padded(gf, dy, cout, dt)
    Py = sp3d.alloc_padded(gf, cout, dt)
    sp3d.sp_upconv2_fwd(Px, to_dev(u), torch.from_numpy(bias).cuda(), Py, gf, cin, cout, dt)
    assert rel_err(f64(volume(gf, Py, cout, dt)), U.upconv2_fwd(widen(x), widen(u), bias)) <= tol
    Pdx = sp3d.alloc_padded(gc, cin, dt)
    sp3d.sp_upconv2_dgrad(Pdy, to_dev(u), Pdx, gf, cin, cout, dt)
    assert rel_err(f64(volume(gc, Pdx, cin, dt)), U.upconv2_dgrad(widen(dy), widen(u))) <= tol
    du = torch.full((2, 2, 2, cin, cout), 7.0, dtype=torch.float32, device="cuda")
    db = torch.full((cout,), 7.0, dtype=torch.float32, device="cuda")
    ws = sp3d.alloc_ws(sp3d.sp_workspace_bytes(sp3d.SP_OP_UPCONV_WGRAD, gf, cin, cout, dt))
    sp3d.sp_upconv2_wgrad(Px, Pdy, du, db, gf, cin, cout, dt, ws)
    ref_du, ref_db = U.upconv2_wgrad(widen(x), widen(dy))
    assert rel_err(f64(du), ref_du) <= tol and rel_err(f64(db), ref_db) <= tol
    du2 = torch.empty_like(du)
    sp3d.sp_upconv2_wgrad(Px, Pdy, du2, None, gf, cin, cout, dt, ws)
    assert torch.equal(du, du2)


@pytest.mark.parametrize("n,dhw,grid,dtype", CASES)
@pytest.mark.parametrize("cin,cout", [(32, 3), (7, 5), (64, 4), (8, 1), (256, 2)])
def test_pointwise_fwd_dgrad_wgrad(n, dhw, grid, dtype, cin, cout):
    g = sp3d.Geom(n, dhw, grid)
    dt, tol = DT[dtype], TOL[dtype]
    x = draw(dtype, (n,) + dhw + (cin,), 6)
    dy = draw(dtype, (n,) + dhw + (cout,), 7)
    p = synth.weights(cin, cout, 8, dtype, taps=(1, 1, 1))
    pw = widen(p).reshape(cin, cout)
    bias = np.linspace(-1, 1, cout).astype(np.float32)
    Px, Pdy = padded(g, x, cin, dt), padded(g, dy, cout, dt)
    Py = sp3d.alloc_padded(g, cout, dt)
    sp3d.sp_pointwise_fwd(Px, to_dev(p), torch.from_numpy(bias).cuda(), Py, g, cin, cout, dt)
    assert rel_err(f64(volume(g, Py, cout, dt)), U.pointwise_fwd(widen(x), pw, bias)) <= tol
    Pdx = sp3d.alloc_padded(g, cin, dt)
    sp3d.sp_pointwise_dgrad(Pdy, to_dev(p), Pdx, g, cin, cout, dt)
    assert rel_err(f64(volume(g, Pdx, cin, dt)), U.pointwise_dgrad(widen(dy), pw)) <= tol
    # with the ReLU mask of the layer input (x clipped at zero stands for a ReLU output)
    xr = np.where(widen(x) > 0, x, np.zeros_like(x))
    Pm, Pdm = padded(g, xr, cin, dt), sp3d.alloc_padded(g, cin, dt)
    sp3d.sp_pointwise_dgrad_relu(Pdy, to_dev(p), Pm, Pdm, g, cin, cout, dt)
    assert rel_err(f64(volume(g, Pdm, cin, dt)), np.where(widen(xr) > 0, U.pointwise_dgrad(widen(dy), pw), 0.0)) <= tol
    sp3d.sp_relu_bwd(Pdx, Pm, Pdx, g, cin, dt)
    assert torch.equal(volume(g, Pdx, cin, dt), volume(g, Pdm, cin, dt))
    dp = torch.empty((cin, cout), dtype=torch.float32, device="cuda")
    db = torch.empty((cout,), dtype=torch.float32, device="cuda")
    ws = sp3d.alloc_ws(sp3d.sp_workspace_bytes(sp3d.SP_OP_POINTWISE_WGRAD, g, cin, cout, dt))
    sp3d.sp_pointwise_wgrad(Px, Pdy, dp, db, g, cin, cout, dt, ws)
    ref_dp, ref_db = U.pointwise_wgrad(widen(x), widen(dy))
    assert rel_err(f64(dp), ref_dp) <= tol and rel_err(f64(db), ref_db) <= tol
    # the whole backward pass in one sweep over the (ReLU) input: the oracle's values, and bit for bit what the two
    # separate calls give on the same input
    guard, Pone = guard_alloc(g.padded_shape + (cin,), Pm.dtype, 5.0)
    dp1, db1 = torch.full_like(dp, 9.0), torch.full_like(db, 9.0)
    sp3d.sp_pointwise_bwd_relu(Pm, Pdy, to_dev(p), Pone, dp1, db1, g, cin, cout, dt, ws)
    assert guards_intact(guard, 5.0)
    assert torch.equal(volume(g, Pone, cin, dt), volume(g, Pdm, cin, dt))
    ref_dp, ref_db = U.pointwise_wgrad(widen(xr), widen(dy))
    assert rel_err(f64(dp1), ref_dp) <= tol and rel_err(f64(db1), ref_db) <= tol
    dp2, db2 = torch.empty_like(dp), torch.empty_like(db)
    sp3d.sp_pointwise_wgrad(Pm, Pdy, dp2, db2, g, cin, cout, dt, ws)
    assert torch.equal(dp1, dp2) and torch.equal(db1, db2)
    dp3 = torch.full_like(dp, 9.0)
    sp3d.sp_pointwise_bwd_relu(Pm, Pdy, to_dev(p), Pone, dp3, None, g, cin, cout, dt, ws)      # no bias gradient
    assert torch.equal(dp3, dp2)
    with pytest.raises(sp3d.Sp3dError) as e:
        sp3d.sp_pointwise_bwd_relu(Pm, Pdy, to_dev(p), Pm, dp3, None, g, cin, cout, dt, ws)   # output on its input
    assert e.value.code == sp3d.SP_EINVAL


def test_pointwise_wgrad_many_partials():
    """Head-sized 1x1x1 weight gradient on a volume large enough for hundreds of per-block partial sums
    (the second-stage reduction then takes its wide, tree-shaped path); run twice: same bits."""
    n, dhw, grid, cin, cout = 1, (96, 128, 192), (2, 4, 1), 32, 3
    g = sp3d.Geom(n, dhw, grid)
    dt, tol = DT["bf16"], TOL["bf16"]
    x = draw("bf16", (n,) + dhw + (cin,), 16)
    dy = draw("bf16", (n,) + dhw + (cout,), 17)
    Px, Pdy = padded(g, x, cin, dt), padded(g, dy, cout, dt)
    ws = sp3d.alloc_ws(sp3d.sp_workspace_bytes(sp3d.SP_OP_POINTWISE_WGRAD, g, cin, cout, dt))
    assert ws.numel() >= 512 * (cin * cout + cout) * 4
    out = []
    for _ in range(2):
        dp = torch.empty((cin, cout), dtype=torch.float32, device="cuda")
        db = torch.empty((cout,), dtype=torch.float32, device="cuda")
        sp3d.sp_pointwise_wgrad(Px, Pdy, dp, db, g, cin, cout, dt, ws)
        out.append((dp, db))
    ref_dp, ref_db = U.pointwise_wgrad(widen(x), widen(dy))
    assert rel_err(f64(out[0][0]), ref_dp) <= tol and rel_err(f64(out[0][1]), ref_db) <= tol
    assert torch.equal(out[0][0], out[1][0]) and torch.equal(out[0][1], out[1][1])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_concat_and_split_bit_exact(dtype):
    g = sp3d.Geom(1, (4, 6, 8), (2, 3, 1))
    dt = DT[dtype]
    tdt = sp3d.torch_dtype(dt)
    a = torch.randn(g.padded_shape + (5,), device="cuda").to(tdt)
    b = torch.randn(g.padded_shape + (3,), device="cuda").to(tdt)
    c = torch.empty(g.padded_shape + (8,), dtype=tdt, device="cuda")
    sp3d.sp_concat(a, 5, b, 3, c, g, dt)
    assert torch.equal(c, torch.cat([a, b], dim=-1))
    a2, b2 = torch.empty_like(a), torch.empty_like(b)
    sp3d.sp_split(c, a2, 5, b2, 3, g, dt)
    assert torch.equal(a2, a) and torch.equal(b2, b)


def test_odd_tile_extent_is_rejected():
    g = sp3d.Geom(1, (6, 8, 8), (2, 2, 2))           # tile depth 3
    x = torch.zeros(g.padded_shape + (4,), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sp3d.Sp3dError) as e:
        sp3d.sp_maxpool2_fwd(x, x, g, 4, sp3d.SP_BF16)
    assert e.value.code == sp3d.SP_EGEOM


# ---- the glue of the configuration-5 stack at its real shapes (grid 4x4x1, fine volumes 256^3 / 128^3 / 64^3) ------

C5_LEVELS = [(256, 32), (128, 64), (64, 128)]       # fine cube edge, channels of the level that is pooled


def _relu_bits(a):
    return np.where(widen(a) > 0, a, np.zeros_like(a))


@pytest.mark.timeout(900)
@pytest.mark.parametrize("edge,c", C5_LEVELS)
def test_configuration_5_pools_real_size(edge, c):
    """The three poolings of the configuration-5 stack at their real shapes: forward, backward and the encoder's
    backward join, every element against the oracle.  The pooled tensor is a ReLU output (half zeros: windows
    with ties are common).  Pooling is window-local, so the oracle is evaluated slab by slab along D to bound
    host memory; selects are compared bit for bit, the join's single rounded sum to half a bf16 ulp."""
    n, dhw, grid, dtype = 1, (edge,) * 3, (4, 4, 1), "bf16"
    gf = sp3d.Geom(n, dhw, grid)
    gc = sp3d.coarse_geom(gf)
    dt = DT[dtype]
    x = _relu_bits(draw(dtype, (n,) + dhw + (c,), 31))
    dy = draw(dtype, (n,) + (edge // 2,) * 3 + (c,), 32)
    skip = draw(dtype, (n,) + dhw + (c,), 33)
    Px, Pdy, Ps = padded(gf, x, c, dt), padded(gc, dy, c, dt), padded(gf, skip, c, dt)
    Py, Pdx, Pj = sp3d.alloc_padded(gc, c, dt), sp3d.alloc_padded(gf, c, dt), sp3d.alloc_padded(gf, c, dt)
    sp3d.sp_maxpool2_fwd(Px, Py, gf, c, dt)
    sp3d.sp_maxpool2_bwd(Px, Pdy, Pdx, gf, c, dt)
    sp3d.sp_maxpool2_bwd_join(Px, Pdy, Ps, Pj, gf, c, dt)
    y, dx, dj = (volume(g_, P, c, dt) for g_, P in ((gc, Py), (gf, Pdx), (gf, Pj)))
    step = 32
    for d0 in range(0, edge, step):
        xs, ds = widen(x[:, d0:d0 + step]), widen(dy[:, d0 // 2:(d0 + step) // 2])
        assert np.array_equal(f64(y[:, d0 // 2:(d0 + step) // 2]), U.maxpool2_fwd(xs)), ("fwd", d0)
        ref = U.maxpool2_bwd(xs, ds)
        assert np.array_equal(f64(dx[:, d0:d0 + step]), ref), ("bwd", d0)
        ref = np.where(xs > 0, ref + widen(skip[:, d0:d0 + step]), 0.0)
        assert rel_err(f64(dj[:, d0:d0 + step]), ref) <= 2.0 ** -8, ("join", d0)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("edge,cin,cout", [(64, 256, 128), (128, 128, 64), (256, 64, 32)])
def test_configuration_5_upconvs_real_size(edge, cin, cout):
    """The three transposed convolutions of the configuration-5 stack at their real shapes (edge = the fine
    side).  The operation is local to a coarse voxel, so forward and data gradient are compared on whole coarse
    D planes (all of H and W: every tile and every segment of a row) -- every plane for the smallest level, the
    first / last planes of every tile and seeded others for the larger ones; the weight gradient, a reduction
    over all voxels, in full for the smallest level and on a seeded 16 x 16 block of (ci, co) pairs for every tap
    otherwise (the definition is independent per pair); the bias gradient in full."""
    n, dhw, grid, dtype = 1, (edge,) * 3, (4, 4, 1), "bf16"
    gf = sp3d.Geom(n, dhw, grid)
    gc = sp3d.coarse_geom(gf)
    dt, tol = DT[dtype], TOL[dtype]
    ce = edge // 2
    x = _relu_bits(draw(dtype, (n,) + (ce,) * 3 + (cin,), 41))
    dy = draw(dtype, (n,) + dhw + (cout,), 42)
    u = synth.weights(cin, cout, 43, dtype, taps=(2, 2, 2))
    bias = (0.1 * np.sin(np.arange(cout))).astype(np.float32)
    ud = widen(u)
    Px, Pdy = padded(gc, x, cin, dt), padded(gf, dy, cout, dt)
    Py, Pdx = sp3d.alloc_padded(gf, cout, dt), sp3d.alloc_padded(gc, cin, dt)
    sp3d.sp_upconv2_fwd(Px, to_dev(u), torch.from_numpy(bias).cuda(), Py, gf, cin, cout, dt)
    sp3d.sp_upconv2_dgrad(Pdy, to_dev(u), Pdx, gf, cin, cout, dt)
    y, dx = volume(gf, Py, cout, dt), volume(gc, Pdx, cin, dt)
    rng = np.random.default_rng(edge)
    td = ce // 4
    if ce <= 32:
        planes = list(range(ce))
    else:
        planes = sorted(set([a * td for a in range(4)] + [a * td + td - 1 for a in range(4)] +
                            [int(v) for v in rng.integers(0, ce, 6)]))
    for d in planes:
        ref = U.upconv2_fwd(widen(x[:, d:d + 1]), ud, bias)
        assert rel_err(f64(y[:, 2 * d:2 * d + 2]), ref) <= tol, ("fwd", d)
        ref = U.upconv2_dgrad(widen(dy[:, 2 * d:2 * d + 2]), ud)
        assert rel_err(f64(dx[:, d:d + 1]), ref) <= tol, ("dgrad", d)
    du = torch.full((2, 2, 2, cin, cout), 7.0, dtype=torch.float32, device="cuda")
    db = torch.full((cout,), 7.0, dtype=torch.float32, device="cuda")
    ws = sp3d.alloc_ws(sp3d.sp_workspace_bytes(sp3d.SP_OP_UPCONV_WGRAD, gf, cin, cout, dt))
    sp3d.sp_upconv2_wgrad(Px, Pdy, du, db, gf, cin, cout, dt, ws)
    if ce <= 32:
        ref_du, ref_db = U.upconv2_wgrad(widen(x), widen(dy))
        assert rel_err(f64(du), ref_du) <= tol
    else:
        ci = np.sort(rng.choice(cin, 16, replace=False))
        co = np.sort(rng.choice(cout, 16, replace=False))
        ref_du, _ = U.upconv2_wgrad(widen(x[..., ci]), widen(dy[..., co]))
        assert rel_err(f64(du)[:, :, :, ci][..., co], ref_du) <= tol
        ref_db = widen(dy).reshape(-1, cout).sum(axis=0)
    assert rel_err(f64(db), ref_db) <= tol


@pytest.mark.timeout(900)
def test_configuration_5_head_real_size():
    """The 1x1x1 classifier 32 -> 3 on 256^3, grid 4x4x1: forward with bias, data gradient, data gradient with
    the ReLU mask of its input, weight and bias gradient -- every element, the oracle evaluated slab by slab
    along D (the operation is voxel-local; the weight gradient is a sum over voxels, added slab by slab)."""
    n, dhw, grid, dtype, cin, cout = 1, (256,) * 3, (4, 4, 1), "bf16", 32, 3
    g = sp3d.Geom(n, dhw, grid)
    dt, tol = DT[dtype], TOL[dtype]
    x = _relu_bits(draw(dtype, (n,) + dhw + (cin,), 51))
    dy = draw(dtype, (n,) + dhw + (cout,), 52)
    p = synth.weights(cin, cout, 53, dtype, taps=(1, 1, 1))
    pw = widen(p).reshape(cin, cout)
    bias = np.array([0.3, -0.2, 0.1], dtype=np.float32)
    Px, Pdy = padded(g, x, cin, dt), padded(g, dy, cout, dt)
    Py, Pdx, Pdm = sp3d.alloc_padded(g, cout, dt), sp3d.alloc_padded(g, cin, dt), sp3d.alloc_padded(g, cin, dt)
    sp3d.sp_pointwise_fwd(Px, to_dev(p), torch.from_numpy(bias).cuda(), Py, g, cin, cout, dt)
    sp3d.sp_pointwise_dgrad(Pdy, to_dev(p), Pdx, g, cin, cout, dt)
    sp3d.sp_pointwise_dgrad_relu(Pdy, to_dev(p), Px, Pdm, g, cin, cout, dt)
    dp = torch.empty((cin, cout), dtype=torch.float32, device="cuda")
    db = torch.empty((cout,), dtype=torch.float32, device="cuda")
    ws = sp3d.alloc_ws(sp3d.sp_workspace_bytes(sp3d.SP_OP_POINTWISE_WGRAD, g, cin, cout, dt))
    sp3d.sp_pointwise_wgrad(Px, Pdy, dp, db, g, cin, cout, dt, ws)
    y, dx, dm = volume(g, Py, cout, dt), volume(g, Pdx, cin, dt), volume(g, Pdm, cin, dt)
    ref_dp, ref_db = np.zeros((cin, cout)), np.zeros(cout)
    step = 32
    for d0 in range(0, 256, step):
        xs, ds = widen(x[:, d0:d0 + step]), widen(dy[:, d0:d0 + step])
        assert rel_err(f64(y[:, d0:d0 + step]), U.pointwise_fwd(xs, pw, bias)) <= tol, ("fwd", d0)
        ref = U.pointwise_dgrad(ds, pw)
        assert rel_err(f64(dx[:, d0:d0 + step]), ref) <= tol, ("dgrad", d0)
        assert rel_err(f64(dm[:, d0:d0 + step]), np.where(xs > 0, ref, 0.0)) <= tol, ("dgrad_relu", d0)
        a, b = U.pointwise_wgrad(xs, ds)
        ref_dp += a
        ref_db += b
    assert rel_err(f64(dp), ref_dp) <= tol and rel_err(f64(db), ref_db) <= tol
