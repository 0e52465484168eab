"""GPU parity of the 2-D variant (geometry flag `flat`: D is a stack of independent slices, 3x3 kernels,
1x2x2 windows; the paper's 2-D U-Net on slabs, Sec. 3) against the fp64 oracle of oracle/flat.py on the
unpartitioned tensor.  Bounds as for the 3-D operations: 1e-2 (bf16) / 1e-5 (f32) on
max_i |g_i - r_i| / max(|r_i|, rms(r)); copies, pooling and the ReLU masks are bit-exact."""
import numpy as np
import pytest
import torch

from oracle import flat as O
from oracle import tiling
from oracle.unet import round_bf16
from paper_1909_03108_amd import sp3d, synth
from gpu_util import DT, TOL, bits, f64, rel_err, to_dev, widen

pytestmark = pytest.mark.gpu


def draw(dtype, shape, seed):
    return synth.normal_volume(shape, seed, dtype)


class Layer:
    """plumbing for one 2-D convolution layer on a tile grid (no arithmetic here)"""

    def __init__(self, n, dhw, grid, cin, cout, dtype, halo=1, grow=0):
        self.g = sp3d.Geom(n, dhw, grid, halo, grow, flat=1)
        self.cin, self.cout, self.dtype, self.dt = cin, cout, dtype, DT[dtype]
        self.ws = {op: sp3d.alloc_ws(sp3d.sp_workspace_bytes(op, self.g, cin, cout, self.dt))
                   for op in (sp3d.SP_OP_FWD, sp3d.SP_OP_DGRAD, sp3d.SP_OP_WGRAD)}

    def padded(self, V, c, exchange=True, poison=True):
        """volume -> padded tiles; the D margins are filled with NaN: nothing may read them"""
        g = self.g
        P = sp3d.alloc_padded(g, c, self.dt)
        if poison:
            P[:, :, :, :, :g.halo] = float("nan")
            P[:, :, :, :, -g.halo:] = float("nan")
        sp3d.sp_partition(to_dev(V), P, g, c, self.dt)
        if exchange:
            sp3d.sp_halo_exchange(P, g, c, self.dt)
        return P

    def volume(self, P, c):
        V = torch.empty((self.g.n, self.g.d, self.g.h, self.g.w, c), dtype=P.dtype, device="cuda")
        sp3d.sp_unpartition(P, V, self.g, c, self.dt)
        return V


SMALL = [
    # n, dhw, grid, cin, cout, dtype
    (1, (3, 8, 8), (1, 2, 2), 5, 8, "f32"),            # the slab input: 5 channels
    (2, (2, 6, 10), (2, 3, 5), 3, 5, "bf16"),          # grid split along the slice axis too
    (1, (1, 16, 64), (1, 2, 1), 32, 32, "bf16"),       # one slice, whole 8 x 32 patches
    (1, (5, 20, 72), (1, 2, 1), 32, 32, "bf16"),       # ragged rows and columns, 5 slices
    (1, (4, 8, 32), (2, 1, 1), 32, 64, "bf16"),
    (1, (16, 8, 64), (1, 2, 1), 64, 64, "bf16"),       # pairs of input chunks, every slot phase
    (1, (3, 12, 40), (1, 1, 1), 128, 64, "bf16"),      # two pairs (first / last)
    (1, (2, 4, 32), (1, 1, 1), 192, 32, "bf16"),       # three pairs
    (1, (7, 5, 33), (1, 1, 1), 96, 32, "bf16"),        # three single chunks (first / middle / last)
    (1, (4, 16, 64), (1, 2, 2), 32, 32, "bf16"),       # whole patches: direct-to-LDS weight gradient
    (1, (3, 16, 40), (1, 2, 1), 5, 32, "bf16"),        # the slab input on the matrix cores (zero-padded channels)
    # tiles narrower than half a patch: several slices side by side in one patch
    (1, (8, 8, 8), (1, 1, 1), 32, 32, "bf16"),         # 8 wide: 3 would fit, 2 divide the 8 slices
    (1, (3, 8, 8), (1, 1, 1), 32, 32, "bf16"),         # 3 slices side by side, one step
    (1, (12, 8, 8), (1, 2, 2), 64, 64, "bf16"),        # 4 x 4 tiles: 4 slices side by side, pairs of chunks
    (1, (6, 16, 24), (1, 1, 2), 128, 64, "bf16"),      # 12 wide: 2 side by side; two launches with partial sums
    (2, (4, 8, 10), (2, 1, 1), 96, 32, "bf16"),        # batch 2, grid over the stack, three launches
    (1, (5, 8, 8), (1, 1, 1), 64, 32, "bf16"),         # 5 slices: no divisor below 4, nothing side by side
    # wide layers on few voxels: the output-stationary kernel
    (1, (4, 8, 8), (1, 2, 2), 512, 128, "bf16"),       # forward, one whole voxel group
    (1, (3, 6, 10), (1, 1, 2), 128, 512, "bf16"),      # data gradient (plain and masked), ragged voxel group
    (1, (5, 16, 8), (1, 2, 1), 640, 256, "bf16"),      # three voxel groups, two groups of output blocks
    # (the cases above fill at most half of the chip and run with 128 voxels per workgroup; these two have more
    # than 128 workgroups of 256 voxels in the forward and in the data-gradient direction)
    (1, (9, 32, 32), (1, 2, 2), 512, 512, "bf16"),     # 36 voxel groups x 4 groups of output blocks, both directions
    (1, (17, 32, 32), (1, 1, 2), 512, 256, "bf16"),    # forward: 68 x 2 workgroups of 256; data gradient: 128-voxel groups
]


@pytest.mark.parametrize("n,dhw,grid,cin,cout,dtype", SMALL)
def test_conv_fwd_dgrad_wgrad_match_oracle(n, dhw, grid, cin, cout, dtype):
    L = Layer(n, dhw, grid, cin, cout, dtype)
    g, dt, tol = L.g, L.dt, TOL[dtype]
    x = draw(dtype, (n,) + dhw + (cin,), 1)
    dz = draw(dtype, (n,) + dhw + (cout,), 2)
    w = synth.weights(cin, cout, 3, dtype, taps=(3, 3))
    bias = np.linspace(-0.5, 0.5, cout).astype(np.float32)
    xmask = draw(dtype, (n,) + dhw + (cin,), 4)

    Px = L.padded(x, cin)
    for relu in (False, True):
        Py = sp3d.alloc_padded(g, cout, dt)
        sp3d.conv3d_fwd(Px, to_dev(w), torch.from_numpy(bias).cuda(), Py, g, cin, cout, dt,
                        sp3d.SP_FLAG_RELU if relu else 0, L.ws[sp3d.SP_OP_FWD])
        ref = O.conv_fwd(widen(x), widen(w), bias.astype(np.float64), relu)
        assert rel_err(f64(L.volume(Py, cout)), ref) <= tol, ("fwd", relu)
        # margins of the output are not written
        got = f64(Py)
        m = np.ones(got.shape, dtype=bool)
        m[(slice(None),) * 4 + (slice(1, -1),) * 3] = False
        assert np.all(got[m] == 0.0)
    Pz = L.padded(dz, cout)
    Pdx = sp3d.alloc_padded(g, cin, dt)
    sp3d.conv3d_dgrad(Pz, to_dev(w), Pdx, g, cin, cout, dt, L.ws[sp3d.SP_OP_DGRAD])
    ref = O.conv_dgrad(widen(dz), widen(w))
    dx = L.volume(Pdx, cin)
    assert rel_err(f64(dx), ref) <= tol
    # with the ReLU mask of the layer input: the same bits where the mask is positive, zero elsewhere
    Pm = L.padded(xmask, cin, exchange=False, poison=False)
    Pdm = sp3d.alloc_padded(g, cin, dt)
    sp3d.conv3d_dgrad_relu(Pz, to_dev(w), Pm, Pdm, g, cin, cout, dt, L.ws[sp3d.SP_OP_DGRAD])
    keep = torch.from_numpy(widen(xmask) > 0).cuda()
    assert torch.equal(L.volume(Pdm, cin), torch.where(keep, dx, torch.zeros_like(dx)))
    # weight and bias gradient
    Pzi = L.padded(dz, cout, exchange=False)
    dw = torch.full((3, 3, cin, cout), 123.0, dtype=torch.float32, device="cuda")
    db = torch.full((cout,), 123.0, dtype=torch.float32, device="cuda")
    sp3d.conv3d_wgrad(Px, Pzi, dw, db, g, cin, cout, dt, L.ws[sp3d.SP_OP_WGRAD])
    assert rel_err(f64(dw), O.conv_wgrad(widen(x), widen(dz))) <= tol
    assert rel_err(f64(db), O.bias_grad(widen(dz))) <= tol


@pytest.mark.parametrize("dhw,grid,ca,cb,cout", [((3, 12, 40), (1, 2, 1), 32, 32, 64),
                                                 ((3, 8, 10), (1, 1, 2), 256, 256, 128),   # output-stationary kernel,
                                                 ((2, 4, 8), (1, 1, 1), 64, 64, 512)])     # forward / data gradient
def test_two_tensor_convolutions_equal_the_concatenated_ones(dhw, grid, ca, cb, cout):
    n = 1
    L = Layer(n, dhw, grid, ca + cb, cout, "bf16")
    g, dt = L.g, L.dt
    xa, xb = draw("bf16", (n,) + dhw + (ca,), 1), draw("bf16", (n,) + dhw + (cb,), 2)
    dz = draw("bf16", (n,) + dhw + (cout,), 3)
    w = to_dev(synth.weights(ca + cb, cout, 4, "bf16", taps=(3, 3)))
    Pa, Pb = L.padded(xa, ca), L.padded(xb, cb)
    Pc = L.padded(np.concatenate([xa, xb], axis=-1), ca + cb)
    Pz, Pzi = L.padded(dz, cout), L.padded(dz, cout, exchange=False)
    y1, y2 = sp3d.alloc_padded(g, cout, dt), sp3d.alloc_padded(g, cout, dt)
    sp3d.conv3d_fwd(Pc, w, None, y1, g, ca + cb, cout, dt, sp3d.SP_FLAG_RELU, L.ws[sp3d.SP_OP_FWD])
    sp3d.conv3d_fwd2(Pa, ca, Pb, cb, w, None, y2, g, cout, dt, sp3d.SP_FLAG_RELU, L.ws[sp3d.SP_OP_FWD])
    assert torch.equal(y1, y2)
    ref = O.conv_fwd(np.concatenate([widen(xa), widen(xb)], axis=-1), f64(w), relu=True)
    assert rel_err(f64(L.volume(y2, cout)), ref) <= 1e-2
    d1 = sp3d.alloc_padded(g, ca + cb, dt)
    da, db_ = sp3d.alloc_padded(g, ca, dt), sp3d.alloc_padded(g, cb, dt)
    sp3d.conv3d_dgrad(Pz, w, d1, g, ca + cb, cout, dt, L.ws[sp3d.SP_OP_DGRAD])
    sp3d.conv3d_dgrad2(Pz, w, da, ca, db_, cb, g, cout, dt, L.ws[sp3d.SP_OP_DGRAD])
    assert torch.equal(L.volume(d1, ca + cb), torch.cat([L.volume(da, ca), L.volume(db_, cb)], dim=-1))
    w1 = torch.empty((3, 3, ca + cb, cout), dtype=torch.float32, device="cuda")
    w2 = torch.empty_like(w1)
    sp3d.conv3d_wgrad(Pc, Pzi, w1, None, g, ca + cb, cout, dt, L.ws[sp3d.SP_OP_WGRAD])
    sp3d.conv3d_wgrad2(Pa, ca, Pb, cb, Pzi, w2, None, g, cout, dt, L.ws[sp3d.SP_OP_WGRAD])
    assert torch.equal(w1, w2)


@pytest.mark.parametrize("c,dtype", [(3, "f32"), (32, "bf16")])
def test_halo_operations_move_only_the_in_slice_regions(c, dtype):
    """pack / unpack / one-pass exchange fill the H and W margins of every slice like the slicing oracle and
    leave the D margins (and the message space of the other 18 regions) as they were"""
    n, dhw, grid = 1, (4, 8, 16), (2, 2, 2)
    g, dt = sp3d.Geom(n, dhw, grid, 1, 0, flat=1), DT[dtype]
    V = draw(dtype, (n,) + dhw + (c,), 7)
    ref = tiling.exchange(tiling.partition(V, grid, 1), 1)
    for one_pass in (False, True):
        P = torch.full(g.padded_shape + (c,), 9.0, dtype=sp3d.torch_dtype(dt), device="cuda")
        sp3d.sp_partition(to_dev(V), P, g, c, dt)
        if one_pass:
            sp3d.sp_halo_exchange(P, g, c, dt)
        else:
            M = torch.full((int(sp3d.sp_msg_elems(g, c)),), 5.0, dtype=P.dtype, device="cuda")
            sp3d.halo_pack(P, M, g, c, dt)
            sp3d.halo_unpack(P, M, g, c, dt)
        got = bits(P)
        assert np.array_equal(got[:, :, :, :, 1:-1], ref[:, :, :, :, 1:-1])
        nine = bits(torch.full((1,), 9.0, dtype=P.dtype))[0]
        assert np.all(got[:, :, :, :, 0] == nine) and np.all(got[:, :, :, :, -1] == nine)


POOL = [  # n, fine dhw, grid, dtype
    (1, (3, 8, 16), (1, 4, 1), "bf16"),
    (2, (2, 12, 8), (2, 3, 2), "f32"),
    (1, (5, 8, 80), (1, 2, 1), "bf16"),
]


@pytest.mark.parametrize("n,dhw,grid,dtype", POOL)
@pytest.mark.parametrize("c", [3, 32])
def test_pooling_bit_exact(n, dhw, grid, dtype, c):
    gf = sp3d.Geom(n, dhw, grid, 1, 0, flat=1)
    gc = sp3d.coarse_geom(gf)
    assert (gc.d, gc.h, gc.w) == (dhw[0], dhw[1] // 2, dhw[2] // 2)
    L = Layer(n, dhw, grid, c, c, dtype)
    Lc = Layer(n, (gc.d, gc.h, gc.w), grid, c, c, dtype)
    dt = DT[dtype]
    x = draw(dtype, (n,) + dhw + (c,), 1)
    x = np.where(widen(x) < 0, np.zeros_like(x), x)          # ties: ReLU-like zeros
    dy = draw(dtype, (n, gc.d, gc.h, gc.w, c), 2)
    skip = draw(dtype, (n,) + dhw + (c,), 3)
    Px = L.padded(x, c, exchange=False)
    Py = sp3d.alloc_padded(gc, c, dt)
    sp3d.sp_maxpool2_fwd(Px, Py, gf, c, dt)
    assert np.array_equal(f64(Lc.volume(Py, c)), O.maxpool_fwd(widen(x)))
    Pdy = Lc.padded(dy, c, exchange=False)
    Pdx = sp3d.alloc_padded(gf, c, dt)
    sp3d.sp_maxpool2_bwd(Px, Pdy, Pdx, gf, c, dt)
    assert np.array_equal(f64(L.volume(Pdx, c)), O.maxpool_bwd(widen(x), widen(dy)))
    Ps = L.padded(skip, c, exchange=False, poison=False)
    Pj = sp3d.alloc_padded(gf, c, dt)
    sp3d.sp_maxpool2_bwd_join(Px, Pdy, Ps, Pj, gf, c, dt)
    sp3d.sp_add(Pdx, Ps, Pdx, gf, c, dt)
    sp3d.sp_relu_bwd(Pdx, Px, Pdx, gf, c, dt)
    assert torch.equal(L.volume(Pdx, c), L.volume(Pj, c))
    ref = np.where(widen(x) > 0, O.maxpool_bwd(widen(x), widen(dy)) + widen(skip), 0.0)
    assert rel_err(f64(L.volume(Pj, c)), ref) <= (2.0 ** -8 if dtype == "bf16" else 1e-6)


UP = [  # n, fine dhw, grid, cin, cout, dtype
    (1, (3, 8, 16), (1, 2, 2), 6, 3, "f32"),
    (1, (2, 8, 16), (1, 2, 1), 16, 8, "bf16"),           # bf16 fallbacks with 8-channel groups
    (1, (5, 8, 80), (1, 2, 1), 64, 32, "bf16"),          # matrix cores; ragged 32-voxel segment
    (2, (2, 4, 128), (1, 1, 2), 32, 32, "bf16"),
    (1, (3, 4, 64), (1, 1, 1), 512, 256, "bf16"),        # wide: one tap per workgroup / weights from global memory
]


@pytest.mark.parametrize("n,dhw,grid,cin,cout,dtype", UP)
def test_upconv_fwd_dgrad_wgrad_match_oracle(n, dhw, grid, cin, cout, dtype):
    gf = sp3d.Geom(n, dhw, grid, 1, 0, flat=1)
    gc = sp3d.coarse_geom(gf)
    cd = (gc.d, gc.h, gc.w)
    Lf, Lc = Layer(n, dhw, grid, cout, cout, dtype), Layer(n, cd, grid, cin, cin, dtype)
    dt, tol = DT[dtype], TOL[dtype]
    x = draw(dtype, (n,) + cd + (cin,), 1)
    dy = draw(dtype, (n,) + dhw + (cout,), 2)
    u = synth.weights(cin, cout, 3, dtype, taps=(2, 2), var=1.0 / cin)
    bias = np.linspace(-1, 1, cout).astype(np.float32)
    Px = Lc.padded(x, cin, exchange=False)
    Py = sp3d.alloc_padded(gf, cout, dt)
    sp3d.sp_upconv2_fwd(Px, to_dev(u), torch.from_numpy(bias).cuda(), Py, gf, cin, cout, dt)
    assert rel_err(f64(Lf.volume(Py, cout)), O.upconv_fwd(widen(x), widen(u), bias.astype(np.float64))) <= tol
    Pdy = Lf.padded(dy, cout, exchange=False)
    Pdx = sp3d.alloc_padded(gc, cin, dt)
    sp3d.sp_upconv2_dgrad(Pdy, to_dev(u), Pdx, gf, cin, cout, dt)
    assert rel_err(f64(Lc.volume(Pdx, cin)), O.upconv_dgrad(widen(dy), widen(u))) <= tol
    du = torch.full((2, 2, cin, cout), 7.0, dtype=torch.float32, device="cuda")
    db = torch.full((cout,), 7.0, dtype=torch.float32, device="cuda")
    ws = sp3d.alloc_ws(sp3d.sp_workspace_bytes(sp3d.SP_OP_UPCONV_WGRAD, gf, cin, cout, dt))
    sp3d.sp_upconv2_wgrad(Px, Pdy, du, db, gf, cin, cout, dt, ws)
    rdu, rdb = O.upconv_wgrad(widen(x), widen(dy))
    assert rel_err(f64(du), rdu) <= tol
    assert rel_err(f64(db), rdb) <= tol


@pytest.mark.parametrize("dhw,grid,chans", [((3, 24, 80), (1, 2, 2), (32, 32, 32)),
                                            ((2, 16, 64), (2, 2, 1), (64, 64, 32)),
                                            ((4, 16, 16), (1, 2, 2), (32, 64, 32)),      # slices side by side, grown boxes
                                            ((2, 8, 16), (1, 2, 2), (512, 512, 128))])   # output-stationary kernel, grown boxes
def test_two_layers_after_one_exchange_of_wide_margins(dhw, grid, chans):
    """halo 2, first layer with grow 1 (no growth along the slice axis), second layer on its own voxels:
    bit for bit the result of two layers with one exchange each on the one-voxel layout"""
    n = 1
    c0, c1, c2 = chans
    x = draw("bf16", (n,) + dhw + (c0,), 1)
    w1 = to_dev(synth.weights(c0, c1, 2, "bf16", taps=(3, 3)))
    w2 = to_dev(synth.weights(c1, c2, 3, "bf16", taps=(3, 3)))
    outs = []
    for halo in (1, 2):
        La, Lb = Layer(n, dhw, grid, c0, c1, "bf16", halo), Layer(n, dhw, grid, c1, c2, "bf16", halo)
        g, dt = La.g, La.dt
        Px = La.padded(x, c0)
        P1, P2 = sp3d.alloc_padded(g, c1, dt), sp3d.alloc_padded(g, c2, dt)
        g1 = g.grown(halo - 1)              # the workspace size depends on the output box
        ws1 = sp3d.alloc_ws(sp3d.sp_workspace_bytes(sp3d.SP_OP_FWD, g1, c0, c1, dt))
        sp3d.conv3d_fwd(Px, w1, None, P1, g1, c0, c1, dt, sp3d.SP_FLAG_RELU, ws1)
        if halo == 1:
            sp3d.sp_halo_exchange(P1, g, c1, dt)
        sp3d.conv3d_fwd(P1, w2, None, P2, g, c1, c2, dt, sp3d.SP_FLAG_RELU, Lb.ws[sp3d.SP_OP_FWD])
        outs.append(Lb.volume(P2, c2))
    assert torch.equal(outs[0], outs[1])
    ref = O.conv_fwd(round_bf16(O.conv_fwd(widen(x), f64(w1), relu=True)), f64(w2), relu=True)
    assert rel_err(f64(outs[1]), ref) <= 1e-2


def _rel_rms(got, ref):
    return float(np.sqrt(np.mean((got - ref) ** 2)) / np.sqrt(np.mean(ref ** 2)))


@pytest.mark.timeout(600)
@pytest.mark.parametrize("convs,channels,dhw", [(2, (32, 64, 128), (3, 32, 32)), (4, (32, 64, 128), (3, 32, 32)),
                                                (2, (32, 512), (2, 16, 16))])      # wide bottom level on 8 x 8 voxels
def test_flat_unet_against_the_composed_oracle(convs, channels, dhw):
    """The 2-D U-Net (slab input with 5 channels, the same architecture with 2-D operations) on a 2 x 2 tile
    grid against the storage-aware oracle chain: free-running forward to 3e-2 element-wise / 1e-2 rms (twice that
    with four convolutions per block),
    free-running backward as a wiring check (0.25 in relative rms: ReLU decisions within the forward error of
    zero flip), a second step bit for bit, and the two-layers-per-exchange layout bit for bit.  The third
    configuration has a 512-channel bottom level: the output-stationary kernel in the forward pass and, with the
    ReLU mask and a grown box, in the backward pass."""
    from oracle import unet as OU
    from paper_1909_03108_amd import unet as PU
    in_ch, classes = 5, 3
    n, grid = 1, (1, 2, 2)
    plan = PU.layer_plan(channels, in_ch, classes, convs, flat=True)
    x = synth.normal_volume((n,) + dhw + (in_ch,), 11, "bf16")
    w_h = {name: synth.weights(shape[2], shape[3], 100 + k, "bf16", taps=shape[:2])
           for k, (name, shape) in enumerate(plan)}
    dl = synth.normal_volume((n,) + dhw + (classes,), 12, "bf16")
    w64 = {k: widen(v) for k, v in w_h.items()}
    A = {}
    ref_logits = OU.forward(widen(x), w64, channels, keep=A, store=OU.round_bf16, convs=convs, flat=True)
    ref_grads, ref_dx = OU.backward(widen(dl), w64, channels, A, store=OU.round_bf16, convs=convs, flat=True)

    wd = {k: to_dev(v) for k, v in w_h.items()}
    net = PU.UNet(n, dhw, grid, wd, channels, in_ch, classes, convs=convs, flat=True)
    logits = net.forward(to_dev(x))
    # 11 stored layers with two convolutions per block, 21 with four: one bf16 rounding each
    emax, erms = (3e-2, 1e-2) if convs == 2 else (6e-2, 2e-2)
    assert rel_err(f64(logits), ref_logits) <= emax and _rel_rms(f64(logits), ref_logits) <= erms
    grads, dx = net.backward(to_dev(dl))
    worst = max([_rel_rms(f64(grads[k]), ref_grads[k]) for k, _ in plan] + [_rel_rms(f64(dx), ref_dx)])
    print("2-D network, free-running backward: worst relative rms %.3f" % worst)
    assert worst <= 0.25
    for k, shape in plan:
        assert tuple(grads[k].shape) == tuple(shape)
    logits2 = net.forward(to_dev(x))
    grads2, dx2 = net.backward(to_dev(dl))
    assert torch.equal(logits2, logits) and torch.equal(dx2, dx)
    for k, _ in plan:
        assert torch.equal(grads2[k], grads[k]), k
    wide = PU.UNet(n, dhw, grid, wd, channels, in_ch, classes, convs=convs, halo=2, flat=True)
    logits3 = wide.forward(to_dev(x))
    grads3, dx3 = wide.backward(to_dev(dl))
    assert torch.equal(logits3, logits) and torch.equal(dx3, dx)
    for k, _ in plan:
        assert torch.equal(grads3[k], grads[k]), k


@pytest.mark.timeout(600)
def test_bench_shape_first_two_layers_full():
    """The shape `bench.py --workload paper2d` times (16 slabs of 512 x 512, grid 1x2x2): the slab layer 5 -> 32 and
    a 32 -> 32 layer, every output element of forward, data gradient and weight gradient against the oracle."""
    n, dhw, grid = 1, (16, 512, 512), (1, 2, 2)
    for cin, cout in ((5, 32), (32, 32)):
        L = Layer(n, dhw, grid, cin, cout, "bf16")
        g, dt = L.g, L.dt
        x = draw("bf16", (n,) + dhw + (cin,), 21)
        dz = draw("bf16", (n,) + dhw + (cout,), 22)
        w = synth.weights(cin, cout, 23, "bf16", taps=(3, 3))
        Px = L.padded(x, cin)
        Py = sp3d.alloc_padded(g, cout, dt)
        sp3d.conv3d_fwd(Px, to_dev(w), None, Py, g, cin, cout, dt, sp3d.SP_FLAG_RELU, L.ws[sp3d.SP_OP_FWD])
        assert rel_err(f64(L.volume(Py, cout)), O.conv_fwd(widen(x), widen(w), relu=True)) <= 1e-2, (cin, "fwd")
        del Py
        Pzi = L.padded(dz, cout, exchange=False)
        dw = torch.empty((3, 3, cin, cout), dtype=torch.float32, device="cuda")
        db = torch.empty((cout,), dtype=torch.float32, device="cuda")
        sp3d.conv3d_wgrad(Px, Pzi, dw, db, g, cin, cout, dt, L.ws[sp3d.SP_OP_WGRAD])
        assert rel_err(f64(dw), O.conv_wgrad(widen(x), widen(dz))) <= 1e-2, (cin, "wgrad")
        assert rel_err(f64(db), O.bias_grad(widen(dz))) <= 1e-2
        dw2 = torch.empty_like(dw)
        sp3d.conv3d_wgrad(Px, Pzi, dw2, None, g, cin, cout, dt, L.ws[sp3d.SP_OP_WGRAD])
        assert torch.equal(dw, dw2)                       # fixed reduction order
        del Px, Pzi
        if cin == 32:
            Pz = L.padded(dz, cout)
            Pdx = sp3d.alloc_padded(g, cin, dt)
            sp3d.conv3d_dgrad(Pz, to_dev(w), Pdx, g, cin, cout, dt, L.ws[sp3d.SP_OP_DGRAD])
            assert rel_err(f64(L.volume(Pdx, cin)), O.conv_dgrad(widen(dz), widen(w))) <= 1e-2, "dgrad"
