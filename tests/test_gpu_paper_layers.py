"""GPU parity of the widest layers of the paper's own network (Sec. 3, "Experimental Results": the first block
has 32 filters and the number doubles after each max-pooling, so the sixth block of the 512^3 network works on
16^3 voxels with 1024 filters) at the shapes `bench.py --workload paper512` / `paper2d` run them: grid 4x4x1
with 4 x 4 x 16 tiles in 3-D, the 16 x 16 images of 16 slabs in 2-D.

All voxels are compared.  A 1024-filter layer costs the plain fp64 oracle minutes per pass, and the
definition is independent per output channel (forward: per column of w; data gradient: per row), so the oracle
is evaluated on all voxels for a seeded subset of the output channels that has at least four channels in
every block of 32 (the unit the kernels tile channels by); weight gradients on seeded entries, each a full
reduction.  The 512 -> 1024 layer is compared on every channel."""
import numpy as np
import pytest
import torch

from oracle import conv3d, flat as O2
from oracle import unet_ops as U
from paper_1909_03108_amd import sp3d, synth
from gpu_util import DT, TOL, f64, progress, rel_err, to_dev, widen
from test_gpu_conv import Layer

pytestmark = pytest.mark.gpu


def _relu_bits(a):
    return np.where(widen(a) > 0, a, np.zeros_like(a))


def _channel_subset(c, per_block, rng):
    """`per_block` channels out of every block of 32, sorted."""
    return np.sort(np.concatenate([32 * b + rng.choice(32, per_block, replace=False) for b in range(c // 32)]))


# the decoder's first block reads concat(skip 512, up-convolved 512): the widest two-tensor layer of the network
WIDE_3D = [(512, 1024, 32), ((512, 512), 512, 8), (1024, 1024, 4)]


@pytest.mark.timeout(1500)
@pytest.mark.parametrize("cin,cout,per_block", WIDE_3D,
                         ids=["%s_to_%d" % (str(c).replace(" ", ""), o) for c, o, _ in WIDE_3D])
def test_paper_bottom_level_3d(cin, cout, per_block):
    two = isinstance(cin, tuple)
    ca, cb = cin if two else (cin, 0)
    ct = ca + cb
    n, dhw, grid = 1, (16, 16, 16), (4, 4, 1)
    L = Layer(n, dhw, grid, ct, cout, "bf16")
    g, dt, tol = L.g, L.dt, TOL["bf16"]
    x = _relu_bits(synth.normal_volume((n,) + dhw + (ct,), 101, "bf16"))
    dz = synth.normal_volume((n,) + dhw + (cout,), 102, "bf16")
    w = synth.weights(ct, cout, 103, "bf16")
    bias = (0.05 * np.cos(np.arange(cout))).astype(np.float32)
    Wd = widen(w)
    rng = np.random.default_rng(ct + cout)
    co = _channel_subset(cout, per_block, rng)
    ci = _channel_subset(ct, min(32, per_block * max(1, ct // cout)), rng)
    w_dev, b_dev = to_dev(w), torch.from_numpy(bias).cuda()
    if two:
        Pa, Pb = L.padded(np.ascontiguousarray(x[..., :ca]), ca), L.padded(np.ascontiguousarray(x[..., ca:]), cb)
    else:
        Pa = L.padded(x, ct)
    Pz = L.padded(dz, cout)
    Py = sp3d.alloc_padded(g, cout, dt)
    if two:
        sp3d.conv3d_fwd2(Pa, ca, Pb, cb, w_dev, b_dev, Py, g, cout, dt, sp3d.SP_FLAG_RELU, L.ws[sp3d.SP_OP_FWD])
    else:
        sp3d.conv3d_fwd(Pa, w_dev, b_dev, Py, g, ct, cout, dt, sp3d.SP_FLAG_RELU, L.ws[sp3d.SP_OP_FWD])
    ref = conv3d.conv3d_fwd(x, np.ascontiguousarray(Wd[..., co]), bias[co].astype(np.float64), relu=True)
    assert rel_err(f64(L.volume(Py, cout))[..., co], ref) <= tol, "fwd"
    progress("%s -> %d: fwd ok" % (cin, cout))
    # data gradient: rows ci of the weights give channels ci of dx
    ref = conv3d.conv3d_dgrad(dz, np.ascontiguousarray(Wd[:, :, :, ci, :]))
    if two:
        Pda, Pdb = sp3d.alloc_padded(g, ca, dt), sp3d.alloc_padded(g, cb, dt)
        sp3d.conv3d_dgrad2(Pz, w_dev, Pda, ca, Pdb, cb, g, cout, dt, L.ws[sp3d.SP_OP_DGRAD])
        dx = torch.cat([L.volume(Pda, ca), L.volume(Pdb, cb)], dim=-1)
        assert rel_err(f64(dx)[..., ci], ref) <= tol, "dgrad2"
    else:
        Pdx, Pdm = sp3d.alloc_padded(g, ct, dt), sp3d.alloc_padded(g, ct, dt)
        sp3d.conv3d_dgrad(Pz, w_dev, Pdx, g, ct, cout, dt, L.ws[sp3d.SP_OP_DGRAD])
        sp3d.conv3d_dgrad_relu(Pz, w_dev, Pa, Pdm, g, ct, cout, dt, L.ws[sp3d.SP_OP_DGRAD])
        dx, dm = L.volume(Pdx, ct), L.volume(Pdm, ct)
        assert rel_err(f64(dx)[..., ci], ref) <= tol, "dgrad"
        assert rel_err(f64(dm)[..., ci], np.where(widen(x)[..., ci] > 0, ref, 0.0)) <= tol, "dgrad_relu"
        assert torch.equal(dm, torch.where(to_dev(x).float() > 0, dx, torch.zeros_like(dx)))
    progress("%s -> %d: dgrad ok" % (cin, cout))
    dw = torch.full((3, 3, 3, ct, cout), 123.0, dtype=torch.float32, device="cuda")
    db = torch.full((cout,), 123.0, dtype=torch.float32, device="cuda")
    if two:
        sp3d.conv3d_wgrad2(Pa, ca, Pb, cb, Pz, dw, db, g, cout, dt, L.ws[sp3d.SP_OP_WGRAD])
    else:
        sp3d.conv3d_wgrad(Pa, Pz, dw, db, g, ct, cout, dt, L.ws[sp3d.SP_OP_WGRAD])
    # seeded entries plus one entry in every (tap, 32 x 32 channel block): each pair of chunks of the kernel
    nb = (ct // 32) * (cout // 32)
    blk = np.arange(27 * nb)
    tap, bi, bo = blk // nb, (blk % nb) // (cout // 32), blk % (cout // 32)
    one_per_block = (tap * ct + 32 * bi + rng.integers(0, 32, blk.size)) * cout + 32 * bo + rng.integers(0, 32, blk.size)
    sel = np.unique(np.concatenate([rng.integers(0, 27 * ct * cout, 8192), one_per_block]))
    assert rel_err(f64(dw).ravel()[sel], conv3d.conv3d_wgrad(x, dz, sel=sel)) <= tol, "wgrad"
    assert rel_err(f64(db), conv3d.bias_grad(dz)) <= tol, "bgrad"


@pytest.mark.timeout(900)
def test_paper_bottom_level_upconv_1024_to_512():
    """The first transposed convolution of the decoder, 1024 -> 512 from 16^3 to 32^3 on 4x4x1 tiles: forward
    and data gradient on every element; the weight gradient for every tap on all 512 output channels and 128
    seeded input channels (four per block of 32); the bias gradient in full."""
    n, dhw, grid, cin, cout = 1, (32, 32, 32), (4, 4, 1), 1024, 512
    gf = sp3d.Geom(n, dhw, grid)
    gc = sp3d.coarse_geom(gf)
    dt, tol = DT["bf16"], TOL["bf16"]
    x = _relu_bits(synth.normal_volume((n, 16, 16, 16, cin), 111, "bf16"))
    dy = synth.normal_volume((n,) + dhw + (cout,), 112, "bf16")
    u = synth.weights(cin, cout, 113, "bf16", taps=(2, 2, 2))
    bias = (0.1 * np.sin(np.arange(cout))).astype(np.float32)

    def padded(g_, V, c):
        P = sp3d.alloc_padded(g_, c, dt)
        sp3d.sp_partition(to_dev(V), P, g_, c, dt)
        return P

    def volume(g_, P, c):
        V = torch.empty((g_.n, g_.d, g_.h, g_.w, c), dtype=P.dtype, device="cuda")
        sp3d.sp_unpartition(P, V, g_, c, dt)
        return V

    Px, Pdy = padded(gc, x, cin), padded(gf, dy, cout)
    Py, Pdx = sp3d.alloc_padded(gf, cout, dt), sp3d.alloc_padded(gc, cin, dt)
    sp3d.sp_upconv2_fwd(Px, to_dev(u), torch.from_numpy(bias).cuda(), Py, gf, cin, cout, dt)
    assert rel_err(f64(volume(gf, Py, cout)), U.upconv2_fwd(widen(x), widen(u), bias)) <= tol
    sp3d.sp_upconv2_dgrad(Pdy, to_dev(u), Pdx, gf, cin, cout, dt)
    assert rel_err(f64(volume(gc, Pdx, cin)), U.upconv2_dgrad(widen(dy), widen(u))) <= tol
    du = torch.full((2, 2, 2, cin, cout), 7.0, dtype=torch.float32, device="cuda")
    db = torch.full((cout,), 7.0, dtype=torch.float32, device="cuda")
    ws = sp3d.alloc_ws(sp3d.sp_workspace_bytes(sp3d.SP_OP_UPCONV_WGRAD, gf, cin, cout, dt))
    sp3d.sp_upconv2_wgrad(Px, Pdy, du, db, gf, cin, cout, dt, ws)
    ci = _channel_subset(cin, 4, np.random.default_rng(7))
    ref_du, ref_db = U.upconv2_wgrad(widen(x[..., ci]), widen(dy))
    assert rel_err(f64(du)[:, :, :, ci], ref_du) <= tol
    assert rel_err(f64(db), ref_db) <= tol


@pytest.mark.timeout(900)
@pytest.mark.parametrize("grid", [(1, 2, 2), (1, 1, 1)])
def test_paper_bottom_level_2d_1024(grid):
    """The 2-D network's sixth block: 1024 -> 1024 with 3x3 kernels on the 16 x 16 images of 16 slabs (the
    output-stationary kernel), every element of forward, data gradient (plain and masked), weight and bias
    gradient against the numpy fp64 oracle of the 2-D variant."""
    n, dhw, cin, cout = 1, (16, 16, 16), 1024, 1024
    g = sp3d.Geom(n, dhw, grid, flat=1)
    dt, tol = DT["bf16"], TOL["bf16"]
    x = _relu_bits(synth.normal_volume((n,) + dhw + (cin,), 121, "bf16"))
    dz = synth.normal_volume((n,) + dhw + (cout,), 122, "bf16")
    w = synth.weights(cin, cout, 123, "bf16", taps=(3, 3))
    bias = (0.05 * np.cos(np.arange(cout))).astype(np.float32)
    ws = {op: sp3d.alloc_ws(sp3d.sp_workspace_bytes(op, g, cin, cout, dt)) for op in (0, 1, 2)}

    def padded(V, c, exchange=True):
        P = sp3d.alloc_padded(g, c, dt)
        sp3d.sp_partition(to_dev(V), P, g, c, dt)
        if exchange:
            sp3d.sp_halo_exchange(P, g, c, dt)
        return P

    def volume(P, c):
        V = torch.empty((n,) + dhw + (c,), dtype=P.dtype, device="cuda")
        sp3d.sp_unpartition(P, V, g, c, dt)
        return V

    Px, Pz = padded(x, cin), padded(dz, cout)
    Py, Pdx, Pdm = (sp3d.alloc_padded(g, c, dt) for c in (cout, cin, cin))
    sp3d.conv3d_fwd(Px, to_dev(w), torch.from_numpy(bias).cuda(), Py, g, cin, cout, dt, sp3d.SP_FLAG_RELU, ws[0])
    assert rel_err(f64(volume(Py, cout)), O2.conv_fwd(widen(x), widen(w), bias.astype(np.float64), True)) <= tol
    sp3d.conv3d_dgrad(Pz, to_dev(w), Pdx, g, cin, cout, dt, ws[1])
    sp3d.conv3d_dgrad_relu(Pz, to_dev(w), Px, Pdm, g, cin, cout, dt, ws[1])
    ref = O2.conv_dgrad(widen(dz), widen(w))
    assert rel_err(f64(volume(Pdx, cin)), ref) <= tol
    assert rel_err(f64(volume(Pdm, cin)), np.where(widen(x) > 0, ref, 0.0)) <= tol
    dw = torch.full((3, 3, cin, cout), 123.0, dtype=torch.float32, device="cuda")
    db = torch.full((cout,), 123.0, dtype=torch.float32, device="cuda")
    sp3d.conv3d_wgrad(Px, Pz, dw, db, g, cin, cout, dt, ws[2])
    assert rel_err(f64(dw), O2.conv_wgrad(widen(x), widen(dz))) <= tol
    assert rel_err(f64(db), O2.bias_grad(widen(dz))) <= tol
