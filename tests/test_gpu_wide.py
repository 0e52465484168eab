"""GPU parity on layouts with margins wider than one voxel, and of a block of convolutions that shares ONE
exchange (the overlap idea of Sec. 1 applied to a short stack): layer i of k computes, besides the tile's own
voxels, the k - i voxels around them that its successors read.

Checked: (1) every operation on a wide-margin layout gives what it gives on the one-voxel layout's oracle;
(2) each layer of a shared-exchange block matches the oracle on the stored output of the layer before,
(3) what a tile computed redundantly in its surround is bit for bit what the neighbour computed for itself,
(4) nothing outside the grown box is written (outside the volume everything stays zero padding)."""
import numpy as np
import pytest
import torch

from oracle import conv3d, tiling
from paper_1909_03108_amd import sp3d, synth
from gpu_util import DT, TOL, bits, f64, guard_alloc, guards_intact, rel_err, to_dev, widen

pytestmark = pytest.mark.gpu


def ws_for(g, cin, cout, dt):
    return {op: sp3d.alloc_ws(sp3d.sp_workspace_bytes(op, g, cin, cout, dt))
            for op in (sp3d.SP_OP_FWD, sp3d.SP_OP_DGRAD, sp3d.SP_OP_WGRAD)}


def exchanged(g, V, c, dt):
    P = sp3d.alloc_padded(g, c, dt)
    sp3d.sp_partition(to_dev(V), P, g, c, dt)
    sp3d.sp_halo_exchange(P, g, c, dt)
    return P


def volume(g, P, c, dt):
    V = torch.empty((g.n, g.d, g.h, g.w, c), dtype=P.dtype, device="cuda")
    sp3d.sp_unpartition(P, V, g, c, dt)
    return V


LAYERS = [  # n, dhw, grid, cin, cout, dtype, halo
    (1, (8, 8, 8), (2, 2, 1), 8, 16, "f32", 2),
    (2, (6, 6, 9), (2, 1, 3), 3, 5, "f32", 3),
    (1, (8, 12, 16), (2, 2, 2), 1, 32, "bf16", 2),       # first-layer kernels
    (1, (12, 20, 72), (2, 2, 1), 32, 32, "bf16", 2),     # ragged patches
    (1, (8, 16, 64), (2, 2, 1), 32, 32, "bf16", 4),      # whole-patch weight-gradient kernel
    (1, (6, 12, 40), (2, 1, 1), 128, 64, "bf16", 3),     # chunk pairs with partial sums
    (1, (4, 8, 16), (1, 2, 2), 32, 64, "bf16", 2),
]


@pytest.mark.parametrize("n,dhw,grid,cin,cout,dtype,h", LAYERS)
def test_layers_on_a_wide_margin_layout(n, dhw, grid, cin, cout, dtype, h):
    g, dt, tol = sp3d.Geom(n, dhw, grid, h), DT[dtype], TOL[dtype]
    ws = ws_for(g, cin, cout, dt)
    x = synth.normal_volume((n,) + dhw + (cin,), 1, dtype)
    dz = synth.normal_volume((n,) + dhw + (cout,), 2, dtype)
    w = synth.weights(cin, cout, 3, dtype)
    bias = np.linspace(-0.5, 0.5, cout).astype(np.float32)
    Px, Pz = exchanged(g, x, cin, dt), exchanged(g, dz, cout, dt)
    Py, Pdx = sp3d.alloc_padded(g, cout, dt), sp3d.alloc_padded(g, cin, dt)
    sp3d.conv3d_fwd(Px, to_dev(w), torch.from_numpy(bias).cuda(), Py, g, cin, cout, dt, sp3d.SP_FLAG_RELU, ws[0])
    assert rel_err(f64(volume(g, Py, cout, dt)), conv3d.conv3d_fwd(x, widen(w), bias.astype(np.float64), True)) <= tol
    sp3d.conv3d_dgrad(Pz, to_dev(w), Pdx, g, cin, cout, dt, ws[1])
    assert rel_err(f64(volume(g, Pdx, cin, dt)), conv3d.conv3d_dgrad(dz, widen(w))) <= tol
    dw = torch.full((3, 3, 3, cin, cout), 9.0, dtype=torch.float32, device="cuda")
    db = torch.full((cout,), 9.0, dtype=torch.float32, device="cuda")
    sp3d.conv3d_wgrad(Px, Pz, dw, db, g, cin, cout, dt, ws[2])
    assert rel_err(f64(dw), conv3d.conv3d_wgrad(x, dz)) <= tol
    assert rel_err(f64(db), conv3d.bias_grad(dz)) <= tol
    # the same bits as on the one-voxel layout: only addresses differ
    g1 = sp3d.Geom(n, dhw, grid)
    ws1 = ws_for(g1, cin, cout, dt)
    Qx, Qy = exchanged(g1, x, cin, dt), sp3d.alloc_padded(g1, cout, dt)
    sp3d.conv3d_fwd(Qx, to_dev(w), torch.from_numpy(bias).cuda(), Qy, g1, cin, cout, dt, sp3d.SP_FLAG_RELU, ws1[0])
    assert torch.equal(volume(g1, Qy, cout, dt), volume(g, Py, cout, dt))
    dw1 = torch.empty_like(dw)
    sp3d.conv3d_wgrad(Qx, exchanged(g1, dz, cout, dt), dw1, None, g1, cin, cout, dt, ws1[2])
    assert torch.equal(dw1, dw)


def grown_box(g, tile_idx, e):
    """padded-coordinate slices of the tile's own voxels grown by e towards the neighbours it has"""
    h, out = g.halo, []
    for i, ng, t in zip(tile_idx, (g.gd, g.gh, g.gw), g.tile):
        out.append(slice(h - (e if i > 0 else 0), h + t + (e if i < ng - 1 else 0)))
    return tuple(out)


def check_grown(g, P, c, dt, e, fill_bits):
    """P (written on top of a fill pattern) holds, in every tile's grown box, the window of the assembled volume,
    and the fill everywhere else."""
    got = bits(P)
    ref = tiling.padded_reference(bits(volume(g, P, c, dt)), (g.gd, g.gh, g.gw), g.halo)
    for n in range(g.n):
        for a in range(g.gd):
            for b in range(g.gh):
                for cc in range(g.gw):
                    box = grown_box(g, (a, b, cc), e)
                    assert np.array_equal(got[n, a, b, cc][box], ref[n, a, b, cc][box]), (a, b, cc)
                    rest = np.ones(got.shape[4:7], dtype=bool)
                    rest[box] = False
                    assert np.all(got[n, a, b, cc][rest] == fill_bits), (a, b, cc)


BLOCKS = [  # n, dhw, grid, channels of the stack (input first), dtype
    (1, (8, 8, 8), (2, 2, 2), (4, 6, 5), "f32"),
    (1, (12, 20, 72), (2, 2, 1), (32, 32, 32), "bf16"),          # ragged patches, two layers
    (1, (12, 12, 48), (3, 2, 2), (32, 32, 32, 32), "bf16"),      # three layers, inner tiles grow on both sides
    (1, (8, 16, 40), (2, 2, 1), (64, 64, 32), "bf16"),           # chunk pairs
    (1, (4, 4, 8), (2, 2, 1), (64, 64, 64), "bf16"),             # masked data gradient with grow on chunk pairs, tiny tiles
    (1, (8, 8, 40), (2, 2, 1), (128, 128, 128), "bf16"),         # the same with partial sums between pairs
    (1, (6, 8, 32), (1, 2, 1), (128, 32, 64, 32), "bf16"),       # partial sums between pairs, grow 2 and 1
]


@pytest.mark.parametrize("n,dhw,grid,chans,dtype", BLOCKS)
def test_block_of_layers_after_one_exchange(n, dhw, grid, chans, dtype):
    k = len(chans) - 1
    g, dt, tol = sp3d.Geom(n, dhw, grid, k), DT[dtype], TOL[dtype]
    tdt = sp3d.torch_dtype(dt)
    fill = 7.0
    fill_bits = bits(torch.tensor([fill], dtype=tdt, device="cuda"))[0]
    x = synth.normal_volume((n,) + dhw + (chans[0],), 1, dtype)
    ws_ = [synth.weights(chans[i], chans[i + 1], 10 + i, dtype) for i in range(k)]
    # forward: one exchange, then layer i with grow = k - i
    P = exchanged(g, x, chans[0], dt)
    acts, prev = [P], x
    bufs = []
    for i in range(1, k + 1):
        cin, cout = chans[i - 1], chans[i]
        buf, Py = guard_alloc(g.padded_shape + (cout,), tdt, fill)
        bufs.append(buf)
        gi = g.grown(k - i)
        sp3d.conv3d_fwd(P, to_dev(ws_[i - 1]), None, Py, gi, cin, cout, dt, sp3d.SP_FLAG_RELU,
                        sp3d.alloc_ws(sp3d.sp_workspace_bytes(sp3d.SP_OP_FWD, gi, cin, cout, dt)))
        assert guards_intact(buf, fill)
        y = volume(g, Py, cout, dt)
        assert rel_err(f64(y), conv3d.conv3d_fwd(prev, widen(ws_[i - 1]), relu=True)) <= tol, ("fwd", i)
        check_grown(g, Py, cout, dt, k - i, fill_bits)
        # beyond the volume an activation is zero padding: put that into the buffer the next layer reads
        # (the fill pattern stands for stale memory; a real buffer starts zeroed and stays zero there)
        zero_outside_grown(g, Py, k - i)
        prev, P = bits(y), Py
        acts.append(Py)
    # backward: d/dz of the last layer exchanged once, then layer i's data gradient with grow = i - 1 and the
    # ReLU mask of its input on that box.  The forward pass leaves layer i - 1's output on a box grown by
    # k - i + 1, which covers it for k = 2 only: longer runs share an exchange in the forward direction alone.
    if k != 2:
        return
    dz = synth.normal_volume((n,) + dhw + (chans[k],), 2, dtype)
    Pg, dprev = exchanged(g, dz, chans[k], dt), dz
    for i in range(k, 0, -1):
        cin, cout = chans[i - 1], chans[i]
        e = i - 1
        assert i == 1 or k - (i - 1) >= e          # the mask exists where it is needed
        gi = g.grown(e)
        wsb = sp3d.alloc_ws(sp3d.sp_workspace_bytes(sp3d.SP_OP_DGRAD, gi, cin, cout, dt))
        # weight gradient of layer i: interiors of dz_i, input with one voxel around the interior
        dw = torch.empty((3, 3, 3, cin, cout), dtype=torch.float32, device="cuda")
        sp3d.conv3d_wgrad(acts[i - 1], Pg, dw, None, g, cin, cout, dt,
                          sp3d.alloc_ws(sp3d.sp_workspace_bytes(sp3d.SP_OP_WGRAD, g, cin, cout, dt)))
        x_in = x if i == 1 else bits(volume(g, acts[i - 1], cin, dt))
        assert rel_err(f64(dw), conv3d.conv3d_wgrad(x_in, dprev)) <= tol, ("wgrad", i)
        buf, Pdx = guard_alloc(g.padded_shape + (cin,), tdt, fill)
        if i > 1:
            sp3d.conv3d_dgrad_relu(Pg, to_dev(ws_[i - 1]), acts[i - 1], Pdx, gi, cin, cout, dt, wsb)
            ref = conv3d.relu_bwd(conv3d.conv3d_dgrad(dprev, widen(ws_[i - 1])), widen(x_in))
        else:
            sp3d.conv3d_dgrad(Pg, to_dev(ws_[i - 1]), Pdx, gi, cin, cout, dt, wsb)
            ref = conv3d.conv3d_dgrad(dprev, widen(ws_[i - 1]))
        assert guards_intact(buf, fill)
        dx = volume(g, Pdx, cin, dt)
        assert rel_err(f64(dx), ref) <= tol, ("dgrad", i)
        check_grown(g, Pdx, cin, dt, e, fill_bits)
        zero_outside_grown(g, Pdx, e)
        Pg, dprev = Pdx, bits(dx)


def zero_outside_grown(g, P, e):
    """zero everything outside every tile's grown box (host side, test plumbing)"""
    keep = torch.zeros(P.shape[:-1], dtype=torch.bool, device="cuda")
    for a in range(g.gd):
        for b in range(g.gh):
            for c in range(g.gw):
                keep[(slice(None), a, b, c) + grown_box(g, (a, b, c), e)] = True
    P.mul_(keep.unsqueeze(-1).to(P.dtype))


def test_two_tensor_block_input_with_grow():
    """concat(a, b) 64 -> 32 with grow 1, then 32 -> 32: same bits as the single-tensor call on the concatenation;
    the data gradient into the two tensors likewise."""
    n, dhw, grid, dt = 1, (8, 12, 40), (2, 2, 1), sp3d.SP_BF16
    g = sp3d.Geom(n, dhw, grid, 2)
    a = synth.normal_volume((n,) + dhw + (32,), 1, "bf16")
    b = synth.normal_volume((n,) + dhw + (32,), 2, "bf16")
    w = to_dev(synth.weights(64, 32, 3, "bf16"))
    g1 = g.grown(1)
    ws = sp3d.alloc_ws(sp3d.sp_workspace_bytes(sp3d.SP_OP_FWD, g1, 64, 32, dt))
    Pa, Pb = exchanged(g, a, 32, dt), exchanged(g, b, 32, dt)
    Pc = exchanged(g, np.concatenate([a, b], axis=-1), 64, dt)
    Y2, Y1 = sp3d.alloc_padded(g, 32, dt), sp3d.alloc_padded(g, 32, dt)
    sp3d.conv3d_fwd2(Pa, 32, Pb, 32, w, None, Y2, g1, 32, dt, sp3d.SP_FLAG_RELU, ws)
    sp3d.conv3d_fwd(Pc, w, None, Y1, g1, 64, 32, dt, sp3d.SP_FLAG_RELU, ws)
    assert torch.equal(Y1, Y2) and bool((Y1[:, :, :, :, 1] != 0).any())        # the surround was written
    dz = exchanged(g, synth.normal_volume((n,) + dhw + (32,), 4, "bf16"), 32, dt)
    wsd = sp3d.alloc_ws(sp3d.sp_workspace_bytes(sp3d.SP_OP_DGRAD, g1, 64, 32, dt))
    Da, Db, Dc = (sp3d.alloc_padded(g, c, dt) for c in (32, 32, 64))
    sp3d.conv3d_dgrad2(dz, w, Da, 32, Db, 32, g1, 32, dt, wsd)
    sp3d.conv3d_dgrad(dz, w, Dc, g1, 64, 32, dt, wsd)
    assert torch.equal(torch.cat([Da, Db], dim=-1), Dc)


GLUE = [  # n, dhw (fine), grid, cin, cout, dtype, halo
    (1, (8, 8, 16), (2, 2, 1), 4, 6, "f32", 2),
    (1, (8, 16, 64), (2, 2, 1), 64, 32, "bf16", 2),      # matrix-core transposed convolution
    (1, (12, 12, 24), (1, 1, 2), 32, 32, "bf16", 3),
]


@pytest.mark.parametrize("n,dhw,grid,cin,cout,dtype,h", GLUE)
def test_glue_operations_on_a_wide_margin_layout(n, dhw, grid, cin, cout, dtype, h):
    """Pooling, transposed convolution, 1x1x1 head and loss read and write interiors only: on a wide-margin
    layout they must give the bits they give on the one-voxel layout (whose parity with the oracle the other
    tests establish)."""
    dt = DT[dtype]
    outs = []
    for halo in (1, h):
        gf = sp3d.Geom(n, dhw, grid, halo)
        gc = sp3d.Geom(n, tuple(e // 2 for e in dhw), grid, halo)
        r = []
        xf = synth.normal_volume((n,) + dhw + (cin,), 1, dtype)
        Pf = exchanged(gf, xf, cin, dt)
        Pp = sp3d.alloc_padded(gc, cin, dt)
        sp3d.sp_maxpool2_fwd(Pf, Pp, gf, cin, dt)
        r.append(volume(gc, Pp, cin, dt))
        dyc = synth.normal_volume((n,) + tuple(e // 2 for e in dhw) + (cin,), 2, dtype)
        Pdyc, Pdf = exchanged(gc, dyc, cin, dt), sp3d.alloc_padded(gf, cin, dt)
        sp3d.sp_maxpool2_bwd(Pf, Pdyc, Pdf, gf, cin, dt)
        r.append(volume(gf, Pdf, cin, dt))
        Pj = sp3d.alloc_padded(gf, cin, dt)
        sp3d.sp_maxpool2_bwd_join(Pf, Pdyc, Pdf, Pj, gf, cin, dt)          # skip gradient: any fine tensor
        r.append(volume(gf, Pj, cin, dt))
        u = to_dev(synth.weights(cin, cout, 3, dtype, taps=(2, 2, 2)))
        Pu = sp3d.alloc_padded(gf, cout, dt)
        sp3d.sp_upconv2_fwd(Pdyc, u, None, Pu, gf, cin, cout, dt)
        r.append(volume(gf, Pu, cout, dt))
        dyf = exchanged(gf, synth.normal_volume((n,) + dhw + (cout,), 4, dtype), cout, dt)
        Pdc = sp3d.alloc_padded(gc, cin, dt)
        sp3d.sp_upconv2_dgrad(dyf, u, Pdc, gf, cin, cout, dt)
        r.append(volume(gc, Pdc, cin, dt))
        du = torch.empty((2, 2, 2, cin, cout), dtype=torch.float32, device="cuda")
        sp3d.sp_upconv2_wgrad(Pdyc, dyf, du, None, gf, cin, cout, dt,
                              sp3d.alloc_ws(sp3d.sp_workspace_bytes(sp3d.SP_OP_UPCONV_WGRAD, gf, cin, cout, dt)))
        r.append(du)
        # head cin -> 3 and the loss on its logits
        p = to_dev(synth.weights(cin, 3, 5, dtype, taps=(1, 1, 1)))
        Pl = sp3d.alloc_padded(gf, 3, dt)
        sp3d.sp_pointwise_fwd(Pf, p, None, Pl, gf, cin, 3, dt)
        r.append(volume(gf, Pl, 3, dt))
        rng = np.random.default_rng(6)
        lab = rng.integers(0, 3, size=(n,) + dhw + (1,)).astype(np.float32)
        lab = synth.f32_to_bf16_bits(lab) if dtype == "bf16" else lab
        Plab, Pdl = exchanged(gf, lab, 1, dt), sp3d.alloc_padded(gf, 3, dt)
        loss = torch.zeros(1, device="cuda")
        sp3d.sp_dice_ce_loss(Pl, Plab, Pdl, loss, None, gf, 3, dt, 0.9, 0.1, 1.0,
                             sp3d.alloc_ws(sp3d.sp_workspace_bytes(sp3d.SP_OP_LOSS, gf, 3, 1, dt)))
        r.append(loss.clone())
        r.append(volume(gf, Pdl, 3, dt))
        Pdh = sp3d.alloc_padded(gf, cin, dt)
        sp3d.sp_pointwise_dgrad(Pdl, p, Pdh, gf, cin, 3, dt)
        r.append(volume(gf, Pdh, cin, dt))
        sp3d.sp_pointwise_dgrad_relu(Pdl, p, Pf, Pdh, gf, cin, 3, dt)
        r.append(volume(gf, Pdh, cin, dt))
        dp = torch.empty((1, 1, 1, cin, 3), dtype=torch.float32, device="cuda")
        sp3d.sp_pointwise_wgrad(Pf, Pdl, dp, None, gf, cin, 3, dt,
                                sp3d.alloc_ws(sp3d.sp_workspace_bytes(sp3d.SP_OP_POINTWISE_WGRAD, gf, cin, 3, dt)))
        r.append(dp)
        outs.append(r)
    for k, (one, wide) in enumerate(zip(*outs)):
        assert torch.equal(one, wide), k
