"""GPU parity of the convolutions that gather their halos (geometry flag SP_HALO_GATHER): the exchange of
margins before a convolution (Fig. 1b; Sec. 2, third paragraph) fused into the convolution itself, which reads
the neighbours' voxels where the exchange would have copied them.  Every result must equal, bit for bit, the
exchange followed by the plain call, and match the fp64 oracle on the unpartitioned volume; the margins towards
neighbours are filled with NaN first to show that nothing reads them."""
import numpy as np
import pytest
import torch

from oracle import conv3d, tiling
from paper_1909_03108_amd import sp3d, synth
from gpu_util import TOL, f64, rel_err, to_dev, widen

pytestmark = pytest.mark.gpu

CASES = [
    # n, dhw, grid, cin, cout                     tiles
    (1, (8, 16, 64), (2, 2, 1), 32, 32),          # 4 x 8 x 64: whole patches, one chunk per march
    (1, (8, 16, 64), (2, 2, 2), 32, 32),          # W split as well: 4 x 8 x 32
    (1, (12, 24, 96), (3, 3, 3), 32, 64),         # tiles with neighbours on both sides, on edges and in the middle
    (1, (80, 16, 64), (2, 2, 1), 32, 32),         # 40 planes per tile: marches cut into D chunks
    (2, (8, 16, 32), (2, 1, 1), 64, 64),          # batch 2; pairs of input chunks summed on chip
    (1, (6, 16, 64), (1, 2, 2), 128, 64),         # two pairs per layer: partial sums between launches
    (1, (8, 8, 64), (2, 1, 2), 96, 32),           # three single chunks (first / middle / last)
    (1, (12, 20, 72), (2, 2, 1), 32, 32),         # ragged patches: forward and data gradient only
]


def margin_masks(g, dhw, grid, c):
    """(towards a neighbour, beyond the volume) as boolean arrays over the padded tensor"""
    ones = np.ones((g.n,) + dhw + (c,), dtype=np.uint8)
    ref = tiling.padded_reference(ones, grid, 1)
    outside = ref == 0
    interior = np.zeros_like(outside)
    interior[(slice(None),) * 4 + (slice(1, -1),) * 3] = True
    return ~outside & ~interior, outside


@pytest.mark.parametrize("n,dhw,grid,cin,cout", CASES)
def test_gathered_halos_equal_exchange_then_convolve(n, dhw, grid, cin, cout):
    g = sp3d.Geom(n, dhw, grid)
    gg = g.with_opts(sp3d.SP_HALO_GATHER)
    dt, tol = sp3d.SP_BF16, TOL["bf16"]
    x = synth.normal_volume((n,) + dhw + (cin,), 21, "bf16")
    dz = synth.normal_volume((n,) + dhw + (cout,), 22, "bf16")
    xmask = synth.normal_volume((n,) + dhw + (cin,), 23, "bf16")
    w = synth.weights(cin, cout, 24, "bf16")
    bias = np.linspace(-0.5, 0.5, cout).astype(np.float32)
    w_d, b_d = to_dev(w), torch.from_numpy(bias).cuda()
    ws = {op: sp3d.alloc_ws(sp3d.sp_workspace_bytes(op, g, cin, cout, dt)) for op in (0, 1, 2)}

    def both(V, c):
        """(partitioned + exchanged, partitioned with NaN in every margin that has a neighbour)"""
        Pe, Pg = sp3d.alloc_padded(g, c, dt), sp3d.alloc_padded(g, c, dt)
        for P in (Pe, Pg):
            sp3d.sp_partition(to_dev(V), P, g, c, dt)
        sp3d.sp_halo_exchange(Pe, g, c, dt)
        towards, _ = margin_masks(g, dhw, grid, c)
        Pg[torch.from_numpy(towards).cuda()] = float("nan")
        return Pe, Pg

    Xe, Xg = both(x, cin)
    Ze, Zg = both(dz, cout)
    whole = g.tile[1] % 8 == 0 and g.tile[2] % 32 == 0

    # forward, bias + ReLU
    Ye, Yg = sp3d.alloc_padded(g, cout, dt), sp3d.alloc_padded(g, cout, dt)
    sp3d.conv3d_fwd(Xe, w_d, b_d, Ye, g, cin, cout, dt, sp3d.SP_FLAG_RELU, ws[0])
    sp3d.conv3d_fwd(Xg, w_d, b_d, Yg, gg, cin, cout, dt, sp3d.SP_FLAG_RELU, ws[0])
    assert torch.equal(Ye, Yg)
    V = torch.empty((n,) + dhw + (cout,), dtype=torch.bfloat16, device="cuda")
    sp3d.sp_unpartition(Yg, V, g, cout, dt)
    assert rel_err(f64(V), conv3d.conv3d_fwd(x, widen(w), bias.astype(np.float64), relu=True)) <= tol
    # data gradient, plain and with the ReLU mask of the layer input
    De, Dg = sp3d.alloc_padded(g, cin, dt), sp3d.alloc_padded(g, cin, dt)
    sp3d.conv3d_dgrad(Ze, w_d, De, g, cin, cout, dt, ws[1])
    sp3d.conv3d_dgrad(Zg, w_d, Dg, gg, cin, cout, dt, ws[1])
    assert torch.equal(De, Dg)
    Pm = sp3d.alloc_padded(g, cin, dt)
    sp3d.sp_partition(to_dev(xmask), Pm, g, cin, dt)
    sp3d.conv3d_dgrad_relu(Ze, w_d, Pm, De, g, cin, cout, dt, ws[1])
    sp3d.conv3d_dgrad_relu(Zg, w_d, Pm, Dg, gg, cin, cout, dt, ws[1])
    assert torch.equal(De, Dg)
    # weight and bias gradient (whole patches only: the flag is refused otherwise)
    dwe = torch.full((3, 3, 3, cin, cout), 1.0, dtype=torch.float32, device="cuda")
    dbe = torch.full((cout,), 1.0, dtype=torch.float32, device="cuda")
    dwg, dbg = torch.full_like(dwe, 2.0), torch.full_like(dbe, 2.0)
    if whole:
        sp3d.conv3d_wgrad(Xe, Ze, dwe, dbe, g, cin, cout, dt, ws[2])
        sp3d.conv3d_wgrad(Xg, Zg, dwg, dbg, gg, cin, cout, dt, ws[2])
        assert torch.equal(dwe, dwg) and torch.equal(dbe, dbg)
        assert rel_err(f64(dwg), conv3d.conv3d_wgrad(x, dz)) <= tol
    else:
        with pytest.raises(sp3d.Sp3dError) as e:
            sp3d.conv3d_wgrad(Xg, Zg, dwg, dbg, gg, cin, cout, dt, ws[2])
        assert e.value.code == sp3d.SP_EUNSUPPORTED
    # the inputs were only read
    towards, _ = margin_masks(g, dhw, grid, cin)
    assert bool(torch.isnan(Xg[torch.from_numpy(towards).cuda()].float()).all())


def test_gathered_halos_two_tensor_forms():
    n, dhw, grid, ca, cb, cout = 1, (8, 16, 64), (2, 2, 2), 32, 32, 64
    g = sp3d.Geom(n, dhw, grid)
    gg = g.with_opts(sp3d.SP_HALO_GATHER)
    dt = sp3d.SP_BF16
    xa = synth.normal_volume((n,) + dhw + (ca,), 31, "bf16")
    xb = synth.normal_volume((n,) + dhw + (cb,), 32, "bf16")
    dz = synth.normal_volume((n,) + dhw + (cout,), 33, "bf16")
    w_d = to_dev(synth.weights(ca + cb, cout, 34, "bf16"))
    ws = {op: sp3d.alloc_ws(sp3d.sp_workspace_bytes(op, g, ca + cb, cout, dt)) for op in (0, 1, 2)}

    def part(V, c, exchange):
        P = sp3d.alloc_padded(g, c, dt)
        sp3d.sp_partition(to_dev(V), P, g, c, dt)
        if exchange:
            sp3d.sp_halo_exchange(P, g, c, dt)
        return P

    Ae, Be, Ze = part(xa, ca, True), part(xb, cb, True), part(dz, cout, True)
    Ag, Bg, Zg = part(xa, ca, False), part(xb, cb, False), part(dz, cout, False)
    Ye, Yg = sp3d.alloc_padded(g, cout, dt), sp3d.alloc_padded(g, cout, dt)
    sp3d.conv3d_fwd2(Ae, ca, Be, cb, w_d, None, Ye, g, cout, dt, sp3d.SP_FLAG_RELU, ws[0])
    sp3d.conv3d_fwd2(Ag, ca, Bg, cb, w_d, None, Yg, gg, cout, dt, sp3d.SP_FLAG_RELU, ws[0])
    assert torch.equal(Ye, Yg)
    outs = []
    for Z, geo in ((Ze, g), (Zg, gg)):
        Da, Db = sp3d.alloc_padded(g, ca, dt), sp3d.alloc_padded(g, cb, dt)
        sp3d.conv3d_dgrad2(Z, w_d, Da, ca, Db, cb, geo, cout, dt, ws[1])
        dw = torch.empty((3, 3, 3, ca + cb, cout), dtype=torch.float32, device="cuda")
        db = torch.empty((cout,), dtype=torch.float32, device="cuda")
        A, B = (Ae, Be) if geo is g else (Ag, Bg)
        sp3d.conv3d_wgrad2(A, ca, B, cb, Z, dw, db, geo, cout, dt, ws[2])
        outs.append((Da, Db, dw, db))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_gather_flag_is_refused_where_no_kernel_gathers():
    dt = sp3d.SP_BF16
    for geo, cin, cout in [(sp3d.Geom(1, (8, 16, 64), (2, 2, 1), halo=2), 32, 32),        # wide margins
                           (sp3d.Geom(1, (8, 16, 64), (2, 2, 1), flat=1), 32, 32),        # 2-D variant
                           (sp3d.Geom(1, (8, 16, 64), (2, 2, 1)), 1, 32),                 # first layer
                           (sp3d.Geom(1, (8, 16, 64), (2, 2, 1)), 8, 16)]:                # odd channel counts
        g = geo.with_opts(sp3d.SP_HALO_GATHER)
        Px, Py = sp3d.alloc_padded(g, cin, dt), sp3d.alloc_padded(g, cout, dt)
        taps = (3, 3) if g.flat else (3, 3, 3)
        w = to_dev(synth.weights(cin, cout, 1, "bf16", taps=taps))
        ws = sp3d.alloc_ws(1 << 20)
        with pytest.raises(sp3d.Sp3dError) as e:
            sp3d.conv3d_fwd(Px, w, None, Py, g, cin, cout, dt, 0, ws)
        assert e.value.code == sp3d.SP_EUNSUPPORTED
