"""GPU parity of the data-movement entry points against the slicing oracle: bit-exact."""
import numpy as np
import pytest
import torch

from oracle import tiling
from paper_1909_03108_amd import sp3d
from gpu_util import DT, bits, guard_alloc, guards_intact, progress, to_dev

pytestmark = pytest.mark.gpu

CASES = [
    # n, dhw, grid, c, dtype
    (1, (32, 32, 32), (2, 2, 1), 8, "f32"),        # configuration 1 geometry
    (1, (16, 16, 64), (4, 4, 1), 32, "bf16"),      # configuration 2/4 grid, small
    (1, (8, 8, 12), (4, 4, 2), 1, "bf16"),         # configuration 3 grid, single channel (2-byte records)
    (1, (8, 8, 12), (4, 4, 2), 32, "bf16"),
    (2, (6, 4, 10), (3, 2, 5), 3, "f32"),          # 12-byte records, batch 2
    (1, (3, 2, 5), (3, 2, 5), 5, "bf16"),          # 1-voxel tiles, 10-byte records
    (1, (5, 7, 9), (1, 1, 1), 4, "bf16"),          # single tile: every margin is zero fill
    (1, (24, 40, 72), (2, 2, 1), 32, "bf16"),      # rows longer than one block pass, ragged
    (1, (4, 6, 260), (2, 3, 2), 16, "f32"),
    # narrow records whose rows are whole multiples of 16 bytes: rows copied as 16-byte pieces at 2- / 4-byte alignment
    (1, (4, 6, 64), (2, 1, 2), 1, "bf16"),         # the CT volume itself: 64-byte rows
    (1, (4, 4, 32), (1, 2, 2), 3, "bf16"),         # class logits: 6-byte records, 96-byte rows
    (2, (4, 4, 8), (2, 1, 2), 3, "f32"),           # 12-byte records, 48-byte rows
    (1, (2, 3, 520), (1, 1, 1), 3, "bf16"),        # rows longer than one pass of a block
]
# margins wider than one voxel (several layers per exchange): n, dhw, grid, c, dtype, halo
WIDE = [
    (1, (16, 16, 64), (4, 4, 1), 32, "bf16", 2),
    (1, (8, 8, 12), (4, 4, 2), 1, "bf16", 2),      # tiles exactly as thick as the margin
    (2, (6, 6, 9), (2, 1, 3), 3, "f32", 3),
    (1, (8, 12, 40), (2, 1, 1), 32, "bf16", 4),
    (1, (5, 7, 9), (1, 1, 1), 4, "bf16", 2),
    (1, (4, 4, 32), (1, 1, 2), 3, "bf16", 3),
]


def make_volume(n, dhw, c, dtype, seed):
    rng = np.random.default_rng(seed)
    if dtype == "bf16":
        return rng.integers(1, 0x7F00, size=(n,) + dhw + (c,), dtype=np.uint16)   # distinct-ish bit patterns
    return rng.standard_normal((n,) + dhw + (c,)).astype(np.float32)


@pytest.mark.parametrize("n,dhw,grid,c,dtype,h", [k + (1,) for k in CASES] + WIDE)
def test_partition_pack_unpack_unpartition_bit_exact(n, dhw, grid, c, dtype, h):
    g = sp3d.Geom(n, dhw, grid, h)
    dt = DT[dtype]
    V = make_volume(n, dhw, c, dtype, 11)
    tdt = sp3d.torch_dtype(dt)
    fill = 7.0
    fill_bits = bits(torch.tensor([fill], dtype=tdt, device="cuda"))[0]

    # partition: interiors written, margins untouched (still the fill value)
    pbuf, P = guard_alloc(g.padded_shape + (c,), tdt, fill)
    sp3d.sp_partition(to_dev(V), P, g, c, dt)
    ref_P = tiling.partition(V, grid, h)
    got = bits(P)
    inner = (slice(None),) * 4 + (slice(h, -h),) * 3
    assert np.array_equal(got[inner], ref_P[inner])
    mask = np.ones(got.shape, dtype=bool)
    mask[inner] = False
    assert np.all(got[mask] == fill_bits)
    assert guards_intact(pbuf, fill)

    # pack
    mbuf, M = guard_alloc((sp3d.sp_msg_elems(g, c),), tdt, fill)
    sp3d.halo_pack(P, M, g, c, dt)
    ref_M = tiling.halo_pack(ref_P, h)
    assert np.array_equal(bits(M).reshape(ref_M.shape), ref_M)
    assert guards_intact(mbuf, fill)

    # unpack: margins from neighbours or zero; interior untouched
    sp3d.halo_unpack(P, M, g, c, dt)
    ref_full = tiling.padded_reference(V, grid, h)
    assert np.array_equal(bits(P), ref_full)
    assert np.array_equal(tiling.halo_unpack(ref_P, ref_M, h), ref_full)
    assert guards_intact(pbuf, fill)

    # the one-pass exchange on a freshly partitioned tensor gives the same padded tiles, margins included
    qbuf, Q = guard_alloc(g.padded_shape + (c,), tdt, fill)
    sp3d.sp_partition(to_dev(V), Q, g, c, dt)
    sp3d.sp_halo_exchange(Q, g, c, dt)
    assert np.array_equal(bits(Q), ref_full)
    assert guards_intact(qbuf, fill)

    # unpartition
    vbuf, V2 = guard_alloc((n,) + dhw + (c,), tdt, fill)
    sp3d.sp_unpartition(P, V2, g, c, dt)
    assert np.array_equal(bits(V2), V)
    assert guards_intact(vbuf, fill)


@pytest.mark.parametrize("n,dhw,grid,c,dtype,h", [k + (1,) for k in CASES[:9]] + WIDE[:4])
def test_border_flags_skip_what_has_no_receiver_and_keep_zero_margins(n, dhw, grid, c, dtype, h):
    """SP_HALO_SKIP_SEND: halo_pack writes exactly the message entries some tile receives (the oracle's
    tiling.delivered) and leaves the others untouched.  SP_HALO_KEEP_ZERO: halo_unpack / sp_halo_exchange write
    exactly the margins that have a neighbour; the margins at the volume border - the positions where the
    zero-padded reference holds padding - are left as they are, so a zeroed array ends up as the full reference."""
    g0 = sp3d.Geom(n, dhw, grid, h)
    g = g0.with_opts(sp3d.SP_HALO_SKIP_SEND | sp3d.SP_HALO_KEEP_ZERO)
    dt = DT[dtype]
    tdt = sp3d.torch_dtype(dt)
    V = make_volume(n, dhw, c, dtype, 12)
    fill = 7.0
    fill_bits = bits(torch.tensor([fill], dtype=tdt, device="cuda"))[0]
    ref_P = tiling.partition(V, grid, h)
    ref_M = tiling.halo_pack(ref_P, h)
    ref_full = tiling.padded_reference(V, grid, h)
    tile = tiling.tile_extents(dhw, grid)
    deliv = np.broadcast_to(tiling.delivered(grid, tile, h)[None, ..., None], ref_M.shape)
    # positions of the padded array that lie outside the volume: where the reference of an all-ones volume is zero
    outside = tiling.padded_reference(np.ones(V.shape, dtype=np.uint8), grid, h) == 0

    pbuf, P = guard_alloc(g.padded_shape + (c,), tdt, fill)
    sp3d.sp_partition(to_dev(V), P, g, c, dt)
    mbuf, M = guard_alloc((sp3d.sp_msg_elems(g, c),), tdt, fill)
    sp3d.halo_pack(P, M, g, c, dt)
    got_M = bits(M).reshape(ref_M.shape)
    assert np.array_equal(got_M[deliv], ref_M[deliv])
    assert np.all(got_M[~deliv] == fill_bits)
    assert guards_intact(mbuf, fill)
    for one_pass in (False, True):
        if one_pass:
            P.fill_(fill)
            sp3d.sp_partition(to_dev(V), P, g, c, dt)
            sp3d.sp_halo_exchange(P, g, c, dt)
        else:
            sp3d.halo_unpack(P, M, g, c, dt)
        got = bits(P)
        assert np.array_equal(got[~outside], ref_full[~outside])
        assert np.all(got[outside] == fill_bits)
        assert guards_intact(pbuf, fill)
    # on a zeroed array the flagged calls give the complete padded tiles
    Q = sp3d.alloc_padded(g, c, dt)
    sp3d.sp_partition(to_dev(V), Q, g, c, dt)
    sp3d.sp_halo_exchange(Q, g, c, dt)
    assert np.array_equal(bits(Q), ref_full)
    # and an unknown flag is an argument error
    with pytest.raises(sp3d.Sp3dError) as e:
        sp3d.sp_halo_exchange(Q, g0.with_opts(8), c, dt)
    assert e.value.code == sp3d.SP_EINVAL


def test_relu_bwd_mask_bit_exact():
    g = sp3d.Geom(1, (6, 4, 10), (3, 2, 5))
    for dtype in ("bf16", "f32"):
        dt = DT[dtype]
        tdt = sp3d.torch_dtype(dt)
        shape = g.padded_shape + (3,)
        y = torch.randn(shape, device="cuda").clamp_min(0).to(tdt)
        y.view(-1)[::7] = -0.0
        dy = torch.randn(shape, device="cuda").to(tdt)
        dz = torch.empty_like(dy)
        sp3d.sp_relu_bwd(dy, y, dz, g, 3, dt)
        ref = torch.where(y > 0, dy, torch.zeros_like(dy))
        assert torch.equal(dz, ref)


# the geometries of the workload list's large configurations: n, dhw, grid, c
CONFIG_GEOMETRIES = [
    (1, (256, 256, 256), (4, 4, 2), 1),      # configuration 3, the CT volume (2-byte records)
    (1, (256, 256, 256), (4, 4, 2), 32),     # configuration 3, 32 channels, W split
    (1, (512, 512, 512), (4, 4, 1), 32),     # configuration 4: 128 x 128 x 512 tiles, 8.6 GB
]


@pytest.mark.timeout(1200)
@pytest.mark.parametrize("n,dhw,grid,c", CONFIG_GEOMETRIES, ids=["c3_c1", "c3_c32", "c4_c32"])
def test_index_ops_bit_exact_at_configuration_geometries(n, dhw, grid, c):
    """partition -> pack -> unpack -> unpartition and the one-pass exchange at the full extents of
    configurations 3 and 4, every element of the padded array, the message array and the reassembled volume
    against the slicing oracle, as raw bits."""
    from paper_1909_03108_amd import synth
    g = sp3d.Geom(n, dhw, grid, 1)
    dt, tdt, h = DT["bf16"], torch.bfloat16, 1
    V = synth.normal_volume((n,) + dhw + (c,), 1234, "bf16")
    fill = 7.0
    fill_bits = bits(torch.tensor([fill], dtype=tdt, device="cuda"))[0]
    Vd = to_dev(V)

    pbuf, P = guard_alloc(g.padded_shape + (c,), tdt, fill)
    sp3d.sp_partition(Vd, P, g, c, dt)
    ref_P = tiling.partition(V, grid, h)
    got = bits(P)
    inner = (slice(None),) * 4 + (slice(h, -h),) * 3
    assert np.array_equal(got[inner], ref_P[inner]), "partition: interiors"
    for ax in (4, 5, 6):            # the six margin slabs of every tile still hold the fill value
        for sl in (slice(0, h), slice(-h, None)):
            idx = [slice(None)] * 8
            idx[ax] = sl
            assert np.all(got[tuple(idx)] == fill_bits), "partition wrote a margin"
    assert guards_intact(pbuf, fill)
    del got

    mbuf, M = guard_alloc((sp3d.sp_msg_elems(g, c),), tdt, fill)
    sp3d.halo_pack(P, M, g, c, dt)
    ref_M = tiling.halo_pack(ref_P, h)
    del ref_P
    assert np.array_equal(bits(M).reshape(ref_M.shape), ref_M), "pack"
    progress("index ops %s c=%d: partition, pack ok" % (dhw, c))
    assert guards_intact(mbuf, fill)
    del ref_M

    sp3d.halo_unpack(P, M, g, c, dt)
    ref_full = tiling.padded_reference(V, grid, h)
    assert np.array_equal(bits(P), ref_full), "unpack"
    progress("index ops %s c=%d: unpack ok" % (dhw, c))
    assert guards_intact(pbuf, fill)

    vbuf, V2 = guard_alloc((n,) + dhw + (c,), tdt, fill)
    sp3d.sp_unpartition(P, V2, g, c, dt)
    assert np.array_equal(bits(V2), V), "unpartition"
    assert guards_intact(vbuf, fill)
    del vbuf, V2

    # the one-pass exchange on a freshly partitioned tensor (reusing P's memory)
    P.fill_(fill)
    sp3d.sp_partition(Vd, P, g, c, dt)
    sp3d.sp_halo_exchange(P, g, c, dt)
    assert np.array_equal(bits(P), ref_full), "one-pass exchange"
    assert guards_intact(pbuf, fill)
