"""Host-side checks of the C-ABI library (no GPU needed): it loads, exports every symbol the
header declares, sizes agree with the slicing oracle, and bad arguments are rejected before
anything is launched."""
import ctypes
import os
import re

import pytest

from oracle import tiling
from paper_1909_03108_amd import sp3d

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000   # non-null, 16-byte aligned; never dereferenced because every call below fails validation


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sp3d.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\([^;{}]*\)\s*;", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = sp3d.lib()
    names = declared_functions()
    assert len(names) >= 14
    for n in names:
        assert hasattr(L, n), n
    assert sorted(sp3d.EXPORTS) == names


@pytest.mark.parametrize("n,dhw,grid,c", [(1, (32, 32, 32), (2, 2, 1), 8), (1, (128, 128, 128), (4, 4, 1), 32),
                                          (1, (256, 256, 256), (4, 4, 2), 1), (2, (6, 4, 8), (3, 2, 4), 5),
                                          (1, (512, 512, 512), (4, 4, 1), 32)])
def test_size_helpers_match_the_oracle_formulas(n, dhw, grid, c):
    g = sp3d.Geom(n, dhw, grid)
    tile = tiling.tile_extents(dhw, grid)
    ntiles = n * grid[0] * grid[1] * grid[2]
    assert sp3d.sp_msg_elems(g, c) == ntiles * tiling.margin_voxels(tile, 1) * c
    assert sp3d.sp_padded_elems(g, c) == ntiles * (tile[0] + 2) * (tile[1] + 2) * (tile[2] + 2) * c
    assert g.padded_shape == (n,) + grid + tuple(t + 2 for t in tile)


def test_margin_voxel_counts_of_the_workload_configurations():
    # per-tile margin voxels for the 16x16x32, 32x32x128, 64x64x128 and 128x128x512 tiles
    for dhw, grid, expect in [((32, 32, 32), (2, 2, 1), 2824), ((128, 128, 128), (4, 4, 1), 19208),
                              ((256, 256, 256), (4, 4, 2), 41992), ((512, 512, 512), (4, 4, 1), 297992)]:
        g = sp3d.Geom(1, dhw, grid)
        assert sp3d.sp_msg_elems(g, 1) == expect * grid[0] * grid[1] * grid[2]


def test_geometry_errors():
    assert sp3d.sp_check_geom(sp3d.Geom(1, (8, 8, 8), (2, 2, 2))) == sp3d.SP_OK
    assert sp3d.sp_check_geom(sp3d.Geom(1, (8, 8, 8), (3, 2, 2))) == sp3d.SP_EGEOM
    assert sp3d.sp_check_geom(sp3d.Geom(1, (8, 8, 8), (2, 2, 2), halo=2)) == sp3d.SP_OK
    assert sp3d.sp_check_geom(sp3d.Geom(1, (8, 8, 8), (2, 2, 2), halo=4)) == sp3d.SP_OK
    assert sp3d.sp_check_geom(sp3d.Geom(1, (8, 8, 8), (2, 2, 2), halo=5)) == sp3d.SP_EUNSUPPORTED
    assert sp3d.sp_check_geom(sp3d.Geom(1, (8, 8, 8), (2, 2, 2), halo=0)) == sp3d.SP_EUNSUPPORTED
    assert sp3d.sp_check_geom(sp3d.Geom(1, (8, 8, 8), (2, 2, 2), halo=-1)) == sp3d.SP_EINVAL
    assert sp3d.sp_check_geom(sp3d.Geom(1, (8, 8, 8), (4, 2, 2), halo=3)) == sp3d.SP_EGEOM     # 2-voxel tiles, 3-wide margin
    # grow: the convolutions' output box may grow by less than the margin width
    assert sp3d.sp_check_geom(sp3d.Geom(1, (8, 8, 8), (2, 2, 2), halo=2, grow=1)) == sp3d.SP_OK
    assert sp3d.sp_check_geom(sp3d.Geom(1, (8, 8, 8), (2, 2, 2), halo=2, grow=2)) == sp3d.SP_EINVAL
    assert sp3d.sp_check_geom(sp3d.Geom(1, (8, 8, 8), (2, 2, 2), halo=1, grow=1)) == sp3d.SP_EINVAL
    assert sp3d.sp_check_geom(sp3d.Geom(1, (8, 8, 8), (2, 2, 2), grow=-1)) == sp3d.SP_EINVAL
    g2 = sp3d.Geom(1, (8, 8, 8), (2, 2, 2), halo=2)
    assert sp3d.sp_padded_elems(g2, 3) == 8 * 8 * 8 * 8 * 3 and g2.padded_shape == (1, 2, 2, 2, 8, 8, 8)
    assert sp3d.sp_msg_elems(g2, 1) == 8 * (8 * 8 * 8 - 4 * 4 * 4)
    assert g2.grown(1).grow == 1 and g2.grown(1).halo == 2
    assert sp3d.sp_check_geom(sp3d.Geom(0, (8, 8, 8), (2, 2, 2))) == sp3d.SP_EINVAL
    assert sp3d.sp_check_geom(sp3d.Geom(1, (8, 8, 8), (2, 0, 2))) == sp3d.SP_EINVAL
    assert sp3d.sp_check_geom(sp3d.Geom(1, (2, 2, 2), (2, 2, 2))) == sp3d.SP_OK     # 1-voxel tiles are legal
    assert sp3d.sp_padded_elems(sp3d.Geom(1, (8, 8, 8), (3, 2, 2)), 4) == 0


def test_flat_geometry_of_the_2d_variant():
    """flat = 1: D is a stack of slices.  The layout is unchanged, a tile may hold fewer slices than the margin is
    wide, only H and W must be even for pooling, and the workspaces are sized for 9 taps / 4 window positions."""
    flat = sp3d.Geom(1, (3, 16, 64), (1, 2, 2), flat=1)
    full = sp3d.Geom(1, (3, 16, 64), (1, 2, 2))
    assert sp3d.sp_check_geom(flat) == sp3d.SP_OK
    assert sp3d.sp_padded_elems(flat, 4) == sp3d.sp_padded_elems(full, 4)
    assert sp3d.sp_msg_elems(flat, 4) == sp3d.sp_msg_elems(full, 4)
    assert flat.grown(0).flat == 1
    bad = sp3d.Geom(1, (3, 16, 64), (1, 2, 2))
    bad.flat = 2
    assert sp3d.sp_check_geom(bad) == sp3d.SP_EINVAL
    assert sp3d.sp_check_geom(sp3d.Geom(1, (2, 16, 64), (2, 2, 2), halo=2, flat=1)) == sp3d.SP_OK     # 1 slice per tile
    assert sp3d.sp_check_geom(sp3d.Geom(1, (2, 16, 64), (2, 2, 2), halo=2)) == sp3d.SP_EGEOM
    assert sp3d.sp_check_geom(sp3d.Geom(1, (4, 2, 64), (1, 2, 2), halo=2, flat=1)) == sp3d.SP_EGEOM    # 1-voxel rows
    gc = sp3d.coarse_geom(flat)
    assert (gc.d, gc.h, gc.w, gc.flat) == (3, 8, 32, 1)
    dt = sp3d.SP_BF16
    # odd slice count: fine for the 1x2x2 windows, not for the 2x2x2 ones
    assert sp3d.sp_workspace_bytes(sp3d.SP_OP_UPCONV_WGRAD, flat, 64, 32, dt) > 0
    with pytest.raises(sp3d.Sp3dError):
        sp3d.sp_workspace_bytes(sp3d.SP_OP_UPCONV_WGRAD, full, 64, 32, dt)
    even_f, even = sp3d.Geom(1, (4, 16, 64), (1, 2, 2), flat=1), sp3d.Geom(1, (4, 16, 64), (1, 2, 2))
    for op, ci, co in [(sp3d.SP_OP_WGRAD, 32, 32), (sp3d.SP_OP_WGRAD, 5, 8)]:
        assert 0 < sp3d.sp_workspace_bytes(op, even_f, ci, co, dt) < sp3d.sp_workspace_bytes(op, even, ci, co, dt)
    assert sp3d.sp_workspace_bytes(sp3d.SP_OP_FWD, even_f, 64, 64, dt) == sp3d.sp_workspace_bytes(
        sp3d.SP_OP_FWD, even, 64, 64, dt)


def test_calls_reject_bad_arguments_before_launching():
    L = sp3d.lib()
    g = sp3d.Geom(1, (8, 8, 8), (2, 2, 2))
    bad = sp3d.Geom(1, (8, 8, 8), (3, 2, 2))
    gp, bp = ctypes.byref(g), ctypes.byref(bad)
    assert L.sp_partition(None, FAKE, gp, 4, sp3d.SP_BF16, None) == sp3d.SP_EINVAL
    assert L.sp_partition(FAKE, FAKE + 8, gp, 4, sp3d.SP_BF16, None) == sp3d.SP_EINVAL      # misaligned
    assert L.sp_partition(FAKE, FAKE, gp, 4, sp3d.SP_BF16, None) == sp3d.SP_EINVAL          # overlap
    assert L.sp_partition(FAKE, FAKE * 16, bp, 4, sp3d.SP_BF16, None) == sp3d.SP_EGEOM
    assert L.sp_unpartition(FAKE, FAKE * 16, gp, 0, sp3d.SP_BF16, None) == sp3d.SP_EINVAL
    assert L.halo_pack(FAKE, FAKE * 16, gp, 4, 7, None) == sp3d.SP_EUNSUPPORTED
    assert L.halo_unpack(FAKE, None, gp, 4, sp3d.SP_BF16, None) == sp3d.SP_EINVAL
    assert L.sp_halo_exchange(None, gp, 4, sp3d.SP_BF16, None) == sp3d.SP_EINVAL
    assert L.sp_halo_exchange(FAKE, bp, 4, sp3d.SP_BF16, None) == sp3d.SP_EGEOM
    assert L.sp_halo_exchange(FAKE + 4, gp, 4, sp3d.SP_BF16, None) == sp3d.SP_EINVAL
    assert L.conv3d_fwd(FAKE, FAKE * 2, None, FAKE * 16, bp, 4, 4, sp3d.SP_F32, 0, None, 0, None) == sp3d.SP_EGEOM
    assert L.conv3d_fwd(FAKE, FAKE * 2, None, FAKE * 16, gp, 4, 4, sp3d.SP_F32, 2, None, 0, None) == sp3d.SP_EINVAL
    assert L.conv3d_fwd(FAKE, FAKE * 2, None, FAKE, gp, 4, 4, sp3d.SP_F32, 0, None, 0, None) == sp3d.SP_EINVAL
    assert L.conv3d_dgrad(FAKE, None, FAKE * 16, gp, 4, 4, sp3d.SP_F32, None, 0, None) == sp3d.SP_EINVAL
    assert L.conv3d_dgrad(FAKE, FAKE * 2, FAKE * 16, gp, -1, 4, sp3d.SP_F32, None, 0, None) == sp3d.SP_EINVAL
    assert L.conv3d_dgrad_relu(FAKE, FAKE * 2, None, FAKE * 16, gp, 4, 4, sp3d.SP_F32, None, 0, None) == sp3d.SP_EINVAL
    assert L.conv3d_dgrad_relu(FAKE, FAKE * 2, FAKE * 16, FAKE * 16, gp, 4, 4, sp3d.SP_F32, None, 0, None) == sp3d.SP_EINVAL
    # weight gradient always needs scratch for its fixed-order reduction
    need = sp3d.sp_workspace_bytes(sp3d.SP_OP_WGRAD, g, 4, 4, sp3d.SP_F32)
    assert need > 0
    assert L.conv3d_wgrad(FAKE, FAKE * 2, FAKE * 4, None, gp, 4, 4, sp3d.SP_F32, None, 0, None) == sp3d.SP_EWORKSPACE
    assert L.conv3d_wgrad(FAKE, FAKE * 2, FAKE * 4, None, gp, 4, 4, sp3d.SP_F32, FAKE * 8, need - 1, None) == sp3d.SP_EWORKSPACE
    assert L.sp_relu_bwd(FAKE, FAKE, None, gp, 4, sp3d.SP_F32, None) == sp3d.SP_EINVAL
    assert L.sp_workspace_bytes(9, gp, 4, 4, sp3d.SP_F32) == ctypes.c_size_t(-1).value
    assert L.sp_workspace_bytes(sp3d.SP_OP_FWD, bp, 4, 4, sp3d.SP_F32) == ctypes.c_size_t(-1).value


def test_few_channel_layers_ask_for_their_padded_copies():
    """bf16 layers with Cin not a multiple of 32 (Cout a multiple) run on zero-padded copies held in the workspace:
    the size helper says so and the calls refuse a missing or short workspace before anything is launched."""
    L = sp3d.lib()
    far = FAKE * 4096
    for g in (sp3d.Geom(1, (8, 8, 32), (2, 2, 1)), sp3d.Geom(1, (3, 8, 32), (1, 2, 1), flat=1)):
        gp = ctypes.byref(g)
        padded32 = sp3d.sp_padded_elems(g, 32) * 2
        for op in (sp3d.SP_OP_FWD, sp3d.SP_OP_WGRAD):
            need = sp3d.sp_workspace_bytes(op, g, 5, 32, sp3d.SP_BF16)
            assert need >= padded32 + sp3d.sp_workspace_bytes(op, g, 32, 32, sp3d.SP_BF16)
            assert need > sp3d.sp_workspace_bytes(op, g, 5, 24, sp3d.SP_BF16)          # Cout 24: the plain kernels
        assert sp3d.sp_workspace_bytes(sp3d.SP_OP_FWD, g, 5, 32, sp3d.SP_F32) == 0
        need = sp3d.sp_workspace_bytes(sp3d.SP_OP_FWD, g, 5, 32, sp3d.SP_BF16)
        assert L.conv3d_fwd(FAKE, FAKE * 2, None, far, gp, 5, 32, sp3d.SP_BF16, 0, None, 0, None) == sp3d.SP_EWORKSPACE
        assert L.conv3d_fwd(FAKE, FAKE * 2, None, far, gp, 5, 32, sp3d.SP_BF16, 0, far * 2, need - 1, None) == sp3d.SP_EWORKSPACE
        need = sp3d.sp_workspace_bytes(sp3d.SP_OP_WGRAD, g, 5, 32, sp3d.SP_BF16)
        assert L.conv3d_wgrad(FAKE, far, far * 2, None, gp, 5, 32, sp3d.SP_BF16, far * 4, need - 1, None) == sp3d.SP_EWORKSPACE


def test_error_strings():
    L = sp3d.lib()
    seen = {L.sp_strerror(c) for c in range(-5, 1)}
    assert len(seen) == 6 and all(s for s in seen)
    assert L.sp_last_hip_error() == 0


def test_glue_calls_reject_bad_arguments_before_launching():
    L = sp3d.lib()
    g = sp3d.Geom(1, (8, 8, 8), (2, 2, 2))
    odd = sp3d.Geom(1, (6, 8, 8), (2, 2, 2))            # tile depth 3: cannot be pooled
    gp, op = ctypes.byref(g), ctypes.byref(odd)
    A, B, C = FAKE, FAKE * 2, FAKE * 4
    assert L.sp_maxpool2_fwd(A, None, gp, 4, sp3d.SP_BF16, None) == sp3d.SP_EINVAL
    assert L.sp_maxpool2_fwd(A, B, op, 4, sp3d.SP_BF16, None) == sp3d.SP_EGEOM
    assert L.sp_maxpool2_bwd(A, B, C + 4, gp, 4, sp3d.SP_BF16, None) == sp3d.SP_EINVAL     # misaligned
    far = FAKE * 64
    assert L.sp_maxpool2_bwd_join(A, B, None, far, gp, 4, sp3d.SP_BF16, None) == sp3d.SP_EINVAL      # no skip gradient
    assert L.sp_maxpool2_bwd_join(A, B, far, A, gp, 4, sp3d.SP_BF16, None) == sp3d.SP_EINVAL         # output over the input
    assert L.sp_maxpool2_bwd_join(A, B, far + 16, far, gp, 4, sp3d.SP_BF16, None) == sp3d.SP_EINVAL  # skip overlaps, not equal
    assert L.sp_maxpool2_bwd_join(A, B, far, far, op, 4, sp3d.SP_BF16, None) == sp3d.SP_EGEOM
    assert L.sp_upconv2_fwd(A, B, None, C, op, 8, 4, sp3d.SP_BF16, None) == sp3d.SP_EGEOM
    assert L.sp_upconv2_fwd(A, B, None, C, gp, 0, 4, sp3d.SP_BF16, None) == sp3d.SP_EINVAL
    assert L.sp_upconv2_dgrad(A, B, C, gp, 8, 4, 9, None) == sp3d.SP_EUNSUPPORTED
    need = sp3d.sp_workspace_bytes(sp3d.SP_OP_UPCONV_WGRAD, g, 8, 4, sp3d.SP_BF16)
    assert need > 0
    assert L.sp_upconv2_wgrad(A, B, C, None, gp, 8, 4, sp3d.SP_BF16, None, 0, None) == sp3d.SP_EWORKSPACE
    assert L.sp_upconv2_wgrad(A, B, C, None, gp, 8, 4, sp3d.SP_BF16, FAKE * 8, need - 1, None) == sp3d.SP_EWORKSPACE
    assert L.sp_pointwise_fwd(A, B, None, C, gp, 8, 3, sp3d.SP_BF16, 4, None) == sp3d.SP_EINVAL         # bad flag
    assert L.sp_pointwise_dgrad(A, None, C, gp, 8, 3, sp3d.SP_BF16, None) == sp3d.SP_EINVAL
    assert L.sp_pointwise_dgrad_relu(A, B, None, far, gp, 8, 3, sp3d.SP_BF16, None) == sp3d.SP_EINVAL
    assert L.sp_pointwise_dgrad_relu(A, B, far, far, gp, 8, 3, sp3d.SP_BF16, None) == sp3d.SP_EINVAL   # mask over the output
    needp = sp3d.sp_workspace_bytes(sp3d.SP_OP_POINTWISE_WGRAD, g, 8, 3, sp3d.SP_BF16)
    assert L.sp_pointwise_wgrad(A, B, C, None, gp, 8, 3, sp3d.SP_BF16, FAKE * 8, needp - 1, None) == sp3d.SP_EWORKSPACE
    assert L.sp_concat(A, 4, B, 0, C, gp, sp3d.SP_BF16, None) == sp3d.SP_EINVAL
    assert L.sp_split(A, B, 4, None, 4, gp, sp3d.SP_BF16, None) == sp3d.SP_EINVAL
    assert L.sp_add(A, B, None, gp, 4, sp3d.SP_BF16, None) == sp3d.SP_EINVAL
    assert L.sp_workspace_bytes(sp3d.SP_OP_UPCONV_WGRAD, op, 8, 4, sp3d.SP_BF16) == ctypes.c_size_t(-1).value


def test_workspace_sizes_of_the_kernel_families():
    """Which kernel family a call will use is visible through its workspace size (host logic only)."""
    g = sp3d.Geom(1, (128, 128, 128), (4, 4, 1))
    frag = 27 * 2 * 64 * 16                                    # packed weight fragments of one 32x32 pair
    assert sp3d.sp_workspace_bytes(sp3d.SP_OP_FWD, g, 32, 32, sp3d.SP_BF16) == frag
    assert sp3d.sp_workspace_bytes(sp3d.SP_OP_FWD, g, 32, 64, sp3d.SP_BF16) == 2 * frag      # one input chunk: no partials
    # fp32 partial sums between the launches of a layer: one value per output element of the patches that cover the
    # tiles (here whole patches: the 128^3 interior voxels), 64 output channels
    partial64 = 4 * 128 ** 3 * 64
    assert sp3d.sp_workspace_bytes(sp3d.SP_OP_FWD, g, 64, 64, sp3d.SP_BF16) == 4 * frag              # one pair of chunks
    assert sp3d.sp_workspace_bytes(sp3d.SP_OP_FWD, g, 96, 64, sp3d.SP_BF16) == 6 * frag + partial64   # three launches
    assert sp3d.sp_workspace_bytes(sp3d.SP_OP_FWD, g, 128, 64, sp3d.SP_BF16) == 8 * frag + partial64  # two pairs
    # ragged tiles: patches of 8 x 32 (one chunk per launch) or 4 x 32 (pairs) voxels are stored whole
    r = sp3d.Geom(1, (4, 10, 40), (1, 1, 1))
    assert sp3d.sp_workspace_bytes(sp3d.SP_OP_FWD, r, 96, 32, sp3d.SP_BF16) == 3 * frag + 4 * 4 * 16 * 64 * 32
    assert sp3d.sp_workspace_bytes(sp3d.SP_OP_FWD, r, 128, 32, sp3d.SP_BF16) == 4 * frag + 4 * 4 * 12 * 64 * 32
    assert sp3d.sp_workspace_bytes(sp3d.SP_OP_DGRAD, g, 32, 64, sp3d.SP_BF16) == 2 * frag           # the kernel's input is dz
    assert sp3d.sp_workspace_bytes(sp3d.SP_OP_FWD, g, 1, 32, sp3d.SP_BF16) == 0               # first-layer kernel
    assert sp3d.sp_workspace_bytes(sp3d.SP_OP_FWD, g, 8, 16, sp3d.SP_F32) == 0                # direct kernel
    for cin, cout in ((32, 32), (64, 128), (1, 32), (3, 5)):
        assert sp3d.sp_workspace_bytes(sp3d.SP_OP_WGRAD, g, cin, cout, sp3d.SP_BF16) > 0


def test_loss_call_rejects_bad_arguments_before_launching():
    L = sp3d.lib()
    g = sp3d.Geom(1, (8, 8, 8), (2, 2, 2))
    gp = ctypes.byref(g)
    need = sp3d.sp_workspace_bytes(sp3d.SP_OP_LOSS, g, 3, 1, sp3d.SP_BF16)
    assert 0 < need < 1 << 20
    A, B, C, W = FAKE, FAKE * 2, FAKE * 4, FAKE * 8
    f = L.sp_dice_ce_loss
    assert f(A, None, C, None, None, gp, 3, sp3d.SP_BF16, 0.9, 0.1, 1.0, W, need, None) == sp3d.SP_EINVAL
    assert f(A, B, None, None, None, gp, 3, sp3d.SP_BF16, 0.9, 0.1, 1.0, W, need, None) == sp3d.SP_EINVAL   # no output
    assert f(A, B, C, None, None, gp, 1, sp3d.SP_BF16, 0.9, 0.1, 1.0, W, need, None) == sp3d.SP_EINVAL
    assert f(A, B, C, None, None, gp, 5, sp3d.SP_BF16, 0.9, 0.1, 1.0, W, need, None) == sp3d.SP_EUNSUPPORTED
    assert f(A, B, C, None, None, gp, 3, sp3d.SP_BF16, -1.0, 0.1, 1.0, W, need, None) == sp3d.SP_EINVAL
    assert f(A, B, C, None, None, gp, 3, sp3d.SP_BF16, 0.9, 0.1, 1.0, W, need - 1, None) == sp3d.SP_EWORKSPACE
    assert f(A, B, C, FAKE + 2, None, gp, 3, sp3d.SP_BF16, 0.9, 0.1, 1.0, W, need, None) == sp3d.SP_EINVAL


def test_geometry_limits():
    # per-tile voxel indices must stay 32-bit
    assert sp3d.sp_check_geom(sp3d.Geom(1, (2048, 2048, 2048), (1, 1, 1))) == sp3d.SP_EGEOM
    assert sp3d.sp_check_geom(sp3d.Geom(1, (2048, 2048, 2048), (2, 2, 2))) == sp3d.SP_OK
    assert sp3d.sp_check_geom(sp3d.Geom(1, (7, 8, 8), (7, 1, 1))) == sp3d.SP_OK


@pytest.mark.timeout(30)
def test_halo_options_and_the_one_tile_grid():
    """sp_geom_t.opts: unknown bits are an argument error; on a grid of one tile every direction leads beyond the
    volume border, so with SP_HALO_SKIP_SEND / SP_HALO_KEEP_ZERO the halo calls have nothing to do and return
    without a launch (checked here without a GPU: a launch would fail); SP_HALO_GATHER is refused where no kernel
    gathers, and sp_gather_supported says so beforehand."""
    L = sp3d.lib()
    one = sp3d.Geom(1, (5, 7, 9), (1, 1, 1), opts=sp3d.SP_HALO_SKIP_SEND | sp3d.SP_HALO_KEEP_ZERO)
    for c, dt in ((4, sp3d.SP_BF16), (3, sp3d.SP_F32), (32, sp3d.SP_BF16)):
        assert L.halo_pack(FAKE, FAKE * 16, ctypes.byref(one), c, dt, None) == sp3d.SP_OK
        assert L.halo_unpack(FAKE, FAKE * 16, ctypes.byref(one), c, dt, None) == sp3d.SP_OK
        assert L.sp_halo_exchange(FAKE, ctypes.byref(one), c, dt, None) == sp3d.SP_OK
    assert sp3d.sp_check_geom(sp3d.Geom(1, (8, 8, 8), (2, 2, 2), opts=8)) == sp3d.SP_EINVAL
    assert sp3d.sp_check_geom(sp3d.Geom(1, (8, 8, 8), (2, 2, 2), opts=7)) == sp3d.SP_OK
    bf = sp3d.SP_BF16
    g = sp3d.Geom(1, (8, 16, 64), (2, 2, 1))
    assert all(sp3d.sp_gather_supported(op, g, 32, 64, bf) for op in (0, 1, 2))
    assert sp3d.sp_gather_supported(sp3d.SP_OP_FWD, sp3d.Geom(1, (12, 20, 72), (2, 2, 1)), 32, 32, bf)       # ragged patches
    assert not sp3d.sp_gather_supported(sp3d.SP_OP_WGRAD, sp3d.Geom(1, (12, 20, 72), (2, 2, 1)), 32, 32, bf)
    assert not sp3d.sp_gather_supported(sp3d.SP_OP_FWD, g, 1, 32, bf)                 # first layer
    assert not sp3d.sp_gather_supported(sp3d.SP_OP_FWD, g, 32, 32, sp3d.SP_F32)
    assert not sp3d.sp_gather_supported(sp3d.SP_OP_FWD, sp3d.Geom(1, (8, 16, 64), (2, 2, 1), halo=2), 32, 32, bf)
    assert not sp3d.sp_gather_supported(sp3d.SP_OP_FWD, sp3d.Geom(1, (8, 16, 64), (2, 2, 1), flat=1), 32, 32, bf)
    gg = g.with_opts(sp3d.SP_HALO_GATHER)
    assert L.conv3d_fwd(FAKE, FAKE * 2, None, FAKE * 16, ctypes.byref(gg), 1, 32, bf, 0, FAKE * 32, 1 << 20, None) == sp3d.SP_EUNSUPPORTED
    assert L.conv3d_wgrad(FAKE, FAKE * 2, FAKE * 4, None, ctypes.byref(sp3d.Geom(1, (12, 20, 72), (2, 2, 1), opts=4)),
                          32, 32, bf, FAKE * 32, 1 << 30, None) == sp3d.SP_EUNSUPPORTED


@pytest.mark.timeout(30)
def test_one_bit_relu_mask_arguments():
    """The bit form of the ReLU mask: size helper, the query, and every argument error of the calls that write or
    read it (all raised before any launch)."""
    L = sp3d.lib()
    bf = sp3d.SP_BF16
    g = sp3d.Geom(1, (8, 16, 64), (2, 2, 1))
    gp = ctypes.byref(g)
    assert sp3d.sp_relu_bits_bytes(g, 64) == sp3d.sp_padded_elems(g, 64) // 8
    assert sp3d.sp_relu_bits_bytes(g, 48) == 0 and sp3d.sp_relu_bits_bytes(g, 0) == 0
    assert sp3d.sp_relu_bits_supported(sp3d.SP_OP_FWD, g, 32, 64, bf)
    assert sp3d.sp_relu_bits_supported(sp3d.SP_OP_DGRAD, g, 32, 64, bf)
    assert sp3d.sp_relu_bits_supported(sp3d.SP_OP_FWD, g, 1, 32, bf)                   # the first layer's kernel
    assert not sp3d.sp_relu_bits_supported(sp3d.SP_OP_DGRAD, g, 1, 32, bf)
    assert not sp3d.sp_relu_bits_supported(sp3d.SP_OP_FWD, g, 32, 32, sp3d.SP_F32)
    assert not sp3d.sp_relu_bits_supported(sp3d.SP_OP_FWD, sp3d.Geom(1, (8, 16, 64), (2, 2, 1), flat=1), 32, 32, bf)
    A, B, C, D = FAKE * 64, FAKE * 128, FAKE * 192, FAKE * 256         # 4 MiB apart: tensors here take 1 MiB
    relu = sp3d.SP_FLAG_RELU
    # no bits pointer, no ReLU, misaligned bits, bits over the output
    assert L.conv3d_fwd_bits(A, FAKE, None, B, None, gp, 32, 32, bf, relu, C, 1 << 30, None) == sp3d.SP_EINVAL
    assert L.conv3d_fwd_bits(A, FAKE, None, B, D, gp, 32, 32, bf, 0, C, 1 << 30, None) == sp3d.SP_EINVAL
    assert L.conv3d_fwd_bits(A, FAKE, None, B, D + 2, gp, 32, 32, bf, relu, C, 1 << 30, None) == sp3d.SP_EINVAL
    assert L.conv3d_fwd_bits(A, FAKE, None, B, B, gp, 32, 32, bf, relu, C, 1 << 30, None) == sp3d.SP_EINVAL
    assert L.conv3d_fwd_bits(A, FAKE, None, B, D, gp, 16, 32, bf, relu, C, 1 << 30, None) == sp3d.SP_EUNSUPPORTED
    assert L.conv3d_fwd2_bits(A, 32, FAKE * 32, 32, FAKE, None, B, None, gp, 32, bf, relu, C, 1 << 30, None) == sp3d.SP_EINVAL
    assert L.conv3d_fwd2_bits(A, 32, FAKE * 32, 32, FAKE, None, B, D, gp, 32, bf, 0, C, 1 << 30, None) == sp3d.SP_EINVAL
    assert L.conv3d_dgrad_bits(A, FAKE, None, B, gp, 32, 32, bf, C, 1 << 30, None) == sp3d.SP_EINVAL
    assert L.conv3d_dgrad_bits(A, FAKE, B, B, gp, 32, 32, bf, C, 1 << 30, None) == sp3d.SP_EINVAL          # bits over dx
    assert L.conv3d_dgrad_bits(A, FAKE, D, B, gp, 16, 32, bf, C, 1 << 30, None) == sp3d.SP_EUNSUPPORTED
    assert L.sp_relu_bits(A, None, gp, 32, bf, None) == sp3d.SP_EINVAL
    assert L.sp_relu_bits(A, A, gp, 32, bf, None) == sp3d.SP_EINVAL
    assert L.sp_relu_bits(A, D, gp, 48, bf, None) == sp3d.SP_EUNSUPPORTED
    assert L.sp_relu_bits(A, D, gp, 32, sp3d.SP_F32, None) == sp3d.SP_EUNSUPPORTED
