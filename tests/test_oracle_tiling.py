"""Pins of the partition / halo oracle: invariants that follow from the paper's statement
(non-overlapping exhaustive patches, margins of half the kernel size from every neighbour,
zero at the volume border) and the transparency claim (tiled result == whole-volume result)."""
import itertools

import numpy as np
import pytest

from oracle import conv3d, tiled, tiling

GRIDS = [((4, 4, 4), (1, 1, 1)), ((4, 4, 4), (2, 2, 2)), ((4, 6, 2), (4, 3, 1)),
         ((3, 2, 5), (3, 2, 5)), ((6, 4, 8), (2, 1, 4)), ((2, 8, 3), (1, 4, 3))]


def vol(rng, dhw, c, n=1):
    return rng.standard_normal((n,) + tuple(dhw) + (c,))


def test_26_directions_in_lexicographic_order():
    assert len(tiling.DIRECTIONS) == 26
    assert tiling.DIRECTIONS == sorted(tiling.DIRECTIONS)
    assert tiling.DIRECTIONS[0] == (-1, -1, -1) and tiling.DIRECTIONS[-1] == (1, 1, 1)
    assert (0, 0, 0) not in tiling.DIRECTIONS


@pytest.mark.parametrize("dhw,grid", GRIDS)
def test_partition_is_exhaustive_and_non_overlapping(rng, dhw, grid):
    """Tag every voxel with a unique number: after partition every tag appears exactly once
    in the interiors, and unpartition restores the volume bit for bit."""
    V = np.arange(2 * np.prod(dhw) * 3, dtype=np.float64).reshape((2,) + dhw + (3,)) + 1
    P = tiling.partition(V, grid)
    inner = P[:, :, :, :, 1:-1, 1:-1, 1:-1, :]
    assert np.array_equal(np.sort(inner.ravel()), np.sort(V.ravel()))
    assert np.count_nonzero(P) == V.size                      # margins untouched (zero)
    assert np.array_equal(tiling.unpartition(P), V)


@pytest.mark.parametrize("dhw,grid", GRIDS)
def test_message_size_and_region_sizes(dhw, grid):
    tile = tiling.tile_extents(dhw, grid)
    sizes = tiling.region_sizes(tile, 1)
    assert sum(sizes) == tiling.margin_voxels(tile, 1)
    td, th, tw = tile
    # 6 faces, 12 edges, 8 corners
    assert sorted(sizes) == sorted([td * th, td * th, td * tw, td * tw, th * tw, th * tw]
                                   + [td] * 4 + [th] * 4 + [tw] * 4 + [1] * 8)


@pytest.mark.parametrize("dhw,grid", GRIDS)
def test_exchange_reproduces_windows_of_the_zero_padded_volume(rng, dhw, grid):
    V = vol(rng, dhw, 2, n=2)
    P = tiling.partition(V, grid)
    assert np.array_equal(tiling.exchange(P), tiling.padded_reference(V, grid))


def test_unpack_overwrites_stale_margins_and_keeps_interior(rng):
    V = vol(rng, (4, 4, 4), 1)
    P = tiling.partition(V, (2, 2, 1))
    M = tiling.halo_pack(P)
    dirty = P.copy()
    dirty[:, :, :, :, 0] = 99.0
    dirty[:, :, :, :, :, :, -1] = 99.0
    assert np.array_equal(tiling.halo_unpack(dirty, M), tiling.padded_reference(V, (2, 2, 1)))


def test_corner_region_comes_from_the_diagonal_neighbour():
    """2x2x2 grid of 1-voxel tiles: tile (0,0,0)'s (+,+,+) corner margin is tile (1,1,1)."""
    V = np.arange(8, dtype=np.float64).reshape(1, 2, 2, 2, 1) + 1
    P = tiling.exchange(tiling.partition(V, (2, 2, 2)))
    assert P[0, 0, 0, 0, 2, 2, 2, 0] == V[0, 1, 1, 1, 0]
    assert P[0, 1, 1, 1, 0, 0, 0, 0] == V[0, 0, 0, 0, 0]
    assert P[0, 0, 0, 0, 0, 0, 0, 0] == 0                      # outside the volume
    # a face neighbour and an edge neighbour
    assert P[0, 0, 0, 0, 2, 1, 1, 0] == V[0, 1, 0, 0, 0]
    assert P[0, 0, 0, 0, 1, 2, 2, 0] == V[0, 0, 1, 1, 0]


@pytest.mark.parametrize("dhw,grid", [((4, 4, 4), (2, 2, 1)), ((4, 6, 4), (2, 3, 2)),
                                      ((3, 2, 2), (3, 2, 2)), ((4, 4, 6), (1, 1, 1))])
def test_tiled_passes_equal_unpartitioned_passes(rng, dhw, grid):
    """The paper's transparency claim, for forward, data-grad and weight-grad."""
    x, g = vol(rng, dhw, 2), vol(rng, dhw, 3)
    w, b = rng.standard_normal((3, 3, 3, 2, 3)), rng.standard_normal(3)
    np.testing.assert_allclose(tiled.tiled_fwd(x, w, b, True, grid), conv3d.conv3d_fwd(x, w, b, True),
                               rtol=0, atol=1e-13)
    np.testing.assert_allclose(tiled.tiled_dgrad(g, w, grid), conv3d.conv3d_dgrad(g, w),
                               rtol=0, atol=1e-12)
    np.testing.assert_allclose(tiled.tiled_wgrad(x, g, grid), conv3d.conv3d_wgrad(x, g),
                               rtol=0, atol=1e-12)


def test_without_edge_and_corner_regions_the_result_is_wrong(rng):
    """Planted mistake (on the CPU): exchanging face margins only, as the paper's 2-D sketch
    might suggest, breaks the tiled == unpartitioned identity at tile edges."""
    x = vol(rng, (4, 4, 4), 1)
    w = rng.standard_normal((3, 3, 3, 1, 1))
    P = tiling.partition(x, (2, 2, 2))
    full = tiling.exchange(P)
    faces_only = P.copy()
    for delta in tiling.DIRECTIONS:
        if sum(abs(d) for d in delta) != 1:
            continue
        sl = tuple({-1: slice(0, 1), 0: slice(1, -1), 1: slice(-1, None)}[d] for d in delta)
        faces_only[(slice(None),) * 4 + sl] = full[(slice(None),) * 4 + sl]
    y_full = conv3d.conv3d_fwd(np.ascontiguousarray(full[:, 0, 0, 0]), w, pad=0)
    y_faces = conv3d.conv3d_fwd(np.ascontiguousarray(faces_only[:, 0, 0, 0]), w, pad=0)
    assert not np.allclose(y_full, y_faces)


def test_overlapping_patch_alternative_gives_the_same_interior(rng):
    """The alternative the paper rejects (Sec. 1: overlapping patches): a patch cut with an
    overlap equal to the number of stacked convolutions yields the same interior values."""
    x = vol(rng, (8, 8, 8), 2)
    w1, w2 = rng.standard_normal((3, 3, 3, 2, 2)), rng.standard_normal((3, 3, 3, 2, 2))
    full = conv3d.conv3d_fwd(conv3d.conv3d_fwd(x, w1, relu=True), w2)
    xp = np.pad(x, ((0, 0), (2, 2), (2, 2), (2, 2), (0, 0)))
    patch = np.ascontiguousarray(xp[:, 4:4 + 8, 0:8, 2:2 + 8])     # tile (1,0,.) of a 2x2 grid + overlap 2
    # inside the volume the first conv must see zeros only beyond the true border
    y1 = conv3d.conv3d_fwd(patch, w1, relu=True, pad=0)
    # positions of y1 that lie outside the true volume must be zero before the second conv
    y1[:, :, 0:1] = 0       # h = -1 of the volume
    y1[:, 5:6] = 0          # d = 8 of the volume
    y2 = conv3d.conv3d_fwd(y1, w2, pad=0)
    np.testing.assert_allclose(y2, full[:, 4:8, 0:4, 2:6], rtol=0, atol=1e-12)


def test_paper_size_arithmetic():
    """Numbers the paper prints (see tests/golden/paper_facts.txt for the citations)."""
    import os
    facts = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_facts.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                facts[line[0]] = [float(v) for v in line[1:]]
    nbytes = (facts["intro_batch"][0] * facts["intro_filters"][0] * facts["intro_side"][0] ** 3
              * facts["intro_bytes_per_value"][0])
    assert facts["intro_min_gb"][0] * 1e9 < nbytes < (facts["intro_min_gb"][0] + 1) * 1e9
    for key in ("pod_64", "pod_128", "pod_256", "pod_512"):
        a, b, dp, sp = facts[key]
        assert a * b * facts["cores_per_tpu"][0] == dp * sp
    assert int(facts["kernel_size"][0] * facts["halo_fraction_of_kernel"][0]) == 1


@pytest.mark.parametrize("dhw,grid,k", [((6, 6, 4), (2, 3, 1), 2), ((6, 6, 6), (2, 2, 2), 3), ((8, 4, 4), (2, 1, 1), 4),
                                        ((4, 4, 4), (1, 1, 1), 2)])
def test_block_after_one_wide_exchange_equals_the_unpartitioned_stack(rng, dhw, grid, k):
    """k conv + ReLU layers after one exchange of k-wide margins (the overlap of Sec. 1 for a short stack):
    every layer's output equals the whole-volume one, provided the redundantly computed surround stops at the
    volume border, where each layer sees zero padding."""
    x = vol(rng, dhw, 2)
    ws = [rng.standard_normal((3, 3, 3, 2, 2)) * 0.3 for _ in range(k)]
    bs = [rng.standard_normal(2) for _ in range(k)]
    ref, y = [], x
    for w, b in zip(ws, bs):
        y = conv3d.conv3d_fwd(y, w, b, relu=True)
        ref.append(y)
    got = tiled.tiled_block_fwd(x, ws, bs, grid)
    for r, g_ in zip(ref, got):
        np.testing.assert_allclose(g_, r, rtol=0, atol=1e-12)
    if max(grid) > 1 or k > 1:
        # planted mistake: convolving beyond the volume border as well changes the last layer near the border
        wrong = tiled.tiled_block_fwd(x, ws, bs, grid, stop_at_border=False)
        assert not np.allclose(wrong[-1], ref[-1])


WIDE = [((4, 4, 4), (1, 1, 1), 2), ((4, 4, 4), (2, 2, 2), 2), ((6, 4, 8), (2, 1, 4), 2), ((6, 6, 3), (2, 2, 1), 3),
        ((8, 4, 4), (2, 1, 1), 4)]


@pytest.mark.parametrize("dhw,grid,h", WIDE)
def test_wider_margins_reproduce_wider_windows(rng, dhw, grid, h):
    """Margins of width h > 1 (several layers per exchange): same invariants as for h = 1."""
    V = vol(rng, dhw, 2, n=2)
    P = tiling.partition(V, grid, h)
    assert np.count_nonzero(P) == np.count_nonzero(V) and np.array_equal(tiling.unpartition(P, h), V)
    assert np.array_equal(tiling.exchange(P, h), tiling.padded_reference(V, grid, h))
    tile = tiling.tile_extents(dhw, grid)
    assert sum(tiling.region_sizes(tile, h)) == tiling.margin_voxels(tile, h) == tiling.halo_pack(P, h).shape[4]


@pytest.mark.parametrize("dhw,grid,h", [((4, 6, 8), (2, 3, 2), 1), ((6, 4, 4), (3, 1, 2), 2), ((3, 3, 3), (1, 1, 1), 1)])
def test_delivered_mask_is_exactly_what_unpack_reads(dhw, grid, h):
    """tiling.delivered() against the receiving side itself: garbage in the entries it calls undelivered does not
    change any padded tile, and every entry it calls delivered does reach some margin (a unique tag planted in the
    message shows up after unpack)."""
    rng = np.random.default_rng(5)
    V = rng.integers(1, 1000, size=(1,) + dhw + (2,)).astype(np.int64)
    P = tiling.partition(V, grid, h)
    M = tiling.halo_pack(P, h)
    tile = tiling.tile_extents(dhw, grid)
    mask = tiling.delivered(grid, tile, h)[None, ..., None] & np.ones_like(M, dtype=bool)
    ref = tiling.halo_unpack(P, M, h)
    assert np.array_equal(tiling.halo_unpack(P, np.where(mask, M, -7), h), ref)
    tags = np.arange(M.size, dtype=np.int64).reshape(M.shape) + 10 ** 6       # unique, and none occurs in V
    got = tiling.halo_unpack(P, tags, h)
    assert set(got[got >= 10 ** 6].tolist()) == set(tags[mask].tolist())
