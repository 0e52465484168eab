"""numpy oracle of spatial partitioning and halo exchange (test infrastructure only).

Follows the paper's Fig. 1 and Sec. 2 (third paragraph):
  (a) the volume is cut into non-overlapping patches (here "tiles") on a grid
      (gd, gh, gw) over the D, H, W axes;
  (b) before a convolution each tile sends its margins -- slabs whose width is
      half the kernel size, h = 1 for 3x3x3 -- to its neighbours, and every
      tile is padded with the margins it received.
The paper's figure draws face margins only; a 3x3x3 kernel also reads across
edges and corners, so all 26 neighbour directions are exchanged.  At the border
of the whole volume nothing is received and the margin is zero ('same' padding).

Everything here is written with array slicing only: no arithmetic on values, so
all results are exact for any dtype.

Layouts (axes): volume V[N,D,H,W,C]; padded tile array
P[N,gd,gh,gw,td+2h,th+2h,tw+2h,C] with the tile's own voxels at [h, h+t) on each
axis; message array M[N,gd,gh,gw,R,C], R = (td+2h)(th+2h)(tw+2h) - td*th*tw,
holding the 26 regions in lexicographic order of (dd,dh,dw) in {-1,0,1}^3
without (0,0,0), each region row-major over its own (d,h,w) extents.
"""
import itertools

import numpy as np

DIRECTIONS = [d for d in itertools.product((-1, 0, 1), repeat=3) if d != (0, 0, 0)]


def tile_extents(shape_dhw, grid):
    (D, H, W), (gd, gh, gw) = shape_dhw, grid
    if D % gd or H % gh or W % gw:
        raise ValueError("grid does not divide the volume")
    return D // gd, H // gh, W // gw


def _send_range(delta, t, h):
    """Own-voxel range (tile-local, unpadded) nearest to the neighbour in direction delta."""
    return {-1: (0, h), 0: (0, t), 1: (t - h, t)}[delta]


def _margin_range(delta, t, h):
    """Range in padded coordinates of the margin lying in direction delta."""
    return {-1: (0, h), 0: (h, h + t), 1: (h + t, 2 * h + t)}[delta]


def region_sizes(tile, h):
    """Voxels in each of the 26 regions, in message order."""
    out = []
    for delta in DIRECTIONS:
        n = 1
        for dl, t in zip(delta, tile):
            n *= h if dl else t
        out.append(n)
    return out


def margin_voxels(tile, h):
    td, th, tw = tile
    return (td + 2 * h) * (th + 2 * h) * (tw + 2 * h) - td * th * tw


def partition(V, grid, h=1):
    """Fig. 1(a): copy each tile into the interior of its padded slot; margins are left zero."""
    N, D, H, W, C = V.shape
    gd, gh, gw = grid
    td, th, tw = tile_extents((D, H, W), grid)
    P = np.zeros((N, gd, gh, gw, td + 2 * h, th + 2 * h, tw + 2 * h, C), dtype=V.dtype)
    for a in range(gd):
        for b in range(gh):
            for c in range(gw):
                P[:, a, b, c, h:h + td, h:h + th, h:h + tw, :] = \
                    V[:, a * td:(a + 1) * td, b * th:(b + 1) * th, c * tw:(c + 1) * tw, :]
    return P


def unpartition(P, h=1):
    """Inverse of partition: drop the margins and reassemble the volume."""
    N, gd, gh, gw, pd, ph, pw, C = P.shape
    td, th, tw = pd - 2 * h, ph - 2 * h, pw - 2 * h
    V = np.empty((N, gd * td, gh * th, gw * tw, C), dtype=P.dtype)
    for a in range(gd):
        for b in range(gh):
            for c in range(gw):
                V[:, a * td:(a + 1) * td, b * th:(b + 1) * th, c * tw:(c + 1) * tw, :] = \
                    P[:, a, b, c, h:h + td, h:h + th, h:h + tw, :]
    return V


def padded_reference(V, grid, h=1):
    """What every padded tile must hold after the exchange, taken straight from the
    zero-padded whole volume: tile (a,b,c) is the window of extents t+2h that starts
    h voxels before the tile's origin."""
    N, D, H, W, C = V.shape
    gd, gh, gw = grid
    td, th, tw = tile_extents((D, H, W), grid)
    Vp = np.zeros((N, D + 2 * h, H + 2 * h, W + 2 * h, C), dtype=V.dtype)
    Vp[:, h:h + D, h:h + H, h:h + W, :] = V
    P = np.empty((N, gd, gh, gw, td + 2 * h, th + 2 * h, tw + 2 * h, C), dtype=V.dtype)
    for a in range(gd):
        for b in range(gh):
            for c in range(gw):
                P[:, a, b, c] = Vp[:, a * td:a * td + td + 2 * h, b * th:b * th + th + 2 * h,
                                   c * tw:c * tw + tw + 2 * h, :]
    return P


def halo_pack(P, h=1):
    """Fig. 1(b), sending side: region delta of a tile's message is the box of the
    tile's own voxels that touches the neighbour in direction delta (width h on the
    axes where delta != 0, the full tile extent elsewhere)."""
    N, gd, gh, gw, pd, ph, pw, C = P.shape
    tile = (pd - 2 * h, ph - 2 * h, pw - 2 * h)
    M = np.empty((N, gd, gh, gw, margin_voxels(tile, h), C), dtype=P.dtype)
    off = 0
    for delta in DIRECTIONS:
        (a0, a1), (b0, b1), (c0, c1) = (_send_range(dl, t, h) for dl, t in zip(delta, tile))
        box = P[:, :, :, :, h + a0:h + a1, h + b0:h + b1, h + c0:h + c1, :]
        n = (a1 - a0) * (b1 - b0) * (c1 - c0)
        M[:, :, :, :, off:off + n, :] = box.reshape(N, gd, gh, gw, n, C)
        off += n
    assert off == M.shape[4]
    return M


def halo_unpack(P, M, h=1):
    """Receiving side: the margin of tile t in direction delta is filled from region
    -delta of the message of tile t+delta; where t+delta is off the grid it is zeros.
    The tile's own voxels are not touched.  Returns a new array."""
    N, gd, gh, gw, pd, ph, pw, C = P.shape
    tile = (pd - 2 * h, ph - 2 * h, pw - 2 * h)
    sizes = region_sizes(tile, h)
    offs = np.concatenate(([0], np.cumsum(sizes)))
    out = P.copy()
    for delta in DIRECTIONS:
        (a0, a1), (b0, b1), (c0, c1) = (_margin_range(dl, t, h) for dl, t in zip(delta, tile))
        shape = (a1 - a0, b1 - b0, c1 - c0)
        src = DIRECTIONS.index(tuple(-dl for dl in delta))
        for a in range(gd):
            for b in range(gh):
                for c in range(gw):
                    na, nb, nc = a + delta[0], b + delta[1], c + delta[2]
                    if 0 <= na < gd and 0 <= nb < gh and 0 <= nc < gw:
                        msg = M[:, na, nb, nc, offs[src]:offs[src + 1], :]
                        out[:, a, b, c, a0:a1, b0:b1, c0:c1, :] = msg.reshape((N,) + shape + (C,))
                    else:
                        out[:, a, b, c, a0:a1, b0:b1, c0:c1, :] = 0
    return out


def delivered(grid, tile, h=1):
    """Which entries of the message array anyone receives: [gd,gh,gw,R] booleans, True for the voxels of a
    region whose direction leads to a tile of the grid.  (Fig. 1b: margins are exchanged between neighbouring
    patches; a patch at the border of the image has no neighbour on that side.)"""
    gd, gh, gw = grid
    sizes = region_sizes(tile, h)
    offs = np.concatenate(([0], np.cumsum(sizes)))
    out = np.zeros((gd, gh, gw, offs[-1]), dtype=bool)
    for k, delta in enumerate(DIRECTIONS):
        for a in range(gd):
            for b in range(gh):
                for c in range(gw):
                    na, nb, nc = a + delta[0], b + delta[1], c + delta[2]
                    if 0 <= na < gd and 0 <= nb < gh and 0 <= nc < gw:
                        out[a, b, c, offs[k]:offs[k + 1]] = True
    return out


def exchange(P, h=1):
    """pack followed by unpack."""
    return halo_unpack(P, halo_pack(P, h), h)
