"""The paper's procedure end to end on the CPU (test infrastructure only).

Sec. 2, third paragraph: exchange the margins of the patches, pad each patch with
the margins received, then convolve each patch on its own.  Composed here from the
slicing oracle (tiling.py) and the direct-convolution oracle (conv3d.py) so that the
claim "the partitioning is transparent" (abstract) can be checked: every function
below must return exactly what its unpartitioned counterpart returns.
"""
import numpy as np

from . import conv3d, tiling


def _per_tile(P):
    N, gd, gh, gw = P.shape[:4]
    for a in range(gd):
        for b in range(gh):
            for c in range(gw):
                yield a, b, c


def tiled_fwd(V, w, bias=None, relu=False, grid=(1, 1, 1), h=1):
    P = tiling.exchange(tiling.partition(V, grid, h), h)
    N, gd, gh, gw, pd, ph, pw, _ = P.shape
    Y = np.zeros((N, gd, gh, gw, pd, ph, pw, w.shape[4]), dtype=np.float64)
    for a, b, c in _per_tile(P):
        Y[:, a, b, c, h:-h, h:-h, h:-h, :] = conv3d.conv3d_fwd(
            np.ascontiguousarray(P[:, a, b, c]), w, bias, relu, pad=0)
    return tiling.unpartition(Y, h)


def tiled_dgrad(dZ, w, grid=(1, 1, 1), h=1):
    """Gather form: exchange the margins of dz, then each tile's dx is the 'valid'
    correlation of its padded dz with the taps mirrored and the channel roles swapped."""
    P = tiling.exchange(tiling.partition(dZ, grid, h), h)
    N, gd, gh, gw, pd, ph, pw, _ = P.shape
    wt = np.ascontiguousarray(np.transpose(np.asarray(w, dtype=np.float64)[::-1, ::-1, ::-1],
                                           (0, 1, 2, 4, 3)))
    X = np.zeros((N, gd, gh, gw, pd, ph, pw, w.shape[3]), dtype=np.float64)
    for a, b, c in _per_tile(P):
        X[:, a, b, c, h:-h, h:-h, h:-h, :] = conv3d.conv3d_fwd(
            np.ascontiguousarray(P[:, a, b, c]), wt, None, False, pad=0)
    return tiling.unpartition(X, h)


def tiled_wgrad(V, dZ, grid=(1, 1, 1), h=1):
    """Each tile correlates its padded x with its own dz; the per-tile results are
    summed over the grid (the sum that a multi-device run does across devices)."""
    Px = tiling.exchange(tiling.partition(V, grid, h), h)
    Pz = tiling.partition(dZ, grid, h)
    dw = np.zeros((3, 3, 3, V.shape[4], dZ.shape[4]), dtype=np.float64)
    for a, b, c in _per_tile(Px):
        dw += conv3d.conv3d_wgrad(np.ascontiguousarray(Px[:, a, b, c]),
                                  np.ascontiguousarray(Pz[:, a, b, c, h:-h, h:-h, h:-h, :]),
                                  pad=0)
    return dw


def _grown(idx, ngrid, t, h, e):
    """Padded-coordinate range of a tile's own voxels grown by e towards the neighbours it has."""
    return h - (e if idx > 0 else 0), h + t + (e if idx < ngrid - 1 else 0)


def tiled_block_fwd(V, ws, bs=None, grid=(1, 1, 1), stop_at_border=True):
    """k = len(ws) stacked conv + ReLU layers after ONE exchange of k-wide margins: the overlapping-patch
    idea of Sec. 1 (each device works on a patch that overlaps its neighbours and so needs nothing from
    them while it runs) applied to a short stack.  Layer i (1-based) is computed by every tile on its own
    voxels plus the k - i voxels around them that the following layers will read; where a tile has no
    neighbour that surround lies beyond the volume, where every layer's output is zero padding, so the box
    does not grow there.  Returns the k layer outputs as whole volumes.
    stop_at_border=False plants the mistake of growing there as well (tests only)."""
    k = len(ws)
    bs = bs or [None] * k
    h = k
    P = tiling.exchange(tiling.partition(V, grid, h), h)
    N, gd, gh, gw, pd, ph, pw, _ = P.shape
    tile = (pd - 2 * h, ph - 2 * h, pw - 2 * h)
    outs = []
    for i, (w, b) in enumerate(zip(ws, bs), 1):
        e = k - i
        Y = np.zeros((N, gd, gh, gw, pd, ph, pw, w.shape[4]), dtype=np.float64)
        for a, bb, c in _per_tile(P):
            if stop_at_border:
                (d0, d1), (h0, h1), (w0, w1) = (_grown(i_, n_, t_, h, e)
                                                for i_, n_, t_ in zip((a, bb, c), (gd, gh, gw), tile))
            else:
                (d0, d1), (h0, h1), (w0, w1) = ((h - e, h + t_ + e) for t_ in tile)
            window = np.ascontiguousarray(P[:, a, bb, c, d0 - 1:d1 + 1, h0 - 1:h1 + 1, w0 - 1:w1 + 1, :])
            Y[:, a, bb, c, d0:d1, h0:h1, w0:w1, :] = conv3d.conv3d_fwd(window, w, b, True, pad=0)
        outs.append(tiling.unpartition(Y, h))
        P = Y
    return outs
