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
