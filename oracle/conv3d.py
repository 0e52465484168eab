"""numpy front end of the C fp64 direct-convolution oracle (test infrastructure only).

Every function is the plain definition of the operation on the *unpartitioned*
NDHWC volume -- the result that the paper's partition / exchange margins / pad /
convolve procedure (Sec. 2, third paragraph; Fig. 1) must reproduce, since the
partitioning is stated to be transparent (abstract).  The backward passes are
the derivatives of that definition (Sec. 3, "Computational efficiency" puts
forward and backward of the convolutions on the path).

Inputs may be float64, float32 or uint16 arrays (uint16 = bf16 bit patterns);
weights and bias are converted to float64; every output is float64.
"""
import ctypes

import numpy as np

from . import build as _build

_lib = None
_DT = {np.dtype(np.float64): 0, np.dtype(np.float32): 1, np.dtype(np.uint16): 2}


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        L, P, I = ctypes.c_long, ctypes.c_void_p, ctypes.c_int
        lib.orc_conv3d_fwd.argtypes = [P, I, P, P, P, L, L, L, L, L, L, I, I, P]
        lib.orc_conv3d_dgrad.argtypes = [P, I, P, P, L, L, L, L, L, L, P]
        lib.orc_conv3d_wgrad.argtypes = [P, I, P, I, P, L, L, L, L, L, L, I, P, L]
        lib.orc_bias_grad.argtypes = [P, I, P, L, L]
        for f in (lib.orc_conv3d_fwd, lib.orc_conv3d_dgrad, lib.orc_conv3d_wgrad,
                  lib.orc_bias_grad):
            f.restype = I
        _lib = lib
    return _lib


def _arr(a):
    a = np.ascontiguousarray(a)
    if a.dtype not in _DT:
        raise TypeError("oracle takes float64, float32 or uint16 (bf16 bits), got %s" % a.dtype)
    return a, _DT[a.dtype]


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _box(box, ext):
    if box is None:
        box = (0, ext[0], 0, ext[1], 0, ext[2])
    b = np.asarray(box, dtype=np.int64)
    assert b.shape == (6,)
    return b


def conv3d_fwd(x, w, bias=None, relu=False, box=None, pad=1):
    """z = bias + sum_taps x[v + tap - pad] . w[tap];  y = relu(z) if relu.

    x [N,D,H,W,Cin], w [3,3,3,Cin,Cout].  pad=1: zero 'same' padding of the
    volume; pad=0: 'valid' convolution of an already padded patch (output
    extents shrink by 2).  box = (d0,d1,h0,h1,w0,w1) selects the output voxels.
    """
    x, xdt = _arr(x)
    w = np.ascontiguousarray(w, dtype=np.float64)
    N, D, H, W, Cin = x.shape
    assert w.shape[:4] == (3, 3, 3, Cin)
    Cout = w.shape[4]
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float64)
    ext = (D - 2 + 2 * pad, H - 2 + 2 * pad, W - 2 + 2 * pad)
    bx = _box(box, ext)
    y = np.empty((N, bx[1] - bx[0], bx[3] - bx[2], bx[5] - bx[4], Cout), dtype=np.float64)
    rc = _load().orc_conv3d_fwd(_ptr(x), xdt, _ptr(w), None if b is None else _ptr(b), _ptr(y),
                                N, D, H, W, Cin, Cout, pad, int(bool(relu)), _ptr(bx))
    if rc:
        raise ValueError("orc_conv3d_fwd: bad arguments (%d)" % rc)
    return y


def conv3d_dgrad(dz, w, box=None):
    """dx[v,ci] = sum_taps sum_co dz[v - tap + 1, co] . w[tap,ci,co]   (dz zero outside)."""
    dz, zdt = _arr(dz)
    w = np.ascontiguousarray(w, dtype=np.float64)
    N, D, H, W, Cout = dz.shape
    assert w.shape[:3] == (3, 3, 3) and w.shape[4] == Cout
    Cin = w.shape[3]
    bx = _box(box, (D, H, W))
    dx = np.empty((N, bx[1] - bx[0], bx[3] - bx[2], bx[5] - bx[4], Cin), dtype=np.float64)
    rc = _load().orc_conv3d_dgrad(_ptr(dz), zdt, _ptr(w), _ptr(dx), N, D, H, W, Cin, Cout,
                                  _ptr(bx))
    if rc:
        raise ValueError("orc_conv3d_dgrad: bad arguments (%d)" % rc)
    return dx


def conv3d_wgrad(x, dz, sel=None, pad=1):
    """dw[tap,ci,co] = sum_v x[v + tap - pad, ci] . dz[v, co].

    Returns the full [3,3,3,Cin,Cout] array, or, when sel (flat indices into it)
    is given, just those entries.  pad=0: x is an already padded patch whose
    extents exceed dz's by 2.
    """
    x, xdt = _arr(x)
    dz, zdt = _arr(dz)
    N, D, H, W, Cout = dz.shape
    Cin = x.shape[4]
    assert x.shape[:4] == (N, D + 2 - 2 * pad, H + 2 - 2 * pad, W + 2 - 2 * pad)
    if sel is None:
        out = np.empty((3, 3, 3, Cin, Cout), dtype=np.float64)
        rc = _load().orc_conv3d_wgrad(_ptr(x), xdt, _ptr(dz), zdt, _ptr(out), N, D, H, W,
                                      Cin, Cout, pad, None, 0)
    else:
        s = np.ascontiguousarray(sel, dtype=np.int64)
        out = np.empty(s.shape, dtype=np.float64)
        rc = _load().orc_conv3d_wgrad(_ptr(x), xdt, _ptr(dz), zdt, _ptr(out), N, D, H, W,
                                      Cin, Cout, pad, _ptr(s), s.size)
    if rc:
        raise ValueError("orc_conv3d_wgrad: bad arguments (%d)" % rc)
    return out


def bias_grad(dz):
    """db[co] = sum over all voxels of dz[., co]."""
    dz, zdt = _arr(dz)
    Cout = dz.shape[-1]
    db = np.empty((Cout,), dtype=np.float64)
    _load().orc_bias_grad(_ptr(dz), zdt, _ptr(db), dz.size // Cout, Cout)
    return db


def relu_bwd(dy, y):
    """dz = dy . [y > 0]  (derivative of max(z,0) taken as 0 at z = 0)."""
    return np.where(np.asarray(y) > 0, np.asarray(dy, dtype=np.float64), 0.0)


def bf16_bits_to_f64(u):
    """Exact widening of bf16 bit patterns (uint16) to float64."""
    u = np.asarray(u, dtype=np.uint16)
    return (u.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
