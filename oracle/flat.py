"""numpy fp64 oracle of the 2-D variant of the network (test infrastructure only).

The paper also trains a 2-D U-Net on 512 x 512 x 5 slabs: the same architecture with the 3-D
convolutions and poolings replaced by 2-D ones (Sec. 3, first paragraph; Table 1, row "2D").
On the NDHWC tensors of this build a 2-D operation treats D as a stack of independent slices:
the 3x3 kernel has extent 1 along D, pooling and transposed-convolution windows are 1 x 2 x 2.
Every function is the plain definition on the unpartitioned tensor, written out tap by tap;
spatial partitioning over H and W must reproduce it (the partitioning is transparent, abstract).

Conventions as in the 3-D oracle: cross-correlation (no tap flip), zero 'same' padding,
x[N,D,H,W,Cin], w[3,3,Cin,Cout] (kh, kw), u[2,2,Cin,Cout], max-pool backward routes the gradient
to the FIRST maximum of a window in (h, w) scan order, ReLU derivative 0 at 0.
Inputs are converted to float64; all outputs are float64.
"""
import numpy as np


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def conv_fwd(x, w, bias=None, relu=False, pad=1):
    """z[n,d,h,w,co] = bias[co] + sum_{kh,kw,ci} x[n,d,h+kh-pad,w+kw-pad,ci] w[kh,kw,ci,co]; y = max(z,0) if relu.
    pad=1: zero 'same' padding in H and W; pad=0: 'valid' convolution of a patch that is already padded
    in H and W (output extents shrink by 2 there).  D is never padded: slices do not interact."""
    x, w = _f64(x), _f64(w)
    assert w.shape[:3] == (3, 3, x.shape[4]) and pad in (0, 1)
    if pad:
        x = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1), (0, 0)))
    N, D, Hp, Wp, _ = x.shape
    H, W = Hp - 2, Wp - 2
    z = np.zeros((N, D, H, W, w.shape[3]))
    for kh in range(3):
        for kw in range(3):
            z += x[:, :, kh:kh + H, kw:kw + W, :] @ w[kh, kw]
    if bias is not None:
        z = z + _f64(bias)
    return np.maximum(z, 0.0) if relu else z


def conv_dgrad(dz, w):
    """dx[n,d,h,w,ci] = sum_{kh,kw,co} dz[n,d,h-kh+1,w-kw+1,co] w[kh,kw,ci,co]   (dz zero outside)."""
    dz, w = _f64(dz), _f64(w)
    N, D, H, W, Co = dz.shape
    assert w.shape[:2] == (3, 3) and w.shape[3] == Co
    p = np.pad(dz, ((0, 0), (0, 0), (1, 1), (1, 1), (0, 0)))
    dx = np.zeros((N, D, H, W, w.shape[2]))
    for kh in range(3):
        for kw in range(3):
            # padded index of dz[h - kh + 1] is h - kh + 2
            dx += p[:, :, 2 - kh:2 - kh + H, 2 - kw:2 - kw + W, :] @ w[kh, kw].T
    return dx


def conv_wgrad(x, dz, pad=1):
    """dw[kh,kw,ci,co] = sum_{n,d,h,w} x[n,d,h+kh-pad,w+kw-pad,ci] dz[n,d,h,w,co].
    pad=0: x is a patch already padded in H and W (its extents exceed dz's by 2 there)."""
    x, dz = _f64(x), _f64(dz)
    if pad:
        x = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1), (0, 0)))
    N, D, H, W, Co = dz.shape
    assert x.shape[:4] == (N, D, H + 2, W + 2)
    Ci = x.shape[4]
    dw = np.zeros((3, 3, Ci, Co))
    zf = dz.reshape(-1, Co)
    for kh in range(3):
        for kw in range(3):
            dw[kh, kw] = x[:, :, kh:kh + H, kw:kw + W, :].reshape(-1, Ci).T @ zf
    return dw


def bias_grad(dz):
    dz = _f64(dz)
    return dz.reshape(-1, dz.shape[-1]).sum(axis=0)


def relu_bwd(dy, y):
    return np.where(np.asarray(y) > 0, _f64(dy), 0.0)


def _windows(x):
    """[N,D,H,W,C] -> [N,D,H/2,W/2,4,C], the window flattened in (h,w) scan order."""
    N, D, H, W, C = x.shape
    assert H % 2 == 0 and W % 2 == 0
    v = x.reshape(N, D, H // 2, 2, W // 2, 2, C)
    return v.transpose(0, 1, 2, 4, 3, 5, 6).reshape(N, D, H // 2, W // 2, 4, C)


def _unwindows(v):
    N, D, H2, W2, _, C = v.shape
    return v.reshape(N, D, H2, W2, 2, 2, C).transpose(0, 1, 2, 4, 3, 5, 6).reshape(N, D, 2 * H2, 2 * W2, C)


def maxpool_fwd(x):
    """y[n,d,h,w,c] = max over the 1x2x2 window starting at (d,2h,2w)."""
    return _windows(_f64(x)).max(axis=4)


def maxpool_bwd(x, dy):
    """dx = dy routed to the first maximum (scan order h,w) of each window, zero elsewhere."""
    v = _windows(_f64(x))
    first = np.argmax(v, axis=4)
    out = np.zeros_like(v)
    np.put_along_axis(out, first[:, :, :, :, None, :], _f64(dy)[:, :, :, :, None, :], axis=4)
    return _unwindows(out)


def upconv_fwd(x, u, bias=None):
    """y[n,d,2h+a,2w+b,co] = bias[co] + sum_ci x[n,d,h,w,ci] u[a,b,ci,co]."""
    x, u = _f64(x), _f64(u)
    N, D, H, W, _ = x.shape
    y = np.einsum("ndhwi,abio->ndhawbo", x, u).reshape(N, D, 2 * H, 2 * W, u.shape[3])
    return y if bias is None else y + _f64(bias)


def upconv_dgrad(dy, u):
    """dx[n,d,h,w,ci] = sum_{a,b,co} dy[n,d,2h+a,2w+b,co] u[a,b,ci,co]."""
    dy, u = _f64(dy), _f64(u)
    N, D, H2, W2, Co = dy.shape
    v = dy.reshape(N, D, H2 // 2, 2, W2 // 2, 2, Co)
    return np.einsum("ndhawbo,abio->ndhwi", v, u)


def upconv_wgrad(x, dy):
    """du[a,b,ci,co] = sum_{n,d,h,w} x[n,d,h,w,ci] dy[n,d,2h+a,2w+b,co]; db[co] = sum dy."""
    x, dy = _f64(x), _f64(dy)
    N, D, H2, W2, Co = dy.shape
    v = dy.reshape(N, D, H2 // 2, 2, W2 // 2, 2, Co)
    return np.einsum("ndhwi,ndhawbo->abio", x, v), dy.sum(axis=(0, 1, 2, 3))
