"""numpy fp64 oracle of the U-Net glue operations around the 3x3x3 convolutions
(test infrastructure only).

The paper's network (Sec. 3, first paragraph) is a 3D U-Net: blocks of convolutions followed by
2x max-pooling on the way down and a symmetric up-sampling path.  The paper does not name the
up-sampling operator or the classifier; the workload list fixes a 2x2x2 stride-2 transposed
convolution, channel concatenation with the skip tensor and a final 1x1x1 convolution.  Every
function here is the plain definition on the unpartitioned NDHWC volume: pooling windows and
transposed-convolution windows never straddle tiles whose extents are even, so partitioning
does not change these results.

Conventions: x[N,D,H,W,C]; up-conv weights u[2,2,2,Cin,Cout]; point-wise weights p[Cin,Cout];
max-pool backward sends the gradient to the FIRST maximum of a window in (d,h,w) scan order.
"""
import numpy as np


def _windows(x):
    """[N,D,H,W,C] -> [N,D/2,H/2,W/2,8,C] with the window flattened in (d,h,w) scan order."""
    N, D, H, W, C = x.shape
    assert D % 2 == 0 and H % 2 == 0 and W % 2 == 0
    v = x.reshape(N, D // 2, 2, H // 2, 2, W // 2, 2, C)
    return v.transpose(0, 1, 3, 5, 2, 4, 6, 7).reshape(N, D // 2, H // 2, W // 2, 8, C)


def _unwindows(v):
    N, D2, H2, W2, _, C = v.shape
    x = v.reshape(N, D2, H2, W2, 2, 2, 2, C).transpose(0, 1, 4, 2, 5, 3, 6, 7)
    return x.reshape(N, 2 * D2, 2 * H2, 2 * W2, C)


def maxpool2_fwd(x):
    """y[n,d,h,w,c] = max over the 2x2x2 window starting at (2d,2h,2w)."""
    return _windows(np.asarray(x, dtype=np.float64)).max(axis=4)


def maxpool2_bwd(x, dy):
    """dx = dy routed to the first maximum (scan order d,h,w) of each window, zero elsewhere."""
    v = _windows(np.asarray(x, dtype=np.float64))
    first = np.argmax(v, axis=4)                               # argmax returns the first occurrence
    out = np.zeros_like(v)
    np.put_along_axis(out, first[:, :, :, :, None, :], np.asarray(dy, dtype=np.float64)[:, :, :, :, None, :],
                      axis=4)
    return _unwindows(out)


def upconv2_fwd(x, u, bias=None):
    """y[n,2d+a,2h+b,2w+c,co] = bias[co] + sum_ci x[n,d,h,w,ci] u[a,b,c,ci,co]."""
    x, u = np.asarray(x, dtype=np.float64), np.asarray(u, dtype=np.float64)
    N, D, H, W, _ = x.shape
    y = np.einsum("ndhwi,abcio->ndahbwco", x, u).reshape(N, 2 * D, 2 * H, 2 * W, u.shape[4])
    return y if bias is None else y + np.asarray(bias, dtype=np.float64)


def upconv2_dgrad(dy, u):
    """dx[n,d,h,w,ci] = sum_{a,b,c,co} dy[n,2d+a,2h+b,2w+c,co] u[a,b,c,ci,co]."""
    dy, u = np.asarray(dy, dtype=np.float64), np.asarray(u, dtype=np.float64)
    N, D2, H2, W2, Co = dy.shape
    v = dy.reshape(N, D2 // 2, 2, H2 // 2, 2, W2 // 2, 2, Co)
    return np.einsum("ndahbwco,abcio->ndhwi", v, u)


def upconv2_wgrad(x, dy):
    """du[a,b,c,ci,co] = sum_{n,d,h,w} x[n,d,h,w,ci] dy[n,2d+a,2h+b,2w+c,co]; db[co] = sum dy."""
    x, dy = np.asarray(x, dtype=np.float64), np.asarray(dy, dtype=np.float64)
    N, D2, H2, W2, Co = dy.shape
    v = dy.reshape(N, D2 // 2, 2, H2 // 2, 2, W2 // 2, 2, Co)
    return np.einsum("ndhwi,ndahbwco->abcio", x, v), dy.sum(axis=(0, 1, 2, 3))


def pointwise_fwd(x, p, bias=None):
    """1x1x1 convolution: y[..., co] = bias[co] + sum_ci x[..., ci] p[ci,co]."""
    y = np.asarray(x, dtype=np.float64) @ np.asarray(p, dtype=np.float64)
    return y if bias is None else y + np.asarray(bias, dtype=np.float64)


def pointwise_dgrad(dy, p):
    return np.asarray(dy, dtype=np.float64) @ np.asarray(p, dtype=np.float64).T


def pointwise_wgrad(x, dy):
    x, dy = np.asarray(x, dtype=np.float64), np.asarray(dy, dtype=np.float64)
    return x.reshape(-1, x.shape[-1]).T @ dy.reshape(-1, dy.shape[-1]), dy.reshape(-1, dy.shape[-1]).sum(axis=0)


def concat(a, b):
    """Channel concatenation [.., Ca] ++ [.., Cb] (skip connection)."""
    return np.concatenate([a, b], axis=-1)


def split(x, ca):
    """Backward of concat: the two channel slices."""
    return x[..., :ca], x[..., ca:]
