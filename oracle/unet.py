"""fp64 oracle of the U-Net convolution stack on the unpartitioned volume (test infrastructure only).

Composes the direct-convolution oracle and the glue oracle in the order of the paper's network
(Sec. 3, first paragraph) as fixed by the workload list: per level `convs` 3x3x3 conv + ReLU (two in
the workload list, four in the paper's own blocks), 2x2x2 max-pool between levels, decoder = transposed
conv, concat (skip, up), `convs` conv + ReLU, final 1x1x1 conv.  Biases are zero.  All arithmetic is fp64.  With `store=None` activations stay fp64 throughout;
with `store=round_bf16` every tensor that the path keeps in memory (each layer output, each
propagated gradient) is rounded to the bf16 storage type first, so that the decisions the path takes
on stored values -- the ReLU mask and the max-pool argmax -- are taken on the same kind of value
as on the device (the workload list fixes bf16 storage with fp32 accumulation).
"""
import numpy as np

from . import conv3d, flat as F2, unet_ops as U3


class _Ops3:
    """the 3-D network: 3x3x3 convolutions, 2x2x2 windows"""
    conv_fwd = staticmethod(lambda x, w, relu=False: conv3d.conv3d_fwd(x, w, relu=relu))
    conv_dgrad = staticmethod(conv3d.conv3d_dgrad)
    conv_wgrad = staticmethod(conv3d.conv3d_wgrad)
    maxpool_fwd, maxpool_bwd = staticmethod(U3.maxpool2_fwd), staticmethod(U3.maxpool2_bwd)
    upconv_fwd, upconv_dgrad = staticmethod(U3.upconv2_fwd), staticmethod(U3.upconv2_dgrad)
    upconv_wgrad = staticmethod(U3.upconv2_wgrad)


class _Ops2:
    """the 2-D network of Sec. 3 (same architecture, 2-D convolutions and poolings): D is a stack of slices"""
    conv_fwd = staticmethod(lambda x, w, relu=False: F2.conv_fwd(x, w, relu=relu))
    conv_dgrad = staticmethod(F2.conv_dgrad)
    conv_wgrad = staticmethod(F2.conv_wgrad)
    maxpool_fwd, maxpool_bwd = staticmethod(F2.maxpool_fwd), staticmethod(F2.maxpool_bwd)
    upconv_fwd, upconv_dgrad = staticmethod(F2.upconv_fwd), staticmethod(F2.upconv_dgrad)
    upconv_wgrad = staticmethod(F2.upconv_wgrad)


U = U3      # channel and point-wise operations are the same in both variants


def round_bf16(a):
    """fp64 -> nearest bf16 (ties to even), returned as fp64."""
    u = np.asarray(a, dtype=np.float64).astype(np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(np.float64)


LETTERS = "abcdefgh"


def forward(x, w, channels, keep=None, store=None, convs=2, flat=False):
    """x [N,D,H,W,Cin] fp64; w: name -> fp64 weights.  Returns logits; fills `keep` with activations.
    flat: the 2-D variant (weights [3,3,Ci,Co] and [2,2,Ci,Co])."""
    O = _Ops2 if flat else _Ops3
    L = len(channels)
    A = {} if keep is None else keep
    q = store if store is not None else (lambda a: a)
    h = np.asarray(x, dtype=np.float64)
    for i in range(L):
        if i > 0:
            h = O.maxpool_fwd(h)
        for k in range(convs):
            name = "enc%d_%s" % (i, LETTERS[k])
            A[name + ".x"] = h
            h = q(O.conv_fwd(h, w[name], relu=True))
        A["enc%d.y" % i] = h
    for i in range(L - 2, -1, -1):
        A["up%d.x" % i] = h
        up = q(O.upconv_fwd(h, w["up%d" % i]))
        h = U.concat(A["enc%d.y" % i], up)
        for k in range(convs):
            name = "dec%d_%s" % (i, LETTERS[k])
            A[name + ".x"] = h
            h = q(O.conv_fwd(h, w[name], relu=True))
        A["dec%d.y" % i] = h
    A["head.x"] = h
    p = w["head"]
    return q(U.pointwise_fwd(h, p.reshape(p.shape[-2], p.shape[-1])))


def backward(dlogits, w, channels, A, store=None, trace=None, convs=2, flat=False):
    """Gradients of <logits, dlogits> with respect to every weight tensor and the input.
    `trace`, if given, receives the stored tensors of the backward pass by name
    ("<layer>.dy" incoming gradient, "<layer>.dx" outgoing gradient, "pool<i>.dy", "skip<i>")."""
    O = _Ops2 if flat else _Ops3
    L = len(channels)
    grads = {}
    T = {} if trace is None else trace
    q = store if store is not None else (lambda a: a)
    p = w["head"].reshape(w["head"].shape[-2], w["head"].shape[-1])
    dp, _ = U.pointwise_wgrad(A["head.x"], dlogits)
    grads["head"] = dp.reshape(w["head"].shape)
    g = q(U.pointwise_dgrad(dlogits, p))
    T["head.dx"] = g

    def conv_bwd(name, x, y, dy):
        T[name + ".dy"] = dy
        dz = conv3d.relu_bwd(dy, y)
        grads[name] = O.conv_wgrad(x, dz)
        dx = q(O.conv_dgrad(dz, w[name]))
        T[name + ".dx"] = dx
        return dx

    def block_bwd(block, g):
        """the `convs` layers of a block, last to first; layer k's output is layer k + 1's input"""
        for k in range(convs - 1, -1, -1):
            name = "%s_%s" % (block, LETTERS[k])
            y = A[block + ".y"] if k == convs - 1 else A["%s_%s.x" % (block, LETTERS[k + 1])]
            g = conv_bwd(name, A[name + ".x"], y, g)
        return g

    skip = {}
    for i in range(0, L - 1):
        c = channels[i]
        g = block_bwd("dec%d" % i, g)
        skip[i], gu = U.split(g, c)
        T["skip%d" % i], T["up%d.dy" % i] = skip[i], gu
        grads["up%d" % i], _ = O.upconv_wgrad(A["up%d.x" % i], gu)
        g = q(O.upconv_dgrad(gu, w["up%d" % i]))
        T["up%d.dx" % i] = g
    for i in range(L - 1, -1, -1):
        if i in skip:
            T["add%d.a" % i] = g
            g = q(g + skip[i])
        g = block_bwd("enc%d" % i, g)
        if i > 0:
            T["pool%d.dy" % i] = g
            g = O.maxpool_bwd(A["enc%d.y" % (i - 1)], g)
            T["pool%d.dx" % i] = g
    return grads, g
