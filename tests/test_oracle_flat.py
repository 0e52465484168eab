"""Pins of the 2-D variant's oracle (oracle/flat.py) to facts that do not come from it: a library routine in
float64 and its autograd, brute-force loops, one-hot shift kernels, the 3-D oracle with the kernel embedded
in its middle D plane, hand-built windows for the tie rule, adjoint identities, and the transparency of the
partitioning over H and W (Sec. 2; Sec. 3 for the 2-D network)."""
import itertools

import numpy as np
import pytest

from oracle import conv3d, flat, tiling

torch = pytest.importorskip("torch")
F = torch.nn.functional


def slices(x):       # [N,D,H,W,C] numpy -> [N*D,C,H,W] torch (every slice an image of a batch)
    N, D, H, W, C = x.shape
    return torch.from_numpy(np.ascontiguousarray(x)).reshape(N * D, H, W, C).permute(0, 3, 1, 2)


def unslices(t, N, D):
    B, C, H, W = t.shape
    return t.permute(0, 2, 3, 1).reshape(N, D, H, W, C).contiguous().numpy()


def kernel(w):       # [3,3,Cin,Cout] -> torch [Cout,Cin,kh,kw]
    return torch.from_numpy(np.ascontiguousarray(w)).permute(3, 2, 0, 1)


def test_forward_against_library_conv2d_and_autograd(rng):
    N, D, H, W, Ci, Co = 2, 3, 5, 6, 3, 4
    x, w, b = rng.standard_normal((N, D, H, W, Ci)), rng.standard_normal((3, 3, Ci, Co)), rng.standard_normal(Co)
    dz = rng.standard_normal((N, D, H, W, Co))
    xt = slices(x).clone().requires_grad_(True)
    wt = kernel(w).clone().requires_grad_(True)
    bt = torch.from_numpy(b).clone().requires_grad_(True)
    y = F.conv2d(xt, wt, bt, padding=1)
    np.testing.assert_allclose(flat.conv_fwd(x, w, b), unslices(y.detach(), N, D), rtol=0, atol=1e-12)
    np.testing.assert_allclose(flat.conv_fwd(x, w, b, relu=True), unslices(torch.relu(y).detach(), N, D), rtol=0,
                               atol=1e-12)
    y.backward(slices(dz))
    np.testing.assert_allclose(flat.conv_dgrad(dz, w), unslices(xt.grad, N, D), rtol=0, atol=1e-12)
    np.testing.assert_allclose(flat.conv_wgrad(x, dz), wt.grad.permute(2, 3, 1, 0).numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(flat.bias_grad(dz), bt.grad.numpy(), rtol=0, atol=1e-12)


def test_forward_brute_force(rng):
    N, D, H, W, Ci, Co = 1, 2, 3, 4, 2, 2
    x, w, b = rng.standard_normal((N, D, H, W, Ci)), rng.standard_normal((3, 3, Ci, Co)), rng.standard_normal(Co)
    y = flat.conv_fwd(x, w, b)
    for d, h, ww, co in itertools.product(range(D), range(H), range(W), range(Co)):
        s = b[co]
        for kh, kw, ci in itertools.product(range(3), range(3), range(Ci)):
            hh, wv = h + kh - 1, ww + kw - 1
            if 0 <= hh < H and 0 <= wv < W:
                s += x[0, d, hh, wv, ci] * w[kh, kw, ci, co]
        assert abs(y[0, d, h, ww, co] - s) < 1e-12


@pytest.mark.parametrize("tap", [t for t in itertools.product(range(3), repeat=2) if t != (1, 1)])
def test_shift_kernels_fix_the_tap_convention_and_slices_do_not_mix(rng, tap):
    """A one-hot tap (kh,kw) reads x at offset tap - 1 inside the slice (no flip, zero fill), never another slice."""
    D, H, W, C = 3, 4, 5, 2
    x = rng.standard_normal((1, D, H, W, C))
    w = np.zeros((3, 3, C, C))
    w[tap] = np.eye(C)
    expect = np.zeros_like(x)
    for d, h, ww in itertools.product(range(D), range(H), range(W)):
        s = (h + tap[0] - 1, ww + tap[1] - 1)
        if 0 <= s[0] < H and 0 <= s[1] < W:
            expect[0, d, h, ww] = x[0, d, s[0], s[1]]
    assert np.array_equal(flat.conv_fwd(x, w), expect)


def test_equals_the_3d_oracle_with_the_kernel_in_the_middle_plane(rng):
    x, w = rng.standard_normal((1, 4, 5, 6, 3)), rng.standard_normal((3, 3, 3, 2))
    dz = rng.standard_normal((1, 4, 5, 6, 2))
    w3 = np.zeros((3, 3, 3, 3, 2))
    w3[1] = w
    np.testing.assert_allclose(flat.conv_fwd(x, w), conv3d.conv3d_fwd(x, w3), rtol=0, atol=1e-12)
    np.testing.assert_allclose(flat.conv_dgrad(dz, w), conv3d.conv3d_dgrad(dz, w3), rtol=0, atol=1e-12)
    np.testing.assert_allclose(flat.conv_wgrad(x, dz), conv3d.conv3d_wgrad(x, dz)[1], rtol=0, atol=1e-11)


def test_adjoint_identities(rng):
    """<conv(x), dz> = <x, dgrad(dz)> = <w, wgrad(x, dz)>: dgrad and wgrad are the transposes of the forward map."""
    x, w = rng.standard_normal((2, 2, 4, 5, 3)), rng.standard_normal((3, 3, 3, 2))
    dz = rng.standard_normal((2, 2, 4, 5, 2))
    lhs = np.sum(flat.conv_fwd(x, w) * dz)
    assert abs(lhs - np.sum(x * flat.conv_dgrad(dz, w))) < 1e-10
    assert abs(lhs - np.sum(w * flat.conv_wgrad(x, dz))) < 1e-10


def test_valid_mode_is_the_inside_of_same_mode(rng):
    x, w = rng.standard_normal((1, 2, 6, 7, 2)), rng.standard_normal((3, 3, 2, 3))
    dz = rng.standard_normal((1, 2, 4, 5, 3))
    assert np.allclose(flat.conv_fwd(x, w, pad=0), flat.conv_fwd(x, w)[:, :, 1:-1, 1:-1], atol=1e-12)
    full = np.zeros((1, 2, 6, 7, 3))
    full[:, :, 1:-1, 1:-1] = dz
    assert np.allclose(flat.conv_wgrad(x, dz, pad=0), flat.conv_wgrad(x, full), atol=1e-12)


@pytest.mark.parametrize("grid", [(1, 2, 2), (1, 1, 3), (2, 3, 1)])
def test_partitioning_over_h_and_w_is_transparent(rng, grid):
    """Exchange the margins, pad each tile with them, convolve each tile on its own (Sec. 2): for the 2-D kernel
    the D margins play no part, whatever the grid does along D."""
    V, w = rng.standard_normal((1, 4, 6, 6, 2)), rng.standard_normal((3, 3, 2, 3))
    dZ = rng.standard_normal((1, 4, 6, 6, 3))
    P = tiling.exchange(tiling.partition(V, grid, 1), 1)
    Pz = tiling.exchange(tiling.partition(dZ, grid, 1), 1)
    Y = np.zeros(P.shape[:7] + (3,))
    X = np.zeros(P.shape[:7] + (2,))
    dw = np.zeros((3, 3, 2, 3))
    wt = np.ascontiguousarray(np.transpose(w[::-1, ::-1], (0, 1, 3, 2)))      # mirrored taps, swapped roles
    for a, b, c in itertools.product(*(range(g) for g in grid)):
        Y[:, a, b, c, 1:-1, 1:-1, 1:-1] = flat.conv_fwd(P[:, a, b, c, 1:-1], w, pad=0)
        X[:, a, b, c, 1:-1, 1:-1, 1:-1] = flat.conv_fwd(Pz[:, a, b, c, 1:-1], wt, pad=0)
        dw += flat.conv_wgrad(P[:, a, b, c, 1:-1], Pz[:, a, b, c, 1:-1, 1:-1, 1:-1], pad=0)
    np.testing.assert_allclose(tiling.unpartition(Y, 1), flat.conv_fwd(V, w), rtol=0, atol=1e-12)
    np.testing.assert_allclose(tiling.unpartition(X, 1), flat.conv_dgrad(dZ, w), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dw, flat.conv_wgrad(V, dZ), rtol=0, atol=1e-11)


def test_pooling_against_library_and_tie_rule(rng):
    N, D = 2, 3
    x = rng.standard_normal((N, D, 4, 6, 2))
    dy = rng.standard_normal((N, D, 2, 3, 2))
    xt = slices(x).clone().requires_grad_(True)
    y = F.max_pool2d(xt, 2)
    assert np.array_equal(flat.maxpool_fwd(x), unslices(y.detach(), N, D))
    y.backward(slices(dy))
    assert np.array_equal(flat.maxpool_bwd(x, dy), unslices(xt.grad, N, D))
    z = np.zeros((1, 2, 2, 2, 1))                 # ties: first in (h, w) scan order, per slice
    g = np.full((1, 2, 1, 1, 1), 5.0)
    dx = flat.maxpool_bwd(z, g)
    assert dx[0, 0, 0, 0, 0] == 5.0 and dx[0, 1, 0, 0, 0] == 5.0 and dx.sum() == 10.0
    z[0, 0, 0, 1, 0] = z[0, 0, 1, 0, 0] = 3.0     # (0,1) comes before (1,0)
    dx = flat.maxpool_bwd(z, g)
    assert dx[0, 0, 0, 1, 0] == 5.0 and dx[0, 0].sum() == 5.0


def test_upconv_against_library_conv_transpose_and_autograd(rng):
    N, D = 2, 2
    x, u, b = rng.standard_normal((N, D, 3, 2, 3)), rng.standard_normal((2, 2, 3, 4)), rng.standard_normal(4)
    dy = rng.standard_normal((N, D, 6, 4, 4))
    xt = slices(x).clone().requires_grad_(True)
    ut = torch.from_numpy(u).permute(2, 3, 0, 1).clone().requires_grad_(True)       # [Cin,Cout,kh,kw]
    bt = torch.from_numpy(b).clone().requires_grad_(True)
    y = F.conv_transpose2d(xt, ut, bt, stride=2)
    np.testing.assert_allclose(flat.upconv_fwd(x, u, b), unslices(y.detach(), N, D), rtol=0, atol=1e-12)
    y.backward(slices(dy))
    np.testing.assert_allclose(flat.upconv_dgrad(dy, u), unslices(xt.grad, N, D), rtol=0, atol=1e-12)
    du, db = flat.upconv_wgrad(x, dy)
    np.testing.assert_allclose(du, ut.grad.permute(2, 3, 0, 1).numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(db, bt.grad.numpy(), rtol=0, atol=1e-11)
