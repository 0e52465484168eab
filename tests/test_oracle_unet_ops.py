"""Pins of the U-Net glue oracle: library routines (torch float64 and its autograd), hand-built
windows for the tie rule, brute-force loops, and adjoint identities."""
import itertools

import numpy as np
import pytest

from oracle import unet_ops as U

torch = pytest.importorskip("torch")
F = torch.nn.functional


def t(x):            # NDHWC numpy -> NCDHW torch
    return torch.from_numpy(np.ascontiguousarray(x)).permute(0, 4, 1, 2, 3)


def n(x):            # back
    return x.permute(0, 2, 3, 4, 1).contiguous().numpy()


def test_maxpool_forward_against_torch_and_brute_force(rng):
    x = rng.standard_normal((2, 4, 6, 2, 3))
    y = U.maxpool2_fwd(x)
    assert np.array_equal(y, n(F.max_pool3d(t(x), 2)))
    for nn_, d, h, w, c in itertools.product(range(2), range(2), range(3), range(1), range(3)):
        win = [x[nn_, 2 * d + a, 2 * h + b, 2 * w + cc, c] for a in range(2) for b in range(2) for cc in range(2)]
        assert y[nn_, d, h, w, c] == max(win)


def test_maxpool_backward_without_ties_matches_autograd(rng):
    x = rng.standard_normal((1, 4, 4, 6, 2))
    dy = rng.standard_normal((1, 2, 2, 3, 2))
    xt = t(x).clone().requires_grad_(True)
    F.max_pool3d(xt, 2).backward(t(dy))
    assert np.array_equal(U.maxpool2_bwd(x, dy), n(xt.grad))


def test_maxpool_backward_tie_rule_first_in_scan_order():
    x = np.zeros((1, 2, 2, 2, 1))                 # all equal: the gradient goes to (0,0,0)
    dy = np.full((1, 1, 1, 1, 1), 5.0)
    dx = U.maxpool2_bwd(x, dy)
    assert dx[0, 0, 0, 0, 0] == 5.0 and dx.sum() == 5.0
    x[0, 0, 1, 1, 0] = 3.0
    x[0, 1, 0, 0, 0] = 3.0                        # two maxima: (0,1,1) comes before (1,0,0)
    dx = U.maxpool2_bwd(x, dy)
    assert dx[0, 0, 1, 1, 0] == 5.0 and dx.sum() == 5.0
    x[0, 0, 0, 1, 0] = 3.0                        # (0,0,1) is earlier still
    assert U.maxpool2_bwd(x, dy)[0, 0, 0, 1, 0] == 5.0


def test_upconv_against_torch_conv_transpose_and_autograd(rng):
    x, u, b = rng.standard_normal((2, 2, 3, 2, 3)), rng.standard_normal((2, 2, 2, 3, 4)), rng.standard_normal(4)
    dy = rng.standard_normal((2, 4, 6, 4, 4))
    xt = t(x).clone().requires_grad_(True)
    wt = torch.from_numpy(u).permute(3, 4, 0, 1, 2).clone().requires_grad_(True)      # [Cin,Cout,kd,kh,kw]
    bt = torch.from_numpy(b).clone().requires_grad_(True)
    y = F.conv_transpose3d(xt, wt, bt, stride=2)
    np.testing.assert_allclose(U.upconv2_fwd(x, u, b), n(y.detach()), atol=1e-12)
    y.backward(t(dy))
    np.testing.assert_allclose(U.upconv2_dgrad(dy, u), n(xt.grad), atol=1e-12)
    du, db = U.upconv2_wgrad(x, dy)
    np.testing.assert_allclose(du, wt.grad.permute(2, 3, 4, 0, 1).numpy(), atol=1e-12)
    np.testing.assert_allclose(db, bt.grad.numpy(), atol=1e-12)


def test_upconv_one_hot_places_the_voxel_in_its_window_slot():
    x = np.zeros((1, 1, 1, 2, 1))
    x[0, 0, 0, 1, 0] = 7.0
    for a, b, c in itertools.product(range(2), repeat=3):
        u = np.zeros((2, 2, 2, 1, 1))
        u[a, b, c, 0, 0] = 1.0
        y = U.upconv2_fwd(x, u)
        assert y[0, a, b, 2 + c, 0] == 7.0 and y.sum() == 7.0


def test_pointwise_against_torch(rng):
    x, p, b = rng.standard_normal((1, 2, 3, 4, 5)), rng.standard_normal((5, 3)), rng.standard_normal(3)
    dy = rng.standard_normal((1, 2, 3, 4, 3))
    xt = t(x).clone().requires_grad_(True)
    wt = torch.from_numpy(p.T.copy())[:, :, None, None, None].clone().requires_grad_(True)
    y = F.conv3d(xt, wt, torch.from_numpy(b))
    np.testing.assert_allclose(U.pointwise_fwd(x, p, b), n(y.detach()), atol=1e-12)
    y.backward(t(dy))
    np.testing.assert_allclose(U.pointwise_dgrad(dy, p), n(xt.grad), atol=1e-12)
    dp, db = U.pointwise_wgrad(x, dy)
    np.testing.assert_allclose(dp, wt.grad[:, :, 0, 0, 0].numpy().T, atol=1e-12)
    np.testing.assert_allclose(db, dy.sum(axis=(0, 1, 2, 3)), atol=1e-12)


def test_adjoint_identities(rng):
    x, u = rng.standard_normal((1, 2, 2, 3, 2)), rng.standard_normal((2, 2, 2, 2, 3))
    g = rng.standard_normal((1, 4, 4, 6, 3))
    lhs = np.vdot(U.upconv2_fwd(x, u), g)
    assert abs(lhs - np.vdot(x, U.upconv2_dgrad(g, u))) < 1e-11
    assert abs(lhs - np.vdot(u, U.upconv2_wgrad(x, g)[0])) < 1e-11
    xf, gy = rng.standard_normal((1, 4, 4, 2, 2)), rng.standard_normal((1, 2, 2, 1, 2))
    # max-pool is linear once the argmax pattern is fixed: <pool(x), g> = <x, pool_bwd(x, g)>
    assert abs(np.vdot(U.maxpool2_fwd(xf), gy) - np.vdot(xf, U.maxpool2_bwd(xf, gy))) < 1e-12


def test_concat_split_roundtrip(rng):
    a, b = rng.standard_normal((1, 2, 2, 2, 3)), rng.standard_normal((1, 2, 2, 2, 5))
    c = U.concat(a, b)
    assert c.shape[-1] == 8 and np.array_equal(c[..., :3], a) and np.array_equal(c[..., 3:], b)
    a2, b2 = U.split(c, 3)
    assert np.array_equal(a2, a) and np.array_equal(b2, b)
