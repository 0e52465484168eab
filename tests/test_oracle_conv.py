"""Pins of the fp64 convolution oracle against facts that do not come from the oracle:
closed forms, special kernels, a library routine, an independent brute force, and the
adjoint / finite-difference identities that tie dgrad and wgrad to the forward pass."""
import itertools

import numpy as np
import pytest

from oracle import brute, conv3d

TAPS = list(itertools.product(range(3), repeat=3))


def rand(rng, *shape):
    return rng.standard_normal(shape)


# ---------------------------------------------------------------- forward definition
@pytest.mark.parametrize("dhw,cin,cout", [((1, 1, 1), 1, 1), ((1, 2, 3), 2, 1), ((2, 1, 4), 1, 3),
                                          ((3, 3, 3), 2, 2), ((4, 2, 5), 3, 2), ((5, 4, 2), 1, 2)])
def test_fwd_vs_scatter_brute_force(rng, dhw, cin, cout):
    x = rand(rng, 2, *dhw, cin)
    w = rand(rng, 3, 3, 3, cin, cout)
    b = rand(rng, cout)
    ref = np.array(brute.conv3d_same_scatter(x.tolist(), w.tolist(), b.tolist()))
    np.testing.assert_allclose(conv3d.conv3d_fwd(x, w, b), ref, rtol=0, atol=1e-12)


def test_identity_kernel_returns_input_exactly(rng):
    x = rand(rng, 1, 4, 5, 6, 3)
    w = np.zeros((3, 3, 3, 3, 3))
    w[1, 1, 1] = np.eye(3)
    assert np.array_equal(conv3d.conv3d_fwd(x, w), x)


@pytest.mark.parametrize("tap", [t for t in TAPS if t != (1, 1, 1)])
def test_shift_kernels_move_the_volume_with_zero_fill(rng, tap):
    """A one-hot tap (kd,kh,kw) with identity channels reads x at offset tap-1: this fixes
    the cross-correlation (no flip) convention and the zero fill, one direction at a time."""
    D, H, W, C = 4, 3, 5, 2
    x = rand(rng, 1, D, H, W, C)
    w = np.zeros((3, 3, 3, C, C))
    w[tap] = np.eye(C)
    expect = np.zeros_like(x)
    for d, h, ww in itertools.product(range(D), range(H), range(W)):
        s = (d + tap[0] - 1, h + tap[1] - 1, ww + tap[2] - 1)
        if 0 <= s[0] < D and 0 <= s[1] < H and 0 <= s[2] < W:
            expect[0, d, h, ww] = x[0, s[0], s[1], s[2]]
    assert np.array_equal(conv3d.conv3d_fwd(x, w), expect)


@pytest.mark.parametrize("dhw", [(1, 1, 1), (2, 2, 2), (1, 4, 3), (5, 4, 6)])
def test_all_ones_closed_form(dhw):
    """x = 1, w = 1: every output counts the taps that fall inside the volume times Cin."""
    cin, cout = 3, 2
    D, H, W = dhw
    y = conv3d.conv3d_fwd(np.ones((1, D, H, W, cin)), np.ones((3, 3, 3, cin, cout)))

    def cnt(a, A):
        return 3 - (a == 0) - (a == A - 1)

    for d, h, ww in itertools.product(range(D), range(H), range(W)):
        assert np.all(y[0, d, h, ww] == cin * cnt(d, D) * cnt(h, H) * cnt(ww, W))


def test_separable_case_against_numpy_correlate(rng):
    """x = a(d) b(h) c(w), w = p (x) q (x) r: y is the product of three 1-D 'same' correlations."""
    a, b, c = rand(rng, 6), rand(rng, 5), rand(rng, 7)
    p, q, r = rand(rng, 3), rand(rng, 3), rand(rng, 3)
    x = np.einsum("d,h,w->dhw", a, b, c)[None, ..., None]
    w = np.einsum("i,j,k->ijk", p, q, r)[..., None, None]
    ya, yb, yc = (np.correlate(v, k, mode="same") for v, k in ((a, p), (b, q), (c, r)))
    np.testing.assert_allclose(conv3d.conv3d_fwd(x, w)[0, ..., 0],
                               np.einsum("d,h,w->dhw", ya, yb, yc), rtol=0, atol=1e-12)


def test_linearity_in_x_and_w(rng):
    x1, x2 = rand(rng, 1, 3, 4, 5, 2), rand(rng, 1, 3, 4, 5, 2)
    w1, w2 = rand(rng, 3, 3, 3, 2, 3), rand(rng, 3, 3, 3, 2, 3)
    f = conv3d.conv3d_fwd
    np.testing.assert_allclose(f(2 * x1 - 3 * x2, w1), 2 * f(x1, w1) - 3 * f(x2, w1), atol=1e-12)
    np.testing.assert_allclose(f(x1, 2 * w1 - 3 * w2), 2 * f(x1, w1) - 3 * f(x1, w2), atol=1e-12)


def test_fwd_against_torch_conv3d_float64(rng):
    torch = pytest.importorskip("torch")
    x, w, b = rand(rng, 2, 5, 6, 7, 3), rand(rng, 3, 3, 3, 3, 4), rand(rng, 4)
    ref = torch.nn.functional.conv3d(torch.from_numpy(x).permute(0, 4, 1, 2, 3),
                                     torch.from_numpy(w).permute(4, 3, 0, 1, 2),
                                     torch.from_numpy(b), padding=1)
    np.testing.assert_allclose(conv3d.conv3d_fwd(x, w, b), ref.permute(0, 2, 3, 4, 1).numpy(),
                               rtol=0, atol=1e-12)


def test_relu_and_bias(rng):
    x, w, b = rand(rng, 1, 3, 3, 3, 2), rand(rng, 3, 3, 3, 2, 2), rand(rng, 2)
    z = conv3d.conv3d_fwd(x, w, b)
    assert np.array_equal(conv3d.conv3d_fwd(x, w, b, relu=True), np.maximum(z, 0))
    np.testing.assert_allclose(z - conv3d.conv3d_fwd(x, w), np.broadcast_to(b, z.shape), atol=1e-12)


def test_box_selects_the_same_values(rng):
    x, w = rand(rng, 2, 6, 5, 7, 2), rand(rng, 3, 3, 3, 2, 3)
    full = conv3d.conv3d_fwd(x, w)
    box = (1, 5, 0, 3, 2, 7)
    assert np.array_equal(conv3d.conv3d_fwd(x, w, box=box), full[:, 1:5, 0:3, 2:7])
    g = rand(rng, 2, 6, 5, 7, 3)
    assert np.array_equal(conv3d.conv3d_dgrad(g, w, box=box), conv3d.conv3d_dgrad(g, w)[:, 1:5, 0:3, 2:7])


def test_valid_mode_equals_same_mode_on_prepadded_input(rng):
    x, w = rand(rng, 1, 4, 5, 3, 2), rand(rng, 3, 3, 3, 2, 2)
    xp = np.pad(x, ((0, 0), (1, 1), (1, 1), (1, 1), (0, 0)))
    assert np.array_equal(conv3d.conv3d_fwd(xp, w, pad=0), conv3d.conv3d_fwd(x, w, pad=1))


def test_storage_dtypes_widen_exactly(rng):
    """f32 and bf16-bit inputs give bit-identical results to the same values passed as f64."""
    x32 = rand(rng, 1, 3, 4, 5, 2).astype(np.float32)
    bits = (x32.view(np.uint32) >> 16).astype(np.uint16)          # truncate: any bf16 pattern
    xbf = (bits.astype(np.uint32) << 16).view(np.float32)
    w = rand(rng, 3, 3, 3, 2, 3)
    assert np.array_equal(conv3d.conv3d_fwd(x32, w), conv3d.conv3d_fwd(x32.astype(np.float64), w))
    assert np.array_equal(conv3d.conv3d_fwd(bits, w), conv3d.conv3d_fwd(xbf.astype(np.float64), w))
    assert np.array_equal(conv3d.bf16_bits_to_f64(bits), xbf.astype(np.float64))


# ---------------------------------------------------------------- backward passes
@pytest.mark.parametrize("dhw,cin,cout", [((1, 1, 1), 1, 1), ((2, 3, 1), 2, 3), ((4, 3, 5), 3, 2)])
def test_adjoint_identities(rng, dhw, cin, cout):
    """<fwd(x,w), g> = <x, dgrad(g,w)> = <w, wgrad(x,g)>: exact in exact arithmetic."""
    x, w, g = rand(rng, 2, *dhw, cin), rand(rng, 3, 3, 3, cin, cout), rand(rng, 2, *dhw, cout)
    lhs = np.vdot(conv3d.conv3d_fwd(x, w), g)
    assert abs(lhs - np.vdot(x, conv3d.conv3d_dgrad(g, w))) <= 1e-11 * max(1, abs(lhs))
    assert abs(lhs - np.vdot(w, conv3d.conv3d_wgrad(x, g))) <= 1e-11 * max(1, abs(lhs))


def test_dgrad_against_torch_autograd(rng):
    torch = pytest.importorskip("torch")
    x, w, g = rand(rng, 1, 4, 3, 5, 2), rand(rng, 3, 3, 3, 2, 3), rand(rng, 1, 4, 3, 5, 3)
    xt = torch.from_numpy(x).permute(0, 4, 1, 2, 3).clone().requires_grad_(True)
    wt = torch.from_numpy(w).permute(4, 3, 0, 1, 2).clone().requires_grad_(True)
    y = torch.nn.functional.conv3d(xt, wt, padding=1)
    y.backward(torch.from_numpy(g).permute(0, 4, 1, 2, 3))
    np.testing.assert_allclose(conv3d.conv3d_dgrad(g, w), xt.grad.permute(0, 2, 3, 4, 1).numpy(),
                               atol=1e-12)
    np.testing.assert_allclose(conv3d.conv3d_wgrad(x, g), wt.grad.permute(2, 3, 4, 1, 0).numpy(),
                               atol=1e-12)
    np.testing.assert_allclose(conv3d.bias_grad(g), g.sum(axis=(0, 1, 2, 3)), atol=1e-12)


def test_central_finite_differences(rng):
    """L = <fwd(x,w), g> is bilinear, so central differences are exact up to rounding."""
    x, w, g = rand(rng, 1, 3, 2, 3, 2), rand(rng, 3, 3, 3, 2, 2), rand(rng, 1, 3, 2, 3, 2)
    dx, dw = conv3d.conv3d_dgrad(g, w), conv3d.conv3d_wgrad(x, g)
    eps = 1e-3

    def L(xx, ww):
        return np.vdot(conv3d.conv3d_fwd(xx, ww), g)

    for idx in [(0, 0, 0, 0, 0), (0, 2, 1, 2, 1), (0, 1, 0, 1, 0)]:
        e = np.zeros_like(x)
        e[idx] = eps
        assert abs((L(x + e, w) - L(x - e, w)) / (2 * eps) - dx[idx]) < 1e-9
    for idx in [(0, 0, 0, 0, 0), (2, 2, 2, 1, 1), (1, 0, 2, 0, 1), (1, 1, 1, 1, 0)]:
        e = np.zeros_like(w)
        e[idx] = eps
        assert abs((L(x, w + e) - L(x, w - e)) / (2 * eps) - dw[idx]) < 1e-9


def test_wgrad_selection_and_valid_mode(rng):
    x, g = rand(rng, 1, 3, 4, 2, 2), rand(rng, 1, 3, 4, 2, 3)
    full = conv3d.conv3d_wgrad(x, g)
    sel = np.array([0, 7, 53, 27 * 6 - 1])
    assert np.array_equal(conv3d.conv3d_wgrad(x, g, sel=sel), full.ravel()[sel])
    xp = np.pad(x, ((0, 0), (1, 1), (1, 1), (1, 1), (0, 0)))
    assert np.array_equal(conv3d.conv3d_wgrad(xp, g, pad=0), full)


def test_relu_backward_rule():
    y = np.array([0.0, 1.0, 0.0, 2.0])
    dy = np.array([5.0, 6.0, -7.0, -8.0])
    assert np.array_equal(conv3d.relu_bwd(dy, y), np.array([0.0, 6.0, 0.0, -8.0]))
