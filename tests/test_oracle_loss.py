"""Pins of the loss oracle (CPU): library cross-entropy, closed forms of the Dice term, finite differences."""
import numpy as np
import pytest

from oracle import loss as OL

torch = pytest.importorskip("torch")


def case(rng, shape=(2, 3, 4, 5), C=3):
    z = rng.standard_normal(shape + (C,)) * 2.0
    lab = rng.integers(0, C, size=shape)
    return z, lab


def test_cross_entropy_term_is_the_library_cross_entropy(rng):
    z, lab = case(rng)
    ours = OL.loss(z, lab, w_dice=0.0, w_ce=1.0)
    ref = torch.nn.functional.cross_entropy(torch.from_numpy(z).reshape(-1, 3), torch.from_numpy(lab).reshape(-1))
    assert abs(ours - ref.item()) < 1e-12
    zt = torch.from_numpy(z).clone().requires_grad_(True)
    torch.nn.functional.cross_entropy(zt.reshape(-1, 3), torch.from_numpy(lab).reshape(-1)).backward()
    np.testing.assert_allclose(OL.gradient(z, lab, w_dice=0.0, w_ce=1.0), zt.grad.numpy(), atol=1e-13)


def test_dice_term_closed_forms():
    C, V = 3, 60
    lab = np.arange(V) % C
    # a confident, correct prediction: p -> one-hot, Dice_c -> (2 n_c + eps) / (2 n_c + eps) = 1, loss -> 0
    z = 60.0 * OL.one_hot(lab, C)
    assert abs(OL.loss(z, lab, 1.0, 0.0)) < 1e-12
    # uniform prediction: p = 1/C, I_c = n_c / C, P_c = V / C, Y_c = n_c  (n_c = V / C = 20)
    z = np.zeros((V, C))
    n = V / C
    dice = (2 * n / C + 1.0) / (V / C + n + 1.0)
    assert abs(OL.loss(z, lab, 1.0, 0.0) - (1.0 - dice)) < 1e-12
    # a confident, wrong prediction (every voxel assigned the next class): I_c = 0
    z = 60.0 * OL.one_hot((lab + 1) % C, C)
    assert abs(OL.loss(z, lab, 1.0, 0.0, eps=1.0) - (1.0 - 1.0 / (2 * n + 1.0))) < 1e-9
    # eps = 0 and an absent class would divide by zero for that class only if p is exactly 0 there: finite otherwise
    assert np.isfinite(OL.loss(np.zeros((V, C)), np.zeros(V, dtype=int), 1.0, 0.0, eps=1.0))


def test_statistics_are_sums_over_all_voxels(rng):
    z, lab = case(rng)
    I, P, Y, nll = OL.stats(z, lab)
    assert abs(P.sum() - lab.size) < 1e-9                       # probabilities of a voxel sum to one
    assert np.array_equal(Y, np.bincount(lab.ravel(), minlength=3).astype(float))
    assert np.all(I <= np.minimum(P, Y) + 1e-12) and nll > 0
    # splitting the volume in two (two "tiles") and adding the statistics gives the same loss
    a, b = OL.stats(z[:1], lab[:1]), OL.stats(z[1:], lab[1:])
    for u, v, w in zip(a, b, (I, P, Y, nll)):
        np.testing.assert_allclose(u + v, w, rtol=1e-13)


@pytest.mark.parametrize("w_dice,w_ce,eps", [(0.9, 0.1, 1.0), (1.0, 0.0, 1.0), (0.5, 0.5, 1e-3)])
def test_gradient_matches_central_differences(rng, w_dice, w_ce, eps):
    z, lab = case(rng, shape=(1, 2, 3, 3))
    g = OL.gradient(z, lab, w_dice, w_ce, eps)
    num = np.zeros_like(z)
    h = 1e-6
    it = np.nditer(z, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        zp, zm = z.copy(), z.copy()
        zp[i] += h
        zm[i] -= h
        num[i] = (OL.loss(zp, lab, w_dice, w_ce, eps) - OL.loss(zm, lab, w_dice, w_ce, eps)) / (2 * h)
    np.testing.assert_allclose(g, num, atol=2e-9)
    # softmax is shift-invariant, so the gradient of every voxel sums to zero over the classes
    assert np.abs(g.sum(axis=-1)).max() < 1e-15


def test_whole_formula_against_autograd_of_an_independent_expression(rng):
    z, lab = case(rng)
    zt = torch.from_numpy(z).clone().requires_grad_(True)
    logp = torch.log_softmax(zt, dim=-1)
    y = torch.nn.functional.one_hot(torch.from_numpy(lab), 3).double()
    p = logp.exp()
    dims = (0, 1, 2, 3)
    dice = (2 * (p * y).sum(dims) + 1.0) / (p.sum(dims) + y.sum(dims) + 1.0)
    L = 0.9 * (1 - dice.mean()) + 0.1 * (-(logp * y).sum(-1)).mean()
    L.backward()
    assert abs(OL.loss(z, lab) - L.item()) < 1e-12
    np.testing.assert_allclose(OL.gradient(z, lab), zt.grad.numpy(), atol=1e-13)
