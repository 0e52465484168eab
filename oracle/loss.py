"""numpy fp64 oracle of the segmentation loss and its gradient (test infrastructure only).

The paper trains with 0.9 x Dice + 0.1 x cross-entropy (Sec. 3, training set-up) and gives no formula.
Reading taken here (the usual soft form of both terms):

  p[v, c]  = softmax over the classes of the logits z[v, :]            v = every voxel of every volume
  CE       = -(1 / V) * sum_v log p[v, label[v]]
  Dice_c   = (2 * sum_v p[v, c] y[v, c] + eps) / (sum_v p[v, c] + sum_v y[v, c] + eps),   y = one-hot label
  loss     = w_dice * (1 - mean_c Dice_c) + w_ce * CE                  (w_dice, w_ce, eps) = (0.9, 0.1, 1)

The sums run over the whole volume, i.e. over all tiles: this is the path's cross-tile reduction.
gradient() is d loss / d z, derived by hand from the definition (quotient rule for Dice_c, then the
softmax Jacobian), not by automatic differentiation.
"""
import numpy as np


def softmax(z):
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(z - z.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def one_hot(labels, classes):
    lab = np.asarray(labels).astype(np.int64)
    assert lab.min() >= 0 and lab.max() < classes
    return (lab[..., None] == np.arange(classes)).astype(np.float64)


def stats(z, labels):
    """per class: I_c = sum p y, P_c = sum p, Y_c = sum y; and the summed -log p[label]."""
    C = np.asarray(z).shape[-1]
    p = softmax(z).reshape(-1, C)
    y = one_hot(labels, C).reshape(-1, C)
    nll = -np.log((p * y).sum(axis=1)).sum()
    return (p * y).sum(axis=0), p.sum(axis=0), y.sum(axis=0), nll


def loss(z, labels, w_dice=0.9, w_ce=0.1, eps=1.0):
    I, P, Y, nll = stats(z, labels)
    V = np.asarray(labels).size
    dice = (2.0 * I + eps) / (P + Y + eps)
    return w_dice * (1.0 - dice.mean()) + w_ce * nll / V


def gradient(z, labels, w_dice=0.9, w_ce=0.1, eps=1.0):
    """d loss / d z, same shape as z."""
    z = np.asarray(z, dtype=np.float64)
    C = z.shape[-1]
    p = softmax(z)
    y = one_hot(labels, C)
    I, P, Y, _ = stats(z, labels)
    V = np.asarray(labels).size
    S = P + Y + eps
    # d loss / d p[v, c]: Dice_c = (2 I_c + eps) / S_c, dI_c/dp = y, dS_c/dp = 1
    g = -(w_dice / C) * (2.0 * y * S - (2.0 * I + eps)) / (S * S)
    # through the softmax: dL/dz_k = p_k (g_k - sum_c g_c p_c); cross-entropy adds (p - y) / V
    return p * (g - (g * p).sum(axis=-1, keepdims=True)) + w_ce * (p - y) / V
