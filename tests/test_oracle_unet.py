"""The composed U-Net oracle against torch autograd in float64 on a tiny network (CPU)."""
import numpy as np
import pytest

from oracle import unet as OU

torch = pytest.importorskip("torch")
F = torch.nn.functional


def weight_shapes(channels, in_ch, classes, convs, nd=3):
    """The weight tensors the oracle's stack reads (name, shape), written out here so that this pin owes nothing
    to the product package: `convs` 3^nd convolutions per encoder level (the first takes the previous level's
    channels), per decoder level a 2^nd transposed convolution to the skip's width and `convs` convolutions (the
    first on concat(skip, up)), and a 1^nd head."""
    plan, prev = [], in_ch
    for i, c in enumerate(channels):
        for k in range(convs):
            plan.append(("enc%d_%s" % (i, "abcd"[k]), (3,) * nd + (c if k else prev, c)))
        prev = c
    for i in reversed(range(len(channels) - 1)):
        c = channels[i]
        plan.append(("up%d" % i, (2,) * nd + (prev, c)))
        for k in range(convs):
            plan.append(("dec%d_%s" % (i, "abcd"[k]), (3,) * nd + (c if k else 2 * c, c)))
        prev = c
    plan.append(("head", (1,) * nd + (prev, classes)))
    return plan


@pytest.mark.parametrize("convs", [2, 4, 1])
def test_unet_oracle_matches_torch_autograd(rng, convs):
    channels, in_ch, classes = (2, 3, 4), 1, 2
    plan = weight_shapes(channels, in_ch, classes, convs)
    w = {name: rng.standard_normal(shape) * 0.4 for name, shape in plan}
    x = rng.standard_normal((1, 4, 8, 4, in_ch))
    dl = rng.standard_normal((1, 4, 8, 4, classes))

    A = {}
    logits = OU.forward(x, w, channels, keep=A, convs=convs)
    grads, dx = OU.backward(dl, w, channels, A, convs=convs)

    tw = {k: torch.from_numpy(v).clone().requires_grad_(True) for k, v in w.items()}
    xt = torch.from_numpy(x).permute(0, 4, 1, 2, 3).clone().requires_grad_(True)

    def conv(h, name):
        return F.relu(F.conv3d(h, tw[name].permute(4, 3, 0, 1, 2), padding=1))

    h, skips = xt, []
    for i in range(len(channels)):
        if i > 0:
            h = F.max_pool3d(h, 2)
        for k in range(convs):
            h = conv(h, "enc%d_%s" % (i, "abcd"[k]))
        skips.append(h)
    for i in range(len(channels) - 2, -1, -1):
        up = F.conv_transpose3d(h, tw["up%d" % i].permute(3, 4, 0, 1, 2), stride=2)
        h = torch.cat([skips[i], up], dim=1)
        for k in range(convs):
            h = conv(h, "dec%d_%s" % (i, "abcd"[k]))
    out = F.conv3d(h, tw["head"].permute(4, 3, 0, 1, 2))
    np.testing.assert_allclose(logits, out.detach().permute(0, 2, 3, 4, 1).numpy(), atol=1e-10)
    out.backward(torch.from_numpy(dl).permute(0, 4, 1, 2, 3))
    np.testing.assert_allclose(dx, xt.grad.permute(0, 2, 3, 4, 1).numpy(), atol=1e-10)
    for name, _ in plan:
        np.testing.assert_allclose(grads[name], tw[name].grad.numpy(), atol=1e-10, err_msg=name)


@pytest.mark.parametrize("convs", [2, 3])
def test_flat_unet_oracle_matches_torch_autograd(rng, convs):
    """the 2-D variant: the library's 3-D routines with kernels / windows of extent 1 along D"""
    channels, in_ch, classes = (2, 3, 4), 5, 2
    plan = weight_shapes(channels, in_ch, classes, convs, nd=2)
    w = {name: rng.standard_normal(shape) * 0.4 for name, shape in plan}
    x = rng.standard_normal((1, 3, 8, 4, in_ch))
    dl = rng.standard_normal((1, 3, 8, 4, classes))
    A = {}
    logits = OU.forward(x, w, channels, keep=A, convs=convs, flat=True)
    grads, dx = OU.backward(dl, w, channels, A, convs=convs, flat=True)

    tw = {k: torch.from_numpy(v).clone().requires_grad_(True) for k, v in w.items()}
    xt = torch.from_numpy(x).permute(0, 4, 1, 2, 3).clone().requires_grad_(True)

    def conv(h, name):
        return F.relu(F.conv3d(h, tw[name].permute(3, 2, 0, 1)[:, :, None], padding=(0, 1, 1)))

    h, skips = xt, []
    for i in range(len(channels)):
        if i > 0:
            h = F.max_pool3d(h, (1, 2, 2))
        for k in range(convs):
            h = conv(h, "enc%d_%s" % (i, "abcd"[k]))
        skips.append(h)
    for i in range(len(channels) - 2, -1, -1):
        up = F.conv_transpose3d(h, tw["up%d" % i].permute(2, 3, 0, 1)[:, :, None], stride=(1, 2, 2))
        h = torch.cat([skips[i], up], dim=1)
        for k in range(convs):
            h = conv(h, "dec%d_%s" % (i, "abcd"[k]))
    out = F.conv3d(h, tw["head"].permute(3, 2, 0, 1)[:, :, None])
    np.testing.assert_allclose(logits, out.detach().permute(0, 2, 3, 4, 1).numpy(), atol=1e-10)
    out.backward(torch.from_numpy(dl).permute(0, 4, 1, 2, 3))
    np.testing.assert_allclose(dx, xt.grad.permute(0, 2, 3, 4, 1).numpy(), atol=1e-10)
    for name, _ in plan:
        np.testing.assert_allclose(grads[name], tw[name].grad.numpy(), atol=1e-10, err_msg=name)


def test_round_bf16_matches_torch():
    a = np.random.default_rng(3).standard_normal(5000) * 13
    ref = torch.from_numpy(a).float().to(torch.bfloat16).double().numpy()
    assert np.array_equal(OU.round_bf16(a), ref)
