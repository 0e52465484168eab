"""The synthetic-input module: reproducible, slab-seeded, rounded to the storage type."""
import numpy as np
import pytest

from paper_1909_03108_amd import synth


def test_bf16_rounding_matches_torch_rne():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(1)
    a = np.concatenate([rng.standard_normal(4096).astype(np.float32) * 37,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38, 1e-40],
                                 dtype=np.float32)])
    ours = synth.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    assert np.array_equal(synth.bf16_bits_to_f32(ours),
                          torch.from_numpy(a).to(torch.bfloat16).float().numpy())


def test_slab_seeding_is_reproducible_and_thread_independent(monkeypatch):
    a = synth.normal_volume((1, 6, 4, 5, 3), 7, "f32")
    monkeypatch.setattr(synth, "_workers", lambda: 1)
    b = synth.normal_volume((1, 6, 4, 5, 3), 7, "f32")
    assert np.array_equal(a, b)
    assert not np.array_equal(a[0, 0], a[0, 1])
    assert not np.array_equal(a, synth.normal_volume((1, 6, 4, 5, 3), 8, "f32"))


def test_distributions():
    x = synth.normal_volume((1, 16, 16, 16, 8), 3, "f32")
    assert abs(x.mean()) < 0.02 and abs(x.std() - 1) < 0.02
    w = synth.bf16_bits_to_f32(synth.weights(32, 32, 5, "bf16"))
    assert w.shape == (3, 3, 3, 32, 32)
    assert abs(w.std() / np.sqrt(2.0 / (27 * 32)) - 1) < 0.03
    ct = synth.bf16_bits_to_f32(synth.ct_like_volume((1, 16, 16, 16, 1), 9, "bf16"))
    assert ct.min() >= -1 and ct.max() <= 1 and ct.std() > 0.3


def test_config_tensors_small():
    x, ws, dy = synth.config_tensors(2, dhw=(8, 8, 8))
    assert x.shape == (1, 8, 8, 8, 32) and x.dtype == np.uint16
    assert [w.shape for w in ws] == [(3, 3, 3, 32, 32)] * 2 and dy.shape == x.shape
    x1, ws1, _ = synth.config_tensors(1, dhw=(4, 4, 4))
    assert x1.dtype == np.float32 and ws1[0].shape == (3, 3, 3, 8, 16)
