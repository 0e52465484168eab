"""Seeded synthetic inputs shaped like the paper's CT workloads.

This module only *draws numbers and rounds them to the storage type*; it holds
none of the method's arithmetic and imports neither the GPU library nor the CPU
oracle, so both sides can be fed the very same arrays.

The paper trains on CT volumes of up to 512^3 voxels with a first block of 32
filters (Sec. 3); those scans are not available here, so every tensor is drawn
from a seeded generator with the same shape:

* activations and upstream gradients ~ N(0,1);
* weights ~ N(0, 2 / (27 Cin)) (He initialisation) unless a variance is given;
* "CT-like" single-channel volumes: Hounsfield-like values uniform in
  [-1000, 1000] plus eight Gaussian blobs, clipped to [-1000, 1000] and scaled
  to [-1, 1].

Large tensors are drawn slab by slab along D, each slab from its own generator
(`numpy.random.Generator(PCG64(SeedSequence([seed, slab])))`), so the values do not
depend on how many threads draw them.
"""
from concurrent.futures import ThreadPoolExecutor
import os

import numpy as np

BASE_SEED = 190903108

# tensor ids inside one configuration
T_INPUT, T_WEIGHT0, T_UPSTREAM = 0, 1, 50


def seed_for(config, tensor):
    """Seed of tensor `tensor` of configuration `config` (1-based, as in the config list)."""
    return BASE_SEED + 100 * int(config) + int(tensor)


def f32_to_bf16_bits(a):
    """Round float32 to bf16 (round to nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    # NaNs never occur in the generated data; plain RNE on the bit pattern
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(u):
    return (np.ascontiguousarray(u, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(
        np.float32)


def _workers():
    return max(1, min(16, len(os.sched_getaffinity(0))))


def _store(a, dtype):
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    raise ValueError(dtype)


def _np_dtype(dtype):
    return {"bf16": np.uint16, "f32": np.float32}[dtype]


def normal_volume(shape, seed, dtype="bf16", std=1.0):
    """N(0, std^2) tensor [N,D,H,W,C], drawn per (n, d)-slab; stored as f32 or bf16 bits."""
    N, D, H, W, C = shape
    out = np.empty(shape, dtype=_np_dtype(dtype))

    def slab(i):
        n, d = divmod(i, D)
        g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, i])))
        a = g.standard_normal((H, W, C), dtype=np.float32)
        if std != 1.0:
            a *= np.float32(std)
        out[n, d] = _store(a, dtype)

    with ThreadPoolExecutor(_workers()) as ex:
        list(ex.map(slab, range(N * D)))
    return out


def weights(cin, cout, seed, dtype="bf16", var=None, taps=(3, 3, 3)):
    """w[kd,kh,kw,Cin,Cout] ~ N(0, var); var defaults to He's 2 / (taps Cin)."""
    ntaps = int(np.prod(taps))
    if var is None:
        var = 2.0 / (ntaps * cin)
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed])))
    a = g.standard_normal(tuple(taps) + (cin, cout), dtype=np.float32) * np.float32(np.sqrt(var))
    return _store(a, dtype)


def ct_like_volume(shape, seed, dtype="bf16"):
    """Single-channel CT-like volume [N,D,H,W,1] in [-1,1]: uniform Hounsfield-like noise
    plus eight Gaussian blobs (amplitude +-U(200,800), sigma U(8,32) voxels scaled to the
    volume size), clipped to [-1000,1000] and divided by 1000."""
    N, D, H, W, C = shape
    assert C == 1
    out = np.empty(shape, dtype=_np_dtype(dtype))
    gb = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 1 << 30])))
    scale = max(D, H, W) / 256.0
    nb = 8
    amp = gb.uniform(200.0, 800.0, (N, nb)) * gb.choice([-1.0, 1.0], (N, nb))
    sig = gb.uniform(8.0, 32.0, (N, nb)) * scale
    cen = gb.uniform(0.0, 1.0, (N, nb, 3)) * np.array([D, H, W])
    hh = np.arange(H, dtype=np.float32)[:, None]
    ww = np.arange(W, dtype=np.float32)[None, :]

    def slab(i):
        n, d = divmod(i, D)
        g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, i])))
        a = g.uniform(-1000.0, 1000.0, (H, W)).astype(np.float32)
        for b in range(nb):
            r2 = (d - cen[n, b, 0]) ** 2 + (hh - cen[n, b, 1]) ** 2 + (ww - cen[n, b, 2]) ** 2
            a += np.float32(amp[n, b]) * np.exp(-r2 / np.float32(2.0 * sig[n, b] ** 2))
        np.clip(a, -1000.0, 1000.0, out=a)
        a /= np.float32(1000.0)
        out[n, d, :, :, 0] = _store(a, dtype)

    with ThreadPoolExecutor(_workers()) as ex:
        list(ex.map(slab, range(N * D)))
    return out


# The five workload configurations (shapes, grids and dtypes) used by tests and bench.
CONFIGS = {
    1: dict(name="c1_fp32_32^3_8to16", n=1, dhw=(32, 32, 32), grid=(2, 2, 1), halo=1,
            dtype="f32", layers=[(8, 16)], relu=[False], passes=("fwd",),
            input="normal", wvar=[1.0 / (27 * 8)]),
    2: dict(name="c2_bf16_128^3_32to32x2", n=1, dhw=(128, 128, 128), grid=(4, 4, 1), halo=1,
            dtype="bf16", layers=[(32, 32), (32, 32)], relu=[True, False],
            passes=("fwd", "dgrad", "wgrad"), input="normal", wvar=[None, None]),
    3: dict(name="c3_bf16_256^3_1to32to32", n=1, dhw=(256, 256, 256), grid=(4, 4, 2), halo=1,
            dtype="bf16", layers=[(1, 32), (32, 32)], relu=[True, True],
            passes=("fwd", "dgrad", "wgrad"), input="ct", wvar=[None, None]),
    4: dict(name="c4_bf16_512^3_32to32", n=1, dhw=(512, 512, 512), grid=(4, 4, 1), halo=1,
            dtype="bf16", layers=[(32, 32)], relu=[False],
            passes=("fwd", "dgrad", "wgrad"), input="normal", wvar=[None]),
}


def config_tensors(cfg_id, dhw=None):
    """Input volume, weights per layer and upstream gradient of a configuration.

    dhw overrides the volume extents (same seeds, same distributions) so that tests can
    run a configuration's recipe at a size the CPU oracle finishes quickly."""
    c = CONFIGS[cfg_id]
    D, H, W = dhw or c["dhw"]
    cin0, cout_last = c["layers"][0][0], c["layers"][-1][1]
    shape_in = (c["n"], D, H, W, cin0)
    if c["input"] == "ct":
        x = ct_like_volume(shape_in, seed_for(cfg_id, T_INPUT), c["dtype"])
    else:
        x = normal_volume(shape_in, seed_for(cfg_id, T_INPUT), c["dtype"])
    ws = [weights(ci, co, seed_for(cfg_id, T_WEIGHT0 + i), c["dtype"], var=c["wvar"][i])
          for i, (ci, co) in enumerate(c["layers"])]
    dy = normal_volume((c["n"], D, H, W, cout_last), seed_for(cfg_id, T_UPSTREAM), c["dtype"])
    return x, ws, dy
