"""Helpers for the GPU parity tests: host<->device plumbing and the error metric."""
import sys
import time

import numpy as np
import torch

from paper_1909_03108_amd import sp3d

DT = {"bf16": sp3d.SP_BF16, "f32": sp3d.SP_F32}


def to_dev(a):
    """numpy float32, or uint16 holding bf16 bit patterns -> device tensor of the same bits."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    assert a.dtype == np.float32
    return torch.from_numpy(a).cuda()


def bits(t):
    """Device tensor -> numpy array of raw storage (uint16 for bf16, float32 otherwise)."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def f64(t):
    """Device tensor -> float64 numpy values."""
    return t.float().cpu().numpy().astype(np.float64)


def widen(a):
    """Storage array (uint16 bf16 bits or float32) -> float64 values."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def rel_err(got, ref):
    """max_i |g_i - r_i| / max(|r_i|, rms(r)): element-wise relative error with the tensor's rms
    as the floor, so that values near a zero crossing do not blow the ratio up."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    den = np.maximum(np.abs(ref), rms if rms > 0 else 1.0)
    return float(np.max(np.abs(got - ref) / den)) if ref.size else 0.0


TOL = {"bf16": 1e-2, "f32": 1e-5}


def guard_alloc(shape, dtype, fill):
    """Device tensor with a 4096-element canary band before and after the payload."""
    n = int(np.prod(shape))
    buf = torch.full((n + 8192,), fill, dtype=dtype, device="cuda")
    return buf, buf[4096:4096 + n].view(shape)


def guards_intact(buf, fill):
    return bool((buf[:4096] == fill).all() and (buf[-4096:] == fill).all())


_T0 = time.time()


def progress(msg):
    """One line on the real stderr (not captured): long oracle passes report their steps."""
    sys.__stderr__.write("[%7.1f s] %s\n" % (time.time() - _T0, msg))
    sys.__stderr__.flush()
