"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

TOL = {"f32": 1e-5, "bf16": 2e-2}
DT = {"f32": 0, "bf16": 1}
TDT = {"f32": torch.float32, "bf16": torch.bfloat16}


def dev(a, dtype="f32"):
    """numpy -> cuda tensor of the storage dtype (values must already be representable)."""
    t = torch.from_numpy(np.ascontiguousarray(a))
    if t.dtype in (torch.float32, torch.float64):
        t = t.to(TDT[dtype])
    return t.cuda()


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64) if t.dtype != torch.int32 else t.cpu().numpy()


def conv_strides(B, C, L):
    """Strides {b, n, c, l} of the paper's [N, B*C, L] layout."""
    return (C * L, B * C * L, L, 1)


def check(gpu, ref, tol, what="", extra=None):
    """Relative parity: norm-wise  max|d| <= tol * max|ref|  and element-wise
    |d| <= tol * (|ref| + rms(ref)).  `extra` is an optional element-wise absolute
    allowance for a documented conditioning term (e.g. fp32 cancellation in x - mean)."""
    gpu = np.asarray(gpu, np.float64)
    ref = np.asarray(ref, np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    assert np.all(np.isfinite(gpu)), what
    d = np.abs(gpu - ref)
    if extra is not None:
        d = np.maximum(d - np.broadcast_to(extra, d.shape), 0.0)
    scale = max(np.abs(ref).max(), 1e-30)
    rms = np.sqrt(np.mean(ref * ref))
    nw = d.max() / scale
    assert nw <= tol, f"{what}: norm-wise rel err {nw:.3e} > {tol}"
    bad = d > tol * (np.abs(ref) + rms) + 1e-30
    assert not bad.any(), f"{what}: {bad.sum()} elements beyond tol; worst {d[bad].max():.3e}"
    return nw
