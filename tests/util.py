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


def check_tail_argmax(ya, ri, gi, absdot, Ci, scale, what=""):
    """Argmax of the one-operator tail (conv -> BatchNorm -> act -> max over points) against the oracle's.

    ya [N, K, L]: the oracle's activated values (float64); ri, gi [N, K]: the oracle's and the device's
    argmax; absdot [N, K, L] = sum_c |w_c| |x_c| at every point; scale [K] = |gamma| * invstd.
    The device decides the maximum on fp32 matrix products whose inputs are exact: a Ci-term dot product
    carries at most Ci * 2^-24 * sum|w||x| of rounding, which BatchNorm scales by |gamma| * invstd and
    the (1-Lipschitz) activation does not enlarge.  So wherever the indices differ, the oracle's value at
    the device's index must be within the sum of that bound at the two positions of the oracle's
    maximum; rows whose activated values are all equal must return index 0 (lowest index among equal
    values).  Returns the number of differing indices."""
    N, K, L = ya.shape
    rv = np.take_along_axis(ya, ri[:, :, None].astype(np.int64), axis=2)[:, :, 0]
    at = np.take_along_axis(ya, gi[:, :, None].astype(np.int64), axis=2)[:, :, 0]
    flat = ya.max(axis=2) == ya.min(axis=2)
    assert np.all(gi[flat] == 0), f"{what}: a row of equal activated values must return index 0"
    bound = Ci * 2.0 ** -24 * absdot * np.asarray(scale)[None, :, None]
    b_at = np.take_along_axis(bound, gi[:, :, None].astype(np.int64), axis=2)[:, :, 0]
    b_ref = np.take_along_axis(bound, ri[:, :, None].astype(np.int64), axis=2)[:, :, 0]
    mism = gi != ri
    assert np.all(at[mism] >= rv[mism] - (b_at + b_ref)[mism]), f"{what}: argmax beyond the fp32 product's rounding bound"
    # an exact tie of the oracle's values at a lower index than the oracle's own cannot happen; at a higher one it
    # means the device skipped the first of two equal values only if they differ in its own arithmetic
    return int(mism.sum())


def bn_preact_fp32(z, gamma, beta, mean, invstd):
    """Pre-activation gamma * xhat + beta of a [N, C, L] tensor as the fp32 kernels form it -- xhat
    rounded to fp32 after the subtraction and after the product, then one fused multiply-add whose
    sign is the sign of the exact sum -- so that the branch an activation's derivative takes at
    elements within rounding of zero is decided in the kernels' precision on both sides."""
    f32 = np.float32
    c = lambda a: np.asarray(a, np.float64).astype(f32)[None, :, None]
    xh = (np.asarray(z, np.float64).astype(f32) - c(mean)) * c(invstd)
    return c(gamma).astype(np.float64) * xh.astype(np.float64) + c(beta).astype(np.float64)
