"""CPU oracle: the plain, unfused, per-model operators.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this package;
only tests, the smoke check and the benchmark's cpu_baseline leg do.  It shares
no code with the HIP library.

Every function here is the ordinary single-model operator from the *left*
column of the paper's operator fusion rules table (appendix "HFTA Operator
Fusion Rules"), written out as its textbook definition in float64 numpy.  The
fused array is mathematically equivalent to B independent models (section "Our
Proposal: HFTA", paragraph "Convergence"), so the reference result for a fused
call is obtained by looping these over b (see ``oracle.array``).

A numpy matmul / einsum is used as a library primitive for the inner
contraction; there is no blocking, fusion or reordering beyond the definition.

Pins: tests/test_oracle_*.py check each function against brute-force Python
loops on tiny shapes, central finite differences, adjoint identities, closed
forms and torch's CPU float64 operators (the *right* column of the same table:
grouped convolution, baddbmm, BatchNorm over B*C channels).
Unpinned: NaN/Inf behaviour (excluded from all tests).
"""
from __future__ import annotations

import math
from typing import Optional, Tuple

import numpy as np

F64 = np.float64


def _f64(a):
    return np.asarray(a, dtype=F64)


# --------------------------------------------------------------------------
# storage rounding (bf16 = upper 16 bits of float32, round to nearest even)
# --------------------------------------------------------------------------
def round_bf16(a) -> np.ndarray:
    """Round float values to the nearest bf16 (ties to even); returns float64.

    Used only where a tensor is *stored* in bf16 between two operators."""
    x = np.asarray(a, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(F64)


def store(a, dtype: str) -> np.ndarray:
    """Value as it reads back from a tensor stored in ``dtype``."""
    if dtype == "bf16":
        return round_bf16(a)
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32).astype(F64)
    if dtype == "f64":
        return _f64(a)
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# Linear  (fusion rules table, row "Linear": w is [Fx, Fy])
# --------------------------------------------------------------------------
def linear_fwd(x, w, bias=None):
    """y[r, j] = bias[j] + sum_k x[r, k] w[k, j];  x:[M,Fx], w:[Fx,Fy]."""
    y = _f64(x) @ _f64(w)
    if bias is not None:
        y = y + _f64(bias)[None, :]
    return y


def linear_bwd(x, w, dy):
    """Returns (dx, dw, dbias) of linear_fwd."""
    x, w, dy = _f64(x), _f64(w), _f64(dy)
    dx = dy @ w.T
    dw = x.T @ dy
    db = dy.sum(axis=0)
    return dx, dw, db


# --------------------------------------------------------------------------
# Conv1d with kernel length 1 (row "Conv1d", L_w = 1, g = 1)
# --------------------------------------------------------------------------
def conv1x1_fwd(x, w, bias=None):
    """y[n, o, l] = bias[o] + sum_c w[o, c] x[n, c, l];  x:[N,Ci,L], w:[Co,Ci]."""
    x, w = _f64(x), _f64(w)
    y = np.einsum("oc,ncl->nol", w, x)
    if bias is not None:
        y = y + _f64(bias)[None, :, None]
    return y


def conv1x1_bwd(x, w, dy):
    x, w, dy = _f64(x), _f64(w), _f64(dy)
    dx = np.einsum("oc,nol->ncl", w, dy)
    dw = np.einsum("nol,ncl->oc", dy, x)
    db = dy.sum(axis=(0, 2))
    return dx, dw, db


# --------------------------------------------------------------------------
# Conv2d / ConvTranspose2d (rows "Conv2d", "ConvT2d"; g = 1, no dilation)
# --------------------------------------------------------------------------
def conv2d_out_size(H: int, k: int, stride: int, pad: int) -> int:
    return (H + 2 * pad - k) // stride + 1


def conv2d_fwd(x, w, bias=None, stride: int = 1, pad: int = 0):
    """Cross-correlation with zero padding.

    y[n,o,i,j] = bias[o] + sum_{c,ky,kx} w[o,c,ky,kx] x[n,c, s*i+ky-p, s*j+kx-p]
    x:[N,Ci,H,W], w:[Co,Ci,kh,kw]."""
    x, w = _f64(x), _f64(w)
    N, Ci, H, W = x.shape
    Co, Ci2, kh, kw = w.shape
    assert Ci == Ci2
    Ho, Wo = conv2d_out_size(H, kh, stride, pad), conv2d_out_size(W, kw, stride, pad)
    xp = np.zeros((N, Ci, H + 2 * pad, W + 2 * pad), F64)
    xp[:, :, pad:pad + H, pad:pad + W] = x
    y = np.zeros((N, Co, Ho, Wo), F64)
    for ky in range(kh):
        for kx in range(kw):
            win = xp[:, :, ky:ky + stride * (Ho - 1) + 1:stride, kx:kx + stride * (Wo - 1) + 1:stride]
            y += np.einsum("oc,ncij->noij", w[:, :, ky, kx], win)
    if bias is not None:
        y = y + _f64(bias)[None, :, None, None]
    return y


def conv2d_bwd(x, w, dy, stride: int = 1, pad: int = 0):
    """Adjoints of conv2d_fwd: (dx, dw, dbias)."""
    x, w, dy = _f64(x), _f64(w), _f64(dy)
    N, Ci, H, W = x.shape
    Co, _, kh, kw = w.shape
    Ho, Wo = dy.shape[2], dy.shape[3]
    xp = np.zeros((N, Ci, H + 2 * pad, W + 2 * pad), F64)
    xp[:, :, pad:pad + H, pad:pad + W] = x
    dxp = np.zeros_like(xp)
    dw = np.zeros_like(w)
    for ky in range(kh):
        for kx in range(kw):
            sl = (slice(None), slice(None),
                  slice(ky, ky + stride * (Ho - 1) + 1, stride),
                  slice(kx, kx + stride * (Wo - 1) + 1, stride))
            dw[:, :, ky, kx] = np.einsum("noij,ncij->oc", dy, xp[sl])
            dxp[sl] += np.einsum("oc,noij->ncij", w[:, :, ky, kx], dy)
    dx = dxp[:, :, pad:pad + H, pad:pad + W]
    db = dy.sum(axis=(0, 2, 3))
    return dx, dw, db


def convT2d_out_size(H: int, k: int, stride: int, pad: int) -> int:
    return (H - 1) * stride - 2 * pad + k


def convT2d_fwd(x, w, bias=None, stride: int = 1, pad: int = 0):
    """Transposed convolution: the adjoint of conv2d w.r.t. its input.

    x:[N,Cx,H,W], w:[Cx,Cy,kh,kw] (input-channel major), y:[N,Cy,Ho,Wo] with
    Ho = (H-1)s - 2p + k.   y[n,o, s*i+ky-p, s*j+kx-p] += x[n,c,i,j] w[c,o,ky,kx]."""
    x, w = _f64(x), _f64(w)
    N, Cx, H, W = x.shape
    Cx2, Cy, kh, kw = w.shape
    assert Cx == Cx2
    Ho, Wo = convT2d_out_size(H, kh, stride, pad), convT2d_out_size(W, kw, stride, pad)
    yp = np.zeros((N, Cy, Ho + 2 * pad, Wo + 2 * pad), F64)
    for ky in range(kh):
        for kx in range(kw):
            yp[:, :, ky:ky + stride * (H - 1) + 1:stride, kx:kx + stride * (W - 1) + 1:stride] += \
                np.einsum("co,ncij->noij", w[:, :, ky, kx], x)
    y = yp[:, :, pad:pad + Ho, pad:pad + Wo]
    if bias is not None:
        y = y + _f64(bias)[None, :, None, None]
    return y


def convT2d_bwd(x, w, dy, stride: int = 1, pad: int = 0):
    """(dx, dw, dbias) of convT2d_fwd."""
    x, w, dy = _f64(x), _f64(w), _f64(dy)
    N, Cx, H, W = x.shape
    _, Cy, kh, kw = w.shape
    Ho, Wo = dy.shape[2], dy.shape[3]
    dyp = np.zeros((N, Cy, Ho + 2 * pad, Wo + 2 * pad), F64)
    dyp[:, :, pad:pad + Ho, pad:pad + Wo] = dy
    dx = np.zeros_like(x)
    dw = np.zeros_like(w)
    for ky in range(kh):
        for kx in range(kw):
            win = dyp[:, :, ky:ky + stride * (H - 1) + 1:stride, kx:kx + stride * (W - 1) + 1:stride]
            dx += np.einsum("co,noij->ncij", w[:, :, ky, kx], win)
            dw[:, :, ky, kx] = np.einsum("ncij,noij->co", x, win)
    db = dy.sum(axis=(0, 2, 3))
    return dx, dw, db


# --------------------------------------------------------------------------
# BatchNorm, training mode (rows "BatchNorm1d", "BatchNorm2d")
# --------------------------------------------------------------------------
def bn_fwd(x, gamma, beta, eps: float = 1e-5, momentum: float = 0.1,
           running_mean=None, running_var=None):
    """x:[N,C,L] (L = 1 for the 2-D case, H*W for 2d).  Per channel c over (n,l):
    mu = mean x, var = mean (x-mu)^2 (biased), y = gamma (x-mu)/sqrt(var+eps) + beta.
    Running estimates use the unbiased variance.
    Returns (y, mean, invstd, new_running_mean, new_running_var)."""
    x = _f64(x)
    N, C, L = x.shape
    m = N * L
    mu = x.mean(axis=(0, 2))
    var = ((x - mu[None, :, None]) ** 2).mean(axis=(0, 2))
    invstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu[None, :, None]) * invstd[None, :, None]
    y = _f64(gamma)[None, :, None] * xhat + _f64(beta)[None, :, None]
    nrm = nrv = None
    if running_mean is not None:
        nrm = (1.0 - momentum) * _f64(running_mean) + momentum * mu
        unbiased = var * (m / (m - 1.0)) if m > 1 else var
        nrv = (1.0 - momentum) * _f64(running_var) + momentum * unbiased
    return y, mu, invstd, nrm, nrv


def bn_eval_fwd(x, gamma, beta, running_mean, running_var, eps: float = 1e-5):
    """Evaluation mode (the fusion rules table keeps every argument of the single-model operator,
    its training flag included): the running estimates take the place of the batch statistics,
    y = gamma (x - running_mean) / sqrt(running_var + eps) + beta; nothing is updated.  x:[N,C,L]."""
    x = _f64(x)
    scale = _f64(gamma) / np.sqrt(_f64(running_var) + eps)
    return (x - _f64(running_mean)[None, :, None]) * scale[None, :, None] + _f64(beta)[None, :, None]


def bn_bwd(x, dy, gamma, mean, invstd):
    """dbeta = sum dy; dgamma = sum dy xhat;
    dx = gamma invstd (dy - dbeta/m - xhat dgamma/m).  Returns (dx, dgamma, dbeta)."""
    x, dy = _f64(x), _f64(dy)
    N, C, L = x.shape
    m = N * L
    xhat = (x - _f64(mean)[None, :, None]) * _f64(invstd)[None, :, None]
    dbeta = dy.sum(axis=(0, 2))
    dgamma = (dy * xhat).sum(axis=(0, 2))
    dx = (_f64(gamma) * _f64(invstd))[None, :, None] * (
        dy - dbeta[None, :, None] / m - xhat * dgamma[None, :, None] / m)
    return dx, dgamma, dbeta


# --------------------------------------------------------------------------
# LayerNorm over the last dim (row "LayerNorm": affine-free LN, then * w + b)
# --------------------------------------------------------------------------
def layernorm_fwd(x, w, b, eps: float = 1e-5):
    """x:[R,E]; returns (y, mean[R], invstd[R])."""
    x = _f64(x)
    mu = x.mean(axis=1)
    var = ((x - mu[:, None]) ** 2).mean(axis=1)
    invstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu[:, None]) * invstd[:, None]
    return xhat * _f64(w)[None, :] + _f64(b)[None, :], mu, invstd


def layernorm_bwd(x, dy, w, mean, invstd):
    """Returns (dx, dw, db)."""
    x, dy, w = _f64(x), _f64(dy), _f64(w)
    E = x.shape[1]
    xhat = (x - _f64(mean)[:, None]) * _f64(invstd)[:, None]
    db = dy.sum(axis=0)
    dw = (dy * xhat).sum(axis=0)
    g = dy * w[None, :]
    dx = _f64(invstd)[:, None] * (g - g.mean(axis=1, keepdims=True)
                                  - xhat * (g * xhat).mean(axis=1, keepdims=True))
    return dx, dw, db


# --------------------------------------------------------------------------
# Max-pool over the point dimension (PointNet's global feature)
# --------------------------------------------------------------------------
def maxpool_points_fwd(x):
    """x:[N,C,L] -> (v[N,C], idx[N,C] int32); ties go to the lowest point index."""
    x = np.asarray(x)
    idx = np.argmax(x, axis=2).astype(np.int32)   # numpy returns the first maximum
    v = np.take_along_axis(x, idx[:, :, None].astype(np.int64), axis=2)[:, :, 0]
    return _f64(v), idx


def maxpool_points_bwd(dv, idx, L: int):
    """dx[n,c,l] = dv[n,c] if l == idx[n,c] else 0."""
    dv = _f64(dv)
    N, C = dv.shape
    dx = np.zeros((N, C, L), F64)
    np.put_along_axis(dx, np.asarray(idx, np.int64)[:, :, None], dv[:, :, None], axis=2)
    return dx


# --------------------------------------------------------------------------
# Pieces of a segmentation head on a concatenation with a tiled (point-independent) part:
# a k=1 convolution over [per-point features | tiled vector] equals the convolution over the
# per-point features plus a per-sample vector broadcast along the points.
# --------------------------------------------------------------------------
def add_sample_bias(z, s):
    """z:[N,C,L], s:[N,C] -> z + s broadcast along the points."""
    return _f64(z) + _f64(s)[:, :, None]


def sum_points(dz):
    """Adjoint of the broadcast: dz:[N,C,L] -> [N,C], the sum over the points."""
    return _f64(dz).sum(axis=2)


def softmax_xent_points(logits, labels):
    """logits:[N,K,L], labels:[N,L] int.  Softmax cross-entropy over the class axis K for every point,
    mean over the N*L points.  Returns (loss, dlogits[N,K,L])."""
    logits = _f64(logits)
    N, K, L = logits.shape
    loss, d = softmax_xent(logits.transpose(0, 2, 1).reshape(N * L, K), np.asarray(labels).reshape(-1))
    return loss, d.reshape(N, L, K).transpose(0, 2, 1)


def maxpool_points_bwd_add(dx, dv, idx):
    """dx:[N,C,L] + (dv[n,c] at l = idx[n,c]): the max-pool's backward added onto another gradient."""
    out = _f64(dx).copy()
    N, C, _ = out.shape
    out[np.arange(N)[:, None], np.arange(C)[None, :], np.asarray(idx, np.int64)] += _f64(dv)
    return out


# --------------------------------------------------------------------------
# Tail of a point-cloud model's per-point MLP as ONE operator:
#   k=1 Conv1d -> training-mode BatchNorm -> activation -> max over points
# (rows "Conv1d", "BatchNorm1d" and the element-wise rows, then the point max-pool).  It is the
# composition of the definitions above with nothing stored between the steps: an operator that
# keeps no intermediate tensor in memory has no storage rounding inside it.
# --------------------------------------------------------------------------
def conv1x1_bn_maxpool_fwd(x, w, bias, gamma, beta, eps: float = 1e-5, momentum: float = 0.1,
                           running_mean=None, running_var=None, act: int = 1, slope: float = 0.2):
    """x:[N,Ci,L], w:[Co,Ci].  Returns (v[N,Co], idx[N,Co], mean, invstd, new_running_mean,
    new_running_var, zhit[N,Co]) with zhit the convolution output at the argmax point."""
    z = conv1x1_fwd(x, w, bias)
    y, mean, invstd, nrm, nrv = bn_fwd(z, gamma, beta, eps, momentum, running_mean, running_var)
    v, idx = maxpool_points_fwd(act_fwd(y, act, slope))
    zhit = np.take_along_axis(z, idx[:, :, None].astype(np.int64), axis=2)[:, :, 0]
    return v, idx, mean, invstd, nrm, nrv, zhit


def conv1x1_bn_maxpool_bwd(x, w, bias, gamma, beta, mean, invstd, dv, idx, act: int = 1, slope: float = 0.2):
    """Backward of the operator above from the gradient dv[N,Co] of its pooled output: max-pool
    scatter -> activation -> BatchNorm -> convolution.  Returns (dx, dw, dbias, dgamma, dbeta)."""
    z = conv1x1_fwd(x, w, bias)
    y = _f64(gamma)[None, :, None] * (z - _f64(mean)[None, :, None]) * _f64(invstd)[None, :, None] \
        + _f64(beta)[None, :, None]
    dy = act_bwd(y, maxpool_points_bwd(dv, idx, z.shape[2]), act, slope)
    dz, dgamma, dbeta = bn_bwd(z, dy, gamma, mean, invstd)
    dx, dw, db = conv1x1_bwd(x, w, dz)
    return dx, dw, db, dgamma, dbeta


# --------------------------------------------------------------------------
# Activations (rows "ReLU", "LeakyReLU", "Tanh"; GELU for the MLP workload)
# --------------------------------------------------------------------------
ACT_NONE, ACT_RELU, ACT_LEAKY, ACT_TANH, ACT_GELU = 0, 1, 2, 3, 4

_erf = np.vectorize(math.erf, otypes=[F64])


def act_fwd(x, act: int, slope: float = 0.2):
    x = _f64(x)
    if act == ACT_NONE:
        return x.copy()
    if act == ACT_RELU:
        return np.where(x > 0, x, 0.0)
    if act == ACT_LEAKY:
        return np.where(x > 0, x, slope * x)
    if act == ACT_TANH:
        return np.tanh(x)
    if act == ACT_GELU:
        return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))
    raise ValueError(act)


def act_bwd(x, dy, act: int, slope: float = 0.2):
    """Gradient w.r.t. the pre-activation x (ReLU/LeakyReLU: the x <= 0 branch
    takes the zero / slope side)."""
    x, dy = _f64(x), _f64(dy)
    if act == ACT_NONE:
        return dy.copy()
    if act == ACT_RELU:
        return np.where(x > 0, dy, 0.0)
    if act == ACT_LEAKY:
        return np.where(x > 0, dy, slope * dy)
    if act == ACT_TANH:
        t = np.tanh(x)
        return dy * (1.0 - t * t)
    if act == ACT_GELU:
        cdf = 0.5 * (1.0 + _erf(x / math.sqrt(2.0)))
        pdf = np.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)
        return dy * (cdf + x * pdf)
    raise ValueError(act)


# --------------------------------------------------------------------------
# Dropout from an explicit keep-mask (row "Dropout")
# --------------------------------------------------------------------------
def dropout_fwd(x, keep_mask, p: float):
    return _f64(x) * _f64(keep_mask) / (1.0 - p)


def dropout_bwd(dy, keep_mask, p: float):
    return _f64(dy) * _f64(keep_mask) / (1.0 - p)


# --------------------------------------------------------------------------
# Per-model losses with mean reduction (appendix "Fused Loss")
# --------------------------------------------------------------------------
def softmax_xent(logits, labels):
    """logits:[R,K], labels:[R] -> (mean loss, dlogits)."""
    z = _f64(logits)
    R = z.shape[0]
    zmax = z.max(axis=1, keepdims=True)
    lse = zmax[:, 0] + np.log(np.exp(z - zmax).sum(axis=1))
    lab = np.asarray(labels, np.int64)
    loss = (lse - z[np.arange(R), lab]).mean()
    p = np.exp(z - lse[:, None])
    p[np.arange(R), lab] -= 1.0
    return float(loss), p / R


def bce_logits(logits, targets):
    """Binary cross-entropy on sigmoid(logits), mean over elements."""
    z, t = _f64(logits), _f64(targets)
    loss = (np.maximum(z, 0.0) - z * t + np.log1p(np.exp(-np.abs(z)))).mean()
    sig = 1.0 / (1.0 + np.exp(-z))
    return float(loss), (sig - t) / z.size


def mse(pred, target):
    d = _f64(pred) - _f64(target)
    return float((d * d).mean()), 2.0 * d / d.size


# --------------------------------------------------------------------------
# Adam (section "Our Proposal: HFTA", paragraph on optimizers; Kingma & Ba)
# --------------------------------------------------------------------------
def adam_step(theta, grad, m, v, lr: float, beta1: float, beta2: float, eps: float,
              weight_decay: float, t: int, decoupled_wd: bool = False):
    """One Adam update of a single model; t is 1-based.

    g' = g + wd*theta (classic L2) or theta *= (1 - lr*wd) first (decoupled);
    m = b1 m + (1-b1) g';  v = b2 v + (1-b2) g'^2;
    theta -= lr * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps).
    Returns (theta, m, v) as float64 (callers store them as float32)."""
    theta, g, m, v = _f64(theta), _f64(grad), _f64(m), _f64(v)
    lr, beta1, beta2, eps, weight_decay = (float(lr), float(beta1), float(beta2),
                                           float(eps), float(weight_decay))
    if decoupled_wd:
        theta = theta * (1.0 - lr * weight_decay)
    else:
        g = g + weight_decay * theta
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    theta = theta - lr * mhat / (np.sqrt(vhat) + eps)
    return theta, m, v


# --------------------------------------------------------------------------
# Adadelta and the step learning-rate schedule (section "Our Proposal: HFTA",
# paragraph on optimizers and learning-rate schedulers: per-model hyper-parameter
# vectors; Zeiler's ADADELTA with a learning-rate factor)
# --------------------------------------------------------------------------
def adadelta_step(theta, grad, sq_avg, acc_delta, lr: float, rho: float, eps: float, weight_decay: float):
    """g' = g + wd*theta;  v = rho v + (1-rho) g'^2;  d = sqrt(u + eps) / sqrt(v + eps) * g';
    u = rho u + (1-rho) d^2;  theta -= lr * d.   Returns (theta, v, u) as float64."""
    theta, g, v, u = _f64(theta), _f64(grad), _f64(sq_avg), _f64(acc_delta)
    lr, rho, eps, weight_decay = float(lr), float(rho), float(eps), float(weight_decay)
    g = g + weight_decay * theta
    v = rho * v + (1.0 - rho) * g * g
    d = np.sqrt(u + eps) / np.sqrt(v + eps) * g
    u = rho * u + (1.0 - rho) * d * d
    return theta - lr * d, v, u


def steplr(base_lr, gamma, step_size, epoch: int):
    """Per-model step schedule: lr_b = base_lr_b * gamma_b ** floor(epoch / step_size_b)."""
    base_lr, gamma = _f64(base_lr), _f64(gamma)
    k = np.floor_divide(int(epoch), np.asarray(step_size, np.int64))
    return base_lr * gamma ** k


# --------------------------------------------------------------------------
# Embedding and scaled-dot-product multi-head attention (fusion rules table rows
# "Embedding" and, built from the Linear rule plus per-model batched products,
# "MultiheadAttention"; the Transformer workloads of section "Methodology")
# --------------------------------------------------------------------------
def embedding_fwd(table, idx, scale: float = 1.0, pos=None):
    """table:[V,E], idx:[R] int -> scale * table[idx] (+ pos[r % len(pos)] if given):[R,E]."""
    y = scale * _f64(table)[np.asarray(idx, np.int64)]
    if pos is not None:
        pos = _f64(pos)
        y = y + pos[np.arange(y.shape[0]) % pos.shape[0]]
    return y


def embedding_bwd(dy, idx, V: int, scale: float = 1.0):
    """dtable[v] = scale * sum over the rows r with idx[r] == v of dy[r]."""
    dy = _f64(dy)
    dt = np.zeros((V, dy.shape[1]), F64)
    np.add.at(dt, np.asarray(idx, np.int64), scale * dy)
    return dt


def softmax_rows(s, scale: float = 1.0, causal: bool = False):
    """Row softmax of scale * s over the last axis; with ``causal`` entry [i, j] takes part only for j <= i."""
    z = scale * _f64(s)
    if causal:
        i, j = np.arange(z.shape[-2])[:, None], np.arange(z.shape[-1])[None, :]
        z = np.where(j <= i, z, -np.inf)
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def softmax_rows_bwd(p, dp, scale: float = 1.0):
    """ds = scale * p * (dp - sum_j dp p)   (masked entries have p = 0, hence ds = 0)."""
    p, dp = _f64(p), _f64(dp)
    return scale * p * (dp - (dp * p).sum(axis=-1, keepdims=True))


def attention_fwd(qkv, heads: int, causal: bool = False, store=None):
    """qkv:[N,S,3E] = [q | k | v] per token; head h owns columns h*d .. (h+1)*d of each block, d = E/heads.
    scores = q_h k_h^T, p = softmax(scores / sqrt(d)), ctx_h = p v_h.  ``store`` rounds the tensors
    the device keeps between the three steps (scores, p).  Returns (ctx[N,S,E], p[N,heads,S,S])."""
    st = store if store is not None else (lambda a: a)
    qkv = _f64(qkv)
    N, S, E3 = qkv.shape
    E = E3 // 3
    d = E // heads
    sp = lambda a: a.reshape(N, S, heads, d).transpose(0, 2, 1, 3)          # [N,H,S,d]
    q, k, v = sp(qkv[..., :E]), sp(qkv[..., E:2 * E]), sp(qkv[..., 2 * E:])
    scores = st(q @ k.transpose(0, 1, 3, 2))
    p = st(softmax_rows(scores, 1.0 / np.sqrt(d), causal))
    ctx = (p @ v).transpose(0, 2, 1, 3).reshape(N, S, E)
    return ctx, p


def attention_bwd(qkv, p, dctx, heads: int, store=None):
    """Backward of attention_fwd from the stored probabilities.  Returns dqkv[N,S,3E]."""
    st = store if store is not None else (lambda a: a)
    qkv, p, dctx = _f64(qkv), _f64(p), _f64(dctx)
    N, S, E3 = qkv.shape
    E = E3 // 3
    d = E // heads
    sp = lambda a: a.reshape(N, S, heads, d).transpose(0, 2, 1, 3)
    un = lambda a: a.transpose(0, 2, 1, 3).reshape(N, S, E)
    q, k, v, dc = sp(qkv[..., :E]), sp(qkv[..., E:2 * E]), sp(qkv[..., 2 * E:]), sp(dctx)
    dv = p.transpose(0, 1, 3, 2) @ dc
    dp = st(dc @ v.transpose(0, 1, 3, 2))
    ds = st(softmax_rows_bwd(p, dp, 1.0 / np.sqrt(d)))
    dq = ds @ k
    dk = ds.transpose(0, 1, 3, 2) @ q
    return np.concatenate([un(dq), un(dk), un(dv)], axis=2)


# --------------------------------------------------------------------------
# Per-sample point transform (the point-cloud models' input / feature transform:
# a matrix predicted per cloud, applied to all its points; one batched product
# per (model, sample), an instance of the Linear rule with the weight indexed by
# the sample as well)
# --------------------------------------------------------------------------
def point_transform_fwd(x, t):
    """x:[N,Ci,L], t:[N,Co,Ci] -> y[n,o,l] = sum_c t[n,o,c] x[n,c,l]."""
    return np.einsum("noc,ncl->nol", _f64(t), _f64(x))


def point_transform_bwd(x, t, dy):
    """Returns (dx[n,c,l] = sum_o t[n,o,c] dy[n,o,l],  dt[n,o,c] = sum_l dy[n,o,l] x[n,c,l])."""
    x, t, dy = _f64(x), _f64(t), _f64(dy)
    return np.einsum("noc,nol->ncl", t, dy), np.einsum("nol,ncl->noc", dy, x)
