"""CPU oracle for a fused call: B separate, unfused, per-model loops.

TEST INFRASTRUCTURE ONLY (see oracle/ops.py).  Each function takes tensors in
the fused layouts of the operator fusion rules table (right column), slices out
model b, runs the ordinary single-model operator from ``oracle.ops`` on it, and
writes the result back into the fused layout.  There is no batching across b.

Layouts:
  conv family / BatchNorm / pool : [N, B*C, L]   (2d: [N, B*C, H, W])
  linear family                  : [B, N, F]
  conv weights [B*Co, Ci, ...], conv-transpose weights [B*Cx, Cy, kh, kw],
  linear weights [B, Fx, Fy], per-channel vectors [B*C] (conv) or [B, F] (linear)
"""
from __future__ import annotations

import numpy as np

from . import ops

F64 = np.float64


def _chan(a, b, C):
    """Model b's channel block of a conv-layout tensor."""
    return a[:, b * C:(b + 1) * C]


# ---------------------------------------------------------------- linear
def linear_fwd(B, x, w, bias=None):
    return np.stack([ops.linear_fwd(x[b], w[b], None if bias is None else bias[b])
                     for b in range(B)])


def linear_bwd(B, x, w, dy):
    r = [ops.linear_bwd(x[b], w[b], dy[b]) for b in range(B)]
    return tuple(np.stack([q[i] for q in r]) for i in range(3))


# ---------------------------------------------------------------- conv1x1
def conv1x1_fwd(B, x, w, bias=None):
    Ci = x.shape[1] // B
    Co = w.shape[0] // B
    y = np.empty((x.shape[0], B * Co, x.shape[2]), F64)
    for b in range(B):
        y[:, b * Co:(b + 1) * Co] = ops.conv1x1_fwd(
            _chan(x, b, Ci), w[b * Co:(b + 1) * Co],
            None if bias is None else bias[b * Co:(b + 1) * Co])
    return y


def conv1x1_bwd(B, x, w, dy):
    Ci = x.shape[1] // B
    Co = w.shape[0] // B
    dx = np.empty(x.shape, F64)
    dw = np.empty(w.shape, F64)
    db = np.empty(B * Co, F64)
    for b in range(B):
        a, c, d = ops.conv1x1_bwd(_chan(x, b, Ci), w[b * Co:(b + 1) * Co], _chan(dy, b, Co))
        dx[:, b * Ci:(b + 1) * Ci] = a
        dw[b * Co:(b + 1) * Co] = c
        db[b * Co:(b + 1) * Co] = d
    return dx, dw, db


# ---------------------------------------------------------------- conv2d (groups = B)
def conv2d_fwd(B, x, w, bias=None, stride=1, pad=0):
    Ci = x.shape[1] // B
    Co = w.shape[0] // B
    ys = [ops.conv2d_fwd(_chan(x, b, Ci), w[b * Co:(b + 1) * Co],
                         None if bias is None else bias[b * Co:(b + 1) * Co], stride, pad)
          for b in range(B)]
    return np.concatenate(ys, axis=1)


def conv2d_bwd(B, x, w, dy, stride=1, pad=0):
    Ci = x.shape[1] // B
    Co = w.shape[0] // B
    r = [ops.conv2d_bwd(_chan(x, b, Ci), w[b * Co:(b + 1) * Co], _chan(dy, b, Co), stride, pad)
         for b in range(B)]
    return (np.concatenate([q[0] for q in r], axis=1),
            np.concatenate([q[1] for q in r], axis=0),
            np.concatenate([q[2] for q in r], axis=0))


def convT2d_fwd(B, x, w, bias=None, stride=1, pad=0):
    Cx = x.shape[1] // B
    Cy = w.shape[1]
    ys = [ops.convT2d_fwd(_chan(x, b, Cx), w[b * Cx:(b + 1) * Cx],
                          None if bias is None else bias[b * Cy:(b + 1) * Cy], stride, pad)
          for b in range(B)]
    return np.concatenate(ys, axis=1)


def convT2d_bwd(B, x, w, dy, stride=1, pad=0):
    Cx = x.shape[1] // B
    Cy = w.shape[1]
    r = [ops.convT2d_bwd(_chan(x, b, Cx), w[b * Cx:(b + 1) * Cx], _chan(dy, b, Cy), stride, pad)
         for b in range(B)]
    return (np.concatenate([q[0] for q in r], axis=1),
            np.concatenate([q[1] for q in r], axis=0),
            np.concatenate([q[2] for q in r], axis=0))


# ---------------------------------------------------------------- BatchNorm
def bn_fwd(B, x, gamma, beta, eps=1e-5, momentum=0.1, running_mean=None, running_var=None,
           layout="conv"):
    """layout "conv": x [N, B*C, L];  layout "linear": x [B, N, C] (per-channel
    vectors then are [B, C], flattened [B*C] is accepted too)."""
    if layout == "linear":
        Bn, N, C = x.shape
        xc = np.transpose(x, (1, 0, 2)).reshape(N, B * C, 1)
        out = bn_fwd(B, xc, np.reshape(gamma, -1), np.reshape(beta, -1), eps, momentum,
                     None if running_mean is None else np.reshape(running_mean, -1),
                     None if running_var is None else np.reshape(running_var, -1), "conv")
        y = out[0].reshape(N, B, C).transpose(1, 0, 2)
        return (y,) + out[1:]
    C = x.shape[1] // B
    y = np.empty(x.shape, F64)
    mean = np.empty(B * C, F64)
    invstd = np.empty(B * C, F64)
    nrm = None if running_mean is None else np.empty(B * C, F64)
    nrv = None if running_var is None else np.empty(B * C, F64)
    for b in range(B):
        s = slice(b * C, (b + 1) * C)
        r = ops.bn_fwd(x[:, s], gamma[s], beta[s], eps, momentum,
                       None if running_mean is None else running_mean[s],
                       None if running_var is None else running_var[s])
        y[:, s], mean[s], invstd[s] = r[0], r[1], r[2]
        if nrm is not None:
            nrm[s], nrv[s] = r[3], r[4]
    return y, mean, invstd, nrm, nrv


def bn_eval_fwd(B, x, gamma, beta, running_mean, running_var, eps=1e-5, layout="conv"):
    """Evaluation-mode BatchNorm of the array: model b's channels with model b's running estimates."""
    if layout == "linear":
        Bn, N, C = x.shape
        xc = np.transpose(x, (1, 0, 2)).reshape(N, B * C, 1)
        y = bn_eval_fwd(B, xc, np.reshape(gamma, -1), np.reshape(beta, -1), np.reshape(running_mean, -1),
                        np.reshape(running_var, -1), eps, "conv")
        return y.reshape(N, B, C).transpose(1, 0, 2)
    C = x.shape[1] // B
    y = np.empty(x.shape, F64)
    for b in range(B):
        s = slice(b * C, (b + 1) * C)
        y[:, s] = ops.bn_eval_fwd(x[:, s], gamma[s], beta[s], running_mean[s], running_var[s], eps)
    return y


def bn_bwd(B, x, dy, gamma, mean, invstd, layout="conv"):
    if layout == "linear":
        Bn, N, C = x.shape
        t = lambda a: np.transpose(a, (1, 0, 2)).reshape(N, B * C, 1)
        dx, dg, dbt = bn_bwd(B, t(x), t(dy), np.reshape(gamma, -1), np.reshape(mean, -1),
                             np.reshape(invstd, -1), "conv")
        return dx.reshape(N, B, C).transpose(1, 0, 2), dg, dbt
    C = x.shape[1] // B
    dx = np.empty(x.shape, F64)
    dg = np.empty(B * C, F64)
    dbt = np.empty(B * C, F64)
    for b in range(B):
        s = slice(b * C, (b + 1) * C)
        dx[:, s], dg[s], dbt[s] = ops.bn_bwd(x[:, s], dy[:, s], gamma[s], mean[s], invstd[s])
    return dx, dg, dbt


# ---------------------------------------------------------------- LayerNorm
def layernorm_fwd(B, x, w, b, eps=1e-5):
    """x:[B, R, E], w,b:[B, E]."""
    r = [ops.layernorm_fwd(x[i], w[i], b[i], eps) for i in range(B)]
    return tuple(np.stack([q[j] for q in r]) for j in range(3))


def layernorm_bwd(B, x, dy, w, mean, invstd):
    r = [ops.layernorm_bwd(x[i], dy[i], w[i], mean[i], invstd[i]) for i in range(B)]
    return tuple(np.stack([q[j] for q in r]) for j in range(3))


# ---------------------------------------------------------------- point max-pool
def maxpool_points_fwd(B, x):
    """x:[N, B*C, L] -> v:[N, B*C], idx:[N, B*C]."""
    C = x.shape[1] // B
    v = np.empty(x.shape[:2], F64)
    idx = np.empty(x.shape[:2], np.int32)
    for b in range(B):
        s = slice(b * C, (b + 1) * C)
        v[:, s], idx[:, s] = ops.maxpool_points_fwd(x[:, s])
    return v, idx


def maxpool_points_bwd(B, dv, idx, L):
    C = dv.shape[1] // B
    dx = np.empty(dv.shape + (L,), F64)
    for b in range(B):
        s = slice(b * C, (b + 1) * C)
        dx[:, s] = ops.maxpool_points_bwd(dv[:, s], idx[:, s], L)
    return dx


# ---------------------------------------------------------------- conv1x1 -> BatchNorm -> act -> point max, one operator
def conv1x1_bn_maxpool_fwd(B, x, w, bias, gamma, beta, eps=1e-5, momentum=0.1, running_mean=None,
                           running_var=None, act=1, slope=0.2):
    """x:[N, B*Ci, L], w:[B*Co, Ci] -> (v[N,B*Co], idx, mean, invstd, new_rm, new_rv, zhit[N,B*Co])."""
    Ci, Co = x.shape[1] // B, w.shape[0] // B
    r = []
    for b in range(B):
        so = slice(b * Co, (b + 1) * Co)
        r.append(ops.conv1x1_bn_maxpool_fwd(
            _chan(x, b, Ci), w[so], None if bias is None else bias[so], gamma[so], beta[so], eps, momentum,
            None if running_mean is None else running_mean[so], None if running_var is None else running_var[so],
            act, slope))
    cat = lambda j, ax: None if r[0][j] is None else np.concatenate([q[j] for q in r], axis=ax)
    return cat(0, 1), cat(1, 1), cat(2, 0), cat(3, 0), cat(4, 0), cat(5, 0), cat(6, 1)


def conv1x1_bn_maxpool_bwd(B, x, w, bias, gamma, beta, mean, invstd, dv, idx, act=1, slope=0.2):
    """dv, idx:[N, B*Co] -> (dx[N,B*Ci,L], dw[B*Co,Ci], dbias[B*Co], dgamma[B*Co], dbeta[B*Co])."""
    Ci, Co = x.shape[1] // B, w.shape[0] // B
    r = []
    for b in range(B):
        so = slice(b * Co, (b + 1) * Co)
        r.append(ops.conv1x1_bn_maxpool_bwd(_chan(x, b, Ci), w[so], None if bias is None else bias[so], gamma[so],
                                            beta[so], mean[so], invstd[so], dv[:, so], idx[:, so], act, slope))
    return (np.concatenate([q[0] for q in r], axis=1),) + tuple(np.concatenate([q[j] for q in r], axis=0)
                                                                  for j in range(1, 5))


# ---------------------------------------------------------------- losses
def softmax_xent(B, logits, labels):
    """logits:[B, R, K], labels:[B, R] -> (loss[B], dlogits[B,R,K]); each model's
    loss is its own mean, so no factor B appears (appendix "Fused Loss")."""
    r = [ops.softmax_xent(logits[b], labels[b]) for b in range(B)]
    return np.array([q[0] for q in r]), np.stack([q[1] for q in r])


def mse(B, pred, target):
    r = [ops.mse(pred[b], target[b]) for b in range(B)]
    return np.array([q[0] for q in r]), np.stack([q[1] for q in r])


def bce_logits(B, logits, targets):
    r = [ops.bce_logits(logits[b], targets[b]) for b in range(B)]
    return np.array([q[0] for q in r]), np.stack([q[1] for q in r])


# ---------------------------------------------------------------- Adam
def adam_step(B, theta, grad, m, v, lr, beta1, beta2, eps, wd, t, decoupled_wd=False):
    """Arena tensors [B, P]; hyper-parameter vectors [B].  State is stored fp32."""
    th = np.empty(theta.shape, np.float32)
    mo = np.empty(theta.shape, np.float32)
    vo = np.empty(theta.shape, np.float32)
    for b in range(B):
        a, c, d = ops.adam_step(theta[b], grad[b], m[b], v[b], lr[b], beta1[b], beta2[b],
                                eps[b], wd[b], t, decoupled_wd)
        th[b], mo[b], vo[b] = a, c, d
    return th, mo, vo


def adadelta_step(B, theta, grad, sq_avg, acc_delta, lr, rho, eps, wd):
    """Arena tensors [B, P]; hyper-parameter vectors [B].  State is stored fp32."""
    th, vo, uo = (np.empty(theta.shape, np.float32) for _ in range(3))
    for b in range(B):
        th[b], vo[b], uo[b] = ops.adadelta_step(theta[b], grad[b], sq_avg[b], acc_delta[b], lr[b], rho[b], eps[b], wd[b])
    return th, vo, uo
