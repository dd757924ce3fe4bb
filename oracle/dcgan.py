"""CPU oracle: one training iteration of ONE DCGAN-style generator/discriminator pair, unfused.

TEST INFRASTRUCTURE ONLY (see oracle/ops.py).  The reference for a fused array
of B GANs is B calls of ``train_iteration``, one model after another (section
"Methodology", paragraph "Baselines": the serial scheme).

Architecture (the GAN workload; fusion rules table rows "Conv2d", "ConvT2d",
"BatchNorm2d" and the element-wise rows): all kernels 4x4.
  generator     z[100,1,1] -ConvT s1 p0-> 4x4 -ConvT s2 p1-> 8x8 -> 16x16 -> 32x32 -> 64x64,
                BatchNorm + ReLU after the first four, tanh after the last; no conv biases;
  discriminator 64x64 -Conv s2 p1-> 32x32 -> 16x16 -> 8x8 -> 4x4 -Conv s1 p0-> 1x1 logit,
                LeakyReLU(0.2) after the first, BatchNorm + LeakyReLU(0.2) after the next three.
One iteration: fake = G(z); discriminator step on loss BCE(D(real), 1) + BCE(D(fake), 0) with the
fake images held constant (each pass normalises with its own batch statistics), Adam on D; generator
step on BCE(D(fake), 1) through the updated discriminator, Adam on G.  Binary cross-entropy on the
logit, mean over the model's own batch.

Storage rounding: every activation / gradient tensor kept in memory between two operators is
rounded once to the storage dtype; BatchNorm statistics, parameter gradients and optimiser state
are float32; arithmetic inside an operator is float64.  Operators whose activation is applied in
the producing kernel's epilogue store only the activated tensor.
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np

from . import ops

BN_EPS = 1e-5
BN_MOMENTUM = 0.1
SLOPE = 0.2


def init_state(params: Dict[str, np.ndarray]) -> dict:
    st = dict(theta={k: v.astype(np.float32).copy() for k, v in params.items()},
              m={k: np.zeros_like(v, np.float32) for k, v in params.items()},
              v={k: np.zeros_like(v, np.float32) for k, v in params.items()}, running={})
    for k, val in params.items():
        if k.endswith(".bn.g"):
            st["running"][k[:-2] + ".rm"] = np.zeros_like(val, np.float32)
            st["running"][k[:-2] + ".rv"] = np.ones_like(val, np.float32)
    return st


def _lowp(theta, dt):
    return {k: (np.asarray(v, np.float64) if ".bn." in k else ops.store(v, dt)) for k, v in theta.items()}


def _bn(x, lp, k, running, sdt):
    rm = None if running is None else running.get(k + ".bn.rm")
    rv = None if running is None else running.get(k + ".bn.rv")
    N, C, H, W = x.shape
    y, mean, invstd, nrm, nrv = ops.bn_fwd(x.reshape(N, C, H * W), lp[k + ".bn.g"], lp[k + ".bn.b"], BN_EPS,
                                           BN_MOMENTUM, rm, rv)
    y = y.reshape(N, C, H, W)
    if running is not None:
        running[k + ".bn.rm"] = np.asarray(nrm, np.float32)
        running[k + ".bn.rv"] = np.asarray(nrv, np.float32)
    return y, ops.store(mean, sdt), ops.store(invstd, sdt)


def gen_forward(spec, lp, z, running):
    """z:[Nb,Cz,1,1] -> (fake:[Nb,3,64,64], saved)."""
    S = lambda a: ops.store(a, spec.dtype)
    sdt = "f64" if spec.dtype == "f64" else "f32"
    saved = []
    a = S(z)
    n = len(spec.g_layers)
    for i, (ci, co, hin, stride, pad) in enumerate(spec.g_layers):
        k = f"g{i}"
        pre = S(ops.convT2d_fwd(a, lp[k + ".w"], None, stride, pad))
        if i < n - 1:
            y, mean, invstd = _bn(pre, lp, k, running, sdt)
            out = S(ops.act_fwd(y, ops.ACT_RELU))
            saved.append((a, pre, mean, invstd))
        else:
            out = S(ops.act_fwd(pre, ops.ACT_TANH))
            saved.append((a, out))
        a = out
    return a, saved


def gen_backward(spec, lp, saved, dfake):
    S = lambda a: ops.store(a, spec.dtype)
    grads = {}
    n = len(spec.g_layers)
    d = dfake
    for i in reversed(range(n)):
        ci, co, hin, stride, pad = spec.g_layers[i]
        k = f"g{i}"
        if i == n - 1:
            ain, out = saved[i]
            dpre = S(d * (1.0 - out * out))               # tanh from its stored output
        else:
            ain, pre, mean, invstd = saved[i]
            y = (pre - mean[None, :, None, None]) * invstd[None, :, None, None] * lp[k + ".bn.g"][None, :, None, None] \
                + lp[k + ".bn.b"][None, :, None, None]
            dy = np.where(y > 0, d, 0.0)
            N_, C_, H_, W_ = pre.shape
            dpre, dg, db = ops.bn_bwd(pre.reshape(N_, C_, H_ * W_), dy.reshape(N_, C_, H_ * W_), lp[k + ".bn.g"],
                                      mean, invstd)
            dpre = dpre.reshape(N_, C_, H_, W_)
            grads[k + ".bn.g"], grads[k + ".bn.b"] = dg, db
            dpre = S(dpre)
        dx, dw, _ = ops.convT2d_bwd(ain, lp[k + ".w"], dpre, stride, pad)
        grads[k + ".w"] = dw
        d = S(dx)
    return grads


def disc_forward(spec, lp, x, running):
    """x:[Nb,3,64,64] -> (logits:[Nb], saved)."""
    S = lambda a: ops.store(a, spec.dtype)
    sdt = "f64" if spec.dtype == "f64" else "f32"
    saved = []
    a = x
    n = len(spec.d_layers)
    for i, (ci, co, hin, stride, pad) in enumerate(spec.d_layers):
        k = f"d{i}"
        pre = ops.conv2d_fwd(a, lp[k + ".w"], None, stride, pad)
        if i == 0:
            out = S(ops.act_fwd(pre, ops.ACT_LEAKY, SLOPE))     # activation in the conv epilogue
            saved.append((a, out))
        elif i < n - 1:
            pre = S(pre)
            y, mean, invstd = _bn(pre, lp, k, running, sdt)
            out = S(ops.act_fwd(y, ops.ACT_LEAKY, SLOPE))
            saved.append((a, pre, mean, invstd))
        else:
            out = S(pre)
            saved.append((a,))
        a = out
    return a.reshape(a.shape[0]), saved


def disc_backward(spec, lp, saved, dlogits, want_dw=True):
    """Returns (grads or None, d/d(input images))."""
    S = lambda a: ops.store(a, spec.dtype)
    grads = {}
    n = len(spec.d_layers)
    d = dlogits.reshape(-1, 1, 1, 1)
    for i in reversed(range(n)):
        ci, co, hin, stride, pad = spec.d_layers[i]
        k = f"d{i}"
        if i == n - 1:
            (ain,) = saved[i]
            dpre = d
        elif i == 0:
            ain, out = saved[i]
            dpre = S(np.where(out > 0, d, SLOPE * d))            # LeakyReLU from its stored output
        else:
            ain, pre, mean, invstd = saved[i]
            y = (pre - mean[None, :, None, None]) * invstd[None, :, None, None] * lp[k + ".bn.g"][None, :, None, None] \
                + lp[k + ".bn.b"][None, :, None, None]
            dy = np.where(y > 0, d, SLOPE * d)
            N_, C_, H_, W_ = pre.shape
            dpre, dg, db = ops.bn_bwd(pre.reshape(N_, C_, H_ * W_), dy.reshape(N_, C_, H_ * W_), lp[k + ".bn.g"],
                                      mean, invstd)
            dpre = dpre.reshape(N_, C_, H_, W_)
            grads[k + ".bn.g"], grads[k + ".bn.b"] = dg, db
            dpre = S(dpre)
        dx, dw, _ = ops.conv2d_bwd(ain, lp[k + ".w"], dpre, stride, pad)
        grads[k + ".w"] = dw
        d = S(dx)
    return (grads if want_dw else None), d


def _adam(state, grads, hp, t):
    for k in state["theta"]:
        g = ops.store(grads[k], "f32")
        th, m, v = ops.adam_step(state["theta"][k], g, state["m"][k], state["v"][k],
                                 hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["wd"], t)
        state["theta"][k] = th.astype(np.float32)
        state["m"][k] = m.astype(np.float32)
        state["v"][k] = v.astype(np.float32)


def train_iteration(spec, gstate, dstate, z, real, hp: Dict[str, float], t: int):
    """One iteration of one GAN; updates both states in place.  z:[Nb,Cz,1,1], real:[Nb,3,64,64].
    Returns dict(loss_d_real, loss_d_fake, loss_g, grads_d, grads_g, fake)."""
    dt = spec.dtype
    S = lambda a: ops.store(a, dt)
    Nb = real.shape[0]
    ones, zeros = np.ones(Nb), np.zeros(Nb)
    glp = _lowp(gstate["theta"], dt)
    fake, gsaved = gen_forward(spec, glp, z, gstate["running"])
    # ---- discriminator step
    dlp = _lowp(dstate["theta"], dt)
    lr_, sv = disc_forward(spec, dlp, S(real), dstate["running"])
    loss_r, dl = ops.bce_logits(lr_, ones)
    g_real, _ = disc_backward(spec, dlp, sv, S(dl))
    lf_, sv = disc_forward(spec, dlp, fake, dstate["running"])
    loss_f, dl = ops.bce_logits(lf_, zeros)
    g_fake, _ = disc_backward(spec, dlp, sv, S(dl))
    # the two passes' gradients are stored as float32 and then added
    grads_d = {k: ops.store(g_real[k], "f32") + ops.store(g_fake[k], "f32") for k in g_real}
    _adam(dstate, grads_d, hp, t)
    # ---- generator step through the updated discriminator
    dlp = _lowp(dstate["theta"], dt)
    lg_, sv = disc_forward(spec, dlp, fake, dstate["running"])
    loss_g, dl = ops.bce_logits(lg_, ones)
    _, dfake = disc_backward(spec, dlp, sv, S(dl), want_dw=False)
    grads_g = gen_backward(spec, glp, gsaved, dfake)
    _adam(gstate, grads_g, hp, t)
    return dict(loss_d_real=loss_r, loss_d_fake=loss_f, loss_g=loss_g, grads_d=grads_d, grads_g=grads_g,
                fake=fake)


def array_train_iteration(spec, gstates: List[dict], dstates: List[dict], inp: dict, t: int):
    """The array's reference: B separate unfused GANs, one after another."""
    outs = []
    for b in range(spec.B):
        hp = {k: float(inp[k][b]) for k in ("lr", "beta1", "beta2", "eps", "wd")}
        cz = spec.g_layers[0][0]
        outs.append(train_iteration(spec, gstates[b], dstates[b], inp["z"][:, cz * b:cz * (b + 1)],
                                    inp["real"][:, 3 * b:3 * b + 3], hp, t))
    return outs
