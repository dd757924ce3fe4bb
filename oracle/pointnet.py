"""CPU oracle: one training step of ONE PointNet-cls-style model, unfused.

TEST INFRASTRUCTURE ONLY (see oracle/ops.py).  The reference for a fused array
of B models is B calls of ``train_step`` -- the paper's "serial" scheme
(section "Methodology", paragraph "Baselines") -- because the fused array is
defined to be equivalent to B independent trainings (section "Our Proposal:
HFTA", paragraph "Convergence").

Architecture (from the workload description, not from any third-party code):
per-point MLP of kernel-length-1 convolutions, each followed by training-mode
BatchNorm and ReLU; max over the point axis; fully connected head where hidden
layers are Linear -> (BatchNorm) -> ReLU, an optional dropout after the last
hidden activation, a final Linear producing logits; softmax cross-entropy with
mean reduction over the model's own batch; Adam.

Storage rounding: every activation / activation-gradient tensor that the
library keeps in memory between two operators is rounded once to the storage
dtype (``ops.store``); statistics, parameter gradients and optimiser state are
float32; arithmetic inside an operator is float64.  The model is written as the
plain chain of single operators (convolution, BatchNorm, ReLU, max over points,
...), each storing its result; an implementation that merges some of them has to
stay within the tolerance of this chain.

``idx_given``: after a chain of floating-point operators the argmax of the max
over points can legitimately differ between two implementations at near-ties,
and from there on the two would differentiate different functions.  A chain-level
comparison therefore may hand the oracle the argmax another implementation took
(after checking it against the oracle's own values): the pooled feature is then
read at those positions and the backward scatters there.  Given as a pair
(argmax, pooled values) the oracle also continues from that pooled tensor (after
the caller has checked it against the oracle's own maximum), so that what follows
the max over points is compared on identical inputs.  Without it the oracle uses
its own argmax (lowest index among equal stored values).
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np

from . import ops


def init_state(params: Dict[str, np.ndarray]) -> Dict[str, Dict[str, np.ndarray]]:
    """Optimiser moments and BatchNorm running statistics for one model."""
    st = dict(theta={k: v.astype(np.float32).copy() for k, v in params.items()},
              m={k: np.zeros_like(v, np.float32) for k, v in params.items()},
              v={k: np.zeros_like(v, np.float32) for k, v in params.items()},
              running={})
    for k, val in params.items():
        if k.endswith(".bn.g"):
            st["running"][k[:-2] + ".rm"] = np.zeros_like(val, np.float32)
            st["running"][k[:-2] + ".rv"] = np.ones_like(val, np.float32)
    return st


def chain_cfg(spec, conv=None, fc="spec", conv_base=0, prefix="", dropout_p=None, fc_bn=None):
    """Description of one chain: per-point layers conv[0] -> conv[-1] named
    ``{prefix}conv{conv_base + i}``, then (unless fc is None) the max over points and the fully
    connected layers ``{prefix}fc{i}``.  Defaults: the whole classification model of ``spec``."""
    return dict(conv=tuple(spec.conv if conv is None else conv), fc=(tuple(spec.fc) if fc == "spec" else fc),
                conv_base=conv_base, prefix=prefix, dtype=spec.dtype,
                fc_bn=spec.fc_bn if fc_bn is None else fc_bn,
                dropout_p=spec.dropout_p if dropout_p is None else dropout_p)


def rounded_params(theta, dt):
    """What the device multiplies with: weights and biases in the storage dtype, BatchNorm affine in fp32."""
    return {k: (ops.store(v, dt) if k.endswith(".w") or (k.endswith(".b") and ".bn." not in k) else
                np.asarray(v, np.float64)) for k, v in theta.items()}


def chain_fwd(cfg, lp, a, drop_mask=None, running=None, new_running=None, bn_eps=1e-5, bn_momentum=0.1,
              idx_given=None):
    """Forward of one chain on a:[Nb,C,L].  Returns (out, ctx): out is the last activation
    [Nb,C',L] (no head) or the last Linear's output [Nb,K].  ctx["idx_own"] / ctx["pooled_own"] are the
    oracle's own argmax and maximum; ctx["idx"] / ctx["pooled"] what the chain continued from."""
    dt, px, cb = cfg["dtype"], cfg["prefix"], cfg["conv_base"]
    S = lambda v: ops.store(v, dt)
    sdt = "f64" if dt == "f64" else "f32"       # saved statistics are float32 on the device
    nconv = len(cfg["conv"]) - 1
    head = cfg["fc"] is not None
    nfc = len(cfg["fc"]) - 1 if head else 0
    new_running = {} if new_running is None else new_running
    saved = {}
    a = np.asarray(a, np.float64)
    for i in range(nconv):
        k = f"{px}conv{cb + i}"
        rm = rv = None
        if running is not None:
            rm, rv = running[k + ".bn.rm"], running[k + ".bn.rv"]
        z = S(ops.conv1x1_fwd(a, lp[k + ".w"], lp[k + ".b"]))
        y, mean, invstd, nrm, nrv = ops.bn_fwd(z, lp[k + ".bn.g"], lp[k + ".bn.b"], bn_eps, bn_momentum, rm, rv)
        mean, invstd = ops.store(mean, sdt), ops.store(invstd, sdt)
        if running is not None:
            new_running[k + ".bn.rm"], new_running[k + ".bn.rv"] = nrm, nrv
        saved[k] = (a, z, y, mean, invstd)
        a = S(ops.act_fwd(y, ops.ACT_RELU))
    ctx = dict(saved=saved, Lp=a.shape[2], idx=None, pooled=None, act=a)
    if not head:
        return a, ctx
    pooled, idx = ops.maxpool_points_fwd(a)
    ctx["idx_own"], ctx["pooled_own"] = idx, pooled
    if idx_given is not None:
        if isinstance(idx_given, tuple):
            idx, pooled = np.asarray(idx_given[0]), np.asarray(idx_given[1], np.float64)
        else:
            idx = np.asarray(idx_given)
            pooled = np.take_along_axis(a, idx[:, :, None].astype(np.int64), axis=2)[:, :, 0]
    ctx["idx"], ctx["pooled"] = idx, pooled

    h = pooled
    for i in range(nfc):
        k = f"{px}fc{i}"
        last = i == nfc - 1
        zl = ops.linear_fwd(h, lp[k + ".w"], lp[k + ".b"])
        if last:
            z = S(zl)
            saved[k] = (h,)
            h = z
            break
        if cfg["fc_bn"]:
            z = S(zl)
            rm = rv = None
            if running is not None:
                rm, rv = running[k + ".bn.rm"], running[k + ".bn.rv"]
            y, mean, invstd, nrm, nrv = ops.bn_fwd(z[:, :, None], lp[k + ".bn.g"], lp[k + ".bn.b"], bn_eps,
                                                   bn_momentum, rm, rv)
            mean, invstd = ops.store(mean, sdt), ops.store(invstd, sdt)
            if running is not None:
                new_running[k + ".bn.rm"], new_running[k + ".bn.rv"] = nrm, nrv
            y = y[:, :, 0]
            hn = S(ops.act_fwd(y, ops.ACT_RELU))
            saved[k] = (h, z, y, mean, invstd)
        else:
            # Linear with the ReLU applied before the single store
            hn = S(ops.act_fwd(zl, ops.ACT_RELU))
            saved[k] = (h, hn)
        if i == nfc - 2 and cfg["dropout_p"] > 0:
            hn = S(ops.dropout_fwd(hn, drop_mask, cfg["dropout_p"]))
        h = hn
    return h, ctx


def chain_bwd(cfg, lp, ctx, d, grads, drop_mask=None, want_dx=False):
    """Backward of one chain from d = gradient of its output (stored).  Fills ``grads``;
    returns the stored gradient of the chain's input if want_dx."""
    dt, px, cb = cfg["dtype"], cfg["prefix"], cfg["conv_base"]
    S = lambda v: ops.store(v, dt)
    nconv = len(cfg["conv"]) - 1
    head = cfg["fc"] is not None
    nfc = len(cfg["fc"]) - 1 if head else 0
    saved, idx = ctx["saved"], ctx["idx"]
    for i in reversed(range(nfc)):
        k = f"{px}fc{i}"
        last = i == nfc - 1
        if not last:
            if i == nfc - 2 and cfg["dropout_p"] > 0:
                d = S(ops.dropout_bwd(d, drop_mask, cfg["dropout_p"]))
            if cfg["fc_bn"]:
                hin, z, y, mean, invstd = saved[k]
                dy = ops.act_bwd(y, d, ops.ACT_RELU)
                dz, dg, dbt = ops.bn_bwd(z[:, :, None], dy[:, :, None], lp[k + ".bn.g"], mean, invstd)
                grads[k + ".bn.g"], grads[k + ".bn.b"] = dg, dbt
                d = S(dz[:, :, 0])
            else:
                hin, hout = saved[k]
                d = S(ops.act_bwd(hout, d, ops.ACT_RELU))   # mask from the stored output
        hin = saved[k][0]
        dx, dw, db = ops.linear_bwd(hin, lp[k + ".w"], d)
        grads[k + ".w"], grads[k + ".b"] = dw, db
        d = S(dx)

    if head:
        d = ops.maxpool_points_bwd(d, idx, ctx["Lp"])      # exact scatter of stored values
    for i in reversed(range(nconv)):
        k = f"{px}conv{cb + i}"
        ain, z, y, mean, invstd = saved[k]
        need_dx = i > 0 or want_dx
        dy = ops.act_bwd(y, d, ops.ACT_RELU)
        dz, dg, dbt = ops.bn_bwd(z, dy, lp[k + ".bn.g"], mean, invstd)
        grads[k + ".bn.g"], grads[k + ".bn.b"] = dg, dbt
        dz = S(dz)
        dx, dw, db = ops.conv1x1_bwd(ain, lp[k + ".w"], dz)
        grads[k + ".w"], grads[k + ".b"] = dw, db
        if need_dx:
            d = S(dx)
    return d if want_dx else None


def forward_backward(spec, theta, points, labels, drop_mask=None, running=None,
                     bn_eps=1e-5, bn_momentum=0.1, idx_given=None):
    """Forward + backward of one model.

    points:[Nb,3,L], labels:[Nb], drop_mask:[Nb,F] or None; idx_given:[Nb,C] or None (module docstring).
    Returns dict(loss, logits, grads{name->float64}, pool_idx, pooled (the oracle's own argmax and
    maximum), last_act (the stored [Nb,C,L] tensor the maximum is taken over), running{...}).
    """
    cfg = chain_cfg(spec)
    lp = rounded_params(theta, spec.dtype)
    new_running = {}
    logits, ctx = chain_fwd(cfg, lp, points, drop_mask, running, new_running, bn_eps, bn_momentum, idx_given)
    loss, dlogits = ops.softmax_xent(logits, labels)
    grads = {}
    chain_bwd(cfg, lp, ctx, ops.store(dlogits, spec.dtype), grads, drop_mask)
    return dict(loss=loss, logits=logits, grads=grads, pool_idx=ctx["idx_own"], pooled=ctx["pooled_own"],
                last_act=ctx["act"], running=new_running)


def train_step(spec, state, points, labels, hp: Dict[str, float], t: int, drop_mask=None, idx_given=None):
    """One fwd + bwd + optimiser step of one model; updates ``state`` in place.
    hp: dict(lr, beta1, beta2, eps, wd) scalars for Adam, dict(lr, rho, eps, wd) for Adadelta.
    Returns the forward/backward dict."""
    out = forward_backward(spec, state["theta"], points, labels, drop_mask, state["running"], idx_given=idx_given)
    for k in state["theta"]:
        g = ops.store(out["grads"][k], "f32")
        if "rho" in hp:     # Adadelta: the two state buffers hold the running square average and the accumulated delta
            th, m, v = ops.adadelta_step(state["theta"][k], g, state["m"][k], state["v"][k],
                                         hp["lr"], hp["rho"], hp["eps"], hp["wd"])
        else:
            th, m, v = ops.adam_step(state["theta"][k], g, state["m"][k], state["v"][k],
                                     hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["wd"], t)
        state["theta"][k] = th.astype(np.float32)
        state["m"][k] = m.astype(np.float32)
        state["v"][k] = v.astype(np.float32)
    for k, val in out["running"].items():
        state["running"][k] = np.asarray(val, np.float32)
    return out


def array_train_step(spec, states: List[dict], inp: dict, t: int, idx_given=None):
    """The array's reference: B separate unfused runs, one after another (idx_given: [B][Nb,C] or None)."""
    outs = []
    for b in range(spec.B):
        hp = {k: float(inp[k][b]) for k in ("lr", "beta1", "beta2", "eps", "wd", "rho") if k in inp}
        mask = None if inp["drop_mask"] is None else inp["drop_mask"][b]
        outs.append(train_step(spec, states[b], inp["points"][:, 3 * b:3 * b + 3, :],
                               inp["labels"][b], hp, t, mask, None if idx_given is None else idx_given[b]))
    return outs
