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
float32; arithmetic inside an operator is float64.  With ``fused_tail`` the last
per-point layer, its BatchNorm, ReLU and the max over points are ONE operator
(``ops.conv1x1_bn_maxpool_fwd`` / ``_bwd``), forward and backward: it keeps no
[N, C, L] tensor, so nothing inside it is rounded; only its pooled output and
its input gradient are stored.
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


def forward_backward(spec, theta, points, labels, drop_mask=None, running=None,
                     bn_eps=1e-5, bn_momentum=0.1, fused_tail=False):
    """Forward + backward of one model.

    points:[Nb,3,L], labels:[Nb], drop_mask:[Nb,F] or None.
    Returns dict(loss, logits, grads{name->float64}, pool_idx, acts{...}, running{...}).
    """
    dt = spec.dtype
    S = lambda a: ops.store(a, dt)
    sdt = "f64" if dt == "f64" else "f32"       # saved statistics are float32 on the device
    lp = {k: (S(v) if k.endswith(".w") or (k.endswith(".b") and ".bn." not in k) else
              np.asarray(v, np.float64)) for k, v in theta.items()}
    nconv = len(spec.conv) - 1
    nfc = len(spec.fc) - 1
    new_running = {}
    saved = {}

    # ---------------- forward: per-point MLP
    a = np.asarray(points, np.float64)
    for i in range(nconv):
        rm = rv = None
        if running is not None:
            rm, rv = running[f"conv{i}.bn.rm"], running[f"conv{i}.bn.rv"]
        if fused_tail and i == nconv - 1:
            pooled, idx, mean, invstd, nrm, nrv, _ = ops.conv1x1_bn_maxpool_fwd(
                a, lp[f"conv{i}.w"], lp[f"conv{i}.b"], lp[f"conv{i}.bn.g"], lp[f"conv{i}.bn.b"], bn_eps,
                bn_momentum, rm, rv, ops.ACT_RELU)
            mean, invstd = ops.store(mean, sdt), ops.store(invstd, sdt)
            if running is not None:
                new_running[f"conv{i}.bn.rm"], new_running[f"conv{i}.bn.rv"] = nrm, nrv
            saved[f"conv{i}"] = (a, None, None, mean, invstd)
            pooled = S(pooled)
            break
        z = S(ops.conv1x1_fwd(a, lp[f"conv{i}.w"], lp[f"conv{i}.b"]))
        y, mean, invstd, nrm, nrv = ops.bn_fwd(z, lp[f"conv{i}.bn.g"], lp[f"conv{i}.bn.b"],
                                               bn_eps, bn_momentum, rm, rv)
        mean, invstd = ops.store(mean, sdt), ops.store(invstd, sdt)
        if running is not None:
            new_running[f"conv{i}.bn.rm"], new_running[f"conv{i}.bn.rv"] = nrm, nrv
        saved[f"conv{i}"] = (a, z, y, mean, invstd)
        a = S(ops.act_fwd(y, ops.ACT_RELU))
    if not fused_tail:
        pooled, idx = ops.maxpool_points_fwd(a)
    Lp = a.shape[2]

    # ---------------- forward: head
    h = pooled
    for i in range(nfc):
        last = i == nfc - 1
        zl = ops.linear_fwd(h, lp[f"fc{i}.w"], lp[f"fc{i}.b"])
        if last:
            z = S(zl)
            saved[f"fc{i}"] = (h,)
            h = z
            break
        if spec.fc_bn:
            z = S(zl)
            rm = rv = None
            if running is not None:
                rm, rv = running[f"fc{i}.bn.rm"], running[f"fc{i}.bn.rv"]
            y, mean, invstd, nrm, nrv = ops.bn_fwd(z[:, :, None], lp[f"fc{i}.bn.g"],
                                                   lp[f"fc{i}.bn.b"], bn_eps, bn_momentum, rm, rv)
            mean, invstd = ops.store(mean, sdt), ops.store(invstd, sdt)
            if running is not None:
                new_running[f"fc{i}.bn.rm"], new_running[f"fc{i}.bn.rv"] = nrm, nrv
            y = y[:, :, 0]
            hn = S(ops.act_fwd(y, ops.ACT_RELU))
            saved[f"fc{i}"] = (h, z, y, mean, invstd)
        else:
            # Linear with the ReLU applied before the single store
            hn = S(ops.act_fwd(zl, ops.ACT_RELU))
            saved[f"fc{i}"] = (h, hn)
        if i == nfc - 2 and spec.dropout_p > 0:
            saved["drop_in"] = hn
            hn = S(ops.dropout_fwd(hn, drop_mask, spec.dropout_p))
        h = hn
    logits = h
    loss, dlogits = ops.softmax_xent(logits, labels)
    d = S(dlogits)

    # ---------------- backward: head
    grads = {}
    for i in reversed(range(nfc)):
        last = i == nfc - 1
        if not last:
            if i == nfc - 2 and spec.dropout_p > 0:
                d = S(ops.dropout_bwd(d, drop_mask, spec.dropout_p))
            if spec.fc_bn:
                hin, z, y, mean, invstd = saved[f"fc{i}"]
                dy = ops.act_bwd(y, d, ops.ACT_RELU)
                dz, dg, dbt = ops.bn_bwd(z[:, :, None], dy[:, :, None], lp[f"fc{i}.bn.g"],
                                         mean, invstd)
                grads[f"fc{i}.bn.g"], grads[f"fc{i}.bn.b"] = dg, dbt
                d = S(dz[:, :, 0])
            else:
                hin, hout = saved[f"fc{i}"]
                d = S(ops.act_bwd(hout, d, ops.ACT_RELU))   # mask from the stored output
        hin = saved[f"fc{i}"][0]
        dx, dw, db = ops.linear_bwd(hin, lp[f"fc{i}.w"], d)
        grads[f"fc{i}.w"], grads[f"fc{i}.b"] = dw, db
        d = S(dx)

    # ---------------- backward: pool and per-point MLP
    if not fused_tail:
        d = ops.maxpool_points_bwd(d, idx, Lp)      # exact scatter of stored values
    for i in reversed(range(nconv)):
        ain, z, y, mean, invstd = saved[f"conv{i}"]
        if fused_tail and i == nconv - 1:
            k = f"conv{i}"
            dx, dw, db, dg, dbt = ops.conv1x1_bn_maxpool_bwd(ain, lp[k + ".w"], lp[k + ".b"], lp[k + ".bn.g"],
                                                             lp[k + ".bn.b"], mean, invstd, d, idx, ops.ACT_RELU)
            grads[k + ".bn.g"], grads[k + ".bn.b"], grads[k + ".w"], grads[k + ".b"] = dg, dbt, dw, db
            if i > 0:
                d = S(dx)
            continue
        dy = ops.act_bwd(y, d, ops.ACT_RELU)
        dz, dg, dbt = ops.bn_bwd(z, dy, lp[f"conv{i}.bn.g"], mean, invstd)
        grads[f"conv{i}.bn.g"], grads[f"conv{i}.bn.b"] = dg, dbt
        dz = S(dz)
        dx, dw, db = ops.conv1x1_bwd(ain, lp[f"conv{i}.w"], dz)
        grads[f"conv{i}.w"], grads[f"conv{i}.b"] = dw, db
        if i > 0:
            d = S(dx)
    return dict(loss=loss, logits=logits, grads=grads, pool_idx=idx, pooled=pooled,
                running=new_running)


def train_step(spec, state, points, labels, hp: Dict[str, float], t: int, drop_mask=None, fused_tail=False):
    """One fwd + bwd + optimiser step of one model; updates ``state`` in place.
    hp: dict(lr, beta1, beta2, eps, wd) scalars for Adam, dict(lr, rho, eps, wd) for Adadelta.
    Returns the forward/backward dict."""
    out = forward_backward(spec, state["theta"], points, labels, drop_mask, state["running"], fused_tail=fused_tail)
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


def array_train_step(spec, states: List[dict], inp: dict, t: int, fused_tail=False):
    """The array's reference: B separate unfused runs, one after another."""
    outs = []
    for b in range(spec.B):
        hp = {k: float(inp[k][b]) for k in ("lr", "beta1", "beta2", "eps", "wd", "rho") if k in inp}
        mask = None if inp["drop_mask"] is None else inp["drop_mask"][b]
        outs.append(train_step(spec, states[b], inp["points"][:, 3 * b:3 * b + 3, :],
                               inp["labels"][b], hp, t, mask, fused_tail))
    return outs
