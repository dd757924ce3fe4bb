"""CPU oracle: one training step of ONE PointNet-segmentation-style model, unfused.

TEST INFRASTRUCTURE ONLY (see oracle/ops.py).  The reference for a fused array
of B models is B calls of ``train_step``, one model after another (section
"Methodology", paragraph "Baselines": the serial scheme).

Architecture (the point-cloud segmentation workload; fusion rules table rows
"Conv1d", "BatchNorm1d", element-wise rows; the max over points as in the
classification model): per-point MLP of k=1 convolutions, each followed by
training-mode BatchNorm and ReLU; the last feature map is also reduced by a max
over the points to a global feature; every per-point feature map, the global
feature tiled over the points and the object-category one-hot tiled over the
points are concatenated along the channel axis and fed to a per-point head of
k=1 convolutions (BatchNorm + ReLU on all but the last), whose output is a score
per part class and point; softmax cross-entropy with mean reduction over all the
model's points; Adam.

The concatenation is written out: the head's input is one stored
[Nb, c_point + c_global, L] tensor (np.concatenate of the feature maps and the
two tiled vectors), its first layer ONE k=1 convolution with ONE
[head[1], c_point + c_global] weight and one store, and the backward is that
convolution's adjoint followed by the adjoints of concatenate and tile (slice;
sum over the points).  How an implementation avoids forming the concatenation
is not the oracle's business.  Storage rounding as in oracle/pointnet.py: every
tensor kept in memory between two operators is rounded once to the storage dtype.
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np

from . import ops
from .pointnet import init_state  # noqa: F401  (same optimiser / running-statistics state)


def forward_backward(spec, theta, points, labels, onehot, running=None, bn_eps=1e-5, bn_momentum=0.1):
    """points:[Nb,3,L], labels:[Nb,L] int, onehot:[Nb,n_cat].  Returns dict(loss, logits, grads, pool_idx, running)."""
    dt = spec.dtype
    S = lambda a: ops.store(a, dt)
    sdt = "f64" if dt == "f64" else "f32"
    lp = {k: (np.asarray(v, np.float64) if ".bn." in k else S(v)) for k, v in theta.items()}
    nconv, nh = len(spec.conv) - 1, len(spec.head) - 1
    new_running, saved = {}, {}

    def bn_relu(name, z):
        rm = rv = None
        if running is not None:
            rm, rv = running[name + ".bn.rm"], running[name + ".bn.rv"]
        y, mean, invstd, nrm, nrv = ops.bn_fwd(z, lp[name + ".bn.g"], lp[name + ".bn.b"], bn_eps, bn_momentum, rm, rv)
        if running is not None:
            new_running[name + ".bn.rm"], new_running[name + ".bn.rv"] = nrm, nrv
        return y, ops.store(mean, sdt), ops.store(invstd, sdt)

    # ---- per-point MLP
    a = np.asarray(points, np.float64)
    feats = []
    for i in range(nconv):
        k = f"conv{i}"
        z = S(ops.conv1x1_fwd(a, lp[k + ".w"], lp[k + ".b"]))
        y, mean, invstd = bn_relu(k, z)
        saved[k] = (a, z, y, mean, invstd)
        a = S(ops.act_fwd(y, ops.ACT_RELU))
        feats.append(a)
    glob, idx = ops.maxpool_points_fwd(a)                      # [Nb, C], exact on stored values
    Nb, L = a.shape[0], a.shape[2]
    tile = lambda v: np.broadcast_to(np.asarray(v, np.float64)[:, :, None], v.shape + (L,))
    cat = np.concatenate(feats + [tile(glob), tile(S(onehot))], axis=1)   # [Nb, c_point + c_global, L]
    # ---- head
    h = cat
    for i in range(nh):
        k = f"head{i}"
        z = S(ops.conv1x1_fwd(h, lp[k + ".w"], lp[k + ".b"]))
        if i == nh - 1:
            saved[k] = (h,)
            h = z
            break
        y, mean, invstd = bn_relu(k, z)
        saved[k] = (h, z, y, mean, invstd)
        h = S(ops.act_fwd(y, ops.ACT_RELU))
    logits = h                                                  # [Nb, n_parts, L]
    flat = logits.transpose(0, 2, 1).reshape(Nb * L, -1)        # one row per point
    loss, dflat = ops.softmax_xent(flat, np.asarray(labels).reshape(-1))
    d = S(dflat.reshape(Nb, L, -1).transpose(0, 2, 1))

    # ---- backward: head
    grads = {}
    for i in reversed(range(nh)):
        k = f"head{i}"
        if i < nh - 1:
            hin, z, y, mean, invstd = saved[k]
            dz, dg, dbt = ops.bn_bwd(z, ops.act_bwd(y, d, ops.ACT_RELU), lp[k + ".bn.g"], mean, invstd)
            grads[k + ".bn.g"], grads[k + ".bn.b"] = dg, dbt
            d = S(dz)
        hin = saved[k][0]
        dx, dw, db = ops.conv1x1_bwd(hin, lp[k + ".w"], d)
        grads[k + ".w"], grads[k + ".b"] = dw, db
        d = S(dx)
    c_point, c4 = sum(spec.conv[1:]), spec.conv[-1]
    dcat = d[:, :c_point]                                       # adjoint of concatenate: slices of the stored gradient
    dglob = S(d[:, c_point:c_point + c4].sum(axis=2))           # adjoint of tile: sum over the points
    # ---- backward: per-point MLP; every feature map also receives its slice of the concatenation's gradient
    off = np.cumsum([0] + list(spec.conv[1:]))
    d = None
    for i in reversed(range(nconv)):
        k = f"conv{i}"
        ain, z, y, mean, invstd = saved[k]
        skip = dcat[:, off[i]:off[i + 1]]
        if i == nconv - 1:
            da = skip.copy()
            np.add.at(da, (np.arange(Nb)[:, None], np.arange(da.shape[1])[None, :], idx), dglob)
            da = S(da)                                           # sparse add onto the stored slice
        else:
            da = S(d + skip)
        dz, dg, dbt = ops.bn_bwd(z, ops.act_bwd(y, da, ops.ACT_RELU), lp[k + ".bn.g"], mean, invstd)
        grads[k + ".bn.g"], grads[k + ".bn.b"] = dg, dbt
        dz = S(dz)
        dx, dw, db = ops.conv1x1_bwd(ain, lp[k + ".w"], dz)
        grads[k + ".w"], grads[k + ".b"] = dw, db
        if i > 0:
            d = S(dx)
    return dict(loss=loss, logits=logits, grads=grads, pool_idx=idx, running=new_running)


def train_step(spec, state, points, labels, onehot, hp: Dict[str, float], t: int):
    out = forward_backward(spec, state["theta"], points, labels, onehot, state["running"])
    for k in state["theta"]:
        g = ops.store(out["grads"][k], "f32")
        th, m, v = ops.adam_step(state["theta"][k], g, state["m"][k], state["v"][k],
                                 hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["wd"], t)
        state["theta"][k] = th.astype(np.float32)
        state["m"][k] = m.astype(np.float32)
        state["v"][k] = v.astype(np.float32)
    for k, val in out["running"].items():
        state["running"][k] = np.asarray(val, np.float32)
    return out


def array_train_step(spec, states: List[dict], inp: dict, t: int):
    """The array's reference: B separate unfused runs, one after another."""
    outs = []
    for b in range(spec.B):
        hp = {k: float(inp[k][b]) for k in ("lr", "beta1", "beta2", "eps", "wd")}
        outs.append(train_step(spec, states[b], inp["points"][:, 3 * b:3 * b + 3, :], inp["labels"][b],
                               inp["onehot"][b], hp, t))
    return outs
