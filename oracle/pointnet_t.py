"""CPU oracle: one training step of ONE PointNet-cls-style model WITH the input / feature
transform sub-networks, unfused.

TEST INFRASTRUCTURE ONLY (see oracle/ops.py).

Architecture (workload description of the point-cloud benchmark; appendix table of
hyper-parameters lists the feature transform as a per-model switch): a transform sub-network is
itself a small classification-style chain (per-point layers k -> 64 -> 128 -> 1024 with BatchNorm
and ReLU, max over points, Linear 1024 -> 512 -> 256 with BatchNorm and ReLU, Linear 256 -> k*k);
its output plus the identity is a k x k matrix per cloud that multiplies every point of the
cloud.  The input transform (k = 3) acts on the coordinates, the feature transform (k = 64) on the
output of the first per-point layer.  Reading: the k*k outputs are taken as T[o][c] (row = output
channel), y[:, l] = T x[:, l]; the other orientation is the same model with the last Linear's
output units relabelled.

Storage rounding as in oracle/pointnet.py: every tensor kept between two operators is rounded once
(T, the transformed points, their gradients).
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np

from . import ops
from . import pointnet as pn

init_state = pn.init_state


def _tnet_cfg(tspec, k: int):
    s = tspec.cls
    return pn.chain_cfg(s, conv=(k,) + tuple(tspec.tnet_conv), fc=(tspec.tnet_conv[-1],) + tuple(tspec.tnet_fc) + (k * k,),
                        prefix=f"t{k}.", dropout_p=0.0, fc_bn=True)


def _transform_fwd(tspec, k, lp, x, running, new_running, S, T_given=None, idx_given=None):
    cfg = _tnet_cfg(tspec, k)
    o, ctx = pn.chain_fwd(cfg, lp, x, None, running, new_running, idx_given=idx_given)
    T_own = S(o + np.eye(k).reshape(1, k * k)).reshape(-1, k, k)
    T = T_own if T_given is None else np.asarray(T_given, np.float64).reshape(-1, k, k)
    return S(ops.point_transform_fwd(x, T)), (cfg, ctx, T, x, T_own)


def _transform_bwd(lp, saved, dy, grads, S, want_dx):
    """dy: stored gradient of the transformed tensor.  Returns the stored gradient of x if want_dx."""
    cfg, ctx, T, x, _ = saved
    k = T.shape[1]
    dx_direct, dT = ops.point_transform_bwd(x, T, dy)
    dx_net = pn.chain_bwd(cfg, lp, ctx, S(dT).reshape(-1, k * k), grads, None, want_dx)
    return S(S(dx_direct) + dx_net) if want_dx else None


def forward_backward(tspec, theta, points, labels, drop_mask=None, running=None, T_given=None, idx_given=None):
    """Forward + backward of one model.  Returns dict(loss, logits, grads, running, T3, T64, pools).

    idx_given: {"main" | k: [Nb,C]} argmax positions to continue from in the main chain / the sub-network
    of size k (oracle/pointnet.py, module docstring); pools: the same keys -> (own argmax, own maximum,
    the stored tensor the maximum is taken over), for checking such positions.

    T_given: {k: [Nb,k,k]} replaces the stored matrix of a sub-network by a given one (the value a
    device run stored) from there on: a matrix entry near 1 has a storage ulp of 2^-8 in bf16, and
    one such last-bit difference moves every point of the cloud, after which the two runs take
    different argmax / ReLU decisions.  T3 / T64 in the result are the oracle's own matrices."""
    T_given = T_given or {}
    idx_given = idx_given or {}
    s = tspec.cls
    S = lambda v: ops.store(v, s.dtype)
    lp = pn.rounded_params(theta, s.dtype)
    new_running: Dict[str, np.ndarray] = {}
    x = np.asarray(points, np.float64)
    sv3 = sv64 = None
    if tspec.input_transform:
        x, sv3 = _transform_fwd(tspec, 3, lp, x, running, new_running, S, T_given.get(3), idx_given.get(3))
    cfg0 = pn.chain_cfg(s, conv=s.conv[:2], fc=None)
    x1, ctx0 = pn.chain_fwd(cfg0, lp, x, None, running, new_running)
    if tspec.feature_transform:
        x1, sv64 = _transform_fwd(tspec, s.conv[1], lp, x1, running, new_running, S, T_given.get(s.conv[1]),
                                  idx_given.get(s.conv[1]))
    cfg1 = pn.chain_cfg(s, conv=s.conv[1:], conv_base=1)
    logits, ctx1 = pn.chain_fwd(cfg1, lp, x1, drop_mask, running, new_running, idx_given=idx_given.get("main"))
    loss, dlogits = ops.softmax_xent(logits, labels)

    grads: Dict[str, np.ndarray] = {}
    d = pn.chain_bwd(cfg1, lp, ctx1, S(dlogits), grads, drop_mask, want_dx=True)
    if tspec.feature_transform:
        d = _transform_bwd(lp, sv64, d, grads, S, True)
    d = pn.chain_bwd(cfg0, lp, ctx0, d, grads, None, want_dx=tspec.input_transform)
    if tspec.input_transform:
        _transform_bwd(lp, sv3, d, grads, S, False)
    pools = {"main": (ctx1["idx_own"], ctx1["pooled_own"], ctx1["act"])}
    for k, sv in ((3, sv3), (s.conv[1], sv64)):
        if sv is not None:
            pools[k] = (sv[1]["idx_own"], sv[1]["pooled_own"], sv[1]["act"])
    return dict(loss=loss, logits=logits, grads=grads, running=new_running,
                T3=None if sv3 is None else sv3[4], T64=None if sv64 is None else sv64[4], pools=pools)


def train_step(tspec, state, points, labels, hp: Dict[str, float], t: int, drop_mask=None, T_given=None, idx_given=None):
    """One fwd + bwd + Adam step of one model; updates ``state`` (see oracle/pointnet.py) in place."""
    out = forward_backward(tspec, state["theta"], points, labels, drop_mask, state["running"], T_given, idx_given)
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


def array_train_step(tspec, states: List[dict], inp: dict, t: int, T_given=None, idx_given=None):
    """The array's reference: B separate unfused runs, one after another.  T_given, idx_given: per model, see forward_backward."""
    outs = []
    for b in range(tspec.cls.B):
        hp = {k: float(inp[k][b]) for k in ("lr", "beta1", "beta2", "eps", "wd")}
        mask = None if inp["drop_mask"] is None else inp["drop_mask"][b]
        outs.append(train_step(tspec, states[b], inp["points"][:, 3 * b:3 * b + 3, :], inp["labels"][b], hp, t,
                               mask, None if T_given is None else T_given[b], None if idx_given is None else idx_given[b]))
    return outs
