"""CPU oracle: one training step of ONE residual MLP-block model, unfused.

TEST INFRASTRUCTURE ONLY (see oracle/ops.py).  The reference for a fused array
of B models is B calls of ``train_step``, one model after another (section
"Methodology", paragraph "Baselines": the serial scheme), because the fused
array is defined to be equivalent to B independent trainings (section "Our
Proposal: HFTA", paragraph "Convergence").

Architecture (the Linear-heavy workload: fusion rules table rows "Linear" and
"LayerNorm" plus element-wise operators): ``blocks`` times

    u = x W1 + b1;  h = GELU(u);  y = h W2 + b2;  s = x + y;  x <- LayerNorm(s) * w + b

with GELU = x * Phi(x) (exact erf form) and LayerNorm over the feature axis
(biased variance, eps = 1e-5); mean-squared-error loss against a target of the
same shape, mean over the model's own R*E elements; Adam with L2 weight decay
added to the gradient.

Storage rounding: every tensor the library keeps in memory between two
operators (u, h, y, s, x and the matching gradients) is rounded once to the
storage dtype; LayerNorm statistics, parameter gradients and optimiser state
are float32; arithmetic inside an operator is float64.
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np

from . import ops

LN_EPS = 1e-5


def init_state(params: Dict[str, np.ndarray]) -> Dict[str, Dict[str, np.ndarray]]:
    return dict(theta={k: v.astype(np.float32).copy() for k, v in params.items()},
                m={k: np.zeros_like(v, np.float32) for k, v in params.items()},
                v={k: np.zeros_like(v, np.float32) for k, v in params.items()})


def forward_backward(spec, theta, x0, target):
    """x0, target: [R, E].  Returns dict(loss, out, grads{name -> float64})."""
    dt = spec.dtype
    S = lambda a: ops.store(a, dt)
    sdt = "f64" if dt == "f64" else "f32"
    # GEMM operands are the storage-dtype copies of the master weights; LayerNorm affine stays fp32
    lp = {k: (np.asarray(v, np.float64) if ".ln." in k else S(v)) for k, v in theta.items()}
    saved = []
    x = S(x0)
    for i in range(spec.blocks):
        k = f"blk{i}"
        u = S(ops.linear_fwd(x, lp[k + ".w1"], lp[k + ".b1"]))
        h = S(ops.act_fwd(u, ops.ACT_GELU))
        y = S(ops.linear_fwd(h, lp[k + ".w2"], lp[k + ".b2"]))
        s = S(x + y)
        o, mu, inv = ops.layernorm_fwd(s, lp[k + ".ln.w"], lp[k + ".ln.b"], LN_EPS)
        mu, inv = ops.store(mu, sdt), ops.store(inv, sdt)
        saved.append((x, u, h, s, mu, inv))
        x = S(o)
    loss, d = ops.mse(x, target)
    d = S(d)
    grads: Dict[str, np.ndarray] = {}
    for i in reversed(range(spec.blocks)):
        k = f"blk{i}"
        xin, u, h, s, mu, inv = saved[i]
        ds, dlw, dlb = ops.layernorm_bwd(s, d, lp[k + ".ln.w"], mu, inv)
        grads[k + ".ln.w"], grads[k + ".ln.b"] = dlw, dlb
        ds = S(ds)
        dh, dw2, db2 = ops.linear_bwd(h, lp[k + ".w2"], ds)
        grads[k + ".w2"], grads[k + ".b2"] = dw2, db2
        du = S(ops.act_bwd(u, S(dh), ops.ACT_GELU))
        dxl, dw1, db1 = ops.linear_bwd(xin, lp[k + ".w1"], du)
        grads[k + ".w1"], grads[k + ".b1"] = dw1, db1
        d = S(ds + S(dxl))
    return dict(loss=loss, out=x, grads=grads)


def train_step(spec, state, x0, target, hp: Dict[str, float], t: int):
    """One fwd + bwd + Adam step of one model; updates ``state`` in place."""
    out = forward_backward(spec, state["theta"], x0, target)
    for k in state["theta"]:
        g = ops.store(out["grads"][k], "f32")
        th, m, v = ops.adam_step(state["theta"][k], g, state["m"][k], state["v"][k],
                                 hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["wd"], t)
        state["theta"][k] = th.astype(np.float32)
        state["m"][k] = m.astype(np.float32)
        state["v"][k] = v.astype(np.float32)
    return out


def array_train_step(spec, states: List[dict], inp: dict, t: int):
    """The array's reference: B separate unfused runs, one after another."""
    outs = []
    for b in range(spec.B):
        hp = {k: float(inp[k][b]) for k in ("lr", "beta1", "beta2", "eps", "wd")}
        outs.append(train_step(spec, states[b], inp["tokens"][b], inp["targets"][b], hp, t))
    return outs
