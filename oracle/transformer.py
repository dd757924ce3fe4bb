"""CPU oracle: one training step of ONE Transformer-encoder language model, unfused.

TEST INFRASTRUCTURE ONLY (see oracle/ops.py).  The reference for a fused array
of B models is B calls of ``train_step``, one model after another (section
"Methodology", paragraph "Baselines": the serial scheme).

Architecture (the Transformer language-model workload; fusion rules table rows
"Embedding", "Linear", "LayerNorm", "MultiheadAttention" /
"TransformerEncoderLayer", element-wise rows): token embedding scaled by
sqrt(E) plus fixed sinusoidal positions; ``layers`` post-norm encoder layers

    a = OutProj(Attention(InProj(x)));  x <- LayerNorm1(x + a)
    y = W2 relu(W1 x + b1) + b2;         x <- LayerNorm2(x + y)

with causal scaled-dot-product attention over ``heads`` heads; a Linear decoder
to the vocabulary; softmax cross-entropy against the next-token targets, mean
over the model's N*S tokens; Adam.  No dropout (its masks would be explicit
inputs like in the classification model).

Storage rounding: every tensor the library keeps in memory between two operators
is rounded once to the storage dtype; LayerNorm statistics, parameter gradients
and optimiser state are float32.
"""
from __future__ import annotations

import math
from typing import Dict, List

import numpy as np

from . import ops

LN_EPS = 1e-5


def positions(S: int, E: int) -> np.ndarray:
    """Fixed sinusoidal position table [S, E]: sin on even columns, cos on odd ones."""
    pe = np.zeros((S, E))
    pos = np.arange(S)[:, None]
    div = np.exp(np.arange(0, E, 2) * (-math.log(10000.0) / E))
    pe[:, 0::2] = np.sin(pos * div)
    pe[:, 1::2] = np.cos(pos * div)[:, :E // 2]
    return pe


def init_state(params: Dict[str, np.ndarray]) -> Dict[str, Dict[str, np.ndarray]]:
    return dict(theta={k: v.astype(np.float32).copy() for k, v in params.items()},
                m={k: np.zeros_like(v, np.float32) for k, v in params.items()},
                v={k: np.zeros_like(v, np.float32) for k, v in params.items()})


def forward_backward(spec, theta, tokens, targets):
    """tokens, targets: [N, S] int.  Returns dict(loss, logits, grads)."""
    dt = spec.dtype
    S_ = lambda a: ops.store(a, dt)
    sdt = "f64" if dt == "f64" else "f32"
    lp = {k: (np.asarray(v, np.float64) if ".ln" in k else S_(v)) for k, v in theta.items()}
    N, S = tokens.shape
    E, Hh, V = spec.E, spec.heads, spec.V
    R = N * S
    pe = ops.store(positions(S, E), sdt)                 # the position table is a float32 input on the device
    x = S_(ops.embedding_fwd(lp["emb"], tokens.reshape(-1), math.sqrt(E), pe))           # [R, E]
    saved = []
    for i in range(spec.layers):
        k = f"l{i}"
        qkv = S_(ops.linear_fwd(x, lp[k + ".in.w"], lp[k + ".in.b"]))
        ctx, p = ops.attention_fwd(qkv.reshape(N, S, 3 * E), Hh, True, S_)
        ctx = S_(ctx).reshape(R, E)
        a = S_(ops.linear_fwd(ctx, lp[k + ".out.w"], lp[k + ".out.b"]))
        s1 = S_(x + a)
        o1, mu1, inv1 = ops.layernorm_fwd(s1, lp[k + ".ln1.w"], lp[k + ".ln1.b"], LN_EPS)
        mu1, inv1 = ops.store(mu1, sdt), ops.store(inv1, sdt)
        x1 = S_(o1)
        h = S_(ops.act_fwd(ops.linear_fwd(x1, lp[k + ".ff1.w"], lp[k + ".ff1.b"]), ops.ACT_RELU))
        y = S_(ops.linear_fwd(h, lp[k + ".ff2.w"], lp[k + ".ff2.b"]))
        s2 = S_(x1 + y)
        o2, mu2, inv2 = ops.layernorm_fwd(s2, lp[k + ".ln2.w"], lp[k + ".ln2.b"], LN_EPS)
        mu2, inv2 = ops.store(mu2, sdt), ops.store(inv2, sdt)
        saved.append((x, qkv, p, ctx, s1, mu1, inv1, x1, h, s2, mu2, inv2))
        x = S_(o2)
    logits = S_(ops.linear_fwd(x, lp["dec.w"], lp["dec.b"]))
    loss, d = ops.softmax_xent(logits, targets.reshape(-1))
    d = S_(d)
    grads: Dict[str, np.ndarray] = {}
    dx, grads["dec.w"], grads["dec.b"] = ops.linear_bwd(x, lp["dec.w"], d)
    d = S_(dx)
    for i in reversed(range(spec.layers)):
        k = f"l{i}"
        xin, qkv, p, ctx, s1, mu1, inv1, x1, h, s2, mu2, inv2 = saved[i]
        ds2, grads[k + ".ln2.w"], grads[k + ".ln2.b"] = ops.layernorm_bwd(s2, d, lp[k + ".ln2.w"], mu2, inv2)
        ds2 = S_(ds2)
        dh, grads[k + ".ff2.w"], grads[k + ".ff2.b"] = ops.linear_bwd(h, lp[k + ".ff2.w"], ds2)
        du = S_(np.where(h > 0, S_(dh), 0.0))                               # ReLU from its stored output
        dx1, grads[k + ".ff1.w"], grads[k + ".ff1.b"] = ops.linear_bwd(x1, lp[k + ".ff1.w"], du)
        d1 = S_(ds2 + S_(dx1))
        ds1, grads[k + ".ln1.w"], grads[k + ".ln1.b"] = ops.layernorm_bwd(s1, d1, lp[k + ".ln1.w"], mu1, inv1)
        ds1 = S_(ds1)
        dctx, grads[k + ".out.w"], grads[k + ".out.b"] = ops.linear_bwd(ctx, lp[k + ".out.w"], ds1)
        dqkv = S_(ops.attention_bwd(qkv.reshape(N, S, 3 * E), p, S_(dctx).reshape(N, S, E), Hh, S_)).reshape(R, 3 * E)
        dxa, grads[k + ".in.w"], grads[k + ".in.b"] = ops.linear_bwd(xin, lp[k + ".in.w"], dqkv)
        d = S_(ds1 + S_(dxa))
    grads["emb"] = ops.embedding_bwd(d, tokens.reshape(-1), V, math.sqrt(E))
    return dict(loss=loss, logits=logits, grads=grads)


def train_step(spec, state, tokens, targets, hp: Dict[str, float], t: int):
    out = forward_backward(spec, state["theta"], tokens, targets)
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
