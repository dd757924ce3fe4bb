"""Pins for the oracle's residual MLP-block model (CPU only).

The model chains operators that are pinned one by one in test_oracle_ops.py; what is pinned
here is the wiring: gradients of the whole chain against central finite differences, the
residual/LayerNorm structure against a special case with a closed form, the per-model
independence that defines the fused array, and the Adam routing of per-model hyper-parameters.
"""
import dataclasses

import numpy as np
import pytest

import hfta_inputs as hi
from oracle import mlp, ops


def tiny(dtype="f64", B=2):
    return hi.MlpSpec(name="tiny", B=B, R=5, E=6, H=7, blocks=2, dtype=dtype, Nb=1)


def test_gradients_match_finite_differences():
    spec = tiny()
    inp = hi.mlp_inputs(spec, seed=11, perturb_ln=True)
    th = {k: v.astype(np.float64) for k, v in inp["params"][0].items()}
    x, tg = inp["tokens"][0].astype(np.float64), inp["targets"][0].astype(np.float64)
    out = mlp.forward_backward(spec, th, x, tg)
    rng = np.random.default_rng(0)
    h = 1e-6
    for name, val in th.items():
        flat = val.reshape(-1)
        for idx in rng.choice(flat.size, size=min(4, flat.size), replace=False):
            keep = flat[idx]
            flat[idx] = keep + h
            lp = mlp.forward_backward(spec, th, x, tg)["loss"]
            flat[idx] = keep - h
            lm = mlp.forward_backward(spec, th, x, tg)["loss"]
            flat[idx] = keep
            fd = (lp - lm) / (2 * h)
            an = out["grads"][name].reshape(-1)[idx]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)) + 1e-8, (name, idx, fd, an)


def test_zero_second_linear_reduces_to_layernorm_of_input():
    """W2 = 0, b2 = 0: each block is x <- LayerNorm(x) * w + b; two blocks of a textbook LayerNorm."""
    spec = tiny()
    inp = hi.mlp_inputs(spec, seed=12, perturb_ln=True)
    th = {k: v.astype(np.float64) for k, v in inp["params"][1].items()}
    for i in range(spec.blocks):
        th[f"blk{i}.w2"][:] = 0
        th[f"blk{i}.b2"][:] = 0
    x = inp["tokens"][1].astype(np.float64)
    out = mlp.forward_backward(spec, th, x, inp["targets"][1])["out"]
    ref = x
    for i in range(spec.blocks):
        mu = ref.mean(axis=1, keepdims=True)
        var = ref.var(axis=1, keepdims=True)          # biased
        ref = (ref - mu) / np.sqrt(var + 1e-5) * th[f"blk{i}.ln.w"] + th[f"blk{i}.ln.b"]
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-12)
    # and the first Linear cannot matter then: its gradient is exactly zero
    g = mlp.forward_backward(spec, th, x, inp["targets"][1])["grads"]
    assert np.abs(g["blk0.w1"]).max() == 0.0


def test_loss_is_mean_square_error_of_the_output():
    spec = tiny()
    inp = hi.mlp_inputs(spec, seed=13)
    th = inp["params"][0]
    out = mlp.forward_backward(spec, th, inp["tokens"][0], inp["targets"][0])
    d = out["out"] - inp["targets"][0].astype(np.float64)
    assert out["loss"] == pytest.approx(float((d * d).sum() / d.size), rel=1e-14)


def test_models_are_independent_and_permutation_equivariant():
    spec = tiny(dtype="bf16", B=3)
    inp = hi.mlp_inputs(spec, seed=14, perturb_ln=True)
    states = [mlp.init_state(p) for p in inp["params"]]
    mlp.array_train_step(spec, states, inp, 1)
    # model 2 trained alone
    s1 = dataclasses.replace(spec, B=1)
    i1 = dict(inp)
    for k in ("tokens", "targets", "lr", "wd", "beta1", "beta2", "eps"):
        i1[k] = inp[k][2:3]
    i1["params"] = inp["params"][2:3]
    alone = [mlp.init_state(inp["params"][2])]
    mlp.array_train_step(s1, alone, i1, 1)
    for k in states[2]["theta"]:
        assert np.array_equal(states[2]["theta"][k], alone[0]["theta"][k]), k
    # permuting the models permutes the results
    perm = [2, 0, 1]
    ip = dict(inp)
    for k in ("tokens", "targets", "lr", "wd", "beta1", "beta2", "eps"):
        ip[k] = inp[k][perm]
    ip["params"] = [inp["params"][j] for j in perm]
    sp = [mlp.init_state(p) for p in ip["params"]]
    mlp.array_train_step(spec, sp, ip, 1)
    for a, j in enumerate(perm):
        for k in sp[a]["theta"]:
            assert np.array_equal(sp[a]["theta"][k], states[j]["theta"][k])


def test_first_adam_step_moves_each_model_by_its_own_learning_rate():
    spec = tiny(dtype="f32", B=2)
    inp = hi.mlp_inputs(spec, seed=15, perturb_ln=True)
    inp["wd"][:] = 0.0
    inp["lr"][:] = (1e-3, 4e-3)
    states = [mlp.init_state(p) for p in inp["params"]]
    outs = mlp.array_train_step(spec, states, inp, 1)
    for b in range(2):
        for k, g in outs[b]["grads"].items():
            delta = states[b]["theta"][k].astype(np.float64) - inp["params"][b][k].astype(np.float64)
            big = np.abs(g) > 1e-6              # where |g| >> eps the first step is -lr * sign(g)
            np.testing.assert_allclose(delta[big], -float(inp["lr"][b]) * np.sign(g[big]), rtol=2e-3, atol=1e-9)


def test_storage_rounding_stays_close_to_exact_arithmetic():
    s64, sbf = tiny("f64", B=1), tiny("bf16", B=1)
    inp = hi.mlp_inputs(sbf, seed=16, perturb_ln=True)
    a = mlp.forward_backward(s64, inp["params"][0], inp["tokens"][0], inp["targets"][0])
    b = mlp.forward_backward(sbf, inp["params"][0], inp["tokens"][0], inp["targets"][0])
    assert b["loss"] == pytest.approx(a["loss"], rel=2e-2)
    for k in a["grads"]:
        scale = np.abs(a["grads"][k]).max() + 1e-12
        assert np.abs(a["grads"][k] - b["grads"][k]).max() <= 5e-2 * scale, k
