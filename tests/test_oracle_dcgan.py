"""Pins for the oracle's DCGAN-style generator/discriminator iteration (CPU only).

The operators are pinned one by one in test_oracle_ops.py; here the wiring is: both optimisation
steps' gradients against central finite differences of the losses they descend, the generator's
first layer against the matrix product it reduces to on a 1x1 input, the output ranges the
architecture fixes, and the per-model independence that defines the fused array.
"""
import copy
import dataclasses

import numpy as np
import pytest

import hfta_inputs as hi
from oracle import dcgan, ops


def setup(dtype="f64", B=1, Nb=2, seed=3):
    spec = hi.dcgan_thin(B, Nb, dtype, div=32, cz=5)
    inp = hi.dcgan_inputs(spec, seed=seed)
    return spec, inp


def d_loss(spec, dtheta, real, fake):
    lp = dcgan._lowp(dtheta, spec.dtype)
    lr_, _ = dcgan.disc_forward(spec, lp, real, None)
    lf_, _ = dcgan.disc_forward(spec, lp, fake, None)
    return ops.bce_logits(lr_, np.ones(len(lr_)))[0] + ops.bce_logits(lf_, np.zeros(len(lf_)))[0]


def g_loss(spec, gtheta, dtheta, z):
    fake, _ = dcgan.gen_forward(spec, dcgan._lowp(gtheta, spec.dtype), z, None)
    lg_, _ = dcgan.disc_forward(spec, dcgan._lowp(dtheta, spec.dtype), fake, None)
    return ops.bce_logits(lg_, np.ones(len(lg_)))[0]


def test_both_steps_match_finite_differences():
    spec, inp = setup()
    z, real = inp["z"].astype(np.float64), inp["real"].astype(np.float64)
    g0 = {k: v.astype(np.float64) for k, v in inp["gparams"][0].items()}
    d0 = {k: v.astype(np.float64) for k, v in inp["dparams"][0].items()}
    gs, ds = dcgan.init_state(inp["gparams"][0]), dcgan.init_state(inp["dparams"][0])
    hp = dict(lr=float(inp["lr"][0]), beta1=0.5, beta2=0.999, eps=1e-8, wd=0.0)
    out = dcgan.train_iteration(spec, gs, ds, z, real, hp, 1)
    d_new = {k: v.astype(np.float64) for k, v in ds["theta"].items()}     # the G step sees the updated D
    rng = np.random.default_rng(1)
    h = 1e-6          # small: a BatchNorm shift moves every element of a channel across the LeakyReLU kink
    for theta, grads, f in ((d0, out["grads_d"], lambda th: d_loss(spec, th, real, out["fake"])),
                            (g0, out["grads_g"], lambda th: g_loss(spec, th, d_new, z))):
        for name, val in theta.items():
            flat = val.reshape(-1)
            for idx in rng.choice(flat.size, size=2, replace=False):
                keep = flat[idx]
                flat[idx] = keep + h
                lp = f(theta)
                flat[idx] = keep - h
                lm = f(theta)
                flat[idx] = keep
                fd = (lp - lm) / (2 * h)
                an = float(np.asarray(grads[name]).reshape(-1)[idx])
                assert abs(fd - an) <= 1e-4 * max(abs(an), abs(fd)) + 1e-8, (name, idx, fd, an)


def test_first_generator_layer_is_a_matrix_product_on_a_1x1_input():
    spec, inp = setup()
    w = inp["gparams"][0]["g0.w"].astype(np.float64)
    z = inp["z"].astype(np.float64)
    ci, co, _, s, p = spec.g_layers[0]
    y = ops.convT2d_fwd(z, w, None, s, p)
    ref = np.einsum("nc,cokl->nokl", z[:, :, 0, 0], w)
    np.testing.assert_allclose(y, ref, rtol=1e-13, atol=1e-15)


def test_shapes_and_ranges():
    spec, inp = setup("bf16", B=1, Nb=3)
    gs, ds = dcgan.init_state(inp["gparams"][0]), dcgan.init_state(inp["dparams"][0])
    hp = dict(lr=float(inp["lr"][0]), beta1=0.5, beta2=0.999, eps=1e-8, wd=0.0)
    out = dcgan.train_iteration(spec, gs, ds, inp["z"], inp["real"], hp, 1)
    assert out["fake"].shape == (3, 3, 64, 64) and np.abs(out["fake"]).max() <= 1.0      # tanh range
    for k in ("loss_d_real", "loss_d_fake", "loss_g"):
        assert 0.0 < out[k] < 5.0
    # at the N(0, 0.02^2) initialisation the logits are near zero: every loss is near log 2
    assert out["loss_d_real"] == pytest.approx(np.log(2.0), abs=0.35)
    assert set(out["grads_d"]) == set(ds["theta"]) and set(out["grads_g"]) == set(gs["theta"])


def test_models_are_independent():
    spec, inp = setup("bf16", B=2, Nb=2, seed=9)
    gs = [dcgan.init_state(p) for p in inp["gparams"]]
    ds = [dcgan.init_state(p) for p in inp["dparams"]]
    dcgan.array_train_iteration(spec, gs, ds, inp, 1)
    # change model 0's data and weights: model 1's results must not move by a bit
    inp2 = copy.deepcopy(inp)
    cz = spec.g_layers[0][0]
    inp2["z"][:, :cz] *= -1.0
    inp2["real"][:, :3] *= 0.5
    inp2["gparams"][0]["g0.w"] *= 2.0
    gs2 = [dcgan.init_state(p) for p in inp2["gparams"]]
    ds2 = [dcgan.init_state(p) for p in inp2["dparams"]]
    dcgan.array_train_iteration(spec, gs2, ds2, inp2, 1)
    for k in gs[1]["theta"]:
        assert np.array_equal(gs[1]["theta"][k], gs2[1]["theta"][k])
    for k in ds[1]["theta"]:
        assert np.array_equal(ds[1]["theta"][k], ds2[1]["theta"][k])
    assert not np.array_equal(ds[0]["theta"]["d0.w"], ds2[0]["theta"]["d0.w"])
