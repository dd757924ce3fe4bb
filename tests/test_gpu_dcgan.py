"""Parity of the fused DCGAN-style array (grouped Conv2d / ConvTranspose2d with groups = B, per-model
BatchNorm, two Adam optimisers) against the oracle: every library call of an iteration checked in
place on the bits it consumed at the per-operator tolerance, the free-running iteration against B
separate unfused oracle GANs, fused == serial."""
import dataclasses

import numpy as np
import pytest
import torch

import hfta_inputs as hi
from oracle import array as oa
from oracle import dcgan as odc
from oracle import ops as oops
from util import TOL, check

pytestmark = pytest.mark.gpu


def H64(t):
    return t.float().cpu().numpy().astype(np.float64)


def probe_for(spec, seen):
    """Per-call checks: the oracle's operator applied to the tensors (bits) the call read."""
    B, Nb, tol = spec.B, spec.Nb, TOL[spec.dtype]
    ftol = 1e-5 if spec.dtype == "f32" else 2e-4          # fp32 outputs (parameter gradients, statistics) of bf16 operands
    ACT = {1: oops.ACT_RELU, 2: oops.ACT_LEAKY, 3: oops.ACT_TANH}

    def img(t, C, hw):                                    # flat or 4-d device tensor -> float64 [Nb, B*C, hw, hw]
        return H64(t).reshape(-1)[:Nb * B * C * hw * hw].reshape(Nb, B * C, hw, hw)

    def cancel(x, g, mean, invstd, weight=None):
        """fp32 rounding of (x - mean), amplified by gamma*invstd (the operator's own conditioning)."""
        amp = np.abs(g) * invstd * (1.0 if weight is None else weight * invstd)
        return 4 * 2.0 ** -24 * amp[None, :, None] * (np.abs(x) + np.abs(mean)[None, :, None])

    def probe(op, **kw):
        torch.cuda.synchronize()
        seen.append(op)
        lay = kw.get("layer", "")
        if op in ("conv2d_fwd", "conv2d_dw", "conv2d_dx"):
            ci, co, st, p = kw["geo"]
            w = H64(kw["w"]).reshape(B * co, ci, 4, 4)
            x = H64(kw["x"])
            if op == "conv2d_fwd":
                y = oa.conv2d_fwd(B, x, w, None, st, p)
                if kw["act"]:
                    y = oops.act_fwd(y, ACT[kw["act"]], 0.2)
                check(H64(kw["y"]), y, tol, f"{lay} conv fwd")
                return
            hin, ho = kw["hw"]
            dx, dw, _ = oa.conv2d_bwd(B, x, w, img(kw["dy"], co, ho), st, p)
            if op == "conv2d_dw":
                check(H64(kw["dw"]).reshape(dw.shape), dw, ftol, f"{lay} conv dW")
            else:
                check(img(kw["dx"], ci, hin), dx, tol, f"{lay} conv dX")
        elif op in ("convT2d_fwd", "convT2d_dw", "convT2d_dx"):
            ci, co, st, p = kw["geo"]
            w = H64(kw["w"]).reshape(B * ci, co, 4, 4)
            x = H64(kw["x"])
            if op == "convT2d_fwd":
                check(H64(kw["y"]), oa.convT2d_fwd(B, x, w, None, st, p), tol, f"{lay} convT fwd")
                return
            hin, ho = kw["hw"]
            dx, dw, _ = oa.convT2d_bwd(B, x, w, img(kw["dy"], co, ho), st, p)
            if op == "convT2d_dw":
                check(H64(kw["dw"]).reshape(dw.shape), dw, ftol, f"{lay} convT dW")
            else:
                check(img(kw["dx"], ci, hin), dx, tol, f"{lay} convT dX")
        elif op == "bn_fwd":
            x = H64(kw["x"])
            n, c = x.shape[:2]
            x3 = x.reshape(n, c, -1)
            g, bt = H64(kw["g"]), H64(kw["b"])
            y, mean, invstd, _, _ = oa.bn_fwd(B, x3, g, bt, 1e-5, 0.1, None, None, "conv")
            check(H64(kw["y"]).reshape(x3.shape), oops.act_fwd(y, ACT[kw["act"]], 0.2), tol, f"{lay} bn",
                  cancel(x3, g, mean, invstd))
            check(H64(kw["mean"]), mean, 1e-5, f"{lay} bn mean")
            check(H64(kw["invstd"]), invstd, 1e-5, f"{lay} bn invstd")
        elif op == "bn_bwd":
            x = H64(kw["x"])
            n, c = x.shape[:2]
            x3 = x.reshape(n, c, -1)
            g, bt, mean, invstd = H64(kw["g"]), H64(kw["b"]), H64(kw["mean"]), H64(kw["invstd"])
            y = oa.bn_fwd(B, x3, g, bt, 1e-5, 0.1, None, None, "conv")[0]
            dy = oops.act_bwd(y, H64(kw["dy"]).reshape(x3.shape), ACT[kw["act"]], 0.2)
            dx, dg, db = oa.bn_bwd(B, x3, dy, g, mean, invstd, "conv")
            mg = np.abs(dg) / (dy.size / dg.size)
            check(H64(kw["dx"]).reshape(x3.shape), dx, tol, f"{lay} bn dx", cancel(x3, g, mean, invstd, mg))
            for got, ref, nm in ((H64(kw["dg"]), dg, "dgamma"), (H64(kw["db"]), db, "dbeta")):
                scale = max(np.abs(ref).max(), np.abs(dy).sum() / ref.size * 1e-3)     # sums of signed terms
                assert np.abs(got.reshape(-1) - ref).max() <= ftol * 10 * scale, f"{lay} bn {nm}"
        elif op == "act_fwd":
            check(H64(kw["y"]), oops.act_fwd(H64(kw["x"]), ACT[kw["act"]], 0.2), tol, f"{lay} act")
        elif op == "act_bwd_from_output":
            y = H64(kw["y"])
            dy = H64(kw["dy"]).reshape(y.shape)
            if kw["act"] == 3:                      # tanh' = 1 - y^2 from the stored output
                ref = dy * (1.0 - y * y)
            else:                                   # LeakyReLU: the output has the input's sign
                ref = oops.act_bwd(y, dy, oops.ACT_LEAKY, 0.2)
            check(H64(kw["dx"]).reshape(y.shape), ref, tol, f"{lay} act bwd")
        elif op == "bce":
            lg, tg = H64(kw["logits"]).reshape(Nb, B).T, H64(kw["targets"]).reshape(Nb, B).T
            loss, d = oa.bce_logits(B, lg, tg)
            check(H64(kw["loss"]), loss, 1e-5, "bce loss")
            check(H64(kw["d"]).reshape(Nb, B).T, d, tol, "bce grad")
        elif op == "grad_add":
            assert np.array_equal(H64(kw["y"]), (kw["a"] + kw["b"]).double().cpu().numpy())
        else:
            raise AssertionError(op)
    return probe


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_dcgan_every_call_in_place(dtype):
    """One whole iteration (generator forward, discriminator step on real + fake, generator step) of
    the 64x64 architecture with channels / 8, B = 2 models, 6 images each: every library call is
    compared in place with the oracle's operator on the bits the call consumed, at the per-operator
    tolerance (2e-2 bf16, 1e-5 fp32; fp32 parameter gradients of bf16 operands 2e-4).  Nothing is
    reloaded from the oracle in between: the device's own tensors flow through the iteration."""
    from paper_2102_02344_amd.arrays import FusedDcgan
    spec = hi.dcgan_thin(2, 6, dtype, div=8, cz=12)
    inp = hi.dcgan_inputs(spec, seed=79)
    arr = FusedDcgan(spec, inp)
    seen = []
    arr.probe = probe_for(spec, seen)
    arr.train_step()
    torch.cuda.synchronize()
    ng, nd = len(spec.g_layers), len(spec.d_layers)
    assert seen.count("convT2d_fwd") == ng and seen.count("convT2d_dw") == ng and seen.count("convT2d_dx") == ng - 1
    assert seen.count("conv2d_fwd") == 3 * nd and seen.count("conv2d_dw") == 2 * nd
    assert seen.count("conv2d_dx") == 2 * (nd - 1) + nd
    assert seen.count("bn_fwd") == (ng - 1) + 3 * (nd - 2) and seen.count("bn_bwd") == (ng - 1) + 3 * (nd - 2)
    assert seen.count("bce") == 3 and seen.count("grad_add") == 1


def rel(a, ref):
    return np.abs(a - ref).max() / max(np.abs(ref).max(), 1e-30)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_iterations_match_the_oracle(dtype):
    from paper_2102_02344_amd.arrays import FusedDcgan
    spec = hi.dcgan_thin(2, 4, dtype, div=16, cz=12)
    inp = hi.dcgan_inputs(spec, seed=77)
    arr = FusedDcgan(spec, inp)
    gs = [odc.init_state(p) for p in inp["gparams"]]
    ds = [odc.init_state(p) for p in inp["dparams"]]
    # a free-running chain of ~60 library calls per iteration (every one of them is held to the
    # per-operator tolerance by test_dcgan_every_call_in_place): per-operator bound times the call
    # count for fp32, times three for bf16 (errors do not add coherently), as the other arrays' chains
    tol = 1e-5 * 60 if dtype == "f32" else 6e-2
    B = spec.B
    # bf16: one iteration -- after an Adam step (+-lr where a noise-level gradient's sign differs) a
    # second free-running bf16 iteration through BatchNorm on 4-image batches is no longer comparable
    for t in ((1, 2) if dtype == "f32" else (1,)):
        print(f"{spec.name}: iteration {t}", flush=True)
        outs = odc.array_train_iteration(spec, gs, ds, inp, t)
        arr.g_forward()
        torch.cuda.synchronize()
        fake = arr.fake.float().cpu().numpy()
        for b in range(B):
            assert rel(fake[:, 3 * b:3 * b + 3], outs[b]["fake"]) <= tol, (b, t)
        arr.d_step()
        torch.cuda.synchronize()
        for b in range(B):
            assert abs(float(arr.loss_d_real[b]) - outs[b]["loss_d_real"]) <= tol * outs[b]["loss_d_real"]
            assert abs(float(arr.loss_d_fake[b]) - outs[b]["loss_d_fake"]) <= tol * outs[b]["loss_d_fake"]
            for name, _ in arr.D.shapes:
                g = arr.D.param_host(arr.D.grad, name, b).astype(np.float64)
                assert rel(g, outs[b]["grads_d"][name]) <= tol, (name, b, t, rel(g, outs[b]["grads_d"][name]))
        arr.D.adam()
        torch.cuda.synchronize()
        if dtype == "bf16":
            # Adam's first step moves every weight by lr, also where the gradient is rounding noise
            # and its sign differs between the two sides (2*lr against weights of 0.02): continue
            # the generator step from the oracle's discriminator so that it is checked on its own
            for b in range(B):
                for name, _ in arr.D.shapes:
                    th = arr.D.param_host(arr.D.theta, name, b).astype(np.float64)
                    assert np.abs(th - ds[b]["theta"][name]).max() <= 2.5 * float(inp["lr"][b]), (name, b)
            arr.D.load_params([ds[b]["theta"] for b in range(B)])
        arr.g_step_backward()
        torch.cuda.synchronize()
        for b in range(B):
            assert abs(float(arr.loss_g[b]) - outs[b]["loss_g"]) <= tol * outs[b]["loss_g"]
            for name, _ in arr.G.shapes:
                g = arr.G.param_host(arr.G.grad, name, b).astype(np.float64)
                assert rel(g, outs[b]["grads_g"][name]) <= tol, (name, b, t, rel(g, outs[b]["grads_g"][name]))
        arr.G.adam()
        torch.cuda.synchronize()
        for b in range(B):
            lr = float(inp["lr"][b])
            for arena, states, gk in ((arr.D, ds, "grads_d"), (arr.G, gs, "grads_g")):
                for name, _ in arena.shapes:
                    th = arena.param_host(arena.theta, name, b).astype(np.float64)
                    ref = states[b]["theta"][name].astype(np.float64)
                    gref = outs[b][gk][name]
                    ok = np.abs(gref) >= 1e-2 * np.abs(gref).max()     # Adam moves by ~lr*sign(g): compare where g is not noise
                    assert np.abs(th - ref)[ok].max() <= max(tol * np.abs(ref).max(), 10 * tol * lr * t), (name, b, t)
                    assert np.abs(th - ref).max() <= 2.5 * lr * t, (name, b, t)


def test_fused_array_equals_models_run_alone():
    from paper_2102_02344_amd.arrays import FusedDcgan
    spec = hi.dcgan_thin(3, 4, "bf16", div=16, cz=12)
    inp = hi.dcgan_inputs(spec, seed=78)
    arr = FusedDcgan(spec, inp)
    arr.train_step()
    torch.cuda.synchronize()
    cz = spec.g_layers[0][0]
    for b in range(spec.B):
        i1 = dict(inp)
        i1["z"] = np.ascontiguousarray(inp["z"][:, cz * b:cz * (b + 1)])
        i1["real"] = np.ascontiguousarray(inp["real"][:, 3 * b:3 * b + 3])
        i1["gparams"], i1["dparams"] = inp["gparams"][b:b + 1], inp["dparams"][b:b + 1]
        for k in ("lr", "beta1", "beta2", "eps", "wd"):
            i1[k] = inp[k][b:b + 1]
        one = FusedDcgan(dataclasses.replace(spec, B=1), i1)
        one.train_step()
        torch.cuda.synchronize()
        for la, lo in ((arr.loss_d_real, one.loss_d_real), (arr.loss_d_fake, one.loss_d_fake), (arr.loss_g, one.loss_g)):
            assert abs(float(la[b]) - float(lo[0])) <= 1e-5 * abs(float(la[b]))
        for A, O in ((arr.D, one.D), (arr.G, one.G)):
            for name, _ in A.shapes:
                ga, go = A.param_host(A.grad, name, b), O.param_host(O.grad, name, 0)
                assert np.abs(ga - go).max() <= 2e-3 * max(np.abs(ga).max(), 1e-30), name
