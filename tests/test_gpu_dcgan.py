"""Whole-iteration parity of the fused DCGAN-style array (grouped Conv2d / ConvTranspose2d with
groups = B, per-model BatchNorm, two Adam optimisers) against B separate unfused oracle GANs."""
import dataclasses

import numpy as np
import pytest
import torch

import hfta_inputs as hi
from oracle import dcgan as odc

pytestmark = pytest.mark.gpu


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
    # a free-running chain of ~60 library calls per iteration: per-operator bound times a few for
    # bf16 (errors do not add coherently), times the call count for fp32
    tol = 1e-5 * 60 if dtype == "f32" else 1e-1
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
