"""Fused Embedding, the multi-head attention core and the Transformer-encoder language-model array
on the GPU against the oracle: operators on their own, every library call of a step in place on
the bits the GPU consumed, the free-running step against B unfused oracle runs, fused == serial."""
import dataclasses
import math

import numpy as np
import pytest
import torch

import hfta_inputs as hi
from oracle import ops as oops
from oracle import transformer as otr
from test_gpu_mlp import probe_for
from util import DT, TOL, check

pytestmark = pytest.mark.gpu
TDT = {"f32": torch.float32, "bf16": torch.bfloat16}


def H64(t):
    return t.cpu().numpy() if t.dtype == torch.int32 else t.float().cpu().numpy().astype(np.float64)


@pytest.fixture(scope="module")
def hb():
    from paper_2102_02344_amd import binding
    return binding


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,N,S,E,H,causal", [(2, 3, 37, 48, 2, 1), (3, 2, 64, 64, 4, 0), (1, 2, 130, 32, 4, 1)])
def test_attention_core(hb, dtype, B, N, S, E, H, causal):
    print(f"attention {dtype} B={B} N={N} S={S} E={E} H={H} causal={causal}", flush=True)
    tdt, st = TDT[dtype], (lambda a: oops.store(a, dtype))
    qkv = hi.normal(201, (B, N, S, 3 * E), dtype)
    QKV = torch.from_numpy(qkv).to(tdt).cuda()
    P = torch.empty(B, N, H, S, S, dtype=tdt, device="cuda")
    CTX = torch.empty(B, N, S, E, dtype=tdt, device="cuda")
    hb.attention_fwd(B, N, S, E, H, DT[dtype], QKV, P, CTX, causal)
    dctx = hi.normal(202, (B, N, S, E), dtype)
    dCTX = torch.from_numpy(dctx).to(tdt).cuda()
    dQKV = torch.empty_like(QKV)
    ws = torch.empty(hb.attention_bwd_workspace_bytes(B, N, S, E, H, DT[dtype]), dtype=torch.uint8, device="cuda")
    hb.attention_bwd(B, N, S, E, H, DT[dtype], QKV, P, dCTX, dQKV, ws)
    gp = H64(P)
    for b in range(B):
        ctx, p = oops.attention_fwd(qkv[b], H, bool(causal), st)
        check(gp[b], p, TOL[dtype], "P")
        check(H64(CTX)[b], ctx, TOL[dtype], "ctx")
        if causal:
            assert np.all(gp[b][..., np.triu_indices(S, 1)[0], np.triu_indices(S, 1)[1]] == 0.0)
        # backward from the probabilities the GPU stored
        check(H64(dQKV)[b], oops.attention_bwd(qkv[b], gp[b], dctx[b], H, st), TOL[dtype], "dqkv")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_embedding(hb, dtype):
    B, R, V, E, S = 3, 500, 40, 24, 7          # 40 rows for 500 positions: every row collects many gradients
    tdt = TDT[dtype]
    table = hi.normal(211, (B, V, E), dtype)
    idx = np.random.default_rng(212).integers(0, V, (B, R)).astype(np.int32)
    idx[0, :50] = 3                             # a long run on one row; rows 30..39 of model 1 stay untouched
    idx[1] = idx[1] % 30
    pos = hi.normal(213, (S, E))
    T, I, Pz = torch.from_numpy(table).to(tdt).cuda(), torch.from_numpy(idx).cuda(), torch.from_numpy(pos).cuda()
    Y = torch.empty(B, R, E, dtype=tdt, device="cuda")
    hb.embedding_fwd(B, R, V, E, DT[dtype], T, I, 1.5, Pz, S, Y)
    dy = hi.normal(214, (B, R, E), dtype)
    dT = torch.full((B, V, E), 7.0, device="cuda")          # must be fully overwritten
    hb.embedding_bwd(B, R, V, E, DT[dtype], torch.from_numpy(dy).to(tdt).cuda(), I, 1.5, dT)
    for b in range(B):
        check(H64(Y)[b], oops.embedding_fwd(table[b], idx[b], 1.5, pos), TOL[dtype], "embedding")
        check(H64(dT)[b], oops.embedding_bwd(dy[b], idx[b], V, 1.5), 1e-5 if dtype == "f32" else 2e-4, "dtable")
    assert float(dT[1, 30:].abs().max()) == 0.0
    Y2 = torch.empty_like(Y)
    hb.embedding_fwd(B, R, V, E, DT[dtype], T, I, 1.0, None, 0, Y2)
    for b in range(B):
        assert np.array_equal(H64(Y2)[b], table[b][idx[b]].astype(np.float64))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("K", [1001, 1000, 8192, 4104, 16])    # odd width; rows kept in registers (ragged, full, fp32 too wide)
def test_softmax_xent_rows(hb, dtype, K):
    B, R = 3, 37
    tdt = TDT[dtype]
    z = hi.normal(221, (B, R, K), dtype, 3.0)
    lab = np.random.default_rng(222).integers(0, K, (B, R)).astype(np.int32)
    Z, L = torch.from_numpy(z).to(tdt).cuda(), torch.from_numpy(lab).cuda()
    loss = torch.empty(B, device="cuda")
    D = torch.empty_like(Z)
    ws = torch.empty(hb.softmax_xent_rows_workspace_bytes(B, R), dtype=torch.uint8, device="cuda")
    hb.softmax_xent_rows(B, R, K, DT[dtype], Z, L, loss, D, ws)
    for b in range(B):
        rl, rd = oops.softmax_xent(z[b], lab[b])
        assert abs(float(loss[b]) - rl) <= 1e-5 * abs(rl)
        check(H64(D)[b], rd, TOL[dtype], "dlogits")


def small(dtype, B=2):
    return hi.TransformerSpec(name=f"tr_small_{dtype}", B=B, N=3, S=37, E=48, heads=2, F=72, layers=2, V=101, dtype=dtype)


def tr_probe(spec, seen):
    base = probe_for(spec, seen)
    B, tol = spec.B, TOL[spec.dtype]
    st = lambda a: oops.store(a, spec.dtype)
    N, S, E, Hh, V = spec.N, spec.S, spec.E, spec.heads, spec.V

    def probe(op, **kw):
        torch.cuda.synchronize()
        if op in ("add", "layernorm_fwd", "layernorm_bwd", "linear_bwd"):
            return base(op, **kw)
        if op == "linear_fwd" and not kw["act"]:
            return base(op, **kw)
        seen.append(op)
        if op == "linear_fwd":                 # ReLU in the epilogue
            Fx = kw["x"].shape[2]
            for b in range(B):
                y = oops.linear_fwd(H64(kw["x"])[b], H64(kw["w"]).reshape(B, Fx, -1)[b], H64(kw["b"]).reshape(B, -1)[b])
                check(H64(kw["y"])[b], oops.act_fwd(y, oops.ACT_RELU), tol, "linear + relu")
        elif op == "embedding_fwd":
            for b in range(B):
                ref = oops.embedding_fwd(H64(kw["table"]).reshape(B, V, E)[b], H64(kw["idx"])[b], math.sqrt(E), H64(kw["pos"]))
                check(H64(kw["y"])[b], ref, tol, "embedding")
        elif op == "embedding_bwd":
            for b in range(B):
                ref = oops.embedding_bwd(H64(kw["dy"])[b], H64(kw["idx"])[b], V, math.sqrt(E))
                check(H64(kw["dtable"]).reshape(B, V, E)[b], ref, 1e-5 if spec.dtype == "f32" else 2e-4, "dtable")
        elif op == "attention_fwd":
            for b in range(B):
                ctx, p = oops.attention_fwd(H64(kw["qkv"])[b].reshape(N, S, 3 * E), Hh, True, st)
                check(H64(kw["p"])[b], p, tol, "P")
                check(H64(kw["ctx"])[b].reshape(N, S, E), ctx, tol, "ctx")
        elif op == "attention_bwd":
            for b in range(B):
                ref = oops.attention_bwd(H64(kw["qkv"])[b].reshape(N, S, 3 * E), H64(kw["p"])[b],
                                         H64(kw["dctx"])[b].reshape(N, S, E), Hh, st)
                check(H64(kw["dqkv"])[b].reshape(N, S, 3 * E), ref, tol, "dqkv")
        elif op == "softmax_xent":
            for b in range(B):
                loss, d = oops.softmax_xent(H64(kw["logits"])[b], H64(kw["labels"])[b])
                assert abs(float(kw["loss"][b]) - loss) <= 1e-5 * abs(loss)
                check(H64(kw["d"])[b], d, tol, "dlogits")
        elif op == "relu_bwd_from_output":
            ref = np.where(H64(kw["y"]) > 0, H64(kw["dy"]), 0.0)
            assert np.array_equal(H64(kw["dx"]), ref)
        else:
            raise AssertionError(op)
    return probe


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_transformer_every_call_in_place_and_chain(dtype):
    from paper_2102_02344_amd.arrays import FusedTransformerLM
    spec = small(dtype)
    inp = hi.transformer_inputs(spec, seed=51, perturb_ln=True)
    arr = FusedTransformerLM(spec, inp)
    seen = []
    arr.forward_backward(tr_probe(spec, seen))
    nl = spec.layers
    assert seen.count("attention_fwd") == nl and seen.count("attention_bwd") == nl and seen.count("linear_bwd") == 4 * nl + 1
    assert seen.count("embedding_fwd") == 1 and seen.count("embedding_bwd") == 1 and seen.count("layernorm_bwd") == 2 * nl
    states = [otr.init_state(inp["params"][b]) for b in range(spec.B)]
    outs = otr.array_train_step(spec, states, inp, 1)
    tol = 6e-2 if dtype == "bf16" else 1e-5 * (22 * nl + 6)
    loss = arr.loss.cpu().numpy()
    for b in range(spec.B):
        assert abs(loss[b] - outs[b]["loss"]) <= tol * abs(outs[b]["loss"]), (b, loss[b], outs[b]["loss"])
    if dtype == "f32":
        for b in range(spec.B):
            for name, _ in arr.shapes:
                g = arr.param_host(arr.grad, name, b).astype(np.float64)
                ref = outs[b]["grads"][name]
                err = np.abs(g - ref).max() / max(np.abs(ref).max(), 1e-30)
                assert err <= tol, (name, b, err)
        arr.adam()
        torch.cuda.synchronize()
        for b in range(spec.B):
            for name, _ in arr.shapes:
                th = arr.param_host(arr.theta, name, b).astype(np.float64)
                assert np.abs(th - states[b]["theta"][name]).max() <= 2.5 * float(inp["lr"][b]), (name, b)


def test_transformer_fused_equals_serial_B1_on_gpu():
    from paper_2102_02344_amd.arrays import FusedTransformerLM
    spec = small("bf16", B=3)
    inp = hi.transformer_inputs(spec, seed=52, perturb_ln=True)
    arr = FusedTransformerLM(spec, inp)
    arr.train_step()
    s1 = dataclasses.replace(spec, B=1)
    i1 = {k: (v[1:2] if isinstance(v, np.ndarray) and k != "pos" else v) for k, v in inp.items()}
    i1["params"] = [inp["params"][1]]
    one = FusedTransformerLM(s1, i1)
    one.train_step()
    torch.cuda.synchronize()
    assert abs(float(arr.loss[1]) - float(one.loss[0])) <= 1e-6 * abs(float(one.loss[0]))
    for name, _ in arr.shapes:
        a, o = arr.param_host(arr.theta, name, 1), one.param_host(one.theta, name, 0)
        assert np.array_equal(a, o), name
