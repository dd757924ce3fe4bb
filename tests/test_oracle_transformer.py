"""Pins for the Transformer-encoder oracle (no GPU needed): the attention core against brute-force
loops and torch's scaled_dot_product_attention; embedding forward/backward by loops; the whole
model against the same network written with torch's CPU float64 operators and differentiated by
autograd; Adam against torch.optim; independence of the models of an array."""
import dataclasses
import math

import numpy as np
import torch
import torch.nn.functional as F

import hfta_inputs as hi
from oracle import ops
from oracle import transformer as otr

T = lambda a: torch.tensor(np.asarray(a, np.float64), dtype=torch.float64)
RNG = np.random.default_rng(77)


def tiny_spec(B=2):
    return hi.TransformerSpec(name="tiny_tr", B=B, N=2, S=5, E=8, heads=2, F=12, layers=2, V=11, dtype="f64")


def test_attention_core_bruteforce_and_library():
    N, S, E, H = 2, 5, 8, 2
    d = E // H
    qkv = RNG.standard_normal((N, S, 3 * E))
    for causal in (False, True):
        ctx, p = ops.attention_fwd(qkv, H, causal)
        for n in range(N):
            for h in range(H):
                q, k, v = (qkv[n, :, j * E + h * d:j * E + (h + 1) * d] for j in range(3))
                for i in range(S):
                    js = [j for j in range(S) if (j <= i or not causal)]
                    sc = [sum(q[i, c] * k[j, c] for c in range(d)) / math.sqrt(d) for j in js]
                    mx = max(sc)
                    w = [math.exp(s_ - mx) for s_ in sc]
                    for jj, j in enumerate(js):
                        assert abs(p[n, h, i, j] - w[jj] / sum(w)) < 1e-12
                    if causal:
                        assert np.all(p[n, h, i, i + 1:] == 0.0)
                    for c in range(d):
                        ref = sum(w[jj] / sum(w) * v[j, c] for jj, j in enumerate(js))
                        assert abs(ctx[n, i, h * d + c] - ref) < 1e-12
        # library routine
        tq = T(qkv).requires_grad_()
        sp = lambda a: a.reshape(N, S, H, d).transpose(1, 2)
        o = F.scaled_dot_product_attention(sp(tq[..., :E]), sp(tq[..., E:2 * E]), sp(tq[..., 2 * E:]), is_causal=causal)
        o = o.transpose(1, 2).reshape(N, S, E)
        np.testing.assert_allclose(ctx, o.detach().numpy(), rtol=0, atol=1e-12)
        r = RNG.standard_normal((N, S, E))
        (o * T(r)).sum().backward()
        np.testing.assert_allclose(ops.attention_bwd(qkv, p, r, H), tq.grad.numpy(), rtol=0, atol=1e-12)


def test_embedding_loops():
    V, E, R = 7, 3, 10
    table, idx, dy = RNG.standard_normal((V, E)), RNG.integers(0, V, R), RNG.standard_normal((R, E))
    pos = RNG.standard_normal((5, E))
    y = ops.embedding_fwd(table, idx, 1.5, pos)
    dt = ops.embedding_bwd(dy, idx, V, 1.5)
    ref = np.zeros((V, E))
    for r in range(R):
        for e in range(E):
            assert abs(y[r, e] - (1.5 * table[idx[r], e] + pos[r % 5, e])) < 1e-15
            ref[idx[r], e] += 1.5 * dy[r, e]
    np.testing.assert_allclose(dt, ref, rtol=0, atol=1e-14)


def torch_loss(spec, tp, tokens, targets):
    N, S = tokens.shape
    E, H = spec.E, spec.heads
    d = E // H
    x = tp["emb"][torch.tensor(tokens.reshape(-1).astype(np.int64))] * math.sqrt(E) + T(otr.positions(S, E)).repeat(N, 1)
    for i in range(spec.layers):
        k = f"l{i}"
        qkv = (x @ tp[k + ".in.w"] + tp[k + ".in.b"]).reshape(N, S, 3 * E)
        sp = lambda a: a.reshape(N, S, H, d).transpose(1, 2)
        o = F.scaled_dot_product_attention(sp(qkv[..., :E]), sp(qkv[..., E:2 * E]), sp(qkv[..., 2 * E:]), is_causal=True)
        a = o.transpose(1, 2).reshape(N * S, E) @ tp[k + ".out.w"] + tp[k + ".out.b"]
        x = F.layer_norm(x + a, (E,), tp[k + ".ln1.w"], tp[k + ".ln1.b"], 1e-5)
        y = F.relu(x @ tp[k + ".ff1.w"] + tp[k + ".ff1.b"]) @ tp[k + ".ff2.w"] + tp[k + ".ff2.b"]
        x = F.layer_norm(x + y, (E,), tp[k + ".ln2.w"], tp[k + ".ln2.b"], 1e-5)
    logits = x @ tp["dec.w"] + tp["dec.b"]
    return F.cross_entropy(logits, torch.tensor(targets.reshape(-1).astype(np.int64))), logits


def test_forward_backward_vs_autograd():
    spec = tiny_spec()
    inp = hi.transformer_inputs(spec, seed=31, perturb_ln=True)
    for b in range(spec.B):
        theta = {k: v.astype(np.float64) for k, v in inp["params"][b].items()}
        out = otr.forward_backward(spec, theta, inp["tokens"][b], inp["targets"][b])
        tp = {k: T(v).requires_grad_() for k, v in theta.items()}
        loss, logits = torch_loss(spec, tp, inp["tokens"][b], inp["targets"][b])
        loss.backward()
        assert abs(out["loss"] - loss.item()) < 1e-12
        np.testing.assert_allclose(out["logits"], logits.detach().numpy(), rtol=0, atol=1e-12)
        for k in theta:
            g = tp[k].grad.numpy()
            assert np.abs(out["grads"][k] - g).max() <= 1e-10 * max(np.abs(g).max(), 1e-3), k


def test_train_step_vs_torch_adam_and_independence():
    spec = tiny_spec(B=3)
    inp = hi.transformer_inputs(spec, seed=32, perturb_ln=True)
    states = [otr.init_state(inp["params"][b]) for b in range(spec.B)]
    tps = [{k: T(v).requires_grad_() for k, v in inp["params"][b].items()} for b in range(spec.B)]
    opts = [torch.optim.Adam(list(tps[b].values()), lr=float(inp["lr"][b])) for b in range(spec.B)]
    for t in (1, 2):
        otr.array_train_step(spec, states, inp, t)
        for b in range(spec.B):
            opts[b].zero_grad()
            torch_loss(spec, tps[b], inp["tokens"][b], inp["targets"][b])[0].backward()
            opts[b].step()
            for k, v in tps[b].items():
                ref = v.detach().numpy()
                assert np.abs(states[b]["theta"][k] - ref).max() <= 2e-6 * max(np.abs(ref).max(), 1e-3), (t, b, k)
    s1 = dataclasses.replace(spec, B=1)
    i1 = {k: (v[1:2] if isinstance(v, np.ndarray) else v) for k, v in inp.items()}
    i1["params"] = [inp["params"][1]]
    alone = [otr.init_state(inp["params"][1])]
    for t in (1, 2):
        otr.array_train_step(s1, alone, i1, t)
    for k in alone[0]["theta"]:
        assert np.array_equal(alone[0]["theta"][k], states[1]["theta"][k]), k


def test_position_table_input_matches_the_definition():
    """The table the input module hands to the device is the oracle's closed form, to float32."""
    from oracle import transformer as otr
    for S, E in ((64, 256), (7, 10)):
        np.testing.assert_array_equal(hi.position_table(S, E), otr.positions(S, E).astype(np.float32))
