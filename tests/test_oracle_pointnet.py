"""Pins for the oracle's whole-model step (no GPU needed).

The per-model PointNet-cls-style step is compared with the same network built
from torch's CPU float64 operators and differentiated by autograd (a library
routine, independent of the oracle's hand-derived backward chain), with finite
differences of the loss, and with torch.optim.Adam for the update.
"""
import dataclasses

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import hfta_inputs as hi
from oracle import pointnet as opn

T = lambda a: torch.tensor(np.asarray(a, np.float64), dtype=torch.float64)


def tiny_spec(fc_bn, p):
    return hi.PointNetClsSpec(name="tiny", B=2, Nb=4, L=9, conv=(3, 5, 7), fc=(7, 6, 5, 4),
                              fc_bn=fc_bn, dropout_p=p, dtype="f64", n_classes=4, config_index=0)


def torch_model_loss(spec, tp, points, labels, mask, pool_at=None):
    a = T(points)
    for i in range(len(spec.conv) - 1):
        z = F.conv1d(a, tp[f"conv{i}.w"][:, :, None], tp[f"conv{i}.b"])
        a = F.relu(F.batch_norm(z, None, None, tp[f"conv{i}.bn.g"], tp[f"conv{i}.bn.b"], training=True, eps=1e-5))
    h = a.max(dim=2).values if pool_at is None else \
        torch.gather(a, 2, torch.tensor(np.asarray(pool_at, np.int64))[:, :, None])[:, :, 0]
    nfc = len(spec.fc) - 1
    for i in range(nfc):
        h = h @ tp[f"fc{i}.w"] + tp[f"fc{i}.b"]
        if i < nfc - 1:
            if spec.fc_bn:
                h = F.batch_norm(h, None, None, tp[f"fc{i}.bn.g"], tp[f"fc{i}.bn.b"], training=True, eps=1e-5)
            h = F.relu(h)
            if i == nfc - 2 and spec.dropout_p > 0:
                h = h * T(mask) / (1 - spec.dropout_p)
    return F.cross_entropy(h, torch.tensor(np.asarray(labels, np.int64))), h


@pytest.mark.parametrize("fc_bn,p", [(True, 0.3), (False, 0.0)])
def test_forward_backward_vs_autograd(fc_bn, p):
    spec = tiny_spec(fc_bn, p)
    inp = hi.pointnet_cls_inputs(spec, seed=5)
    for b in range(spec.B):
        theta = {k: v.astype(np.float64) + 0.05 * np.random.default_rng(b).standard_normal(v.shape)
                 for k, v in inp["params"][b].items()}
        pts = inp["points"][:, 3 * b:3 * b + 3, :]
        mask = None if inp["drop_mask"] is None else inp["drop_mask"][b]
        out = opn.forward_backward(spec, theta, pts, inp["labels"][b], mask)
        tp = {k: T(v).requires_grad_() for k, v in theta.items()}
        loss, logits = torch_model_loss(spec, tp, pts, inp["labels"][b], mask)
        loss.backward()
        assert abs(out["loss"] - loss.item()) < 1e-12
        np.testing.assert_allclose(out["logits"], logits.detach().numpy(), rtol=0, atol=1e-12)
        for k in theta:
            g = tp[k].grad.numpy()
            assert np.abs(out["grads"][k] - g).max() <= 1e-10 * max(np.abs(g).max(), 1e-3), k


def test_loss_gradient_finite_difference():
    spec = tiny_spec(True, 0.3)
    inp = hi.pointnet_cls_inputs(spec, seed=6)
    theta = {k: v.astype(np.float64) for k, v in inp["params"][0].items()}
    pts, lab, mask = inp["points"][:, 0:3, :], inp["labels"][0], inp["drop_mask"][0]
    out = opn.forward_backward(spec, theta, pts, lab, mask)
    rng = np.random.default_rng(0)
    for k in ("conv0.w", "conv1.b", "fc0.w", "fc1.bn.g", "fc2.w", "conv0.bn.b"):
        for _ in range(3):
            i = tuple(rng.integers(0, s) for s in theta[k].shape)
            h = 1e-6
            tp, tm = {n: v.copy() for n, v in theta.items()}, {n: v.copy() for n, v in theta.items()}
            tp[k][i] += h; tm[k][i] -= h
            fd = (opn.forward_backward(spec, tp, pts, lab, mask)["loss"]
                  - opn.forward_backward(spec, tm, pts, lab, mask)["loss"]) / (2 * h)
            assert abs(fd - out["grads"][k][i]) < 1e-6 * max(1.0, abs(fd)), (k, i)


def test_train_steps_vs_torch_adam_and_independence():
    spec = tiny_spec(True, 0.3)
    inp = hi.pointnet_cls_inputs(spec, seed=7)
    states = [opn.init_state(inp["params"][b]) for b in range(spec.B)]
    tparams = [{k: T(v).requires_grad_() for k, v in inp["params"][b].items()} for b in range(spec.B)]
    opts = [torch.optim.Adam(list(tparams[b].values()), lr=float(inp["lr"][b]),
                             betas=(float(inp["beta1"][b]), float(inp["beta2"][b])),
                             eps=float(inp["eps"][b])) for b in range(spec.B)]
    for t in range(1, 4):
        outs = opn.array_train_step(spec, states, inp, t)
        for b in range(spec.B):
            opts[b].zero_grad()
            loss, _ = torch_model_loss(spec, tparams[b], inp["points"][:, 3 * b:3 * b + 3, :],
                                       inp["labels"][b], inp["drop_mask"][b])
            loss.backward()
            opts[b].step()
            assert abs(outs[b]["loss"] - loss.item()) < 1e-4 * t
    for b in range(spec.B):
        for k in tparams[b]:
            ref = tparams[b][k].detach().numpy()
            # float32 optimiser state in the oracle vs float64 in torch
            assert np.abs(states[b]["theta"][k] - ref).max() < 2e-4, k
    # model 0 of the array == model 0 trained alone (B = 1), bit for bit
    spec1 = dataclasses.replace(spec, B=1)
    alone = [opn.init_state(inp["params"][0])]
    inp1 = {k: (v[:1] if isinstance(v, np.ndarray) and k != "points" else v) for k, v in inp.items()}
    inp1["points"] = inp["points"][:, 0:3, :]
    inp1["params"] = inp["params"][:1]
    for t in range(1, 4):
        opn.array_train_step(spec1, alone, inp1, t)
    for k in alone[0]["theta"]:
        assert np.array_equal(alone[0]["theta"][k], states[0]["theta"][k])
    # running statistics follow torch's convention (momentum 0.1, unbiased variance)
    assert all(np.all(np.isfinite(v)) for v in states[0]["running"].values())


def test_inputs_recipe():
    spec = hi.spec_c0()
    a, b = hi.pointnet_cls_inputs(spec), hi.pointnet_cls_inputs(spec)
    assert np.array_equal(a["points"], b["points"]) and np.array_equal(a["labels"], b["labels"])
    pts = a["points"].reshape(spec.Nb, spec.B, 3, spec.L)
    r = np.sqrt((pts.astype(np.float64) ** 2).sum(axis=2))
    assert r.max() <= 1.0 + 1e-6 and 0.6 < np.mean(r) < 0.9      # E[r] = 3/4 in the unit ball
    assert a["labels"].min() >= 0 and a["labels"].max() < 16
    assert np.all((a["lr"] >= 1e-4) & (a["lr"] <= 1e-2))
    # model b's data does not depend on B
    big = hi.pointnet_cls_inputs(dataclasses.replace(spec, B=3))
    assert np.array_equal(big["points"][:, :6], a["points"])
    # bf16 snapping yields bf16-representable values
    c1 = hi.pointnet_cls_inputs(hi.spec_c1(B=2, Nb=2, L=50))
    u = c1["points"].view(np.uint32)
    assert np.all(u & 0xFFFF == 0)
    assert c1["drop_mask"].shape == (2, 2, 256) and 0.5 < c1["drop_mask"].mean() < 0.9


def test_given_argmax():
    """Handing the oracle its own argmax changes nothing; handing it other positions gives the model
    whose global feature is read at those positions (checked against autograd on torch.gather)."""
    spec = tiny_spec(True, 0.3)
    inp = hi.pointnet_cls_inputs(spec, seed=8)
    theta = {k: v.astype(np.float64) for k, v in inp["params"][0].items()}
    pts, lab, mask = inp["points"][:, 0:3, :], inp["labels"][0], inp["drop_mask"][0]
    own = opn.forward_backward(spec, theta, pts, lab, mask)
    same = opn.forward_backward(spec, theta, pts, lab, mask, idx_given=own["pool_idx"])
    assert same["loss"] == own["loss"] and all(np.array_equal(same["grads"][k], own["grads"][k]) for k in theta)
    assert np.array_equal(np.take_along_axis(own["last_act"], own["pool_idx"][:, :, None].astype(np.int64), axis=2)[:, :, 0],
                          own["pooled"])
    pair = opn.forward_backward(spec, theta, pts, lab, mask, idx_given=(own["pool_idx"], own["pooled"]))
    assert pair["loss"] == own["loss"] and all(np.array_equal(pair["grads"][k], own["grads"][k]) for k in theta)
    other = (own["pool_idx"] + 1) % spec.L
    out = opn.forward_backward(spec, theta, pts, lab, mask, idx_given=other)
    assert np.array_equal(out["pool_idx"], own["pool_idx"])          # the oracle's own argmax is still reported
    tp = {k: T(v).requires_grad_() for k, v in theta.items()}
    loss, _ = torch_model_loss(spec, tp, pts, lab, mask, pool_at=other)
    loss.backward()
    assert abs(out["loss"] - loss.item()) < 1e-12
    for k in theta:
        g = tp[k].grad.numpy()
        assert np.abs(out["grads"][k] - g).max() <= 1e-10 * max(np.abs(g).max(), 1e-3), k
