"""Pins for the oracle of the PointNet-cls model with input / feature transform sub-networks
(no GPU needed): the same network built from torch's CPU float64 operators (conv1d, batch_norm,
max, matmul, bmm) and differentiated by autograd; special cases that have a closed form."""
import dataclasses

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import hfta_inputs as hi
from oracle import pointnet as opn
from oracle import pointnet_t as opt

T = lambda a: torch.tensor(np.asarray(a, np.float64), dtype=torch.float64)


def tiny(input_transform=True, feature_transform=True):
    cls = hi.PointNetClsSpec(name="tiny_t", B=2, Nb=4, L=9, conv=(3, 5, 7), fc=(7, 6, 4), fc_bn=True, dropout_p=0.3,
                             dtype="f64", n_classes=4, config_index=0)
    return hi.PointNetTSpec(cls=cls, tnet_conv=(4, 6), tnet_fc=(5,), input_transform=input_transform,
                            feature_transform=feature_transform)


def bn(x, g, b):
    return F.batch_norm(x, None, None, g, b, training=True, eps=1e-5)


def torch_tnet(ts, tp, k, x):
    a = x
    for i in range(len(ts.tnet_conv)):
        a = F.relu(bn(F.conv1d(a, tp[f"t{k}.conv{i}.w"][:, :, None], tp[f"t{k}.conv{i}.b"]),
                      tp[f"t{k}.conv{i}.bn.g"], tp[f"t{k}.conv{i}.bn.b"]))
    h = a.max(dim=2).values
    n = len(ts.tnet_fc)
    for i in range(n):
        h = F.relu(bn(h @ tp[f"t{k}.fc{i}.w"] + tp[f"t{k}.fc{i}.b"], tp[f"t{k}.fc{i}.bn.g"], tp[f"t{k}.fc{i}.bn.b"]))
    h = h @ tp[f"t{k}.fc{n}.w"] + tp[f"t{k}.fc{n}.b"]
    Tm = (h + torch.eye(k, dtype=torch.float64).reshape(1, k * k)).reshape(-1, k, k)
    return torch.bmm(Tm, x), Tm                              # y[n] = T[n] x[n]


def torch_loss(ts, tp, points, labels, mask):
    s = ts.cls
    x = T(points)
    if ts.input_transform:
        x, _ = torch_tnet(ts, tp, 3, x)
    a = x
    for i in range(len(s.conv) - 1):
        a = F.relu(bn(F.conv1d(a, tp[f"conv{i}.w"][:, :, None], tp[f"conv{i}.b"]), tp[f"conv{i}.bn.g"], tp[f"conv{i}.bn.b"]))
        if i == 0 and ts.feature_transform:
            a, _ = torch_tnet(ts, tp, s.conv[1], a)
    h = a.max(dim=2).values
    nfc = len(s.fc) - 1
    for i in range(nfc):
        h = h @ tp[f"fc{i}.w"] + tp[f"fc{i}.b"]
        if i < nfc - 1:
            h = F.relu(bn(h, tp[f"fc{i}.bn.g"], tp[f"fc{i}.bn.b"]))
            if i == nfc - 2 and s.dropout_p > 0:
                h = h * T(mask) / (1 - s.dropout_p)
    return F.cross_entropy(h, torch.tensor(np.asarray(labels, np.int64))), h


@pytest.mark.parametrize("it,ft", [(True, True), (True, False), (False, True)])
def test_forward_backward_vs_autograd(it, ft):
    ts = tiny(it, ft)
    inp = hi.pointnet_t_inputs(ts, seed=11)
    names = [n for n, _ in hi.pointnet_t_param_shapes(ts)]
    assert set(names) == set(inp["params"][0])
    for b in range(ts.cls.B):
        theta = {k: v.astype(np.float64) + 0.05 * np.random.default_rng(b).standard_normal(v.shape)
                 for k, v in inp["params"][b].items()}
        pts, mask = inp["points"][:, 3 * b:3 * b + 3, :], inp["drop_mask"][b]
        out = opt.forward_backward(ts, theta, pts, inp["labels"][b], mask)
        tp = {k: T(v).requires_grad_() for k, v in theta.items()}
        loss, logits = torch_loss(ts, tp, pts, inp["labels"][b], mask)
        loss.backward()
        assert abs(out["loss"] - loss.item()) < 1e-12
        np.testing.assert_allclose(out["logits"], logits.detach().numpy(), rtol=0, atol=1e-11)
        assert set(out["grads"]) == set(theta)
        for k in theta:
            g = tp[k].grad.numpy()
            assert np.abs(out["grads"][k] - g).max() <= 1e-9 * max(np.abs(g).max(), 1e-3), k


def test_identity_transform_is_the_plain_model():
    """With the last Linear of each sub-network zero the matrices are the identity: loss, logits and
    the gradients of the main network equal the model without sub-networks; the sub-networks still
    receive gradients (through their last Linear's weights only where its input is nonzero)."""
    ts = tiny()
    inp = hi.pointnet_t_inputs(ts, seed=12)
    theta = {k: v.astype(np.float64) for k, v in inp["params"][0].items()}
    n = len(ts.tnet_fc)
    for k in (3, ts.cls.conv[1]):
        theta[f"t{k}.fc{n}.w"][:] = 0
        theta[f"t{k}.fc{n}.b"][:] = 0
    pts, lab, mask = inp["points"][:, 0:3, :], inp["labels"][0], inp["drop_mask"][0]
    out = opt.forward_backward(ts, theta, pts, lab, mask)
    plain = opn.forward_backward(ts.cls, {k: v for k, v in theta.items() if not k.startswith("t")}, pts, lab, mask)
    assert np.array_equal(out["T3"], np.broadcast_to(np.eye(3), out["T3"].shape))
    assert abs(out["loss"] - plain["loss"]) < 1e-13
    for k, g in plain["grads"].items():
        assert np.abs(out["grads"][k] - g).max() <= 1e-11 * max(np.abs(g).max(), 1e-3), k
    # dL/dT3[n] = sum_l dx'[n,:,l] x[n,:,l]^T reaches the last bias unchanged
    assert np.abs(out["grads"][f"t3.fc{n}.b"]).max() > 0


def test_storage_rounding_and_train_step():
    """bf16 storage: the transformed points and the matrices are stored values; a training step
    updates every parameter of every sub-network."""
    ts = dataclasses.replace(tiny(), cls=dataclasses.replace(tiny().cls, dtype="bf16"))
    inp = hi.pointnet_t_inputs(ts, seed=13)
    states = [opn.init_state(p) for p in inp["params"]]
    before = [{k: v.copy() for k, v in st["theta"].items()} for st in states]
    outs = opt.array_train_step(ts, states, inp, 1)
    for b, o in enumerate(outs):
        assert np.array_equal(o["T3"], hi.snap(o["T3"], "bf16"))
        moved = [k for k in before[b] if not np.array_equal(before[b][k], states[b]["theta"][k])]
        assert len(moved) >= len(before[b]) - 8, sorted(set(before[b]) - set(moved))   # biases in front of a BatchNorm stay
        assert any(k.startswith("t3.") for k in moved) and any(k.startswith("t5.") for k in moved)
        assert set(o["running"]) == {k[:-2] + s for k in before[b] if k.endswith(".bn.g") for s in (".rm", ".rv")}


def test_given_matrices():
    """Handing the oracle its own stored matrices changes nothing; handing it other matrices gives
    the model whose transform output is that matrix (here: the identity = no transform): same loss,
    same gradients downstream of the feature transform (the first layer still receives the gradient
    that flows back through the sub-network)."""
    ts = tiny()
    inp = hi.pointnet_t_inputs(ts, seed=14)
    theta = {k: v.astype(np.float64) for k, v in inp["params"][0].items()}
    pts, lab, mask = inp["points"][:, 0:3, :], inp["labels"][0], inp["drop_mask"][0]
    own = opt.forward_backward(ts, theta, pts, lab, mask)
    same = opt.forward_backward(ts, theta, pts, lab, mask, T_given={3: own["T3"], ts.cls.conv[1]: own["T64"]})
    assert same["loss"] == own["loss"] and all(np.array_equal(same["grads"][k], own["grads"][k]) for k in theta)
    Nb, k2 = ts.cls.Nb, ts.cls.conv[1]
    eye = {3: np.broadcast_to(np.eye(3), (Nb, 3, 3)), k2: np.broadcast_to(np.eye(k2), (Nb, k2, k2))}
    ident = opt.forward_backward(ts, theta, pts, lab, mask, T_given=eye)
    plain = opn.forward_backward(ts.cls, {k: v for k, v in theta.items() if not k.startswith("t")}, pts, lab, mask)
    assert abs(ident["loss"] - plain["loss"]) < 1e-13
    for k, g in plain["grads"].items():
        if not k.startswith("conv0."):
            assert np.abs(ident["grads"][k] - g).max() <= 1e-11 * max(np.abs(g).max(), 1e-3), k
    assert np.abs(ident["grads"]["conv0.w"] - plain["grads"]["conv0.w"]).max() > 1e-6
    assert np.array_equal(ident["T3"], own["T3"])          # the oracle's own matrices are still reported
