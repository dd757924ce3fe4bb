"""Pins for the segmentation-style oracle step (no GPU needed): the same network written with
torch's CPU float64 operators as ONE 4944-style convolution over an explicit concatenation
(torch.cat + expand) and differentiated by autograd; the identity that lets an implementation
split the first head weight into a per-point block and a once-per-sample block; Adam against torch.optim;
independence of the models of an array."""
import dataclasses

import numpy as np
import torch
import torch.nn.functional as F

import hfta_inputs as hi
from oracle import pointnet_seg as ops_seg

T = lambda a: torch.tensor(np.asarray(a, np.float64), dtype=torch.float64)


def tiny_spec(B=2):
    conv = (3, 4, 6, 5)
    return hi.PointNetSegSpec(name="tiny_seg", B=B, Nb=3, L=7, conv=conv, head=(sum(conv[1:]) + conv[-1] + 3, 6, 5, 4),
                              dtype="f64", n_cat=3, n_parts=4)


def torch_loss(spec, tp, points, labels, onehot):
    a = T(points)
    feats = []
    for i in range(len(spec.conv) - 1):
        z = F.conv1d(a, tp[f"conv{i}.w"][:, :, None], tp[f"conv{i}.b"])
        a = F.relu(F.batch_norm(z, None, None, tp[f"conv{i}.bn.g"], tp[f"conv{i}.bn.b"], training=True, eps=1e-5))
        feats.append(a)
    L = a.shape[2]
    g = a.max(dim=2).values
    cat = torch.cat(feats + [g[:, :, None].expand(-1, -1, L), T(onehot)[:, :, None].expand(-1, -1, L)], dim=1)
    nh = len(spec.head) - 1
    h = cat
    for i in range(nh):
        w = tp[f"head{i}.w"]                 # head0.w: [Co, c_point + c_global], one convolution
        h = F.conv1d(h, w[:, :, None], tp[f"head{i}.b"])
        if i < nh - 1:
            h = F.relu(F.batch_norm(h, None, None, tp[f"head{i}.bn.g"], tp[f"head{i}.bn.b"], training=True, eps=1e-5))
    return F.cross_entropy(h, torch.tensor(np.asarray(labels, np.int64))), h


def test_forward_backward_vs_autograd():
    spec = tiny_spec()
    inp = hi.pointnet_seg_inputs(spec, seed=11)
    assert spec.head[0] == spec.c_point + spec.c_global
    for b in range(spec.B):
        theta = {k: v.astype(np.float64) + 0.05 * np.random.default_rng(b).standard_normal(v.shape)
                 for k, v in inp["params"][b].items()}
        pts = inp["points"][:, 3 * b:3 * b + 3, :]
        out = ops_seg.forward_backward(spec, theta, pts, inp["labels"][b], inp["onehot"][b])
        tp = {k: T(v).requires_grad_() for k, v in theta.items()}
        loss, logits = torch_loss(spec, tp, pts, inp["labels"][b], inp["onehot"][b])
        loss.backward()
        assert abs(out["loss"] - loss.item()) < 1e-12
        np.testing.assert_allclose(out["logits"], logits.detach().numpy(), rtol=0, atol=1e-12)
        for k in theta:
            g = tp[k].grad.numpy()
            assert np.abs(out["grads"][k] - g).max() <= 1e-10 * max(np.abs(g).max(), 1e-3), k


def test_train_step_vs_torch_adam_and_independence():
    spec = tiny_spec(B=3)
    inp = hi.pointnet_seg_inputs(spec, seed=12)
    states = [ops_seg.init_state(inp["params"][b]) for b in range(spec.B)]
    tps = [{k: T(v).requires_grad_() for k, v in inp["params"][b].items()} for b in range(spec.B)]
    opts = [torch.optim.Adam(list(tps[b].values()), lr=float(inp["lr"][b]), betas=(0.9, 0.999), eps=1e-8) for b in range(spec.B)]
    for t in (1, 2):
        ops_seg.array_train_step(spec, states, inp, t)
        for b in range(spec.B):
            opts[b].zero_grad()
            loss, _ = torch_loss(spec, tps[b], inp["points"][:, 3 * b:3 * b + 3, :], inp["labels"][b], inp["onehot"][b])
            loss.backward()
            opts[b].step()
            for k, v in tps[b].items():
                ref = v.detach().numpy()
                # parameters are kept as float32 between steps by the oracle
                assert np.abs(states[b]["theta"][k] - ref).max() <= 2e-6 * max(np.abs(ref).max(), 1e-3), (t, b, k)
    # model 1 of the array equals that model trained alone
    s1 = dataclasses.replace(spec, B=1)
    i1 = {k: (v[1:2] if isinstance(v, np.ndarray) and v.shape[:1] == (spec.B,) else v) for k, v in inp.items()}
    i1["points"] = inp["points"][:, 3:6, :]
    i1["params"] = [inp["params"][1]]
    alone = [ops_seg.init_state(inp["params"][1])]
    for t in (1, 2):
        ops_seg.array_train_step(s1, alone, i1, t)
    for k in alone[0]["theta"]:
        assert np.array_equal(alone[0]["theta"][k], states[1]["theta"][k]), k


def test_inputs_recipe():
    spec = hi.spec_c2()
    assert spec.head[0] == 4944 and spec.c_point == 2880 and spec.c_global == 2064
    thin = hi.seg_thin(2, 2, 40, "bf16")
    inp = hi.pointnet_seg_inputs(thin)
    assert inp["points"].shape == (2, 6, 40) and inp["labels"].shape == (2, 2, 40) and inp["labels"].max() < 50
    assert np.all(np.linalg.norm(inp["points"][:, :3, :].astype(np.float64), axis=1) <= 1.0 + 1e-2)
    assert np.array_equal(inp["onehot"].sum(axis=2), np.ones((2, 2)))
    shapes = dict(hi.pointnet_seg_param_shapes(thin))
    assert shapes["head0.w"] == (thin.head[1], thin.c_point + thin.c_global) and "head0.wg" not in shapes


def test_split_first_head_layer_identity():
    """A k=1 convolution over [per-point maps | tiled vector] equals the convolution of the per-point
    block plus the tiled block's product taken once per sample and broadcast along the points, and its
    adjoint hands the tiled part the point-sum of the output gradient: the decomposition the device
    uses, checked here on the oracle's own operators in float64."""
    from oracle import ops
    rng = np.random.default_rng(3)
    Nb, Cp, Cg, Co, L = 3, 5, 4, 6, 7
    xp, t = rng.standard_normal((Nb, Cp, L)), rng.standard_normal((Nb, Cg))
    w, b, dy = rng.standard_normal((Co, Cp + Cg)), rng.standard_normal(Co), rng.standard_normal((Nb, Co, L))
    cat = np.concatenate([xp, np.broadcast_to(t[:, :, None], (Nb, Cg, L))], axis=1)
    y = ops.conv1x1_fwd(cat, w, b)
    hg = ops.linear_fwd(t, w[:, Cp:].T.copy(), None)
    np.testing.assert_allclose(ops.add_sample_bias(ops.conv1x1_fwd(xp, w[:, :Cp].copy(), b), hg), y, rtol=0, atol=1e-12)
    dx, dw, _ = ops.conv1x1_bwd(cat, w, dy)
    dxp, dwp, _ = ops.conv1x1_bwd(xp, w[:, :Cp].copy(), dy)
    dt, dwg, _ = ops.linear_bwd(t, w[:, Cp:].T.copy(), ops.sum_points(dy))
    np.testing.assert_allclose(dxp, dx[:, :Cp], rtol=0, atol=1e-12)
    np.testing.assert_allclose(dt, dx[:, Cp:].sum(axis=2), rtol=0, atol=1e-12)
    np.testing.assert_allclose(np.concatenate([dwp, dwg.T], axis=1), dw, rtol=0, atol=1e-12)
