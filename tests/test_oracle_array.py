"""Pins for the oracle's fused-array level (no GPU needed).

The oracle runs B separate unfused loops.  The paper's fusion rules table says
those B operators equal ONE existing operator on concatenated tensors (grouped
convolution with G = B, baddbmm, BatchNorm over B*C channels, ...).  Here the
right-hand column is evaluated with torch's CPU float64 operators and autograd,
an implementation independent of the oracle, and the two must agree.  Also:
B = 1 reduces to the plain op, model i of the array equals model i alone,
models do not talk to each other, and the loss-scaling identities of the
appendix "Fused Loss" (eqs. 1-5) hold.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import array as oa
from oracle import ops

RNG = np.random.default_rng(99)
T = lambda a: torch.tensor(np.asarray(a, np.float64), dtype=torch.float64)


def rnd(*s):
    return RNG.standard_normal(s)


def close(a, b, tol=1e-11):
    a = a.detach().numpy() if isinstance(a, torch.Tensor) else np.asarray(a, np.float64)
    b = b.detach().numpy() if isinstance(b, torch.Tensor) else np.asarray(b, np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    assert np.abs(a - b).max() <= tol * max(np.abs(b).max(), 1e-30), np.abs(a - b).max()


def test_linear_is_baddbmm():
    B, M, Fx, Fy = 3, 5, 4, 6
    x, w, b, dy = rnd(B, M, Fx), rnd(B, Fx, Fy), rnd(B, Fy), rnd(B, M, Fy)
    tx, tw, tb = T(x).requires_grad_(), T(w).requires_grad_(), T(b).requires_grad_()
    ty = torch.baddbmm(tb[:, None, :], tx, tw)
    close(oa.linear_fwd(B, x, w, b), ty)
    ty.backward(T(dy))
    dx, dw, db = oa.linear_bwd(B, x, w, dy)
    close(dx, tx.grad); close(dw, tw.grad); close(db, tb.grad)


def test_conv1x1_is_grouped_conv1d():
    B, N, Ci, Co, L = 3, 2, 4, 5, 7
    x, w, b, dy = rnd(N, B * Ci, L), rnd(B * Co, Ci), rnd(B * Co), rnd(N, B * Co, L)
    tx, tw, tb = T(x).requires_grad_(), T(w).requires_grad_(), T(b).requires_grad_()
    ty = F.conv1d(tx, tw[:, :, None], tb, groups=B)
    close(oa.conv1x1_fwd(B, x, w, b), ty)
    ty.backward(T(dy))
    dx, dw, db = oa.conv1x1_bwd(B, x, w, dy)
    close(dx, tx.grad); close(dw, tw.grad); close(db, tb.grad)


@pytest.mark.parametrize("k,s,p,H", [(4, 2, 1, 8), (4, 1, 0, 4), (3, 1, 1, 5)])
def test_conv2d_is_grouped_conv2d(k, s, p, H):
    B, N, Ci, Co = 3, 2, 2, 3
    x, w, b = rnd(N, B * Ci, H, H), rnd(B * Co, Ci, k, k), rnd(B * Co)
    tx, tw, tb = T(x).requires_grad_(), T(w).requires_grad_(), T(b).requires_grad_()
    ty = F.conv2d(tx, tw, tb, stride=s, padding=p, groups=B)
    y = oa.conv2d_fwd(B, x, w, b, s, p)
    close(y, ty)
    dy = rnd(*y.shape)
    ty.backward(T(dy))
    dx, dw, db = oa.conv2d_bwd(B, x, w, dy, s, p)
    close(dx, tx.grad); close(dw, tw.grad); close(db, tb.grad)
    # groups = B is a dense convolution with block-diagonal weights
    wd = np.zeros((B * Co, B * Ci, k, k))
    for g in range(B):
        wd[g * Co:(g + 1) * Co, g * Ci:(g + 1) * Ci] = w[g * Co:(g + 1) * Co]
    close(y, ops.conv2d_fwd(x, wd, b, s, p))


@pytest.mark.parametrize("k,s,p,H", [(4, 2, 1, 4), (4, 1, 0, 1)])
def test_convT2d_is_grouped_convT2d(k, s, p, H):
    B, N, Cx, Cy = 3, 2, 3, 2
    x, w, b = rnd(N, B * Cx, H, H), rnd(B * Cx, Cy, k, k), rnd(B * Cy)
    tx, tw, tb = T(x).requires_grad_(), T(w).requires_grad_(), T(b).requires_grad_()
    ty = F.conv_transpose2d(tx, tw, tb, stride=s, padding=p, groups=B)
    y = oa.convT2d_fwd(B, x, w, b, s, p)
    close(y, ty)
    dy = rnd(*y.shape)
    ty.backward(T(dy))
    dx, dw, db = oa.convT2d_bwd(B, x, w, dy, s, p)
    close(dx, tx.grad); close(dw, tw.grad); close(db, tb.grad)


@pytest.mark.parametrize("layout", ["conv", "linear"])
def test_bn_is_batchnorm_over_BC_channels(layout):
    B, N, C, L = 3, 4, 5, 6
    eps, mom = 1e-5, 0.1
    g, bt = rnd(B * C), rnd(B * C)
    rm, rv = rnd(B * C), RNG.random(B * C) + 0.5
    if layout == "conv":
        x = rnd(N, B * C, L) * 2 + 0.3
        tx = T(x).requires_grad_()
        txc = tx
    else:
        x = rnd(B, N, C) * 2 + 0.3
        tx = T(x).requires_grad_()
        txc = tx.permute(1, 0, 2).reshape(N, B * C)       # the table's [N, B, C] view
    tg, tb = T(g).requires_grad_(), T(bt).requires_grad_()
    trm, trv = T(rm).clone(), T(rv).clone()
    ty = F.batch_norm(txc, trm, trv, tg, tb, training=True, momentum=mom, eps=eps)
    y, mean, invstd, nrm, nrv = oa.bn_fwd(B, x, g, bt, eps, mom, rm, rv, layout)
    tyl = ty if layout == "conv" else ty.reshape(N, B, C).permute(1, 0, 2)
    close(y, tyl); close(nrm, trm); close(nrv, trv)
    dy = rnd(*x.shape)
    tyl.backward(T(dy))
    dx, dg, dbt = oa.bn_bwd(B, x, dy, g, mean, invstd, layout)
    close(dx, tx.grad, 1e-10); close(dg, tg.grad, 1e-10); close(dbt, tb.grad, 1e-10)


def test_layernorm_rule():
    B, R, E = 3, 4, 6
    x, w, b, dy = rnd(B, R, E), rnd(B, E), rnd(B, E), rnd(B, R, E)
    tx, tw, tb = T(x).requires_grad_(), T(w).requires_grad_(), T(b).requires_grad_()
    ty = F.layer_norm(tx, (E,), eps=1e-5) * tw[:, None, :] + tb[:, None, :]
    y, mean, invstd = oa.layernorm_fwd(B, x, w, b, 1e-5)
    close(y, ty)
    ty.backward(T(dy))
    dx, dw, db = oa.layernorm_bwd(B, x, dy, w, mean, invstd)
    close(dx, tx.grad, 1e-10); close(dw, tw.grad); close(db, tb.grad)


def test_maxpool_points_vs_torch():
    B, N, C, L = 2, 3, 4, 11
    x = rnd(N, B * C, L)
    x[0, 0, :] = 0.0               # tie row
    v, idx = oa.maxpool_points_fwd(B, x)
    tv, ti = F.max_pool1d(T(x), L, return_indices=True)
    assert np.array_equal(v, tv[:, :, 0].numpy())
    assert idx[0, 0] == 0
    m = np.ones(idx.shape, bool); m[0, 0] = False
    assert np.array_equal(idx[m], ti[:, :, 0].numpy()[m])
    dv = rnd(N, B * C)
    dx = oa.maxpool_points_bwd(B, dv, idx, L)
    assert np.array_equal(dx.sum(axis=2), dv)
    assert np.count_nonzero(dx) == dv.size


def test_losses_vs_torch():
    B, R, K = 3, 5, 7
    z, lab = rnd(B, R, K), RNG.integers(0, K, (B, R))
    tz = T(z).requires_grad_()
    per = torch.stack([F.cross_entropy(tz[b], torch.tensor(lab[b])) for b in range(B)])
    loss, dz = oa.softmax_xent(B, z, lab)
    close(loss, per)
    per.sum().backward()
    close(dz, tz.grad)
    t = RNG.integers(0, 2, (B, R, 1)).astype(float)
    zz = rnd(B, R, 1)
    tzz = T(zz).requires_grad_()
    per = torch.stack([F.binary_cross_entropy_with_logits(tzz[b], T(t[b])) for b in range(B)])
    loss, dzz = oa.bce_logits(B, zz, t)
    close(loss, per)
    per.sum().backward()
    close(dzz, tzz.grad)


def test_adam_vs_torch_optim():
    B, P, steps = 3, 17, 4
    th0 = rnd(B, P).astype(np.float32)
    lr = np.array([1e-3, 3e-3, 1e-2]); b1 = np.array([0.8, 0.9, 0.95]); b2 = np.array([0.99, 0.999, 0.9])
    eps = np.array([1e-8, 1e-6, 1e-8]); wd = np.array([0.0, 0.1, 0.3])
    grads = [rnd(B, P) for _ in range(steps)]
    for decoupled in (False, True):
        th, m, v = th0.copy(), np.zeros((B, P), np.float32), np.zeros((B, P), np.float32)
        tparams = [T(th0[b]).requires_grad_() for b in range(B)]
        Opt = torch.optim.AdamW if decoupled else torch.optim.Adam
        opts = [Opt([tparams[b]], lr=lr[b], betas=(b1[b], b2[b]), eps=eps[b], weight_decay=wd[b])
                for b in range(B)]
        for t in range(1, steps + 1):
            th, m, v = oa.adam_step(B, th, grads[t - 1], m, v, lr, b1, b2, eps, wd, t, decoupled)
            for b in range(B):
                tparams[b].grad = T(grads[t - 1][b])
                opts[b].step()
        for b in range(B):
            # the oracle stores its state in float32 between steps
            close(th[b], tparams[b], 1e-6)


def test_adam_routes_hyperparameters_per_model():
    B, P = 3, 9
    th0, g = rnd(B, P).astype(np.float32), rnd(B, P)
    z = np.zeros((B, P), np.float32)
    lr = np.array([1e-2, 0.0, 1e-3])
    hp = dict(beta1=np.full(B, 0.9), beta2=np.full(B, 0.999), eps=np.full(B, 1e-8), wd=np.zeros(B))
    th, _, _ = oa.adam_step(B, th0, g, z, z, lr, hp["beta1"], hp["beta2"], hp["eps"], hp["wd"], 1)
    assert np.array_equal(th[1], th0[1])
    assert np.all(th[0] != th0[0]) and np.all(th[2] != th0[2])
    # step 1 moves every element by lr_b (up to eps): |delta_0| / |delta_2| = lr_0 / lr_2
    np.testing.assert_allclose(np.abs(th[0] - th0[0]) / np.abs(th[2] - th0[2]), 10.0, rtol=1e-3)


def test_B1_and_independence():
    B, N, Ci, Co, L = 3, 2, 3, 4, 5
    x, w, b = rnd(N, B * Ci, L), rnd(B * Co, Ci), rnd(B * Co)
    y = oa.conv1x1_fwd(B, x, w, b)
    for i in range(B):
        # model i of the array == model i alone (B = 1 call == the plain operator)
        alone = oa.conv1x1_fwd(1, x[:, i * Ci:(i + 1) * Ci], w[i * Co:(i + 1) * Co], b[i * Co:(i + 1) * Co])
        assert np.array_equal(alone, y[:, i * Co:(i + 1) * Co])
        assert np.array_equal(alone, ops.conv1x1_fwd(x[:, i * Ci:(i + 1) * Ci], w[i * Co:(i + 1) * Co],
                                                     b[i * Co:(i + 1) * Co]))
    # perturbing model 2 leaves models 0 and 1 bit-identical
    x2 = x.copy(); x2[:, 2 * Ci:] += 1.0
    y2 = oa.conv1x1_fwd(B, x2, w, b)
    assert np.array_equal(y2[:, :2 * Co], y[:, :2 * Co]) and not np.array_equal(y2[:, 2 * Co:], y[:, 2 * Co:])
    # permuting the models permutes the results
    perm = [2, 0, 1]
    xp = np.concatenate([x[:, i * Ci:(i + 1) * Ci] for i in perm], axis=1)
    wp = np.concatenate([w[i * Co:(i + 1) * Co] for i in perm]); bp = np.concatenate([b[i * Co:(i + 1) * Co] for i in perm])
    yp = oa.conv1x1_fwd(B, xp, wp, bp)
    assert np.array_equal(yp, np.concatenate([y[:, i * Co:(i + 1) * Co] for i in perm], axis=1))


def test_loss_scaling_identities():
    """Appendix "Fused Loss": with mean reduction over the array,
    grad_theta_b l_b = B * grad_theta_b L (eq. 3); with sum reduction no factor (eq. 5);
    the sums run over the B models."""
    B, M, Fx, K = 4, 6, 5, 3
    x, w, b = rnd(B, M, Fx), rnd(B, Fx, K), rnd(B, K)
    lab = RNG.integers(0, K, (B, M))
    # per-model gradients from the oracle (each loss is the model's own mean)
    logits = oa.linear_fwd(B, x, w, b)
    loss, dlogits = oa.softmax_xent(B, logits, lab)
    _, dw, _ = oa.linear_bwd(B, x, w, dlogits)
    # one backward pass through the fused scalar, by autograd
    tw = T(w).requires_grad_()
    tl = torch.baddbmm(T(b)[:, None, :], T(x), tw)
    per = torch.stack([F.cross_entropy(tl[i], torch.tensor(lab[i])) for i in range(B)])
    close(loss, per)
    (g_mean,) = torch.autograd.grad(per.mean(), tw, retain_graph=True)
    (g_scaled,) = torch.autograd.grad(B * per.mean(), tw, retain_graph=True)
    (g_sum,) = torch.autograd.grad(per.sum(), tw)
    close(dw, B * g_mean.numpy())
    close(dw, g_scaled)
    close(dw, g_sum)
    # cross gradients vanish: model 0's loss does not move model 1's weights
    (g0,) = torch.autograd.grad(F.cross_entropy(
        torch.baddbmm(T(b)[:, None, :], T(x), tw)[0], torch.tensor(lab[0])), tw)
    assert np.all(g0[1:].numpy() == 0)
