"""Pins for the CPU oracle's single-model operators (no GPU needed).

Each pin is something other than the oracle itself: brute-force Python loops on
tiny inputs, central finite differences, adjoint identities, closed forms and
invariants.  They are chosen so that a dropped term, a wrong sign or index, or
a transposed operand fails at least one of them.
"""
import math

import numpy as np
import pytest

from oracle import ops

RNG = np.random.default_rng(1234)


def rnd(*shape):
    return RNG.standard_normal(shape)


def fd_grad(f, x, h=1e-6):
    """Central finite-difference gradient of scalar f at x (float64)."""
    x = np.array(x, dtype=np.float64)
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    while not it.finished:
        i = it.multi_index
        old = x[i]
        x[i] = old + h
        fp = f(x)
        x[i] = old - h
        fm = f(x)
        x[i] = old
        g[i] = (fp - fm) / (2 * h)
        it.iternext()
    return g


def close(a, b, tol=1e-6):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    scale = max(np.abs(b).max(), 1e-30)
    assert a.shape == b.shape
    assert np.abs(a - b).max() <= tol * scale, (np.abs(a - b).max(), scale)


# ------------------------------------------------------------------ linear
def test_linear_bruteforce_and_orientation():
    M, Fx, Fy = 3, 4, 5
    x, w, b = rnd(M, Fx), rnd(Fx, Fy), rnd(Fy)
    y = ops.linear_fwd(x, w, b)
    ref = np.zeros((M, Fy))
    for r in range(M):
        for j in range(Fy):
            s = b[j]
            for k in range(Fx):
                s += x[r, k] * w[k, j]
            ref[r, j] = s
    close(y, ref, 1e-13)
    # identity weights return x + bias
    close(ops.linear_fwd(x, np.eye(Fx), np.arange(Fx)), x + np.arange(Fx), 1e-15)


def test_linear_bwd_fd():
    M, Fx, Fy = 3, 4, 5
    x, w, b, c = rnd(M, Fx), rnd(Fx, Fy), rnd(Fy), rnd(M, Fy)
    dx, dw, db = ops.linear_bwd(x, w, c)
    close(dx, fd_grad(lambda t: (ops.linear_fwd(t, w, b) * c).sum(), x))
    close(dw, fd_grad(lambda t: (ops.linear_fwd(x, t, b) * c).sum(), w))
    close(db, fd_grad(lambda t: (ops.linear_fwd(x, w, t) * c).sum(), b))


# ------------------------------------------------------------------ conv1x1
def test_conv1x1_bruteforce_and_linear_special_case():
    N, Ci, Co, L = 2, 3, 4, 5
    x, w, b = rnd(N, Ci, L), rnd(Co, Ci), rnd(Co)
    y = ops.conv1x1_fwd(x, w, b)
    ref = np.zeros((N, Co, L))
    for n in range(N):
        for o in range(Co):
            for l in range(L):
                ref[n, o, l] = b[o] + sum(w[o, c] * x[n, c, l] for c in range(Ci))
    close(y, ref, 1e-13)
    # L = 1 reduces to Linear with the weight transposed
    x1 = rnd(N, Ci, 1)
    close(ops.conv1x1_fwd(x1, w, b)[:, :, 0], ops.linear_fwd(x1[:, :, 0], w.T, b), 1e-13)


def test_conv1x1_bwd_fd():
    N, Ci, Co, L = 2, 3, 4, 5
    x, w, b, c = rnd(N, Ci, L), rnd(Co, Ci), rnd(Co), rnd(N, Co, L)
    dx, dw, db = ops.conv1x1_bwd(x, w, c)
    close(dx, fd_grad(lambda t: (ops.conv1x1_fwd(t, w, b) * c).sum(), x))
    close(dw, fd_grad(lambda t: (ops.conv1x1_fwd(x, t, b) * c).sum(), w))
    close(db, fd_grad(lambda t: (ops.conv1x1_fwd(x, w, t) * c).sum(), b))


# ------------------------------------------------------------------ conv2d
def conv2d_loops(x, w, b, s, p):
    N, Ci, H, W = x.shape
    Co, _, kh, kw = w.shape
    Ho, Wo = (H + 2 * p - kh) // s + 1, (W + 2 * p - kw) // s + 1
    y = np.zeros((N, Co, Ho, Wo))
    for n in range(N):
        for o in range(Co):
            for i in range(Ho):
                for j in range(Wo):
                    acc = b[o]
                    for c in range(Ci):
                        for ky in range(kh):
                            for kx in range(kw):
                                yy, xx = s * i + ky - p, s * j + kx - p
                                if 0 <= yy < H and 0 <= xx < W:
                                    acc += w[o, c, ky, kx] * x[n, c, yy, xx]
                    y[n, o, i, j] = acc
    return y


@pytest.mark.parametrize("k,s,p,H", [(4, 2, 1, 6), (4, 1, 0, 4), (3, 1, 1, 5), (1, 1, 0, 3), (4, 2, 1, 8)])
def test_conv2d_bruteforce(k, s, p, H):
    N, Ci, Co = 2, 2, 3
    x, w, b = rnd(N, Ci, H, H + 1), rnd(Co, Ci, k, k), rnd(Co)
    close(ops.conv2d_fwd(x, w, b, s, p), conv2d_loops(x, w, b, s, p), 1e-13)


def test_conv2d_special_cases():
    N, Ci, Co, H = 2, 3, 2, 5
    x = rnd(N, Ci, H, H)
    # k = 1 on the flattened image is the k=1 Conv1d
    w1, b = rnd(Co, Ci), rnd(Co)
    close(ops.conv2d_fwd(x, w1[:, :, None, None], b).reshape(N, Co, H * H),
          ops.conv1x1_fwd(x.reshape(N, Ci, H * H), w1, b), 1e-13)
    # all-ones 3x3 kernel, pad 1: box sum over all channels
    y = ops.conv2d_fwd(x, np.ones((1, Ci, 3, 3)), None, 1, 1)
    xp = np.pad(x.sum(axis=1), ((0, 0), (1, 1), (1, 1)))
    box = sum(xp[:, a:a + H, c:c + H] for a in range(3) for c in range(3))
    close(y[:, 0], box, 1e-13)
    # shift equivariance away from the borders (stride 1, no pad)
    w = rnd(Co, Ci, 3, 3)
    y0 = ops.conv2d_fwd(x, w)
    xs = np.roll(x, 1, axis=3)
    ys = ops.conv2d_fwd(xs, w)
    close(ys[:, :, :, 1:], y0[:, :, :, :-1], 1e-13)


@pytest.mark.parametrize("k,s,p,H", [(4, 2, 1, 6), (4, 1, 0, 4), (3, 2, 0, 7)])
def test_conv2d_bwd_fd_and_adjoint(k, s, p, H):
    N, Ci, Co = 2, 2, 3
    x, w, b = rnd(N, Ci, H, H), rnd(Co, Ci, k, k), rnd(Co)
    y = ops.conv2d_fwd(x, w, b, s, p)
    c = rnd(*y.shape)
    dx, dw, db = ops.conv2d_bwd(x, w, c, s, p)
    close(dx, fd_grad(lambda t: (ops.conv2d_fwd(t, w, b, s, p) * c).sum(), x))
    close(dw, fd_grad(lambda t: (ops.conv2d_fwd(x, t, b, s, p) * c).sum(), w))
    close(db, fd_grad(lambda t: (ops.conv2d_fwd(x, w, t, s, p) * c).sum(), b))
    # <conv(x), c> == <x, conv^T(c)>
    lhs = (ops.conv2d_fwd(x, w, None, s, p) * c).sum()
    assert abs(lhs - (x * dx).sum()) <= 1e-11 * abs(lhs)


def convT2d_loops(x, w, b, s, p):
    N, Cx, H, W = x.shape
    _, Cy, kh, kw = w.shape
    Ho, Wo = (H - 1) * s - 2 * p + kh, (W - 1) * s - 2 * p + kw
    y = np.zeros((N, Cy, Ho, Wo)) + b[None, :, None, None]
    for n in range(N):
        for c in range(Cx):
            for i in range(H):
                for j in range(W):
                    for o in range(Cy):
                        for ky in range(kh):
                            for kx in range(kw):
                                yy, xx = s * i + ky - p, s * j + kx - p
                                if 0 <= yy < Ho and 0 <= xx < Wo:
                                    y[n, o, yy, xx] += x[n, c, i, j] * w[c, o, ky, kx]
    return y


@pytest.mark.parametrize("k,s,p,H", [(4, 2, 1, 3), (4, 1, 0, 1), (3, 2, 0, 3)])
def test_convT2d_bruteforce_adjoint_fd(k, s, p, H):
    N, Cx, Cy = 2, 3, 2
    x, w, b = rnd(N, Cx, H, H), rnd(Cx, Cy, k, k), rnd(Cy)
    y = ops.convT2d_fwd(x, w, b, s, p)
    close(y, convT2d_loops(x, w, b, s, p), 1e-13)
    # ConvT is the adjoint of Conv2d w.r.t. its input, with the same weight tensor
    # read as [Co=Cx, Ci=Cy, kh, kw]:  <convT(x), u> == <x, conv(u)>
    u = rnd(*y.shape)
    lhs = (ops.convT2d_fwd(x, w, None, s, p) * u).sum()
    rhs = (x * ops.conv2d_fwd(u, w, None, s, p)).sum()
    assert abs(lhs - rhs) <= 1e-11 * max(abs(lhs), 1e-30)
    dx, dw, db = ops.convT2d_bwd(x, w, u, s, p)
    close(dx, fd_grad(lambda t: (ops.convT2d_fwd(t, w, b, s, p) * u).sum(), x))
    close(dw, fd_grad(lambda t: (ops.convT2d_fwd(x, t, b, s, p) * u).sum(), w))
    close(db, fd_grad(lambda t: (ops.convT2d_fwd(x, w, t, s, p) * u).sum(), b))


# ------------------------------------------------------------------ BatchNorm
def test_bn_fwd_invariants_and_closed_forms():
    N, C, L = 4, 3, 7
    x = rnd(N, C, L) * 3 + 1.5
    g, b = rnd(C), rnd(C)
    eps = 1e-3
    y, mean, invstd, rm, rv = ops.bn_fwd(x, g, b, eps, 0.1, np.zeros(C), np.ones(C))
    # per channel: mean(y) = beta, var_biased(y) = gamma^2 var / (var + eps)
    var = x.var(axis=(0, 2))
    close(y.mean(axis=(0, 2)), b, 1e-12)
    close(y.var(axis=(0, 2)), g * g * var / (var + eps), 1e-12)
    close(mean, x.mean(axis=(0, 2)), 1e-13)
    close(invstd, 1 / np.sqrt(var + eps), 1e-13)
    m = N * L
    close(rm, 0.1 * x.mean(axis=(0, 2)), 1e-13)
    close(rv, 0.9 + 0.1 * var * m / (m - 1), 1e-13)
    # constant input -> y = beta
    yc = ops.bn_fwd(np.full((N, C, L), 2.5), g, b, eps)[0]
    close(yc, np.broadcast_to(b[None, :, None], yc.shape), 1e-12)
    # hand-computed two-element channel: x = {1, 3}: mu = 2, var = 1
    y2 = ops.bn_fwd(np.array([[[1.0]], [[3.0]]]), np.array([2.0]), np.array([0.5]), 0.0)[0]
    close(y2[:, 0, 0], [0.5 - 2.0, 0.5 + 2.0], 1e-14)


def test_bn_bwd_fd_and_invariants():
    N, C, L = 3, 2, 4
    x, dy, g, b = rnd(N, C, L), rnd(N, C, L), rnd(C), rnd(C)
    eps = 1e-2
    _, mean, invstd, _, _ = ops.bn_fwd(x, g, b, eps)
    dx, dg, dbt = ops.bn_bwd(x, dy, g, mean, invstd)
    close(dx, fd_grad(lambda t: (ops.bn_fwd(t, g, b, eps)[0] * dy).sum(), x), 1e-6)
    close(dg, fd_grad(lambda t: (ops.bn_fwd(x, t, b, eps)[0] * dy).sum(), g))
    close(dbt, fd_grad(lambda t: (ops.bn_fwd(x, g, t, eps)[0] * dy).sum(), b))
    xhat = (x - mean[None, :, None]) * invstd[None, :, None]
    assert np.abs(dx.sum(axis=(0, 2))).max() < 1e-12
    # sum dx*xhat = gamma invstd dgamma (1 - sum xhat^2 / m) = gamma invstd dgamma eps invstd^2
    close((dx * xhat).sum(axis=(0, 2)), g * invstd * dg * eps * invstd ** 2, 1e-10)


# ------------------------------------------------------------------ LayerNorm
def test_layernorm_fwd_bwd():
    R, E = 3, 6
    x, w, b, dy = rnd(R, E) * 2 + 1, rnd(E), rnd(E), rnd(R, E)
    eps = 1e-3
    y, mean, invstd = ops.layernorm_fwd(x, w, b, eps)
    for r in range(R):
        mu = sum(x[r]) / E
        var = sum((x[r] - mu) ** 2) / E
        close(y[r], (x[r] - mu) / math.sqrt(var + eps) * w + b, 1e-13)
    dx, dw, db = ops.layernorm_bwd(x, dy, w, mean, invstd)
    close(dx, fd_grad(lambda t: (ops.layernorm_fwd(t, w, b, eps)[0] * dy).sum(), x))
    close(dw, fd_grad(lambda t: (ops.layernorm_fwd(x, t, b, eps)[0] * dy).sum(), w))
    close(db, fd_grad(lambda t: (ops.layernorm_fwd(x, w, t, eps)[0] * dy).sum(), b))


# ------------------------------------------------------------------ max-pool
def test_maxpool_bruteforce_ties_permutation():
    N, C, L = 3, 4, 9
    x = rnd(N, C, L)
    v, idx = ops.maxpool_points_fwd(x)
    for n in range(N):
        for c in range(C):
            best, bi = x[n, c, 0], 0
            for l in range(1, L):
                if x[n, c, l] > best:
                    best, bi = x[n, c, l], l
            assert v[n, c] == best and idx[n, c] == bi
    assert idx.dtype == np.int32
    # ties: all-equal and post-ReLU-zero rows return index 0; first of equal maxima wins
    z = np.zeros((1, 2, 5))
    z[0, 1] = [-1, 3, 3, 0, 3]
    v, idx = ops.maxpool_points_fwd(z)
    assert idx.tolist() == [[0, 1]] and v.tolist() == [[0.0, 3.0]]
    # permuting the point axis permutes indices and keeps values
    perm = RNG.permutation(L)
    v2, idx2 = ops.maxpool_points_fwd(x[:, :, perm])
    assert np.array_equal(v2, ops.maxpool_points_fwd(x)[0])
    assert np.array_equal(perm[idx2], ops.maxpool_points_fwd(x)[1])
    # backward is the exact scatter
    dv = rnd(N, C)
    dx = ops.maxpool_points_bwd(dv, idx2, L)
    assert np.count_nonzero(dx) == N * C
    close(dx, fd_grad(lambda t: (ops.maxpool_points_fwd(t)[0] * dv).sum(), x[:, :, perm]), 1e-6)


# ------------------------------------------------------------------ activations, dropout
@pytest.mark.parametrize("act", [ops.ACT_RELU, ops.ACT_LEAKY, ops.ACT_TANH, ops.ACT_GELU])
def test_activations(act):
    x = rnd(4, 5)
    x[np.abs(x) < 1e-3] = 0.5
    dy = rnd(4, 5)
    y = ops.act_fwd(x, act, 0.2)
    for i in range(4):
        for j in range(5):
            t = x[i, j]
            ref = {ops.ACT_RELU: max(t, 0.0), ops.ACT_LEAKY: t if t > 0 else 0.2 * t,
                   ops.ACT_TANH: math.tanh(t),
                   ops.ACT_GELU: t * 0.5 * math.erfc(-t / math.sqrt(2))}[act]
            assert abs(y[i, j] - ref) < 1e-14
    close(ops.act_bwd(x, dy, act, 0.2), fd_grad(lambda t: (ops.act_fwd(t, act, 0.2) * dy).sum(), x))
    # the kink belongs to the non-positive side
    z = np.zeros(1)
    assert ops.act_bwd(z, np.ones(1), ops.ACT_RELU)[0] == 0.0
    assert ops.act_bwd(z, np.ones(1), ops.ACT_LEAKY, 0.2)[0] == 0.2


def test_gelu_known_values():
    # Phi(0) = 1/2; Phi(1) = 0.8413447460685429 (standard normal table)
    close(ops.act_fwd(np.array([0.0, 1.0, -1.0]), ops.ACT_GELU),
          [0.0, 0.8413447460685429, -(1 - 0.8413447460685429)], 1e-14)


def test_dropout():
    x = rnd(3, 4)
    mask = (RNG.random((3, 4)) > 0.3).astype(np.uint8)
    y = ops.dropout_fwd(x, mask, 0.3)
    assert np.all(y[mask == 0] == 0)
    close(y[mask == 1], x[mask == 1] / 0.7, 1e-15)
    close(ops.dropout_bwd(x, mask, 0.3), y, 1e-15)


# ------------------------------------------------------------------ losses
def test_losses_closed_forms_and_fd():
    R, K = 4, 5
    z = rnd(R, K)
    lab = RNG.integers(0, K, R)
    loss, dz = ops.softmax_xent(z, lab)
    ref = np.mean([-math.log(math.exp(z[r, lab[r]]) / sum(math.exp(t) for t in z[r])) for r in range(R)])
    assert abs(loss - ref) < 1e-13
    close(dz, fd_grad(lambda t: ops.softmax_xent(t, lab)[0], z))
    # uniform logits: loss = log K
    assert abs(ops.softmax_xent(np.zeros((2, K)), [0, 1])[0] - math.log(K)) < 1e-14
    t = RNG.integers(0, 2, (R, 1)).astype(float)
    zz = rnd(R, 1)
    loss, dzz = ops.bce_logits(zz, t)
    sig = 1 / (1 + np.exp(-zz))
    assert abs(loss - (-(t * np.log(sig) + (1 - t) * np.log(1 - sig))).mean()) < 1e-13
    close(dzz, fd_grad(lambda q: ops.bce_logits(q, t)[0], zz))
    p, q = rnd(R, K), rnd(R, K)
    loss, dp = ops.mse(p, q)
    assert abs(loss - ((p - q) ** 2).sum() / (R * K)) < 1e-14
    close(dp, fd_grad(lambda u: ops.mse(u, q)[0], p))


# ------------------------------------------------------------------ Adam
def test_adam_closed_forms():
    P = 7
    th0, g = rnd(P), rnd(P)
    lr, eps = 3e-3, 1e-8
    # step 1 from zero moments: delta = -lr g / (|g| + eps)  (bias correction cancels)
    th, m, v = ops.adam_step(th0, g, np.zeros(P), np.zeros(P), lr, 0.9, 0.999, eps, 0.0, 1)
    close(th - th0, -lr * g / (np.abs(g) + eps), 1e-9)
    close(m, 0.1 * g, 1e-12)
    close(v, 0.001 * g * g, 1e-12)
    # constant gradient for t steps: theta_t = theta_0 - t lr g / (|g| + eps)
    th, m, v = th0.copy(), np.zeros(P), np.zeros(P)
    for t in range(1, 6):
        th, m, v = ops.adam_step(th, g, m, v, lr, 0.8, 0.95, eps, 0.0, t)
    close(th - th0, -5 * lr * g / (np.abs(g) + eps), 1e-9)
    # lr = 0 leaves the parameters untouched
    th, _, _ = ops.adam_step(th0, g, np.zeros(P), np.zeros(P), 0.0, 0.9, 0.999, eps, 0.1, 1)
    assert np.array_equal(th, th0)
    # L2 weight decay enters through the gradient; decoupled decay shrinks theta first
    wd = 0.3
    th_l2, m_l2, _ = ops.adam_step(th0, g, np.zeros(P), np.zeros(P), lr, 0.9, 0.999, eps, wd, 1)
    close(m_l2, 0.1 * (g + wd * th0), 1e-12)
    th_dw, m_dw, _ = ops.adam_step(th0, g, np.zeros(P), np.zeros(P), lr, 0.9, 0.999, eps, wd, 1, True)
    close(m_dw, 0.1 * g, 1e-12)
    close(th_dw, th0 * (1 - lr * wd) - lr * g / (np.abs(g) + eps), 1e-9)


# ------------------------------------------------------------------ storage rounding
def test_round_bf16_matches_definition():
    # bf16 keeps 8 significant bits: 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1.0)
    assert ops.round_bf16(np.float32(1 + 2 ** -8)) == 1.0
    assert ops.round_bf16(np.float32(1 + 3 * 2 ** -8)) == 1 + 2 ** -6   # tie -> even mantissa
    assert ops.round_bf16(np.float32(1 + 2 ** -8 + 2 ** -12)) == 1 + 2 ** -7
    x = np.float32(RNG.standard_normal(1000))
    r = ops.round_bf16(x)
    assert np.all(np.abs(r - x) <= np.abs(x) * 2 ** -8)
    # idempotent, and equal to torch's cast (library routine)
    import torch
    assert np.array_equal(ops.round_bf16(r), r)
    assert np.array_equal(r, torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy())


# ------------------------------------------------------------------ conv1x1 -> BatchNorm -> act -> point max, one operator
@pytest.mark.parametrize("act", [ops.ACT_NONE, ops.ACT_RELU, ops.ACT_LEAKY])
def test_conv_bn_maxpool_operator(act):
    """Pins of the one-operator tail: brute-force loops for the forward; the statistics in closed
    form from the input's first and second moments (mean = w E[x] + b, var = w Cov(x) w^T);
    central finite differences of sum(v * r) for every gradient; the bias gradient is zero
    because BatchNorm removes any per-channel constant."""
    N, Ci, Co, L = 3, 4, 5, 7
    x, w, b = rnd(N, Ci, L), rnd(Co, Ci), rnd(Co)
    g, bt = rnd(Co), rnd(Co)
    g[0] = -abs(g[0])                                   # a negative scale: the maximum sits at the minimum of z
    eps, slope = 1e-3, 0.3
    v, idx, mean, invstd, nrm, nrv, zhit = ops.conv1x1_bn_maxpool_fwd(x, w, b, g, bt, eps, 0.1, np.zeros(Co), np.ones(Co),
                                                                        act, slope)
    # brute force
    m = N * L
    for c in range(Co):
        zs = [[sum(w[c, i] * x[n, i, l] for i in range(Ci)) + b[c] for l in range(L)] for n in range(N)]
        mu = sum(sum(r) for r in zs) / m
        var = sum(sum((q - mu) ** 2 for q in r) for r in zs) / m
        assert abs(mean[c] - mu) < 1e-12 and abs(invstd[c] - 1 / math.sqrt(var + eps)) < 1e-10
        assert abs(nrm[c] - 0.1 * mu) < 1e-12 and abs(nrv[c] - (0.9 + 0.1 * var * m / (m - 1))) < 1e-12
        for n in range(N):
            ys = [g[c] * (q - mu) / math.sqrt(var + eps) + bt[c] for q in zs[n]]
            if act == ops.ACT_RELU:
                ys = [max(q, 0.0) for q in ys]
            elif act == ops.ACT_LEAKY:
                ys = [q if q > 0 else slope * q for q in ys]
            best = max(range(L), key=lambda l: (ys[l], -l))
            assert idx[n, c] == best and abs(v[n, c] - ys[best]) < 1e-12 and abs(zhit[n, c] - zs[n][best]) < 1e-12
    # closed form of the statistics from the moments of x
    xf = x.transpose(1, 0, 2).reshape(Ci, -1)
    ex, cov = xf.mean(axis=1), np.cov(xf, bias=True)
    close(mean, w @ ex + b, 1e-12)
    close(1 / invstd ** 2 - eps, np.einsum("ci,ij,cj->c", w, cov, w), 1e-12)
    # gradients by central differences of sum(v * r); the argmax is locally constant
    r = rnd(N, Co)
    dx, dw, db, dg, dbt = ops.conv1x1_bn_maxpool_bwd(x, w, b, g, bt, mean, invstd, r, idx, act, slope)
    f = lambda x_, w_, b_, g_, bt_: float((ops.conv1x1_bn_maxpool_fwd(x_, w_, b_, g_, bt_, eps, 0.1, None, None, act, slope)[0] * r).sum())
    close(dx, fd_grad(lambda q: f(q, w, b, g, bt), x), 1e-5)
    close(dw, fd_grad(lambda q: f(x, q, b, g, bt), w), 1e-5)
    close(dg, fd_grad(lambda q: f(x, w, b, q, bt), g), 1e-5)
    close(dbt, fd_grad(lambda q: f(x, w, b, g, q), bt), 1e-5)
    assert np.abs(db).max() < 1e-12 and np.abs(fd_grad(lambda q: f(x, w, q, g, bt), b)).max() < 1e-6


def test_segmentation_head_pieces():
    """Brute-force loops; the broadcast/sum pair is an adjoint pair; the per-point loss against the
    row form on an explicit transpose and by finite differences."""
    N, C, L, K = 2, 3, 5, 4
    z, s, dz = rnd(N, C, L), rnd(N, C), rnd(N, C, L)
    y = ops.add_sample_bias(z, s)
    for n in range(N):
        for c in range(C):
            for l in range(L):
                assert y[n, c, l] == z[n, c, l] + s[n, c]
    sp = ops.sum_points(dz)
    assert abs((ops.add_sample_bias(np.zeros_like(z), s) * dz).sum() - (s * sp).sum()) < 1e-12     # <B s, dz> = <s, B^T dz>
    logits, labels = rnd(N, K, L), RNG.integers(0, K, (N, L))
    loss, d = ops.softmax_xent_points(logits, labels)
    ref = 0.0
    for n in range(N):
        for l in range(L):
            col = logits[n, :, l]
            ref += math.log(sum(math.exp(q) for q in col)) - col[labels[n, l]]
    assert abs(loss - ref / (N * L)) < 1e-12
    close(d, fd_grad(lambda q: ops.softmax_xent_points(q, labels)[0], logits), 1e-6)
    dx, dv = rnd(N, C, L), rnd(N, C)
    idx = RNG.integers(0, L, (N, C))
    out = ops.maxpool_points_bwd_add(dx, dv, idx)
    close(out, dx + ops.maxpool_points_bwd(dv, idx, L), 1e-15)


def test_adadelta_and_steplr_vs_library_and_closed_forms():
    """torch.optim.Adadelta / StepLR (library routines, float64) over several steps with weight
    decay; first step from zero state in closed form; lr = 0 leaves the parameters untouched."""
    import torch
    P = 9
    th0 = rnd(P)
    grads = [rnd(P) for _ in range(4)]
    lr, rho, eps, wd = 0.7, 0.85, 1e-6, 0.05
    tp = torch.tensor(th0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adadelta([tp], lr=lr, rho=rho, eps=eps, weight_decay=wd)
    th, v, u = th0.copy(), np.zeros(P), np.zeros(P)
    for g in grads:
        tp.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        th, v, u = ops.adadelta_step(th, g, v, u, lr, rho, eps, wd)
        close(th, tp.detach().numpy(), 1e-12)
    g = grads[0]
    th1, v1, u1 = ops.adadelta_step(th0, g, np.zeros(P), np.zeros(P), lr, rho, eps, 0.0)
    d = math.sqrt(eps) / np.sqrt((1 - rho) * g * g + eps) * g
    close(v1, (1 - rho) * g * g, 1e-14)
    close(u1, (1 - rho) * d * d, 1e-12)
    close(th1 - th0, -lr * d, 1e-12)
    assert np.array_equal(ops.adadelta_step(th0, g, v, u, 0.0, rho, eps, wd)[0], th0)
    # step schedule against the library, per-model factor and period
    base, gam, step = np.array([0.1, 0.02, 0.5]), np.array([0.5, 0.1, 0.9]), np.array([1, 3, 4])
    for b in range(3):
        q = torch.nn.Parameter(torch.zeros(1))
        o = torch.optim.SGD([q], lr=float(base[b]))
        sch = torch.optim.lr_scheduler.StepLR(o, step_size=int(step[b]), gamma=float(gam[b]))
        for epoch in range(10):
            assert abs(ops.steplr(base, gam, step, epoch)[b] - o.param_groups[0]["lr"]) <= 1e-12 * base[b]
            o.step()
            sch.step()


def test_point_transform_bruteforce_and_adjoints():
    N, Ci, Co, L = 2, 3, 4, 5
    x, t, dy = rnd(N, Ci, L), rnd(N, Co, Ci), rnd(N, Co, L)
    y = ops.point_transform_fwd(x, t)
    for n in range(N):
        for o in range(Co):
            for l in range(L):
                assert abs(y[n, o, l] - sum(t[n, o, c] * x[n, c, l] for c in range(Ci))) < 1e-13
    dx, dt = ops.point_transform_bwd(x, t, dy)
    close(dx, fd_grad(lambda q: float((ops.point_transform_fwd(q, t) * dy).sum()), x), 1e-6)
    close(dt, fd_grad(lambda q: float((ops.point_transform_fwd(x, q) * dy).sum()), t), 1e-6)
    # samples do not mix: changing sample 1's matrix leaves sample 0's output untouched
    t2 = t.copy(); t2[1] += 1.0
    assert np.array_equal(ops.point_transform_fwd(x, t2)[0], y[0])


def test_bn_eval_fwd_pins():
    """Evaluation-mode BatchNorm: torch's batch_norm with training=False (a library routine); the closed
    form at the running estimates themselves (x = running_mean -> beta); and the link to training mode:
    with the running estimates set to a batch's own mean and biased variance it reproduces that batch's
    training-mode output."""
    import torch
    import torch.nn.functional as F
    rng = np.random.default_rng(91)
    x = rng.standard_normal((5, 4, 7)) * 2 + 1
    g, b = rng.standard_normal(4), rng.standard_normal(4)
    rm, rv = rng.standard_normal(4), rng.uniform(0.3, 2.0, 4)
    y = ops.bn_eval_fwd(x, g, b, rm, rv, 1e-3)
    T = lambda a: torch.tensor(a, dtype=torch.float64)
    ref = F.batch_norm(T(x), T(rm), T(rv), T(g), T(b), training=False, eps=1e-3).numpy()
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-13)
    at_mean = ops.bn_eval_fwd(np.broadcast_to(rm[None, :, None], x.shape), g, b, rm, rv)
    np.testing.assert_allclose(at_mean, np.broadcast_to(b[None, :, None], x.shape), rtol=0, atol=1e-15)
    yt, mu, invstd, _, _ = ops.bn_fwd(x, g, b, 1e-5)
    np.testing.assert_allclose(ops.bn_eval_fwd(x, g, b, mu, 1.0 / invstd ** 2 - 1e-5, 1e-5), yt, rtol=0, atol=1e-12)
