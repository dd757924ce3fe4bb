"""Parity at the full sizes of the BASELINE configs, in the launch configuration the benchmark
times.  A full oracle run is out of reach there (hundreds of GFLOP of float64), so:
GEMM / convolution outputs are checked on seeded samples of output coordinates, each recomputed
by the oracle's definition as an independent dot product from the very input bits the GPU read;
reduction-type outputs (statistics, pooled maxima, parameter gradients of sampled channels,
Adam) are checked in full for sampled channels / in full."""
import numpy as np
import pytest
import torch

import hfta_inputs as hi
from oracle import ops as oops
from util import DT, TOL, bn_preact_fp32, check_tail_argmax

pytestmark = pytest.mark.gpu
bf = torch.bfloat16


def f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def rel_ok(got, ref, tol, what):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    scale = np.sqrt(np.mean(ref * ref)) + 1e-30
    bad = np.abs(got - ref) > tol * (np.abs(ref) + scale)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} samples beyond tol, worst {np.abs(got - ref)[bad].max():.3e}"


@pytest.mark.parametrize("fused_tail", [True, False])
def test_c1_full_size_step_sampled(fused_tail):
    """Config 1 as benchmarked: B=8, bf16, 32 clouds x 2500 points per model (``fused_tail`` is the
    benchmark's configuration; the unfused tail is the path other storage types take)."""
    from paper_2102_02344_amd.arrays import FusedPointNetCls
    spec = hi.spec_c1()
    inp = hi.pointnet_cls_inputs(spec)
    arr = FusedPointNetCls(spec, inp, fused_tail=fused_tail)
    B, Nb, L = spec.B, spec.Nb, spec.L
    rng = np.random.default_rng(5)
    tol = TOL["bf16"]
    seen = []

    def chan(t, b, C, c):          # [Nb, L] slice of channel (b, c) of a [Nb, B*C, L] tensor
        return f64(t[:, b * C + c, :])

    def probe(op, **kw):
        lay = kw.get("layer", "")
        if op == "conv1x1_fwd" and lay in ("conv0", "conv4"):
            print("full-size check", op, lay, flush=True)
            x, y = kw["x"], kw["y"]
            Ci, Co = x.shape[1] // B, y.shape[1] // B
            w = kw["w"].view(B, Co, Ci)
            bias = kw["b"].view(B, Co)
            S = 3000
            n, b, o, l = (rng.integers(0, m, S) for m in (Nb, B, Co, L))
            nt, bt, ot, lt = (torch.from_numpy(a).cuda() for a in (n, b, o, l))
            ci = torch.arange(Ci, device="cuda")
            xs = f64(x[nt[:, None], (bt * Ci)[:, None] + ci[None, :], lt[:, None]])          # [S, Ci]
            ws = f64(w[bt, ot])                                                                 # [S, Ci]
            ref = (xs * ws).sum(axis=1) + f64(bias[bt, ot])
            rel_ok(f64(y[nt, bt * Co + ot, lt]), ref, tol, f"{lay} fwd")
            seen.append(op + lay)
        elif op == "bn_fwd_maxpool":
            print("full-size check", op, flush=True)
            C = kw["x"].shape[1] // B
            for b, c in zip(rng.integers(0, B, 12), rng.integers(0, C, 12)):
                z = chan(kw["x"], b, C, c)
                k = b * C + c
                g, bt_ = float(kw["g"][k]), float(kw["b"][k])
                y, mean, invstd, _, _ = oops.bn_fwd(z[:, None, :], [g], [bt_], 1e-5)
                assert abs(float(kw["mean"][k]) - mean[0]) <= 1e-5 * (abs(mean[0]) + np.sqrt(1 / invstd[0] ** 2))
                assert abs(float(kw["invstd"][k]) - invstd[0]) <= 1e-5 * invstd[0]
                ya = oops.store(oops.act_fwd(y[:, 0, :], oops.ACT_RELU), "bf16")
                v, idx = oops.maxpool_points_fwd(ya[:, None, :])
                gv, gi = f64(kw["v"][b, :, c]), kw["idx"][b, :, c].cpu().numpy()
                rel_ok(gv, v[:, 0], tol, "pooled")
                mism = gi != idx[:, 0]
                if mism.any():      # legitimate only at a near-tie of the maximum
                    at = ya[np.arange(Nb), gi]
                    assert np.all(at[mism] >= v[mism, 0] - tol * (np.abs(v[mism, 0]) + np.abs(ya).max()))
            seen.append(op)
        elif op == "bn_bwd_maxpool":
            print("full-size check", op, flush=True)
            C = kw["x"].shape[1] // B
            for b, c in zip(rng.integers(0, B, 8), rng.integers(0, C, 8)):
                z = chan(kw["x"], b, C, c)
                k = b * C + c
                g, bt_ = float(kw["g"][k]), float(kw["b"][k])
                mean, invstd = float(kw["mean"][k]), float(kw["invstd"][k])
                dv, idx = f64(kw["dv"][b, :, c]), kw["idx"][b, :, c].cpu().numpy()
                dy = oops.maxpool_points_bwd(dv[:, None], idx[:, None], L)[:, 0, :]
                y = g * (z - mean) * invstd + bt_
                gdy = oops.act_bwd(y, dy, oops.ACT_RELU)
                dx, dg, dbt = oops.bn_bwd(z[:, None, :], gdy[:, None, :], [g], [mean], [invstd])
                rel_ok(chan(kw["dx"], b, C, c), dx[:, 0, :], tol, "bn+pool dx")
                sc = np.abs(dv).sum()
                assert abs(float(kw["dg"][k]) - dg[0]) <= 2e-4 * max(abs(dg[0]), 1e-2 * sc)
                assert abs(float(kw["db"][k]) - dbt[0]) <= 2e-4 * max(abs(dbt[0]), 1e-2 * sc)
            seen.append(op)
        elif op == "conv1x1_bn_bwd" and lay in ("conv0", "conv2", "conv3"):
            # BatchNorm backward + convolution backward in one call (3 -> 64 without a data gradient,
            # 64 -> 64, 64 -> 128): ONE seeded model of the eight in full, every output, against the
            # oracle's chain of the two single operators with dz stored in between (the models of an
            # array share nothing, so the oracle runs that model alone on the bits the GPU read)
            print("full-size check", op, lay, flush=True)
            b = int(rng.integers(0, B))
            Co = kw["z"].shape[1] // B
            Ci = kw["x"].shape[1] // B
            so, si = slice(b * Co, (b + 1) * Co), slice(b * Ci, (b + 1) * Ci)
            z, dy, x = f64(kw["z"][:, so, :]), f64(kw["dy"][:, so, :]), f64(kw["x"][:, si, :])
            g, bt_, mean, invstd = (f64(kw[n_])[so] for n_ in ("g", "bt", "mean", "invstd"))
            w = f64(kw["w"].view(B, Co, Ci)[b])
            dz, dg, dbt = oops.bn_bwd(z, oops.act_bwd(bn_preact_fp32(z, g, bt_, mean, invstd), dy, oops.ACT_RELU), g, mean, invstd)
            sc = np.abs(dy).sum(axis=(0, 2))
            assert np.all(np.abs(f64(kw["dg"])[so] - dg) <= 2e-4 * np.maximum(np.abs(dg), 1e-2 * sc)), f"{lay} dgamma"
            assert np.all(np.abs(f64(kw["dbt"])[so] - dbt) <= 2e-4 * np.maximum(np.abs(dbt), 1e-2 * sc)), f"{lay} dbeta"
            dzs = oops.store(dz, "bf16")
            dx, dw, db = oops.conv1x1_bwd(x, w, dzs)
            if kw["dx"] is not None:
                rel_ok(f64(kw["dx"][:, si, :]), dx, tol, f"{lay} dX")
            # dz rounds the other way for a few elements in a thousand (fp32 against float64 arithmetic),
            # each moving one term of a weight-gradient element by one bf16 ulp (2^-8 of the term).  The
            # flips are not independent: behind a ReLU that is off, dz = -sc (mb + xhat mg) takes one value
            # per distinct stored z, so all points of a channel that share a z value flip together.  Worst
            # case (every term flips) is 2^-8 of the sum of magnitudes; the bound here is 1e-4 of it (or 1e-2
            # of the element itself), and 3e-4 in root mean square over the layer's weight gradient.
            gw = f64(kw["dw"].view(B, Co, Ci)[b])
            terms = np.einsum("nol,ncl->oc", np.abs(dzs), np.abs(x))
            ratio = np.abs(gw - dw) / np.maximum(np.abs(dw), 1e-2 * terms)
            assert ratio.max() <= 1e-2, f"{lay} dW: worst {ratio.max():.3e} at {np.unravel_index(ratio.argmax(), ratio.shape)}, " \
                                        f"{(ratio > 1e-2).sum()} of {ratio.size} beyond"
            assert np.sqrt(np.mean((gw - dw) ** 2)) <= 3e-4 * np.sqrt(np.mean(dw ** 2)), f"{lay} dW (rms)"
            assert np.all(np.abs(f64(kw["db"])[so] - db) <= 2e-4 * np.abs(dzs).sum(axis=(0, 2))), f"{lay} dbias"
            seen.append(op + lay)
        elif op == "conv1x1_bwd" and lay == "conv4":
            print("full-size check", op, lay, flush=True)
            x, dy = kw["x"], kw["dy"]
            Ci, Co = x.shape[1] // B, dy.shape[1] // B
            dw = kw["dw"].view(B, Co, Ci)
            w = kw["w"].view(B, Co, Ci)
            for b, o, c in zip(rng.integers(0, B, 24), rng.integers(0, Co, 24), rng.integers(0, Ci, 24)):
                ref = (chan(dy, b, Co, o) * chan(x, b, Ci, c)).sum()
                terms = np.abs(chan(dy, b, Co, o) * chan(x, b, Ci, c)).sum()
                assert abs(float(dw[b, o, c]) - ref) <= 2e-4 * max(abs(ref), 1e-2 * terms), "conv4 dW"
            S = 2000
            n, b, c, l = (rng.integers(0, m, S) for m in (Nb, B, Ci, L))
            nt, bt, ct, lt = (torch.from_numpy(a).cuda() for a in (n, b, c, l))
            co = torch.arange(Co, device="cuda")
            dys = f64(dy[nt[:, None], (bt * Co)[:, None] + co[None, :], lt[:, None]])         # [S, Co]
            ws = f64(w[bt, :, ct])                                                              # [S, Co]
            rel_ok(f64(kw["dx"][nt, bt * Ci + ct, lt]), (dys * ws).sum(axis=1), tol, "conv4 dX")
            seen.append(op + lay)

        elif op == "conv1x1_bn_maxpool_fwd":
            # sampled channels of every model, all 32 x 2500 points of each: the oracle's composition of the
            # four single operators on those channels (BatchNorm is per channel, so a channel subset is exact)
            print("full-size check", op, flush=True)
            x = kw["x"]
            Co, Ci = kw["idx"].shape[2], x.shape[1] // B
            w, bias = f64(kw["w"].view(B, Co, Ci)), f64(kw["b"]).reshape(B, Co)
            g, bt_ = f64(kw["g"]).reshape(B, Co), f64(kw["bt"]).reshape(B, Co)
            nm = nd = 0
            for b in range(B):
                oc = np.sort(rng.choice(Co, 16, replace=False))
                xb = f64(x[:, b * Ci:(b + 1) * Ci, :])
                rv, ri, mean, invstd, _, _, rz = oops.conv1x1_bn_maxpool_fwd(xb, w[b, oc], bias[b, oc], g[b, oc], bt_[b, oc],
                                                                             1e-5, 0.1, None, None, oops.ACT_RELU)
                z = oops.conv1x1_fwd(xb, w[b, oc], bias[b, oc])
                ez2, var = (z ** 2).mean(axis=(0, 2)), 1.0 / invstd ** 2 - 1e-5
                gm, gis = f64(kw["mean"]).reshape(B, Co)[b, oc], f64(kw["invstd"]).reshape(B, Co)[b, oc]
                assert np.all(np.abs(gm - mean) <= 1e-5 * (np.abs(mean) + np.sqrt(var) + np.sqrt(ez2))), "mean"
                assert np.all(np.abs(gis - invstd) <= invstd * (1e-5 + 2e-6 * ez2 / (var + 1e-5))), "invstd"
                ya = oops.act_fwd(oops.bn_fwd(z, g[b, oc], bt_[b, oc], 1e-5)[0], oops.ACT_RELU)
                gi = kw["idx"][b][:, torch.from_numpy(oc).cuda()].cpu().numpy()                  # [Nb, 16]
                rel_ok(f64(kw["v"][b][:, torch.from_numpy(oc).cuda()]), oops.store(rv, "bf16"), tol, "pooled")
                nm += check_tail_argmax(ya, ri, gi, oops.conv1x1_fwd(np.abs(xb), np.abs(w[b, oc]), None), Ci,
                                        np.abs(g[b, oc]) * invstd, "one-operator tail at full size")
                nd += gi.size
                zat = np.take_along_axis(z, gi[:, :, None].astype(np.int64), axis=2)[:, :, 0]
                assert np.abs(f64(kw["zhit"][b][:, torch.from_numpy(oc).cuda()]) - zat).max() <= 1e-5 * np.abs(z).max()
            print(f"one-operator tail at config-1 size: {nm} of {nd} sampled argmax decisions differ from the oracle's", flush=True)
            seen.append(op)
        elif op == "conv1x1_bn_maxpool_bwd":
            # one whole model: the oracle's backward composition (max-pool scatter -> ReLU -> BatchNorm ->
            # convolution) on all 1024 channels and all points, every output of that model compared
            print("full-size check", op, "(one model through the oracle, about a minute of float64)", flush=True)
            x = kw["x"]
            Co, Ci = kw["idx"].shape[2], x.shape[1] // B
            b = int(rng.integers(0, B))
            xb = f64(x[:, b * Ci:(b + 1) * Ci, :])
            sl = slice(b * Co, (b + 1) * Co)
            dx, dw, _, dg, dbt = oops.conv1x1_bn_maxpool_bwd(
                xb, f64(kw["w"].view(B, Co, Ci)[b]), f64(kw["b"]).reshape(B, Co)[b], f64(kw["g"])[sl], f64(kw["bt"])[sl],
                f64(kw["mean"])[sl], f64(kw["invstd"])[sl], f64(kw["dv"][b]), kw["idx"][b].cpu().numpy(), oops.ACT_RELU)
            rel_ok(f64(kw["dx"][:, b * Ci:(b + 1) * Ci, :]), dx, tol, "one-operator tail dX")
            rel_ok(f64(kw["dw"].view(B, Co, Ci)[b]), dw, 2e-4, "one-operator tail dW")
            sc = np.abs(f64(kw["dv"][b])).sum(axis=0)
            assert np.all(np.abs(f64(kw["dg"])[sl] - dg) <= 2e-4 * np.maximum(np.abs(dg), 1e-2 * sc)), "dgamma"
            assert np.all(np.abs(f64(kw["dbt"])[sl] - dbt) <= 2e-4 * np.maximum(np.abs(dbt), 1e-2 * sc)), "dbeta"
            seen.append(op)

    arr.forward_backward(probe)
    torch.cuda.synchronize()
    tail = ({"conv1x1_bn_maxpool_fwd", "conv1x1_bn_maxpool_bwd"} if fused_tail
            else {"conv1x1_fwdconv4", "bn_fwd_maxpool", "bn_bwd_maxpool", "conv1x1_bwdconv4"})
    assert set(seen) == {"conv1x1_fwdconv0", "conv1x1_bn_bwdconv0", "conv1x1_bn_bwdconv2", "conv1x1_bn_bwdconv3"} | tail
    assert np.all(np.isfinite(arr.loss.cpu().numpy()))
    # Adam over the whole arena, in full, from the gradients the GPU just produced
    th0, g = f64(arr.theta), f64(arr.grad)
    arr.adam()
    torch.cuda.synchronize()
    th1 = f64(arr.theta)
    for j, (name, shp) in enumerate(arr.shapes):
        o, n = arr.seg_offsets[j], arr.seg_offsets[j + 1] - arr.seg_offsets[j]
        sl = slice(B * o, B * (o + n))
        for b in range(B):
            sb = slice(B * o + b * n, B * o + (b + 1) * n)
            ref, _, _ = oops.adam_step(th0[sb], g[sb], np.zeros(n), np.zeros(n), inp["lr"][b], inp["beta1"][b],
                                       inp["beta2"][b], inp["eps"][b], inp["wd"][b], 1)
            assert np.abs(th1[sb] - ref).max() <= 1e-5 * max(np.abs(ref).max(), 1e-30), name
    assert torch.equal(arr.lowp, arr.theta.to(bf))


@pytest.mark.parametrize("Fx,Fy", [(512, 2048), (2048, 512)])
def test_c4_linear_full_size_sampled(Fx, Fy):
    """Config 4's GEMMs: B=16 models, 32 x 128 = 4096 tokens per model, bf16."""
    from paper_2102_02344_amd import binding as hb
    B, M = 16, 4096
    g = torch.Generator(device="cuda").manual_seed(40 + Fx)
    X = torch.randn(B, M, Fx, device="cuda", generator=g).to(bf)
    W = (torch.randn(B, Fx, Fy, device="cuda", generator=g) * (6.0 / Fx) ** 0.5).to(bf)
    bias = torch.randn(B, Fy, device="cuda", generator=g).to(bf)
    dY = torch.randn(B, M, Fy, device="cuda", generator=g).to(bf)
    Y = torch.empty(B, M, Fy, device="cuda", dtype=bf)
    dX = torch.empty_like(X)
    dW = torch.empty(B, Fx, Fy, device="cuda")
    db = torch.empty(B, Fy, device="cuda")
    ws = torch.empty(max(4, hb.linear_bwd_workspace_bytes(B, M, Fx, Fy, DT["bf16"])), dtype=torch.uint8, device="cuda")
    hb.linear_fwd(B, M, Fx, Fy, DT["bf16"], X, W, bias, Y, hb.ACT_GELU)
    hb.linear_bwd(B, M, Fx, Fy, DT["bf16"], X, W, dY, dX, dW, db, ws)
    torch.cuda.synchronize()
    rng = np.random.default_rng(7)
    S = 4096
    b, r, i, j = (torch.from_numpy(rng.integers(0, m, S)).cuda() for m in (B, M, Fx, Fy))
    ref = (f64(X[b, r, :]) * f64(W[b, :, j])).sum(axis=1) + f64(bias[b, j])
    rel_ok(f64(Y[b, r, j]), oops.act_fwd(ref, oops.ACT_GELU), TOL["bf16"], "Y = gelu(XW + b)")
    for act, oact in ((hb.ACT_NONE, oops.ACT_NONE), (hb.ACT_RELU, oops.ACT_RELU)):   # the persistent kernel's epilogues
        hb.linear_fwd(B, M, Fx, Fy, DT["bf16"], X, W, bias, Y, act)
        torch.cuda.synchronize()
        rel_ok(f64(Y[b, r, j]), oops.act_fwd(ref, oact), TOL["bf16"], f"Y = act{act}(XW + b)")
    rel_ok(f64(dX[b, r, i]), (f64(dY[b, r, :]) * f64(W[b, i, :])).sum(axis=1), TOL["bf16"], "dX")
    rel_ok(f64(dW[b, i, j]), (f64(X[b, :, i]) * f64(dY[b, :, j])).sum(axis=1), 2e-4, "dW")
    rel_ok(f64(db), f64(dY).sum(axis=1), 2e-4, "dbias")


def test_c4_fused_reductions_full_size():
    """Config 4's element-wise operators with reductions folded in (GELU backward + bias gradient,
    LayerNorm backward + residual sum + bias gradient), B=16 models x 4096 tokens, bf16: sampled
    elements / rows by the oracle's definitions, the sums against the stored tensors."""
    from paper_2102_02344_amd import binding as hb
    B, R, E, H = 16, 4096, 512, 2048
    g = torch.Generator(device="cuda").manual_seed(44)
    Z = torch.randn(B, R, H, device="cuda", generator=g).to(bf)
    dA = torch.randn(B, R, H, device="cuda", generator=g).to(bf)
    dZ = torch.empty_like(Z)
    db1 = torch.empty(B, H, device="cuda")
    hb.act_bwd_colsum(B, R, H, DT["bf16"], Z, dA, dZ, db1, hb.ACT_GELU)
    torch.cuda.synchronize()
    rng = np.random.default_rng(11)
    S = 8192
    b, r, j = (torch.from_numpy(rng.integers(0, m, S)).cuda() for m in (B, R, H))
    rel_ok(f64(dZ[b, r, j]), oops.act_bwd(f64(Z[b, r, j]), f64(dA[b, r, j]), oops.ACT_GELU), TOL["bf16"], "gelu backward")
    rel_ok(f64(db1), dZ.double().sum(dim=1).cpu().numpy(), 2e-4, "bias gradient = column sums of the stored dZ")
    del Z, dA, dZ

    X = (torch.randn(B, R, E, device="cuda", generator=g) * 2 + 0.5).to(bf)
    w = torch.randn(B, E, device="cuda", generator=g) * 0.5 + 1.0
    bt = torch.randn(B, E, device="cuda", generator=g) * 0.2
    d1 = torch.randn(B, R, E, device="cuda", generator=g).to(bf)
    d2 = torch.randn(B, R, E, device="cuda", generator=g).to(bf)
    SM, SI = torch.empty(B, R, device="cuda"), torch.empty(B, R, device="cuda")
    Y, dX = torch.empty_like(X), torch.empty_like(X)
    dw, db, dxs = (torch.empty(B, E, device="cuda") for _ in range(3))
    ws = torch.empty(hb.layernorm_bwd_sums_workspace_bytes(B, R, E), dtype=torch.uint8, device="cuda")
    hb.layernorm_fwd(B, R, E, DT["bf16"], X, w, bt, 1e-5, SM, SI, Y)
    hb.layernorm_bwd_sums(B, R, E, DT["bf16"], X, d1, d2, w, SM, SI, dX, dw, db, dxs, ws)
    torch.cuda.synchronize()
    dsum = (d1.float() + d2.float()).to(bf)                 # the pair as a stored sum
    for bb in (0, 7, 15):
        rows = np.sort(rng.choice(R, 64, replace=False))
        x = f64(X[bb, rows])
        mean = x.mean(axis=1)
        invstd = 1.0 / np.sqrt(x.var(axis=1) + 1e-5)
        rel_ok(f64(SM[bb, rows]), mean, 1e-5, "row mean")
        rel_ok(f64(SI[bb, rows]), invstd, 1e-5, "row 1/std")
        rdx, _, _ = oops.layernorm_bwd(x, f64(dsum[bb, rows]), f64(w[bb]), mean, invstd)
        rel_ok(f64(dX[bb, rows]), rdx, TOL["bf16"], "LayerNorm dX rows")
    xhat = (X.double() - SM.double()[:, :, None]) * SI.double()[:, :, None]
    rel_ok(f64(dw), (dsum.double() * xhat).sum(dim=1).cpu().numpy(), 2e-4, "LayerNorm dw")
    rel_ok(f64(db), dsum.double().sum(dim=1).cpu().numpy(), 2e-4, "LayerNorm db")
    rel_ok(f64(dxs), dX.double().sum(dim=1).cpu().numpy(), 2e-4, "column sums of the stored dX")


def _gen(seed):
    return torch.Generator(device="cuda").manual_seed(seed)


def _host_slices(T, Nb, B, C, b, imgs=None, chans=None):
    """float64 [n, C', H, W] slice of model b (and of a sample / channel subset) of an [Nb, B*C, H, W] tensor."""
    v = T.view(Nb, B, C, T.shape[2], T.shape[3])[:, b]
    if imgs is not None:
        v = v[imgs]
    if chans is not None:
        v = v[:, chans]
    return f64(v)


@pytest.mark.parametrize("path", ["implicit", "lowered"])
@pytest.mark.parametrize("Ci,Co,H,s,p", hi.DCGAN_D_LAYERS)
def test_c3_conv2d_full_size(Ci, Co, H, s, p, path):
    """Config 3's discriminator layers at full size (B=10 models, 64 images per model, 4x4 kernels, bf16),
    on both convolution paths (implicit GEMM without a workspace; column-buffer lowering with one).
    References are the oracle's conv2d_fwd / conv2d_bwd on gathered slices of the tensors the GPU read:
    output and data gradient of four sampled images of two sampled models in full, the weight gradient
    (a reduction over all 64 images) for eight sampled output channels of those models in full."""
    from paper_2102_02344_amd import binding as hb
    B, Nb, k = 10, 64, 4
    Ho = (H + 2 * p - k) // s + 1
    print(f"conv2d {Ci}->{Co} {H}x{H} s{s} p{p} {path}", flush=True)
    g = _gen(300 + Ci)
    X = (torch.rand(Nb, B * Ci, H, H, device="cuda", generator=g) * 2 - 1).to(bf)
    W = (torch.randn(B * Co, Ci, k, k, device="cuda", generator=g) * 0.02).to(bf)
    dY = torch.randn(Nb, B * Co, Ho, Ho, device="cuda", generator=g).to(bf)
    Y = torch.empty_like(dY)
    dX = torch.empty_like(X)
    dW = torch.empty(B * Co, Ci, k, k, device="cuda")
    geo = (B, Nb, Ci, Co, H, H, k, k, s, p, DT["bf16"])
    if path == "lowered":
        nws = max(hb.conv2d_grouped_bwd_workspace_bytes(*geo), hb.conv2d_grouped_fwd_workspace_bytes(*geo))
    else:
        nws = hb.conv2d_grouped_bwd_min_workspace_bytes(*geo)
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda") if nws else None
    hb.conv2d_grouped_fwd(*geo, X, W, None, Y, workspace=ws if path == "lowered" else None)
    hb.conv2d_grouped_bwd(*geo, X, W, dY, dX, dW, None, ws)
    torch.cuda.synchronize()
    rng = np.random.default_rng(9 + Ci)
    for b in rng.choice(B, 2, replace=False):
        imgs = np.sort(rng.choice(Nb, 4, replace=False))
        wb = f64(W[b * Co:(b + 1) * Co])
        xb = _host_slices(X, Nb, B, Ci, b, imgs)
        rel_ok(_host_slices(Y, Nb, B, Co, b, imgs), oops.conv2d_fwd(xb, wb, None, s, p), TOL["bf16"], "Y")
        dx, _, _ = oops.conv2d_bwd(xb, wb, _host_slices(dY, Nb, B, Co, b, imgs), s, p)
        rel_ok(_host_slices(dX, Nb, B, Ci, b, imgs), dx, TOL["bf16"], "dX")
        oc = np.sort(rng.choice(Co, min(8, Co), replace=False))
        _, dw, _ = oops.conv2d_bwd(_host_slices(X, Nb, B, Ci, b), wb[oc], _host_slices(dY, Nb, B, Co, b, chans=oc), s, p)
        rel_ok(f64(dW[b * Co:(b + 1) * Co][oc]), dw, 2e-4, "dW")


@pytest.mark.parametrize("path", ["implicit", "lowered"])
@pytest.mark.parametrize("Cx,Cy,H,s,p", hi.DCGAN_G_LAYERS)
def test_c3_convT2d_full_size(Cx, Cy, H, s, p, path):
    """Config 3's generator layers (ConvTranspose2d, weights [B*Cx, Cy, 4, 4]) at full size, as the array
    calls them: forward = the grouped convolution's data-gradient form, data gradient = its forward,
    weight gradient = its weight gradient with input and output gradient exchanged.  References:
    the oracle's convT2d_fwd / convT2d_bwd on gathered slices (four images of two models in full;
    weight gradient of eight sampled input channels over all 64 images)."""
    from paper_2102_02344_amd import binding as hb
    B, Nb, k = 10, 64, 4
    Ho = (H - 1) * s - 2 * p + k
    print(f"convT2d {Cx}->{Cy} {H}x{H} s{s} p{p} {path}", flush=True)
    g = _gen(400 + Cx)
    X = torch.randn(Nb, B * Cx, H, H, device="cuda", generator=g).to(bf)
    W = (torch.randn(B * Cx, Cy, k, k, device="cuda", generator=g) * 0.02).to(bf)
    dY = torch.randn(Nb, B * Cy, Ho, Ho, device="cuda", generator=g).to(bf)
    Y = torch.empty_like(dY)
    dX = torch.empty_like(X)
    dW = torch.empty(B * Cx, Cy, k, k, device="cuda")
    geo = (B, Nb, Cy, Cx, Ho, Ho, k, k, s, p, DT["bf16"])          # the convolution this layer is the transpose of
    if path == "lowered":
        nws = max(hb.conv2d_grouped_bwd_workspace_bytes(*geo), hb.conv2d_grouped_fwd_workspace_bytes(*geo))
    else:
        nws = hb.conv2d_grouped_bwd_min_workspace_bytes(*geo)
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda") if nws else None
    hb.conv2d_grouped_bwd(*geo, None, W, X, Y, None, None, ws)                                   # ConvT forward
    hb.conv2d_grouped_fwd(*geo, dY, W, None, dX, workspace=ws if path == "lowered" else None)    # ConvT data gradient
    hb.conv2d_grouped_bwd(*geo, dY, None, X, None, dW, None, ws)                                 # ConvT weight gradient
    torch.cuda.synchronize()
    rng = np.random.default_rng(19 + Cx)
    for b in rng.choice(B, 2, replace=False):
        imgs = np.sort(rng.choice(Nb, 4, replace=False))
        wb = f64(W[b * Cx:(b + 1) * Cx])
        xb = _host_slices(X, Nb, B, Cx, b, imgs)
        rel_ok(_host_slices(Y, Nb, B, Cy, b, imgs), oops.convT2d_fwd(xb, wb, None, s, p), TOL["bf16"], "ConvT Y")
        dx, _, _ = oops.convT2d_bwd(xb, wb, _host_slices(dY, Nb, B, Cy, b, imgs), s, p)
        rel_ok(_host_slices(dX, Nb, B, Cx, b, imgs), dx, TOL["bf16"], "ConvT dX")
        ic = np.sort(rng.choice(Cx, min(8, Cx), replace=False))
        _, dw, _ = oops.convT2d_bwd(_host_slices(X, Nb, B, Cx, b, chans=ic), wb[ic], _host_slices(dY, Nb, B, Cy, b), s, p)
        rel_ok(f64(dW[b * Cx:(b + 1) * Cx][ic]), dw, 2e-4, "ConvT dW")


def test_c2_full_size_step_sampled():
    """Config 2 as benchmarked: B=6, bf16, 16 clouds x 2500 points per model, 2880-channel
    concatenation.  The calls that are new at this size (convolutions over channel slices of the
    concatenation buffers, K = 2880 and 512 -> 2048 GEMMs, the head's strided support operators)
    are checked on seeded samples recomputed from the bits the GPU read."""
    from paper_2102_02344_amd.arrays import FusedPointNetSeg
    spec = hi.spec_c2()
    inp = hi.pointnet_seg_inputs(spec)
    arr = FusedPointNetSeg(spec, inp)
    B, Nb, L = spec.B, spec.Nb, spec.L
    rng = np.random.default_rng(21)
    tol = TOL["bf16"]
    seen = []
    S = 1500

    def v4(t, C):                      # [Nb, B*C, L] or [Nb, B, C, L] -> [Nb, B, C, L] view
        return t if t.dim() == 4 else t.view(Nb, B, C, L)

    def pick(*dims):
        return [torch.from_numpy(rng.integers(0, m, S)).cuda() for m in dims]

    def probe(op, **kw):
        lay = kw.get("layer", "")
        if op in ("conv1x1_fwd", "conv1x1_fwd_sample_bias") and lay in ("conv4", "head0", "head3"):
            # sampled outputs; the reference of each is the oracle's operator on its gathered input column
            # (head0: the convolution over the 2880 per-point channels plus the per-sample term)
            print("full-size check", op, lay, flush=True)
            Co = kw["y"].shape[1] // B
            w = kw["w"].view(B, Co, -1)
            Ci = w.shape[2]
            x, y = v4(kw["x"], Ci), v4(kw["y"], Co)
            n, b, o, l = pick(Nb, B, Co, L)
            cols, rows = f64(x[n, b, :, l]), f64(w[b, o])                                   # [S, Ci] each
            bias = f64(kw["s"][b, n, o]) if op == "conv1x1_fwd_sample_bias" else f64(kw["b"].view(B, Co)[b, o])
            ref = np.array([oops.conv1x1_fwd(cols[i][None, :, None], rows[i][None, :], bias[i:i + 1])[0, 0, 0] for i in range(S)])
            rel_ok(f64(y[n, b, o, l]), ref, tol, f"{lay} fwd")
            seen.append("conv1x1_fwd" + lay)
        elif op == "softmax_xent_points":
            K = kw["logits"].shape[1] // B
            lg, d = v4(kw["logits"], K), v4(kw["d"], K)
            n, b, l = pick(Nb, B, L)
            z = f64(lg[n, b, :, l])                                                         # [S, K]
            lab = kw["labels"][b, n, l].cpu().numpy()
            lse = np.log(np.exp(z - z.max(axis=1, keepdims=True)).sum(axis=1)) + z.max(axis=1)
            p = np.exp(z - lse[:, None])
            p[np.arange(S), lab] -= 1.0
            rel_ok(f64(d[n, b, :, l]), p / (Nb * L), tol, "dlogits")
            for bb in range(B):                                                             # the loss in full, per model
                zb = f64(lg[:, bb]).transpose(0, 2, 1).reshape(Nb * L, K)
                rl, _ = oops.softmax_xent(zb, kw["labels"][bb].cpu().numpy().reshape(-1))
                assert abs(float(kw["loss"][bb]) - rl) <= 1e-5 * abs(rl)
            seen.append(op)
        elif op == "sum_points":
            C = kw["s"].shape[2]
            for b, n, c in zip(*(rng.integers(0, m, 16) for m in (B, Nb, C))):
                ref = f64(v4(kw["x"], C)[n, b, c]).sum()
                assert abs(float(kw["s"][b, n, c]) - ref) <= tol * max(abs(ref), 1e-2 * np.abs(f64(v4(kw["x"], C)[n, b, c])).sum())
            seen.append(op)
        elif op == "add_strided":
            C = kw["y"].shape[1] // B
            n, b, c, l = pick(Nb, B, C, L)
            ref = f64(v4(kw["a"], C)[n, b, c, l]) + f64(v4(kw["b"], C)[n, b, c, l])
            rel_ok(f64(v4(kw["y"], C)[n, b, c, l]), oops.store(ref, "bf16"), 1e-6, op)
            seen.append(op)
        elif op == "maxpool_points_bwd_add":
            C = kw["dv"].shape[2]
            idx = kw["idx"].long()
            got = torch.gather(kw["dx"], 3, idx.permute(1, 0, 2).unsqueeze(3))[..., 0]       # [Nb, B, C] at the argmax
            was = torch.gather(kw["dx0"], 3, idx.permute(1, 0, 2).unsqueeze(3))[..., 0]
            ref = oops.store(f64(was) + f64(kw["dv"]).transpose(1, 0, 2), "bf16")
            assert np.abs(f64(got) - ref).max() <= 1e-6 * max(np.abs(ref).max(), 1e-30)
            # everything else is untouched: the number of changed elements is at most one per (n, b, c)
            assert int((kw["dx"] != kw["dx0"]).sum()) <= Nb * B * C
            seen.append(op)
        elif op == "conv1x1_bwd" and lay in ("head0", "conv4"):
            print("full-size check", op, lay, flush=True)
            Co = kw["dy"].shape[1] // B
            w = kw["w"].view(B, Co, -1)
            Ci = w.shape[2]
            x, dy, dx = v4(kw["x"], Ci), v4(kw["dy"], Co), v4(kw["dx"], Ci)
            # data gradient at sampled points: the oracle's backward on the gathered gradient columns, per model
            n, b, c, l = pick(Nb, B, Ci, L)
            got, cols = f64(dx[n, b, c, l]), f64(dy[n, b, :, l])                            # [S], [S, Co]
            bh, ch = b.cpu().numpy(), c.cpu().numpy()
            ref = np.empty(S)
            for bb in range(B):
                m_ = bh == bb
                if m_.any():
                    rdx, _, _ = oops.conv1x1_bwd(np.zeros((int(m_.sum()), Ci, 1)), f64(w[bb]), cols[m_][:, :, None])
                    ref[m_] = rdx[np.arange(int(m_.sum())), ch[m_], 0]
            rel_ok(got, ref, tol, f"{lay} dX")
            # weight gradient of sampled (model, output, input) channels: the full reduction over samples and points
            dw = kw["dw"].view(B, Co, Ci)
            for b_, o, c_ in zip(*(rng.integers(0, m, 16) for m in (B, Co, Ci))):
                d_, x_ = f64(dy[:, b_, o:o + 1]), f64(x[:, b_, c_:c_ + 1])                  # [Nb, 1, L] each
                _, rdw, _ = oops.conv1x1_bwd(x_, np.zeros((1, 1)), d_)
                terms = np.abs(d_ * x_).sum()
                assert abs(float(dw[b_, o, c_]) - rdw[0, 0]) <= 2e-4 * max(abs(rdw[0, 0]), 1e-2 * terms), f"{lay} dW"
            seen.append(op + lay)

    arr.forward_backward(probe)
    torch.cuda.synchronize()
    assert set(seen) == {"conv1x1_fwdconv4", "conv1x1_fwdhead0", "conv1x1_fwdhead3", "softmax_xent_points",
                         "sum_points", "add_strided", "maxpool_points_bwd_add", "conv1x1_bwdhead0", "conv1x1_bwdconv4"}
    assert np.all(np.isfinite(arr.loss.cpu().numpy()))


def test_t0_attention_full_size_sampled():
    """The attention core at the Transformer workload's size (B=8, 32 sequences of 64 tokens, width
    256, 4 heads, bf16, causal): sampled probabilities, context and gradient entries recomputed by
    their definitions from the bits the GPU read and stored."""
    from paper_2102_02344_amd import binding as hb
    B, N, S, E, H = 8, 32, 64, 256, 4
    d = E // H
    g = torch.Generator(device="cuda").manual_seed(61)
    QKV = torch.randn(B, N, S, 3 * E, device="cuda", generator=g).to(bf)
    dCTX = torch.randn(B, N, S, E, device="cuda", generator=g).to(bf)
    P = torch.empty(B, N, H, S, S, device="cuda", dtype=bf)
    CTX = torch.empty(B, N, S, E, device="cuda", dtype=bf)
    dQKV = torch.empty_like(QKV)
    ws = torch.empty(hb.attention_bwd_workspace_bytes(B, N, S, E, H, DT["bf16"]), dtype=torch.uint8, device="cuda")
    hb.attention_fwd(B, N, S, E, H, DT["bf16"], QKV, P, CTX, 1)
    hb.attention_bwd(B, N, S, E, H, DT["bf16"], QKV, P, dCTX, dQKV, ws)
    torch.cuda.synchronize()
    rng = np.random.default_rng(62)
    K_ = 400
    for b, n, h in zip(*(rng.integers(0, m, 6) for m in (B, N, H))):
        q, k, v = (f64(QKV[b, n, :, j * E + h * d:j * E + (h + 1) * d]) for j in range(3))
        sc = oops.store(q @ k.T, "bf16")
        p = oops.softmax_rows(sc, 1.0 / np.sqrt(d), True)
        gp = f64(P[b, n, h])
        rel_ok(gp, oops.store(p, "bf16"), TOL["bf16"], "P")
        assert np.all(np.triu(gp, 1) == 0.0)
        rel_ok(f64(CTX[b, n, :, h * d:(h + 1) * d]), gp @ v, TOL["bf16"], "ctx")          # from the stored probabilities
        dc = f64(dCTX[b, n, :, h * d:(h + 1) * d])
        dp = oops.store(dc @ v.T, "bf16")
        ds = oops.store(oops.softmax_rows_bwd(gp, dp, 1.0 / np.sqrt(d)), "bf16")
        rel_ok(f64(dQKV[b, n, :, h * d:(h + 1) * d]), ds @ k, TOL["bf16"], "dq")
        rel_ok(f64(dQKV[b, n, :, E + h * d:E + (h + 1) * d]), ds.T @ q, TOL["bf16"], "dk")
        rel_ok(f64(dQKV[b, n, :, 2 * E + h * d:2 * E + (h + 1) * d]), gp.T @ dc, TOL["bf16"], "dv")


def test_c1_with_transform_subnetworks_full_size():
    """Config 1 with both transform sub-networks at the benchmarked size.  With the last Linear of
    each sub-network zero the matrices are identities, so loss and the main network's gradients must
    equal the plain config 1 array bit for bit (same kernels, same inputs; the transformed tensors
    are exact copies); the sub-networks still receive finite, nonzero gradients.  One exception: the
    first layer's backward also produces a data gradient here (for the input transform), which is
    another instantiation of the kernel with another number of workgroups per model, so its weight and
    bias gradients are the same sums in another fp32 order."""
    from paper_2102_02344_amd.arrays import FusedPointNetCls, FusedPointNetClsT
    ts = hi.PointNetTSpec(cls=hi.spec_c1())
    inp = hi.pointnet_t_inputs(ts)
    n = len(ts.tnet_fc)
    for p in inp["params"]:
        for k in hi.tnet_sizes(ts):
            p[f"t{k}.fc{n}.w"][:] = 0
            p[f"t{k}.fc{n}.b"][:] = 0
    arr = FusedPointNetClsT(ts, inp)
    print("full-size check: transform array, identity matrices", flush=True)
    arr.forward_backward()
    torch.cuda.synchronize()
    plain = FusedPointNetCls(ts.cls, dict(inp, params=[{k: v for k, v in p.items() if not k.startswith("t")}
                                                       for p in inp["params"]]))
    plain.forward_backward()
    torch.cuda.synchronize()
    assert torch.equal(arr.loss, plain.loss) and bool(torch.isfinite(arr.loss).all())
    for name, _ in plain.shapes:
        if name.startswith("conv0."):
            # the first layer runs another instantiation of the backward kernel here, and its two BatchNorm-backward
            # reductions come from its own pass (its output goes through the feature transform) where the plain
            # array hands them down from the next layer's kernel: fp32 summation orders, single bf16 roundings of dz
            ga, gp = arr.g(name).double(), plain.g(name).double()
            ref = "conv0.w" if name == "conv0.b" else name       # the bias gradient is a sum of dz that cancels: no scale of its own
            assert float((ga - gp).abs().max()) <= 3e-4 * plain.g(ref).abs().max().item(), name
            continue
        assert torch.equal(arr.g(name), plain.g(name)), name
    for k in hi.tnet_sizes(ts):
        g = arr.g(f"t{k}.fc{n}.w")
        assert bool(torch.isfinite(g).all()) and float(g.abs().max()) > 0, k
