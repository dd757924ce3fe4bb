"""GPU parity: every entry point of the C ABI against the CPU oracle, element by
element, on the same seeded inputs.  Sizes span several 128x128 tiles plus a
ragged tail; both storage dtypes.  Index outputs must match bit for bit."""
import numpy as np
import pytest
import torch

import hfta_inputs as hi
from oracle import array as oa
from oracle import ops as oops
from util import DT, TDT, TOL, bn_preact_fp32, check, check_tail_argmax, conv_strides, dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hb():
    from paper_2102_02344_amd import binding
    return binding


def empty(shape, dtype):
    return torch.empty(shape, dtype=TDT[dtype] if isinstance(dtype, str) else dtype, device="cuda")


def f32_tol(dtype):
    """fp32 outputs (parameter gradients, statistics) accumulate in fp32 from exactly
    representable inputs; hold them to a tighter bound than the bf16 storage tolerance."""
    return 1e-5 if dtype == "f32" else 2e-4


# ------------------------------------------------------------------ linear
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,M,Fx,Fy", [(3, 300, 200, 260), (2, 5, 1024, 16), (1, 129, 7, 3), (4, 32, 256, 512),
                                        # many models, ragged 256x256 tiles: all three forms take the compute-bound kernel
                                        (100, 320, 264, 200), (50, 260, 136, 300),
                                        # more tiles than compute units, odd k-tile counts: the persistent form
                                        (40, 520, 520, 520), (12, 1100, 264, 1032)])
def test_linear_fwd_bwd(hb, dtype, B, M, Fx, Fy):
    print(f"linear {dtype} B={B} M={M} Fx={Fx} Fy={Fy}", flush=True)
    x = hi.normal(1, (B, M, Fx), dtype)
    w = hi.normal(2, (B, Fx, Fy), dtype, 1.0 / np.sqrt(Fx))
    b = hi.normal(3, (B, Fy), dtype)
    dy = hi.normal(4, (B, M, Fy), dtype)
    X, W, Bi, dY = dev(x, dtype), dev(w, dtype), dev(b, dtype), dev(dy, dtype)
    Y = empty((B, M, Fy), dtype)
    hb.linear_fwd(B, M, Fx, Fy, DT[dtype], X, W, Bi, Y)
    check(host(Y), oa.linear_fwd(B, x, w, b), TOL[dtype], "Y")
    # fused activation epilogue
    hb.linear_fwd(B, M, Fx, Fy, DT[dtype], X, W, Bi, Y, hb.ACT_RELU)
    check(host(Y), oops.act_fwd(oa.linear_fwd(B, x, w, b), oops.ACT_RELU), TOL[dtype], "relu(Y)")
    hb.linear_fwd(B, M, Fx, Fy, DT[dtype], X, W, None, Y, hb.ACT_GELU)
    check(host(Y), oops.act_fwd(oa.linear_fwd(B, x, w, None), oops.ACT_GELU), TOL[dtype], "gelu(Y)")
    dX = empty((B, M, Fx), dtype)
    dW = empty((B, Fx, Fy), torch.float32)
    db = empty((B, Fy), torch.float32)
    nws = hb.linear_bwd_workspace_bytes(B, M, Fx, Fy, DT[dtype])
    ws = torch.empty(max(nws, 4), dtype=torch.uint8, device="cuda")
    hb.linear_bwd(B, M, Fx, Fy, DT[dtype], X, W, dY, dX, dW, db, ws)
    rdx, rdw, rdb = oa.linear_bwd(B, x, w, dy)
    check(host(dX), rdx, TOL[dtype], "dX")
    check(host(dW), rdw, f32_tol(dtype), "dW")
    check(host(db), rdb, f32_tol(dtype), "dbias")


def test_linear_identity_and_B1(hb):
    # identity weights return X + bias exactly; B = 1 equals model 0 of a B = 2 call
    B, M, F = 2, 70, 96
    x = hi.normal(5, (B, M, F))
    w = np.stack([np.eye(F, dtype=np.float32)] * B)
    b = hi.normal(6, (B, F))
    X, W, Bi = dev(x), dev(w), dev(b)
    Y = empty((B, M, F), "f32")
    hb.linear_fwd(B, M, F, F, 0, X, W, Bi, Y)
    assert np.array_equal(host(Y), (x + b[:, None, :]).astype(np.float32).astype(np.float64))
    w2 = hi.normal(7, (B, F, F))
    W2 = dev(w2)
    hb.linear_fwd(B, M, F, F, 0, X, W2, Bi, Y)
    Y1 = empty((1, M, F), "f32")
    hb.linear_fwd(1, M, F, F, 0, X[:1].contiguous(), W2[:1].contiguous(), Bi[:1].contiguous(), Y1)
    assert torch.equal(Y1[0], Y[0])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,M,Fx,Fy,act", [(8, 32, 1024, 512, 0), (3, 32, 512, 256, 1), (2, 7, 256, 40, 0),
                                           (2, 64, 200, 130, 3), (2, 65, 256, 128, 0), (2, 4, 16, 16, 1)])
def test_linear_fwd_with_workspace(hb, dtype, B, M, Fx, Fy, act):
    """Few rows per model: the reduction is split over workgroups, the partial products are added in
    a fixed order with bias and activation; otherwise (M > 64, short K) the call is the plain forward."""
    print(f"linear_fwd_ws {dtype} B={B} M={M} Fx={Fx} Fy={Fy} act={act}", flush=True)
    x = hi.normal(41, (B, M, Fx), dtype)
    w = hi.normal(42, (B, Fx, Fy), dtype, 1.0 / np.sqrt(Fx))
    b = hi.normal(43, (B, Fy), dtype)
    X, W, Bi = dev(x, dtype), dev(w, dtype), dev(b, dtype)
    nws = hb.linear_fwd_workspace_bytes(B, M, Fx, Fy, DT[dtype])
    assert (nws > 0) == (M <= 64 and Fx >= (128 if dtype == "bf16" else 64))
    ws = torch.empty(max(nws, 4), dtype=torch.uint8, device="cuda")
    Y = empty((B, M, Fy), dtype)
    hb.linear_fwd_ws(B, M, Fx, Fy, DT[dtype], X, W, Bi, Y, act, 0.1, ws)
    ref = oops.act_fwd(oa.linear_fwd(B, x, w, b), act, 0.1)
    check(host(Y), ref, TOL[dtype], "Y")
    Y2 = empty((B, M, Fy), dtype)
    hb.linear_fwd_ws(B, M, Fx, Fy, DT[dtype], X, W, None, Y2, act, 0.1, ws)
    check(host(Y2), oops.act_fwd(oa.linear_fwd(B, x, w, None), act, 0.1), TOL[dtype], "Y without bias")
    Y3 = empty((B, M, Fy), dtype)
    hb.linear_fwd_ws(B, M, Fx, Fy, DT[dtype], X, W, Bi, Y3, act, 0.1, ws)
    assert torch.equal(Y, Y3)
    if nws > 0:
        with pytest.raises(RuntimeError):
            hb.linear_fwd_ws(B, M, Fx, Fy, DT[dtype], X, W, Bi, Y3, act, 0.1, None)


# ------------------------------------------------------------------ conv1x1
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Nb,Ci,Co,L", [(3, 2, 70, 150, 300), (2, 3, 3, 64, 250), (2, 2, 128, 40, 129),
                                          (2, 4, 64, 64, 500), (2, 3, 3, 64, 1300), (3, 2, 4, 24, 132),
                                          (2, 2, 128, 64, 260), (2, 2, 256, 520, 260), (2, 2, 520, 256, 132),
                                          (1, 2, 200, 512, 132),
                                          # more 256x256 tiles than compute units: the persistent GEMM form
                                          (3, 32, 264, 520, 520),
                                          # ... with rows of points only 8-byte aligned (8-byte loads and stores)
                                          (3, 32, 264, 520, 524)])
def test_conv1x1_fwd_bwd(hb, dtype, B, Nb, Ci, Co, L):
    print(f"conv1x1 {dtype} B={B} Nb={Nb} Ci={Ci} Co={Co} L={L}", flush=True)
    x = hi.normal(11, (Nb, B * Ci, L), dtype)
    w = hi.normal(12, (B * Co, Ci), dtype, 1.0 / np.sqrt(Ci))
    b = hi.normal(13, (B * Co,), dtype)
    dy = hi.normal(14, (Nb, B * Co, L), dtype)
    X, W, Bi, dY = dev(x, dtype), dev(w, dtype), dev(b, dtype), dev(dy, dtype)
    xs, ys = conv_strides(B, Ci, L), conv_strides(B, Co, L)
    Y = empty((Nb, B * Co, L), dtype)
    hb.conv1x1_fwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, W, Bi, Y, ys)
    check(host(Y), oa.conv1x1_fwd(B, x, w, b), TOL[dtype], "Y")
    # fused activation epilogue (select kind), with and without the bias
    hb.conv1x1_fwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, W, Bi, Y, ys, hb.ACT_LEAKY, 0.2)
    check(host(Y), oops.act_fwd(oa.conv1x1_fwd(B, x, w, b), oops.ACT_LEAKY, 0.2), TOL[dtype], "leaky(Y)")
    hb.conv1x1_fwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, W, None, Y, ys, hb.ACT_RELU)
    check(host(Y), oops.act_fwd(oa.conv1x1_fwd(B, x, w, None), oops.ACT_RELU), TOL[dtype], "relu(Y, no bias)")
    dX = empty((Nb, B * Ci, L), dtype)
    dW = empty((B * Co, Ci), torch.float32)
    db = empty((B * Co,), torch.float32)
    nws = hb.conv1x1_bwd_workspace_bytes(B, Nb, Ci, Co, L, DT[dtype])
    ws = torch.empty(max(nws, 4), dtype=torch.uint8, device="cuda")
    hb.conv1x1_bwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, W, dY, ys, dX, xs, dW, db, ws)
    rdx, rdw, rdb = oa.conv1x1_bwd(B, x, w, dy)
    check(host(dX), rdx, TOL[dtype], "dX")
    check(host(dW), rdw, f32_tol(dtype), "dW")
    check(host(db), rdb, f32_tol(dtype), "dbias")
    # bit-reproducible (fixed-order split reduction, no atomics)
    dW2 = empty((B * Co, Ci), torch.float32)
    hb.conv1x1_bwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, W, dY, ys, None, None, dW2, None, ws)
    assert torch.equal(dW, dW2)


@pytest.mark.parametrize("L", [1028, 1040])
def test_weight_gradient_split_reduction_on_large_tiles(hb, L):
    """Few large output tiles and a long reduction: the weight gradient runs split over k on the
    256x256-tile kernel (ragged Co, ragged last k-tile, splits that cross sample boundaries; rows of
    L points 8- or 16-byte aligned) and its fixed-order reduction; Linear case: one segment."""
    dtype = "bf16"
    B, Nb, Ci, Co = 3, 16, 512, 500
    print(f"conv1x1 dW large tiles B={B} Nb={Nb} Ci={Ci} Co={Co} L={L}", flush=True)
    x = hi.normal(21, (Nb, B * Ci, L), dtype)
    w = hi.normal(22, (B * Co, Ci), dtype, 1.0 / np.sqrt(Ci))
    dy = hi.normal(23, (Nb, B * Co, L), dtype)
    X, W, dY = dev(x, dtype), dev(w, dtype), dev(dy, dtype)
    xs, ys = conv_strides(B, Ci, L), conv_strides(B, Co, L)
    dW = empty((B * Co, Ci), torch.float32)
    nws = hb.conv1x1_bwd_workspace_bytes(B, Nb, Ci, Co, L, DT[dtype])
    assert nws > 0
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    hb.conv1x1_bwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, W, dY, ys, None, None, dW, None, ws)
    _, rdw, _ = oa.conv1x1_bwd(B, x, w, dy)
    check(host(dW), rdw, f32_tol(dtype), "dW")
    dW2 = empty((B * Co, Ci), torch.float32)
    hb.conv1x1_bwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, W, dY, ys, None, None, dW2, None, ws)
    assert torch.equal(dW, dW2)

    B, M, Fx, Fy = 4, 8200, 512, 760
    print(f"linear dW large tiles B={B} M={M} Fx={Fx} Fy={Fy}", flush=True)
    x = hi.normal(24, (B, M, Fx), dtype)
    w = hi.normal(25, (B, Fx, Fy), dtype, 1.0 / np.sqrt(Fx))
    dy = hi.normal(26, (B, M, Fy), dtype)
    dW = empty((B, Fx, Fy), torch.float32)
    nws = hb.linear_bwd_workspace_bytes(B, M, Fx, Fy, DT[dtype])
    assert nws > 0
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    hb.linear_bwd(B, M, Fx, Fy, DT[dtype], dev(x, dtype), dev(w, dtype), dev(dy, dtype), None, dW, None, ws)
    _, rdw, _ = oa.linear_bwd(B, x, w, dy)
    check(host(dW), rdw, f32_tol(dtype), "linear dW")


def test_conv1x1_cross_talk_and_linear_special_case(hb):
    B, Nb, Ci, Co, L = 3, 2, 32, 48, 140
    x = hi.normal(15, (Nb, B * Ci, L))
    w = hi.normal(16, (B * Co, Ci))
    X, W = dev(x), dev(w)
    xs, ys = conv_strides(B, Ci, L), conv_strides(B, Co, L)
    Y = empty((Nb, B * Co, L), "f32")
    hb.conv1x1_fwd(B, Nb, Ci, Co, L, 0, X, xs, W, None, Y, ys)
    # perturbing model 2's input and weights leaves models 0 and 1 bit-identical
    x2 = x.copy(); x2[:, 2 * Ci:] += 1.0
    w2 = w.copy(); w2[2 * Co:] *= 2.0
    Y2 = empty((Nb, B * Co, L), "f32")
    hb.conv1x1_fwd(B, Nb, Ci, Co, L, 0, dev(x2), xs, dev(w2), None, Y2, ys)
    assert torch.equal(Y[:, :2 * Co], Y2[:, :2 * Co]) and not torch.equal(Y[:, 2 * Co:], Y2[:, 2 * Co:])
    # L = 1 is the fused Linear with the weight transposed
    x1 = hi.normal(17, (Nb, B * Ci, 1))
    Yc = empty((Nb, B * Co, 1), "f32")
    hb.conv1x1_fwd(B, Nb, Ci, Co, 1, 0, dev(x1), conv_strides(B, Ci, 1), W, None, Yc, conv_strides(B, Co, 1))
    xl = np.ascontiguousarray(x1.reshape(Nb, B, Ci).transpose(1, 0, 2))
    wl = np.ascontiguousarray(w.reshape(B, Co, Ci).transpose(0, 2, 1))
    Yl = empty((B, Nb, Co), "f32")
    hb.linear_fwd(B, Nb, Ci, Co, 0, dev(xl), dev(wl), None, Yl)
    check(host(Yc).reshape(Nb, B, Co).transpose(1, 0, 2), host(Yl), 1e-6, "conv(L=1) vs linear")


# ------------------------------------------------------------------ BatchNorm
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Nb,C,L,act", [(3, 4, 5, 300, 1), (2, 3, 7, 250, 0), (2, 2, 64, 131, 2), (2, 8, 3, 1024, 1)])
def test_bn_conv_layout(hb, dtype, B, Nb, C, L, act):
    print(f"bn conv {dtype} B={B} Nb={Nb} C={C} L={L} act={act}", flush=True)
    x = hi.snap(hi.normal(21, (Nb, B * C, L)) * 2.0 + 3.0, dtype)
    g = (hi.normal(22, (B * C,)) * 0.5 + 1.0).astype(np.float32)
    bt = hi.normal(23, (B * C,)) * 0.3
    rm, rv = hi.normal(24, (B * C,)), np.abs(hi.normal(25, (B * C,))) + 0.5
    dy = hi.normal(26, (Nb, B * C, L), dtype)
    s = conv_strides(B, C, L)
    X, dY = dev(x, dtype), dev(dy, dtype)
    G, Bt, RM, RV = dev(g), dev(bt), dev(rm), dev(rv)
    SM, SI = empty((B * C,), torch.float32), empty((B * C,), torch.float32)
    Y = empty(x.shape, dtype)
    hb.bn_fwd(B, Nb, C, L, DT[dtype], X, s, G, Bt, 1e-5, 0.1, RM, RV, SM, SI, Y, s, act, 0.2)
    ry, rmean, rinv, nrm, nrv = oa.bn_fwd(B, x, g, bt, 1e-5, 0.1, rm, rv)
    oact = {0: oops.ACT_NONE, 1: oops.ACT_RELU, 2: oops.ACT_LEAKY}[act]
    check(host(Y), oops.act_fwd(ry, oact, 0.2), TOL[dtype], "Y")
    check(host(SM), rmean, 1e-5, "mean")
    check(host(SI), rinv, 1e-5, "invstd")
    check(host(RM), nrm, 1e-5, "running_mean")
    check(host(RV), nrv, 1e-5, "running_var")
    dX = empty(x.shape, dtype)
    dG, dB = empty((B * C,), torch.float32), empty((B * C,), torch.float32)
    DS = empty((B * C,), torch.float32)
    hb.bn_bwd(B, Nb, C, L, DT[dtype], X, s, dY, s, G, Bt, SM, SI, dX, s, dG, dB, act, 0.2, DS)
    # dx_sum is the per-channel sum of dX as stored (the producer layer's bias gradient)
    gdx = host(dX)
    assert np.abs(host(DS) - gdx.sum(axis=(0, 2))).max() <= 1e-5 * np.abs(gdx).sum(axis=(0, 2)).max()
    # the oracle takes the activation mask from its own float64 pre-activation; elements whose
    # pre-activation is within rounding of zero may legitimately take the other branch in fp32
    knife = np.abs(ry) < 1e-5 * (np.abs(ry - bt[None, :, None]) + np.abs(bt)[None, :, None])
    assert knife.sum() == 0, "regenerate inputs: pre-activation on the kink"
    gdy = oops.act_bwd(ry, dy, oact, 0.2)
    rdx, rdg, rdb = oa.bn_bwd(B, x, gdy, g, rmean, rinv)
    check(host(dX), rdx, TOL[dtype], "dX")
    check(host(dG), rdg, f32_tol(dtype), "dgamma")
    check(host(dB), rdb, f32_tol(dtype), "dbeta")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,Nb,Ci,Co,L,act,bias", [
    (2, 3, 64, 64, 2500, 1, True),     # config 1's middle layers: streaming kernel, ragged last slice (2500 = 19 * 128 + 68)
    (2, 2, 64, 128, 300, 2, True),     # single W tile of 128 rows
    (1, 2, 128, 320, 260, 1, False),   # three W tiles (ragged: 320 = 2 * 128 + 64), 128-deep reduction, no conv bias
    (2, 2, 24, 40, 100, 0, True),      # not the streaming kernel's shape: the two operators run one after the other
    (2, 13, 256, 264, 2500, 1, True),  # a wide layer: the persistent 256 x 256 GEMM kernel leaves the partial sums (ragged row and column tiles)
    (2, 2, 256, 264, 502, 1, True),    # rows that are only 4-byte aligned (L % 4 == 2): no vector path anywhere
])
def test_conv1x1_bn_fwd(hb, dtype, B, Nb, Ci, Co, L, act, bias):
    """Conv1d k=1 + training BatchNorm + activation in one call against the composition of the two
    single operators of the oracle (z stored and rounded, statistics of the stored z)."""
    print(f"conv1x1+bn {dtype} B={B} Nb={Nb} {Ci}->{Co} L={L} act={act} bias={bias}", flush=True)
    x = hi.normal(301, (Nb, B * Ci, L), dtype)
    w = hi.normal(302, (B * Co, Ci), dtype, 1.0 / np.sqrt(Ci))
    b = (hi.normal(303, (B * Co,), dtype) * 2.0) if bias else None      # a large bias: the statistics are shifted by it
    g = (hi.normal(304, (B * Co,)) * 0.5 + 1.0).astype(np.float32)
    bt = hi.normal(305, (B * Co,)) * 0.3
    rm, rv = hi.normal(306, (B * Co,)), np.abs(hi.normal(307, (B * Co,))) + 0.5
    xs, zs = conv_strides(B, Ci, L), conv_strides(B, Co, L)
    X, W, Bi = dev(x, dtype), dev(w, dtype), (dev(b, dtype) if bias else None)
    G, Bt, RM, RV = dev(g), dev(bt), dev(rm), dev(rv)
    SM, SI = empty((B * Co,), torch.float32), empty((B * Co,), torch.float32)
    Z, Y = empty((Nb, B * Co, L), dtype), empty((Nb, B * Co, L), dtype)
    nws = hb.conv1x1_bn_fwd_workspace_bytes(B, Nb, Ci, Co, L, DT[dtype])
    ws = torch.empty(max(nws, 8), dtype=torch.uint8, device="cuda")
    hb.conv1x1_bn_fwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, W, Bi, G, Bt, 1e-5, 0.1, RM, RV, SM, SI, Z, zs, Y, zs, act, 0.2, ws)
    rz = oa.conv1x1_fwd(B, x, w, b)
    check(host(Z), rz, TOL[dtype], "Z")
    # the BatchNorm is checked on the bits the device stored for Z (what its statistics are taken from)
    zdev = host(Z).astype(np.float64)
    ry, rmean, rinv, nrm, nrv = oa.bn_fwd(B, zdev, g, bt, 1e-5, 0.1, rm, rv)
    oact = {0: oops.ACT_NONE, 1: oops.ACT_RELU, 2: oops.ACT_LEAKY}[act]
    check(host(Y), oops.act_fwd(ry, oact, 0.2), TOL[dtype], "Y")
    check(host(SM), rmean, 1e-5, "mean")
    check(host(SI), rinv, 1e-5, "invstd")
    check(host(RM), nrm, 1e-5, "running_mean")
    check(host(RV), nrv, 1e-5, "running_var")
    # and the same call without a workspace (the two-operator path) agrees
    Z2, Y2 = empty((Nb, B * Co, L), dtype), empty((Nb, B * Co, L), dtype)
    SM2, SI2 = empty((B * Co,), torch.float32), empty((B * Co,), torch.float32)
    hb.conv1x1_bn_fwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, W, Bi, G, Bt, 1e-5, 0.1, None, None, SM2, SI2, Z2, zs, Y2, zs, act, 0.2, None)
    assert np.array_equal(host(Z2), host(Z)), "Z differs between the two paths"
    check(host(SM2), host(SM), 1e-5, "mean (two-operator path)")
    check(host(SI2), host(SI), 1e-5, "invstd (two-operator path)")
    check(host(Y2), host(Y), TOL[dtype], "Y (two-operator path)")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,Nb,Ci,Co,L,act,want_dx", [
    (2, 3, 64, 64, 2500, 1, True),     # config 1's middle layers: ragged last slice, several slices per workgroup
    (3, 2, 64, 128, 300, 2, True),     # 128 output channels (two dW tiles per wavefront)
    (2, 2, 128, 128, 644, 1, True),    # both channel tiles 128 wide
    (2, 2, 128, 64, 260, 0, True),     # 128 -> 64, no activation
    (2, 4, 3, 64, 500, 1, False),      # a network's first layer: three input channels, no data gradient
    (2, 2, 3, 64, 132, 1, True),       # ... with a data gradient (rows of W not 8-byte aligned: element loads)
    (2, 2, 24, 40, 132, 1, True),      # channel counts below the tiles (zero padding inside the kernel)
    (300, 2, 64, 64, 260, 1, True),    # many models: one workgroup per model walks all its slices
    (2, 2, 64, 200, 128, 1, True),     # not the one-pass kernel's shape: the two operators, dz in the workspace
    (2, 2, 64, 64, 130, 1, True),      # L % 4 == 2: the one-pass kernel's channel counts, but not its alignment
])
def test_conv1x1_bn_bwd(hb, dtype, B, Nb, Ci, Co, L, act, want_dx):
    """BatchNorm backward + k=1 convolution backward in one call against the oracle's chain of the two
    single operators with dz stored (rounded) in between.

    The device forms dz in fp32 and rounds it to the storage type; the oracle forms it in float64.
    The two roundings differ where the float64 value lies within the fp32 noise of dz of a bf16
    rounding boundary -- between one element in 10^4 and a few in 10^3, each by one bf16 ulp
    (2^-8..2^-7 of |dz|) -- so an element of dW, a sum of Nb * L products dz * x, can be off by a
    few ulps of its largest terms: no tighter element-wise bound than the storage type's own holds
    for it.  What the flips cannot do is move the error's root mean square: sqrt(5e-3) * 2^-8 ~ 3e-4
    of rms(dW) at most.  So dW is held element-wise to the bf16 tolerance and in rms to 3e-4 (fp32
    storage: 1e-5 element-wise); a dropped term, a wrong index or a misplaced tile is an error of
    order one in either measure."""
    print(f"conv1x1+bn bwd {dtype} B={B} Nb={Nb} {Ci}->{Co} L={L} act={act} dx={want_dx}", flush=True)
    x = hi.normal(311, (Nb, B * Ci, L), dtype)
    w = hi.normal(312, (B * Co, Ci), dtype, 1.0 / np.sqrt(Ci))
    z = hi.snap(hi.normal(313, (Nb, B * Co, L)) * 2.0 + 1.5, dtype)
    g = (hi.normal(314, (B * Co,)) * 0.5 + 1.0).astype(np.float32)
    bt = hi.normal(315, (B * Co,)) * 0.3
    dy = hi.normal(316, (Nb, B * Co, L), dtype)
    xs, zs = conv_strides(B, Ci, L), conv_strides(B, Co, L)
    # the oracle takes the activation mask from its own float64 pre-activation; an element whose
    # pre-activation is within rounding of zero may legitimately take the other branch in fp32, so
    # the few such elements of a large tensor are moved off the kink before either side sees them
    for _ in range(4):
        ry, rmean, rinv, _, _ = oa.bn_fwd(B, z, g, bt, 1e-5, 0.1, None, None)
        knife = np.abs(ry) < 1e-5 * (np.abs(ry - bt[None, :, None]) + np.abs(bt)[None, :, None])
        if act == 0 or knife.sum() == 0:
            break
        z = hi.snap(np.where(knife, z + 0.5, z), dtype)
    assert act == 0 or knife.sum() == 0, "pre-activation on the kink"
    X, W, Z, dY, G, Bt = dev(x, dtype), dev(w, dtype), dev(z, dtype), dev(dy, dtype), dev(g), dev(bt)
    SM, SI = dev(rmean.astype(np.float32)), dev(rinv.astype(np.float32))
    oact = {0: oops.ACT_NONE, 1: oops.ACT_RELU, 2: oops.ACT_LEAKY}[act]
    dX = empty((Nb, B * Ci, L), dtype) if want_dx else None
    dW, db = empty((B * Co, Ci), torch.float32), empty((B * Co,), torch.float32)
    dG, dB = empty((B * Co,), torch.float32), empty((B * Co,), torch.float32)
    nws = hb.conv1x1_bn_bwd_workspace_bytes(B, Nb, Ci, Co, L, DT[dtype])
    assert nws > 0
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    hb.conv1x1_bn_bwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, W, Z, zs, dY, zs, G, Bt, SM, SI, dX, xs if want_dx else None,
                      dW, db, dG, dB, act, 0.2, ws)
    rmean32, rinv32 = rmean.astype(np.float32).astype(np.float64), rinv.astype(np.float32).astype(np.float64)
    rdz, rdg, rdb = oa.bn_bwd(B, z, oops.act_bwd(ry, dy, oact, 0.2), g, rmean32, rinv32)
    check(host(dG), rdg, f32_tol(dtype), "dgamma")
    check(host(dB), rdb, f32_tol(dtype), "dbeta")
    dzs = oops.store(rdz, dtype)
    rdx, rdw, rdbias = oa.conv1x1_bwd(B, x, w, dzs)
    if want_dx:
        check(host(dX), rdx, TOL[dtype], "dX")
    check(host(dW), rdw, 1e-5 if dtype == "f32" else TOL[dtype], "dW")
    err = host(dW).astype(np.float64) - rdw
    assert np.sqrt(np.mean(err * err)) <= (1e-5 if dtype == "f32" else 3e-4) * np.sqrt(np.mean(rdw * rdw)), "dW (rms)"
    # dbias is a sum of terms that cancel (sum dz = 0 up to rounding): bound against the sum of magnitudes
    assert np.abs(host(db) - rdbias).max() <= f32_tol(dtype) * np.abs(dzs).sum(axis=(0, 2)).max(), "dbias"
    # bit-reproducible, and no output depends on what the workspace held before
    ws.fill_(0xff)
    dW2, db2 = empty((B * Co, Ci), torch.float32), empty((B * Co,), torch.float32)
    dX2 = empty((Nb, B * Ci, L), dtype) if want_dx else None
    hb.conv1x1_bn_bwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, W, Z, zs, dY, zs, G, Bt, SM, SI, dX2, xs if want_dx else None,
                      dW2, db2, dG, dB, act, 0.2, ws)
    assert torch.equal(dW, dW2) and torch.equal(db, db2)
    if want_dx:
        assert torch.equal(dX, dX2)
    # the block's two reductions handed in (here: its own, as dbeta and dgamma hold them) instead of taken in a
    # pass over dY and Z: the same constants, hence the same bits everywhere
    S = torch.stack([dB, dG], dim=1).contiguous()
    dG3, dB3 = empty((B * Co,), torch.float32), empty((B * Co,), torch.float32)
    hb.conv1x1_bn_bwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, W, Z, zs, dY, zs, G, Bt, SM, SI, dX2, xs if want_dx else None,
                      dW2, db2, dG3, dB3, act, 0.2, ws, sums=S)
    assert torch.equal(dW, dW2) and torch.equal(db, db2) and torch.equal(dG, dG3) and torch.equal(dB, dB3)
    if want_dx:
        assert torch.equal(dX, dX2)
    with pytest.raises(RuntimeError):
        hb.conv1x1_bn_bwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, W, Z, zs, dY, zs, G, Bt, SM, SI, dX2, xs if want_dx else None,
                          dW2, db2, dG, dB, act, 0.2, None)


@pytest.mark.parametrize("B,Nb,Ci,Co,L,in_act,act,want_y", [
    (2, 3, 64, 64, 2500, 1, 1, False),   # config 1's middle layers: ragged last slice, activated output not formed
    (3, 2, 64, 128, 300, 1, 1, True),    # 64 -> 128 with the activated output stored (what feeds the one-operator tail)
    (2, 2, 128, 128, 644, 2, 0, False),  # 128-deep reduction, LeakyReLU on the input block, none on this one
    (2, 2, 24, 72, 132, 0, 2, True),     # channel counts below the tiles, no activation on the input block
    (2, 3, 32, 64, 260, 2, 1, False),    # LeakyReLU on the input block where its sums are handed down
])
def test_conv1x1_bn_prenorm(hb, B, Nb, Ci, Co, L, in_act, act, want_y):
    """A chain of conv -> BatchNorm -> act blocks in which the activated tensor between two blocks is never
    stored: the second block takes the first one's stored pre-activation and BatchNorm constants and forms
    its input on load.  Forward and backward must equal, bit for bit, the plain pair of calls on the stored
    activated tensor (same arithmetic, same kernels), and the forward is checked against the oracle's chain."""
    dtype = "bf16"
    print(f"conv1x1+bn prenorm B={B} Nb={Nb} {Ci}->{Co} L={L} in_act={in_act} act={act} y={want_y}", flush=True)
    assert hb.conv1x1_bn_prenorm_supported(B, Nb, Ci, Co, L, DT[dtype])
    xpre = hi.snap(hi.normal(321, (Nb, B * Ci, L)) * 1.5 + 0.4, dtype)
    gi = (hi.normal(322, (B * Ci,)) * 0.5 + 1.0).astype(np.float32)
    bi = (hi.normal(323, (B * Ci,)) * 0.3).astype(np.float32)
    w = hi.normal(324, (B * Co, Ci), dtype, 1.0 / np.sqrt(Ci))
    b = hi.normal(325, (B * Co,), dtype)
    g = (hi.normal(326, (B * Co,)) * 0.5 + 1.0).astype(np.float32)
    bt = (hi.normal(327, (B * Co,)) * 0.3).astype(np.float32)
    dy = hi.normal(328, (Nb, B * Co, L), dtype)
    xs, zs = conv_strides(B, Ci, L), conv_strides(B, Co, L)
    Xp, Gi, Bi, W, Bs, G, Bt, dY = dev(xpre, dtype), dev(gi), dev(bi), dev(w, dtype), dev(b, dtype), dev(g), dev(bt), dev(dy, dtype)
    f32 = torch.float32
    # the input block's BatchNorm on the device: its statistics, and (for the plain pair) its stored output
    MI, II, X = empty((B * Ci,), f32), empty((B * Ci,), f32), empty((Nb, B * Ci, L), dtype)
    hb.bn_fwd(B, Nb, Ci, L, DT[dtype], Xp, xs, Gi, Bi, 1e-5, 0.1, None, None, MI, II, X, xs, in_act, 0.2)
    nws = max(hb.conv1x1_bn_fwd_workspace_bytes(B, Nb, Ci, Co, L, DT[dtype]), hb.conv1x1_bn_bwd_workspace_bytes(B, Nb, Ci, Co, L, DT[dtype]))
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    out = {}
    for kind in ("plain", "prenorm"):
        Z, Y = empty((Nb, B * Co, L), dtype), (empty((Nb, B * Co, L), dtype) if want_y else None)
        SM, SI = empty((B * Co,), f32), empty((B * Co,), f32)
        RM, RV = dev(np.zeros(B * Co, np.float32)), dev(np.ones(B * Co, np.float32))
        dX, dW, db = empty((Nb, B * Ci, L), dtype), empty((B * Co, Ci), f32), empty((B * Co,), f32)
        dG, dB = empty((B * Co,), f32), empty((B * Co,), f32)
        ws.fill_(0x5a)
        if kind == "plain":
            hb.conv1x1_bn_fwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, W, Bs, G, Bt, 1e-5, 0.1, RM, RV, SM, SI, Z, zs, Y,
                              zs if want_y else None, act, 0.2, ws)
            hb.conv1x1_bn_bwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, W, Z, zs, dY, zs, G, Bt, SM, SI, dX, xs, dW, db, dG, dB, act, 0.2, ws)
        else:
            hb.conv1x1_bn_prenorm_fwd(B, Nb, Ci, Co, L, DT[dtype], Xp, xs, Gi, Bi, MI, II, in_act, 0.2, W, Bs, G, Bt, 1e-5, 0.1,
                                      RM, RV, SM, SI, Z, zs, Y, zs if want_y else None, act, 0.2, ws)
            hb.conv1x1_bn_prenorm_bwd(B, Nb, Ci, Co, L, DT[dtype], Xp, xs, Gi, Bi, MI, II, in_act, 0.2, W, Z, zs, dY, zs, G, Bt,
                                      SM, SI, dX, xs, dW, db, dG, dB, act, 0.2, ws)
        out[kind] = dict(Z=Z, Y=Y, SM=SM, SI=SI, RM=RM, RV=RV, dX=dX, dW=dW, db=db, dG=dG, dB=dB)
    for k, v in out["plain"].items():
        if v is not None:
            assert torch.equal(v, out["prenorm"][k]), f"{k} differs from the plain pair on the stored activated tensor"
    # against the oracle: its own chain with the activated tensor stored (rounded) in between
    oin = {0: oops.ACT_NONE, 1: oops.ACT_RELU, 2: oops.ACT_LEAKY}[in_act]
    ry_in = oa.bn_fwd(B, xpre, gi, bi, 1e-5, 0.1, None, None)[0]
    xo = oops.store(oops.act_fwd(ry_in, oin, 0.2), dtype)
    check(host(X), xo, TOL[dtype], "input block's activated tensor")
    rz = oa.conv1x1_fwd(B, host(X).astype(np.float64), w, b)      # on the bits the device formed on load (equal to X, shown above)
    check(host(out["prenorm"]["Z"]), rz, TOL[dtype], "Z")
    zdev = host(out["prenorm"]["Z"]).astype(np.float64)
    ry, rmean, rinv, _, _ = oa.bn_fwd(B, zdev, g, bt, 1e-5, 0.1, None, None)
    check(host(out["prenorm"]["SM"]), rmean, 1e-5, "mean")
    check(host(out["prenorm"]["SI"]), rinv, 1e-5, "invstd")
    if want_y:
        oact = {0: oops.ACT_NONE, 1: oops.ACT_RELU, 2: oops.ACT_LEAKY}[act]
        check(host(out["prenorm"]["Y"]), oops.act_fwd(ry, oact, 0.2), TOL[dtype], "Y")
    # the backward call also leaves the input block's two reductions (sum g, sum g xhat over dX as stored and
    # the input block's pre-activation) where the kernel has room for them: nothing else changes by a bit, and
    # the sums are those of the oracle's BatchNorm backward of that block on the device's dX
    assert hb.conv1x1_bn_prenorm_bwd_gives_sums(B, Nb, Ci, Co, L, DT[dtype]) == (Ci <= 64)
    S = torch.full((B * Ci, 2), float("nan"), dtype=f32, device="cuda")
    if Ci <= 64:
        pz = out["prenorm"]
        dX, dW, db = empty((Nb, B * Ci, L), dtype), empty((B * Co, Ci), f32), empty((B * Co,), f32)
        dG, dB = empty((B * Co,), f32), empty((B * Co,), f32)
        ws.fill_(0xa5)
        hb.conv1x1_bn_prenorm_bwd(B, Nb, Ci, Co, L, DT[dtype], Xp, xs, Gi, Bi, MI, II, in_act, 0.2, W, pz["Z"], zs, dY, zs, G, Bt,
                                  pz["SM"], pz["SI"], dX, xs, dW, db, dG, dB, act, 0.2, ws, in_sums=S)
        for k, v in dict(dX=dX, dW=dW, db=db, dG=dG, dB=dB).items():
            assert torch.equal(v, pz[k]), f"{k} changes when the input block's sums are asked for"
        mi, ii = host(MI).astype(np.float64), host(II).astype(np.float64)
        pre = bn_preact_fp32(xpre, gi, bi, mi, ii)             # the mask in the kernels' precision
        gr = oops.act_bwd(pre, host(dX).astype(np.float64), oin, 0.2)
        _, rdg, rdb = oa.bn_bwd(B, xpre, gr, gi, mi, ii)
        check(host(S)[:, 0], rdb, f32_tol(dtype), "input block's sum g")
        check(host(S)[:, 1], rdg, f32_tol(dtype), "input block's sum g xhat")
    else:
        with pytest.raises(RuntimeError):
            hb.conv1x1_bn_prenorm_bwd(B, Nb, Ci, Co, L, DT[dtype], Xp, xs, Gi, Bi, MI, II, in_act, 0.2, W, out["prenorm"]["Z"], zs,
                                      dY, zs, G, Bt, out["prenorm"]["SM"], out["prenorm"]["SI"], out["prenorm"]["dX"], xs,
                                      out["prenorm"]["dW"], out["prenorm"]["db"], out["prenorm"]["dG"], out["prenorm"]["dB"],
                                      act, 0.2, ws, in_sums=S)
    # an input the kernels do not take comes back as a status code with nothing launched
    with pytest.raises(RuntimeError):
        hb.conv1x1_bn_prenorm_fwd(B, Nb, Ci, Co, L, DT["f32"], Xp, xs, Gi, Bi, MI, II, in_act, 0.2, W, Bs, G, Bt, 1e-5, 0.1,
                                  None, None, SM, SI, Z, zs, None, None, act, 0.2, ws)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("Nb", [32, 5, 64, 100])      # up to 64 samples: the column-in-registers kernels
def test_bn_linear_layout_and_independence(hb, dtype, Nb):
    B, C = 3, 300
    x = hi.snap(hi.normal(31, (B, Nb, C)) * 1.5 - 0.7, dtype)
    g, bt = (hi.normal(32, (B, C)) * 0.5 + 1.0), hi.normal(33, (B, C)) * 0.3
    dy = hi.normal(34, (B, Nb, C), dtype)
    s = (Nb * C, C, 1, 1)
    X, dY, G, Bt = dev(x, dtype), dev(dy, dtype), dev(g), dev(bt)
    SM, SI = empty((B, C), torch.float32), empty((B, C), torch.float32)
    Y = empty(x.shape, dtype)
    hb.bn_fwd(B, Nb, C, 1, DT[dtype], X, s, G, Bt, 1e-5, 0.1, None, None, SM, SI, Y, s, hb.ACT_RELU, 0.0)
    ry, rmean, rinv, _, _ = oa.bn_fwd(B, x, g, bt, 1e-5, 0.1, None, None, "linear")
    check(host(Y), oops.act_fwd(ry, oops.ACT_RELU), TOL[dtype], "Y")
    check(host(SM).reshape(-1), rmean, 1e-5, "mean")
    dX = empty(x.shape, dtype)
    dG, dB = empty((B, C), torch.float32), empty((B, C), torch.float32)
    DS = empty((B, C), torch.float32)
    hb.bn_bwd(B, Nb, C, 1, DT[dtype], X, s, dY, s, G, Bt, SM, SI, dX, s, dG, dB, hb.ACT_RELU, 0.0, DS)
    assert np.abs(host(DS) - host(dX).sum(axis=1)).max() <= 1e-5 * np.abs(host(dX)).sum(axis=1).max()
    rdx, rdg, rdb = oa.bn_bwd(B, x, oops.act_bwd(ry, dy, oops.ACT_RELU), g, rmean, rinv, "linear")
    check(host(dX), rdx, TOL[dtype], "dX")
    check(host(dG).reshape(-1), rdg, f32_tol(dtype), "dgamma")
    check(host(dB).reshape(-1), rdb, f32_tol(dtype), "dbeta")
    # models never share statistics: changing model 1's data leaves models 0 and 2 bit-identical
    x2 = x.copy(); x2[1] = x2[1] * 2 + 1
    Y2 = empty(x.shape, dtype)
    hb.bn_fwd(B, Nb, C, 1, DT[dtype], dev(hi.snap(x2, dtype), dtype), s, G, Bt, 1e-5, 0.1, None, None, SM, SI, Y2, s,
              hb.ACT_RELU, 0.0)
    assert torch.equal(Y[0], Y2[0]) and torch.equal(Y[2], Y2[2]) and not torch.equal(Y[1], Y2[1])


def test_bn_invariants_large_mean(hb):
    # |mean| >> std: the shifted sums must keep fp32 accuracy; mean(y) = beta, var(y) = gamma^2 var/(var+eps)
    B, Nb, C, L = 2, 4, 3, 1000
    x = (hi.normal(35, (Nb, B * C, L)) * 0.01 + 100.0).astype(np.float32)
    g, bt = np.full(B * C, 2.0, np.float32), np.full(B * C, 0.5, np.float32)
    s = conv_strides(B, C, L)
    SM, SI = empty((B * C,), torch.float32), empty((B * C,), torch.float32)
    Y = empty(x.shape, "f32")
    hb.bn_fwd(B, Nb, C, L, 0, dev(x), s, dev(g), dev(bt), 1e-5, 0.1, None, None, SM, SI, Y, s)
    ry, rmean, rinv, _, _ = oa.bn_fwd(B, x, g, bt, 1e-5)
    check(host(SM), rmean, 1e-6, "mean")
    check(host(SI), rinv, 1e-4, "invstd")
    y = host(Y)
    assert np.abs(y.mean(axis=(0, 2)) - 0.5).max() < 1e-3


# ------------------------------------------------------------------ point max-pool
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Nb,C,L", [(2, 3, 50, 2500), (3, 2, 7, 250), (1, 1, 5, 3), (2, 2, 33, 64)])
def test_maxpool_points(hb, dtype, B, Nb, C, L):
    print(f"maxpool {dtype} B={B} Nb={Nb} C={C} L={L}", flush=True)
    x = hi.normal(41, (Nb, B * C, L), dtype)
    x = np.maximum(x, 0.0)                     # post-ReLU: many exact ties at zero
    x[0, 0, :] = 0.0                           # all-equal row -> index 0
    if L > 2:
        x[0, 1, :] = -1.0; x[0, 1, 1] = 3.0; x[0, 1, L - 1] = 3.0   # first of equal maxima wins
    X = dev(x, dtype)
    xs = conv_strides(B, C, L)
    # result lands directly in the linear layout [B][Nb][C]
    vs = (Nb * C, C, 1)
    V, I = empty((B, Nb, C), dtype), empty((B, Nb, C), torch.int32)
    hb.maxpool_points(B, Nb, C, L, DT[dtype], X, xs, V, I, vs)
    rv, ri = oa.maxpool_points_fwd(B, x)
    rv = rv.reshape(Nb, B, C).transpose(1, 0, 2)
    ri = ri.reshape(Nb, B, C).transpose(1, 0, 2)
    assert np.array_equal(I.cpu().numpy(), ri)             # bit-exact indices
    assert np.array_equal(host(V), rv)                     # values are copies
    assert I[0, 0, 0].item() == 0
    dv = hi.normal(42, (B, Nb, C), dtype)
    dX = empty(x.shape, dtype)
    hb.maxpool_points_bwd(B, Nb, C, L, DT[dtype], dev(dv, dtype), I, vs, dX, xs)
    rdx = oa.maxpool_points_bwd(B, dv.transpose(1, 0, 2).reshape(Nb, B * C), ri.transpose(1, 0, 2).reshape(Nb, B * C), L)
    assert np.array_equal(host(dX), rdx)


# ------------------------------------------------------------------ Adam
@pytest.mark.parametrize("gdtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,P", [(3, 4096 + 8), (2, 1023), (8, 100_000)])
def test_adam(hb, gdtype, B, P):
    hp = hi.adam_hparams(51, B)
    th = hi.normal(52, (B, P)) * 0.1
    m, v = np.zeros((B, P), np.float32), np.zeros((B, P), np.float32)
    TH, M_, V_ = dev(th), dev(m), dev(v)
    LP = empty((B, P), torch.bfloat16)
    H = {k: dev(a) for k, a in hp.items()}
    for dec in (0, 1):
        th_r, m_r, v_r = th.copy(), m.copy(), v.copy()
        TH.copy_(dev(th)); M_.zero_(); V_.zero_()
        for t in range(1, 4):
            g = hi.normal(60 + t, (B, P), gdtype)
            hb.adam_step(B, P, DT[gdtype], TH, dev(g, gdtype), M_, V_, LP, H["lr"], H["beta1"], H["beta2"], H["eps"],
                         H["wd"], t, dec)
            th_r, m_r, v_r = oa.adam_step(B, th_r, g, m_r, v_r, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"],
                                          hp["wd"], t, bool(dec))
        check(host(TH), th_r, 1e-5, "theta")
        check(host(M_), m_r, 1e-5, "m")
        check(host(V_), v_r, 1e-5, "v")
        assert torch.equal(LP, TH.to(torch.bfloat16))      # the low-precision copy is RNE of the new theta


def test_adam_closed_form_and_routing(hb):
    B, P = 3, 1000
    th0 = hi.normal(53, (B, P))
    g = hi.normal(54, (B, P))
    lr = np.array([1e-2, 0.0, 1e-3], np.float32)
    z = np.zeros(B, np.float32)
    TH, M_, V_ = dev(th0), dev(np.zeros((B, P), np.float32)), dev(np.zeros((B, P), np.float32))
    G = dev(g)
    b1, b2, eps = dev(np.full(B, 0.8, np.float32)), dev(np.full(B, 0.95, np.float32)), dev(np.full(B, 1e-8, np.float32))
    for t in range(1, 6):
        hb.adam_step(B, P, 0, TH, G, M_, V_, None, dev(lr), b1, b2, eps, dev(z), t)
    th = host(TH)
    # constant gradient: theta_t = theta_0 - t lr g/(|g| + eps); lr = 0 leaves model 1 bit-unchanged
    assert np.array_equal(th[1], th0[1].astype(np.float64))
    for b in (0, 2):
        ref = th0[b] - 5 * lr[b] * g[b] / (np.abs(g[b]) + 1e-8)
        assert np.abs(th[b] - ref).max() < 2e-6


@pytest.mark.parametrize("gdtype,segs", [("f32", (0, 12, 40, 1064)), ("bf16", (0, 5, 31, 1000))])
def test_adadelta_arena_and_steplr(hb, gdtype, segs):
    """Adadelta over a parameter-major arena with per-model lr / rho / eps / weight decay (one
    launch for all models; the second segment table has sizes that are not multiples of 4), its
    learning rates produced on the device by the per-model step schedule."""
    B, P = 3, segs[-1]
    rng = np.random.default_rng(91)
    base = np.array([1.0, 0.5, 0.0], np.float32)          # model 2: lr = 0, parameters must not move
    gam = np.array([0.5, 0.1, 0.9], np.float32)
    step = np.array([1, 2, 3], np.int32)
    rho = np.array([0.9, 0.8, 0.95], np.float32)
    eps = np.array([1e-6, 1e-5, 1e-6], np.float32)
    wd = np.array([0.0, 0.05, 0.1], np.float32)
    # arena layout: segment j holds [B][n_j]
    def to_arena(a):                                       # [B, P] -> flat parameter-major
        return np.concatenate([a[:, segs[j]:segs[j + 1]].reshape(-1) for j in range(len(segs) - 1)])
    def from_arena(f):
        out = np.empty((B, P), np.float64)
        o = 0
        for j in range(len(segs) - 1):
            n = segs[j + 1] - segs[j]
            out[:, segs[j]:segs[j + 1]] = f[o:o + B * n].reshape(B, n)
            o += B * n
        return out
    th = (hi.normal(92, (B, P)) * 0.1).astype(np.float32)
    TH = dev(to_arena(th))
    V_, U_ = dev(np.zeros(B * P, np.float32)), dev(np.zeros(B * P, np.float32))
    LP = empty((B * P,), torch.bfloat16)
    LR = empty((B,), torch.float32)
    Hd = {k: dev(a) for k, a in dict(base=base, gam=gam, rho=rho, eps=eps, wd=wd).items()}
    STEP = torch.from_numpy(step).cuda()
    th_r, v_r, u_r = th.astype(np.float64), np.zeros((B, P)), np.zeros((B, P))
    for epoch in range(4):
        hb.steplr(B, Hd["base"], Hd["gam"], STEP, epoch, LR)
        lr_r = oops.steplr(base, gam, step, epoch)
        assert np.abs(host(LR) - lr_r).max() <= 1e-6 * max(lr_r.max(), 1e-30)
        g = hi.normal(100 + epoch, (B, P), gdtype)
        hb.adadelta_step_multi(B, list(segs), DT[gdtype], TH, dev(to_arena(g), gdtype), V_, U_, LP, LR, Hd["rho"],
                               Hd["eps"], Hd["wd"])
        th_r, v_r, u_r = oa.adadelta_step(B, th_r, g, v_r, u_r, host(LR), rho, eps, wd)
    check(from_arena(host(TH)), th_r, 1e-5, "theta")
    check(from_arena(host(V_)), v_r, 1e-5, "square_avg")
    check(from_arena(host(U_)), u_r, 2e-5, "acc_delta")
    assert np.array_equal(from_arena(host(TH))[2], th[2].astype(np.float64))     # lr = 0
    assert torch.equal(LP, TH.to(torch.bfloat16))


# ------------------------------------------------------------------ support ops
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_activations_dropout(hb, dtype):
    n = 10_007
    x = hi.normal(71, (n,), dtype)
    x[np.abs(x) < 1e-3] = 0.25
    dy = hi.normal(72, (n,), dtype)
    X, dY = dev(x, dtype), dev(dy, dtype)
    Y, dX = empty((n,), dtype), empty((n,), dtype)
    for act, oact in ((hb.ACT_RELU, oops.ACT_RELU), (hb.ACT_LEAKY, oops.ACT_LEAKY), (hb.ACT_TANH, oops.ACT_TANH),
                      (hb.ACT_GELU, oops.ACT_GELU)):
        hb.act_fwd(n, DT[dtype], X, Y, act, 0.2)
        check(host(Y), oops.act_fwd(x, oact, 0.2), TOL[dtype], f"act{act}")
        hb.act_bwd(n, DT[dtype], X, dY, dX, act, 0.2, 0)
        check(host(dX), oops.act_bwd(x, dy, oact, 0.2), TOL[dtype], f"dact{act}")
        if act != hb.ACT_GELU:
            yst = host(Y)
            hb.act_bwd(n, DT[dtype], Y, dY, dX, act, 0.2, 1)
            ref = oops.act_bwd(x, dy, oact, 0.2) if act != hb.ACT_TANH else dy * (1 - yst * yst)
            check(host(dX), ref, TOL[dtype], f"dact{act} from output")
    mask = (np.random.default_rng(73).random(n) > 0.3).astype(np.uint8)
    hb.dropout(n, DT[dtype], X, dev(mask), 0.3, Y)
    check(host(Y), oops.dropout_fwd(x, mask, 0.3), TOL[dtype], "dropout")
    # per-channel bias + activation in place on an [Nb][K][HW] tensor
    Nb, K, HW = 3, 10, 37
    t = hi.normal(74, (Nb, K, HW), dtype)
    bias = hi.normal(75, (K,), dtype)
    Tt = dev(t, dtype)
    hb.bias_act_nchw(Nb, K, HW, DT[dtype], Tt, dev(bias, dtype), hb.ACT_TANH, 0.0)
    check(host(Tt), np.tanh(t.astype(np.float64) + bias[None, :, None]), TOL[dtype], "bias_act")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,R,E", [(3, 200, 512), (2, 7, 100), (2, 300, 1016)])
def test_layernorm(hb, dtype, B, R, E):
    x = hi.snap(hi.normal(81, (B, R, E)) * 2 + 0.5, dtype)
    w, b = hi.normal(82, (B, E)) * 0.5 + 1.0, hi.normal(83, (B, E)) * 0.2
    dy = hi.normal(84, (B, R, E), dtype)
    X, dY, Wt, Bt = dev(x, dtype), dev(dy, dtype), dev(w), dev(b)
    SM, SI = empty((B, R), torch.float32), empty((B, R), torch.float32)
    Y = empty(x.shape, dtype)
    hb.layernorm_fwd(B, R, E, DT[dtype], X, Wt, Bt, 1e-5, SM, SI, Y)
    ry, rmean, rinv = oa.layernorm_fwd(B, x, w, b, 1e-5)
    check(host(Y), ry, TOL[dtype], "Y")
    check(host(SM), rmean, 1e-5, "mean")
    dX = empty(x.shape, dtype)
    dw, db = empty((B, E), torch.float32), empty((B, E), torch.float32)
    ws = torch.empty(hb.layernorm_bwd_workspace_bytes(B, R, E), dtype=torch.uint8, device="cuda")
    hb.layernorm_bwd(B, R, E, DT[dtype], X, dY, Wt, SM, SI, dX, dw, db, ws)
    rdx, rdw, rdb = oa.layernorm_bwd(B, x, dy, w, rmean, rinv)
    check(host(dX), rdx, TOL[dtype], "dX")
    check(host(dw), rdw, f32_tol(dtype), "dw")
    check(host(db), rdb, f32_tol(dtype), "db")
    # the residual-block form: gradient given as a pair summed on load, column sums of dX on the side
    ws = torch.empty(hb.layernorm_bwd_sums_workspace_bytes(B, R, E), dtype=torch.uint8, device="cuda")
    dy2 = hi.normal(85, (B, R, E), dtype)
    dxs = empty((B, E), torch.float32)
    epv = 8 if dtype == "bf16" else 4
    if E % epv != 0 or E // epv > 128:         # not a row of at most 128 whole 16-byte pieces: unsupported
        with pytest.raises(RuntimeError):
            hb.layernorm_bwd_sums(B, R, E, DT[dtype], X, dY, dev(dy2, dtype), Wt, SM, SI, dX, dw, db, dxs, ws)
        return
    for second in (dy2, None):
        hb.layernorm_bwd_sums(B, R, E, DT[dtype], X, dY, None if second is None else dev(second, dtype), Wt, SM, SI, dX, dw,
                              db, dxs, ws)
        dsum = dy if second is None else oops.store(dy.astype(np.float64) + second, dtype)
        rdx, rdw, rdb = oa.layernorm_bwd(B, x, dsum, w, rmean, rinv)
        check(host(dX), rdx, TOL[dtype], "dX (sums)")
        check(host(dw), rdw, f32_tol(dtype), "dw (sums)")
        check(host(db), rdb, f32_tol(dtype), "db (sums)")
        check(host(dxs), host(dX).astype(np.float64).sum(axis=1), f32_tol(dtype), "column sums of the stored dX")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,M,F,act", [(3, 200, 264, "GELU"), (2, 70, 4104, "RELU"), (2, 1, 8, "TANH"), (1, 4100, 128, "LEAKY"),
                                       # many models: the one-pass form (at least 128 workgroups)
                                       (16, 70, 1024, "GELU"), (40, 133, 520, "RELU"), (130, 65, 8, "LEAKY")])
def test_act_bwd_with_bias_gradient(hb, dtype, B, M, F, act):
    """Activation backward fused with the column sums of its result = the two separate operators."""
    print(f"act_bwd_colsum {dtype} B={B} M={M} F={F} {act}", flush=True)
    a, oa_act = getattr(hb, "ACT_" + act), getattr(oops, "ACT_" + act)
    z, dy = hi.normal(61, (B, M, F), dtype), hi.normal(62, (B, M, F), dtype)
    dx, db = empty((B, M, F), dtype), empty((B, F), torch.float32)
    hb.act_bwd_colsum(B, M, F, DT[dtype], dev(z, dtype), dev(dy, dtype), dx, db, a, 0.2)
    rdx = oops.act_bwd(z, dy, oa_act, 0.2)
    check(host(dx), rdx, TOL[dtype], "dx")
    # the sums are of the values as stored
    stored = host(dx).astype(np.float64)
    check(host(db), stored.sum(axis=1), f32_tol(dtype), "dbias vs stored dx")
    check(host(db), oops.store(rdx, dtype).sum(axis=1), 5 * TOL[dtype], "dbias vs oracle")
    if F % 8 == 0 and dtype == "bf16":
        with pytest.raises(RuntimeError):            # 100 columns: no whole 16-byte pieces
            hb.act_bwd_colsum(B, M, 100, DT[dtype], dev(z, dtype), dev(dy, dtype), dx, db, a, 0.2)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_losses(hb, dtype):
    B, R, K = 3, 77, 16
    z = hi.normal(91, (B, R, K), dtype) * 2
    lab = np.random.default_rng(92).integers(0, K, (B, R)).astype(np.int32)
    loss, dz = empty((B,), torch.float32), empty((B, R, K), dtype)
    hb.softmax_xent(B, R, K, DT[dtype], dev(z, dtype), dev(lab), loss, dz)
    rl, rdz = oa.softmax_xent(B, z, lab)
    check(host(loss), rl, 1e-5, "xent loss")
    check(host(dz), rdz, TOL[dtype], "dlogits")
    R2 = 5000
    p, t = hi.normal(93, (B, R2), dtype), hi.normal(94, (B, R2), dtype)
    dp = empty((B, R2), dtype)
    hb.mse(B, R2, DT[dtype], dev(p, dtype), dev(t, dtype), loss, dp)
    rl, rdp = oa.mse(B, p, t)
    check(host(loss), rl, 1e-5, "mse loss")
    check(host(dp), rdp, TOL[dtype], "dpred")
    tb = (np.random.default_rng(95).random((B, R2)) > 0.5).astype(np.float32)
    hb.bce_logits(B, R2, DT[dtype], dev(p, dtype), dev(tb, dtype), loss, dp)
    rl, rdp = oa.bce_logits(B, p, tb)
    check(host(loss), rl, 1e-5, "bce loss")
    check(host(dp), rdp, TOL[dtype], "dlogits(bce)")
    # long contiguous rows: full-width gradient launch + one-workgroup loss sum per model
    R3 = 65536 + 24
    p, t = hi.normal(96, (B, R3), dtype), hi.normal(97, (B, R3), dtype)
    dp = empty((B, R3), dtype)
    hb.mse(B, R3, DT[dtype], dev(p, dtype), dev(t, dtype), loss, dp)
    rl, rdp = oa.mse(B, p, t)
    check(host(loss), rl, 1e-5, "mse loss (long rows)")
    check(host(dp), rdp, TOL[dtype], "dpred (long rows)")
    tb = (np.random.default_rng(98).random((B, R3)) > 0.5).astype(np.float32)
    hb.bce_logits(B, R3, DT[dtype], dev(p, dtype), dev(tb, dtype), loss, dp)
    rl, rdp = oa.bce_logits(B, p, tb)
    check(host(loss), rl, 1e-5, "bce loss (long rows)")
    check(host(dp), rdp, TOL[dtype], "dlogits(bce, long rows)")


# ------------------------------------------------------------------ grouped Conv2d / ConvTranspose2d
CONV_CASES = [
    # B, Nb, Ci, Co, H, k, s, p
    (3, 2, 5, 7, 12, 4, 2, 1),      # ragged channels
    (2, 2, 3, 64, 16, 4, 2, 1),     # first discriminator layer shape (3 -> 64)
    (2, 3, 16, 130, 32, 4, 2, 1),   # two row tiles, two pixel tiles
    (2, 4, 64, 1, 4, 4, 1, 0),      # last discriminator layer: 4x4 -> 1x1
    (2, 2, 6, 9, 9, 3, 1, 1),       # generic 3x3
    (1, 1, 8, 8, 10, 1, 1, 0),      # k = 1
    (2, 2, 32, 24, 32, 4, 2, 1),    # data gradient on the parity-class kernel (16x16 outputs, >= 32 channels); regrouped weights
    (1, 2, 40, 10, 34, 4, 2, 1),    # the same with a 17-wide class grid (no 4-pixel pieces)
    (1, 2, 32, 9, 32, 4, 2, 1),     # the same with K = 36: weights gathered tap by tap
    (2, 5, 32, 100, 4, 4, 1, 0),    # generator's first layer seen as a convolution: whole-image window, batched-GEMM path
    (2, 3, 5, 3, 3, 3, 1, 0),       # whole-image window with K = 45 (no 16-byte pieces)
    (2, 3, 264, 40, 8, 4, 2, 1),    # 4x4 outputs: 8 samples per column tile, ragged sample tail; forward reduction (K = 4224) split four ways
    (1, 5, 40, 48, 8, 4, 2, 1),     # weight gradient with two 4x4 samples per k-tile and an odd number of samples
    (1, 3, 16, 300, 16, 4, 2, 1),   # forward on 128-row tiles, two 8x8 samples per column tile, ragged rows and samples
    (1, 2, 32, 512, 8, 4, 2, 1),    # data gradient with a long reduction (K = 2048) on 64-row class-pair tiles
    (2, 2, 3, 20, 80, 4, 2, 1),     # few-channel data gradient: 40x40 q grid (ragged 32x8 tiles), Co not a multiple of 8
    (1, 3, 1, 9, 12, 4, 2, 1),      # the same with one channel and a q grid smaller than a tile
]


def conv_workspaces(hb, path, args):
    """(forward workspace, backward workspace) that select the implicit-GEMM kernels or the
    column-buffer lowering onto the batched GEMM kernels."""
    if path == "implicit":
        n = hb.conv2d_grouped_bwd_min_workspace_bytes(*args)
        return None, (torch.empty(n, dtype=torch.uint8, device="cuda") if n else None)
    nf, nb = hb.conv2d_grouped_fwd_workspace_bytes(*args), hb.conv2d_grouped_bwd_workspace_bytes(*args)
    return (torch.empty(max(nf, 4), dtype=torch.uint8, device="cuda"),
            torch.empty(max(nb, 4), dtype=torch.uint8, device="cuda"))


@pytest.mark.parametrize("path", ["implicit", "lowered"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Nb,Ci,Co,H,k,s,p", CONV_CASES)
def test_conv2d_grouped(hb, dtype, B, Nb, Ci, Co, H, k, s, p, path):
    print(f"conv2d {path} {dtype} B={B} Nb={Nb} Ci={Ci} Co={Co} H={H} k={k} s={s} p={p}", flush=True)
    Wd = H + 2 if k > 1 and s == 1 and H > 4 else H
    x = hi.normal(101, (Nb, B * Ci, H, Wd), dtype)
    w = hi.normal(102, (B * Co, Ci, k, k), dtype, 1.0 / np.sqrt(Ci * k * k))
    b = hi.normal(103, (B * Co,), dtype)
    ry = oa.conv2d_fwd(B, x, w, b, s, p)
    Ho, Wo = ry.shape[2], ry.shape[3]
    dy = hi.normal(104, ry.shape, dtype)
    X, W, Bi, dY = dev(x, dtype), dev(w, dtype), dev(b, dtype), dev(dy, dtype)
    Y = empty(ry.shape, dtype)
    wsf, ws = conv_workspaces(hb, path, (B, Nb, Ci, Co, H, Wd, k, k, s, p, DT[dtype]))
    hb.conv2d_grouped_fwd(B, Nb, Ci, Co, H, Wd, k, k, s, p, DT[dtype], X, W, Bi, Y, workspace=wsf)
    check(host(Y), ry, TOL[dtype], "Y")
    hb.conv2d_grouped_fwd(B, Nb, Ci, Co, H, Wd, k, k, s, p, DT[dtype], X, W, None, Y, hb.ACT_LEAKY, 0.2, workspace=wsf)
    check(host(Y), oops.act_fwd(oa.conv2d_fwd(B, x, w, None, s, p), oops.ACT_LEAKY, 0.2), TOL[dtype], "leaky(Y)")
    dX = empty(x.shape, dtype)
    dW = empty(w.shape, torch.float32)
    db = empty((B * Co,), torch.float32)
    hb.conv2d_grouped_bwd(B, Nb, Ci, Co, H, Wd, k, k, s, p, DT[dtype], X, W, dY, dX, dW, db, ws)
    rdx, rdw, rdb = oa.conv2d_bwd(B, x, w, dy, s, p)
    check(host(dX), rdx, TOL[dtype], "dX")
    check(host(dW), rdw, f32_tol(dtype), "dW")
    check(host(db), rdb, f32_tol(dtype), "dbias")


@pytest.mark.parametrize("path", ["implicit", "lowered"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Nb,Cx,Cy,H,k,s,p", [(3, 2, 10, 6, 4, 4, 2, 1), (2, 3, 20, 12, 1, 4, 1, 0), (2, 2, 8, 3, 8, 4, 2, 1)])
def test_convT2d_through_conv_entry_points(hb, dtype, B, Nb, Cx, Cy, H, k, s, p, path):
    """Fused ConvTranspose2d: forward = the data-gradient form of the grouped conv, its input
    gradient = the forward form, its weight gradient = the weight-gradient form with X and dY
    exchanged (weights [B*Cx, Cy, kh, kw] are read as conv weights [B*Co=Cx, Ci=Cy, kh, kw])."""
    x = hi.normal(111, (Nb, B * Cx, H, H), dtype)
    w = hi.normal(112, (B * Cx, Cy, k, k), dtype, 1.0 / np.sqrt(Cx * 4))
    ry = oa.convT2d_fwd(B, x, w, None, s, p)
    Ho = ry.shape[2]
    dy = hi.normal(113, ry.shape, dtype)
    X, W, dY = dev(x, dtype), dev(w, dtype), dev(dy, dtype)
    Y = empty(ry.shape, dtype)
    conv = (B, Nb, Cy, Cx, Ho, Ho, k, k, s, p, DT[dtype])     # the conv whose input is ConvT's output
    wsf, ws = conv_workspaces(hb, path, conv)
    hb.conv2d_grouped_bwd(*conv, None, W, X, Y, None, None, ws)
    check(host(Y), ry, TOL[dtype], "convT fwd")
    bias = hi.normal(114, (B * Cy,), dtype)
    hb.bias_act_nchw(Nb, B * Cy, Ho * Ho, DT[dtype], Y, dev(bias, dtype), hb.ACT_TANH, 0.0)
    check(host(Y), np.tanh(oa.convT2d_fwd(B, x, w, bias, s, p)), TOL[dtype], "tanh(convT + bias)")
    rdx, rdw, _ = oa.convT2d_bwd(B, x, w, dy, s, p)
    dX = empty(x.shape, dtype)
    hb.conv2d_grouped_fwd(*conv, dY, W, None, dX, workspace=wsf)
    check(host(dX), rdx, TOL[dtype], "convT dX")
    dW = empty(w.shape, torch.float32)
    hb.conv2d_grouped_bwd(*conv, dY, None, X, None, dW, None, ws)
    check(host(dW), rdw, f32_tol(dtype), "convT dW")


# ------------------------------------------------------------------ BatchNorm + activation + point max-pool, fused
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Nb,C,L", [(2, 9, 40, 500), (3, 4, 7, 250), (2, 32, 16, 2500), (1, 2, 3, 5)])
def test_bn_maxpool_fused(hb, dtype, B, Nb, C, L):
    print(f"bn+pool {dtype} B={B} Nb={Nb} C={C} L={L}", flush=True)
    x = hi.snap(hi.normal(121, (Nb, B * C, L)) * 1.5 + 0.5, dtype)
    g = (hi.normal(122, (B * C,)) * 0.5 + 1.0).astype(np.float32)
    g[0] = -abs(g[0])                          # a negative scale: the maximum sits at the minimum of x
    bt = (hi.normal(123, (B * C,)) * 0.3).astype(np.float32)
    bt[1 % (B * C)] = -5.0                     # a channel that the ReLU clips everywhere: all-zero ties -> index 0
    s = conv_strides(B, C, L)
    vs = (Nb * C, C, 1)
    X, G, Bt = dev(x, dtype), dev(g), dev(bt)
    SM, SI = empty((B * C,), torch.float32), empty((B * C,), torch.float32)
    V, I = empty((B, Nb, C), dtype), empty((B, Nb, C), torch.int32)
    hb.bn_fwd_maxpool(B, Nb, C, L, DT[dtype], X, s, G, Bt, 1e-5, 0.1, None, None, SM, SI, V, I, vs, hb.ACT_RELU)
    # (1) bit-identical to the two stand-alone operators
    SM2, SI2 = empty((B * C,), torch.float32), empty((B * C,), torch.float32)
    Y = empty(x.shape, dtype)
    V2, I2 = empty((B, Nb, C), dtype), empty((B, Nb, C), torch.int32)
    hb.bn_fwd(B, Nb, C, L, DT[dtype], X, s, G, Bt, 1e-5, 0.1, None, None, SM2, SI2, Y, s, hb.ACT_RELU)
    hb.maxpool_points(B, Nb, C, L, DT[dtype], Y, s, V2, I2, vs)
    assert torch.equal(SM, SM2) and torch.equal(SI, SI2)
    assert torch.equal(I, I2) and torch.equal(V, V2)
    # (2) against the oracle's composition; an index may differ only at a near-tie of the maximum
    ry, rmean, rinv, _, _ = oa.bn_fwd(B, x, g, bt, 1e-5)
    ya = oops.store(oops.act_fwd(ry, oops.ACT_RELU), dtype)
    rv, ri = oa.maxpool_points_fwd(B, ya)
    t3 = lambda a: a.reshape(Nb, B, C).transpose(1, 0, 2)
    check(host(V), t3(rv), TOL[dtype], "pooled")
    gi = I.cpu().numpy()
    mism = gi != t3(ri)
    if mism.any():
        at = np.take_along_axis(ya, gi.transpose(1, 0, 2).reshape(Nb, B * C, 1).astype(np.int64), axis=2)[:, :, 0]
        assert np.all(t3(at)[mism] >= t3(rv)[mism] - TOL[dtype] * (np.abs(t3(rv)[mism]) + np.abs(ya).max()))
    assert mism.mean() <= 0.02
    assert int(gi[(1 % (B * C)) // C, 0, (1 % (B * C)) % C]) == 0
    # backward: equals scatter + BatchNorm backward
    dv = hi.normal(124, (B, Nb, C), dtype)
    dV = dev(dv, dtype)
    dX = empty(x.shape, dtype)
    dG, dB, DS = (empty((B * C,), torch.float32) for _ in range(3))
    hb.bn_bwd_maxpool(B, Nb, C, L, DT[dtype], X, s, dV, I, vs, G, Bt, SM, SI, dX, s, dG, dB, hb.ACT_RELU, 0.0, DS)
    dy = oa.maxpool_points_bwd(B, dv.transpose(1, 0, 2).reshape(Nb, B * C), gi.transpose(1, 0, 2).reshape(Nb, B * C), L)
    gdy = oops.act_bwd(ry, dy, oops.ACT_RELU)
    rdx, rdg, rdb = oa.bn_bwd(B, x, gdy, g, host(SM), host(SI))
    check(host(dX), rdx, TOL[dtype], "dX")
    sc = np.abs(dv).sum(axis=1).max()
    assert np.abs(host(dG) - rdg).max() <= f32_tol(dtype) * max(np.abs(rdg).max(), sc * 1e-2), "dgamma"
    assert np.abs(host(dB) - rdb).max() <= f32_tol(dtype) * max(np.abs(rdb).max(), sc * 1e-2), "dbeta"
    dX2 = empty(x.shape, dtype)
    dYd = empty(x.shape, dtype)
    dG2, dB2 = empty((B * C,), torch.float32), empty((B * C,), torch.float32)
    hb.maxpool_points_bwd(B, Nb, C, L, DT[dtype], dV, I, vs, dYd, s)
    hb.bn_bwd(B, Nb, C, L, DT[dtype], X, s, dYd, s, G, Bt, SM, SI, dX2, s, dG2, dB2, hb.ACT_RELU, 0.0)
    check(host(dX), host(dX2), 1e-5 if dtype == "f32" else 8e-3, "fused vs unfused dX")


# ------------------------------------------------------------------ BatchNorm, evaluation mode
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Nb,C,L,layout,act", [(3, 4, 5, 300, "conv", 1), (2, 3, 7, 131, "conv", 2), (2, 33, 70, 1, "linear", 1),
                                                  (2, 6, 4, 9000, "conv", 0)])
def test_bn_eval_fwd(hb, dtype, B, Nb, C, L, layout, act):
    """Running estimates in place of batch statistics; conv layout (vector and scalar rows, the wide
    workgroup) and the [N, B, C] layout; writing in place; models never share estimates."""
    print(f"bn eval {dtype} B={B} Nb={Nb} C={C} L={L} {layout} act={act}", flush=True)
    oact = {0: oops.ACT_NONE, 1: oops.ACT_RELU, 2: oops.ACT_LEAKY}[act]
    g = (hi.normal(71, (B * C,)) * 0.5 + 1.0).astype(np.float32)
    bt = (hi.normal(72, (B * C,)) * 0.3).astype(np.float32)
    rm = (hi.normal(73, (B * C,)) * 0.5).astype(np.float32)
    rv = (0.5 + np.abs(hi.normal(74, (B * C,)))).astype(np.float32)
    if layout == "conv":
        x = hi.normal(75, (Nb, B * C, L), dtype)
        xs = conv_strides(B, C, L)
        ref = oops.act_fwd(oa.bn_eval_fwd(B, x, g, bt, rm, rv, 1e-5), oact, 0.2)
    else:
        x = hi.normal(75, (B, Nb, C), dtype)
        xs = (Nb * C, C, 1, 1)
        ref = oops.act_fwd(oa.bn_eval_fwd(B, x, g, bt, rm, rv, 1e-5, "linear"), oact, 0.2)
    X = dev(x, dtype)
    Y = torch.full(x.shape, float("nan"), dtype=TDT[dtype], device="cuda")
    G, Bt, RM, RV = dev(g), dev(bt), dev(rm), dev(rv)
    hb.bn_eval_fwd(B, Nb, C, L, DT[dtype], X, xs, G, Bt, RM, RV, 1e-5, Y, xs, act, 0.2)
    extra = 4 * 2.0 ** -24 * np.abs(g / np.sqrt(rv + 1e-5)) * (1.0 + np.abs(rm))       # fp32 rounding of (x - mean) * scale
    ex = extra[None, :, None] * (np.abs(x) + 1) if layout == "conv" else extra.reshape(B, 1, C) * (np.abs(x) + 1)
    check(host(Y), ref, TOL[dtype], "y", ex)
    assert torch.equal(RM, dev(rm)) and torch.equal(RV, dev(rv))          # nothing is updated
    hb.bn_eval_fwd(B, Nb, C, L, DT[dtype], X, xs, G, Bt, RM, RV, 1e-5, X, xs, act, 0.2)      # in place
    assert torch.equal(X, Y)
    # independence: another model's estimates do not touch model 0's output
    rv2 = rv.copy()
    rv2[C:] *= 3.0
    Y2 = torch.empty_like(Y)
    hb.bn_eval_fwd(B, Nb, C, L, DT[dtype], dev(x, dtype), xs, G, Bt, RM, dev(rv2), 1e-5, Y2, xs, act, 0.2)
    if layout == "conv":
        assert torch.equal(Y2[:, :C], Y[:, :C]) and not torch.equal(Y2[:, C:], Y[:, C:])
    else:
        assert torch.equal(Y2[0], Y[0]) and not torch.equal(Y2[1], Y[1])


# ------------------------------------------------------------------ conv1x1 -> BatchNorm -> point max-pool, fused backward
@pytest.mark.parametrize("B,Nb,Ci,Co,L,act", [(2, 5, 16, 40, 300, 1), (2, 3, 128, 136, 260, 1), (3, 4, 64, 72, 132, 2),
                                               (1, 2, 8, 1024, 8, 0)])
def test_conv1x1_bn_maxpool_bwd_fused(hb, B, Nb, Ci, Co, L, act):
    """The fused backward never forms the dense [Nb, B*Co, L] gradient; it must equal the chain
    point-max backward -> BatchNorm backward -> conv1x1 backward of the oracle, and the library's
    own unfused chain, to the bf16 tolerance (the references round the dense gradient to bf16
    before the two contractions, the fused operator has no such tensor)."""
    dtype = "bf16"
    print(f"conv+bn+pool bwd B={B} Nb={Nb} Ci={Ci} Co={Co} L={L} act={act}", flush=True)
    x = hi.snap(np.maximum(hi.normal(131, (Nb, B * Ci, L)) + 0.3, 0.0), dtype)      # like a post-ReLU activation
    w = hi.normal(132, (B * Co, Ci), dtype, 1.0 / np.sqrt(Ci))
    bias = hi.normal(133, (B * Co,), dtype, 0.1)
    g = (hi.normal(134, (B * Co,)) * 0.3 + 1.0).astype(np.float32)
    g[0] = -abs(g[0])
    bt = (hi.normal(135, (B * Co,)) * 0.3).astype(np.float32)
    slope = 0.2
    oact = {0: oops.ACT_NONE, 1: oops.ACT_RELU, 2: oops.ACT_LEAKY}[act]
    z = oops.store(oa.conv1x1_fwd(B, x, w, bias), dtype)
    ry, rmean, rinv, _, _ = oa.bn_fwd(B, z, g, bt, 1e-5)
    ya = oops.store(oops.act_fwd(ry, oact, slope), dtype)
    rv, ri = oa.maxpool_points_fwd(B, ya)
    dv = hi.normal(136, (B, Nb, Co), dtype)
    sx, sz = conv_strides(B, Ci, L), conv_strides(B, Co, L)
    vs = (Nb * Co, Co, 1)
    t3 = lambda a: np.ascontiguousarray(a.reshape(Nb, B, Co).transpose(1, 0, 2))
    idx = t3(ri).astype(np.int32)
    mean32, inv32 = rmean.astype(np.float32), rinv.astype(np.float32)
    # oracle chain
    dy = oa.maxpool_points_bwd(B, dv.transpose(1, 0, 2).reshape(Nb, B * Co), ri, L)
    gdy = oops.act_bwd(ry, dy, oact, slope)
    rdz, rdg, rdb = oa.bn_bwd(B, z, gdy, g, mean32, inv32)
    rdx, rdw, _ = oa.conv1x1_bwd(B, x, w, rdz)                 # exact composition (no rounding of dz)
    rdx_r, rdw_r, _ = oa.conv1x1_bwd(B, x, w, oops.store(rdz, dtype))
    X, W, Bi, Z = dev(x, dtype), dev(w, dtype), dev(bias, dtype), dev(z, dtype)
    G, Bt, SM, SI = dev(g), dev(bt), dev(mean32), dev(inv32)
    dV, I = dev(dv, dtype), torch.from_numpy(idx).cuda()
    dX = empty(x.shape, dtype)
    dW = empty((B * Co, Ci), torch.float32)
    dB0, dG, dBt = (empty((B * Co,), torch.float32) for _ in range(3))
    nws = hb.conv1x1_bn_maxpool_bwd_workspace_bytes(B, Nb, Ci, Co, L, DT[dtype])
    assert nws > 0
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    hb.conv1x1_bn_maxpool_bwd(B, Nb, Ci, Co, L, DT[dtype], X, sx, W, Bi, Z, sz, None, None, dV, I, vs, G, Bt, SM, SI, dX,
                              sx, dW, dB0, dG, dBt, act, slope, ws)
    sc = np.abs(dv).sum(axis=1).max()
    assert np.abs(host(dG) - rdg).max() <= f32_tol(dtype) * max(np.abs(rdg).max(), sc * 1e-2), "dgamma"
    assert np.abs(host(dBt) - rdb).max() <= f32_tol(dtype) * max(np.abs(rdb).max(), sc * 1e-2), "dbeta"
    assert float(dB0.abs().max()) == 0.0
    # Conditioning term: the operator normalises the convolution output it recomputes from X and W
    # (through the Gram matrix), the chain normalises the stored, bf16-rounded z.  The two differ by
    # at most 2^-9 |z| per element, which the dense term scales by gamma * invstd^2 * dgamma / M.
    M = Nb * L
    coef = np.abs(g * rinv * rinv * rdg) / M * 2.0 ** -9                       # [B*Co]
    xa, za = np.abs(x).reshape(Nb, B, Ci, L), np.abs(z).reshape(Nb, B, Co, L)
    cf, wa = coef.reshape(B, Co), np.abs(w).reshape(B, Co, Ci)
    ex_dw = (cf[:, :, None] * np.einsum("nbcl,nbil->bci", za, xa)).reshape(B * Co, Ci)
    ex_dx = np.einsum("bci,nbcl->nbil", wa * cf[:, :, None], za).reshape(Nb, B * Ci, L)
    e1 = check(host(dX), rdx, TOL[dtype], "dX vs exact composition", ex_dx)
    e2 = check(host(dW), rdw, TOL[dtype], "dW vs exact composition", ex_dw)
    e3 = check(host(dX), rdx_r, TOL[dtype], "dX vs chain with stored dz", ex_dx)
    e4 = check(host(dW), rdw_r, TOL[dtype], "dW vs chain with stored dz", ex_dw)
    raw = lambda a, r: np.abs(a - r).max() / np.abs(r).max()
    print(f"   raw norm-wise err: dX {raw(host(dX), rdx):.2e}, dW {raw(host(dW), rdw):.2e}", flush=True)
    assert raw(host(dX), rdx) <= TOL[dtype] and raw(host(dW), rdw) <= TOL[dtype]
    print(f"   conditioning allowance / rms: dX {ex_dx.max() / np.sqrt((rdx ** 2).mean()):.2e}, "
          f"dW {ex_dw.max() / np.sqrt((rdw ** 2).mean()):.2e}", flush=True)
    print(f"   rel err: dX {e1:.2e} / {e3:.2e}, dW {e2:.2e} / {e4:.2e}", flush=True)
    # the library's own unfused chain on the same inputs
    dZ = empty(z.shape, dtype)
    dG2, dB2 = empty((B * Co,), torch.float32), empty((B * Co,), torch.float32)
    hb.bn_bwd_maxpool(B, Nb, Co, L, DT[dtype], Z, sz, dV, I, vs, G, Bt, SM, SI, dZ, sz, dG2, dB2, act, slope)
    dX2 = empty(x.shape, dtype)
    dW2 = empty((B * Co, Ci), torch.float32)
    n2 = hb.conv1x1_bwd_workspace_bytes(B, Nb, Ci, Co, L, DT[dtype])
    ws2 = torch.empty(max(n2, 4), dtype=torch.uint8, device="cuda")
    hb.conv1x1_bwd(B, Nb, Ci, Co, L, DT[dtype], X, sx, W, dZ, sz, dX2, sx, dW2, None, ws2)
    check(host(dX), host(dX2), 2 * TOL[dtype], "fused vs unfused dX", ex_dx)    # both sides carry their own bf16 rounding
    check(host(dW), host(dW2), 2 * TOL[dtype], "fused vs unfused dW", ex_dw)
    assert torch.equal(dG, dG2) or np.abs(host(dG) - host(dG2)).max() <= 1e-5 * max(np.abs(rdg).max(), sc * 1e-2)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Nb,C,L,act", [(3, 5, 10, 37, 1), (2, 4, 64, 260, 2), (1, 3, 7, 1, 0), (2, 40, 16, 2500, 1)])
def test_bn_apply_fwd(hb, B, Nb, C, L, act, dtype):
    """Normalisation with given statistics: against the oracle's normalisation by given estimates, on
    statistics chosen freely (not those of the input), and bit for bit what the training forward
    stored when handed the statistics it saved."""
    print(f"bn apply B={B} Nb={Nb} C={C} L={L} act={act} {dtype}", flush=True)
    oact = {0: oops.ACT_NONE, 1: oops.ACT_RELU, 2: oops.ACT_LEAKY}[act]
    x = hi.snap(hi.normal(171, (Nb, B * C, L)) * 1.3 + 0.2, dtype)
    g = (hi.normal(172, (B * C,)) * 0.5 + 1.0).astype(np.float32)
    bt = (hi.normal(173, (B * C,)) * 0.3).astype(np.float32)
    mean = (hi.normal(174, (B * C,)) * 0.4).astype(np.float32)
    invstd = (np.abs(hi.normal(175, (B * C,))) * 0.5 + 0.5).astype(np.float32)
    var = 1.0 / invstd.astype(np.float64) ** 2                  # the oracle takes a variance and eps: eps = 0
    ref = oops.act_fwd(oa.bn_eval_fwd(B, x, g, bt, mean, var, 0.0), oact, 0.2)
    sx = conv_strides(B, C, L)
    X, G, Bt, Y = dev(x, dtype), dev(g), dev(bt), empty((Nb, B * C, L), dtype)
    hb.bn_apply_fwd(B, Nb, C, L, DT[dtype], X, sx, G, Bt, dev(mean), dev(invstd), Y, sx, act, 0.2)
    extra = 4 * 2.0 ** -24 * np.abs(g * invstd) * (1.0 + np.abs(mean))
    check(host(Y), ref, TOL[dtype], "y", extra[None, :, None] * (np.abs(x) + 1))
    f32 = torch.float32
    SM, SI, Y1, Y2 = empty((B * C,), f32), empty((B * C,), f32), empty((Nb, B * C, L), dtype), empty((Nb, B * C, L), dtype)
    hb.bn_fwd(B, Nb, C, L, DT[dtype], X, sx, G, Bt, 1e-5, 0.1, None, None, SM, SI, Y1, sx, act, 0.2)
    hb.bn_apply_fwd(B, Nb, C, L, DT[dtype], X, sx, G, Bt, SM, SI, Y2, sx, act, 0.2)
    assert torch.equal(Y1, Y2)


@pytest.mark.parametrize("B,Nb,Ci,Co,L,in_act,saved", [(2, 3, 128, 1024, 644, 1, True), (2, 4, 64, 200, 260, 2, False),
                                                        (3, 2, 24, 72, 132, 1, True)])
def test_conv1x1_bn_maxpool_prenorm(hb, B, Nb, Ci, Co, L, in_act, saved):
    """The one-operator tail at the end of a chain whose activated tensors are not stored: its input given as
    the previous block's pre-activation and BatchNorm constants must give, bit for bit, what the plain
    operator gives on that block's stored output (forward and backward; with and without the moments the
    forward saved), the plain operator being the one checked against the oracle above."""
    dtype = "bf16"
    print(f"conv+bn+pool prenorm B={B} Nb={Nb} Ci={Ci} Co={Co} L={L} in_act={in_act} saved={saved}", flush=True)
    xpre = hi.snap(hi.normal(151, (Nb, B * Ci, L)) * 1.5 + 0.4, dtype)
    gi = (hi.normal(152, (B * Ci,)) * 0.5 + 1.0).astype(np.float32)
    bi = (hi.normal(153, (B * Ci,)) * 0.3).astype(np.float32)
    w = hi.normal(154, (B * Co, Ci), dtype, 1.0 / np.sqrt(Ci))
    bias = hi.normal(155, (B * Co,), dtype, 0.1)
    g = (hi.normal(156, (B * Co,)) * 0.3 + 1.0).astype(np.float32)
    g[::3] = -np.abs(g[::3])
    bt = (hi.normal(157, (B * Co,)) * 0.3).astype(np.float32)
    bt[1::7] = -6.0                                     # rows clipped flat by the ReLU: the rare path that re-reads X at point 0
    dv = hi.normal(158, (B, Nb, Co), dtype)
    sx, vs = conv_strides(B, Ci, L), (Nb * Co, Co, 1)
    f32 = torch.float32
    Xp, Gi, Bi_, W, Bs, G, Bt, dV = dev(xpre, dtype), dev(gi), dev(bi), dev(w, dtype), dev(bias, dtype), dev(g), dev(bt), dev(dv, dtype)
    MI, II, X = empty((B * Ci,), f32), empty((B * Ci,), f32), empty((Nb, B * Ci, L), dtype)
    hb.bn_fwd(B, Nb, Ci, L, DT[dtype], Xp, sx, Gi, Bi_, 1e-5, 0.1, None, None, MI, II, X, sx, in_act, 0.2)
    nws = max(hb.conv1x1_bn_maxpool_fwd_workspace_bytes(B, Nb, Ci, Co, L, DT[dtype]),
              hb.conv1x1_bn_maxpool_bwd_workspace_bytes(B, Nb, Ci, Co, L, DT[dtype]))
    assert nws > 0
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    out = {}
    for kind in ("plain", "prenorm", "written"):
        SM, SI = empty((B * Co,), f32), empty((B * Co,), f32)
        RM, RV = dev(np.zeros(B * Co, np.float32)), dev(np.ones(B * Co, np.float32))
        V, I = empty((B, Nb, Co), dtype), torch.empty(B, Nb, Co, dtype=torch.int32, device="cuda")
        ZH = empty((B, Nb, Co), f32)
        SAV = empty((hb.conv1x1_bn_maxpool_saved_floats(B, Ci, Co),), f32) if saved else None
        dX, dW, db = empty((Nb, B * Ci, L), dtype), empty((B * Co, Ci), f32), empty((B * Co,), f32)
        dG, dB = empty((B * Co,), f32), empty((B * Co,), f32)
        ws.fill_(0x5a)
        if kind == "plain":
            hb.conv1x1_bn_maxpool_fwd(B, Nb, Ci, Co, L, DT[dtype], X, sx, W, Bs, G, Bt, 1e-5, 0.1, RM, RV, SM, SI, V, I, vs, ZH, SAV,
                                      1, 0.0, ws)
            hb.conv1x1_bn_maxpool_bwd(B, Nb, Ci, Co, L, DT[dtype], X, sx, W, Bs, None, None, ZH, SAV, dV, I, vs, G, Bt, SM, SI, dX,
                                      sx, dW, db, dG, dB, 1, 0.0, ws)
        elif kind == "written":        # the forward's first kernel writes the activated input out; plain backward on that
            XA = torch.full((Nb, B * Ci, L), float("nan"), dtype=TDT[dtype], device="cuda")
            hb.conv1x1_bn_maxpool_prenorm_fwd(B, Nb, Ci, Co, L, DT[dtype], Xp, sx, Gi, Bi_, MI, II, in_act, 0.2, W, Bs, G, Bt, 1e-5,
                                              0.1, RM, RV, SM, SI, V, I, vs, ZH, SAV, 1, 0.0, ws, Xact=XA, xas=sx)
            assert torch.equal(XA, X), "the activated input written on the way differs from the stored one"
            hb.conv1x1_bn_maxpool_bwd(B, Nb, Ci, Co, L, DT[dtype], XA, sx, W, Bs, None, None, ZH, SAV, dV, I, vs, G, Bt, SM, SI, dX,
                                      sx, dW, db, dG, dB, 1, 0.0, ws)
        else:
            hb.conv1x1_bn_maxpool_prenorm_fwd(B, Nb, Ci, Co, L, DT[dtype], Xp, sx, Gi, Bi_, MI, II, in_act, 0.2, W, Bs, G, Bt, 1e-5,
                                              0.1, RM, RV, SM, SI, V, I, vs, ZH, SAV, 1, 0.0, ws)
            hb.conv1x1_bn_maxpool_prenorm_bwd(B, Nb, Ci, Co, L, DT[dtype], Xp, sx, Gi, Bi_, MI, II, in_act, 0.2, W, Bs, ZH, SAV, dV, I,
                                              vs, G, Bt, SM, SI, dX, sx, dW, db, dG, dB, 1, 0.0, ws)
        out[kind] = dict(V=V, I=I, ZH=ZH, SM=SM, SI=SI, RM=RM, RV=RV, dX=dX, dW=dW, db=db, dG=dG, dB=dB)
    for k, v in out["plain"].items():
        for kind in ("prenorm", "written"):
            assert torch.equal(v, out[kind][k]), f"{k} ({kind}) differs from the plain operator on the stored activated tensor"
    assert bool(torch.isfinite(out["prenorm"]["dX"].float()).all()) and float(out["prenorm"]["dW"].abs().max()) > 0


@pytest.mark.parametrize("B,Nb,Ci,Co,L,act", [(2, 5, 16, 40, 300, 1), (2, 3, 128, 136, 260, 1), (3, 4, 64, 72, 132, 2),
                                               (2, 3, 8, 1024, 8, 0), (1, 2, 128, 300, 1156, 1)])
def test_conv1x1_bn_maxpool_fwd_bwd_one_operator(hb, B, Nb, Ci, Co, L, act):
    """Forward and backward of the one-operator tail against the oracle's composition (which
    rounds nothing inside the operator).  The argmax is decided on fp32 matrix products on the
    GPU and in float64 by the oracle: indices must agree except at near-ties of the maximum,
    and the backward is checked on the GPU's own indices."""
    dtype = "bf16"
    print(f"conv+bn+pool one operator B={B} Nb={Nb} Ci={Ci} Co={Co} L={L} act={act}", flush=True)
    x = hi.snap(np.maximum(hi.normal(141, (Nb, B * Ci, L)) + 0.3, 0.0), dtype)
    w = hi.normal(142, (B * Co, Ci), dtype, 1.0 / np.sqrt(Ci))
    bias = hi.normal(143, (B * Co,), dtype, 0.1)
    g = (hi.normal(144, (B * Co,)) * 0.3 + 1.0).astype(np.float32)
    g[::3] = -np.abs(g[::3])                            # negative scales: the maximum sits at the minimum of z
    bt = (hi.normal(145, (B * Co,)) * 0.3).astype(np.float32)
    bt[1::7] = -6.0                                     # every point clipped by a ReLU: the row's values are all equal
    g[5] = 0.0                                          # zero scale: all equal whatever the activation
    slope, eps, mom = 0.2, 1e-5, 0.1
    oact = {0: oops.ACT_NONE, 1: oops.ACT_RELU, 2: oops.ACT_LEAKY}[act]
    rm0 = (hi.normal(146, (B * Co,)) * 0.1).astype(np.float32)
    rv0 = (1.0 + 0.1 * np.abs(hi.normal(147, (B * Co,)))).astype(np.float32)
    rv, ri, rmean, rinv, nrm, nrv, rz = oa.conv1x1_bn_maxpool_fwd(B, x, w, bias, g, bt, eps, mom, rm0, rv0, oact, slope)
    sx = conv_strides(B, Ci, L)
    vs = (Nb * Co, Co, 1)
    t3 = lambda a: np.ascontiguousarray(a.reshape(Nb, B, Co).transpose(1, 0, 2))
    X, W, Bi = dev(x, dtype), dev(w, dtype), dev(bias, dtype)
    G, Bt, RM, RV = dev(g), dev(bt), dev(rm0), dev(rv0)
    SM, SI = empty((B * Co,), torch.float32), empty((B * Co,), torch.float32)
    V = empty((B, Nb, Co), dtype)
    I = torch.empty(B, Nb, Co, dtype=torch.int32, device="cuda")
    ZH = empty((B, Nb, Co), torch.float32)
    SAV = empty((hb.conv1x1_bn_maxpool_saved_floats(B, Ci, Co),), torch.float32)
    nws = max(hb.conv1x1_bn_maxpool_fwd_workspace_bytes(B, Nb, Ci, Co, L, DT[dtype]),
              hb.conv1x1_bn_maxpool_bwd_workspace_bytes(B, Nb, Ci, Co, L, DT[dtype]))
    assert nws > 0
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    hb.conv1x1_bn_maxpool_fwd(B, Nb, Ci, Co, L, DT[dtype], X, sx, W, Bi, G, Bt, eps, mom, RM, RV, SM, SI, V, I, vs, ZH, SAV,
                              act, slope, ws)
    # statistics: fp32 Gram matrix; the variance loses relative accuracy E[z^2] / var
    m = Nb * L
    gm, gi_ = host(SM), host(SI)
    z = oa.conv1x1_fwd(B, x, w, bias)
    ez2 = (z ** 2).mean(axis=(0, 2))
    var = 1.0 / rinv ** 2 - eps
    assert np.all(np.abs(gm - rmean) <= 1e-5 * (np.abs(rmean) + np.sqrt(var) + np.sqrt(ez2))), "mean"
    assert np.all(np.abs(gi_ - rinv) <= rinv * (1e-5 + 2e-6 * ez2 / (var + eps))), "invstd"
    assert np.abs(host(RM) - nrm).max() <= 1e-5 * max(np.abs(nrm).max(), 1.0)
    assert np.all(np.abs(host(RV) - nrv) <= 1e-5 * np.abs(nrv) + 2e-7 * ez2), "running_var"
    # pooled value, argmax, z at the argmax
    gv, gi, gz = host(V), host(I), host(ZH)
    y = oa.bn_fwd(B, z, g, bt, eps)[0]
    ya = oops.act_fwd(y, oact, slope)
    check(gv, t3(oops.store(rv, dtype)), TOL[dtype], "pooled")
    assert gi.min() >= 0 and gi.max() < L
    gi_nk = gi.transpose(1, 0, 2).reshape(Nb, B * Co)
    nmism = check_tail_argmax(ya, ri, gi_nk, oa.conv1x1_fwd(B, np.abs(x), np.abs(w), None), Ci, np.abs(g) * rinv, "one-operator tail")
    nflat = int((ya.max(axis=2) == ya.min(axis=2)).sum())
    zat = np.take_along_axis(z, gi.transpose(1, 0, 2).reshape(Nb, B * Co, 1).astype(np.int64), axis=2)[:, :, 0]
    assert np.abs(gz - t3(zat)).max() <= 1e-5 * np.abs(z).max(), "z at the argmax"
    # backward from the forward's own outputs, against the oracle's composition on the same indices
    dv = hi.normal(148, (B, Nb, Co), dtype)
    idx_o = gi.transpose(1, 0, 2).reshape(Nb, B * Co)
    rdx, rdw, rdb, rdg, rdbt = oa.conv1x1_bn_maxpool_bwd(B, x, w, bias, g, bt, gm, gi_, dv.transpose(1, 0, 2).reshape(Nb, B * Co),
                                                         idx_o, oact, slope)
    dV = dev(dv, dtype)
    dX = empty(x.shape, dtype)
    dW = empty((B * Co, Ci), torch.float32)
    dB0, dG, dBt = (empty((B * Co,), torch.float32) for _ in range(3))
    hb.conv1x1_bn_maxpool_bwd(B, Nb, Ci, Co, L, DT[dtype], X, sx, W, Bi, None, None, ZH, SAV, dV, I, vs, G, Bt, SM, SI, dX, sx,
                              dW, dB0, dG, dBt, act, slope, ws)
    sc = np.abs(dv).sum(axis=1).max()
    assert np.abs(host(dG) - rdg).max() <= f32_tol(dtype) * max(np.abs(rdg).max(), sc * 1e-2), "dgamma"
    assert np.abs(host(dBt) - rdbt).max() <= f32_tol(dtype) * max(np.abs(rdbt).max(), sc * 1e-2), "dbeta"
    # a bias under a BatchNorm has no gradient (the oracle's is rounding of the fp32 statistics it was given)
    assert float(dB0.abs().max()) == 0.0 and np.abs(rdb).max() <= 1e-5 * sc
    e1 = check(host(dX), rdx, TOL[dtype], "dX")
    e2 = check(host(dW), rdw, 2e-4, "dW")               # fp32 output, no storage rounding anywhere in the operator
    print(f"   argmax differing from the oracle's: {nmism} of {gi.size} ({nflat} rows of equal values); rel err dX {e1:.2e} dW {e2:.2e}", flush=True)
    # the same backward without the saved moments of the forward (recomputed from X)
    dX2, dW2 = empty(x.shape, dtype), empty((B * Co, Ci), torch.float32)
    hb.conv1x1_bn_maxpool_bwd(B, Nb, Ci, Co, L, DT[dtype], X, sx, W, Bi, None, None, ZH, None, dV, I, vs, G, Bt, SM, SI, dX2,
                              sx, dW2, dB0, dG, dBt, act, slope, ws)
    check(host(dX2), rdx, TOL[dtype], "dX (moments recomputed)")
    check(host(dW2), rdw, 2e-4, "dW (moments recomputed)")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Nb,Ci,Co,L", [(2, 3, 3, 3, 300), (2, 4, 64, 64, 260), (3, 2, 24, 40, 131)])
def test_point_transform(hb, dtype, B, Nb, Ci, Co, L):
    """Per-sample matrices applied to the points (3x3 input transform, 64x64 feature transform)."""
    print(f"point transform {dtype} B={B} Nb={Nb} Ci={Ci} Co={Co} L={L}", flush=True)
    x = hi.normal(231, (Nb, B * Ci, L), dtype)
    t = hi.normal(232, (B, Nb, Co, Ci), dtype, 1.0 / np.sqrt(Ci))
    dy = hi.normal(233, (Nb, B * Co, L), dtype)
    X, T, dY = dev(x, dtype), dev(t, dtype), dev(dy, dtype)
    xs, ys = conv_strides(B, Ci, L), conv_strides(B, Co, L)
    Y, dX, dT = empty((Nb, B * Co, L), dtype), empty((Nb, B * Ci, L), dtype), empty((B, Nb, Co, Ci), dtype)
    hb.point_transform_fwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, T, Y, ys)
    hb.point_transform_bwd(B, Nb, Ci, Co, L, DT[dtype], X, xs, T, dY, ys, dX, xs, dT)
    for b in range(B):
        xb, dyb = x[:, b * Ci:(b + 1) * Ci], dy[:, b * Co:(b + 1) * Co]
        check(host(Y)[:, b * Co:(b + 1) * Co], oops.point_transform_fwd(xb, t[b]), TOL[dtype], "Y")
        rdx, rdt = oops.point_transform_bwd(xb, t[b], dyb)
        check(host(dX)[:, b * Ci:(b + 1) * Ci], rdx, TOL[dtype], "dX")
        check(host(dT)[b], rdt, TOL[dtype], "dT")
