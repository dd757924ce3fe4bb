"""Whole-step parity of the PointNet-cls array with input / feature transform sub-networks on the
GPU against B separate unfused oracle runs: forward + backward + Adam, fp32 and bf16."""
import dataclasses

import numpy as np
import pytest
import torch

import hfta_inputs as hi
from oracle import pointnet as opn
from oracle import pointnet_t as opt

pytestmark = pytest.mark.gpu

# Free-running chain: the per-operator bound (1e-5 fp32, 2e-2 bf16) accumulates over ~100 library
# calls through three BatchNorm'd heads; norm-wise per tensor and model.  The oracle continues from the
# matrices the device stored (a last-bit difference in a bf16 matrix entry near 1 is 2^-8 relative
# and moves every point of the cloud, after which argmax and ReLU decisions differ); the matrices
# themselves are compared to the oracle's own within four storage ulps.  The fp32 case is the sharp one
# (same wiring, same entry points except the one-operator tail, which has its own tests); in bf16 the
# error scales with the storage precision (fp32: 4e-5 observed; bf16 at 32 samples per head: 0.05-0.14 in the
# Frobenius norm, single entries up to 0.3 where a ReLU decision differs).  The oracle is the plain chain
# (it stores, i.e. rounds, the convolution output and the activation of every tail, where the device's
# one-operator tails round neither), so it also continues from the pooled features the device produced,
# after each has been checked against the oracle's own maximum.
TOL = {"f32": 5e-4, "bf16": 0.2}          # Frobenius norm of a gradient tensor; loss; parameters after Adam
TOL_MAX = {"f32": 5e-4, "bf16": 0.5}     # largest entry: a flipped argmax or ReLU moves single entries
# (the oracle's sub-networks are the plain chain, which stores the last per-point layer's output and its
# activation; the device's one-operator tail rounds neither: two more storage ulps on that path)
T_TOL = {"f32": 1e-5, "bf16": 4 * 2.0 ** -7}


def tspec(dtype, it=True, ft=True, L=260):
    # BatchNorm over the Nb samples of a head amplifies rounding noise; bf16 gets more samples
    cls = hi.PointNetClsSpec(name=f"t_{dtype}", B=2, Nb=8 if dtype == "f32" else 32, L=L, conv=(3, 64, 64, 128, 256), fc=(256, 64, 16),
                             fc_bn=True, dropout_p=0.3, dtype=dtype, config_index=1)
    return hi.PointNetTSpec(cls=cls, tnet_conv=(64, 128, 256), tnet_fc=(64, 32), input_transform=it, feature_transform=ft)


def noise_level_gradient(ts, name):
    """Biases in front of a BatchNorm (exactly zero gradient) and the shift of the BatchNorm in
    front of a max over points that feeds a Linear + BatchNorm (zero up to channels clipped by the ReLU)."""
    px, _, rest = name.rpartition("conv") if "conv" in name else name.rpartition("fc")
    if name.endswith(".b") and ".bn." not in name:
        if "conv" in name:
            return True
        nfc = len(ts.tnet_fc) + 1 if name.startswith("t") else len(ts.cls.fc) - 1
        return int(name.split("fc")[1][0]) < nfc - 1
    if name.endswith(".bn.b") and "conv" in name:
        last = len(ts.tnet_conv) - 1 if name.startswith("t") else len(ts.cls.conv) - 2
        return int(name.split("conv")[1][0]) == last
    return False


@pytest.mark.parametrize("dtype,it,ft", [("f32", True, True), ("bf16", True, True), ("bf16", True, False),
                                         ("f32", False, True)])
def test_transform_array_against_serial_oracle(dtype, it, ft):
    from paper_2102_02344_amd.arrays import FusedPointNetClsT
    ts = tspec(dtype, it, ft)
    print(f"pointnet with transforms {dtype} input={it} feature={ft}", flush=True)
    inp = hi.pointnet_t_inputs(ts)
    arr = FusedPointNetClsT(ts, inp)
    states = [opn.init_state(inp["params"][b]) for b in range(ts.cls.B)]
    tol = TOL[dtype]
    for t in (1, 2):
        arr.forward_backward()
        torch.cuda.synchronize()
        loss = arr.loss.cpu().numpy()
        Tg = [{tn["k"]: tn["T"][b].float().cpu().numpy().astype(np.float64) for tn in (arr.t_in, arr.t_feat) if tn is not None}
              for b in range(ts.cls.B)]
        # ... and from the device's three max-over-points (argmax positions and pooled values, each checked
        # against the oracle's own stored activations and maximum below; oracle/pointnet.py)
        chains = [("main", arr.rest)] + [(tn["k"], tn["chain"]) for tn in (arr.t_in, arr.t_feat) if tn is not None]
        Ig = [{key: (ch.pool_idx[b].cpu().numpy(), ch.pooled[b].float().cpu().numpy().astype(np.float64)) for key, ch in chains}
              for b in range(ts.cls.B)]
        outs = opt.array_train_step(ts, states, inp, t, T_given=Tg, idx_given=Ig)
        ptol = 1e-5 if dtype == "f32" else 2e-2
        for b in range(ts.cls.B):
            for key, _ in chains:
                own, v, ya = outs[b]["pools"][key]
                gi, gv = Ig[b][key]
                at = np.take_along_axis(ya, gi[:, :, None].astype(np.int64), axis=2)[:, :, 0]
                assert np.all(at >= v - ptol * (np.abs(v) + np.abs(ya).max())), (t, b, key)      # a near-tie of the oracle's maximum
                assert np.abs(gv - v).max() <= 3 * ptol * max(np.abs(v).max(), 1e-30), (t, b, key)   # pooled value, chain tolerance
        for b in range(ts.cls.B):
            assert abs(loss[b] - outs[b]["loss"]) <= tol * abs(outs[b]["loss"]), (t, b, loss[b], outs[b]["loss"])
            for k, key in ((3, "T3"), (ts.cls.conv[1], "T64")):
                if k in Tg[b]:
                    assert np.abs(Tg[b][k] - outs[b][key]).max() <= T_TOL[dtype] * max(1.0, np.abs(outs[b][key]).max()), (t, b, key)
            wmax = max(np.abs(outs[b]["grads"][n]).max() for n, _ in arr.shapes if n.endswith(".w"))
            for name, _ in arr.shapes:
                g = arr.param_host(arr.grad, name, b).astype(np.float64)
                ref = outs[b]["grads"][name]
                if noise_level_gradient(ts, name):
                    assert np.abs(g).max() <= 2e-2 * wmax and np.abs(ref).max() <= 2e-2 * wmax, (name, np.abs(g).max(), wmax)
                    continue
                err = np.abs(g - ref).max() / max(np.abs(ref).max(), 1e-30)
                errf = np.linalg.norm(g - ref) / max(np.linalg.norm(ref), 1e-30)
                assert errf <= tol and err <= TOL_MAX[dtype], (t, name, b, errf, err)
        arr.adam()
        torch.cuda.synchronize()
        for b in range(ts.cls.B):
            lr = float(inp["lr"][b])
            for name, _ in arr.shapes:
                if noise_level_gradient(ts, name):
                    continue
                th = arr.param_host(arr.theta, name, b).astype(np.float64)
                ref = states[b]["theta"][name].astype(np.float64)
                gref = outs[b]["grads"][name]
                ok = np.abs(gref) >= 1e-2 * np.abs(gref).max()      # Adam's early steps are ~lr*sign(g)
                assert np.abs(th - ref)[ok].max() <= max(tol * np.abs(ref).max(), 10 * tol * lr * t), (t, name, b)
                assert np.abs(th - ref).max() <= 2.5 * lr * t, (t, name, b)
        # the oracle continues from ITS parameters; keep the two sides together for step 2
        arr.load_params([{k: v for k, v in st["theta"].items()} for st in states])


def test_identity_transform_equals_plain_array():
    """Sub-networks whose last Linear is zero give identity matrices: the array's loss and the
    main network's gradients equal those of the array without sub-networks (same kernels, same bits,
    up to the storage rounding of the transformed tensors, which is exact for an identity)."""
    from paper_2102_02344_amd.arrays import FusedPointNetCls, FusedPointNetClsT
    ts = tspec("bf16")
    inp = hi.pointnet_t_inputs(ts)
    n = len(ts.tnet_fc)
    for p in inp["params"]:
        for k in (3, ts.cls.conv[1]):
            p[f"t{k}.fc{n}.w"][:] = 0
            p[f"t{k}.fc{n}.b"][:] = 0
    arr = FusedPointNetClsT(ts, inp)
    plain_inp = dict(inp, params=[{k: v for k, v in p.items() if not k.startswith("t")} for p in inp["params"]])
    plain = FusedPointNetCls(ts.cls, plain_inp)
    arr.forward_backward(); plain.forward_backward()
    torch.cuda.synchronize()
    eye = torch.eye(3, device="cuda", dtype=arr.t_in["T"].dtype).expand_as(arr.t_in["T"])
    assert torch.equal(arr.t_in["T"], eye)
    assert torch.equal(arr.loss, plain.loss)
    for name, _ in plain.shapes:
        if name.startswith("conv0."):
            # the first layer's two BatchNorm-backward reductions come from the next layer's kernel in the plain
            # array and from the layer's own pass here (its output goes through the feature transform first): another
            # fp32 summation order of two means, which moves single bf16 roundings of dz
            ref = "conv0.w" if name == "conv0.b" else name       # the bias gradient is a sum of dz that cancels: no scale of its own
            d, scale = (arr.g(name) - plain.g(name)).abs().max(), plain.g(ref).abs().max()
            assert float(d) <= 3e-4 * float(scale), name
            continue
        assert torch.equal(arr.g(name), plain.g(name)), name
    assert float(arr.g(f"t3.fc{n}.b").abs().max()) > 0
