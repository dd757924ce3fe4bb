"""hfta_linear_fwd_static, the entry point for callers that cannot allocate device memory: its
split partials live in a device array inside the library, so it takes no workspace.  Checked through
the C ABI against hfta_linear_fwd_ws (same kernels and split count: bit-equal) and against the oracle
at the stated tolerances, on two calls in a row, the second with a smaller input (the array keeps the
first call's contents)."""
import numpy as np
import pytest
import torch

import hfta_inputs as hi
from oracle import array as oa
from oracle import ops as oops
from util import DT, TDT, TOL, check, dev, host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_linear_fwd_static_matches_workspace_entry(dtype):
    from paper_2102_02344_amd import binding as hb
    # (B, M, Fx, Fy): config 1's first head layer, then a smaller, ragged one; both take the split path
    for case, (B, M, Fx, Fy) in enumerate([(8, 32, 1024, 512), (3, 5, 520, 72)]):
        print(f"linear_fwd_static {dtype} B={B} M={M} Fx={Fx} Fy={Fy}", flush=True)
        need = hb.linear_fwd_workspace_bytes(B, M, Fx, Fy, DT[dtype])
        assert 0 < need <= hb.linear_fwd_static_max_bytes()
        x = hi.normal(11 + case, (B, M, Fx), dtype)
        w = hi.normal(21 + case, (B, Fx, Fy), dtype, 1.0 / np.sqrt(Fx))
        b = hi.normal(31 + case, (B, Fy), dtype)
        X, W, Bi = dev(x, dtype), dev(w, dtype), dev(b, dtype)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        Yw = torch.empty((B, M, Fy), dtype=TDT[dtype], device="cuda")
        Ys = torch.full((B, M, Fy), float("nan"), dtype=TDT[dtype], device="cuda")
        hb.linear_fwd_ws(B, M, Fx, Fy, DT[dtype], X, W, Bi, Yw, hb.ACT_RELU, 0.0, ws)
        hb.linear_fwd_static(B, M, Fx, Fy, DT[dtype], X, W, Bi, Ys, hb.ACT_RELU, 0.0)
        torch.cuda.synchronize()
        assert torch.equal(Yw, Ys)
        check(host(Ys), oops.act_fwd(oa.linear_fwd(B, x, w, b), oops.ACT_RELU), TOL[dtype], "Y")


def test_linear_fwd_static_rejects_oversize_and_passes_unsplit_shapes():
    from paper_2102_02344_amd import binding as hb
    one = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(hb.HftaError) as e:
        hb.linear_fwd_static(9, 64, 8192, 2048, 1, one, one, None, one)
    assert e.value.status == hb.EWORKSPACE
    # many rows per model: no split, no scratch; equals hfta_linear_fwd
    B, M, Fx, Fy = 2, 200, 72, 136
    x = hi.normal(5, (B, M, Fx), "bf16")
    w = hi.normal(6, (B, Fx, Fy), "bf16", 1.0 / np.sqrt(Fx))
    X, W = dev(x, "bf16"), dev(w, "bf16")
    Y0 = torch.empty((B, M, Fy), dtype=torch.bfloat16, device="cuda")
    Y1 = torch.empty_like(Y0)
    assert hb.linear_fwd_workspace_bytes(B, M, Fx, Fy, 1) == 0
    hb.linear_fwd(B, M, Fx, Fy, 1, X, W, None, Y0)
    hb.linear_fwd_static(B, M, Fx, Fy, 1, X, W, None, Y1)
    torch.cuda.synchronize()
    assert torch.equal(Y0, Y1)
    check(host(Y1), oa.linear_fwd(B, x, w, None), TOL["bf16"], "Y")
