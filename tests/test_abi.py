"""The C-ABI library loads, exports every symbol include/hfta.h declares, and
rejects bad arguments before any launch (runs without a GPU)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2102_02344_amd import binding
    return binding


def declared_symbols():
    src = open(os.path.join(ROOT, "include", "hfta.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(hfta_[a-z0-9_]+)\s*\(", src)))


def test_exports_every_declared_symbol(lib):
    names = declared_symbols()
    assert len(names) >= 25
    raw = lib.raw()
    for n in names:
        assert hasattr(raw, n), n
    assert set(names) == set(lib.EXPORTS)
    assert lib.version() >= 100
    assert lib.status_string(0) == "ok" and "workspace" in lib.status_string(-3)


def test_validation_precedes_launch(lib):
    raw = lib.raw()
    s4 = (C.c_int64 * 4)(12, 24, 4, 1)
    bad_l = (C.c_int64 * 4)(12, 24, 4, 2)
    one = C.c_void_p(16)      # never dereferenced: validation fails first
    # B <= 0, null pointers, bad dtype
    assert raw.hfta_linear_fwd(0, 4, 4, 4, 0, one, one, None, one, 0, 0.0, None) == lib.EINVAL
    assert raw.hfta_linear_fwd(1, 4, 4, 4, 0, None, one, None, one, 0, 0.0, None) == lib.EINVAL
    assert raw.hfta_linear_fwd(1, 4, 4, 4, 7, one, one, None, one, 0, 0.0, None) == lib.EINVAL
    assert raw.hfta_linear_fwd(1, 4, 4, 4, 0, one, one, None, one, 99, 0.0, None) == lib.EINVAL
    assert raw.hfta_linear_fwd(1, 1 << 20, 1 << 12, 4, 0, one, one, None, one, 0, 0.0, None) == lib.EINVAL
    need = raw.hfta_linear_fwd_workspace_bytes(8, 32, 1024, 512, 1)
    assert need > 0 and raw.hfta_linear_fwd_workspace_bytes(8, 128, 1024, 512, 1) == 0
    assert raw.hfta_linear_fwd_ws(8, 32, 1024, 512, 1, one, one, None, one, 0, 0.0, one, need - 1, None) == lib.EWORKSPACE
    assert raw.hfta_linear_fwd_ws(8, 32, 1024, 512, 1, one, None, None, one, 0, 0.0, one, need, None) == lib.EINVAL
    # the entry point without a workspace: same validation; shapes whose partials exceed its built-in array
    assert raw.hfta_linear_fwd_static_max_bytes() == 8 << 20
    assert raw.hfta_linear_fwd_static(8, 32, 1024, 512, 1, one, None, None, one, 0, 0.0, None) == lib.EINVAL
    assert raw.hfta_linear_fwd_static(0, 32, 1024, 512, 1, one, one, None, one, 0, 0.0, None) == lib.EINVAL
    assert raw.hfta_linear_fwd_workspace_bytes(9, 64, 8192, 2048, 1) > 8 << 20
    assert raw.hfta_linear_fwd_static(9, 64, 8192, 2048, 1, one, one, None, one, 0, 0.0, None) == lib.EWORKSPACE
    # stride_l != 1 is not implemented for the conv family
    assert raw.hfta_conv1x1_fwd(1, 2, 3, 4, 4, 0, one, bad_l, one, None, one, s4, 0, 0.0, None) == lib.EUNSUPPORTED
    assert raw.hfta_conv1x1_fwd(1, 2, 3, 4, 4, 0, one, None, one, None, one, s4, 0, 0.0, None) == lib.EINVAL
    # workspace too small / missing
    need = raw.hfta_conv1x1_bwd_workspace_bytes(8, 32, 128, 1024, 2500, 1)
    assert need > 0
    assert raw.hfta_conv1x1_bwd(8, 32, 128, 1024, 2500, 1, one, s4, one, one, s4, None, None, one, None,
                                None, 0, None) == lib.EWORKSPACE
    assert raw.hfta_conv1x1_bwd(8, 32, 128, 1024, 2500, 1, one, s4, one, one, s4, None, None, one, None,
                                one, need - 1, None) == lib.EWORKSPACE
    assert raw.hfta_bn_fwd(1, 2, 3, 4, 0, one, bad_l, one, one, 1e-5, 0.1, None, None, one, one, one, bad_l,
                           0, 0.0, None) == lib.EUNSUPPORTED
    assert raw.hfta_bn_fwd(1, 2, 3, 4, 0, one, s4, one, one, 1e-5, 0.1, one, None, one, one, one, s4,
                           0, 0.0, None) == lib.EINVAL
    assert raw.hfta_bn_fwd(1, 2, 3, 4, 0, one, s4, one, one, 1e-5, 0.1, None, None, one, one, one, s4,
                           lib.ACT_TANH, 0.0, None) == lib.EUNSUPPORTED
    assert raw.hfta_bn_eval_fwd(1, 2, 3, 4, 0, one, s4, one, one, one, None, 1e-5, one, s4, 0, 0.0, None) == lib.EINVAL
    assert raw.hfta_bn_eval_fwd(1, 2, 3, 4, 0, one, bad_l, one, one, one, one, 1e-5, one, bad_l, 0, 0.0, None) == lib.EUNSUPPORTED
    assert raw.hfta_bn_eval_fwd(1, 2, 3, 4, 0, one, s4, one, one, one, one, 1e-5, one, s4, lib.ACT_GELU, 0.0, None) == lib.EUNSUPPORTED
    assert raw.hfta_adam_step(2, 8, 0, one, one, one, one, None, one, one, one, one, one, 0, 0, None) == lib.EINVAL
    assert raw.hfta_adam_step(2, 0, 0, one, one, one, one, None, one, one, one, one, one, 1, 0, None) == lib.EINVAL
    assert raw.hfta_maxpool_points(1, 1, 1, 0, 0, one, s4, one, one, (C.c_int64 * 3)(1, 1, 1), None) == lib.EINVAL
    assert raw.hfta_dropout(8, 0, one, one, 1.0, one, None) == lib.EINVAL
    assert raw.hfta_act_bwd(8, 0, one, one, one, lib.ACT_GELU, 0.0, 1, None) == lib.EUNSUPPORTED
    assert raw.hfta_layernorm_bwd(1, 4, 8, 0, one, one, one, one, one, one, one, one, None, 0, None) == lib.EWORKSPACE


def test_validation_of_the_wider_entry_points(lib):
    """One-operator tail, segmentation support operators, Adadelta / StepLR, Embedding / attention,
    point transform: bad arguments come back as status codes before anything is launched."""
    raw = lib.raw()
    one = C.c_void_p(256)
    s4 = (C.c_int64 * 4)(128 * 2500, 8 * 128 * 2500, 2500, 1)
    bad_l = (C.c_int64 * 4)(128 * 2500, 8 * 128 * 2500, 2500, 2)
    v3 = (C.c_int64 * 3)(32 * 1024, 1024, 1)
    # ---- conv + BatchNorm + max over points as one operator
    assert raw.hfta_conv1x1_bn_maxpool_fwd_workspace_bytes(8, 32, 128, 1024, 2500, 1) > 0
    assert raw.hfta_conv1x1_bn_maxpool_fwd_workspace_bytes(8, 32, 128, 1024, 2500, 0) == 0      # fp32: not built
    assert raw.hfta_conv1x1_bn_maxpool_fwd_workspace_bytes(8, 32, 136, 1024, 2500, 1) == 0      # Ci > 128
    assert raw.hfta_conv1x1_bn_maxpool_fwd_workspace_bytes(8, 32, 128, 1024, 2502, 1) == 0      # L % 4
    assert raw.hfta_conv1x1_bn_maxpool_saved_floats(8, 128, 1024) == 8 * (128 * 128 + 128 + 1024 * 128)

    def tail_fwd(B=8, Nb=32, Ci=128, Co=1024, L=2500, dt=1, X=one, xs=s4, act=1, ws=one, nws=1 << 40):
        return raw.hfta_conv1x1_bn_maxpool_fwd(B, Nb, Ci, Co, L, dt, X, xs, one, None, one, one, 1e-5, 0.1, None,
                                               None, one, one, one, one, v3, one, None, act, 0.0, ws, nws, None)
    assert tail_fwd(X=None) == lib.EINVAL
    assert tail_fwd(B=0) == lib.EINVAL
    assert tail_fwd(dt=0) == lib.EUNSUPPORTED
    assert tail_fwd(Ci=136) == lib.EUNSUPPORTED
    assert tail_fwd(Co=1032) == lib.EUNSUPPORTED
    assert tail_fwd(L=2502) == lib.EUNSUPPORTED
    assert tail_fwd(xs=bad_l) == lib.EUNSUPPORTED
    assert tail_fwd(act=lib.ACT_TANH) == lib.EUNSUPPORTED
    assert tail_fwd(ws=None, nws=0) == lib.EWORKSPACE
    assert tail_fwd(nws=1024) == lib.EWORKSPACE

    def tail_bwd(Z=None, zhit=one, ws=one, nws=1 << 40, dt=1):
        return raw.hfta_conv1x1_bn_maxpool_bwd(8, 32, 128, 1024, 2500, dt, one, s4, one, None, Z, s4 if Z else None,
                                               zhit, None, one, one, v3, one, one, one, one, one, s4, one, None,
                                               one, one, 1, 0.0, ws, nws, None)
    assert tail_bwd(Z=one, zhit=one) == lib.EINVAL            # exactly one of Z / zhit
    assert tail_bwd(Z=None, zhit=None) == lib.EINVAL
    assert tail_bwd(dt=0) == lib.EUNSUPPORTED
    assert tail_bwd(ws=None, nws=0) == lib.EWORKSPACE

    # the same tail with its input normalised on load
    def tailp_fwd(ig=one, in_act=1, dt=1, ws=one, nws=1 << 40, xs=s4, xa=None, xas=None):
        return raw.hfta_conv1x1_bn_maxpool_prenorm_fwd(8, 32, 128, 1024, 2500, dt, one, xs, ig, one, one, one, in_act, 0.0,
                                                       one, None, one, one, 1e-5, 0.1, None, None, one, one, one, one,
                                                       v3, one, None, 1, 0.0, xa, xas, ws, nws, None)
    assert tailp_fwd(xa=one, xas=None) == lib.EINVAL
    assert tailp_fwd(xa=one, xas=bad_l) == lib.EUNSUPPORTED
    assert tailp_fwd(xa=C.c_void_p(258), xas=s4) == lib.EUNSUPPORTED          # 8-byte alignment
    assert tailp_fwd(ig=None) == lib.EINVAL
    assert tailp_fwd(in_act=lib.ACT_TANH) == lib.EUNSUPPORTED
    assert tailp_fwd(dt=0) == lib.EUNSUPPORTED
    assert tailp_fwd(xs=bad_l) == lib.EUNSUPPORTED
    assert tailp_fwd(ws=None, nws=0) == lib.EWORKSPACE

    def tailp_bwd(ig=one, in_act=1, zhit=one, ws=one, nws=1 << 40):
        return raw.hfta_conv1x1_bn_maxpool_prenorm_bwd(8, 32, 128, 1024, 2500, 1, one, s4, ig, one, one, one, in_act, 0.0,
                                                       one, None, zhit, None, one, one, v3, one, one, one, one, one, s4,
                                                       one, None, one, one, 1, 0.0, ws, nws, None)
    assert tailp_bwd(ig=None) == lib.EINVAL
    assert tailp_bwd(zhit=None) == lib.EINVAL
    assert tailp_bwd(in_act=lib.ACT_TANH) == lib.EUNSUPPORTED
    assert tailp_bwd(ws=None, nws=0) == lib.EWORKSPACE

    # ---- normalisation with given statistics
    def bn_apply(B=8, mean=one, xs=s4, act=1):
        return raw.hfta_bn_apply_fwd(B, 32, 128, 2500, 1, one, xs, one, one, mean, one, one, s4, act, 0.0, None)
    assert bn_apply(B=0) == lib.EINVAL
    assert bn_apply(mean=None) == lib.EINVAL
    assert bn_apply(xs=bad_l) == lib.EUNSUPPORTED
    assert bn_apply(act=lib.ACT_TANH) == lib.EUNSUPPORTED

    # ---- conv + BatchNorm as one call per direction
    assert raw.hfta_conv1x1_bn_fwd_workspace_bytes(8, 32, 64, 64, 2500, 1) == 8 * 32 * 20 * 64 * 2 * 4
    assert raw.hfta_conv1x1_bn_fwd_workspace_bytes(8, 32, 64, 64, 2500, 0) == 0               # fp32: the two operators, no workspace
    assert raw.hfta_conv1x1_bn_bwd_one_pass(8, 32, 64, 128, 2500, 1) == 1
    assert raw.hfta_conv1x1_bn_bwd_one_pass(8, 32, 64, 128, 2500, 0) == 0                     # fp32
    assert raw.hfta_conv1x1_bn_bwd_one_pass(8, 32, 128, 136, 2500, 1) == 0                    # Co > 128
    assert raw.hfta_conv1x1_bn_bwd_one_pass(8, 32, 64, 64, 2502, 1) == 0                      # L % 4
    assert raw.hfta_conv1x1_bn_bwd_one_pass(0, 32, 64, 64, 2500, 1) == 0
    small = raw.hfta_conv1x1_bn_bwd_workspace_bytes(8, 32, 64, 64, 2500, 1)
    assert 0 < small < 8 * 32 * 64 * 2500 * 2                  # constants and partials, not a dz-sized buffer
    assert raw.hfta_conv1x1_bn_bwd_workspace_bytes(8, 32, 64, 64, 2500, 0) > 8 * 32 * 64 * 2500 * 4     # the two operators: dz + theirs
    s64 = (C.c_int64 * 4)(64 * 2500, 8 * 64 * 2500, 2500, 1)
    bad64 = (C.c_int64 * 4)(64 * 2500, 8 * 64 * 2500, 2500, 2)

    def cb_fwd(B=8, X=one, xs=s64, rm=None, rv=None, act=1, eps=1e-5):
        return raw.hfta_conv1x1_bn_fwd(B, 32, 64, 64, 2500, 1, X, xs, one, None, one, one, eps, 0.1, rm, rv, one, one,
                                       one, s64, one, s64, act, 0.0, None, 0, None)
    assert cb_fwd(X=None) == lib.EINVAL
    assert cb_fwd(B=0) == lib.EINVAL
    assert cb_fwd(rm=one) == lib.EINVAL                        # running statistics come as a pair
    assert cb_fwd(eps=-1.0) == lib.EINVAL
    assert cb_fwd(act=lib.ACT_TANH) == lib.EUNSUPPORTED
    assert cb_fwd(xs=bad64) == lib.EUNSUPPORTED

    def cb_bwd(B=8, Z=one, dX=one, W=one, dxs=s64, dW=one, act=1, ws=one, nws=1 << 40, dys=s64):
        return raw.hfta_conv1x1_bn_bwd(B, 32, 64, 64, 2500, 1, one, s64, W, Z, s64, one, dys, one, one, one, one,
                                       dX, dxs, dW, None, one, one, None, act, 0.0, ws, nws, None)
    assert cb_bwd(Z=None) == lib.EINVAL
    assert cb_bwd(B=0) == lib.EINVAL
    assert cb_bwd(dW=None) == lib.EINVAL
    assert cb_bwd(W=None) == lib.EINVAL                        # a data gradient needs the weights ...
    assert cb_bwd(dxs=None) == lib.EINVAL                      # ... and its strides
    assert cb_bwd(act=lib.ACT_GELU) == lib.EUNSUPPORTED
    assert cb_bwd(dys=bad64) == lib.EUNSUPPORTED
    assert cb_bwd(ws=None, nws=0) == lib.EWORKSPACE
    assert cb_bwd(nws=small - 1) == lib.EWORKSPACE

    # ---- ... and with the input given as the previous block's stored pre-activation
    assert raw.hfta_conv1x1_bn_prenorm_supported(8, 32, 64, 128, 2500, 1) == 1
    assert raw.hfta_conv1x1_bn_prenorm_supported(8, 32, 64, 128, 2500, 0) == 0                # fp32
    assert raw.hfta_conv1x1_bn_prenorm_supported(8, 32, 3, 64, 2500, 1) == 0                  # Ci % 8
    assert raw.hfta_conv1x1_bn_prenorm_supported(8, 32, 128, 1024, 2500, 1) == 0              # Co > 128
    assert raw.hfta_conv1x1_bn_prenorm_supported(8, 32, 64, 32, 2500, 1) == 0                 # Co < 64
    assert raw.hfta_conv1x1_bn_fwd(8, 32, 64, 64, 2500, 0, one, s64, one, None, one, one, 1e-5, 0.1, None, None, one, one,
                                   one, s64, one, None, 1, 0.0, None, 0, None) == lib.EINVAL   # an output without strides

    def pn_fwd(dt=1, Ci=64, ig=one, in_act=1, ws=one, nws=1 << 40, Y=None, ys=None):
        return raw.hfta_conv1x1_bn_prenorm_fwd(8, 32, Ci, 64, 2500, dt, one, s64, ig, one, one, one, in_act, 0.0, one, None,
                                               one, one, 1e-5, 0.1, None, None, one, one, one, s64, Y, ys, 1, 0.0, ws, nws, None)
    assert pn_fwd(ig=None) == lib.EINVAL
    assert pn_fwd(Y=one, ys=None) == lib.EINVAL
    assert pn_fwd(dt=0) == lib.EUNSUPPORTED
    assert pn_fwd(Ci=60) == lib.EUNSUPPORTED
    assert pn_fwd(in_act=lib.ACT_TANH) == lib.EUNSUPPORTED
    assert pn_fwd(ws=None, nws=0) == lib.EWORKSPACE

    def pn_bwd(dt=1, ig=one, dW=one, W=one, ws=one, nws=1 << 40, dX=one, isum=None, Ci=64):
        return raw.hfta_conv1x1_bn_prenorm_bwd(8, 32, Ci, 64, 2500, dt, one, s64, ig, one, one, one, 1, 0.0, W, one, s64, one,
                                               s64, one, one, one, one, dX, s64, dW, None, one, one, None, isum, 1, 0.0, ws,
                                               nws, None)
    assert raw.hfta_conv1x1_bn_prenorm_bwd_gives_sums(8, 32, 64, 128, 2500, 1) == 1
    assert raw.hfta_conv1x1_bn_prenorm_bwd_gives_sums(8, 32, 128, 128, 2500, 1) == 0          # Ci > 64
    assert raw.hfta_conv1x1_bn_prenorm_bwd_gives_sums(8, 32, 64, 128, 2500, 0) == 0           # fp32
    assert pn_bwd(isum=one, dX=None) == lib.EINVAL             # the sums are taken where dX is stored
    assert pn_bwd(isum=one, Ci=128) == lib.EUNSUPPORTED
    assert pn_bwd(ig=None) == lib.EINVAL
    assert pn_bwd(dW=None) == lib.EINVAL
    assert pn_bwd(W=None) == lib.EINVAL
    assert pn_bwd(dt=0) == lib.EUNSUPPORTED
    assert pn_bwd(nws=small - 1) == lib.EWORKSPACE

    # ---- strided support operators of the segmentation head
    c3 = (C.c_int64 * 3)(16 * 64, 64, 1)
    assert raw.hfta_add_sample_bias(1, 2, 64, 0, 1, one, s4, one, c3, one, s4, None) == lib.EINVAL
    assert raw.hfta_add_sample_bias(1, 2, 64, 8, 1, one, bad_l, one, c3, one, s4, None) == lib.EUNSUPPORTED
    assert raw.hfta_sum_points(1, 2, 64, 8, 1, None, s4, one, c3, None) == lib.EINVAL
    assert raw.hfta_add_strided(1, 2, 64, 8, 9, one, s4, one, s4, one, s4, None) == lib.EINVAL
    assert raw.hfta_maxpool_points_bwd_add(1, 2, 64, 8, 1, one, None, c3, one, s4, None) == lib.EINVAL
    need = raw.hfta_softmax_xent_points_workspace_bytes(6, 16, 2500)
    assert need > 0
    assert raw.hfta_softmax_xent_points(6, 16, 50, 2500, 1, one, s4, one, one, one, s4, one, need - 1,
                                        None) == lib.EWORKSPACE
    assert raw.hfta_softmax_xent_points(6, 16, 0, 2500, 1, one, s4, one, one, one, s4, one, need, None) == lib.EINVAL

    # ---- Adadelta and the step schedule
    offs = (C.c_int64 * 3)(0, 8, 24)
    bad_offs = (C.c_int64 * 3)(0, 8, 8)
    assert raw.hfta_adadelta_step_multi(0, 2, offs, 0, one, one, one, one, None, one, one, one, one, None) == lib.EINVAL
    assert raw.hfta_adadelta_step_multi(2, 2, bad_offs, 0, one, one, one, one, None, one, one, one, one,
                                        None) == lib.EINVAL
    assert raw.hfta_adadelta_step_multi(2, 2, offs, 0, one, one, None, one, None, one, one, one, one, None) == lib.EINVAL
    assert raw.hfta_adadelta_step_multi(2, 10 ** 6, offs, 0, one, one, one, one, None, one, one, one, one,
                                        None) in (lib.EINVAL, lib.EUNSUPPORTED)
    assert raw.hfta_steplr(0, one, one, one, 3, one, None) == lib.EINVAL
    assert raw.hfta_steplr(4, one, one, one, -1, one, None) == lib.EINVAL
    assert raw.hfta_steplr(4, one, None, one, 3, one, None) == lib.EINVAL

    # ---- element-wise backward operators with reductions folded in
    assert raw.hfta_act_bwd_colsum(0, 64, 64, 1, one, one, one, one, 1, 0.0, None) == lib.EINVAL
    assert raw.hfta_act_bwd_colsum(2, 64, 64, 1, one, None, one, one, 1, 0.0, None) == lib.EINVAL
    assert raw.hfta_act_bwd_colsum(2, 64, 64, 1, one, one, one, None, 1, 0.0, None) == lib.EINVAL
    assert raw.hfta_act_bwd_colsum(2, 64, 64, 1, one, one, one, one, 99, 0.0, None) == lib.EINVAL
    assert raw.hfta_act_bwd_colsum(2, 64, 100, 1, one, one, one, one, 1, 0.0, None) == lib.EUNSUPPORTED   # 100 bf16: no whole pieces
    assert raw.hfta_act_bwd_colsum(2, 64, 64, 1, C.c_void_p(264), one, one, one, 1, 0.0, None) == lib.EUNSUPPORTED  # 8-byte aligned
    need = raw.hfta_layernorm_bwd_sums_workspace_bytes(2, 64, 512)
    assert need > raw.hfta_layernorm_bwd_workspace_bytes(2, 64, 512) > 0

    def ln_sums(B=2, E=512, X=one, dxs=one, ws=one, nws=need, dy2=None):
        return raw.hfta_layernorm_bwd_sums(B, 64, E, 1, X, one, dy2, one, one, one, one, one, one, dxs, ws, nws, None)
    assert ln_sums(B=0) == lib.EINVAL
    assert ln_sums(X=None) == lib.EINVAL
    assert ln_sums(dxs=None) == lib.EINVAL
    assert ln_sums(ws=None) == lib.EWORKSPACE
    assert ln_sums(nws=need - 1) == lib.EWORKSPACE
    assert ln_sums(E=100, nws=1 << 30) == lib.EUNSUPPORTED            # 100 bf16: no whole pieces
    assert ln_sums(E=2048, nws=1 << 30) == lib.EUNSUPPORTED           # more than 128 pieces per row
    assert ln_sums(dy2=C.c_void_p(264)) == lib.EUNSUPPORTED           # second gradient only 8-byte aligned

    # ---- Embedding, attention core, wide-class cross-entropy, per-sample point transform
    assert raw.hfta_embedding_fwd(2, 64, 0, 32, 1, one, one, 1.0, None, 0, one, None) == lib.EINVAL
    assert raw.hfta_embedding_bwd(2, 7681, 100, 32, 1, one, one, 1.0, one, None) == lib.EUNSUPPORTED
    assert raw.hfta_attention_fwd(2, 4, 16, 30, 4, 1, one, one, one, 1, None) == lib.EINVAL          # E % H
    assert raw.hfta_attention_fwd(64, 128, 16, 32, 16, 1, one, one, one, 1, None) == lib.EUNSUPPORTED  # B*N*H
    need = raw.hfta_attention_bwd_workspace_bytes(2, 4, 16, 32, 4, 1)
    assert need > 0
    assert raw.hfta_attention_bwd(2, 4, 16, 32, 4, 1, one, one, one, one, one, need - 1, None) == lib.EWORKSPACE
    need = raw.hfta_softmax_xent_rows_workspace_bytes(2, 64)
    assert need > 0
    assert raw.hfta_softmax_xent_rows(2, 64, 1000, 1, one, one, one, one, None, 0, None) == lib.EWORKSPACE
    assert raw.hfta_softmax_xent_rows(2, 64, 0, 1, one, one, one, one, one, need, None) == lib.EINVAL
    assert raw.hfta_point_transform_fwd(1, 2, 64, 64, 8, 1, one, bad_l, one, one, s4, None) == lib.EUNSUPPORTED
    assert raw.hfta_point_transform_fwd(300, 300, 64, 64, 8, 1, one, s4, one, one, s4, None) == lib.EUNSUPPORTED
    assert raw.hfta_point_transform_bwd(1, 2, 64, 64, 8, 1, one, s4, one, None, s4, one, s4, one, None) == lib.EINVAL
