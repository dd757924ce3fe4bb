"""Thin ctypes binding over libhfta.so: argument marshalling only.

Every function has the name and argument order of its C entry point in
``include/hfta.h``; tensors are ``torch`` CUDA tensors (used for device memory
and streams only) or ``None``; stride arguments are Python sequences.  A
non-zero status raises ``HftaError``.  There is no CPU fallback: if the library
is missing the import fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhfta.so")

F32, BF16 = 0, 1
ACT_NONE, ACT_RELU, ACT_LEAKY, ACT_TANH, ACT_GELU = 0, 1, 2, 3, 4
OK, EINVAL, EUNSUPPORTED, EWORKSPACE, ELAUNCH = 0, -1, -2, -3, -4


class HftaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2102_02344_amd.build` "
                          "(or __graft_entry__.build()) first")
    return C.CDLL(LIB_PATH)


_lib = _load()

_i, _i64, _f, _p, _sz = C.c_int, C.c_int64, C.c_float, C.c_void_p, C.c_size_t
_s4 = C.POINTER(C.c_int64)

_SIGS = {
    "hfta_status_string": (C.c_char_p, [_i]),
    "hfta_version": (_i, []),
    "hfta_linear_fwd": (_i, [_i, _i, _i, _i, _i, _p, _p, _p, _p, _i, _f, _p]),
    "hfta_linear_fwd_workspace_bytes": (_sz, [_i, _i, _i, _i, _i]),
    "hfta_linear_fwd_ws": (_i, [_i, _i, _i, _i, _i, _p, _p, _p, _p, _i, _f, _p, _sz, _p]),
    "hfta_linear_fwd_static_max_bytes": (_sz, []),
    "hfta_linear_fwd_static": (_i, [_i, _i, _i, _i, _i, _p, _p, _p, _p, _i, _f, _p]),
    "hfta_linear_bwd_workspace_bytes": (_sz, [_i, _i, _i, _i, _i]),
    "hfta_linear_bwd": (_i, [_i, _i, _i, _i, _i, _p, _p, _p, _p, _p, _p, _p, _sz, _p]),
    "hfta_conv1x1_fwd": (_i, [_i, _i, _i, _i, _i, _i, _p, _s4, _p, _p, _p, _s4, _i, _f, _p]),
    "hfta_conv1x1_fwd_sample_bias": (_i, [_i, _i, _i, _i, _i, _i, _p, _s4, _p, _p, _s4, _p, _s4, _i, _f, _p]),
    "hfta_conv1x1_bn_fwd_workspace_bytes": (_sz, [_i, _i, _i, _i, _i, _i]),
    "hfta_conv1x1_bn_fwd": (_i, [_i, _i, _i, _i, _i, _i, _p, _s4, _p, _p, _p, _p, _f, _f, _p, _p, _p, _p, _p, _s4, _p, _s4,
                                 _i, _f, _p, _sz, _p]),
    "hfta_conv1x1_bn_bwd_one_pass": (_i, [_i, _i, _i, _i, _i, _i]),
    "hfta_conv1x1_bn_bwd_workspace_bytes": (_sz, [_i, _i, _i, _i, _i, _i]),
    "hfta_conv1x1_bn_bwd": (_i, [_i, _i, _i, _i, _i, _i, _p, _s4, _p, _p, _s4, _p, _s4, _p, _p, _p, _p, _p, _s4, _p, _p, _p, _p,
                                 _p, _i, _f, _p, _sz, _p]),
    "hfta_conv1x1_bn_prenorm_supported": (_i, [_i, _i, _i, _i, _i, _i]),
    "hfta_conv1x1_bn_prenorm_fwd": (_i, [_i, _i, _i, _i, _i, _i, _p, _s4, _p, _p, _p, _p, _i, _f, _p, _p, _p, _p, _f, _f, _p, _p,
                                         _p, _p, _p, _s4, _p, _s4, _i, _f, _p, _sz, _p]),
    "hfta_conv1x1_bn_prenorm_bwd": (_i, [_i, _i, _i, _i, _i, _i, _p, _s4, _p, _p, _p, _p, _i, _f, _p, _p, _s4, _p, _s4, _p, _p, _p,
                                         _p, _p, _s4, _p, _p, _p, _p, _p, _p, _i, _f, _p, _sz, _p]),
    "hfta_conv1x1_bn_prenorm_bwd_gives_sums": (_i, [_i, _i, _i, _i, _i, _i]),
    "hfta_conv1x1_bwd_workspace_bytes": (_sz, [_i, _i, _i, _i, _i, _i]),
    "hfta_conv1x1_bwd": (_i, [_i, _i, _i, _i, _i, _i, _p, _s4, _p, _p, _s4, _p, _s4, _p, _p, _p, _sz, _p]),
    "hfta_conv2d_grouped_fwd": (_i, [_i] * 11 + [_p, _p, _p, _p, _i, _f, _p, _sz, _p]),
    "hfta_conv2d_grouped_fwd_workspace_bytes": (_sz, [_i] * 11),
    "hfta_conv2d_grouped_bwd_min_workspace_bytes": (_sz, [_i] * 11),
    "hfta_conv2d_grouped_bwd_workspace_bytes": (_sz, [_i] * 11),
    "hfta_conv2d_grouped_bwd": (_i, [_i] * 11 + [_p, _p, _p, _p, _p, _p, _p, _sz, _p]),
    "hfta_bn_fwd": (_i, [_i, _i, _i, _i, _i, _p, _s4, _p, _p, _f, _f, _p, _p, _p, _p, _p, _s4, _i, _f, _p]),
    "hfta_bn_apply_fwd": (_i, [_i, _i, _i, _i, _i, _p, _s4, _p, _p, _p, _p, _p, _s4, _i, _f, _p]),
    "hfta_bn_eval_fwd": (_i, [_i, _i, _i, _i, _i, _p, _s4, _p, _p, _p, _p, _f, _p, _s4, _i, _f, _p]),
    "hfta_bn_bwd": (_i, [_i, _i, _i, _i, _i, _p, _s4, _p, _s4, _p, _p, _p, _p, _p, _s4, _p, _p, _p, _i, _f, _p]),
    "hfta_bn_fwd_maxpool": (_i, [_i, _i, _i, _i, _i, _p, _s4, _p, _p, _f, _f, _p, _p, _p, _p, _p, _p, _s4, _i, _f, _p]),
    "hfta_bn_bwd_maxpool": (_i, [_i, _i, _i, _i, _i, _p, _s4, _p, _p, _s4, _p, _p, _p, _p, _p, _s4, _p, _p, _p, _i, _f, _p]),
    "hfta_conv1x1_bn_maxpool_bwd_workspace_bytes": (_sz, [_i] * 6),
    "hfta_conv1x1_bn_maxpool_bwd": (_i, [_i] * 6 + [_p] * 21 + [_i, _f, _p, _sz, _p]),
    "hfta_conv1x1_bn_maxpool_prenorm_fwd": (_i, [_i] * 6 + [_p] * 6 + [_i, _f] + [_p] * 4 + [_f, _f] + [_p] * 9 + [_i, _f, _p, _s4, _p, _sz, _p]),
    "hfta_conv1x1_bn_maxpool_prenorm_bwd": (_i, [_i] * 6 + [_p] * 6 + [_i, _f] + [_p] * 17 + [_i, _f, _p, _sz, _p]),
    "hfta_point_transform_fwd": (_i, [_i] * 6 + [_p] * 6),
    "hfta_point_transform_bwd": (_i, [_i] * 6 + [_p] * 9),
    "hfta_softmax_xent_rows_workspace_bytes": (_sz, [_i, _i]),
    "hfta_softmax_xent_rows": (_i, [_i] * 4 + [_p] * 5 + [_sz, _p]),
    "hfta_embedding_fwd": (_i, [_i] * 5 + [_p, _p, _f, _p, _i, _p, _p]),
    "hfta_embedding_bwd": (_i, [_i] * 5 + [_p, _p, _f, _p, _p]),
    "hfta_attention_fwd": (_i, [_i] * 6 + [_p, _p, _p, _i, _p]),
    "hfta_attention_bwd_workspace_bytes": (_sz, [_i] * 6),
    "hfta_attention_bwd": (_i, [_i] * 6 + [_p, _p, _p, _p, _p, _sz, _p]),
    "hfta_adadelta_step_multi": (_i, [_i, _i, _s4, _i] + [_p] * 9 + [_p]),
    "hfta_steplr": (_i, [_i, _p, _p, _p, _i, _p, _p]),
    "hfta_add_sample_bias": (_i, [_i] * 5 + [_p] * 7),
    "hfta_sum_points": (_i, [_i] * 5 + [_p] * 5),
    "hfta_add_strided": (_i, [_i] * 5 + [_p] * 7),
    "hfta_maxpool_points_bwd_add": (_i, [_i] * 5 + [_p] * 6),
    "hfta_softmax_xent_points_workspace_bytes": (_sz, [_i] * 3),
    "hfta_softmax_xent_points": (_i, [_i] * 5 + [_p] * 7 + [_sz, _p]),
    "hfta_conv1x1_bn_maxpool_saved_floats": (_sz, [_i] * 3),
    "hfta_conv1x1_bn_maxpool_fwd_workspace_bytes": (_sz, [_i] * 6),
    "hfta_conv1x1_bn_maxpool_fwd": (_i, [_i] * 6 + [_p] * 6 + [_f, _f] + [_p] * 9 + [_i, _f, _p, _sz, _p]),
    "hfta_maxpool_points": (_i, [_i, _i, _i, _i, _i, _p, _s4, _p, _p, _s4, _p]),
    "hfta_maxpool_points_bwd": (_i, [_i, _i, _i, _i, _i, _p, _p, _s4, _p, _s4, _p]),
    "hfta_adam_step": (_i, [_i, _i64, _i, _p, _p, _p, _p, _p, _p, _p, _p, _p, _p, _i, _i, _p]),
    "hfta_adam_step_multi": (_i, [_i, _i, _s4, _i, _p, _p, _p, _p, _p, _p, _p, _p, _p, _p, _i, _i, _p]),
    "hfta_act_fwd": (_i, [_i64, _i, _p, _p, _i, _f, _p]),
    "hfta_act_bwd": (_i, [_i64, _i, _p, _p, _p, _i, _f, _i, _p]),
    "hfta_act_bwd_colsum": (_i, [_i, _i, _i, _i, _p, _p, _p, _p, _i, _f, _p]),
    "hfta_bias_act_nchw": (_i, [_i64, _i64, _i64, _i, _p, _p, _i, _f, _p]),
    "hfta_dropout": (_i, [_i64, _i, _p, _p, _f, _p, _p]),
    "hfta_add": (_i, [_i64, _i, _p, _p, _p, _p]),
    "hfta_layernorm_fwd": (_i, [_i, _i, _i, _i, _p, _p, _p, _f, _p, _p, _p, _p]),
    "hfta_layernorm_bwd_workspace_bytes": (_sz, [_i, _i, _i]),
    "hfta_layernorm_bwd": (_i, [_i, _i, _i, _i, _p, _p, _p, _p, _p, _p, _p, _p, _p, _sz, _p]),
    "hfta_layernorm_bwd_sums_workspace_bytes": (_sz, [_i, _i, _i]),
    "hfta_layernorm_bwd_sums": (_i, [_i, _i, _i, _i, _p, _p, _p, _p, _p, _p, _p, _p, _p, _p, _p, _sz, _p]),
    "hfta_softmax_xent": (_i, [_i, _i, _i, _i, _p, _p, _p, _p, _p]),
    "hfta_bce_logits": (_i, [_i, _i64, _i, _p, _p, _p, _p, _p]),
    "hfta_bce_logits_strided": (_i, [_i, _i64, _i, _p, _p, _p, _p, _i64, _i64, _p]),
    "hfta_mse": (_i, [_i, _i64, _i, _p, _p, _p, _p, _p]),
}
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(_lib, _name)
    _fn.restype, _fn.argtypes = _res, _args

EXPORTS = tuple(_SIGS)


def status_string(status: int) -> str:
    return _lib.hfta_status_string(int(status)).decode()


def version() -> int:
    return _lib.hfta_version()


def _ptr(t) -> Optional[int]:
    """Device pointer of a tensor (None -> NULL); raw ints pass through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _strides(s: Optional[Sequence[int]], n: int = 4):
    if s is None:
        return None
    assert len(s) == n, (s, n)
    return (C.c_int64 * n)(*[int(v) for v in s])


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _check(rc: int, where: str) -> None:
    if rc != OK:
        raise HftaError(rc, where)


def _ws(workspace):
    if workspace is None:
        return None, 0
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


# ---------------------------------------------------------------- entry points
def linear_fwd(B, M, Fx, Fy, dtype, X, W, bias, Y, act=ACT_NONE, act_slope=0.0, stream=None):
    _check(_lib.hfta_linear_fwd(B, M, Fx, Fy, dtype, _ptr(X), _ptr(W), _ptr(bias), _ptr(Y), act, act_slope,
                                _stream(stream)), "hfta_linear_fwd")


def linear_fwd_workspace_bytes(B, M, Fx, Fy, dtype) -> int:
    return _lib.hfta_linear_fwd_workspace_bytes(B, M, Fx, Fy, dtype)


def linear_fwd_ws(B, M, Fx, Fy, dtype, X, W, bias, Y, act=ACT_NONE, act_slope=0.0, workspace=None, stream=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_linear_fwd_ws(B, M, Fx, Fy, dtype, _ptr(X), _ptr(W), _ptr(bias), _ptr(Y), act, act_slope,
                                   wp, wb, _stream(stream)), "hfta_linear_fwd_ws")


def linear_fwd_static_max_bytes() -> int:
    return _lib.hfta_linear_fwd_static_max_bytes()


def linear_fwd_static(B, M, Fx, Fy, dtype, X, W, bias, Y, act=ACT_NONE, act_slope=0.0, stream=None):
    _check(_lib.hfta_linear_fwd_static(B, M, Fx, Fy, dtype, _ptr(X), _ptr(W), _ptr(bias), _ptr(Y), act, act_slope,
                                       _stream(stream)), "hfta_linear_fwd_static")


def linear_bwd_workspace_bytes(B, M, Fx, Fy, dtype) -> int:
    return _lib.hfta_linear_bwd_workspace_bytes(B, M, Fx, Fy, dtype)


def linear_bwd(B, M, Fx, Fy, dtype, X, W, dY, dX, dW, dbias, workspace=None, stream=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_linear_bwd(B, M, Fx, Fy, dtype, _ptr(X), _ptr(W), _ptr(dY), _ptr(dX), _ptr(dW), _ptr(dbias),
                                wp, wb, _stream(stream)), "hfta_linear_bwd")


def conv1x1_fwd(B, Nb, Ci, Co, L, dtype, X, xs, W, bias, Y, ys, act=ACT_NONE, act_slope=0.0, stream=None):
    _check(_lib.hfta_conv1x1_fwd(B, Nb, Ci, Co, L, dtype, _ptr(X), _strides(xs), _ptr(W), _ptr(bias), _ptr(Y),
                                 _strides(ys), act, act_slope, _stream(stream)), "hfta_conv1x1_fwd")


def conv1x1_fwd_sample_bias(B, Nb, Ci, Co, L, dtype, X, xs, W, S, ss, Y, ys, act=ACT_NONE, act_slope=0.0, stream=None):
    _check(_lib.hfta_conv1x1_fwd_sample_bias(B, Nb, Ci, Co, L, dtype, _ptr(X), _strides(xs), _ptr(W), _ptr(S),
                                             _strides(ss, 3), _ptr(Y), _strides(ys), act, act_slope, _stream(stream)),
           "hfta_conv1x1_fwd_sample_bias")


def conv1x1_bn_fwd_workspace_bytes(B, Nb, Ci, Co, L, dtype) -> int:
    return _lib.hfta_conv1x1_bn_fwd_workspace_bytes(B, Nb, Ci, Co, L, dtype)


def conv1x1_bn_fwd(B, Nb, Ci, Co, L, dtype, X, xs, W, bias, gamma, beta, eps, momentum, running_mean, running_var,
                   save_mean, save_invstd, Z, zs, Y, ys, act=ACT_NONE, act_slope=0.0, workspace=None, stream=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_conv1x1_bn_fwd(B, Nb, Ci, Co, L, dtype, _ptr(X), _strides(xs), _ptr(W), _ptr(bias), _ptr(gamma),
                                    _ptr(beta), eps, momentum, _ptr(running_mean), _ptr(running_var), _ptr(save_mean),
                                    _ptr(save_invstd), _ptr(Z), _strides(zs), _ptr(Y), _strides(ys), act, act_slope,
                                    wp, wb, _stream(stream)), "hfta_conv1x1_bn_fwd")


def conv1x1_bn_bwd_one_pass(B, Nb, Ci, Co, L, dtype) -> bool:
    return bool(_lib.hfta_conv1x1_bn_bwd_one_pass(B, Nb, Ci, Co, L, dtype))


def conv1x1_bn_bwd_workspace_bytes(B, Nb, Ci, Co, L, dtype) -> int:
    return _lib.hfta_conv1x1_bn_bwd_workspace_bytes(B, Nb, Ci, Co, L, dtype)


def conv1x1_bn_bwd(B, Nb, Ci, Co, L, dtype, X, xs, W, Z, zs, dY, dys, gamma, beta, save_mean, save_invstd, dX, dxs, dW,
                   dbias, dgamma, dbeta, act=ACT_NONE, act_slope=0.0, workspace=None, stream=None, sums=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_conv1x1_bn_bwd(B, Nb, Ci, Co, L, dtype, _ptr(X), _strides(xs), _ptr(W), _ptr(Z), _strides(zs),
                                    _ptr(dY), _strides(dys), _ptr(gamma), _ptr(beta), _ptr(save_mean), _ptr(save_invstd),
                                    _ptr(dX), _strides(dxs), _ptr(dW), _ptr(dbias), _ptr(dgamma), _ptr(dbeta),
                                    _ptr(sums), act, act_slope, wp, wb, _stream(stream)), "hfta_conv1x1_bn_bwd")


def conv1x1_bn_prenorm_supported(B, Nb, Ci, Co, L, dtype) -> bool:
    return bool(_lib.hfta_conv1x1_bn_prenorm_supported(B, Nb, Ci, Co, L, dtype))


def conv1x1_bn_prenorm_bwd_gives_sums(B, Nb, Ci, Co, L, dtype) -> bool:
    return bool(_lib.hfta_conv1x1_bn_prenorm_bwd_gives_sums(B, Nb, Ci, Co, L, dtype))


def conv1x1_bn_prenorm_fwd(B, Nb, Ci, Co, L, dtype, Xpre, xs, in_gamma, in_beta, in_mean, in_invstd, in_act, in_slope, W, bias,
                           gamma, beta, eps, momentum, running_mean, running_var, save_mean, save_invstd, Z, zs, Y, ys,
                           act=ACT_NONE, act_slope=0.0, workspace=None, stream=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_conv1x1_bn_prenorm_fwd(B, Nb, Ci, Co, L, dtype, _ptr(Xpre), _strides(xs), _ptr(in_gamma), _ptr(in_beta),
                                            _ptr(in_mean), _ptr(in_invstd), in_act, in_slope, _ptr(W), _ptr(bias), _ptr(gamma),
                                            _ptr(beta), eps, momentum, _ptr(running_mean), _ptr(running_var), _ptr(save_mean),
                                            _ptr(save_invstd), _ptr(Z), _strides(zs), _ptr(Y), _strides(ys), act, act_slope,
                                            wp, wb, _stream(stream)), "hfta_conv1x1_bn_prenorm_fwd")


def conv1x1_bn_prenorm_bwd(B, Nb, Ci, Co, L, dtype, Xpre, xs, in_gamma, in_beta, in_mean, in_invstd, in_act, in_slope, W, Z, zs,
                           dY, dys, gamma, beta, save_mean, save_invstd, dX, dxs, dW, dbias, dgamma, dbeta, act=ACT_NONE,
                           act_slope=0.0, workspace=None, stream=None, sums=None, in_sums=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_conv1x1_bn_prenorm_bwd(B, Nb, Ci, Co, L, dtype, _ptr(Xpre), _strides(xs), _ptr(in_gamma), _ptr(in_beta),
                                            _ptr(in_mean), _ptr(in_invstd), in_act, in_slope, _ptr(W), _ptr(Z), _strides(zs),
                                            _ptr(dY), _strides(dys), _ptr(gamma), _ptr(beta), _ptr(save_mean),
                                            _ptr(save_invstd), _ptr(dX), _strides(dxs), _ptr(dW), _ptr(dbias), _ptr(dgamma),
                                            _ptr(dbeta), _ptr(sums), _ptr(in_sums), act, act_slope, wp, wb,
                                            _stream(stream)),
           "hfta_conv1x1_bn_prenorm_bwd")


def conv1x1_bwd_workspace_bytes(B, Nb, Ci, Co, L, dtype) -> int:
    return _lib.hfta_conv1x1_bwd_workspace_bytes(B, Nb, Ci, Co, L, dtype)


def conv1x1_bwd(B, Nb, Ci, Co, L, dtype, X, xs, W, dY, dys, dX, dxs, dW, dbias, workspace=None, stream=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_conv1x1_bwd(B, Nb, Ci, Co, L, dtype, _ptr(X), _strides(xs), _ptr(W), _ptr(dY), _strides(dys),
                                 _ptr(dX), _strides(dxs), _ptr(dW), _ptr(dbias), wp, wb, _stream(stream)),
           "hfta_conv1x1_bwd")


def conv2d_grouped_fwd_workspace_bytes(B, Nb, Ci, Co, H, W_, kh, kw, stride, pad, dtype) -> int:
    return _lib.hfta_conv2d_grouped_fwd_workspace_bytes(B, Nb, Ci, Co, H, W_, kh, kw, stride, pad, dtype)


def conv2d_grouped_fwd(B, Nb, Ci, Co, H, W_, kh, kw, stride, pad, dtype, X, Wt, bias, Y, act=ACT_NONE,
                       act_slope=0.0, workspace=None, stream=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_conv2d_grouped_fwd(B, Nb, Ci, Co, H, W_, kh, kw, stride, pad, dtype, _ptr(X), _ptr(Wt),
                                        _ptr(bias), _ptr(Y), act, act_slope, wp, wb, _stream(stream)),
           "hfta_conv2d_grouped_fwd")


def conv2d_grouped_bwd_min_workspace_bytes(B, Nb, Ci, Co, H, W_, kh, kw, stride, pad, dtype) -> int:
    return _lib.hfta_conv2d_grouped_bwd_min_workspace_bytes(B, Nb, Ci, Co, H, W_, kh, kw, stride, pad, dtype)


def conv2d_grouped_bwd_workspace_bytes(B, Nb, Ci, Co, H, W_, kh, kw, stride, pad, dtype) -> int:
    return _lib.hfta_conv2d_grouped_bwd_workspace_bytes(B, Nb, Ci, Co, H, W_, kh, kw, stride, pad, dtype)


def conv2d_grouped_bwd(B, Nb, Ci, Co, H, W_, kh, kw, stride, pad, dtype, X, Wt, dY, dX, dW, dbias,
                       workspace=None, stream=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_conv2d_grouped_bwd(B, Nb, Ci, Co, H, W_, kh, kw, stride, pad, dtype, _ptr(X), _ptr(Wt),
                                        _ptr(dY), _ptr(dX), _ptr(dW), _ptr(dbias), wp, wb, _stream(stream)),
           "hfta_conv2d_grouped_bwd")


def bn_fwd(B, Nb, C_, L, dtype, X, xs, gamma, beta, eps, momentum, running_mean, running_var, save_mean,
           save_invstd, Y, ys, act=ACT_NONE, act_slope=0.0, stream=None):
    _check(_lib.hfta_bn_fwd(B, Nb, C_, L, dtype, _ptr(X), _strides(xs), _ptr(gamma), _ptr(beta), eps, momentum,
                            _ptr(running_mean), _ptr(running_var), _ptr(save_mean), _ptr(save_invstd), _ptr(Y),
                            _strides(ys), act, act_slope, _stream(stream)), "hfta_bn_fwd")


def bn_apply_fwd(B, Nb, C_, L, dtype, X, xs, gamma, beta, mean, invstd, Y, ys, act=ACT_NONE, act_slope=0.0, stream=None):
    _check(_lib.hfta_bn_apply_fwd(B, Nb, C_, L, dtype, _ptr(X), _strides(xs), _ptr(gamma), _ptr(beta), _ptr(mean), _ptr(invstd),
                                  _ptr(Y), _strides(ys), act, act_slope, _stream(stream)), "hfta_bn_apply_fwd")


def bn_eval_fwd(B, Nb, C_, L, dtype, X, xs, gamma, beta, running_mean, running_var, eps, Y, ys, act=ACT_NONE,
                act_slope=0.0, stream=None):
    _check(_lib.hfta_bn_eval_fwd(B, Nb, C_, L, dtype, _ptr(X), _strides(xs), _ptr(gamma), _ptr(beta), _ptr(running_mean),
                                 _ptr(running_var), eps, _ptr(Y), _strides(ys), act, act_slope, _stream(stream)),
           "hfta_bn_eval_fwd")


def bn_bwd(B, Nb, C_, L, dtype, X, xs, dY, dys, gamma, beta, save_mean, save_invstd, dX, dxs, dgamma, dbeta,
           act=ACT_NONE, act_slope=0.0, dx_sum=None, stream=None):
    _check(_lib.hfta_bn_bwd(B, Nb, C_, L, dtype, _ptr(X), _strides(xs), _ptr(dY), _strides(dys), _ptr(gamma),
                            _ptr(beta), _ptr(save_mean), _ptr(save_invstd), _ptr(dX), _strides(dxs), _ptr(dgamma),
                            _ptr(dbeta), _ptr(dx_sum), act, act_slope, _stream(stream)), "hfta_bn_bwd")


def bn_fwd_maxpool(B, Nb, C_, L, dtype, X, xs, gamma, beta, eps, momentum, running_mean, running_var, save_mean,
                   save_invstd, V, idx, vs, act=ACT_NONE, act_slope=0.0, stream=None):
    _check(_lib.hfta_bn_fwd_maxpool(B, Nb, C_, L, dtype, _ptr(X), _strides(xs), _ptr(gamma), _ptr(beta), eps,
                                    momentum, _ptr(running_mean), _ptr(running_var), _ptr(save_mean),
                                    _ptr(save_invstd), _ptr(V), _ptr(idx), _strides(vs, 3), act, act_slope,
                                    _stream(stream)), "hfta_bn_fwd_maxpool")


def bn_bwd_maxpool(B, Nb, C_, L, dtype, X, xs, dV, idx, vs, gamma, beta, save_mean, save_invstd, dX, dxs, dgamma,
                   dbeta, act=ACT_NONE, act_slope=0.0, dx_sum=None, stream=None):
    _check(_lib.hfta_bn_bwd_maxpool(B, Nb, C_, L, dtype, _ptr(X), _strides(xs), _ptr(dV), _ptr(idx),
                                    _strides(vs, 3), _ptr(gamma), _ptr(beta), _ptr(save_mean), _ptr(save_invstd),
                                    _ptr(dX), _strides(dxs), _ptr(dgamma), _ptr(dbeta), _ptr(dx_sum), act,
                                    act_slope, _stream(stream)), "hfta_bn_bwd_maxpool")


def conv1x1_bn_maxpool_bwd_workspace_bytes(B, Nb, Ci, Co, L, dtype) -> int:
    return _lib.hfta_conv1x1_bn_maxpool_bwd_workspace_bytes(B, Nb, Ci, Co, L, dtype)


def conv1x1_bn_maxpool_bwd(B, Nb, Ci, Co, L, dtype, X, xs, W, bias, Z, zs, zhit, saved_moments, dV, idx, vs, gamma, beta,
                           save_mean, save_invstd, dX, dxs, dW, dbias, dgamma, dbeta, act=ACT_NONE, act_slope=0.0,
                           workspace=None, stream=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_conv1x1_bn_maxpool_bwd(B, Nb, Ci, Co, L, dtype, _ptr(X), _strides(xs), _ptr(W), _ptr(bias),
                                            _ptr(Z), None if zs is None else _strides(zs), _ptr(zhit),
                                            _ptr(saved_moments), _ptr(dV), _ptr(idx), _strides(vs, 3), _ptr(gamma),
                                            _ptr(beta), _ptr(save_mean), _ptr(save_invstd), _ptr(dX), _strides(dxs),
                                            _ptr(dW), _ptr(dbias), _ptr(dgamma), _ptr(dbeta), act, act_slope, wp, wb,
                                            _stream(stream)), "hfta_conv1x1_bn_maxpool_bwd")


def conv1x1_bn_maxpool_prenorm_fwd(B, Nb, Ci, Co, L, dtype, Xpre, xs, in_gamma, in_beta, in_mean, in_invstd, in_act, in_slope, W,
                                   bias, gamma, beta, eps, momentum, running_mean, running_var, save_mean, save_invstd, V, idx,
                                   vs, zhit, saved_moments, act=ACT_NONE, act_slope=0.0, workspace=None, stream=None, Xact=None,
                                   xas=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_conv1x1_bn_maxpool_prenorm_fwd(B, Nb, Ci, Co, L, dtype, _ptr(Xpre), _strides(xs), _ptr(in_gamma),
                                                    _ptr(in_beta), _ptr(in_mean), _ptr(in_invstd), in_act, in_slope, _ptr(W),
                                                    _ptr(bias), _ptr(gamma), _ptr(beta), eps, momentum, _ptr(running_mean),
                                                    _ptr(running_var), _ptr(save_mean), _ptr(save_invstd), _ptr(V), _ptr(idx),
                                                    _strides(vs, 3), _ptr(zhit), _ptr(saved_moments), act, act_slope, _ptr(Xact),
                                                    _strides(xas), wp, wb,
                                                    _stream(stream)), "hfta_conv1x1_bn_maxpool_prenorm_fwd")


def conv1x1_bn_maxpool_prenorm_bwd(B, Nb, Ci, Co, L, dtype, Xpre, xs, in_gamma, in_beta, in_mean, in_invstd, in_act, in_slope, W,
                                   bias, zhit, saved_moments, dV, idx, vs, gamma, beta, save_mean, save_invstd, dX, dxs, dW,
                                   dbias, dgamma, dbeta, act=ACT_NONE, act_slope=0.0, workspace=None, stream=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_conv1x1_bn_maxpool_prenorm_bwd(B, Nb, Ci, Co, L, dtype, _ptr(Xpre), _strides(xs), _ptr(in_gamma),
                                                    _ptr(in_beta), _ptr(in_mean), _ptr(in_invstd), in_act, in_slope, _ptr(W),
                                                    _ptr(bias), _ptr(zhit), _ptr(saved_moments), _ptr(dV), _ptr(idx),
                                                    _strides(vs, 3), _ptr(gamma), _ptr(beta), _ptr(save_mean),
                                                    _ptr(save_invstd), _ptr(dX), _strides(dxs), _ptr(dW), _ptr(dbias),
                                                    _ptr(dgamma), _ptr(dbeta), act, act_slope, wp, wb, _stream(stream)),
           "hfta_conv1x1_bn_maxpool_prenorm_bwd")


def conv1x1_bn_maxpool_saved_floats(B, Ci, Co):
    return _lib.hfta_conv1x1_bn_maxpool_saved_floats(B, Ci, Co)


def conv1x1_bn_maxpool_fwd_workspace_bytes(B, Nb, Ci, Co, L, dtype):
    return _lib.hfta_conv1x1_bn_maxpool_fwd_workspace_bytes(B, Nb, Ci, Co, L, dtype)


def conv1x1_bn_maxpool_fwd(B, Nb, Ci, Co, L, dtype, X, xs, W, bias, gamma, beta, eps, momentum, running_mean, running_var,
                           save_mean, save_invstd, V, idx, vs, zhit, saved_moments, act=ACT_NONE, act_slope=0.0,
                           workspace=None, stream=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_conv1x1_bn_maxpool_fwd(B, Nb, Ci, Co, L, dtype, _ptr(X), _strides(xs), _ptr(W), _ptr(bias),
                                            _ptr(gamma), _ptr(beta), eps, momentum, _ptr(running_mean),
                                            _ptr(running_var), _ptr(save_mean), _ptr(save_invstd), _ptr(V), _ptr(idx),
                                            _strides(vs, 3), _ptr(zhit), _ptr(saved_moments), act, act_slope, wp, wb,
                                            _stream(stream)), "hfta_conv1x1_bn_maxpool_fwd")


def maxpool_points(B, Nb, C_, L, dtype, X, xs, V, idx, vs, stream=None):
    _check(_lib.hfta_maxpool_points(B, Nb, C_, L, dtype, _ptr(X), _strides(xs), _ptr(V), _ptr(idx),
                                    _strides(vs, 3), _stream(stream)), "hfta_maxpool_points")


def maxpool_points_bwd(B, Nb, C_, L, dtype, dV, idx, vs, dX, dxs, stream=None):
    _check(_lib.hfta_maxpool_points_bwd(B, Nb, C_, L, dtype, _ptr(dV), _ptr(idx), _strides(vs, 3), _ptr(dX),
                                        _strides(dxs), _stream(stream)), "hfta_maxpool_points_bwd")


def adam_step(B, P, grad_dtype, theta, grad, m, v, theta_lowp, lr, beta1, beta2, eps, weight_decay, step_t,
              decoupled_wd=0, stream=None):
    _check(_lib.hfta_adam_step(B, P, grad_dtype, _ptr(theta), _ptr(grad), _ptr(m), _ptr(v), _ptr(theta_lowp),
                               _ptr(lr), _ptr(beta1), _ptr(beta2), _ptr(eps), _ptr(weight_decay), step_t,
                               decoupled_wd, _stream(stream)), "hfta_adam_step")


def adam_step_multi(B, seg_offsets, grad_dtype, theta, grad, m, v, theta_lowp, lr, beta1, beta2, eps,
                    weight_decay, step_t, decoupled_wd=0, stream=None):
    nseg = len(seg_offsets) - 1
    _check(_lib.hfta_adam_step_multi(B, nseg, _strides(seg_offsets, nseg + 1), grad_dtype, _ptr(theta), _ptr(grad),
                                     _ptr(m), _ptr(v), _ptr(theta_lowp), _ptr(lr), _ptr(beta1), _ptr(beta2),
                                     _ptr(eps), _ptr(weight_decay), step_t, decoupled_wd, _stream(stream)),
           "hfta_adam_step_multi")


def act_fwd(count, dtype, X, Y, act, slope=0.0, stream=None):
    _check(_lib.hfta_act_fwd(count, dtype, _ptr(X), _ptr(Y), act, slope, _stream(stream)), "hfta_act_fwd")


def act_bwd(count, dtype, Z, dY, dX, act, slope=0.0, from_output=0, stream=None):
    _check(_lib.hfta_act_bwd(count, dtype, _ptr(Z), _ptr(dY), _ptr(dX), act, slope, from_output, _stream(stream)),
           "hfta_act_bwd")


def act_bwd_colsum(B, M, F, dtype, Z, dY, dX, dbias, act, slope=0.0, stream=None):
    _check(_lib.hfta_act_bwd_colsum(B, M, F, dtype, _ptr(Z), _ptr(dY), _ptr(dX), _ptr(dbias), act, slope, _stream(stream)),
           "hfta_act_bwd_colsum")


def bias_act_nchw(Nb, K, HW, dtype, Y, bias, act=ACT_NONE, slope=0.0, stream=None):
    _check(_lib.hfta_bias_act_nchw(Nb, K, HW, dtype, _ptr(Y), _ptr(bias), act, slope, _stream(stream)),
           "hfta_bias_act_nchw")


def add(count, dtype, A, B, Y, stream=None):
    _check(_lib.hfta_add(count, dtype, _ptr(A), _ptr(B), _ptr(Y), _stream(stream)), "hfta_add")


def dropout(count, dtype, X, mask, p, Y, stream=None):
    _check(_lib.hfta_dropout(count, dtype, _ptr(X), _ptr(mask), p, _ptr(Y), _stream(stream)), "hfta_dropout")


def layernorm_fwd(B, R, E, dtype, X, w, b, eps, save_mean, save_invstd, Y, stream=None):
    _check(_lib.hfta_layernorm_fwd(B, R, E, dtype, _ptr(X), _ptr(w), _ptr(b), eps, _ptr(save_mean),
                                   _ptr(save_invstd), _ptr(Y), _stream(stream)), "hfta_layernorm_fwd")


def layernorm_bwd_workspace_bytes(B, R, E) -> int:
    return _lib.hfta_layernorm_bwd_workspace_bytes(B, R, E)


def layernorm_bwd(B, R, E, dtype, X, dY, w, save_mean, save_invstd, dX, dw, db, workspace=None, stream=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_layernorm_bwd(B, R, E, dtype, _ptr(X), _ptr(dY), _ptr(w), _ptr(save_mean), _ptr(save_invstd),
                                   _ptr(dX), _ptr(dw), _ptr(db), wp, wb, _stream(stream)), "hfta_layernorm_bwd")


def layernorm_bwd_sums_workspace_bytes(B, R, E) -> int:
    return _lib.hfta_layernorm_bwd_sums_workspace_bytes(B, R, E)


def layernorm_bwd_sums(B, R, E, dtype, X, dY, dY2, w, save_mean, save_invstd, dX, dw, db, dx_colsum, workspace=None,
                       stream=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_layernorm_bwd_sums(B, R, E, dtype, _ptr(X), _ptr(dY), _ptr(dY2), _ptr(w), _ptr(save_mean),
                                        _ptr(save_invstd), _ptr(dX), _ptr(dw), _ptr(db), _ptr(dx_colsum), wp, wb,
                                        _stream(stream)), "hfta_layernorm_bwd_sums")


def softmax_xent(B, R, K, dtype, logits, labels, loss, dlogits, stream=None):
    _check(_lib.hfta_softmax_xent(B, R, K, dtype, _ptr(logits), _ptr(labels), _ptr(loss), _ptr(dlogits),
                                  _stream(stream)), "hfta_softmax_xent")


def bce_logits(B, R, dtype, logits, targets, loss, dlogits, stream=None):
    _check(_lib.hfta_bce_logits(B, R, dtype, _ptr(logits), _ptr(targets), _ptr(loss), _ptr(dlogits),
                                _stream(stream)), "hfta_bce_logits")


def bce_logits_strided(B, R, dtype, logits, targets, loss, dlogits, stride_b, stride_r, stream=None):
    _check(_lib.hfta_bce_logits_strided(B, R, dtype, _ptr(logits), _ptr(targets), _ptr(loss), _ptr(dlogits),
                                        stride_b, stride_r, _stream(stream)), "hfta_bce_logits_strided")


def mse(B, R, dtype, pred, target, loss, dpred, stream=None):
    _check(_lib.hfta_mse(B, R, dtype, _ptr(pred), _ptr(target), _ptr(loss), _ptr(dpred), _stream(stream)), "hfta_mse")


def raw():
    """The ctypes library handle (for status-code tests that must not raise)."""
    return _lib


def add_sample_bias(B, Nb, C, L, dtype, Z, zs, S, ss, Y, ys, stream=None):
    _check(_lib.hfta_add_sample_bias(B, Nb, C, L, dtype, _ptr(Z), _strides(zs), _ptr(S), _strides(ss, 3), _ptr(Y),
                                     _strides(ys), _stream(stream)), "hfta_add_sample_bias")


def sum_points(B, Nb, C, L, dtype, X, xs, S, ss, stream=None):
    _check(_lib.hfta_sum_points(B, Nb, C, L, dtype, _ptr(X), _strides(xs), _ptr(S), _strides(ss, 3), _stream(stream)),
           "hfta_sum_points")


def add_strided(B, Nb, C, L, dtype, A, as_, Bt, bs, Y, ys, stream=None):
    _check(_lib.hfta_add_strided(B, Nb, C, L, dtype, _ptr(A), _strides(as_), _ptr(Bt), _strides(bs), _ptr(Y),
                                 _strides(ys), _stream(stream)), "hfta_add_strided")


def maxpool_points_bwd_add(B, Nb, C, L, dtype, dV, idx, vs, dX, dxs, stream=None):
    _check(_lib.hfta_maxpool_points_bwd_add(B, Nb, C, L, dtype, _ptr(dV), _ptr(idx), _strides(vs, 3), _ptr(dX),
                                            _strides(dxs), _stream(stream)), "hfta_maxpool_points_bwd_add")


def softmax_xent_points_workspace_bytes(B, Nb, L):
    return _lib.hfta_softmax_xent_points_workspace_bytes(B, Nb, L)


def softmax_xent_points(B, Nb, K, L, dtype, logits, ls, labels, loss, dlogits, ds, workspace=None, stream=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_softmax_xent_points(B, Nb, K, L, dtype, _ptr(logits), _strides(ls), _ptr(labels), _ptr(loss),
                                         _ptr(dlogits), _strides(ds), wp, wb, _stream(stream)), "hfta_softmax_xent_points")


def adadelta_step_multi(B, seg_offsets, grad_dtype, theta, grad, square_avg, acc_delta, theta_lowp, lr, rho, eps,
                        weight_decay, stream=None):
    nseg = len(seg_offsets) - 1
    _check(_lib.hfta_adadelta_step_multi(B, nseg, _strides(seg_offsets, nseg + 1), grad_dtype, _ptr(theta), _ptr(grad),
                                         _ptr(square_avg), _ptr(acc_delta), _ptr(theta_lowp), _ptr(lr), _ptr(rho),
                                         _ptr(eps), _ptr(weight_decay), _stream(stream)), "hfta_adadelta_step_multi")


def steplr(B, base_lr, gamma, step_size, epoch, lr, stream=None):
    _check(_lib.hfta_steplr(B, _ptr(base_lr), _ptr(gamma), _ptr(step_size), epoch, _ptr(lr), _stream(stream)),
           "hfta_steplr")


def embedding_fwd(B, R, V, E, dtype, table, idx, scale, pos, S, out, stream=None):
    _check(_lib.hfta_embedding_fwd(B, R, V, E, dtype, _ptr(table), _ptr(idx), scale, _ptr(pos), S, _ptr(out),
                                   _stream(stream)), "hfta_embedding_fwd")


def embedding_bwd(B, R, V, E, dtype, dY, idx, scale, dtable, stream=None):
    _check(_lib.hfta_embedding_bwd(B, R, V, E, dtype, _ptr(dY), _ptr(idx), scale, _ptr(dtable), _stream(stream)),
           "hfta_embedding_bwd")


def attention_fwd(B, N, S, E, H, dtype, QKV, P, CTX, causal=0, stream=None):
    _check(_lib.hfta_attention_fwd(B, N, S, E, H, dtype, _ptr(QKV), _ptr(P), _ptr(CTX), causal, _stream(stream)),
           "hfta_attention_fwd")


def attention_bwd_workspace_bytes(B, N, S, E, H, dtype):
    return _lib.hfta_attention_bwd_workspace_bytes(B, N, S, E, H, dtype)


def attention_bwd(B, N, S, E, H, dtype, QKV, P, dCTX, dQKV, workspace=None, stream=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_attention_bwd(B, N, S, E, H, dtype, _ptr(QKV), _ptr(P), _ptr(dCTX), _ptr(dQKV), wp, wb,
                                   _stream(stream)), "hfta_attention_bwd")


def softmax_xent_rows_workspace_bytes(B, R):
    return _lib.hfta_softmax_xent_rows_workspace_bytes(B, R)


def softmax_xent_rows(B, R, K, dtype, logits, labels, loss, dlogits, workspace=None, stream=None):
    wp, wb = _ws(workspace)
    _check(_lib.hfta_softmax_xent_rows(B, R, K, dtype, _ptr(logits), _ptr(labels), _ptr(loss), _ptr(dlogits), wp, wb,
                                       _stream(stream)), "hfta_softmax_xent_rows")


def point_transform_fwd(B, Nb, Ci, Co, L, dtype, X, xs, T, Y, ys, stream=None):
    _check(_lib.hfta_point_transform_fwd(B, Nb, Ci, Co, L, dtype, _ptr(X), _strides(xs), _ptr(T), _ptr(Y), _strides(ys),
                                         _stream(stream)), "hfta_point_transform_fwd")


def point_transform_bwd(B, Nb, Ci, Co, L, dtype, X, xs, T, dY, dys, dX, dxs, dT, stream=None):
    _check(_lib.hfta_point_transform_bwd(B, Nb, Ci, Co, L, dtype, _ptr(X), None if xs is None else _strides(xs), _ptr(T),
                                         _ptr(dY), _strides(dys), _ptr(dX), None if dxs is None else _strides(dxs),
                                         _ptr(dT), _stream(stream)), "hfta_point_transform_bwd")
