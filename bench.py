#!/usr/bin/env python3
"""Benchmark of the fused training array on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--repeats R] [--workload all|c0|c1|c2|c3|c4|c1t|t0] [--skip-serial] [--skip-cpu]

A step is one forward + backward + Adam pass of the whole fused array over one
synthetic batch that is already resident in HBM.  Prints ONE JSON line:
fused samples/s summed over the B models (`value`), the same B models run one
after another through the library with B = 1 (`serial_b1`), the roofline of the
kernel that dominates the step (timed live with HIP events on the launch stream)
and the CPU oracle timed on a bounded sample (`cpu_baseline`).
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time
from collections import defaultdict

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth


# ------------------------------------------------------------------ tracing proxy
class Tracer:
    """Wraps the binding so that selected entry points (one kernel each, or a named short
    sequence) are bracketed by HIP events on the stream they launch on (torch's current stream)."""

    SINGLE_KERNEL = ("conv1x1_fwd", "conv1x1_bwd", "bn_fwd", "bn_bwd", "maxpool_points", "maxpool_points_bwd",
                     "adam_step_multi", "linear_fwd", "linear_fwd_ws", "linear_bwd", "bn_fwd_maxpool", "bn_bwd_maxpool",
                     "act_fwd", "act_bwd", "act_bwd_colsum", "add", "layernorm_fwd", "layernorm_bwd", "layernorm_bwd_sums",
                     "conv2d_grouped_fwd", "conv2d_grouped_bwd", "bias_act_nchw", "conv1x1_bn_maxpool_fwd",
                     "add_sample_bias", "sum_points", "add_strided", "softmax_xent_points",
                     "attention_fwd", "attention_bwd", "embedding_fwd", "embedding_bwd", "softmax_xent", "softmax_xent_rows",
                     "point_transform_fwd", "point_transform_bwd",
                     "conv1x1_bn_maxpool_bwd", "conv1x1_bn_fwd", "conv1x1_bn_bwd", "conv1x1_bn_prenorm_fwd",
                     "conv1x1_bn_prenorm_bwd", "conv1x1_bn_maxpool_prenorm_fwd", "conv1x1_bn_maxpool_prenorm_bwd")

    def __init__(self, hb, torch):
        self._hb, self._torch = hb, torch
        self.events = []            # (label, bytes, start, end)
        self.enabled = False
        self.only = None            # when set: bracket only the calls with this label

    def __getattr__(self, name):
        fn = getattr(self._hb, name)
        if not callable(fn) or name not in self.SINGLE_KERNEL:
            return fn

        def wrapped(*a, **kw):
            if not self.enabled:
                return fn(*a, **kw)
            if self.only is not None and kernel_label(name, a) != self.only:
                return fn(*a, **kw)
            s = self._torch.cuda.Event(enable_timing=True)
            e = self._torch.cuda.Event(enable_timing=True)
            s.record()
            r = fn(*a, **kw)
            e.record()
            self.events.append((kernel_label(name, a), algorithmic_bytes(name, a), s, e, algorithmic_flops(name, a)))
            return r
        return wrapped

    def summary(self):
        self._torch.cuda.synchronize()
        tot = defaultdict(lambda: [0, 0.0, 0.0, 0.0])   # label -> [launches, ms, bytes, flop]
        for label, nbytes, s, e, fl in self.events:
            t = tot[label]
            t[0] += 1
            t[1] += s.elapsed_time(e)
            t[2] += nbytes
            t[3] += fl
        return tot


def _es(dtype):
    return 2 if dtype == 1 else 4


def kernel_label(name, a):
    """Kernel symbol family an entry point launches (matches the rocprofv3 kernel names)."""
    if name in ("bn_fwd", "bn_bwd"):
        lay = "linear" if a[3] == 1 else "conv"
        return f"{name}_{lay}_kernel"
    if name == "conv1x1_bn_fwd":
        B, Nb, Ci, Co, L, dt = a[:6]
        if dt == 1 and Ci % 8 == 0 and L % 4 == 0 and ((Ci <= 128 and Co >= 64) or (Ci <= 256 and Co >= 512)):
            return "conv1x1_bn_fwd: conv1x1_stream_kernel(+statistics) + bn_stats_part_kernel (+ bn_apply_conv_kernel)"
        return "conv1x1_bn_fwd: conv1x1 kernel (batched GEMM, + statistics in its 256x256 form; K <= 4: vector kernel) + BatchNorm kernels"
    if name == "conv1x1_bn_prenorm_fwd":     # the same kernels as the plain call, the input normalised on load
        return "conv1x1_bn_fwd: conv1x1_stream_kernel(+statistics) + bn_stats_part_kernel (+ bn_apply_conv_kernel)"
    if name == "conv1x1_bn_prenorm_bwd":
        return "conv1x1_bn_bwd: bn_bwd_conv_coef_kernel or bn_bwd_coef_sums_kernel + cbb_kernel + cbb_reduce_kernel"
    if name == "conv1x1_bn_bwd":
        B, Nb, Ci, Co, L, dt = a[:6]
        if dt == 1 and Ci <= 128 and Co <= 128 and L % 4 == 0:
            return "conv1x1_bn_bwd: bn_bwd_conv_coef_kernel or bn_bwd_coef_sums_kernel + cbb_kernel + cbb_reduce_kernel"
        return "conv1x1_bn_bwd: bn_bwd_conv_kernel + conv1x1 backward kernels"
    if name == "conv1x1_fwd":
        B, Nb, Ci, Co, L, dt = a[:6]
        if dt == 1 and Ci <= 4 and L % 4 == 0:
            return "conv1x1_tinyk_kernel"
        if dt == 1 and Ci % 8 == 0 and L % 4 == 0 and ((Ci <= 128 and Co >= 64) or (Ci <= 256 and Co >= 512)):
            return "conv1x1_stream_kernel"
        if dt == 1 and big_gemm(B * Nb, Co, L, Ci):
            return big_name(B * Nb, Co, L) + "(fwd)"
        return "gemm_pf_kernel(fwd)" if dt == 1 else "gemm_kernel(fwd)"
    if name == "linear_fwd_ws" and a[1] <= 64:
        return ("gemm_pf_kernel" if a[4] == 1 else "gemm_kernel") + "(fwd, split)+splitk_bias_act_kernel"
    if name in ("linear_fwd", "linear_fwd_ws"):
        if a[4] == 1 and big_gemm(a[0], a[1], a[3], a[2]):
            return big_name(a[0], a[1], a[3]) + "(fwd)"
        return "gemm_pf_kernel(fwd)" if a[4] == 1 else "gemm_kernel(fwd)"
    if name == "linear_bwd":           # the MLP array asks for dX, dW and dbias in separate calls
        B, M, Fx, Fy, dt = a[:5]
        if a[8] is not None and a[9] is not None:      # one call for everything (the Transformer array)
            return "linear_bwd: gemm(dX) + gemm(dW) + splitk_reduce_kernel + colsum_kernel"
        if a[8] is not None:
            return (big_name(B, M, Fx) if dt == 1 and big_gemm(B, M, Fx, Fy) else "gemm_pf_kernel") + "(dX)"
        if a[9] is not None:
            sp = big_splits(B, Fx, Fy, M) if dt == 1 else 0
            return (big_name(B, Fx, Fy, sp) if sp else "gemm_pf_kernel") + "(dW)"
        return "colsum_kernel"
    if name == "layernorm_bwd_sums":
        return "layernorm_bwd_kernel"
    if name in ("act_fwd", "act_bwd", "act_bwd_colsum", "add", "layernorm_fwd", "layernorm_bwd", "bias_act_nchw"):
        return name + "_kernel"
    if name in ("attention_fwd", "attention_bwd"):
        return name + ": batched head GEMMs + softmax_rows kernel"
    if name in ("embedding_fwd", "embedding_bwd", "softmax_xent"):
        return name + "_kernel"
    if name == "softmax_xent_rows":
        return "xent_rows_kernel"
    if name in ("point_transform_fwd", "point_transform_bwd"):
        return name + ": batched GEMM per (model, cloud)"
    if name in ("add_sample_bias", "add_strided"):
        return "row_add_kernel"
    if name == "sum_points":
        return "sum_points_kernel"
    if name == "softmax_xent_points":
        return "xent_points_kernel"
    if name in ("conv2d_grouped_fwd", "conv2d_grouped_bwd"):
        B, Nb, Ci, Co, H, W, kh, kw, stride, pad, dt = a[:11]
        p2 = lambda v: v > 0 and v & (v - 1) == 0
        ig = dt == 1 and (kh, kw, stride, pad) == (4, 4, 2, 1) and p2(H // 2) and p2(W // 2) and W >= 8 and H * W >= 64
        full = H == kh and W == kw and pad == 0     # whole-image window: a batched Linear
        small = "full_%s_small_kernel" if Co <= 8 else "gemm(%s, whole-image window)"
        if name == "conv2d_grouped_fwd":       # sample-folded implicit GEMM, else the column-buffer lowering
            if full:
                return small % "fwd"
            return "conv_ig_fwd_kernel<4,4,2>" if ig else "conv2d fwd: im2col_lds_kernel + gemm"
        if a[14] is not None:                  # dX and dW are asked for in separate calls
            if full:
                return small % "dx"
            if dt == 1 and (kh, kw, stride, pad) == (4, 4, 2, 1) and Ci <= 4:
                return "conv_dx_fewc_kernel"
            return ("ig_pack_class_w_kernel + conv_ig_fwd_kernel<2,2,1,pair>" if ig and Ci >= 32
                    else "conv2d dX: pack_dy_kernel + gemm + col2im_lds_kernel")
        if full:
            return small % "dw"
        return ("conv_ig_dw_kernel + ig_split_reduce_kernel" if ig and Co >= 32 and W <= 64
                else "conv2d dW: pack_dy_kernel + im2col_lds_kernel + gemm")
    if name == "conv1x1_bwd":          # called with either dX or dW requested, never both
        B, Nb, Ci, Co, L, dt = a[:6]
        k = "gemm_pf_kernel" if dt == 1 else "gemm_kernel"
        if a[11] is not None:
            if (dt == 1 and Co % 8 == 0 and L % 4 == 0 and a[15] is not None
                    and ((Co <= 128 and Ci >= 64) or (Co <= 256 and Ci >= 512))):
                return "conv1x1_stream_kernel(dX)"
            return (big_name(B * Nb, Ci, L) if dt == 1 and big_gemm(B * Nb, Ci, L, Co) else k) + "(dX)"
        sp = big_splits(B, Co, Ci, L, Nb) if dt == 1 else 0
        if sp:
            k = big_name(B, Co, Ci, sp)
        return k + "(dW)+splitk_reduce_kernel"
    if name in ("bn_fwd_maxpool", "bn_bwd_maxpool"):
        return name + "_kernel"
    if name in ("conv1x1_bn_maxpool_fwd", "conv1x1_bn_maxpool_prenorm_fwd"):      # the same kernels, the input normalised on load
        return "conv1x1_bn_maxpool_fwd: fbp_main_kernel + gram_kernel + 4 small"
    if name in ("conv1x1_bn_maxpool_bwd", "conv1x1_bn_maxpool_prenorm_bwd"):
        saved = a[13] if name == "conv1x1_bn_maxpool_bwd" else a[17]
        return "conv1x1_bn_maxpool_bwd: cbp_dx_kernel + 5 small" + ("" if saved is not None else " + gram_kernel")
    return {"maxpool_points": "maxpool_fwd_kernel", "maxpool_points_bwd": "maxpool_bwd_kernel",
            "adam_step_multi": "adam_multi_kernel"}[name]


def big_gemm(G, M, N, K):
    """The 256x256-tile kernel's dispatch rule (compute-bound shapes)."""
    return M >= 192 and N >= 192 and K >= 256 and ((M + 255) // 256) * ((N + 255) // 256) * G >= 192


def big_name(G, M, N, splits=1):
    """Persistent form of the 256x256-tile kernel: more workgroups than compute units and output
    rows (fp32 partial rows when split) that take whole 8- or 16-byte pieces."""
    tiles = ((M + 255) // 256) * ((N + 255) // 256) * G * splits
    return "gemm_bigp_kernel" if tiles > 256 and N % 4 == 0 else "gemm_big_kernel"


def big_splits(G, M, N, K, S=1):
    """Split count the library's cost model picks for a weight gradient on the 256x256-tile kernel
    (rounds of 256 workgroups, a fixed prologue / epilogue in k-tile units, the partial buffer's
    traffic), or 0 when the shape does not take that kernel."""
    if M < 192 or N < 192 or K < 256:
        return 0
    t256, tt = ((M + 255) // 256) * ((N + 255) // 256) * G, S * ((K + 63) // 64)
    if tt < 32:
        return 0
    best, best_cost = 0, 0.0
    for s in range(1, 33):
        if tt // s < 16:
            break
        if t256 * s < 192:
            continue
        rounds = (t256 * s + 255) // 256
        cost = rounds * (tt / s + 4.0) + (0.2 * t256 / 256.0 * s if s > 1 else 0.0)
        if best == 0 or cost < best_cost:
            best, best_cost = s, cost
    return best


def algorithmic_flops(name, a):
    if name in ("linear_fwd", "linear_fwd_ws", "linear_bwd"):
        B, M, Fx, Fy = a[:4]
        if name == "linear_bwd" and a[8] is None and a[9] is None:
            return 0.0
        both = name == "linear_bwd" and a[8] is not None and a[9] is not None
        return (4.0 if both else 2.0) * B * M * Fx * Fy
    if name in ("conv1x1_fwd", "conv1x1_bwd", "conv1x1_bn_fwd"):
        B, Nb, Ci, Co, L = a[:5]
        return 2.0 * B * Nb * Ci * Co * L
    if name in ("conv1x1_bn_bwd", "conv1x1_bn_prenorm_bwd"):       # weight gradient, and the data gradient if asked for
        B, Nb, Ci, Co, L = a[:5]
        dx = a[17] if name == "conv1x1_bn_bwd" else a[23]
        return (4.0 if dx is not None else 2.0) * B * Nb * Ci * Co * L
    if name == "conv1x1_bn_prenorm_fwd":
        B, Nb, Ci, Co, L = a[:5]
        return 2.0 * B * Nb * Ci * Co * L
    if name in ("attention_fwd", "attention_bwd"):      # 2 (forward) / 4 (backward) products of S x S x d per head
        B, N, S, E, H = a[:5]
        return (2 if name == "attention_fwd" else 4) * 2.0 * B * N * S * S * E
    if name in ("conv1x1_bn_maxpool_fwd", "conv1x1_bn_maxpool_prenorm_fwd"):      # the Ci -> Co product (its output is reduced, never stored) + the Gram matrix
        B, Nb, Ci, Co, L = a[:5]
        return 2.0 * B * Nb * Ci * (Co + Ci) * L
    if name in ("conv1x1_bn_maxpool_bwd", "conv1x1_bn_maxpool_prenorm_bwd"):      # the Ci -> Ci product of the data gradient (+ the Gram matrix if not saved)
        B, Nb, Ci, Co, L = a[:5]
        saved = a[13] if name == "conv1x1_bn_maxpool_bwd" else a[17]
        return (2.0 if saved is not None else 4.0) * B * Nb * Ci * Ci * L
    if name in ("conv2d_grouped_fwd", "conv2d_grouped_bwd"):
        B, Nb, Ci, Co, H, W, kh, kw, st, pad = a[:10]
        Ho, Wo = (H + 2 * pad - kh) // st + 1, (W + 2 * pad - kw) // st + 1
        return 2.0 * B * Nb * Ho * Wo * Ci * Co * kh * kw
    return 0.0


def algorithmic_bytes(name, a):
    """Bytes that must cross HBM once: every operand in once, every result out once."""
    if name == "bn_fwd":
        B, Nb, C, L, dt = a[:5]
        return 2 * B * Nb * C * L * _es(dt)
    if name == "bn_bwd":
        B, Nb, C, L, dt = a[:5]
        return 3 * B * Nb * C * L * _es(dt)
    if name == "bn_fwd_maxpool":
        B, Nb, C, L, dt = a[:5]
        return B * Nb * C * (L * _es(dt) + _es(dt) + 4)
    if name == "bn_bwd_maxpool":
        B, Nb, C, L, dt = a[:5]
        return B * Nb * C * (2 * L * _es(dt) + _es(dt) + 4)
    if name == "conv1x1_fwd":
        B, Nb, Ci, Co, L, dt = a[:6]
        return (B * Nb * (Ci + Co) * L + B * Co * (Ci + 1)) * _es(dt)
    if name in ("conv1x1_bn_fwd", "conv1x1_bn_prenorm_fwd"):       # x and W in, z out; z in, y out (if y is asked for)
        B, Nb, Ci, Co, L, dt = a[:6]
        y = a[20] if name == "conv1x1_bn_fwd" else a[26]
        return (B * Nb * (Ci + (3 if y is not None else 1) * Co) * L + B * Co * (Ci + 1)) * _es(dt)
    if name in ("conv1x1_bn_bwd", "conv1x1_bn_prenorm_bwd"):
        # BatchNorm backward as the method defines it reads dY and z twice (the batch means, then the gradient);
        # then x in and dX out; dz itself is not counted.  (Where the successor's kernel hands the two means' sums
        # down, the first read does not happen: the counters' traffic is then below this figure.)
        B, Nb, Ci, Co, L, dt = a[:6]
        has_dx = (a[17] if name == "conv1x1_bn_bwd" else a[23]) is not None
        return (B * Nb * (4 * Co + (2 if has_dx else 1) * Ci) * L + B * Co * Ci) * _es(dt) + B * Co * (Ci + 3) * 4
    if name in ("linear_fwd", "linear_fwd_ws"):
        B, M, Fx, Fy, dt = a[:5]
        return B * (M * Fx + Fx * Fy + Fy + M * Fy) * _es(dt)
    if name == "conv1x1_bwd":
        B, Nb, Ci, Co, L, dt = a[:6]
        if a[11] is not None:          # dX = W^T dY: dY and W in, dX out
            return (B * Nb * (Ci + Co) * L + B * Co * Ci) * _es(dt)
        return B * Nb * (Ci + Co) * L * _es(dt) + B * Co * Ci * 4      # dW (fp32) = dY X^T
    if name in ("conv1x1_bn_maxpool_fwd", "conv1x1_bn_maxpool_prenorm_fwd"):      # x in, W in, pooled + argmax + z at the argmax out
        B, Nb, Ci, Co, L, dt = a[:6]
        return B * Nb * Ci * L * _es(dt) + B * Co * Ci * _es(dt) + B * Nb * Co * (_es(dt) + 4 + 4)
    if name in ("conv1x1_bn_maxpool_bwd", "conv1x1_bn_maxpool_prenorm_bwd"):      # x in, dx out, W in, dW (fp32) out, pooled gradient + argmax in
        B, Nb, Ci, Co, L, dt = a[:6]
        return 2 * B * Nb * Ci * L * _es(dt) + B * Co * Ci * (_es(dt) + 4) + B * Nb * Co * (_es(dt) + 4 + _es(dt))
    if name == "linear_bwd":
        B, M, Fx, Fy, dt = a[:5]
        if a[8] is not None and a[9] is not None:      # x, W, dy in; dx, dW (fp32), dbias out
            return B * (2 * M * Fx + Fx * Fy + M * Fy) * _es(dt) + B * (Fx * Fy + Fy) * 4
        if a[8] is not None:
            return B * (M * Fy + Fx * Fy + M * Fx) * _es(dt)
        if a[9] is not None:
            return B * (M * Fx + M * Fy) * _es(dt) + B * Fx * Fy * 4
        return B * M * Fy * _es(dt)
    if name in ("conv2d_grouped_fwd", "conv2d_grouped_bwd"):
        B, Nb, Ci, Co, H, W, kh, kw, st, pad, dt = a[:11]
        Ho, Wo = (H + 2 * pad - kh) // st + 1, (W + 2 * pad - kw) // st + 1
        act_bytes = B * Nb * (Ci * H * W + Co * Ho * Wo) * _es(dt)
        wbytes = B * Co * Ci * kh * kw
        if name == "conv2d_grouped_bwd" and a[14] is None:
            return act_bytes + wbytes * 4          # dW is fp32
        return act_bytes + wbytes * _es(dt)
    if name == "bias_act_nchw":
        return 2 * a[0] * a[1] * a[2] * _es(a[3])
    if name == "attention_fwd":               # qkv in, probabilities and context out
        B, N, S, E, H, dt = a[:6]
        return B * N * S * (4 * E + H * S) * _es(dt)
    if name == "attention_bwd":               # qkv, probabilities, dctx in, dqkv out
        B, N, S, E, H, dt = a[:6]
        return B * N * S * (7 * E + H * S) * _es(dt)
    if name in ("embedding_fwd", "embedding_bwd"):
        B, R, V, E, dt = a[:5]
        return B * R * E * 2 * _es(dt) if name == "embedding_fwd" else B * (R * E * _es(dt) + V * E * 4)
    if name in ("softmax_xent", "softmax_xent_rows"):
        return 2 * a[0] * a[1] * a[2] * _es(a[3])
    if name in ("add_sample_bias", "softmax_xent_points"):
        return 2 * a[0] * a[1] * a[2] * a[3] * _es(a[4])
    if name == "add_strided":
        return 3 * a[0] * a[1] * a[2] * a[3] * _es(a[4])
    if name == "sum_points":
        return a[0] * a[1] * a[2] * a[3] * _es(a[4])
    if name == "point_transform_fwd":         # x in, y out, one small matrix per cloud
        B, Nb, Ci, Co, L, dt = a[:6]
        return B * Nb * ((Ci + Co) * L + Ci * Co) * _es(dt)
    if name == "point_transform_bwd":         # x, dy in; dx (if asked for) and the matrix gradient out
        B, Nb, Ci, Co, L, dt = a[:6]
        return B * Nb * ((Ci + Co + (Ci if a[11] is not None else 0)) * L + 2 * Ci * Co) * _es(dt)
    if name == "act_fwd":
        return 2 * a[0] * _es(a[1])
    if name in ("act_bwd", "add"):
        return 3 * a[0] * _es(a[1])
    if name == "act_bwd_colsum":              # z, dy in, dx out (the column sums are 4 bytes per column)
        return 3 * a[0] * a[1] * a[2] * _es(a[3])
    if name == "layernorm_fwd":
        return 2 * a[0] * a[1] * a[2] * _es(a[3])
    if name == "layernorm_bwd":
        return 3 * a[0] * a[1] * a[2] * _es(a[3])
    if name == "layernorm_bwd_sums":          # x, dy (and dy2) in, dx out
        return (4 if a[6] is not None else 3) * a[0] * a[1] * a[2] * _es(a[3])
    if name == "maxpool_points":
        B, Nb, C, L, dt = a[:5]
        return B * Nb * C * (L * _es(dt) + _es(dt) + 4)
    if name == "maxpool_points_bwd":
        B, Nb, C, L, dt = a[:5]
        return B * Nb * C * (L * _es(dt) + _es(dt) + 4)
    if name == "adam_step_multi":
        B, off = a[0], a[1]
        return B * off[-1] * (4 * 4 + 3 * 4 + (2 if a[7] is not None else 0))
    return 0


# ------------------------------------------------------------------ legs
def time_steps(arr, torch, steps, warmup):
    for _ in range(warmup):
        arr.train_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        arr.train_step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def ops_report(torch, binding):
    """Operator-level rooflines at the shapes of the other BASELINE configs (not the headline
    line): config 4's MLP GEMMs against the bf16 MFMA peak, config 3's grouped 4x4 stride-2
    convolutions, each timed with HIP events on the launch stream."""
    hb = binding
    bf = torch.bfloat16
    MFMA_PEAK = 2500.0          # TFLOP/s, dense bf16

    def timeit(fn, n=100, warm=30):
        # the first entry timed after new tensors were made ran 10-20 % slow with 30 warm-up launches alone (clocks
        # and caches had not settled): a few milliseconds of the same launches first, then the warm-up proper
        for _ in range(3 * warm):
            fn()
        torch.cuda.synchronize()
        for _ in range(warm):
            fn()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for _ in range(n):
            fn()
        e.record()
        torch.cuda.synchronize()
        return s.elapsed_time(e) / n * 1e-3

    out = []
    B, M = 16, 4096
    for fx, fy in ((512, 2048), (2048, 512)):
        X = torch.randn(B, M, fx, device="cuda").to(bf)
        W = (torch.randn(B, fx, fy, device="cuda") / fx ** 0.5).to(bf)
        bias = torch.randn(B, fy, device="cuda").to(bf)
        Y = torch.empty(B, M, fy, device="cuda", dtype=bf)
        dY = torch.randn(B, M, fy, device="cuda").to(bf)
        dX = torch.empty_like(X)
        dW = torch.empty(B, fx, fy, device="cuda")
        ws = torch.empty(max(4, hb.linear_bwd_workspace_bytes(B, M, fx, fy, 1)), dtype=torch.uint8, device="cuda")
        fl = 2.0 * B * M * fx * fy
        for name, fn in (("linear_fwd", lambda: hb.linear_fwd(B, M, fx, fy, 1, X, W, bias, Y)),
                         ("linear_fwd+gelu", lambda: hb.linear_fwd(B, M, fx, fy, 1, X, W, bias, Y, hb.ACT_GELU)),
                         ("linear_dX", lambda: hb.linear_bwd(B, M, fx, fy, 1, None, W, dY, dX, None, None, None)),
                         ("linear_dW", lambda: hb.linear_bwd(B, M, fx, fy, 1, X, None, dY, None, dW, None, ws))):
            t = timeit(fn)
            out.append(dict(op=name, workload=f"c4 B=16 M=4096 {fx}->{fy} bf16", ms=t * 1e3, bound="mfma",
                            achieved=fl / t / 1e12, peak=MFMA_PEAK, unit="TFLOP/s", frac=fl / t / 1e12 / MFMA_PEAK))
    B, Nb = 10, 64
    for ci, co, H in ((3, 64, 64), (64, 128, 32), (128, 256, 16), (256, 512, 8)):
        Ho = H // 2
        X = torch.randn(Nb, B * ci, H, H, device="cuda").to(bf)
        W = (torch.randn(B * co, ci, 4, 4, device="cuda") * 0.02).to(bf)
        Y = torch.empty(Nb, B * co, Ho, Ho, device="cuda", dtype=bf)
        dY = torch.randn_like(Y)
        dX = torch.empty_like(X)
        dW = torch.empty(B * co, ci, 4, 4, device="cuda")
        geo = (B, Nb, ci, co, H, H, 4, 4, 2, 1, 1)
        ws = torch.empty(max(4, hb.conv2d_grouped_bwd_workspace_bytes(*geo), hb.conv2d_grouped_fwd_workspace_bytes(*geo)),
                         dtype=torch.uint8, device="cuda")
        nmin = hb.conv2d_grouped_bwd_min_workspace_bytes(*geo)
        wmin = torch.empty(nmin, dtype=torch.uint8, device="cuda") if nmin else None
        fl = 2.0 * B * Nb * Ho * Ho * ci * co * 16
        for name, fn in (("conv2d_fwd", lambda: hb.conv2d_grouped_fwd(*geo, X, W, None, Y, workspace=ws)),
                         ("conv2d_dX", lambda: hb.conv2d_grouped_bwd(*geo, None, W, dY, dX, None, None, ws)),
                         ("conv2d_dW", lambda: hb.conv2d_grouped_bwd(*geo, X, None, dY, None, dW, None, ws)),
                         ("conv2d_fwd (no workspace: no split of the reduction)", lambda: hb.conv2d_grouped_fwd(*geo, X, W, None, Y)),
                         ("conv2d_dX (no workspace: fallback that gathers single taps, no regrouped weights)", lambda: hb.conv2d_grouped_bwd(*geo, None, W, dY, dX, None, None, None)),
                         ("conv2d_dW (minimal workspace: fewest partial slices)", lambda: hb.conv2d_grouped_bwd(*geo, X, None, dY, None, dW, None, wmin))):
            t = timeit(fn)
            out.append(dict(op=name, workload=f"c3 B=10 Nb=64 {ci}->{co} {H}x{H} k4 s2 p1 bf16", ms=t * 1e3, bound="mfma",
                            achieved=fl / t / 1e12, peak=MFMA_PEAK, unit="TFLOP/s", frac=fl / t / 1e12 / MFMA_PEAK))
    return out


MFMA_PEAK_TFLOPS = 2500.0    # MI355X dense bf16 MFMA
BF16_RIDGE = MFMA_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)   # flop per byte above which a GEMM is MFMA-bound


class Workload:
    """What the legs of the benchmark need to know about one BASELINE configuration."""

    def __init__(self, name):
        import hfta_inputs as hi
        from paper_2102_02344_amd import arrays
        self.name = name
        if name in ("c0", "c1"):
            from oracle import pointnet as oracle_model
            self.spec = hi.spec_c1() if name == "c1" else hi.spec_c0()
            self.inp = hi.pointnet_cls_inputs(self.spec)
            self.cls = arrays.FusedPointNetCls
            self.per_model_keys = ("labels",)
            self.config = {"workload": self.spec.name, "B": self.spec.B, "batch_per_model": self.spec.Nb,
                           "points": self.spec.L, "conv": list(self.spec.conv), "fc": list(self.spec.fc),
                           "step": "fwd+bwd+Adam"}
        elif name == "c1t":
            from oracle import pointnet_t as oracle_model
            self.spec = hi.PointNetTSpec(cls=hi.spec_c1())
            self.inp = hi.pointnet_t_inputs(self.spec)
            self.cls = arrays.FusedPointNetClsT
            self.per_model_keys = ("labels",)
            c = self.spec.cls
            self.config = {"workload": self.spec.name, "B": c.B, "batch_per_model": c.Nb, "points": c.L,
                           "conv": list(c.conv), "fc": list(c.fc),
                           "transform_subnetworks": {"sizes": hi.tnet_sizes(self.spec), "conv": list(self.spec.tnet_conv),
                                                     "fc": list(self.spec.tnet_fc)}, "step": "fwd+bwd+Adam"}
        elif name == "c2":
            from oracle import pointnet_seg as oracle_model
            self.spec = hi.spec_c2()
            self.inp = hi.pointnet_seg_inputs(self.spec)
            self.cls = arrays.FusedPointNetSeg
            self.per_model_keys = ("labels", "onehot", "category")
            self.config = {"workload": self.spec.name, "B": self.spec.B, "batch_per_model": self.spec.Nb,
                           "points": self.spec.L, "conv": list(self.spec.conv), "head": list(self.spec.head),
                           "step": "fwd+bwd+Adam"}
        elif name == "t0":
            from oracle import transformer as oracle_model
            self.spec = hi.spec_t0()
            self.inp = hi.transformer_inputs(self.spec)
            self.cls = arrays.FusedTransformerLM
            self.per_model_keys = ("tokens", "targets")
            self.config = {"workload": self.spec.name, "B": self.spec.B, "sequences_per_model": self.spec.N,
                           "tokens_per_sequence": self.spec.S, "width": self.spec.E, "heads": self.spec.heads,
                           "ffn": self.spec.F, "layers": self.spec.layers, "vocab": self.spec.V, "step": "fwd+bwd+Adam"}
        elif name == "c3":
            from oracle import dcgan as oracle_model
            self.spec = hi.spec_c3()
            self.inp = hi.dcgan_inputs(self.spec)
            self.cls = arrays.FusedDcgan
            self.per_model_keys = ()
            self.config = {"workload": self.spec.name, "B": self.spec.B, "images_per_model": self.spec.Nb,
                           "image": "64x64x3", "generator": [l[:2] for l in self.spec.g_layers],
                           "discriminator": [l[:2] for l in self.spec.d_layers],
                           "step": "D step (real + fake) + G step, two Adam optimisers"}
        else:
            from oracle import mlp as oracle_model
            self.spec = hi.spec_c4()
            self.inp = hi.mlp_inputs(self.spec)
            self.cls = arrays.FusedMlp
            self.per_model_keys = ("tokens", "targets")
            self.config = {"workload": self.spec.name, "B": self.spec.B, "sequences_per_model": self.spec.Nb,
                           "tokens_per_sequence": self.spec.R // self.spec.Nb, "width": self.spec.E,
                           "hidden": self.spec.H, "blocks": self.spec.blocks, "step": "fwd+bwd+Adam"}
        self.oracle = oracle_model
        self.samples = self.spec.B * self.spec.Nb

    def one_model(self, b):
        """(spec, inputs) of model b alone: the serial scheme's unit."""
        s1 = self.spec.with_cls(B=1) if self.name == "c1t" else dataclasses.replace(self.spec, B=1)
        i1 = dict(self.inp)
        if self.name in ("c0", "c1", "c1t", "c2"):
            i1["points"] = np.ascontiguousarray(self.inp["points"][:, 3 * b:3 * b + 3])
        if self.name in ("c0", "c1", "c1t"):
            i1["drop_mask"] = None if self.inp["drop_mask"] is None else self.inp["drop_mask"][b:b + 1]
        for k in self.per_model_keys + ("lr", "beta1", "beta2", "eps", "wd"):
            i1[k] = self.inp[k][b:b + 1]          # ("pos" of the Transformer workload is shared by the models)
        if self.name == "c3":
            cz = self.spec.g_layers[0][0]
            i1["z"] = np.ascontiguousarray(self.inp["z"][:, cz * b:cz * (b + 1)])
            i1["real"] = np.ascontiguousarray(self.inp["real"][:, 3 * b:3 * b + 3])
            i1["gparams"], i1["dparams"] = self.inp["gparams"][b:b + 1], self.inp["dparams"][b:b + 1]
        else:
            i1["params"] = self.inp["params"][b:b + 1]
        return s1, i1

    def cpu_baseline(self):
        """The oracle as it stands on a bounded sample of one model; its cost is linear in the sample."""
        import hfta_inputs as hi
        if self.name in ("c0", "c1"):
            small = dataclasses.replace(self.spec, B=1, Nb=min(16, self.spec.Nb))
            inp = hi.pointnet_cls_inputs(small)
            nsamp = small.Nb
            what = f"1 model x {small.Nb} clouds x {small.L} points"
        elif self.name == "c1t":
            small = self.spec.with_cls(B=1, Nb=8)
            inp = hi.pointnet_t_inputs(small)
            nsamp = small.Nb
            what = f"1 model x {small.Nb} clouds x {small.L} points, with transform sub-networks"
        elif self.name == "c2":
            small = dataclasses.replace(self.spec, B=1, Nb=2)
            inp = hi.pointnet_seg_inputs(small)
            nsamp = small.Nb
            what = f"1 model x {small.Nb} clouds x {small.L} points"
        elif self.name == "t0":
            small = dataclasses.replace(self.spec, B=1, N=8)
            inp = hi.transformer_inputs(small)
            nsamp = small.N
            what = f"1 model x {small.N} sequences x {small.S} tokens, {small.layers} layers, vocabulary {small.V}"
        elif self.name == "c3":
            small = dataclasses.replace(self.spec, B=1, Nb=4)
            inp = hi.dcgan_inputs(small)
            nsamp = small.Nb
            what = f"1 generator/discriminator pair x {small.Nb} images"
        else:
            seqs = 4
            small = dataclasses.replace(self.spec, B=1, R=seqs * (self.spec.R // self.spec.Nb), Nb=seqs)
            inp = hi.mlp_inputs(small)
            nsamp = seqs
            what = f"1 model x {seqs} sequences x {self.spec.R // self.spec.Nb} tokens, {small.blocks} blocks"
        if self.name == "c3":
            gs, ds = [self.oracle.init_state(inp["gparams"][0])], [self.oracle.init_state(inp["dparams"][0])]
            t0 = time.perf_counter()
            self.oracle.array_train_iteration(small, gs, ds, inp, 1)
        else:
            states = [self.oracle.init_state(inp["params"][0])]
            t0 = time.perf_counter()
            self.oracle.array_train_step(small, states, inp, 1)
        dt = time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        return dict(value=nsamp / dt, unit="samples/s", cores=int(cores), kind="oracle",
                    sample=f"{what}, one fwd+bwd+Adam step ({dt:.1f} s), numpy float64; host has "
                           f"{os.cpu_count()} logical cores")


def _stats(xs):
    return dict(mean=float(np.mean(xs)), min=float(np.min(xs)), max=float(np.max(xs)))


def run_workload(name, args, torch, arrays, binding):
    """All legs of one workload: fused (REPEATS timed regions of `steps` steps each), the same models
    one after another with B = 1, the CPU oracle on a bounded sample, the per-entry table and the
    roofline of the entry with the largest share of a step."""
    wl = Workload(name)
    spec, inp = wl.spec, wl.inp
    tracer = Tracer(binding, torch)
    arrays.hb = tracer
    unf = args.unfused if name == "c1" else 0
    arr = wl.cls(spec, inp, unfused_layers=tuple(range(unf))) if unf else wl.cls(spec, inp)
    if unf:
        wl.config["unfused_per_point_layers"] = unf
    # Warm-up.  Its last steps bracket EVERY traced entry point with HIP events: the per-kernel table,
    # and which entry has the largest share of a step.  (Two events per call cost host time, about
    # as much as a whole step of config 1 for ~50 calls, so the timed region cannot carry them all.)
    survey = max(1, min(2, args.warmup))
    for _ in range(max(0, args.warmup - survey)):
        arr.train_step()
    torch.cuda.synchronize()
    tracer.enabled = True
    for _ in range(survey):
        arr.train_step()
    tot = tracer.summary()
    per_kernel = {k: dict(launches_per_step=v[0] // survey, ms_per_step=v[1] / survey,
                          GBps=(v[2] / 1e9) / (v[1] / 1e3) if v[1] > 0 else None,
                          TFLOPs=(v[3] / 1e12) / (v[1] / 1e3) if v[1] > 0 and v[3] > 0 else None)
                  for k, v in sorted(tot.items(), key=lambda kv: -kv[1][1])}
    dom = max(tot.items(), key=lambda kv: kv[1][1])[0]
    # Timed regions: only the dominant entry's launches are bracketed, live, inside them
    tracer.events = []
    tracer.only = dom
    secs = []
    for _ in range(args.repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            arr.train_step()
        torch.cuda.synchronize()
        secs.append((time.perf_counter() - t0) / args.steps)
    tracer.enabled = False
    sec = float(np.mean(secs))
    nsteps = args.steps * args.repeats
    dv = tracer.summary()[dom]
    samples = wl.samples
    # HBM bytes per launch of that entry from the committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    # runs of this same command (profiles/<workload>_traffic.json); null when not collected
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"{name}_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(dom)
    common = dict(kernel=dom, traffic=traffic, avg_launch_us=1e3 * dv[1] / dv[0],
                  launches_per_step=dv[0] // nsteps, algorithmic_bytes_per_launch=dv[2] / dv[0],
                  share_of_step=(dv[1] / nsteps) / (sec * 1e3))
    if dv[3] > 0 and dv[3] / dv[2] > BF16_RIDGE and spec.dtype == "bf16":
        achieved = (dv[3] / 1e12) / (dv[1] / 1e3)
        roofline = dict(bound="mfma", achieved=achieved, peak=MFMA_PEAK_TFLOPS, unit="TFLOP/s",
                        frac=achieved / MFMA_PEAK_TFLOPS, algorithmic_flop_per_launch=dv[3] / dv[0], **common)
    else:
        achieved = (dv[2] / dv[0]) / 1e9 / ((dv[1] / dv[0]) / 1e3)
        roofline = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=achieved / HBM_PEAK_GBS, **common)
    del arr
    torch.cuda.empty_cache()

    serial = None
    if not args.skip_serial:
        arrays.hb = binding
        nser = max(3, args.steps // 4)
        rep = np.zeros(args.repeats)
        for b in range(spec.B):          # one model resident at a time: B models, one after another
            s1, i1 = wl.one_model(b)
            mdl = wl.cls(s1, i1)
            rep += np.array([time_steps(mdl, torch, nser, 2 if r == 0 else 0) for r in range(args.repeats)])
            del mdl
        ssec = float(rep.mean())
        serial = dict(value=samples / ssec, unit="samples/s", ms_per_step_all_models=ssec * 1e3,
                      ms_per_step_all_models_stats=_stats(rep * 1e3), fused_speedup=ssec / sec,
                      steps_per_model=nser, repeats=args.repeats)
        torch.cuda.empty_cache()

    cpu = None if args.skip_cpu else wl.cpu_baseline()
    return {
        "value": samples / sec, "unit": "samples/s", "ms_per_step": sec * 1e3,
        "repeats": args.repeats, "value_stats": _stats([samples / t for t in secs]),
        "ms_per_step_stats": _stats([t * 1e3 for t in secs]),
        "dtype": spec.dtype, "data": "synthetic", "config": wl.config,
        "roofline": roofline, "serial_b1": serial, "cpu_baseline": cpu, "kernels": per_kernel,
        "kernels_note": f"per-entry HIP-event times from the last {survey} warm-up step(s); the roofline entry is timed inside the timed regions",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--repeats", type=int, default=3, help="timed regions of --steps steps each; mean / min / max are reported")
    ap.add_argument("--workload", default="all", choices=["all", "c0", "c1", "c1t", "c2", "c3", "c4", "t0"],
                    help="all (default): config 1 as the headline line plus a `workloads` block with configs 0, 2, 3, 4 "
                         "and the operator table; a name: that workload alone")
    ap.add_argument("--unfused", type=int, default=0,
                    help="config 1 only: run the first K per-point layers (and their share of Adam) model by model "
                         "(partial fusion); the headline line is K = 0")
    ap.add_argument("--skip-serial", action="store_true")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--skip-ops", action="store_true", help="leave the operator table out of the default run")
    ap.add_argument("--ops-report", default=None,
                    help="also write the operator table (GEMMs at config 4 shapes, conv2d at config 3 shapes) as JSON here")
    ap.add_argument("--copy-ref", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (models are independent and would shard over "
              "the model index without any exchange); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2102_02344_amd import arrays, binding

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)

    if args.copy_ref:
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device="cuda")      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    head_name = "c1" if args.workload == "all" else args.workload
    t_start = time.perf_counter()
    head = run_workload(head_name, args, torch, arrays, binding)
    out = {
        "metric": "fused train samples/sec summed over B models",
        "value": head["value"], "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
    }
    out.update({k: v for k, v in head.items() if k not in out})
    if args.workload == "all":
        # the other BASELINE configurations, same legs each: the small fp32 case, the segmentation
        # array, the GAN array and the MLP-block array (one JSON line carries all five)
        out["workloads"] = {}
        for name in ("c0", "c2", "c3", "c4"):
            print(f"bench.py: {name} ... ({time.perf_counter() - t_start:.0f} s so far)", file=sys.stderr, flush=True)
            w = run_workload(name, args, torch, arrays, binding)
            w.pop("kernels_note", None)
            out["workloads"][name] = w
    if args.ops_report or (args.workload == "all" and not args.skip_ops):
        print(f"bench.py: operator table ... ({time.perf_counter() - t_start:.0f} s so far)", file=sys.stderr, flush=True)
        ops = ops_report(torch, binding)
        if args.ops_report:
            with open(args.ops_report, "w") as f:
                json.dump(ops, f, indent=1)
        if args.workload == "all":
            out["operators"] = ops
            out["operators_note"] = ("entry points timed alone with HIP events (120 warm-up + 100 launches): fused Linear at "
                                     "config 4 shapes, grouped conv2d at config 3 shapes, against the dense bf16 MFMA peak")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
