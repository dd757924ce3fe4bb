"""Fused training arrays: B models of one architecture trained as one job.

This module only sequences calls into the C ABI (``binding``) and owns the
device buffers; every arithmetic step runs in the HIP kernels.  Parameters
live in a parameter-major arena (each fused parameter is one ``[B][...]``
tensor, as the fusion rules table concatenates weights along the model
dimension), so one ``adam_step_multi`` launch updates all B models with their
own learning rate, betas and weight decay.

Layouts: point-wise activations ``[Nb, B*C, L]`` (the table's Conv1d /
BatchNorm1d layout), head activations ``[B, Nb, F]`` (the table's baddbmm
layout); the max-pool writes straight from the first into the second.
"""
from __future__ import annotations

from typing import Dict, List, Tuple

import numpy as np
import torch

from . import binding as hb

_TDT = {"f32": torch.float32, "bf16": torch.bfloat16}
_DT = {"f32": hb.F32, "bf16": hb.BF16}


def _cs(B, C, L):
    return (C * L, B * C * L, L, 1)


def _bn_bwd_one_pass(B, Nb, ci, co, L, dt):
    """True when ``conv1x1_bn_bwd`` runs this layer as one streaming kernel (dz never stored).  Layers it
    would run as the two single operators are called as such here, with dz in one of the array's
    gradient buffers instead of a workspace of that size."""
    return hb.conv1x1_bn_bwd_one_pass(B, Nb, ci, co, L, dt)


class ParamArena:
    """Parameter-major storage of B models' parameters, gradients and Adam state.

    Fused parameter j is one ``[B][n_j]`` tensor (the fusion rules table concatenates weights
    along the model dimension); the arena is those back to back, so a GEMM sees ``[B][Fx][Fy]`` /
    ``[B][Co][Ci]`` directly and ONE ``adam_step_multi`` launch walks every parameter of every
    model with that model's own learning rate, betas and weight decay."""

    def _init_arena(self, shapes, B: int, inp: dict, dtype: str, dev):
        self.shapes: List[Tuple[str, Tuple[int, ...]]] = shapes
        self._index = {n: j for j, (n, _) in enumerate(shapes)}
        off = [0]
        for _, shp in shapes:
            off.append(off[-1] + int(np.prod(shp)))
        self.seg_offsets = off
        P = off[-1]
        self.P = P
        f32 = dict(dtype=torch.float32, device=dev)
        self.theta = torch.empty(B * P, **f32)
        self.grad = torch.zeros(B * P, **f32)
        self.m = torch.zeros(B * P, **f32)
        self.v = torch.zeros(B * P, **f32)
        self.lowp = torch.empty(B * P, dtype=torch.bfloat16, device=dev) if dtype == "bf16" else None
        host = np.empty(B * P, np.float32)
        for j, (name, shp) in enumerate(shapes):
            n = off[j + 1] - off[j]
            blk = np.stack([inp["params"][b][name].reshape(-1) for b in range(B)])
            host[B * off[j]:B * off[j] + B * n] = blk.reshape(-1)
        self.theta.copy_(torch.from_numpy(host))
        if self.lowp is not None:
            self.lowp.copy_(self.theta)           # initial cast only; afterwards Adam writes it
        self.hp = {k: torch.from_numpy(np.asarray(inp[k], np.float32)).to(dev)
                   for k in ("lr", "beta1", "beta2", "eps", "wd")}
        self.t = 0

    def load_params(self, params) -> None:
        """Overwrite the master weights (and their storage-dtype copy) with per-model values:
        ``params[b][name]`` float32 arrays.  Optimiser moments are left as they are."""
        host = np.empty(self.B * self.P, np.float32)
        off = self.seg_offsets
        for j, (name, shp) in enumerate(self.shapes):
            n = off[j + 1] - off[j]
            blk = np.stack([np.asarray(params[b][name], np.float32).reshape(-1) for b in range(self.B)])
            host[self.B * off[j]:self.B * off[j] + self.B * n] = blk.reshape(-1)
        self.theta.copy_(torch.from_numpy(host))
        if self.lowp is not None:
            self.lowp.copy_(self.theta)

    def _seg(self, buf: torch.Tensor, name: str) -> torch.Tensor:
        j = self._index[name]
        o, n = self.seg_offsets[j], self.seg_offsets[j + 1] - self.seg_offsets[j]
        return buf[self.B * o:self.B * (o + n)]

    def w(self, name: str) -> torch.Tensor:
        """Weights as the GEMMs read them (storage dtype)."""
        return self._seg(self.lowp if self.lowp is not None else self.theta, name)

    def master(self, name: str) -> torch.Tensor:
        return self._seg(self.theta, name)

    def g(self, name: str) -> torch.Tensor:
        return self._seg(self.grad, name)

    def param_host(self, buf: torch.Tensor, name: str, b: int) -> np.ndarray:
        shp = dict(self.shapes)[name]
        return self._seg(buf, name).view(self.B, *shp)[b].float().cpu().numpy()

    def adam(self):
        self.t += 1
        hb.adam_step_multi(self.B, self.seg_offsets, hb.F32, self.theta, self.grad, self.m, self.v, self.lowp,
                           self.hp["lr"], self.hp["beta1"], self.hp["beta2"], self.hp["eps"], self.hp["wd"], self.t)

    def adam_partial(self, unfused_prefixes):
        """Partially fused optimiser (section "Results", partial-fusion study): parameters whose name
        starts with one of ``unfused_prefixes`` are stepped model by model (B launches of the
        single-arena kernel each), the contiguous runs of all other parameters stay fused."""
        self.t += 1
        B, off, names = self.B, self.seg_offsets, [n for n, _ in self.shapes]
        unf = [any(n.startswith(p) for p in unfused_prefixes) for n in names]
        lp = self.lowp
        hp = self.hp
        j = 0
        while j < len(names):
            if unf[j]:
                n = off[j + 1] - off[j]
                for b in range(B):
                    o = B * off[j] + b * n
                    hb.adam_step(1, n, hb.F32, self.theta[o:], self.grad[o:], self.m[o:], self.v[o:],
                                 None if lp is None else lp[o:], hp["lr"][b:], hp["beta1"][b:], hp["beta2"][b:],
                                 hp["eps"][b:], hp["wd"][b:], self.t)
                j += 1
                continue
            j1 = j
            while j1 < len(names) and not unf[j1]:
                j1 += 1
            o = B * off[j]
            rel = [off[q] - off[j] for q in range(j, j1 + 1)]
            hb.adam_step_multi(B, rel, hb.F32, self.theta[o:], self.grad[o:], self.m[o:], self.v[o:],
                               None if lp is None else lp[o:], hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["wd"],
                               self.t)
            j = j1

    def adadelta(self, rho: torch.Tensor, eps: torch.Tensor):
        """Adadelta instead of Adam (``rho``, ``eps``: device ``[B]``); the two state buffers hold
        the running square average and the accumulated squared delta."""
        self.t += 1
        hb.adadelta_step_multi(self.B, self.seg_offsets, hb.F32, self.theta, self.grad, self.m, self.v, self.lowp,
                               self.hp["lr"], rho, eps, self.hp["wd"])

    def steplr(self, base_lr: torch.Tensor, gamma: torch.Tensor, step_size: torch.Tensor, epoch: int):
        """Per-model step schedule: rewrites the device learning-rate vector the optimisers read."""
        hb.steplr(self.B, base_lr, gamma, step_size, epoch, self.hp["lr"])

    def train_step(self):
        loss = self.forward_backward()
        self.adam()
        return loss


class FusedPointNetCls(ParamArena):
    """PointNet-classification-style array (per-point k=1 convolutions + BatchNorm +
    ReLU, max over points, fully connected head, softmax cross-entropy, Adam)."""

    def train_step(self):
        loss = self.forward_backward()
        if self.unfused:
            self.adam_partial([f"conv{i}." for i in self.unfused])
        else:
            self.adam()
        return loss

    BN_EPS = 1e-5
    BN_MOMENTUM = 0.1

    def __init__(self, spec, inp: dict, device: str = "cuda", fused_tail: bool = True, unfused_layers=(),
                 tail_prenorm: bool = False):
        """``unfused_layers``: indices of per-point layers (convolution + BatchNorm, forward and
        backward, and their share of the optimiser) that run model by model -- B launches with B = 1
        on the same buffers -- instead of once for the whole array: the partial fusion of the
        paper's sensitivity study.  The last per-point layer stays fused when ``fused_tail`` applies.
        ``tail_prenorm``: the layer in front of the one-operator tail skips its normalisation pass and
        the tail's first kernel forms (and writes) the activated tensor instead; same bits, and on the
        headline shape the same time within noise (the kernel that takes the work on is bound by its
        matrix products and slows down by what the pass cost), hence off by default."""
        self.spec = spec
        self.unfused = frozenset(int(i) for i in unfused_layers)
        self.B, self.Nb, self.L = spec.B, spec.Nb, spec.L
        self.dtype = spec.dtype
        self.dt = _DT[spec.dtype]
        self.tdt = _TDT[spec.dtype]
        self.dev = torch.device(device)
        B, Nb, L = self.B, self.Nb, self.L

        import hfta_inputs as hi
        self._init_arena(hi.pointnet_cls_param_shapes(spec), B, inp, spec.dtype, self.dev)
        f32 = dict(dtype=torch.float32, device=self.dev)

        # ---- BatchNorm running statistics / saved statistics -------------------
        self.running: Dict[str, torch.Tensor] = {}
        self.saved: Dict[str, torch.Tensor] = {}
        for name, shp in self.shapes:
            if name.endswith(".bn.g"):
                k = name[:-2]
                self.running[k + ".rm"] = torch.zeros(B * shp[0], **f32)
                self.running[k + ".rv"] = torch.ones(B * shp[0], **f32)
                self.saved[k + ".mean"] = torch.empty(B * shp[0], **f32)
                self.saved[k + ".invstd"] = torch.empty(B * shp[0], **f32)

        # ---- activations ----------------------------------------------------------
        act = dict(dtype=self.tdt, device=self.dev)
        self.nconv = len(spec.conv) - 1
        self.nfc = len(spec.fc) - 1
        # The last per-point layer, its BatchNorm, ReLU and the max over points run as one operator,
        # forward and backward, where the library supports the shape: its [Nb, B*C, L] output and the
        # gradient of that tensor are then never allocated.
        self.fused_tail = False
        if fused_tail and self.nconv >= 2:
            geo = (B, Nb, spec.conv[-2], spec.conv[-1], L, self.dt)
            self.fused_tail_ws = max(hb.conv1x1_bn_maxpool_fwd_workspace_bytes(*geo),
                                     hb.conv1x1_bn_maxpool_bwd_workspace_bytes(*geo))
            self.fused_tail = hb.conv1x1_bn_maxpool_fwd_workspace_bytes(*geo) > 0
        nz = self.nconv - 1 if self.fused_tail else self.nconv
        self.z = [torch.empty(Nb, B * c, L, **act) for c in spec.conv[1:1 + nz]]
        # prenorm[i]: layer i takes layer i-1's stored pre-activation and normalises it on load (forward and
        # backward), so the activated tensor a[i-1] between the two is never stored.  The layer in front of the
        # tail keeps its activated output (the tail operator reads it).
        self.prenorm = [False] * self.nconv
        if not self.unfused:
            for i in range(1, self.nconv - 1):
                self.prenorm[i] = hb.conv1x1_bn_prenorm_supported(B, Nb, spec.conv[i], spec.conv[i + 1], L, self.dt)
        # ... unless the tail is the one-operator form: its first kernel normalises on load and writes the activated
        # tensor out on the way (tail_x), so that layer skips its own normalisation pass over the tensor
        self.tail_prenorm = bool(tail_prenorm) and self.fused_tail and not self.unfused and self.nconv >= 2
        self.tail_x = None
        if self.tail_prenorm:
            self.prenorm[self.nconv - 1] = True
            self.tail_x = torch.empty(Nb, B * spec.conv[-2], L, **act)
        self.a = [None if self.prenorm[i + 1] else torch.empty(Nb, B * c, L, **act)
                  for i, c in enumerate(spec.conv[1:-1])]                        # the last layer's is never stored
        self._atmp = None
        cmax = max(spec.conv[1:1 + nz])
        self.dbuf = [torch.empty(Nb * B * cmax * L, **act) for _ in range(2)]
        Cp = spec.conv[-1]
        self.pooled = torch.empty(B, Nb, Cp, **act)
        self.pool_idx = torch.empty(B, Nb, Cp, dtype=torch.int32, device=self.dev)
        if self.fused_tail:
            self.zhit = torch.empty(B, Nb, Cp, **f32)
            self.tail_moments = torch.empty(hb.conv1x1_bn_maxpool_saved_floats(B, spec.conv[-2], Cp), **f32)
        self.fz = [torch.empty(B, Nb, f, **act) for f in spec.fc[1:]]
        self.fh = [torch.empty(B, Nb, f, **act) for f in spec.fc[1:-1]]
        self.fdrop = torch.empty(B, Nb, spec.fc[-2], **act) if spec.dropout_p > 0 else None
        fmax = max(spec.fc)
        self.fd = [torch.empty(B * Nb * fmax, **act) for _ in range(2)]
        self.loss = torch.empty(B, **f32)
        ws = 4
        self.one_pass = [_bn_bwd_one_pass(B, Nb, spec.conv[i], spec.conv[i + 1], L, self.dt) for i in range(self.nconv)]
        # bn_sums[i]: the two reductions of layer i's BatchNorm backward, left by layer i+1's backward call (which
        # holds layer i's pre-activation and output gradient in registers anyway) so that layer i's call skips its
        # own pass over the two tensors
        self.bn_sums = [None] * self.nconv
        for i in range(1, self.nconv):
            if self.prenorm[i] and i < self.nconv - 1 and self.one_pass[i - 1] and \
                    hb.conv1x1_bn_prenorm_bwd_gives_sums(B, Nb, spec.conv[i], spec.conv[i + 1], L, self.dt):
                self.bn_sums[i - 1] = torch.empty(B * spec.conv[i], 2, **f32)
        for i in range(self.nconv):
            ws = max(ws, hb.conv1x1_bwd_workspace_bytes(B, Nb, spec.conv[i], spec.conv[i + 1], L, self.dt),
                     hb.conv1x1_bn_fwd_workspace_bytes(B, Nb, spec.conv[i], spec.conv[i + 1], L, self.dt))
            if i < self.nconv - 1:
                if i in self.unfused:
                    ws = max(ws, hb.conv1x1_bn_bwd_workspace_bytes(1, Nb, spec.conv[i], spec.conv[i + 1], L, self.dt))
                elif self.one_pass[i]:
                    ws = max(ws, hb.conv1x1_bn_bwd_workspace_bytes(B, Nb, spec.conv[i], spec.conv[i + 1], L, self.dt))
        for i in range(self.nfc):
            ws = max(ws, hb.linear_bwd_workspace_bytes(B, Nb, spec.fc[i], spec.fc[i + 1], self.dt),
                     hb.linear_fwd_workspace_bytes(B, Nb, spec.fc[i], spec.fc[i + 1], self.dt))
        if not self.fused_tail:
            self.fused_tail_ws = 0
        ws = max(ws, self.fused_tail_ws)
        self.ws = torch.empty(ws, dtype=torch.uint8, device=self.dev)

        # ---- inputs -----------------------------------------------------------------
        self.points = torch.from_numpy(inp["points"]).to(self.tdt).to(self.dev)
        self.labels = torch.from_numpy(inp["labels"]).to(self.dev)
        self.drop_mask = None
        if spec.dropout_p > 0:
            self.drop_mask = torch.from_numpy(inp["drop_mask"]).to(self.dev)

    # ------------------------------------------------------------------ one step
    def _act(self, i):
        """Activated output of per-point layer i: the stored tensor, or -- for a layer whose consumer normalises
        on load, and only for tests that look at every tensor -- the same bits written out from the stored
        pre-activation and the saved statistics."""
        if self.a[i] is not None:
            return self.a[i]
        s, B, Nb, L = self.spec, self.B, self.Nb, self.L
        co, k, cs = s.conv[i + 1], f"conv{i}", _cs(self.B, s.conv[i + 1], self.L)
        if self._atmp is None:
            self._atmp = torch.empty(Nb * B * max(s.conv[1:-1]) * L, dtype=self.tdt, device=self.dev)
        t = self._atmp[:Nb * B * co * L].view(Nb, B * co, L)
        hb.bn_apply_fwd(B, Nb, co, L, self.dt, self.z[i], cs, self.master(k + ".bn.g"), self.master(k + ".bn.b"),
                        self.saved[k + ".bn.mean"], self.saved[k + ".bn.invstd"], t, cs, hb.ACT_RELU)
        return t

    def forward_backward(self, probe=None):
        """One forward + backward pass.  ``probe(op, **tensors)``, if given, is called after
        every library call with the tensors that call read and wrote (tests use it to check
        each operator in place against the oracle on the very bits the GPU consumed)."""
        s, B, Nb, L, dt = self.spec, self.B, self.Nb, self.L, self.dt
        eps, mom = self.BN_EPS, self.BN_MOMENTUM
        P = probe if probe is not None else (lambda op, **kw: None)
        # per-point MLP
        x, ci = self.points, s.conv[0]
        for i in range(self.nconv):
            co = s.conv[i + 1]
            k = f"conv{i}"
            if i == self.nconv - 1 and self.fused_tail:
                vs = (Nb * co, co, 1)
                tail = (self.w(k + ".w"), self.w(k + ".b"), self.master(k + ".bn.g"), self.master(k + ".bn.b"), eps, mom,
                        self.running[k + ".bn.rm"], self.running[k + ".bn.rv"], self.saved[k + ".bn.mean"],
                        self.saved[k + ".bn.invstd"], self.pooled, self.pool_idx, vs, self.zhit, self.tail_moments,
                        hb.ACT_RELU, 0.0, self.ws)
                if self.tail_prenorm:
                    kp = f"conv{i - 1}"
                    hb.conv1x1_bn_maxpool_prenorm_fwd(B, Nb, ci, co, L, dt, self.z[i - 1], _cs(B, ci, L),
                                                      self.master(kp + ".bn.g"), self.master(kp + ".bn.b"),
                                                      self.saved[kp + ".bn.mean"], self.saved[kp + ".bn.invstd"],
                                                      hb.ACT_RELU, 0.0, *tail, Xact=self.tail_x, xas=_cs(B, ci, L))
                    x = self.tail_x
                else:
                    hb.conv1x1_bn_maxpool_fwd(B, Nb, ci, co, L, dt, x, _cs(B, ci, L), *tail)
                P("conv1x1_bn_maxpool_fwd", layer=k, x=x, w=self.w(k + ".w"), b=self.w(k + ".b"),
                  g=self.master(k + ".bn.g"), bt=self.master(k + ".bn.b"), v=self.pooled, idx=self.pool_idx,
                  mean=self.saved[k + ".bn.mean"], invstd=self.saved[k + ".bn.invstd"], zhit=self.zhit)
                ci = co
                break
            if i in self.unfused and i < self.nconv - 1:
                self._layer_fwd_unfused(i, x, ci, co)
                x, ci = self.a[i], co
                continue
            if i < self.nconv - 1:
                # convolution + BatchNorm + ReLU in one call: the convolution's epilogue leaves the
                # statistics' partial sums, so z is read once for the normalisation -- or not at all here,
                # where the next layer normalises it on load (y is None)
                y = self.a[i]
                bnp = (self.master(k + ".bn.g"), self.master(k + ".bn.b"), eps, mom, self.running[k + ".bn.rm"],
                       self.running[k + ".bn.rv"], self.saved[k + ".bn.mean"], self.saved[k + ".bn.invstd"])
                if self.prenorm[i]:
                    kp = f"conv{i - 1}"
                    hb.conv1x1_bn_prenorm_fwd(B, Nb, ci, co, L, dt, self.z[i - 1], _cs(B, ci, L), self.master(kp + ".bn.g"),
                                              self.master(kp + ".bn.b"), self.saved[kp + ".bn.mean"],
                                              self.saved[kp + ".bn.invstd"], hb.ACT_RELU, 0.0, self.w(k + ".w"),
                                              self.w(k + ".b"), *bnp, self.z[i], _cs(B, co, L), y,
                                              None if y is None else _cs(B, co, L), hb.ACT_RELU, 0.0, self.ws)
                else:
                    hb.conv1x1_bn_fwd(B, Nb, ci, co, L, dt, x, _cs(B, ci, L), self.w(k + ".w"), self.w(k + ".b"), *bnp,
                                      self.z[i], _cs(B, co, L), y, None if y is None else _cs(B, co, L), hb.ACT_RELU, 0.0,
                                      self.ws)
                if probe is not None:
                    P("conv1x1_fwd", layer=k, x=self._act(i - 1) if self.prenorm[i] else x, w=self.w(k + ".w"),
                      b=self.w(k + ".b"), y=self.z[i])
                    P("bn_fwd", layer=k, layout="conv", x=self.z[i], g=self.master(k + ".bn.g"), b=self.master(k + ".bn.b"),
                      y=self._act(i), mean=self.saved[k + ".bn.mean"], invstd=self.saved[k + ".bn.invstd"])
                x, ci = y, co
                continue
            hb.conv1x1_fwd(B, Nb, ci, co, L, dt, x, _cs(B, ci, L), self.w(k + ".w"), self.w(k + ".b"),
                           self.z[i], _cs(B, co, L))
            P("conv1x1_fwd", layer=k, x=x, w=self.w(k + ".w"), b=self.w(k + ".b"), y=self.z[i])
            if i == self.nconv - 1:
                # last per-point layer: BatchNorm + ReLU + max over points in one operator; the
                # activated [Nb, B*C, L] tensor is never written
                vs = (Nb * co, co, 1)
                hb.bn_fwd_maxpool(B, Nb, co, L, dt, self.z[i], _cs(B, co, L), self.master(k + ".bn.g"),
                                  self.master(k + ".bn.b"), eps, mom, self.running[k + ".bn.rm"],
                                  self.running[k + ".bn.rv"], self.saved[k + ".bn.mean"],
                                  self.saved[k + ".bn.invstd"], self.pooled, self.pool_idx, vs, hb.ACT_RELU)
                P("bn_fwd_maxpool", layer=k, x=self.z[i], g=self.master(k + ".bn.g"), b=self.master(k + ".bn.b"),
                  v=self.pooled, idx=self.pool_idx, mean=self.saved[k + ".bn.mean"],
                  invstd=self.saved[k + ".bn.invstd"])
                ci = co
                break
        Cp = ci
        # head
        h, fx = self.pooled, s.fc[0]
        for i in range(self.nfc):
            fy = s.fc[i + 1]
            k = f"fc{i}"
            last = i == self.nfc - 1
            if last or s.fc_bn:
                hb.linear_fwd_ws(B, Nb, fx, fy, dt, h, self.w(k + ".w"), self.w(k + ".b"), self.fz[i], workspace=self.ws)
                P("linear_fwd", layer=k, x=h, w=self.w(k + ".w"), b=self.w(k + ".b"), y=self.fz[i], act=0)
                if not last:
                    ls = (Nb * fy, fy, 1, 1)
                    hb.bn_fwd(B, Nb, fy, 1, dt, self.fz[i], ls, self.master(k + ".bn.g"), self.master(k + ".bn.b"),
                              eps, mom, self.running[k + ".bn.rm"], self.running[k + ".bn.rv"],
                              self.saved[k + ".bn.mean"], self.saved[k + ".bn.invstd"], self.fh[i], ls, hb.ACT_RELU)
                    P("bn_fwd", layer=k, layout="linear", x=self.fz[i], g=self.master(k + ".bn.g"),
                      b=self.master(k + ".bn.b"), y=self.fh[i], mean=self.saved[k + ".bn.mean"],
                      invstd=self.saved[k + ".bn.invstd"])
            else:
                hb.linear_fwd_ws(B, Nb, fx, fy, dt, h, self.w(k + ".w"), self.w(k + ".b"), self.fh[i], hb.ACT_RELU,
                                 workspace=self.ws)
                P("linear_fwd", layer=k, x=h, w=self.w(k + ".w"), b=self.w(k + ".b"), y=self.fh[i], act=1)
            if last:
                h = self.fz[i]
            else:
                h = self.fh[i]
                if i == self.nfc - 2 and s.dropout_p > 0:
                    hb.dropout(B * Nb * fy, dt, h, self.drop_mask, s.dropout_p, self.fdrop)
                    P("dropout", x=h, mask=self.drop_mask, y=self.fdrop)
                    h = self.fdrop
            fx = fy
        logits = h
        K = s.fc[-1]
        d = self.fd[0][:B * Nb * K]
        hb.softmax_xent(B, Nb, K, dt, logits, self.labels, self.loss, d)
        P("softmax_xent", logits=logits, labels=self.labels, loss=self.loss, d=d.view(B, Nb, K))

        # backward: head
        cur = 0
        for i in reversed(range(self.nfc)):
            fx, fy = s.fc[i], s.fc[i + 1]
            k = f"fc{i}"
            last = i == self.nfc - 1
            if not last:
                n = B * Nb * fy
                if i == self.nfc - 2 and s.dropout_p > 0:
                    nd = self.fd[cur ^ 1][:n]
                    hb.dropout(n, dt, d, self.drop_mask, s.dropout_p, nd)
                    P("dropout", x=d.view(B, Nb, fy), mask=self.drop_mask, y=nd.view(B, Nb, fy))
                    d, cur = nd, cur ^ 1
                nd = self.fd[cur ^ 1][:n]
                if s.fc_bn:
                    ls = (Nb * fy, fy, 1, 1)
                    hb.bn_bwd(B, Nb, fy, 1, dt, self.fz[i], ls, d, ls, self.master(k + ".bn.g"),
                              self.master(k + ".bn.b"), self.saved[k + ".bn.mean"], self.saved[k + ".bn.invstd"],
                              nd, ls, self.g(k + ".bn.g"), self.g(k + ".bn.b"), hb.ACT_RELU, 0.0, self.g(k + ".b"))
                    P("bn_bwd", layer=k, layout="linear", x=self.fz[i], dy=d.view(B, Nb, fy),
                      g=self.master(k + ".bn.g"), b=self.master(k + ".bn.b"), mean=self.saved[k + ".bn.mean"],
                      invstd=self.saved[k + ".bn.invstd"], dx=nd.view(B, Nb, fy), dg=self.g(k + ".bn.g"),
                      db=self.g(k + ".bn.b"))
                else:
                    hb.act_bwd(n, dt, self.fh[i], d, nd, hb.ACT_RELU, 0.0, 1)
                    P("relu_bwd_from_output", y=self.fh[i], dy=d.view(B, Nb, fy), dx=nd.view(B, Nb, fy))
                d, cur = nd, cur ^ 1
            if i == 0:
                hin = self.pooled
            elif i == self.nfc - 1 and s.dropout_p > 0:
                hin = self.fdrop
            else:
                hin = self.fh[i - 1]
            nd = self.fd[cur ^ 1][:B * Nb * fx]
            # a bias that feeds a BatchNorm gets its gradient from that BatchNorm's backward (dx_sum)
            own_db = self.g(k + ".b") if (last or not s.fc_bn) else None
            hb.linear_bwd(B, Nb, fx, fy, dt, hin, self.w(k + ".w"), d, nd, self.g(k + ".w"), own_db, self.ws)
            P("linear_bwd", layer=k, x=hin, w=self.w(k + ".w"), dy=d.view(B, Nb, fy), dx=nd.view(B, Nb, fx),
              dw=self.g(k + ".w"), db=self.g(k + ".b"))
            d, cur = nd, cur ^ 1

        # backward: pool and per-point MLP
        Cp = s.conv[-1]
        dpool = d
        da = None
        cur = 0
        for i in reversed(range(self.nconv)):
            ci, co = s.conv[i], s.conv[i + 1]
            k = f"conv{i}"
            cs = _cs(B, co, L)
            if i == self.nconv - 1 and self.fused_tail:
                xin, dxin = self.a[i - 1], self.dbuf[cur][:Nb * B * ci * L]
                tail = (self.zhit, self.tail_moments, dpool, self.pool_idx, (Nb * co, co, 1), self.master(k + ".bn.g"),
                        self.master(k + ".bn.b"), self.saved[k + ".bn.mean"], self.saved[k + ".bn.invstd"], dxin,
                        _cs(B, ci, L), self.g(k + ".w"), self.g(k + ".b"), self.g(k + ".bn.g"), self.g(k + ".bn.b"),
                        hb.ACT_RELU, 0.0, self.ws)
                if self.tail_prenorm:
                    xin = self.tail_x
                hb.conv1x1_bn_maxpool_bwd(B, Nb, ci, co, L, dt, xin, _cs(B, ci, L), self.w(k + ".w"), self.w(k + ".b"),
                                          None, None, *tail)
                P("conv1x1_bn_maxpool_bwd", layer=k, x=xin, w=self.w(k + ".w"), b=self.w(k + ".b"),
                  dv=dpool.view(B, Nb, co), idx=self.pool_idx, g=self.master(k + ".bn.g"),
                  bt=self.master(k + ".bn.b"), mean=self.saved[k + ".bn.mean"], invstd=self.saved[k + ".bn.invstd"],
                  dx=dxin.view(Nb, B * ci, L), dw=self.g(k + ".w"), db=self.g(k + ".b"), dg=self.g(k + ".bn.g"),
                  dbt=self.g(k + ".bn.b"))
                da = dxin
                continue
            xin = self.points if i == 0 else self.a[i - 1]
            if i < self.nconv - 1 and (i in self.unfused or self.one_pass[i]):
                # BatchNorm backward + convolution backward in one call: dz stays on chip.  The data
                # gradient goes to the other buffer (dY is still being read while it is written).
                dxin = None if i == 0 else self.dbuf[cur ^ 1][:Nb * B * ci * L]
                if i in self.unfused:
                    self._layer_bwd_unfused(i, xin, ci, co, da, dxin)
                else:
                    bnp = (self.master(k + ".bn.g"), self.master(k + ".bn.b"), self.saved[k + ".bn.mean"],
                           self.saved[k + ".bn.invstd"])
                    out = (dxin, None if i == 0 else _cs(B, ci, L), self.g(k + ".w"), self.g(k + ".b"), self.g(k + ".bn.g"),
                           self.g(k + ".bn.b"), hb.ACT_RELU, 0.0, self.ws, None, self.bn_sums[i])
                    if self.prenorm[i]:
                        kp = f"conv{i - 1}"
                        hb.conv1x1_bn_prenorm_bwd(B, Nb, ci, co, L, dt, self.z[i - 1], _cs(B, ci, L), self.master(kp + ".bn.g"),
                                                  self.master(kp + ".bn.b"), self.saved[kp + ".bn.mean"],
                                                  self.saved[kp + ".bn.invstd"], hb.ACT_RELU, 0.0, self.w(k + ".w"),
                                                  self.z[i], cs, da, cs, *bnp, *out, self.bn_sums[i - 1])
                        if probe is not None:
                            xin = self._act(i - 1)
                    else:
                        hb.conv1x1_bn_bwd(B, Nb, ci, co, L, dt, xin, _cs(B, ci, L), self.w(k + ".w"), self.z[i], cs, da, cs,
                                          *bnp, *out)
                    P("conv1x1_bn_bwd", layer=k, x=xin, w=self.w(k + ".w"), z=self.z[i], dy=da.view(Nb, B * co, L),
                      g=self.master(k + ".bn.g"), bt=self.master(k + ".bn.b"), mean=self.saved[k + ".bn.mean"],
                      invstd=self.saved[k + ".bn.invstd"], dx=None if i == 0 else dxin.view(Nb, B * ci, L),
                      dw=self.g(k + ".w"), db=self.g(k + ".b"), dg=self.g(k + ".bn.g"), dbt=self.g(k + ".bn.b"))
                da, cur = dxin, cur ^ 1
                continue
            dz = self.dbuf[cur ^ 1][:Nb * B * co * L]
            if i == self.nconv - 1:     # BatchNorm backward through the max over points
                hb.bn_bwd_maxpool(B, Nb, co, L, dt, self.z[i], cs, dpool, self.pool_idx, (Nb * co, co, 1),
                                  self.master(k + ".bn.g"), self.master(k + ".bn.b"), self.saved[k + ".bn.mean"],
                                  self.saved[k + ".bn.invstd"], dz, cs, self.g(k + ".bn.g"), self.g(k + ".bn.b"),
                                  hb.ACT_RELU, 0.0, self.g(k + ".b"))
                P("bn_bwd_maxpool", layer=k, x=self.z[i], dv=dpool.view(B, Nb, co), idx=self.pool_idx,
                  g=self.master(k + ".bn.g"), b=self.master(k + ".bn.b"), mean=self.saved[k + ".bn.mean"],
                  invstd=self.saved[k + ".bn.invstd"], dx=dz.view(Nb, B * co, L), dg=self.g(k + ".bn.g"),
                  db=self.g(k + ".bn.b"))
            else:
                hb.bn_bwd(B, Nb, co, L, dt, self.z[i], cs, da, cs, self.master(k + ".bn.g"), self.master(k + ".bn.b"),
                          self.saved[k + ".bn.mean"], self.saved[k + ".bn.invstd"], dz, cs, self.g(k + ".bn.g"),
                          self.g(k + ".bn.b"), hb.ACT_RELU, 0.0, self.g(k + ".b"))
                P("bn_bwd", layer=k, layout="conv", x=self.z[i], dy=da.view(Nb, B * co, L),
                  g=self.master(k + ".bn.g"), b=self.master(k + ".bn.b"), mean=self.saved[k + ".bn.mean"],
                  invstd=self.saved[k + ".bn.invstd"], dx=dz.view(Nb, B * co, L), dg=self.g(k + ".bn.g"),
                  db=self.g(k + ".bn.b"))
            dxin = None if i == 0 else self.dbuf[cur][:Nb * B * ci * L]
            # data gradient and weight gradient as two calls: one GEMM launch each (plus the weight
            # gradient's split-K reduction), so a caller can time them separately
            if i > 0:
                hb.conv1x1_bwd(B, Nb, ci, co, L, dt, None, None, self.w(k + ".w"), dz, cs,
                               dxin, _cs(B, ci, L), None, None, self.ws)
            hb.conv1x1_bwd(B, Nb, ci, co, L, dt, xin, _cs(B, ci, L), None, dz, cs,
                           None, None, self.g(k + ".w"), None, self.ws)
            P("conv1x1_bwd", layer=k, x=xin, w=self.w(k + ".w"), dy=dz.view(Nb, B * co, L),
              dx=None if i == 0 else dxin.view(Nb, B * ci, L), dw=self.g(k + ".w"), db=self.g(k + ".b"))
            da = dxin
        return self.loss




def _unfused_methods():
    def _off(t, n):
        return t.view(-1)[n:]

    def _layer_fwd_unfused(self, i, x, ci, co):
        B, Nb, L, dt, k = self.B, self.Nb, self.L, self.dt, f"conv{i}"
        xs, cs = _cs(B, ci, L), _cs(B, co, L)
        for b in range(B):
            # the same operator as the fused array's (convolution + BatchNorm + ReLU), one model at a time
            hb.conv1x1_bn_fwd(1, Nb, ci, co, L, dt, _off(x, b * ci * L), xs, _off(self.w(k + ".w"), b * co * ci),
                              _off(self.w(k + ".b"), b * co), _off(self.master(k + ".bn.g"), b * co),
                              _off(self.master(k + ".bn.b"), b * co), self.BN_EPS, self.BN_MOMENTUM,
                              _off(self.running[k + ".bn.rm"], b * co), _off(self.running[k + ".bn.rv"], b * co),
                              _off(self.saved[k + ".bn.mean"], b * co), _off(self.saved[k + ".bn.invstd"], b * co),
                              _off(self.z[i], b * co * L), cs, _off(self.a[i], b * co * L), cs, hb.ACT_RELU, 0.0, self.ws)

    def _layer_bwd_unfused(self, i, xin, ci, co, da, dxin):
        B, Nb, L, dt, k = self.B, self.Nb, self.L, self.dt, f"conv{i}"
        xs, cs = _cs(B, ci, L), _cs(B, co, L)
        for b in range(B):      # the same operator as the fused array's, one model at a time
            hb.conv1x1_bn_bwd(1, Nb, ci, co, L, dt, _off(xin, b * ci * L), xs, _off(self.w(k + ".w"), b * co * ci),
                              _off(self.z[i], b * co * L), cs, _off(da, b * co * L), cs,
                              _off(self.master(k + ".bn.g"), b * co), _off(self.master(k + ".bn.b"), b * co),
                              _off(self.saved[k + ".bn.mean"], b * co), _off(self.saved[k + ".bn.invstd"], b * co),
                              None if dxin is None else _off(dxin, b * ci * L), None if dxin is None else xs,
                              _off(self.g(k + ".w"), b * co * ci), _off(self.g(k + ".b"), b * co),
                              _off(self.g(k + ".bn.g"), b * co), _off(self.g(k + ".bn.b"), b * co), hb.ACT_RELU, 0.0, self.ws)

    FusedPointNetCls._layer_fwd_unfused = _layer_fwd_unfused
    FusedPointNetCls._layer_bwd_unfused = _layer_bwd_unfused


_unfused_methods()


class FusedMlp(ParamArena):
    """Residual MLP-block array: x <- LayerNorm(x + W2 GELU(W1 x + b1) + b2), `blocks` times, MSE
    loss per model, Adam with per-model lr and weight decay.  Activations are ``[B, R, F]`` (the
    fusion rules table's baddbmm layout); every Linear is one batched GEMM over the B weight sets."""

    LN_EPS = 1e-5

    def __init__(self, spec, inp: dict, device: str = "cuda"):
        import hfta_inputs as hi
        self.spec = spec
        self.B, self.R, self.E, self.H = spec.B, spec.R, spec.E, spec.H
        self.dtype = spec.dtype
        self.dt = _DT[spec.dtype]
        self.tdt = _TDT[spec.dtype]
        self.dev = torch.device(device)
        B, R, E, H = self.B, self.R, self.E, self.H
        self._init_arena(hi.mlp_param_shapes(spec), B, inp, spec.dtype, self.dev)
        f32 = dict(dtype=torch.float32, device=self.dev)
        act = dict(dtype=self.tdt, device=self.dev)
        nb = spec.blocks
        self.x = [torch.from_numpy(inp["tokens"]).to(self.tdt).to(self.dev)] + \
                 [torch.empty(B, R, E, **act) for _ in range(nb)]
        self.target = torch.from_numpy(inp["targets"]).to(self.tdt).to(self.dev)
        self.u = [torch.empty(B, R, H, **act) for _ in range(nb)]
        self.h = [torch.empty(B, R, H, **act) for _ in range(nb)]
        self.s = [torch.empty(B, R, E, **act) for _ in range(nb)]
        self.y = torch.empty(B, R, E, **act)
        self.ln_mean = [torch.empty(B * R, **f32) for _ in range(nb)]
        self.ln_invstd = [torch.empty(B * R, **f32) for _ in range(nb)]
        self.dE = [torch.empty(B, R, E, **act) for _ in range(3)]
        self.dH = [torch.empty(B, R, H, **act) for _ in range(2)]
        self.loss = torch.empty(B, **f32)
        ws = max(4, hb.layernorm_bwd_workspace_bytes(B, R, E), hb.layernorm_bwd_sums_workspace_bytes(B, R, E),
                 hb.linear_bwd_workspace_bytes(B, R, E, H, self.dt),
                 hb.linear_bwd_workspace_bytes(B, R, H, E, self.dt))
        self.ws = torch.empty(ws, dtype=torch.uint8, device=self.dev)

    def forward_backward(self, probe=None):
        """One forward + backward pass; ``probe(op, **tensors)`` as in FusedPointNetCls."""
        B, R, E, H, dt = self.B, self.R, self.E, self.H, self.dt
        P = probe if probe is not None else (lambda op, **kw: None)
        nb = self.spec.blocks
        for i in range(nb):
            k = f"blk{i}"
            x = self.x[i]
            hb.linear_fwd(B, R, E, H, dt, x, self.w(k + ".w1"), self.w(k + ".b1"), self.u[i])
            P("linear_fwd", layer=k + ".1", x=x, w=self.w(k + ".w1"), b=self.w(k + ".b1"), y=self.u[i], act=0)
            hb.act_fwd(B * R * H, dt, self.u[i], self.h[i], hb.ACT_GELU)
            P("act_fwd", layer=k, x=self.u[i], y=self.h[i], act=hb.ACT_GELU)
            hb.linear_fwd(B, R, H, E, dt, self.h[i], self.w(k + ".w2"), self.w(k + ".b2"), self.y)
            P("linear_fwd", layer=k + ".2", x=self.h[i], w=self.w(k + ".w2"), b=self.w(k + ".b2"), y=self.y, act=0)
            hb.add(B * R * E, dt, x, self.y, self.s[i])
            P("add", a=x, b=self.y, y=self.s[i])
            hb.layernorm_fwd(B, R, E, dt, self.s[i], self.master(k + ".ln.w"), self.master(k + ".ln.b"), self.LN_EPS,
                             self.ln_mean[i], self.ln_invstd[i], self.x[i + 1])
            P("layernorm_fwd", layer=k, x=self.s[i], w=self.master(k + ".ln.w"), b=self.master(k + ".ln.b"),
              y=self.x[i + 1], mean=self.ln_mean[i], invstd=self.ln_invstd[i])
        d = self.dE[0]
        hb.mse(B, R * E, dt, self.x[nb], self.target, self.loss, d)
        P("mse", pred=self.x[nb], target=self.target, loss=self.loss, d=d)
        # A block's incoming gradient is the pair (ga, gb) whose sum it is: the LayerNorm backward adds
        # them on load (no stored sum) and also emits the column sums of its result, the second
        # Linear's bias gradient.  (Rows of E that are not whole 16-byte pieces: the separate calls.)
        epv = 8 if dt == hb.BF16 else 4
        fused_ln = E % epv == 0 and E // epv <= 128
        ga, gb, free = self.dE[0], None, [self.dE[1], self.dE[2]]
        for i in reversed(range(nb)):
            k = f"blk{i}"
            ds = free.pop()
            if fused_ln:
                hb.layernorm_bwd_sums(B, R, E, dt, self.s[i], ga, gb, self.master(k + ".ln.w"), self.ln_mean[i],
                                      self.ln_invstd[i], ds, self.g(k + ".ln.w"), self.g(k + ".ln.b"), self.g(k + ".b2"),
                                      self.ws)
            else:
                if gb is not None:
                    hb.add(B * R * E, dt, ga, gb, ga)
                hb.layernorm_bwd(B, R, E, dt, self.s[i], ga, self.master(k + ".ln.w"), self.ln_mean[i], self.ln_invstd[i],
                                 ds, self.g(k + ".ln.w"), self.g(k + ".ln.b"), self.ws)
                hb.linear_bwd(B, R, H, E, dt, None, None, ds, None, None, self.g(k + ".b2"), None)
            P("layernorm_bwd", layer=k, x=self.s[i], dy=ga, dy2=gb if fused_ln else None, w=self.master(k + ".ln.w"),
              mean=self.ln_mean[i], invstd=self.ln_invstd[i], dx=ds, dw=self.g(k + ".ln.w"), db=self.g(k + ".ln.b"))
            # data gradient and weight gradient as separate calls (one kernel each), so a caller can
            # time them separately
            hb.linear_bwd(B, R, H, E, dt, None, self.w(k + ".w2"), ds, self.dH[0], None, None, None)
            hb.linear_bwd(B, R, H, E, dt, self.h[i], None, ds, None, self.g(k + ".w2"), None, self.ws)
            P("linear_bwd", layer=k + ".2", x=self.h[i], w=self.w(k + ".w2"), dy=ds, dx=self.dH[0],
              dw=self.g(k + ".w2"), db=self.g(k + ".b2"))
            # GELU backward and the first Linear's bias gradient (column sums of its result) in one pass
            # (whole 16-byte pieces along H; otherwise the two separate calls)
            if H % epv == 0:
                hb.act_bwd_colsum(B, R, H, dt, self.u[i], self.dH[0], self.dH[1], self.g(k + ".b1"), hb.ACT_GELU)
            else:
                hb.act_bwd(B * R * H, dt, self.u[i], self.dH[0], self.dH[1], hb.ACT_GELU)
                hb.linear_bwd(B, R, E, H, dt, None, None, self.dH[1], None, None, self.g(k + ".b1"), None)
            P("act_bwd", layer=k, x=self.u[i], dy=self.dH[0], dx=self.dH[1], act=hb.ACT_GELU)
            # nothing consumes the gradient of the array's input: the first block computes no data
            # gradient of its first Linear
            dxl = ga                                   # this block's incoming gradient is dead: reuse it
            if i > 0:
                hb.linear_bwd(B, R, E, H, dt, None, self.w(k + ".w1"), self.dH[1], dxl, None, None, None)
            hb.linear_bwd(B, R, E, H, dt, self.x[i], None, self.dH[1], None, self.g(k + ".w1"), None, self.ws)
            P("linear_bwd", layer=k + ".1", x=self.x[i], w=self.w(k + ".w1"), dy=self.dH[1], dx=dxl if i > 0 else None,
              dw=self.g(k + ".w1"), db=self.g(k + ".b1"))
            if gb is not None:
                free.append(gb)
            ga, gb = ds, dxl                           # the next block down receives ds + dxl
        return self.loss


class _Arena(ParamArena):
    """A stand-alone parameter arena (one optimiser's worth of parameters)."""

    def __init__(self, shapes, B, params, hp_inp, dtype, dev):
        self.B = B
        inp = dict(hp_inp)
        inp["params"] = params
        self._init_arena(shapes, B, inp, dtype, dev)
        self.grad2 = torch.zeros_like(self.grad)      # second pass of a step that sums two passes

    def g2(self, name):
        return self._seg(self.grad2, name)


class FusedDcgan:
    """B generator/discriminator pairs trained as one job: every Conv2d / ConvTranspose2d is one
    grouped implicit GEMM with groups = B, BatchNorm keeps per-model statistics, one Adam launch
    per network updates all B models (per-model lr).  Activations are ``[Nb, B*C, H, W]``."""

    BN_EPS = 1e-5
    BN_MOMENTUM = 0.1
    SLOPE = 0.2

    def __init__(self, spec, inp: dict, device: str = "cuda"):
        import hfta_inputs as hi
        self.spec = spec
        self.probe = None          # tests: called after every library call with the tensors it read and wrote
        self.B, self.Nb = spec.B, spec.Nb
        self.dt, self.tdt = _DT[spec.dtype], _TDT[spec.dtype]
        self.dev = torch.device(device)
        B, Nb = self.B, self.Nb
        gsh, dsh = hi.dcgan_param_shapes(spec)
        self.G = _Arena(gsh, B, inp["gparams"], inp, spec.dtype, self.dev)
        self.D = _Arena(dsh, B, inp["dparams"], inp, spec.dtype, self.dev)
        f32 = dict(dtype=torch.float32, device=self.dev)
        act = dict(dtype=self.tdt, device=self.dev)
        self.z = torch.from_numpy(inp["z"]).to(self.tdt).to(self.dev)
        self.real = torch.from_numpy(inp["real"]).to(self.tdt).to(self.dev)
        self.running, self.saved = {}, {}
        for arena in (self.G, self.D):
            for name, shp in arena.shapes:
                if name.endswith(".bn.g"):
                    k = name[:-2]
                    self.running[k + ".rm"] = torch.zeros(B * shp[0], **f32)
                    self.running[k + ".rv"] = torch.ones(B * shp[0], **f32)
                    self.saved[k + ".mean"] = torch.empty(B * shp[0], **f32)
                    self.saved[k + ".invstd"] = torch.empty(B * shp[0], **f32)
        # generator activations: pre-BatchNorm and activated, per layer
        self.g_pre, self.g_act = [], []
        for (ci, co, hin, s, p) in spec.g_layers:
            ho = (hin - 1) * s - 2 * p + 4
            self.g_pre.append(torch.empty(Nb, B * co, ho, ho, **act))
            self.g_act.append(torch.empty(Nb, B * co, ho, ho, **act))
        self.g_act[-1] = self.g_pre[-1]                 # tanh runs in place on the last layer
        self.fake = self.g_pre[-1]
        self.d_pre, self.d_act = [], []
        for (ci, co, hin, s, p) in spec.d_layers:
            ho = (hin + 2 * p - 4) // s + 1
            self.d_pre.append(torch.empty(Nb, B * co, ho, ho, **act))
            self.d_act.append(torch.empty(Nb, B * co, ho, ho, **act))
        self.d_act[0] = self.d_pre[0]                   # LeakyReLU in the first conv's epilogue
        self.logits = self.d_pre[-1]
        big = max(max(t.numel() for t in self.g_pre), max(t.numel() for t in self.d_pre), self.real.numel())
        self.dbuf = [torch.empty(big, **act) for _ in range(2)]
        self.ones = torch.ones(Nb, B, **act)
        self.zeros = torch.zeros(Nb, B, **act)
        self.dlogits = torch.empty(Nb, B, **act)
        self.loss_d_real = torch.empty(B, **f32)
        self.loss_d_fake = torch.empty(B, **f32)
        self.loss_g = torch.empty(B, **f32)
        ws = 4
        for (ci, co, hin, s, p) in spec.d_layers:
            geo = (B, Nb, ci, co, hin, hin, 4, 4, s, p, self.dt)
            ws = max(ws, hb.conv2d_grouped_bwd_workspace_bytes(*geo), hb.conv2d_grouped_fwd_workspace_bytes(*geo))
        for (ci, co, hin, s, p) in spec.g_layers:
            ho = (hin - 1) * s - 2 * p + 4
            geo = (B, Nb, co, ci, ho, ho, 4, 4, s, p, self.dt)
            ws = max(ws, hb.conv2d_grouped_bwd_workspace_bytes(*geo), hb.conv2d_grouped_fwd_workspace_bytes(*geo))
        # large enough for the column-buffer lowering of every layer (its sample-folded GEMMs)
        self.ws = torch.empty(ws, dtype=torch.uint8, device=self.dev)

    def _P(self, op, **kw):
        if self.probe is not None:
            self.probe(op, **kw)

    # ------------------------------------------------------------------ generator
    def g_forward(self):
        B, Nb, dt, s = self.B, self.Nb, self.dt, self.spec
        x = self.z
        n = len(s.g_layers)
        for i, (ci, co, hin, st, p) in enumerate(s.g_layers):
            k = f"g{i}"
            ho = (hin - 1) * st - 2 * p + 4
            # ConvTranspose2d forward = the data-gradient form of the grouped convolution
            hb.conv2d_grouped_bwd(B, Nb, co, ci, ho, ho, 4, 4, st, p, dt, None, self.G.w(k + ".w"), x,
                                  self.g_pre[i], None, None, self.ws)
            self._P("convT2d_fwd", layer=k, x=x, w=self.G.w(k + ".w"), y=self.g_pre[i], geo=(ci, co, st, p))
            if i < n - 1:
                cs = _cs(B, co, ho * ho)
                hb.bn_fwd(B, Nb, co, ho * ho, dt, self.g_pre[i], cs, self.G.master(k + ".bn.g"),
                          self.G.master(k + ".bn.b"), self.BN_EPS, self.BN_MOMENTUM, self.running[k + ".bn.rm"],
                          self.running[k + ".bn.rv"], self.saved[k + ".bn.mean"], self.saved[k + ".bn.invstd"],
                          self.g_act[i], cs, hb.ACT_RELU)
                self._P("bn_fwd", layer=k, x=self.g_pre[i], g=self.G.master(k + ".bn.g"), b=self.G.master(k + ".bn.b"),
                        y=self.g_act[i], mean=self.saved[k + ".bn.mean"], invstd=self.saved[k + ".bn.invstd"],
                        act=hb.ACT_RELU)
            else:
                pre = self.g_pre[i].clone() if self.probe is not None else None
                hb.bias_act_nchw(Nb, B * co, ho * ho, dt, self.g_pre[i], None, hb.ACT_TANH)
                self._P("act_fwd", layer=k, x=pre, y=self.g_pre[i], act=hb.ACT_TANH)
            x = self.g_act[i]
        return self.fake

    def g_backward(self, dfake):
        B, Nb, dt, s = self.B, self.Nb, self.dt, self.spec
        n = len(s.g_layers)
        d = dfake
        for i in reversed(range(n)):
            ci, co, hin, st, p = s.g_layers[i]
            k = f"g{i}"
            ho = (hin - 1) * st - 2 * p + 4
            cnt = Nb * B * co * ho * ho
            dpre = self._other(d)[:cnt]
            if i == n - 1:
                hb.act_bwd(cnt, dt, self.fake, d, dpre, hb.ACT_TANH, 0.0, 1)
                self._P("act_bwd_from_output", layer=k, y=self.fake, dy=d[:cnt], dx=dpre, act=hb.ACT_TANH)
            else:
                cs = _cs(B, co, ho * ho)
                hb.bn_bwd(B, Nb, co, ho * ho, dt, self.g_pre[i], cs, d, cs, self.G.master(k + ".bn.g"),
                          self.G.master(k + ".bn.b"), self.saved[k + ".bn.mean"], self.saved[k + ".bn.invstd"],
                          dpre, cs, self.G.g(k + ".bn.g"), self.G.g(k + ".bn.b"), hb.ACT_RELU, 0.0)
                self._P("bn_bwd", layer=k, x=self.g_pre[i], dy=d[:cnt], g=self.G.master(k + ".bn.g"),
                        b=self.G.master(k + ".bn.b"), mean=self.saved[k + ".bn.mean"], invstd=self.saved[k + ".bn.invstd"],
                        dx=dpre, dg=self.G.g(k + ".bn.g"), db=self.G.g(k + ".bn.b"), act=hb.ACT_RELU)
            xin = self.z if i == 0 else self.g_act[i - 1]
            # ConvTranspose2d weight gradient = the convolution's with input and output gradient exchanged
            hb.conv2d_grouped_bwd(B, Nb, co, ci, ho, ho, 4, 4, st, p, dt, dpre, None, xin, None,
                                  self.G.g(k + ".w"), None, self.ws)
            self._P("convT2d_dw", layer=k, x=xin, w=self.G.w(k + ".w"), dy=dpre, dw=self.G.g(k + ".w"), geo=(ci, co, st, p),
                    hw=(hin, ho))
            if i > 0:
                dx = self._other(dpre)[:Nb * B * ci * hin * hin]      # the incoming gradient's buffer: it is dead
                # ConvTranspose2d data gradient = the convolution's forward
                hb.conv2d_grouped_fwd(B, Nb, co, ci, ho, ho, 4, 4, st, p, dt, dpre, self.G.w(k + ".w"), None, dx,
                                      workspace=self.ws)
                self._P("convT2d_dx", layer=k, x=xin, w=self.G.w(k + ".w"), dy=dpre, dx=dx, geo=(ci, co, st, p), hw=(hin, ho))
                d = dx

    def _other(self, t):
        """The ping-pong gradient buffer that `t` does not live in."""
        return self.dbuf[1] if t.data_ptr() == self.dbuf[0].data_ptr() else self.dbuf[0]

    # ------------------------------------------------------------------ discriminator
    def d_forward(self, x):
        B, Nb, dt, s = self.B, self.Nb, self.dt, self.spec
        n = len(s.d_layers)
        self._d_in = x
        for i, (ci, co, hin, st, p) in enumerate(s.d_layers):
            k = f"d{i}"
            ho = (hin + 2 * p - 4) // st + 1
            if i == 0:
                hb.conv2d_grouped_fwd(B, Nb, ci, co, hin, hin, 4, 4, st, p, dt, x, self.D.w(k + ".w"), None,
                                      self.d_pre[i], hb.ACT_LEAKY, self.SLOPE, workspace=self.ws)
                self._P("conv2d_fwd", layer=k, x=x, w=self.D.w(k + ".w"), y=self.d_pre[i], geo=(ci, co, st, p), act=hb.ACT_LEAKY)
            else:
                hb.conv2d_grouped_fwd(B, Nb, ci, co, hin, hin, 4, 4, st, p, dt, x, self.D.w(k + ".w"), None,
                                      self.d_pre[i], workspace=self.ws)
                self._P("conv2d_fwd", layer=k, x=x, w=self.D.w(k + ".w"), y=self.d_pre[i], geo=(ci, co, st, p), act=hb.ACT_NONE)
                if i < n - 1:
                    cs = _cs(B, co, ho * ho)
                    hb.bn_fwd(B, Nb, co, ho * ho, dt, self.d_pre[i], cs, self.D.master(k + ".bn.g"),
                              self.D.master(k + ".bn.b"), self.BN_EPS, self.BN_MOMENTUM, self.running[k + ".bn.rm"],
                              self.running[k + ".bn.rv"], self.saved[k + ".bn.mean"], self.saved[k + ".bn.invstd"],
                              self.d_act[i], cs, hb.ACT_LEAKY, self.SLOPE)
                    self._P("bn_fwd", layer=k, x=self.d_pre[i], g=self.D.master(k + ".bn.g"), b=self.D.master(k + ".bn.b"),
                            y=self.d_act[i], mean=self.saved[k + ".bn.mean"], invstd=self.saved[k + ".bn.invstd"],
                            act=hb.ACT_LEAKY)
            x = self.d_act[i]
        return self.logits

    def d_backward(self, grad_of, want_dw=True, want_dx=False):
        """Backward from ``self.dlogits``; ``grad_of(name)`` names where a parameter gradient goes."""
        B, Nb, dt, s = self.B, self.Nb, self.dt, self.spec
        n = len(s.d_layers)
        d = self.dlogits
        for i in reversed(range(n)):
            ci, co, hin, st, p = s.d_layers[i]
            k = f"d{i}"
            ho = (hin + 2 * p - 4) // st + 1
            cnt = Nb * B * co * ho * ho
            if i == n - 1:
                dpre = d
            else:
                dpre = self._other(d)[:cnt]
                if i == 0:
                    hb.act_bwd(cnt, dt, self.d_act[0], d, dpre, hb.ACT_LEAKY, self.SLOPE, 1)
                    self._P("act_bwd_from_output", layer=k, y=self.d_act[0], dy=d[:cnt], dx=dpre, act=hb.ACT_LEAKY)
                else:
                    cs = _cs(B, co, ho * ho)
                    # without weight gradients the BatchNorm parameter gradients go to the spare buffer
                    tgt = grad_of if want_dw else self.D.g2
                    hb.bn_bwd(B, Nb, co, ho * ho, dt, self.d_pre[i], cs, d, cs, self.D.master(k + ".bn.g"),
                              self.D.master(k + ".bn.b"), self.saved[k + ".bn.mean"], self.saved[k + ".bn.invstd"],
                              dpre, cs, tgt(k + ".bn.g"), tgt(k + ".bn.b"), hb.ACT_LEAKY, self.SLOPE)
                    self._P("bn_bwd", layer=k, x=self.d_pre[i], dy=d[:cnt], g=self.D.master(k + ".bn.g"),
                            b=self.D.master(k + ".bn.b"), mean=self.saved[k + ".bn.mean"], invstd=self.saved[k + ".bn.invstd"],
                            dx=dpre, dg=tgt(k + ".bn.g"), db=tgt(k + ".bn.b"), act=hb.ACT_LEAKY)
            xin = self._d_in if i == 0 else self.d_act[i - 1]
            need_dx = i > 0 or want_dx
            if want_dw:
                hb.conv2d_grouped_bwd(B, Nb, ci, co, hin, hin, 4, 4, st, p, dt, xin, None, dpre, None,
                                      grad_of(k + ".w"), None, self.ws)
                self._P("conv2d_dw", layer=k, x=xin, w=self.D.w(k + ".w"), dy=dpre, dw=grad_of(k + ".w"), geo=(ci, co, st, p),
                        hw=(hin, ho))
            if need_dx:
                dx = self._other(dpre)[:Nb * B * ci * hin * hin]
                hb.conv2d_grouped_bwd(B, Nb, ci, co, hin, hin, 4, 4, st, p, dt, None, self.D.w(k + ".w"), dpre, dx,
                                      None, None, self.ws)
                self._P("conv2d_dx", layer=k, x=xin, w=self.D.w(k + ".w"), dy=dpre, dx=dx, geo=(ci, co, st, p), hw=(hin, ho))
                d = dx
        return d

    def _bce(self, targets, loss):
        hb.bce_logits_strided(self.B, self.Nb, self.dt, self.logits, targets, loss, self.dlogits, 1, self.B)
        self._P("bce", logits=self.logits, targets=targets, loss=loss, d=self.dlogits)

    # ------------------------------------------------------------------ one iteration
    def d_step(self):
        """Discriminator step on BCE(D(real), 1) + BCE(D(fake), 0); `fake` must be current."""
        self.d_forward(self.real)
        self._bce(self.ones, self.loss_d_real)
        self.d_backward(self.D.g)
        self.d_forward(self.fake)
        self._bce(self.zeros, self.loss_d_fake)
        self.d_backward(self.D.g2)
        g1 = self.D.grad.clone() if self.probe is not None else None
        hb.add(self.D.grad.numel(), hb.F32, self.D.grad, self.D.grad2, self.D.grad)
        self._P("grad_add", a=g1, b=self.D.grad2, y=self.D.grad)

    def g_step_backward(self):
        """Generator loss BCE(D(fake), 1) through the current discriminator, back to G's parameters."""
        self.d_forward(self.fake)
        self._bce(self.ones, self.loss_g)
        dfake = self.d_backward(None, want_dw=False, want_dx=True)
        self.g_backward(dfake)

    def train_step(self):
        self.g_forward()
        self.d_step()
        self.D.adam()
        self.g_step_backward()
        self.G.adam()
        return self.loss_g


class FusedPointNetSeg(ParamArena):
    """PointNet-segmentation-style array: per-point k=1 convolutions + BatchNorm + ReLU, max over the
    points of the last feature map, then a per-point head on the concatenation of every feature map,
    the tiled global feature and the tiled category one-hot; softmax cross-entropy per point; Adam.

    Nothing is copied to concatenate: every per-point layer writes its activation into its channel
    slice of one ``[Nb, B*c_point, L]`` buffer (strides), the head's first convolution reads that
    buffer as one 2880-channel input, and the tiled part enters as ``[global | one-hot] @ Wg + bias`` once
    per sample, added in that convolution's accumulators as a per-(sample, channel) bias.  Backward mirrors it: the head's data gradient lands in a
    buffer of the same shape, and each per-point layer adds its slice to the gradient from the
    next layer."""

    BN_EPS = 1e-5
    BN_MOMENTUM = 0.1

    def __init__(self, spec, inp: dict, device: str = "cuda"):
        self.spec = spec
        self.B, self.Nb, self.L = spec.B, spec.Nb, spec.L
        self.dtype, self.dt, self.tdt = spec.dtype, _DT[spec.dtype], _TDT[spec.dtype]
        self.dev = torch.device(device)
        B, Nb, L = self.B, self.Nb, self.L
        import hfta_inputs as hi
        # The layer list's first head weight [head[1], c_point + c_global] is stored as two arena
        # tensors: its per-point columns as a k=1 convolution weight ``head0.w`` [co, c_point], and its
        # tiled columns transposed, ``head0.wg`` [c_global, co], the weight of a Linear applied once per
        # sample (a convolution over channels that are constant along the points).
        self.param_shapes = hi.pointnet_seg_param_shapes(spec)
        shapes = []
        for name, shp in self.param_shapes:
            if name == "head0.w":
                shapes += [("head0.w", (shp[0], spec.c_point)), ("head0.wg", (spec.c_global, shp[0]))]
            else:
                shapes.append((name, shp))
        self._init_arena(shapes, B, {**inp, "params": [self._split_head0(p) for p in inp["params"]]}, spec.dtype, self.dev)
        f32 = dict(dtype=torch.float32, device=self.dev)
        act = dict(dtype=self.tdt, device=self.dev)
        self.running: Dict[str, torch.Tensor] = {}
        self.saved: Dict[str, torch.Tensor] = {}
        for name, shp in self.shapes:
            if name.endswith(".bn.g"):
                k = name[:-2]
                self.running[k + ".rm"] = torch.zeros(B * shp[0], **f32)
                self.running[k + ".rv"] = torch.ones(B * shp[0], **f32)
                self.saved[k + ".mean"] = torch.empty(B * shp[0], **f32)
                self.saved[k + ".invstd"] = torch.empty(B * shp[0], **f32)
        self.nconv, self.nh = len(spec.conv) - 1, len(spec.head) - 1
        self.Cp, self.Cg, self.C4 = spec.c_point, spec.c_global, spec.conv[-1]
        self.off = [0]
        for c in spec.conv[1:]:
            self.off.append(self.off[-1] + c)
        Cp, Cg = self.Cp, self.Cg
        self.cat = torch.empty(Nb, B * Cp, L, **act)
        self.dcat = torch.empty(Nb, B * Cp, L, **act)
        self.cat_strides = (Cp * L, B * Cp * L, L, 1)
        self.z = [torch.empty(Nb, B * c, L, **act) for c in spec.conv[1:]]
        self.gfeat = torch.zeros(B, Nb, Cg, **act)
        self.gfeat[:, :, self.C4:] = torch.from_numpy(inp["onehot"]).to(self.tdt).to(self.dev)
        self.pool_idx = torch.zeros(B, Nb, Cg, dtype=torch.int32, device=self.dev)
        self.gvs = (Nb * Cg, Cg, 1)
        H = spec.head
        self.hg = torch.empty(B, Nb, H[1], **act)
        self.dhg = torch.empty(B, Nb, H[1], **act)
        self.dgfeat = torch.empty(B, Nb, Cg, **act)
        self.zh = [torch.empty(Nb, B * c, L, **act) for c in H[1:]]
        self.ah = [torch.empty(Nb, B * c, L, **act) for c in H[1:-1]]
        cmax = max(max(spec.conv[1:]), max(H[1:]))
        self.dbuf = [torch.empty(Nb * B * cmax * L, **act) for _ in range(3)]
        self.loss = torch.empty(B, **f32)
        ws = max(4, hb.softmax_xent_points_workspace_bytes(B, Nb, L), hb.linear_bwd_workspace_bytes(B, Nb, Cg, H[1], self.dt),
                 hb.linear_fwd_workspace_bytes(B, Nb, Cg, H[1], self.dt))
        self.one_pass = [_bn_bwd_one_pass(B, Nb, spec.conv[i], spec.conv[i + 1], L, self.dt) for i in range(self.nconv)]
        for i in range(self.nconv):
            ws = max(ws, hb.conv1x1_bwd_workspace_bytes(B, Nb, spec.conv[i], spec.conv[i + 1], L, self.dt),
                     hb.conv1x1_bn_fwd_workspace_bytes(B, Nb, spec.conv[i], spec.conv[i + 1], L, self.dt))
            if self.one_pass[i]:
                ws = max(ws, hb.conv1x1_bn_bwd_workspace_bytes(B, Nb, spec.conv[i], spec.conv[i + 1], L, self.dt))
        for i in range(self.nh):
            ws = max(ws, hb.conv1x1_bwd_workspace_bytes(B, Nb, Cp if i == 0 else H[i], H[i + 1], L, self.dt),
                     hb.conv1x1_bn_fwd_workspace_bytes(B, Nb, Cp if i == 0 else H[i], H[i + 1], L, self.dt))
        self.ws = torch.empty(ws, dtype=torch.uint8, device=self.dev)
        self.points = torch.from_numpy(inp["points"]).to(self.tdt).to(self.dev)
        self.labels = torch.from_numpy(inp["labels"]).to(self.dev)

    def _split_head0(self, p: dict) -> dict:
        """Per-model parameters of the layer list -> the arena's tensors (a re-layout, no arithmetic)."""
        q = dict(p)
        w = np.asarray(p["head0.w"], np.float32)
        q["head0.w"] = np.ascontiguousarray(w[:, :self.spec.c_point])
        q["head0.wg"] = np.ascontiguousarray(w[:, self.spec.c_point:].T)
        return q

    def load_params(self, params) -> None:
        super().load_params([self._split_head0(p) for p in params])

    def param_host(self, buf: torch.Tensor, name: str, b: int) -> np.ndarray:
        """Parameter ``name`` of the layer list for model b (the first head weight re-assembled)."""
        if name == "head0.w":
            return np.concatenate([super().param_host(buf, "head0.w", b), super().param_host(buf, "head0.wg", b).T], axis=1)
        return super().param_host(buf, name, b)

    def _slice(self, buf, i):
        """Channel slice i of a concatenation buffer: (tensor whose data pointer is the slice's first
        element, for the ABI; the same slice as a [Nb, B, C, L] view, for tests)."""
        o, c = self.off[i], self.spec.conv[i + 1]
        return buf.view(-1)[o * self.L:], buf.view(self.Nb, self.B, self.Cp, self.L)[:, :, o:o + c, :]

    def forward_backward(self, probe=None):
        s, B, Nb, L, dt = self.spec, self.B, self.Nb, self.L, self.dt
        eps, mom = self.BN_EPS, self.BN_MOMENTUM
        P = probe if probe is not None else (lambda op, **kw: None)
        cst, Cp, Cg, C4, H = self.cat_strides, self.Cp, self.Cg, self.C4, s.head
        bn = lambda k: (self.master(k + ".bn.g"), self.master(k + ".bn.b"))
        st = lambda k: (self.saved[k + ".bn.mean"], self.saved[k + ".bn.invstd"])
        # ---- per-point MLP: each activation goes straight into its slice of the concatenation
        x, xs, xv, ci = self.points, _cs(B, 3, L), self.points, 3
        for i in range(self.nconv):
            co, k = s.conv[i + 1], f"conv{i}"
            a, av = self._slice(self.cat, i)
            # convolution + BatchNorm + ReLU in one call (z is read once, for the normalisation)
            hb.conv1x1_bn_fwd(B, Nb, ci, co, L, dt, x, xs, self.w(k + ".w"), self.w(k + ".b"), *bn(k), eps, mom,
                              self.running[k + ".bn.rm"], self.running[k + ".bn.rv"], *st(k), self.z[i], _cs(B, co, L),
                              a, cst, hb.ACT_RELU, 0.0, self.ws)
            P("conv1x1_fwd", layer=k, x=xv, w=self.w(k + ".w"), b=self.w(k + ".b"), y=self.z[i])
            P("bn_fwd", layer=k, x=self.z[i], g=bn(k)[0], b=bn(k)[1], y=av, mean=st(k)[0], invstd=st(k)[1])
            x, xs, xv, ci = a, cst, av, co
        hb.maxpool_points(B, Nb, C4, L, dt, x, cst, self.gfeat, self.pool_idx, self.gvs)
        P("maxpool_points", x=xv, v=self.gfeat[:, :, :C4], idx=self.pool_idx[:, :, :C4])
        # ---- head: first layer = per-point block over the concatenation + once-per-sample block
        # the tiled block's product (with the layer's bias) once per sample ...
        hb.linear_fwd_ws(B, Nb, Cg, H[1], dt, self.gfeat, self.w("head0.wg"), self.w("head0.b"), self.hg, workspace=self.ws)
        P("linear_fwd", layer="head0.wg", x=self.gfeat, w=self.w("head0.wg"), b=self.w("head0.b"), y=self.hg)
        h, hs, hv, ci = self.cat, cst, self.cat, Cp
        for i in range(self.nh):
            co, k = H[i + 1], f"head{i}"
            cs = _cs(B, co, L)
            if i == 0:      # ... enters the convolution over the per-point block as its per-sample bias: one store
                hb.conv1x1_fwd_sample_bias(B, Nb, ci, co, L, dt, h, hs, self.w(k + ".w"), self.hg, (Nb * co, co, 1),
                                           self.zh[i], cs)
                P("conv1x1_fwd_sample_bias", layer=k, x=hv, w=self.w(k + ".w"), s=self.hg, y=self.zh[i])
            elif i < self.nh - 1:
                hb.conv1x1_bn_fwd(B, Nb, ci, co, L, dt, h, hs, self.w(k + ".w"), self.w(k + ".b"), *bn(k), eps, mom,
                                  self.running[k + ".bn.rm"], self.running[k + ".bn.rv"], *st(k), self.zh[i], cs,
                                  self.ah[i], cs, hb.ACT_RELU, 0.0, self.ws)
                P("conv1x1_fwd", layer=k, x=hv, w=self.w(k + ".w"), b=self.w(k + ".b"), y=self.zh[i])
            else:
                hb.conv1x1_fwd(B, Nb, ci, co, L, dt, h, hs, self.w(k + ".w"), self.w(k + ".b"), self.zh[i], cs)
                P("conv1x1_fwd", layer=k, x=hv, w=self.w(k + ".w"), b=self.w(k + ".b"), y=self.zh[i])
            if i == self.nh - 1:
                break
            if i == 0:
                hb.bn_fwd(B, Nb, co, L, dt, self.zh[i], cs, *bn(k), eps, mom, self.running[k + ".bn.rm"],
                          self.running[k + ".bn.rv"], *st(k), self.ah[i], cs, hb.ACT_RELU)
            P("bn_fwd", layer=k, x=self.zh[i], g=bn(k)[0], b=bn(k)[1], y=self.ah[i], mean=st(k)[0], invstd=st(k)[1])
            h, hs, hv, ci = self.ah[i], cs, self.ah[i], co
        K = H[-1]
        logits = self.zh[-1]
        d = self.dbuf[0][:Nb * B * K * L]
        hb.softmax_xent_points(B, Nb, K, L, dt, logits, _cs(B, K, L), self.labels, self.loss, d, _cs(B, K, L), self.ws)
        P("softmax_xent_points", logits=logits, labels=self.labels, loss=self.loss, d=d.view(Nb, B * K, L))

        # ---- backward: head
        cur = 0
        for i in reversed(range(self.nh)):
            ci, co, k = (Cp if i == 0 else H[i]), H[i + 1], f"head{i}"
            cs = _cs(B, co, L)
            if i < self.nh - 1:
                dz = self.dbuf[cur ^ 1][:Nb * B * co * L]
                hb.bn_bwd(B, Nb, co, L, dt, self.zh[i], cs, d, cs, *bn(k), *st(k), dz, cs, self.g(k + ".bn.g"),
                          self.g(k + ".bn.b"), hb.ACT_RELU, 0.0, self.g(k + ".b"))
                P("bn_bwd", layer=k, x=self.zh[i], dy=d.view(Nb, B * co, L), g=bn(k)[0], b=bn(k)[1], mean=st(k)[0],
                  invstd=st(k)[1], dx=dz.view(Nb, B * co, L), dg=self.g(k + ".bn.g"), db=self.g(k + ".bn.b"))
                d, cur = dz, cur ^ 1
            hin, hs = (self.cat, cst) if i == 0 else (self.ah[i - 1], _cs(B, ci, L))
            dx, dxs = (self.dcat, cst) if i == 0 else (self.dbuf[cur ^ 1][:Nb * B * ci * L], _cs(B, ci, L))
            hb.conv1x1_bwd(B, Nb, ci, co, L, dt, None, None, self.w(k + ".w"), d, cs, dx, dxs, None, None, self.ws)
            own_db = self.g(k + ".b") if i == self.nh - 1 else None      # else from the BatchNorm backward
            hb.conv1x1_bwd(B, Nb, ci, co, L, dt, hin, hs, None, d, cs, None, None, self.g(k + ".w"), own_db, self.ws)
            P("conv1x1_bwd", layer=k, x=hin, w=self.w(k + ".w"), dy=d.view(Nb, B * co, L),
              dx=dx.view(Nb, B * ci, L), dw=self.g(k + ".w"), db=self.g(k + ".b"))
            if i == 0:
                hb.sum_points(B, Nb, co, L, dt, d, cs, self.dhg, (Nb * co, co, 1))
                P("sum_points", x=d.view(Nb, B * co, L), s=self.dhg)
                hb.linear_bwd(B, Nb, Cg, co, dt, self.gfeat, self.w("head0.wg"), self.dhg, self.dgfeat,
                              self.g("head0.wg"), None, self.ws)
                P("linear_bwd", layer="head0.wg", x=self.gfeat, w=self.w("head0.wg"), dy=self.dhg, dx=self.dgfeat,
                  dw=self.g("head0.wg"))
            else:
                d, cur = dx, cur ^ 1

        # ---- backward: per-point MLP; each layer adds its slice of the concatenation's gradient
        dnext = None
        for i in reversed(range(self.nconv)):
            ci, co, k = s.conv[i], s.conv[i + 1], f"conv{i}"
            cs = _cs(B, co, L)
            sl, slv = self._slice(self.dcat, i)
            if i == self.nconv - 1:
                before = slv.clone() if probe is not None else None
                hb.maxpool_points_bwd_add(B, Nb, co, L, dt, self.dgfeat, self.pool_idx, self.gvs, sl, cst)
                P("maxpool_points_bwd_add", dx0=before, dv=self.dgfeat[:, :, :C4], idx=self.pool_idx[:, :, :C4], dx=slv)
                da, das, dav = sl, cst, slv
            else:
                dsum = self.dbuf[2][:Nb * B * co * L]
                hb.add_strided(B, Nb, co, L, dt, dnext, cs, sl, cst, dsum, cs)
                P("add_strided", a=dnext.view(Nb, B * co, L), b=slv, y=dsum.view(Nb, B * co, L))
                da, das, dav = dsum, cs, dsum.view(Nb, B * co, L)
            if self.one_pass[i]:
                # BatchNorm backward + convolution backward in one call (dz stays on chip)
                if i > 0:
                    xin, xs, xinv = self._slice(self.cat, i - 1)[0], cst, self._slice(self.cat, i - 1)[1]
                    dnext = self.dbuf[1][:Nb * B * ci * L]
                else:
                    xin, xs, xinv, dnext = self.points, _cs(B, 3, L), self.points, None
                hb.conv1x1_bn_bwd(B, Nb, ci, co, L, dt, xin, xs, self.w(k + ".w"), self.z[i], cs, da, das, *bn(k), *st(k),
                                  dnext, None if i == 0 else _cs(B, ci, L), self.g(k + ".w"), self.g(k + ".b"),
                                  self.g(k + ".bn.g"), self.g(k + ".bn.b"), hb.ACT_RELU, 0.0, self.ws)
                P("conv1x1_bn_bwd", layer=k, x=xinv, w=self.w(k + ".w"), z=self.z[i], dy=dav, g=bn(k)[0], bt=bn(k)[1],
                  mean=st(k)[0], invstd=st(k)[1], dx=None if i == 0 else dnext.view(Nb, B * ci, L), dw=self.g(k + ".w"),
                  db=self.g(k + ".b"), dg=self.g(k + ".bn.g"), dbt=self.g(k + ".bn.b"))
                continue
            dz = self.dbuf[0][:Nb * B * co * L]
            hb.bn_bwd(B, Nb, co, L, dt, self.z[i], cs, da, das, *bn(k), *st(k), dz, cs, self.g(k + ".bn.g"),
                      self.g(k + ".bn.b"), hb.ACT_RELU, 0.0, self.g(k + ".b"))
            P("bn_bwd", layer=k, x=self.z[i], dy=dav, g=bn(k)[0], b=bn(k)[1], mean=st(k)[0], invstd=st(k)[1],
              dx=dz.view(Nb, B * co, L), dg=self.g(k + ".bn.g"), db=self.g(k + ".bn.b"))
            if i > 0:
                xin, xs = self._slice(self.cat, i - 1)[0], cst
                xinv = self._slice(self.cat, i - 1)[1]
                dnext = self.dbuf[1][:Nb * B * ci * L]
                hb.conv1x1_bwd(B, Nb, ci, co, L, dt, None, None, self.w(k + ".w"), dz, cs, dnext, _cs(B, ci, L),
                               None, None, self.ws)
            else:
                xin, xs, xinv, dnext = self.points, _cs(B, 3, L), self.points, None
            hb.conv1x1_bwd(B, Nb, ci, co, L, dt, xin, xs, None, dz, cs, None, None, self.g(k + ".w"), None, self.ws)
            P("conv1x1_bwd", layer=k, x=xinv, w=self.w(k + ".w"), dy=dz.view(Nb, B * co, L),
              dx=None if i == 0 else dnext.view(Nb, B * ci, L), dw=self.g(k + ".w"), db=self.g(k + ".b"))
        return self.loss


class FusedTransformerLM(ParamArena):
    """Transformer-encoder language-model array: fused Embedding (scaled, plus fixed positions), post-norm
    encoder layers with causal multi-head attention (projections are fused Linears, the per-head
    products run as batched GEMMs on column blocks of the packed projection), Linear decoder, softmax
    cross-entropy per token, Adam.  Activations are ``[B, R, F]`` with R = N*S tokens per model."""

    LN_EPS = 1e-5

    def __init__(self, spec, inp: dict, device: str = "cuda"):
        import hfta_inputs as hi
        from math import sqrt
        self.spec = spec
        self.B, self.N, self.S, self.E, self.F, self.V, self.Hh = spec.B, spec.N, spec.S, spec.E, spec.F, spec.V, spec.heads
        self.R = spec.N * spec.S
        self.dtype, self.dt, self.tdt = spec.dtype, _DT[spec.dtype], _TDT[spec.dtype]
        self.dev = torch.device(device)
        B, R, E, F, V, N, S, Hh = self.B, self.R, self.E, self.F, self.V, self.N, self.S, self.Hh
        self._init_arena(hi.transformer_param_shapes(spec), B, inp, spec.dtype, self.dev)
        f32 = dict(dtype=torch.float32, device=self.dev)
        act = dict(dtype=self.tdt, device=self.dev)
        nl = spec.layers
        self.scale = sqrt(E)
        self.tokens = torch.from_numpy(inp["tokens"].reshape(B, R)).to(self.dev)
        self.targets = torch.from_numpy(inp["targets"].reshape(B, R)).to(self.dev)
        self.pos = torch.from_numpy(np.ascontiguousarray(inp["pos"], np.float32)).to(self.dev)   # fixed position table, an input
        self.x = [torch.empty(B, R, E, **act) for _ in range(nl + 1)]
        self.qkv = [torch.empty(B, R, 3 * E, **act) for _ in range(nl)]
        self.p = [torch.empty(B, N, Hh, S, S, **act) for _ in range(nl)]
        self.ctx = [torch.empty(B, R, E, **act) for _ in range(nl)]
        self.s1 = [torch.empty(B, R, E, **act) for _ in range(nl)]
        self.x1 = [torch.empty(B, R, E, **act) for _ in range(nl)]
        self.h = [torch.empty(B, R, F, **act) for _ in range(nl)]
        self.s2 = [torch.empty(B, R, E, **act) for _ in range(nl)]
        self.tmpE = torch.empty(B, R, E, **act)
        self.stats = [[torch.empty(B * R, **f32) for _ in range(4)] for _ in range(nl)]   # mean1, invstd1, mean2, invstd2
        self.logits = torch.empty(B, R, V, **act)
        self.dlogits = torch.empty(B, R, V, **act)
        self.dE = [torch.empty(B, R, E, **act) for _ in range(4)]
        self.dF = [torch.empty(B, R, F, **act) for _ in range(2)]
        self.dqkv = torch.empty(B, R, 3 * E, **act)
        self.loss = torch.empty(B, **f32)
        ws = max(4, hb.layernorm_bwd_workspace_bytes(B, R, E), hb.attention_bwd_workspace_bytes(B, N, S, E, Hh, self.dt),
                 hb.softmax_xent_rows_workspace_bytes(B, R),
                 hb.linear_bwd_workspace_bytes(B, R, E, 3 * E, self.dt), hb.linear_bwd_workspace_bytes(B, R, E, F, self.dt),
                 hb.linear_bwd_workspace_bytes(B, R, F, E, self.dt), hb.linear_bwd_workspace_bytes(B, R, E, V, self.dt))
        self.ws = torch.empty(ws, dtype=torch.uint8, device=self.dev)

    def _lin_bwd(self, P, name, M, Fx, Fy, x, dy, dx):
        hb.linear_bwd(self.B, M, Fx, Fy, self.dt, x, self.w(name + ".w"), dy, dx, self.g(name + ".w"), self.g(name + ".b"), self.ws)
        P("linear_bwd", layer=name, x=x, w=self.w(name + ".w"), dy=dy, dx=dx, dw=self.g(name + ".w"), db=self.g(name + ".b"))

    def forward_backward(self, probe=None):
        B, R, E, F, V, N, S, Hh, dt = self.B, self.R, self.E, self.F, self.V, self.N, self.S, self.Hh, self.dt
        P = probe if probe is not None else (lambda op, **kw: None)
        nl = self.spec.layers
        hb.embedding_fwd(B, R, V, E, dt, self.w("emb"), self.tokens, self.scale, self.pos, S, self.x[0])
        P("embedding_fwd", table=self.w("emb"), idx=self.tokens, pos=self.pos, y=self.x[0])
        for i in range(nl):
            k, x = f"l{i}", self.x[i]
            mu1, inv1, mu2, inv2 = self.stats[i]
            hb.linear_fwd(B, R, E, 3 * E, dt, x, self.w(k + ".in.w"), self.w(k + ".in.b"), self.qkv[i])
            P("linear_fwd", layer=k + ".in", x=x, w=self.w(k + ".in.w"), b=self.w(k + ".in.b"), y=self.qkv[i], act=0)
            hb.attention_fwd(B, N, S, E, Hh, dt, self.qkv[i], self.p[i], self.ctx[i], 1)
            P("attention_fwd", qkv=self.qkv[i], p=self.p[i], ctx=self.ctx[i])
            hb.linear_fwd(B, R, E, E, dt, self.ctx[i], self.w(k + ".out.w"), self.w(k + ".out.b"), self.tmpE)
            P("linear_fwd", layer=k + ".out", x=self.ctx[i], w=self.w(k + ".out.w"), b=self.w(k + ".out.b"), y=self.tmpE, act=0)
            hb.add(B * R * E, dt, x, self.tmpE, self.s1[i])
            P("add", a=x, b=self.tmpE, y=self.s1[i])
            hb.layernorm_fwd(B, R, E, dt, self.s1[i], self.master(k + ".ln1.w"), self.master(k + ".ln1.b"), self.LN_EPS,
                             mu1, inv1, self.x1[i])
            P("layernorm_fwd", layer=k + ".ln1", x=self.s1[i], w=self.master(k + ".ln1.w"), b=self.master(k + ".ln1.b"),
              y=self.x1[i], mean=mu1, invstd=inv1)
            hb.linear_fwd(B, R, E, F, dt, self.x1[i], self.w(k + ".ff1.w"), self.w(k + ".ff1.b"), self.h[i], hb.ACT_RELU)
            P("linear_fwd", layer=k + ".ff1", x=self.x1[i], w=self.w(k + ".ff1.w"), b=self.w(k + ".ff1.b"), y=self.h[i], act=1)
            hb.linear_fwd(B, R, F, E, dt, self.h[i], self.w(k + ".ff2.w"), self.w(k + ".ff2.b"), self.tmpE)
            P("linear_fwd", layer=k + ".ff2", x=self.h[i], w=self.w(k + ".ff2.w"), b=self.w(k + ".ff2.b"), y=self.tmpE, act=0)
            hb.add(B * R * E, dt, self.x1[i], self.tmpE, self.s2[i])
            P("add", a=self.x1[i], b=self.tmpE, y=self.s2[i])
            hb.layernorm_fwd(B, R, E, dt, self.s2[i], self.master(k + ".ln2.w"), self.master(k + ".ln2.b"), self.LN_EPS,
                             mu2, inv2, self.x[i + 1])
            P("layernorm_fwd", layer=k + ".ln2", x=self.s2[i], w=self.master(k + ".ln2.w"), b=self.master(k + ".ln2.b"),
              y=self.x[i + 1], mean=mu2, invstd=inv2)
        hb.linear_fwd(B, R, E, V, dt, self.x[nl], self.w("dec.w"), self.w("dec.b"), self.logits)
        P("linear_fwd", layer="dec", x=self.x[nl], w=self.w("dec.w"), b=self.w("dec.b"), y=self.logits, act=0)
        hb.softmax_xent_rows(B, R, V, dt, self.logits, self.targets, self.loss, self.dlogits, self.ws)
        P("softmax_xent", logits=self.logits, labels=self.targets, loss=self.loss, d=self.dlogits)
        # ---- backward
        d = self.dE[0]
        self._lin_bwd(P, "dec", R, E, V, self.x[nl], self.dlogits, d)
        for i in reversed(range(nl)):
            k = f"l{i}"
            mu1, inv1, mu2, inv2 = self.stats[i]
            ds2, t1, t2 = self.dE[1], self.dE[2], self.dE[3]
            hb.layernorm_bwd(B, R, E, dt, self.s2[i], d, self.master(k + ".ln2.w"), mu2, inv2, ds2,
                             self.g(k + ".ln2.w"), self.g(k + ".ln2.b"), self.ws)
            P("layernorm_bwd", layer=k + ".ln2", x=self.s2[i], dy=d, w=self.master(k + ".ln2.w"), mean=mu2, invstd=inv2,
              dx=ds2, dw=self.g(k + ".ln2.w"), db=self.g(k + ".ln2.b"))
            self._lin_bwd(P, k + ".ff2", R, F, E, self.h[i], ds2, self.dF[0])
            hb.act_bwd(B * R * F, dt, self.h[i], self.dF[0], self.dF[1], hb.ACT_RELU, 0.0, 1)
            P("relu_bwd_from_output", y=self.h[i], dy=self.dF[0], dx=self.dF[1])
            self._lin_bwd(P, k + ".ff1", R, E, F, self.x1[i], self.dF[1], t1)
            hb.add(B * R * E, dt, ds2, t1, t2)
            P("add", a=ds2, b=t1, y=t2)
            ds1 = self.dE[1]                                   # ds2 is consumed
            hb.layernorm_bwd(B, R, E, dt, self.s1[i], t2, self.master(k + ".ln1.w"), mu1, inv1, ds1,
                             self.g(k + ".ln1.w"), self.g(k + ".ln1.b"), self.ws)
            P("layernorm_bwd", layer=k + ".ln1", x=self.s1[i], dy=t2, w=self.master(k + ".ln1.w"), mean=mu1, invstd=inv1,
              dx=ds1, dw=self.g(k + ".ln1.w"), db=self.g(k + ".ln1.b"))
            self._lin_bwd(P, k + ".out", R, E, E, self.ctx[i], ds1, t1)            # t1 = dctx
            hb.attention_bwd(B, N, S, E, Hh, dt, self.qkv[i], self.p[i], t1, self.dqkv, self.ws)
            P("attention_bwd", qkv=self.qkv[i], p=self.p[i], dctx=t1, dqkv=self.dqkv)
            self._lin_bwd(P, k + ".in", R, E, 3 * E, self.x[i], self.dqkv, t2)
            hb.add(B * R * E, dt, ds1, t2, self.dE[0])
            P("add", a=ds1, b=t2, y=self.dE[0])
            d = self.dE[0]
        hb.embedding_bwd(B, R, V, E, dt, d, self.tokens, self.scale, self.g("emb"))
        P("embedding_bwd", dy=d, idx=self.tokens, dtable=self.g("emb"))
        return self.loss


class _PointChain:
    """One chain of a point-cloud model inside a ParamArena: per-point layers (k=1 convolution,
    BatchNorm, ReLU) named ``{prefix}conv{conv_base+i}``, then, if ``fc`` is given, the max over
    points and the fully connected layers ``{prefix}fc{i}`` (hidden ones with BatchNorm and ReLU,
    dropout after the last hidden one).  The last per-point layer, its BatchNorm, ReLU and the max
    run as one operator where the library has it.  ``fwd`` returns the chain's output tensor,
    ``bwd`` takes the gradient of that tensor."""

    def __init__(self, arena, prefix, conv, fc, conv_base, fc_bn=True, dropout_p=0.0, drop_mask=None):
        A = self.A = arena
        self.px, self.conv, self.fc, self.cb = prefix, tuple(conv), None if fc is None else tuple(fc), conv_base
        self.fc_bn, self.dropout_p, self.drop_mask = fc_bn, dropout_p, drop_mask
        B, Nb, L, dt = A.B, A.Nb, A.L, A.dt
        act = dict(dtype=A.tdt, device=A.dev)
        f32 = dict(dtype=torch.float32, device=A.dev)
        self.nconv = len(self.conv) - 1
        self.head = self.fc is not None
        self.nfc = len(self.fc) - 1 if self.head else 0
        self.fused_tail = False
        ws = 4
        if self.head and self.nconv >= 2:
            geo = (B, Nb, self.conv[-2], self.conv[-1], L, dt)
            wt = A.w(f"{prefix}conv{conv_base + self.nconv - 1}.w")     # the one-operator tail wants 16-byte aligned weights
            self.fused_tail = hb.conv1x1_bn_maxpool_fwd_workspace_bytes(*geo) > 0 and wt.data_ptr() % 16 == 0
            if self.fused_tail:
                ws = max(ws, hb.conv1x1_bn_maxpool_fwd_workspace_bytes(*geo), hb.conv1x1_bn_maxpool_bwd_workspace_bytes(*geo))
        nz = self.nconv - 1 if self.fused_tail else self.nconv
        self.z = [torch.empty(Nb, B * c, L, **act) for c in self.conv[1:1 + nz]]
        na = self.nconv if not self.head else self.nconv - 1            # a chain without a head keeps its last activation
        # prenorm[i]: layer i normalises layer i-1's stored pre-activation on load, a[i-1] is never stored
        # (the layer in front of the tail keeps its output: the tail operator reads it)
        self.prenorm = [False] * self.nconv
        for i in range(1, na):
            self.prenorm[i] = hb.conv1x1_bn_prenorm_supported(B, Nb, self.conv[i], self.conv[i + 1], L, dt)
        self.a = [None if (i + 1 < na and self.prenorm[i + 1]) else torch.empty(Nb, B * c, L, **act)
                  for i, c in enumerate(self.conv[1:1 + na])]
        cmax = max(self.conv)
        self.dbuf = [torch.empty(Nb * B * cmax * L, **act) for _ in range(2)]
        self.one_pass = [_bn_bwd_one_pass(B, Nb, self.conv[i], self.conv[i + 1], L, dt) for i in range(self.nconv)]
        # bn_sums[i]: layer i's two BatchNorm-backward reductions, left by layer i+1's backward call
        self.bn_sums = [None] * self.nconv
        for i in range(1, self.nconv):
            if self.prenorm[i] and self.one_pass[i] and self.one_pass[i - 1] and not (self.head and i == self.nconv - 1) and \
                    hb.conv1x1_bn_prenorm_bwd_gives_sums(B, Nb, self.conv[i], self.conv[i + 1], L, dt):
                self.bn_sums[i - 1] = torch.empty(B * self.conv[i], 2, **f32)
        for i in range(self.nconv):
            ws = max(ws, hb.conv1x1_bwd_workspace_bytes(B, Nb, self.conv[i], self.conv[i + 1], L, dt),
                     hb.conv1x1_bn_fwd_workspace_bytes(B, Nb, self.conv[i], self.conv[i + 1], L, dt))
            if self.one_pass[i]:
                ws = max(ws, hb.conv1x1_bn_bwd_workspace_bytes(B, Nb, self.conv[i], self.conv[i + 1], L, dt))
        if self.head:
            Cp = self.conv[-1]
            self.pooled = torch.empty(B, Nb, Cp, **act)
            self.pool_idx = torch.empty(B, Nb, Cp, dtype=torch.int32, device=A.dev)
            if self.fused_tail:
                self.zhit = torch.empty(B, Nb, Cp, **f32)
                self.moments = torch.empty(hb.conv1x1_bn_maxpool_saved_floats(B, self.conv[-2], Cp), **f32)
            self.fz = [torch.empty(B, Nb, f, **act) for f in self.fc[1:]]
            self.fh = [torch.empty(B, Nb, f, **act) for f in self.fc[1:-1]]
            self.fdrop = torch.empty(B, Nb, self.fc[-2], **act) if dropout_p > 0 else None
            self.fd = [torch.empty(B * Nb * max(self.fc), **act) for _ in range(2)]
            for i in range(self.nfc):
                ws = max(ws, hb.linear_bwd_workspace_bytes(B, Nb, self.fc[i], self.fc[i + 1], dt),
                         hb.linear_fwd_workspace_bytes(B, Nb, self.fc[i], self.fc[i + 1], dt))
        self.ws_bytes = ws

    def _bn(self, k):
        A = self.A
        return (A.master(k + ".bn.g"), A.master(k + ".bn.b"), A.BN_EPS, A.BN_MOMENTUM, A.running[k + ".bn.rm"],
                A.running[k + ".bn.rv"], A.saved[k + ".bn.mean"], A.saved[k + ".bn.invstd"])

    def fwd(self, x):
        """x: [Nb, B*conv[0], L] contiguous.  Returns the last activation (no head) or the last Linear's output."""
        A = self.A
        B, Nb, L, dt, ws = A.B, A.Nb, A.L, A.dt, A.ws
        self.x_in = x
        ci = self.conv[0]
        for i in range(self.nconv):
            co, k = self.conv[i + 1], f"{self.px}conv{self.cb + i}"
            tail = self.head and i == self.nconv - 1
            if tail and self.fused_tail:
                hb.conv1x1_bn_maxpool_fwd(B, Nb, ci, co, L, dt, x, _cs(B, ci, L), A.w(k + ".w"), A.w(k + ".b"), *self._bn(k),
                                          self.pooled, self.pool_idx, (Nb * co, co, 1), self.zhit, self.moments,
                                          hb.ACT_RELU, 0.0, ws)
                break
            if not tail:
                y = self.a[i]
                ys = None if y is None else _cs(B, co, L)
                if self.prenorm[i]:
                    kp = f"{self.px}conv{self.cb + i - 1}"
                    hb.conv1x1_bn_prenorm_fwd(B, Nb, ci, co, L, dt, self.z[i - 1], _cs(B, ci, L), A.master(kp + ".bn.g"),
                                              A.master(kp + ".bn.b"), A.saved[kp + ".bn.mean"], A.saved[kp + ".bn.invstd"],
                                              hb.ACT_RELU, 0.0, A.w(k + ".w"), A.w(k + ".b"), *self._bn(k), self.z[i],
                                              _cs(B, co, L), y, ys, hb.ACT_RELU, 0.0, ws)
                else:
                    hb.conv1x1_bn_fwd(B, Nb, ci, co, L, dt, x, _cs(B, ci, L), A.w(k + ".w"), A.w(k + ".b"), *self._bn(k),
                                      self.z[i], _cs(B, co, L), y, ys, hb.ACT_RELU, 0.0, ws)
                x, ci = y, co
                continue
            hb.conv1x1_fwd(B, Nb, ci, co, L, dt, x, _cs(B, ci, L), A.w(k + ".w"), A.w(k + ".b"), self.z[i], _cs(B, co, L))
            hb.bn_fwd_maxpool(B, Nb, co, L, dt, self.z[i], _cs(B, co, L), *self._bn(k), self.pooled, self.pool_idx,
                              (Nb * co, co, 1), hb.ACT_RELU)
            break
        if not self.head:
            return x
        h = self.pooled
        for i in range(self.nfc):
            fx, fy, k = self.fc[i], self.fc[i + 1], f"{self.px}fc{i}"
            last = i == self.nfc - 1
            if last or self.fc_bn:
                hb.linear_fwd_ws(B, Nb, fx, fy, dt, h, A.w(k + ".w"), A.w(k + ".b"), self.fz[i], workspace=ws)
                if last:
                    return self.fz[i]
                ls = (Nb * fy, fy, 1, 1)
                hb.bn_fwd(B, Nb, fy, 1, dt, self.fz[i], ls, *self._bn(k), self.fh[i], ls, hb.ACT_RELU)
            else:
                hb.linear_fwd_ws(B, Nb, fx, fy, dt, h, A.w(k + ".w"), A.w(k + ".b"), self.fh[i], hb.ACT_RELU, workspace=ws)
            h = self.fh[i]
            if i == self.nfc - 2 and self.dropout_p > 0:
                hb.dropout(B * Nb * fy, dt, h, self.drop_mask, self.dropout_p, self.fdrop)
                h = self.fdrop

    def bwd(self, d, want_dx):
        """d: gradient of the chain's output (flat, storage dtype).  Parameter gradients go to the
        arena; returns the gradient of the chain's input (flat view of an own buffer) if want_dx."""
        A = self.A
        B, Nb, L, dt, ws = A.B, A.Nb, A.L, A.dt, A.ws
        cur = 0
        for i in reversed(range(self.nfc)):
            fx, fy, k = self.fc[i], self.fc[i + 1], f"{self.px}fc{i}"
            last = i == self.nfc - 1
            if not last:
                n = B * Nb * fy
                if i == self.nfc - 2 and self.dropout_p > 0:
                    nd = self.fd[cur ^ 1][:n]
                    hb.dropout(n, dt, d, self.drop_mask, self.dropout_p, nd)
                    d, cur = nd, cur ^ 1
                nd = self.fd[cur ^ 1][:n]
                if self.fc_bn:
                    ls = (Nb * fy, fy, 1, 1)
                    hb.bn_bwd(B, Nb, fy, 1, dt, self.fz[i], ls, d, ls, A.master(k + ".bn.g"), A.master(k + ".bn.b"),
                              A.saved[k + ".bn.mean"], A.saved[k + ".bn.invstd"], nd, ls, A.g(k + ".bn.g"),
                              A.g(k + ".bn.b"), hb.ACT_RELU, 0.0, A.g(k + ".b"))
                else:
                    hb.act_bwd(n, dt, self.fh[i], d, nd, hb.ACT_RELU, 0.0, 1)
                d, cur = nd, cur ^ 1
            if i == 0:
                hin = self.pooled
            elif i == self.nfc - 1 and self.dropout_p > 0:
                hin = self.fdrop
            else:
                hin = self.fh[i - 1]
            nd = self.fd[cur ^ 1][:B * Nb * fx]
            own_db = A.g(k + ".b") if (last or not self.fc_bn) else None
            hb.linear_bwd(B, Nb, fx, fy, dt, hin, A.w(k + ".w"), d, nd, A.g(k + ".w"), own_db, ws)
            d, cur = nd, cur ^ 1

        da, cur = d, 0      # da never lives in dbuf[cur]
        for i in reversed(range(self.nconv)):
            ci, co, k = self.conv[i], self.conv[i + 1], f"{self.px}conv{self.cb + i}"
            cs, xs = _cs(B, co, L), _cs(B, ci, L)
            xin = self.x_in if i == 0 else self.a[i - 1]
            need_dx = i > 0 or want_dx
            tail = self.head and i == self.nconv - 1
            bn = (A.master(k + ".bn.g"), A.master(k + ".bn.b"), A.saved[k + ".bn.mean"], A.saved[k + ".bn.invstd"])
            if tail and self.fused_tail:
                # the operator always writes dX: give it a buffer even when nobody reads it
                dxo = self.dbuf[cur][:Nb * B * ci * L]
                hb.conv1x1_bn_maxpool_bwd(B, Nb, ci, co, L, dt, xin, xs, A.w(k + ".w"), A.w(k + ".b"), None, None, self.zhit,
                                          self.moments, da, self.pool_idx, (Nb * co, co, 1), *bn, dxo, xs, A.g(k + ".w"),
                                          A.g(k + ".b"), A.g(k + ".bn.g"), A.g(k + ".bn.b"), hb.ACT_RELU, 0.0, ws)
                da, cur = (dxo if need_dx else None), cur ^ 1
                continue
            if not tail and self.one_pass[i]:
                # BatchNorm backward + convolution backward in one call; its dX must not share da's buffer
                dxin = self.dbuf[cur][:Nb * B * ci * L] if need_dx else None
                out = (dxin, xs if need_dx else None, A.g(k + ".w"), A.g(k + ".b"), A.g(k + ".bn.g"), A.g(k + ".bn.b"),
                       hb.ACT_RELU, 0.0, ws, None, self.bn_sums[i])
                if self.prenorm[i]:
                    kp = f"{self.px}conv{self.cb + i - 1}"
                    hb.conv1x1_bn_prenorm_bwd(B, Nb, ci, co, L, dt, self.z[i - 1], xs, A.master(kp + ".bn.g"),
                                              A.master(kp + ".bn.b"), A.saved[kp + ".bn.mean"], A.saved[kp + ".bn.invstd"],
                                              hb.ACT_RELU, 0.0, A.w(k + ".w"), self.z[i], cs, da, cs, *bn, *out,
                                              self.bn_sums[i - 1])
                else:
                    hb.conv1x1_bn_bwd(B, Nb, ci, co, L, dt, xin, xs, A.w(k + ".w"), self.z[i], cs, da, cs, *bn, *out)
                da, cur = dxin, cur ^ 1
                continue
            dz = self.dbuf[cur][:Nb * B * co * L]
            dxin = self.dbuf[cur ^ 1][:Nb * B * ci * L] if need_dx else None       # over da, which the BatchNorm has consumed
            if tail:
                hb.bn_bwd_maxpool(B, Nb, co, L, dt, self.z[i], cs, da, self.pool_idx, (Nb * co, co, 1), *bn, dz, cs,
                                  A.g(k + ".bn.g"), A.g(k + ".bn.b"), hb.ACT_RELU, 0.0, A.g(k + ".b"))
            else:
                hb.bn_bwd(B, Nb, co, L, dt, self.z[i], cs, da, cs, *bn, dz, cs, A.g(k + ".bn.g"), A.g(k + ".bn.b"),
                          hb.ACT_RELU, 0.0, A.g(k + ".b"))
            if need_dx:
                hb.conv1x1_bwd(B, Nb, ci, co, L, dt, None, None, A.w(k + ".w"), dz, cs, dxin, xs, None, None, ws)
            hb.conv1x1_bwd(B, Nb, ci, co, L, dt, xin, xs, None, dz, cs, None, None, A.g(k + ".w"), None, ws)
            da = dxin
        return da if want_dx else None


class FusedPointNetClsT(ParamArena):
    """PointNet-classification-style array whose models carry the input (3x3) and / or feature
    (64x64) transform sub-networks: each is a small chain of the same fused operators whose output
    plus the identity is a matrix per (model, cloud), applied to all points of the cloud by
    ``point_transform_fwd``; its gradient comes back through ``point_transform_bwd``."""

    BN_EPS = 1e-5
    BN_MOMENTUM = 0.1

    def __init__(self, tspec, inp: dict, device: str = "cuda"):
        import hfta_inputs as hi
        spec = tspec.cls
        self.tspec, self.spec = tspec, spec
        self.B, self.Nb, self.L = spec.B, spec.Nb, spec.L
        self.dtype, self.dt, self.tdt = spec.dtype, _DT[spec.dtype], _TDT[spec.dtype]
        self.dev = torch.device(device)
        B, Nb, L = self.B, self.Nb, self.L
        self._init_arena(hi.pointnet_t_param_shapes(tspec), B, inp, spec.dtype, self.dev)
        f32 = dict(dtype=torch.float32, device=self.dev)
        act = dict(dtype=self.tdt, device=self.dev)
        self.running: Dict[str, torch.Tensor] = {}
        self.saved: Dict[str, torch.Tensor] = {}
        for name, shp in self.shapes:
            if name.endswith(".bn.g"):
                k = name[:-2]
                self.running[k + ".rm"] = torch.zeros(B * shp[0], **f32)
                self.running[k + ".rv"] = torch.ones(B * shp[0], **f32)
                self.saved[k + ".mean"] = torch.empty(B * shp[0], **f32)
                self.saved[k + ".invstd"] = torch.empty(B * shp[0], **f32)
        self.points = torch.from_numpy(np.ascontiguousarray(inp["points"])).to(self.dev).to(self.tdt)
        self.labels = torch.from_numpy(np.ascontiguousarray(inp["labels"])).to(self.dev)
        self.drop_mask = None
        if spec.dropout_p > 0:
            self.drop_mask = torch.from_numpy(np.ascontiguousarray(inp["drop_mask"])).to(self.dev)
        self.loss = torch.empty(B, **f32)

        def tnet(k):
            ch = _PointChain(self, f"t{k}.", (k,) + tuple(tspec.tnet_conv),
                             (tspec.tnet_conv[-1],) + tuple(tspec.tnet_fc) + (k * k,), 0)
            eye = torch.eye(k, **act).reshape(1, 1, k * k).expand(B, Nb, k * k).contiguous()
            return dict(k=k, chain=ch, eye=eye, T=torch.empty(B, Nb, k, k, **act), dT=torch.empty(B, Nb, k, k, **act),
                        y=torch.empty(Nb, B * k, L, **act), dx=torch.empty(Nb * B * k * L, **act))

        self.t_in = tnet(3) if tspec.input_transform else None
        self.block0 = _PointChain(self, "", spec.conv[:2], None, 0)
        self.t_feat = tnet(spec.conv[1]) if tspec.feature_transform else None
        self.rest = _PointChain(self, "", spec.conv[1:], spec.fc, 1, spec.fc_bn, spec.dropout_p, self.drop_mask)
        self.dlogits = torch.empty(B * Nb * spec.fc[-1], **act)
        chains = [self.block0, self.rest] + [t["chain"] for t in (self.t_in, self.t_feat) if t is not None]
        self.ws = torch.empty(max(c.ws_bytes for c in chains), dtype=torch.uint8, device=self.dev)

    def _transform_fwd(self, t, x):
        B, Nb, L, dt, k = self.B, self.Nb, self.L, self.dt, t["k"]
        o = t["chain"].fwd(x)
        hb.add(B * Nb * k * k, dt, o, t["eye"], t["T"])
        t["x"] = x
        hb.point_transform_fwd(B, Nb, k, k, L, dt, x, _cs(B, k, L), t["T"], t["y"], _cs(B, k, L))
        return t["y"]

    def _transform_bwd(self, t, dy, want_dx):
        B, Nb, L, dt, k = self.B, self.Nb, self.L, self.dt, t["k"]
        cs = _cs(B, k, L)
        hb.point_transform_bwd(B, Nb, k, k, L, dt, t["x"], cs, t["T"], dy, cs, t["dx"] if want_dx else None,
                               cs if want_dx else None, t["dT"])
        dnet = t["chain"].bwd(t["dT"].view(-1), want_dx)
        if not want_dx:
            return None
        hb.add(Nb * B * k * L, dt, t["dx"], dnet, t["dx"])
        return t["dx"]

    def forward_backward(self):
        s, B, Nb, dt = self.spec, self.B, self.Nb, self.dt
        x = self.points
        if self.t_in is not None:
            x = self._transform_fwd(self.t_in, x)
        x = self.block0.fwd(x)
        if self.t_feat is not None:
            x = self._transform_fwd(self.t_feat, x)
        logits = self.rest.fwd(x)
        hb.softmax_xent(B, Nb, s.fc[-1], dt, logits, self.labels, self.loss, self.dlogits)
        d = self.rest.bwd(self.dlogits, True)
        if self.t_feat is not None:
            d = self._transform_bwd(self.t_feat, d, True)
        d = self.block0.bwd(d, self.t_in is not None)
        if self.t_in is not None:
            self._transform_bwd(self.t_in, d, False)
        return self.loss

    def train_step(self):
        loss = self.forward_backward()
        self.adam()
        return loss
