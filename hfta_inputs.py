"""Seeded synthetic inputs for the fused-array workloads.

This module serves both the CPU oracle and the HIP path and therefore holds
none of the method's arithmetic: it only draws random numbers, shapes them like
the paper's workloads (point clouds of 2500 points / 16 classes standing in for
ShapeNet-part, 64x64x3 images standing in for LSUN; section "Methodology",
paragraph on PointNet and DCGAN) and lays them out as the operator fusion rules
table prescribes (conv family ``[N, B*C, L]``, linear family ``[B, N, F]``).

Everything is numpy; values destined for bf16 storage are snapped to
bf16-representable float32 with ``torch``'s own cast (a library conversion, not
ours) so that both sides start from identical bits.

Model ``b`` draws from its own child stream, so its data does not depend on B.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------
# helpers
# --------------------------------------------------------------------------
def config_seed(config_index: int) -> int:
    return 1000 * config_index + 7


def model_streams(seed: int, B: int) -> List[np.random.Generator]:
    """One independent generator per model, spawned in order of b."""
    ss = np.random.SeedSequence(seed)
    return [np.random.default_rng(s) for s in ss.spawn(B)]


def snap(a: np.ndarray, dtype: str) -> np.ndarray:
    """Return float32 values exactly representable in the storage dtype."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype in ("f32", "f64"):     # "f64": oracle-only mode without storage rounding
        return a
    if dtype == "bf16":
        import torch

        return torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    raise ValueError(dtype)


def unit_ball_points(rng: np.random.Generator, n: int, L: int) -> np.ndarray:
    """Points uniform in the unit ball, shape [n, 3, L]."""
    d = rng.standard_normal((n, 3, L))
    d /= np.linalg.norm(d, axis=1, keepdims=True)
    r = rng.random((n, 1, L)) ** (1.0 / 3.0)
    return d * r


def uniform_fan_in(rng: np.random.Generator, shape: Sequence[int], fan_in: int,
                   gain_sq: float) -> np.ndarray:
    """U(-sqrt(gain_sq/fan_in), +sqrt(gain_sq/fan_in))."""
    bound = math.sqrt(gain_sq / fan_in)
    return rng.uniform(-bound, bound, size=tuple(shape))


def log_uniform(rng: np.random.Generator, lo: float, hi: float) -> float:
    return float(math.exp(rng.uniform(math.log(lo), math.log(hi))))


# --------------------------------------------------------------------------
# PointNet-classification-style fused array
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class PointNetClsSpec:
    """Layer list of a PointNet-cls-style array (all models share it)."""
    name: str
    B: int
    Nb: int                 # clouds per model per step
    L: int                  # points per cloud
    conv: Tuple[int, ...]   # channel chain of the per-point MLP, starts at 3
    fc: Tuple[int, ...]     # channel chain after the pool, ends at n_classes
    fc_bn: bool             # BatchNorm on the hidden FC layers
    dropout_p: float        # dropout after the last hidden FC activation (0 = none)
    dtype: str              # "f32" or "bf16" (storage; master weights fp32)
    lr_range: Tuple[float, float] = (1e-4, 1e-2)
    beta1_range: Optional[Tuple[float, float]] = None  # None -> 0.9 for all
    n_classes: int = 16
    config_index: int = 0


def spec_c0() -> PointNetClsSpec:
    return PointNetClsSpec(name="c0_pointnet_cls_B2_fp32", B=2, Nb=4, L=256,
                           conv=(3, 64, 128, 1024), fc=(1024, 256, 16), fc_bn=False,
                           dropout_p=0.0, dtype="f32", config_index=0)


def spec_c1(B: int = 8, Nb: int = 32, L: int = 2500, dtype: str = "bf16") -> PointNetClsSpec:
    return PointNetClsSpec(name=f"c1_pointnet_cls_B{B}_{dtype}", B=B, Nb=Nb, L=L,
                           conv=(3, 64, 64, 64, 128, 1024), fc=(1024, 512, 256, 16),
                           fc_bn=True, dropout_p=0.3, dtype=dtype,
                           beta1_range=(0.8, 0.95), config_index=1)


def pointnet_cls_param_shapes(spec: PointNetClsSpec) -> List[Tuple[str, Tuple[int, ...]]]:
    """Per-model parameter list, in arena order.

    conv weights are ``[Co, Ci]`` (kernel length 1), linear weights ``[Fx, Fy]``
    as in the fusion rules table (baddbmm orientation).
    """
    out: List[Tuple[str, Tuple[int, ...]]] = []
    for i in range(len(spec.conv) - 1):
        ci, co = spec.conv[i], spec.conv[i + 1]
        out += [(f"conv{i}.w", (co, ci)), (f"conv{i}.b", (co,)),
                (f"conv{i}.bn.g", (co,)), (f"conv{i}.bn.b", (co,))]
    nfc = len(spec.fc) - 1
    for i in range(nfc):
        fx, fy = spec.fc[i], spec.fc[i + 1]
        out += [(f"fc{i}.w", (fx, fy)), (f"fc{i}.b", (fy,))]
        if spec.fc_bn and i < nfc - 1:
            out += [(f"fc{i}.bn.g", (fy,)), (f"fc{i}.bn.b", (fy,))]
    return out


def pointnet_cls_inputs(spec: PointNetClsSpec, seed: Optional[int] = None) -> Dict[str, object]:
    """Draw everything one training step needs.

    Returns a dict with
      points   float32 [Nb, B*3, L]  (snapped to spec.dtype)
      labels   int32   [B, Nb]
      params   list over b of dict name -> float32 array (fp32 master values)
      lr, beta1, beta2, eps, wd : float32 [B]
      drop_mask uint8 [B, Nb, fc[-2]]  (1 = keep), or None
    """
    seed = config_seed(spec.config_index) if seed is None else seed
    rngs = model_streams(seed, spec.B)
    B, Nb, L = spec.B, spec.Nb, spec.L
    points = np.empty((Nb, B * 3, L), dtype=np.float32)
    labels = np.empty((B, Nb), dtype=np.int32)
    params = []
    lr = np.empty(B, np.float32)
    beta1 = np.full(B, 0.9, np.float32)
    beta2 = np.full(B, 0.999, np.float32)
    eps = np.full(B, 1e-8, np.float32)
    wd = np.zeros(B, np.float32)
    mask = None
    if spec.dropout_p > 0:
        mask = np.empty((B, Nb, spec.fc[-2]), dtype=np.uint8)
    for b, rng in enumerate(rngs):
        points[:, 3 * b:3 * b + 3, :] = unit_ball_points(rng, Nb, L)
        labels[b] = rng.integers(0, spec.n_classes, size=Nb)
        p = {}
        for name, shape in pointnet_cls_param_shapes(spec):
            if name.endswith(".bn.g"):
                p[name] = np.ones(shape, np.float32)
            elif name.endswith(".bn.b"):
                p[name] = np.zeros(shape, np.float32)
            elif name.endswith(".w"):
                fan_in = shape[1] if name.startswith("conv") else shape[0]
                p[name] = uniform_fan_in(rng, shape, fan_in, 6.0).astype(np.float32)
            else:  # bias of conv / linear: fan_in of the layer it belongs to
                wshape = dict(pointnet_cls_param_shapes(spec))[name[:-2] + ".w"]
                fan_in = wshape[1] if name.startswith("conv") else wshape[0]
                p[name] = uniform_fan_in(rng, shape, fan_in, 1.0).astype(np.float32)
        params.append(p)
        lr[b] = log_uniform(rng, *spec.lr_range)
        if spec.beta1_range is not None:
            beta1[b] = rng.uniform(*spec.beta1_range)
        if mask is not None:
            mask[b] = (rng.random((Nb, spec.fc[-2])) >= spec.dropout_p).astype(np.uint8)
    return dict(points=snap(points, spec.dtype), labels=labels, params=params,
                lr=lr, beta1=beta1, beta2=beta2, eps=eps, wd=wd, drop_mask=mask)


# --------------------------------------------------------------------------
# PointNet-cls with the input / feature transform sub-networks
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class PointNetTSpec:
    """A PointNet-cls array whose models carry transform sub-networks: per-point layers
    k -> tnet_conv..., max over points, Linear layers tnet_fc... -> k*k; k = 3 on the coordinates
    (input transform), k = cls.conv[1] on the first layer's output (feature transform)."""
    cls: PointNetClsSpec
    tnet_conv: Tuple[int, ...] = (64, 128, 1024)
    tnet_fc: Tuple[int, ...] = (512, 256)
    input_transform: bool = True
    feature_transform: bool = True

    # what generic drivers ask of a spec
    B = property(lambda self: self.cls.B)
    Nb = property(lambda self: self.cls.Nb)
    L = property(lambda self: self.cls.L)
    dtype = property(lambda self: self.cls.dtype)
    name = property(lambda self: self.cls.name + "_transforms")

    def with_cls(self, **kw) -> "PointNetTSpec":
        return dataclasses.replace(self, cls=dataclasses.replace(self.cls, **kw))


def tnet_sizes(tspec: PointNetTSpec) -> List[int]:
    """Matrix sizes of the sub-networks, largest first: in arena order the only parameter whose
    size is not a multiple of 8 (the 9 biases of the 3x3 matrix) then comes last, so every weight
    matrix of every model starts on a 16-byte boundary."""
    return ([tspec.cls.conv[1]] if tspec.feature_transform else []) + ([3] if tspec.input_transform else [])


def pointnet_t_param_shapes(tspec: PointNetTSpec) -> List[Tuple[str, Tuple[int, ...]]]:
    out = list(pointnet_cls_param_shapes(tspec.cls))
    for k in tnet_sizes(tspec):
        conv = (k,) + tuple(tspec.tnet_conv)
        fc = (tspec.tnet_conv[-1],) + tuple(tspec.tnet_fc) + (k * k,)
        for i in range(len(conv) - 1):
            out += [(f"t{k}.conv{i}.w", (conv[i + 1], conv[i])), (f"t{k}.conv{i}.b", (conv[i + 1],)),
                    (f"t{k}.conv{i}.bn.g", (conv[i + 1],)), (f"t{k}.conv{i}.bn.b", (conv[i + 1],))]
        for i in range(len(fc) - 1):
            out += [(f"t{k}.fc{i}.w", (fc[i], fc[i + 1])), (f"t{k}.fc{i}.b", (fc[i + 1],))]
            if i < len(fc) - 2:
                out += [(f"t{k}.fc{i}.bn.g", (fc[i + 1],)), (f"t{k}.fc{i}.bn.b", (fc[i + 1],))]
    return out


def pointnet_t_inputs(tspec: PointNetTSpec, seed: Optional[int] = None) -> Dict[str, object]:
    """pointnet_cls_inputs plus the sub-networks' parameters (same initialisation rule; the last
    Linear of a sub-network is scaled by 0.1 so that the matrices start near the identity)."""
    spec = tspec.cls
    inp = pointnet_cls_inputs(spec, seed)
    seed = config_seed(spec.config_index) if seed is None else seed
    rngs = model_streams(seed + 7919, spec.B)
    shapes = pointnet_t_param_shapes(tspec)
    sd = dict(shapes)
    for b, rng in enumerate(rngs):
        p = inp["params"][b]
        for name, shape in shapes:
            if name in p:
                continue
            conv = ".conv" in name
            if name.endswith(".bn.g"):
                p[name] = np.ones(shape, np.float32)
            elif name.endswith(".bn.b"):
                p[name] = np.zeros(shape, np.float32)
            else:
                wshape = shape if name.endswith(".w") else sd[name[:-2] + ".w"]
                fan_in = wshape[1] if conv else wshape[0]
                v = uniform_fan_in(rng, shape, fan_in, 6.0 if name.endswith(".w") else 1.0)
                last = (not conv) and name.split(".")[1] == f"fc{len(tspec.tnet_fc)}"
                p[name] = (v * (0.1 if last else 1.0)).astype(np.float32)
    return inp


# --------------------------------------------------------------------------
# PointNet-segmentation-style fused array (BASELINE config 2)
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class PointNetSegSpec:
    """Per-point MLP, max over points, then a per-point head on the concatenation of every
    per-point feature map, the tiled global feature and the tiled object-category one-hot."""
    name: str
    B: int
    Nb: int
    L: int
    conv: Tuple[int, ...]     # per-point MLP channel chain, starts at 3
    head: Tuple[int, ...]     # head channel chain; head[0] = sum(conv[1:]) + conv[-1] + n_cat, ends at n_parts
    dtype: str
    n_cat: int = 16
    n_parts: int = 50
    lr_range: Tuple[float, float] = (1e-4, 1e-2)
    config_index: int = 2

    @property
    def c_point(self) -> int:          # channels of the concatenated per-point features
        return sum(self.conv[1:])

    @property
    def c_global(self) -> int:         # tiled part: global feature + category one-hot
        return self.conv[-1] + self.n_cat


def spec_c2(B: int = 6, Nb: int = 16, L: int = 2500, dtype: str = "bf16") -> PointNetSegSpec:
    conv = (3, 64, 128, 128, 512, 2048)
    return PointNetSegSpec(name=f"c2_pointnet_seg_B{B}_{dtype}", B=B, Nb=Nb, L=L, conv=conv,
                           head=(sum(conv[1:]) + conv[-1] + 16, 256, 256, 128, 50), dtype=dtype)


def seg_thin(B: int, Nb: int, L: int, dtype: str, div: int = 8) -> PointNetSegSpec:
    """Config 2's layer list with every hidden width divided by ``div`` (oracle-sized cases)."""
    conv = (3,) + tuple(max(8, c // div) for c in (64, 128, 128, 512, 2048))
    head_hidden = tuple(max(8, c // div) for c in (256, 256, 128))
    return PointNetSegSpec(name=f"c2_thin{div}_B{B}_{dtype}", B=B, Nb=Nb, L=L, conv=conv,
                           head=(sum(conv[1:]) + conv[-1] + 16,) + head_hidden + (50,), dtype=dtype)


def pointnet_seg_param_shapes(spec: PointNetSegSpec) -> List[Tuple[str, Tuple[int, ...]]]:
    """Per-model parameters of the layer list.  The first head layer has ONE ``[head[1], head[0]]``
    weight over the whole concatenation (per-point features, then the tiled global feature, then the
    tiled one-hot); how an implementation stores it is its own business."""
    out: List[Tuple[str, Tuple[int, ...]]] = []
    for i in range(len(spec.conv) - 1):
        ci, co = spec.conv[i], spec.conv[i + 1]
        out += [(f"conv{i}.w", (co, ci)), (f"conv{i}.b", (co,)), (f"conv{i}.bn.g", (co,)), (f"conv{i}.bn.b", (co,))]
    nh = len(spec.head) - 1
    for i in range(nh):
        ci, co = spec.head[i], spec.head[i + 1]
        out += [(f"head{i}.w", (co, ci)), (f"head{i}.b", (co,))]
        if i < nh - 1:
            out += [(f"head{i}.bn.g", (co,)), (f"head{i}.bn.b", (co,))]
    return out


def pointnet_seg_inputs(spec: PointNetSegSpec, seed: Optional[int] = None) -> Dict[str, object]:
    """points float32 [Nb, B*3, L]; labels int32 [B, Nb, L] (part of every point); category int32
    [B, Nb] and its one-hot float32 [B, Nb, n_cat]; params; lr, beta1, beta2, eps, wd [B]."""
    seed = config_seed(spec.config_index) if seed is None else seed
    rngs = model_streams(seed, spec.B)
    B, Nb, L = spec.B, spec.Nb, spec.L
    points = np.empty((Nb, B * 3, L), dtype=np.float32)
    labels = np.empty((B, Nb, L), dtype=np.int32)
    cat = np.empty((B, Nb), dtype=np.int32)
    params = []
    lr = np.empty(B, np.float32)
    shapes = pointnet_seg_param_shapes(spec)
    for b, rng in enumerate(rngs):
        points[:, 3 * b:3 * b + 3, :] = unit_ball_points(rng, Nb, L)
        labels[b] = rng.integers(0, spec.n_parts, size=(Nb, L))
        cat[b] = rng.integers(0, spec.n_cat, size=Nb)
        p = {}
        for name, shape in shapes:
            layer = name.split(".")[0]
            fan_in = dict(shapes)[layer + ".w"][1]
            if name.endswith(".bn.g"):
                p[name] = np.ones(shape, np.float32)
            elif name.endswith(".bn.b"):
                p[name] = np.zeros(shape, np.float32)
            elif name.endswith(".w"):
                p[name] = uniform_fan_in(rng, shape, fan_in, 6.0).astype(np.float32)
            else:
                p[name] = uniform_fan_in(rng, shape, fan_in, 1.0).astype(np.float32)
        params.append(p)
        lr[b] = log_uniform(rng, *spec.lr_range)
    onehot = np.zeros((B, Nb, spec.n_cat), np.float32)
    np.put_along_axis(onehot, cat[:, :, None].astype(np.int64), 1.0, axis=2)
    return dict(points=snap(points, spec.dtype), labels=labels, category=cat, onehot=onehot, params=params, lr=lr,
                beta1=np.full(B, 0.9, np.float32), beta2=np.full(B, 0.999, np.float32),
                eps=np.full(B, 1e-8, np.float32), wd=np.zeros(B, np.float32))


# --------------------------------------------------------------------------
# Transformer-encoder language-model fused array (the paper's secondary Transformer workload;
# synthetic token streams stand in for its text corpus)
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class TransformerSpec:
    name: str
    B: int
    N: int                  # sequences per model per step
    S: int                  # tokens per sequence
    E: int                  # model width
    heads: int
    F: int                  # feed-forward width
    layers: int
    V: int                  # vocabulary size
    dtype: str
    lr_range: Tuple[float, float] = (1e-4, 1e-3)
    config_index: int = 5

    @property
    def Nb(self) -> int:    # samples (sequences) per model per step
        return self.N


def spec_t0(B: int = 8, N: int = 32, S: int = 64, E: int = 256, heads: int = 4, F: int = 1024, layers: int = 2,
            V: int = 8192, dtype: str = "bf16") -> TransformerSpec:
    return TransformerSpec(name=f"t0_transformer_lm_B{B}_{dtype}", B=B, N=N, S=S, E=E, heads=heads, F=F, layers=layers,
                           V=V, dtype=dtype)


def transformer_param_shapes(spec: TransformerSpec) -> List[Tuple[str, Tuple[int, ...]]]:
    """Per-model parameters in arena order; Linear weights are [Fx, Fy] (baddbmm orientation)."""
    E, F, V = spec.E, spec.F, spec.V
    out: List[Tuple[str, Tuple[int, ...]]] = [("emb", (V, E))]
    for i in range(spec.layers):
        k = f"l{i}"
        out += [(k + ".in.w", (E, 3 * E)), (k + ".in.b", (3 * E,)), (k + ".out.w", (E, E)), (k + ".out.b", (E,)),
                (k + ".ln1.w", (E,)), (k + ".ln1.b", (E,)), (k + ".ff1.w", (E, F)), (k + ".ff1.b", (F,)),
                (k + ".ff2.w", (F, E)), (k + ".ff2.b", (E,)), (k + ".ln2.w", (E,)), (k + ".ln2.b", (E,))]
    out += [("dec.w", (E, V)), ("dec.b", (V,))]
    return out


def position_table(S: int, E: int) -> np.ndarray:
    """The fixed sinusoidal position table of the encoder, float32 [S, E] (an input constant of the
    model, shared by all B models): sin(pos / 10000^(2i/E)) on even columns, cos on odd ones."""
    pos = np.arange(S, dtype=np.float64)[:, None]
    div = np.exp(np.arange(0, E, 2, dtype=np.float64) * (-np.log(10000.0) / E))
    pe = np.zeros((S, E))
    pe[:, 0::2] = np.sin(pos * div)
    pe[:, 1::2] = np.cos(pos * div)[:, :E // 2]
    return pe.astype(np.float32)


def transformer_inputs(spec: TransformerSpec, seed: Optional[int] = None, perturb_ln: bool = False) -> Dict[str, object]:
    """tokens, targets int32 [B, N, S] (targets = the next token of a stream of N*S+1 uniform tokens);
    pos float32 [S, E] (position_table); params; lr, beta1, beta2, eps, wd [B]."""
    seed = config_seed(spec.config_index) if seed is None else seed
    rngs = model_streams(seed, spec.B)
    B, N, S = spec.B, spec.N, spec.S
    tokens = np.empty((B, N, S), np.int32)
    targets = np.empty((B, N, S), np.int32)
    params = []
    lr = np.empty(B, np.float32)
    for b, rng in enumerate(rngs):
        stream = rng.integers(0, spec.V, size=N * S + 1)
        tokens[b] = stream[:-1].reshape(N, S)
        targets[b] = stream[1:].reshape(N, S)
        p = {}
        for name, shape in transformer_param_shapes(spec):
            if name == "emb":
                p[name] = rng.uniform(-0.1, 0.1, size=shape).astype(np.float32)
            elif ".ln" in name:
                base = 1.0 if name.endswith(".w") else 0.0
                p[name] = (base + (0.1 * rng.standard_normal(shape) if perturb_ln else 0.0)) * np.ones(shape)
                p[name] = p[name].astype(np.float32)
            elif name.endswith(".w"):
                p[name] = uniform_fan_in(rng, shape, shape[0], 3.0).astype(np.float32)
            else:
                p[name] = np.zeros(shape, np.float32) if not perturb_ln else (0.05 * rng.standard_normal(shape)).astype(np.float32)
        params.append(p)
        lr[b] = log_uniform(rng, *spec.lr_range)
    return dict(tokens=tokens, targets=targets, pos=position_table(S, spec.E), params=params, lr=lr,
                beta1=np.full(B, 0.9, np.float32), beta2=np.full(B, 0.999, np.float32), eps=np.full(B, 1e-8, np.float32),
                wd=np.zeros(B, np.float32))


# --------------------------------------------------------------------------
# operator-level cases (shapes of the other workloads)
# --------------------------------------------------------------------------
def normal(seed: int, shape: Sequence[int], dtype: str = "f32", scale: float = 1.0) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return snap(rng.standard_normal(tuple(shape)) * scale, dtype)


def uniform(seed: int, shape: Sequence[int], lo: float, hi: float, dtype: str = "f32") -> np.ndarray:
    rng = np.random.default_rng(seed)
    return snap(rng.uniform(lo, hi, size=tuple(shape)), dtype)


def adam_hparams(seed: int, B: int, lr=(1e-4, 1e-2), beta1=(0.8, 0.95), beta2=(0.9, 0.999),
                 wd=(0.0, 0.1)) -> Dict[str, np.ndarray]:
    """Per-model optimiser hyper-parameter vectors (the fusible ones of the
    hyper-parameter list table)."""
    rng = np.random.default_rng(seed)
    return dict(
        lr=np.exp(rng.uniform(math.log(lr[0]), math.log(lr[1]), B)).astype(np.float32),
        beta1=rng.uniform(*beta1, B).astype(np.float32),
        beta2=rng.uniform(*beta2, B).astype(np.float32),
        eps=np.full(B, 1e-8, np.float32),
        wd=rng.uniform(*wd, B).astype(np.float32),
    )


# DCGAN layer table (BASELINE config 3): (Ci, Co, H_in, stride, pad); 4x4 kernels.
DCGAN_D_LAYERS = ((3, 64, 64, 2, 1), (64, 128, 32, 2, 1), (128, 256, 16, 2, 1),
                  (256, 512, 8, 2, 1), (512, 1, 4, 1, 0))
# generator: transposed convolutions, listed as (Ci, Co, H_in, stride, pad)
DCGAN_G_LAYERS = ((100, 512, 1, 1, 0), (512, 256, 4, 2, 1), (256, 128, 8, 2, 1),
                  (128, 64, 16, 2, 1), (64, 3, 32, 2, 1))


def dcgan_weights(seed: int, B: int, shape: Sequence[int], dtype: str = "bf16") -> np.ndarray:
    """N(0, 0.02^2) weights, one set per model, concatenated on the leading dim."""
    rngs = model_streams(seed, B)
    w = np.concatenate([r.standard_normal(tuple(shape)) * 0.02 for r in rngs], axis=0)
    return snap(w, dtype)


# --------------------------------------------------------------------------
# Transformer-MLP-block fused array (BASELINE config 4)
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class MlpSpec:
    """`blocks` residual blocks x <- LayerNorm(x + W2 GELU(W1 x + b1) + b2) on R rows of E features."""
    name: str
    B: int
    R: int                  # rows (tokens) per model per step
    E: int                  # model width
    H: int                  # hidden width
    blocks: int
    dtype: str
    Nb: int = 32            # sequences per model per step (R = Nb * tokens per sequence)
    lr_range: Tuple[float, float] = (1e-5, 1e-3)
    wd_range: Tuple[float, float] = (0.0, 0.1)
    config_index: int = 4


def spec_c4(B: int = 16, R: int = 4096, E: int = 512, H: int = 2048, blocks: int = 8,
            dtype: str = "bf16") -> MlpSpec:
    return MlpSpec(name=f"c4_mlp_blocks_B{B}_{dtype}", B=B, R=R, E=E, H=H, blocks=blocks, dtype=dtype)


def mlp_param_shapes(spec: MlpSpec) -> List[Tuple[str, Tuple[int, ...]]]:
    """Per-model parameter list in arena order; Linear weights are [Fx, Fy] (baddbmm orientation)."""
    out: List[Tuple[str, Tuple[int, ...]]] = []
    for i in range(spec.blocks):
        out += [(f"blk{i}.w1", (spec.E, spec.H)), (f"blk{i}.b1", (spec.H,)),
                (f"blk{i}.w2", (spec.H, spec.E)), (f"blk{i}.b2", (spec.E,)),
                (f"blk{i}.ln.w", (spec.E,)), (f"blk{i}.ln.b", (spec.E,))]
    return out


def mlp_inputs(spec: MlpSpec, seed: Optional[int] = None, perturb_ln: bool = False) -> Dict[str, object]:
    """tokens, targets: float32 [B, R, E] ~ N(0,1) snapped to spec.dtype; params: list over b of
    dict name -> float32; lr log-uniform, wd uniform, beta = (0.9, 0.999), eps = 1e-8: float32 [B].
    perturb_ln draws the LayerNorm affine around (1, 0) instead of exactly there (tests)."""
    seed = config_seed(spec.config_index) if seed is None else seed
    rngs = model_streams(seed, spec.B)
    x = np.empty((spec.B, spec.R, spec.E), np.float32)
    tg = np.empty_like(x)
    params = []
    lr = np.empty(spec.B, np.float32)
    wd = np.empty(spec.B, np.float32)
    for b, rng in enumerate(rngs):
        x[b] = rng.standard_normal((spec.R, spec.E))
        tg[b] = rng.standard_normal((spec.R, spec.E))
        p = {}
        for name, shp in mlp_param_shapes(spec):
            if name.endswith(".ln.w"):
                p[name] = (1.0 + (0.1 * rng.standard_normal(shp) if perturb_ln else 0.0) * np.ones(shp)).astype(np.float32)
            elif name.endswith(".ln.b"):
                p[name] = ((0.1 * rng.standard_normal(shp) if perturb_ln else 0.0) * np.ones(shp)).astype(np.float32)
            elif len(shp) == 2:
                p[name] = uniform_fan_in(rng, shp, shp[0], 6.0).astype(np.float32)
            else:
                fan_in = spec.E if name.endswith(".b1") else spec.H
                p[name] = uniform_fan_in(rng, shp, fan_in, 1.0).astype(np.float32)
        params.append(p)
        lr[b] = log_uniform(rng, *spec.lr_range)
        wd[b] = rng.uniform(*spec.wd_range)
    sd = "f32" if spec.dtype == "f64" else spec.dtype
    return dict(tokens=snap(x, sd), targets=snap(tg, sd), params=params, lr=lr, wd=wd,
                beta1=np.full(spec.B, 0.9, np.float32), beta2=np.full(spec.B, 0.999, np.float32),
                eps=np.full(spec.B, 1e-8, np.float32))


# --------------------------------------------------------------------------
# DCGAN-style fused array (BASELINE config 3)
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class DcganSpec:
    """B generator/discriminator pairs; layers as (Ci, Co, H_in, stride, pad), 4x4 kernels."""
    name: str
    B: int
    Nb: int                          # images per model per step
    g_layers: Tuple[Tuple[int, int, int, int, int], ...]
    d_layers: Tuple[Tuple[int, int, int, int, int], ...]
    dtype: str
    lr_range: Tuple[float, float] = (1e-4, 5e-4)
    config_index: int = 3


def spec_c3(B: int = 10, Nb: int = 64, dtype: str = "bf16") -> DcganSpec:
    return DcganSpec(name=f"c3_dcgan_B{B}_{dtype}", B=B, Nb=Nb, g_layers=DCGAN_G_LAYERS,
                     d_layers=DCGAN_D_LAYERS, dtype=dtype)


def dcgan_thin(B: int, Nb: int, dtype: str, div: int = 16, cz: int = 12) -> DcganSpec:
    """The same 64x64 architecture with every channel count divided by `div` (tests)."""
    g = tuple((cz if i == 0 else max(ci // div, 2), co if i == 4 else max(co // div, 2), h, s, p)
              for i, (ci, co, h, s, p) in enumerate(DCGAN_G_LAYERS))
    d = tuple((ci if i == 0 else max(ci // div, 2), co if i == 4 else max(co // div, 2), h, s, p)
              for i, (ci, co, h, s, p) in enumerate(DCGAN_D_LAYERS))
    return DcganSpec(name=f"dcgan_thin{div}_B{B}_{dtype}", B=B, Nb=Nb, g_layers=g, d_layers=d, dtype=dtype)


def dcgan_param_shapes(spec: DcganSpec):
    """(generator list, discriminator list) of (name, shape) per model, arena order.
    ConvTranspose weights are [Cin, Cout, 4, 4], Conv weights [Cout, Cin, 4, 4]."""
    g, d = [], []
    for i, (ci, co, _, _, _) in enumerate(spec.g_layers):
        g.append((f"g{i}.w", (ci, co, 4, 4)))
        if i < len(spec.g_layers) - 1:
            g += [(f"g{i}.bn.g", (co,)), (f"g{i}.bn.b", (co,))]
    for i, (ci, co, _, _, _) in enumerate(spec.d_layers):
        d.append((f"d{i}.w", (co, ci, 4, 4)))
        if 0 < i < len(spec.d_layers) - 1:
            d += [(f"d{i}.bn.g", (co,)), (f"d{i}.bn.b", (co,))]
    return g, d


def dcgan_inputs(spec: DcganSpec, seed: Optional[int] = None) -> Dict[str, object]:
    """z: float32 [Nb, B*Cz, 1, 1] ~ N(0,1); real: [Nb, B*3, 64, 64] ~ U(-1,1) (both snapped to the
    storage dtype); gparams / dparams: lists over b of dict name -> float32 (weights N(0, 0.02^2),
    BatchNorm scale N(1, 0.02^2), shift 0); lr log-uniform per model, beta = (0.5, 0.999), eps 1e-8, wd 0."""
    seed = config_seed(spec.config_index) if seed is None else seed
    rngs = model_streams(seed, spec.B)
    cz = spec.g_layers[0][0]
    H = spec.d_layers[0][2]
    z = np.empty((spec.Nb, spec.B * cz, 1, 1), np.float32)
    real = np.empty((spec.Nb, spec.B * 3, H, H), np.float32)
    gsh, dsh = dcgan_param_shapes(spec)
    gparams, dparams = [], []
    lr = np.empty(spec.B, np.float32)
    for b, rng in enumerate(rngs):
        z[:, cz * b:cz * (b + 1)] = rng.standard_normal((spec.Nb, cz, 1, 1))
        real[:, 3 * b:3 * b + 3] = rng.uniform(-1.0, 1.0, (spec.Nb, 3, H, H))
        for shapes, out in ((gsh, gparams), (dsh, dparams)):
            p = {}
            for name, shp in shapes:
                if name.endswith(".bn.g"):
                    p[name] = (1.0 + 0.02 * rng.standard_normal(shp)).astype(np.float32)
                elif name.endswith(".bn.b"):
                    p[name] = np.zeros(shp, np.float32)
                else:
                    p[name] = (0.02 * rng.standard_normal(shp)).astype(np.float32)
            out.append(p)
        lr[b] = log_uniform(rng, *spec.lr_range)
    sd = "f32" if spec.dtype == "f64" else spec.dtype
    return dict(z=snap(z, sd), real=snap(real, sd), gparams=gparams, dparams=dparams, lr=lr,
                beta1=np.full(spec.B, 0.5, np.float32), beta2=np.full(spec.B, 0.999, np.float32),
                eps=np.full(spec.B, 1e-8, np.float32), wd=np.zeros(spec.B, np.float32))
