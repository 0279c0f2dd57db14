"""Seeded synthetic inputs for the merged-operator workloads.

This module is the ONLY code shared by the CPU oracle's tests and the GPU path's
tests/bench.  It holds no operator arithmetic: it draws random tensors with the
shapes and distributions of the five workloads, describes the layer shapes of the
networks those workloads are built from, and converts between float32 and bf16
bit patterns (storage conversion of inputs, not part of any operator).

Seeding: model ``m`` of workload ``cfg`` draws everything from its own
``numpy.random.Generator(PCG64(20091306 + 1000*cfg + m))`` in a fixed order, and
merged tensors are the per-model tensors concatenated in model order -- so
permuting the models of a merged input is exactly a re-ordering of slices.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

BASE_SEED = 20091306


def model_rng(cfg: int, m: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * cfg + m))


# ----------------------------------------------------------------------------- bf16 storage
def bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> uint16 bf16 bit patterns, round to nearest, ties to even (NaN kept NaN)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        r[nan] = np.uint16(0x7FC0)
    return r


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float32 (exact)."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def on_bf16_grid(a: np.ndarray) -> np.ndarray:
    """float32 values rounded to the nearest bf16, returned as float32."""
    return bf16_to_f32(bf16_bits(a)).reshape(np.shape(a))


def _store(a: np.ndarray, bf16: bool) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return on_bf16_grid(a) if bf16 else a


def _normal(rng, shape, mean=0.0, std=1.0):
    return (mean + std * rng.standard_normal(shape)).astype(np.float32)


# ----------------------------------------------------------------------------- workload 1
def tiny_layer(M: int = 2, cfg: int = 1, bf16: bool = False, order: Optional[List[int]] = None
               ) -> Dict[str, np.ndarray]:
    """Workload 1: linear 64->64 on [8,64] rows, per-model LayerNorm, then a 3x3 conv (own input).

    ``order`` lists which model seeds occupy slices 0..M-1 (default identity) -- used by the
    model-permutation tests.
    """
    order = list(range(M)) if order is None else list(order)
    per = []
    for m in order:
        r = model_rng(cfg, m)
        per.append(dict(
            X=_normal(r, (8, 64)),
            W=_normal(r, (64, 64), 0.0, 0.02),
            b=_normal(r, (64,), 0.0, 0.02),
            gamma=_normal(r, (64,), 1.0, 0.02),
            beta=_normal(r, (64,), 0.0, 0.02),
            conv_x=_normal(r, (16, 8, 8)),
            conv_w=_normal(r, (16, 16, 3, 3), 0.0, 0.05),
        ))
    out = dict(
        X=np.stack([p["X"] for p in per]),                       # [M, 8, 64]
        W=np.stack([p["W"] for p in per]),                       # [M, 64, 64]
        b=np.stack([p["b"] for p in per]),                       # [M, 64]
        gamma=np.concatenate([p["gamma"] for p in per]),         # [M*64]
        beta=np.concatenate([p["beta"] for p in per]),           # [M*64]
        conv_x=np.concatenate([p["conv_x"] for p in per])[None], # [1, M*16, 8, 8]
        conv_w=np.concatenate([p["conv_w"] for p in per]),       # [M*16, 16, 3, 3]
    )
    return {k: _store(v, bf16) for k, v in out.items()}


# ----------------------------------------------------------------------------- workloads 2 and 5
@dataclass(frozen=True)
class EncoderShape:
    hidden: int = 768
    heads: int = 12
    ffn: int = 3072
    layers: int = 1
    seq: int = 128
    batch: int = 1          # sequences per model

    @property
    def head_dim(self) -> int:
        return self.hidden // self.heads


ENCODER_LAYER_KEYS = ("Wqkv", "bqkv", "Wo", "bo", "ln1_g", "ln1_b", "W1", "b1", "W2", "b2",
                      "ln2_g", "ln2_b")


def relative_positions(seq: int, hidden: int) -> np.ndarray:
    """The sinusoid encodings of the relative distances seq, seq-1, ..., -seq+1 (an input tensor of the
    relative-position attention, shared by all models): row p = [sin(pos f_0..), cos(pos f_0..)] for
    pos = seq - p and f_i = 10000^(-2i/hidden)."""
    pos = np.arange(seq, -seq, -1, dtype=np.float64)
    inv = 1.0 / (10000.0 ** (np.arange(0, hidden, 2, dtype=np.float64) / hidden))
    ang = pos[:, None] * inv[None, :]
    return np.concatenate([np.sin(ang), np.cos(ang)], axis=1).astype(np.float32)


def encoder_stack(M: int, shape: EncoderShape, cfg: int = 2, bf16: bool = True,
                  order: Optional[List[int]] = None, rel: bool = False) -> Dict[str, object]:
    """Post-LN encoder layers: X[M, batch*seq, hidden] ~ N(0,1); weights/biases ~ N(0,0.02);
    LayerNorm gamma ~ 1+N(0,0.02), beta ~ N(0,0.02).  Returns {"X":..., "layers":[{key: merged}]}.
    Wqkv has column blocks [Q | K | V].  rel: also the parameters of relative-position attention per layer
    (position projection Wr[hidden, hidden], query biases rwb, rrb ~ N(0,0.02)) and "R" = relative_positions."""
    order = list(range(M)) if order is None else list(order)
    Hd, F = shape.hidden, shape.ffn
    xs, per_layer = [], [dict((k, []) for k in ENCODER_LAYER_KEYS) for _ in range(shape.layers)]
    for m in order:
        r = model_rng(cfg, m)
        xs.append(_normal(r, (shape.batch * shape.seq, Hd)))
        for L in range(shape.layers):
            d = per_layer[L]
            d["Wqkv"].append(_normal(r, (Hd, 3 * Hd), 0.0, 0.02))
            d["bqkv"].append(_normal(r, (3 * Hd,), 0.0, 0.02))
            d["Wo"].append(_normal(r, (Hd, Hd), 0.0, 0.02))
            d["bo"].append(_normal(r, (Hd,), 0.0, 0.02))
            d["ln1_g"].append(_normal(r, (Hd,), 1.0, 0.02))
            d["ln1_b"].append(_normal(r, (Hd,), 0.0, 0.02))
            d["W1"].append(_normal(r, (Hd, F), 0.0, 0.02))
            d["b1"].append(_normal(r, (F,), 0.0, 0.02))
            d["W2"].append(_normal(r, (F, Hd), 0.0, 0.02))
            d["b2"].append(_normal(r, (Hd,), 0.0, 0.02))
            d["ln2_g"].append(_normal(r, (Hd,), 1.0, 0.02))
            d["ln2_b"].append(_normal(r, (Hd,), 0.0, 0.02))
            if rel:                                    # relative-position attention: drawn last, so the rest is unchanged
                d.setdefault("Wr", []).append(_normal(r, (Hd, Hd), 0.0, 0.02))
                d.setdefault("rwb", []).append(_normal(r, (Hd,), 0.0, 0.02))
                d.setdefault("rrb", []).append(_normal(r, (Hd,), 0.0, 0.02))
    layers = []
    for d in per_layer:
        merged = {}
        for k, lst in d.items():
            a = np.concatenate(lst) if k.startswith("ln") else np.stack(lst)
            merged[k] = _store(a, bf16)
        layers.append(merged)
    out = {"X": _store(np.stack(xs), bf16), "layers": layers}
    if rel:
        out["R"] = _store(relative_positions(shape.seq, Hd), bf16)
    return out


# ----------------------------------------------------------------------------- workloads 3 and 4
@dataclass(frozen=True)
class ConvSpec:
    name: str
    cin: int            # per-model input channels
    cout: int           # per-model output channels
    k: int
    stride: int
    pad: int
    groups: int         # per-model groups g (merged groups = M*g)
    relu: bool          # ReLU directly after this conv's BatchNorm (before any residual add: no)


@dataclass(frozen=True)
class BottleneckSpec:
    conv1: ConvSpec
    conv2: ConvSpec
    conv3: ConvSpec
    down: Optional[ConvSpec]     # projection shortcut (first block of a stage) or None


@dataclass(frozen=True)
class ResNetSpec:
    image: int
    stem: ConvSpec
    blocks: List[BottleneckSpec] = field(default_factory=list)

    def convs(self) -> List[ConvSpec]:
        out = [self.stem]
        for b in self.blocks:
            out += [b.conv1, b.conv2, b.conv3] + ([b.down] if b.down else [])
        return out

    @property
    def out_channels(self) -> int:
        return self.blocks[-1].conv3.cout


def resnet_spec(cardinality: int = 1, base_width: int = 64, image: int = 224, width_div: int = 1,
                depths=(3, 4, 6, 3)) -> ResNetSpec:
    """Bottleneck ResNet: stem 7x7/2 + max-pool 3x3/2, stages of [1x1, 3x3, 1x1] blocks with the
    stride on the 3x3 conv of a stage's first block and a 1x1 projection shortcut there.
    ResNet-50: cardinality 1, base_width 64.  ResNeXt-50 32x4d: cardinality 32, base_width 4.
    ``width_div``/``image``/``depths`` shrink the network for tests (channel counts divided)."""
    c0 = 64 // width_div
    stem = ConvSpec("stem", 3, c0, 7, 2, 3, 1, True)
    blocks, inplanes = [], c0
    for si, (planes_full, nblk) in enumerate(zip((64, 128, 256, 512), depths)):
        planes = planes_full // width_div
        width = int(planes * (base_width / 64.0)) * cardinality
        stage_stride = 1 if si == 0 else 2
        for j in range(nblk):
            s = stage_stride if j == 0 else 1
            nm = "s%db%d" % (si + 1, j)
            c1 = ConvSpec(nm + ".conv1", inplanes, width, 1, 1, 0, 1, True)
            c2 = ConvSpec(nm + ".conv2", width, width, 3, s, 1, cardinality, True)
            c3 = ConvSpec(nm + ".conv3", width, planes * 4, 1, 1, 0, 1, False)
            dn = ConvSpec(nm + ".down", inplanes, planes * 4, 1, s, 0, 1, False) if j == 0 else None
            blocks.append(BottleneckSpec(c1, c2, c3, dn))
            inplanes = planes * 4
    return ResNetSpec(image, stem, blocks)


def resnet_params(spec: ResNetSpec, M: int, cfg: int = 3, bf16: bool = True,
                  order: Optional[List[int]] = None, batch: int = 1) -> Dict[str, object]:
    """x[batch, M*3, image, image] ~ N(0,1) (model m's ``batch`` images are its first draw, so batch 1
    reproduces the single-image inputs).  Per conv: Kaiming-normal weight, std = sqrt(2/(cig*k*k));
    BatchNorm gamma ~ 1+N(0,0.02), beta ~ N(0,0.02), running mean ~ N(0,0.1), var ~ U(0.5,1.5).
    BatchNorm vectors stay float32 (they are per-channel constants, not activations)."""
    order = list(range(M)) if order is None else list(order)
    convs = spec.convs()
    xs = []
    acc = {c.name: dict(w=[], gamma=[], beta=[], mean=[], var=[]) for c in convs}
    for m in order:
        r = model_rng(cfg, m)
        xs.append(_normal(r, (batch, 3, spec.image, spec.image)))
        for c in convs:
            cig = c.cin // c.groups
            std = float(np.sqrt(2.0 / (cig * c.k * c.k)))
            a = acc[c.name]
            a["w"].append(_normal(r, (c.cout, cig, c.k, c.k), 0.0, std))
            a["gamma"].append(_normal(r, (c.cout,), 1.0, 0.02))
            a["beta"].append(_normal(r, (c.cout,), 0.0, 0.02))
            a["mean"].append(_normal(r, (c.cout,), 0.0, 0.1))
            a["var"].append(r.uniform(0.5, 1.5, (c.cout,)).astype(np.float32))
    params = {}
    for c in convs:
        a = acc[c.name]
        params[c.name] = dict(
            w=_store(np.concatenate(a["w"]), bf16),
            gamma=np.concatenate(a["gamma"]), beta=np.concatenate(a["beta"]),
            mean=np.concatenate(a["mean"]), var=np.concatenate(a["var"]))
    return {"x": _store(np.concatenate(xs, axis=1), bf16), "params": params}
