"""Full-size synthetic inputs drawn directly in GPU memory (torch's seeded CUDA generator).

Same shapes, layouts and distributions as the numpy generators of this package, for the sizes
where drawing on the host would take minutes (the 12-layer, 32-model encoder stack holds 2.7 G
weights).  No operator arithmetic here: only random draws, and a cast to the storage dtype.
Tests that need host copies of what was drawn copy the slices back from the device.
"""
from __future__ import annotations

from typing import Dict

import torch

from . import BASE_SEED, EncoderShape, ResNetSpec


def _gen(cfg: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(BASE_SEED + 1000 * cfg)
    return g


def _normal(g, shape, mean, std, dtype, device):
    t = torch.empty(shape, dtype=torch.float32, device=device)
    t.normal_(mean, std, generator=g)
    return t.to(dtype)


def encoder_stack_device(M: int, shape: EncoderShape, cfg: int = 5, dtype=torch.bfloat16,
                         device="cuda") -> Dict[str, object]:
    """X[M, batch*seq, hidden] ~ N(0,1); matrices ~ N(0,0.02) in ``dtype``; biases ~ N(0,0.02) and
    LayerNorm gamma ~ 1+N(0,0.02), beta ~ N(0,0.02) in float32 (values on the bf16 grid)."""
    g = _gen(cfg, device)
    Hd, F, N = shape.hidden, shape.ffn, shape.batch * shape.seq
    f32 = lambda t: t.to(torch.float32)
    X = _normal(g, (M, N, Hd), 0.0, 1.0, dtype, device)
    layers = []
    for _ in range(shape.layers):
        layers.append(dict(
            Wqkv=_normal(g, (M, Hd, 3 * Hd), 0.0, 0.02, dtype, device),
            bqkv=f32(_normal(g, (M, 3 * Hd), 0.0, 0.02, dtype, device)),
            Wo=_normal(g, (M, Hd, Hd), 0.0, 0.02, dtype, device),
            bo=f32(_normal(g, (M, Hd), 0.0, 0.02, dtype, device)),
            ln1_g=f32(_normal(g, (M * Hd,), 1.0, 0.02, dtype, device)),
            ln1_b=f32(_normal(g, (M * Hd,), 0.0, 0.02, dtype, device)),
            W1=_normal(g, (M, Hd, F), 0.0, 0.02, dtype, device),
            b1=f32(_normal(g, (M, F), 0.0, 0.02, dtype, device)),
            W2=_normal(g, (M, F, Hd), 0.0, 0.02, dtype, device),
            b2=f32(_normal(g, (M, Hd), 0.0, 0.02, dtype, device)),
            ln2_g=f32(_normal(g, (M * Hd,), 1.0, 0.02, dtype, device)),
            ln2_b=f32(_normal(g, (M * Hd,), 0.0, 0.02, dtype, device)),
        ))
    return {"X": X, "layers": layers}


def resnet_params_device(spec: ResNetSpec, M: int, cfg: int = 3, dtype=torch.bfloat16,
                         device="cuda") -> Dict[str, object]:
    """x[1, M*3, image, image] ~ N(0,1); conv weights Kaiming-normal std = sqrt(2/(cig k k));
    BatchNorm gamma ~ 1+N(0,0.02), beta ~ N(0,0.02), mean ~ N(0,0.1), var ~ U(0.5,1.5), float32."""
    g = _gen(cfg, device)
    x = _normal(g, (1, M * 3, spec.image, spec.image), 0.0, 1.0, dtype, device)
    params = {}
    for c in spec.convs():
        cig = c.cin // c.groups
        std = (2.0 / (cig * c.k * c.k)) ** 0.5
        n = M * c.cout
        var = torch.empty(n, dtype=torch.float32, device=device).uniform_(0.5, 1.5, generator=g)
        params[c.name] = dict(
            w=_normal(g, (n, cig, c.k, c.k), 0.0, std, dtype, device),
            gamma=_normal(g, (n,), 1.0, 0.02, torch.float32, device),
            beta=_normal(g, (n,), 0.0, 0.02, torch.float32, device),
            mean=_normal(g, (n,), 0.0, 0.1, torch.float32, device),
            var=var)
    return {"x": x, "params": params}
