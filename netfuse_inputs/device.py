"""Full-size synthetic inputs drawn directly in GPU memory (torch's seeded CUDA generator).

Same shapes, layouts and distributions as the numpy generators of this package, for the sizes
where drawing on the host would take minutes (the 12-layer, 32-model encoder stack holds 2.7 G
weights).  Seeding follows the same rule as the host generators: model ``m`` of workload ``cfg``
draws everything from its own generator seeded ``BASE_SEED + 1000*cfg + m`` in a fixed order into
its own slice of the merged tensors, so permuting the models is a re-ordering of slices (the
values differ from the numpy generators': the two random streams are different algorithms).
No operator arithmetic here: only random draws, and a cast to the storage dtype.
Tests that need host copies of what was drawn copy the slices back from the device.
"""
from __future__ import annotations

from typing import Dict

import torch

from . import BASE_SEED, EncoderShape, ResNetSpec


def _gen(cfg: int, m: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(BASE_SEED + 1000 * cfg + m)
    return g


def _fill(dst: torch.Tensor, g, mean, std):
    """dst (a slice of a merged tensor, any dtype) <- N(mean, std) drawn in float32, cast on store."""
    if dst.dtype == torch.float32 and dst.is_contiguous():
        dst.normal_(mean, std, generator=g)
    else:
        t = torch.empty(dst.shape, dtype=torch.float32, device=dst.device)
        t.normal_(mean, std, generator=g)
        dst.copy_(t)


def encoder_stack_device(M: int, shape: EncoderShape, cfg: int = 5, dtype=torch.bfloat16,
                         device="cuda", rel: bool = False) -> Dict[str, object]:
    """X[M, batch*seq, hidden] ~ N(0,1); matrices ~ N(0,0.02) in ``dtype``; biases ~ N(0,0.02) and
    LayerNorm gamma ~ 1+N(0,0.02), beta ~ N(0,0.02) in float32 (values on the bf16 grid)."""
    Hd, F, N = shape.hidden, shape.ffn, shape.batch * shape.seq
    e = lambda *s, dt=dtype: torch.empty(s, dtype=dt, device=device)
    X = e(M, N, Hd)
    layers = [dict(Wqkv=e(M, Hd, 3 * Hd), bqkv=e(M, 3 * Hd), Wo=e(M, Hd, Hd), bo=e(M, Hd), ln1_g=e(M * Hd),
                   ln1_b=e(M * Hd), W1=e(M, Hd, F), b1=e(M, F), W2=e(M, F, Hd), b2=e(M, Hd), ln2_g=e(M * Hd),
                   ln2_b=e(M * Hd)) for _ in range(shape.layers)]
    for m in range(M):
        g = _gen(cfg, m, device)
        _fill(X[m], g, 0.0, 1.0)
        for L in layers:
            for k in ("Wqkv", "bqkv", "Wo", "bo"):
                _fill(L[k][m], g, 0.0, 0.02)
            _fill(L["ln1_g"][m * Hd:(m + 1) * Hd], g, 1.0, 0.02)
            _fill(L["ln1_b"][m * Hd:(m + 1) * Hd], g, 0.0, 0.02)
            for k in ("W1", "b1", "W2", "b2"):
                _fill(L[k][m], g, 0.0, 0.02)
            _fill(L["ln2_g"][m * Hd:(m + 1) * Hd], g, 1.0, 0.02)
            _fill(L["ln2_b"][m * Hd:(m + 1) * Hd], g, 0.0, 0.02)
            if rel:
                for k, shp in (("Wr", (M, Hd, Hd)), ("rwb", (M, Hd)), ("rrb", (M, Hd))):
                    if k not in L:
                        L[k] = e(*shp)
                    _fill(L[k][m], g, 0.0, 0.02)
    for L in layers:                      # per-feature vectors are float32 operands (values on the storage grid)
        for k in ("bqkv", "bo", "ln1_g", "ln1_b", "b1", "b2", "ln2_g", "ln2_b") + (("rwb", "rrb") if rel else ()):
            L[k] = L[k].to(torch.float32)
    out = {"X": X, "layers": layers}
    if rel:
        from . import relative_positions
        out["R"] = torch.from_numpy(relative_positions(shape.seq, Hd)).to(device=device, dtype=dtype)
    return out


def resnet_params_device(spec: ResNetSpec, M: int, cfg: int = 3, dtype=torch.bfloat16,
                         device="cuda", batch: int = 1) -> Dict[str, object]:
    """x[batch, M*3, image, image] ~ N(0,1); conv weights Kaiming-normal std = sqrt(2/(cig k k));
    BatchNorm gamma ~ 1+N(0,0.02), beta ~ N(0,0.02), mean ~ N(0,0.1), var ~ U(0.5,1.5), float32."""
    x = torch.empty((batch, M * 3, spec.image, spec.image), dtype=dtype, device=device)
    f32 = lambda n: torch.empty(n, dtype=torch.float32, device=device)
    params = {}
    for c in spec.convs():
        n = M * c.cout
        params[c.name] = dict(w=torch.empty((n, c.cin // c.groups, c.k, c.k), dtype=dtype, device=device),
                              gamma=f32(n), beta=f32(n), mean=f32(n), var=f32(n))
    for m in range(M):
        g = _gen(cfg, m, device)
        _fill(x[:, 3 * m:3 * (m + 1)], g, 0.0, 1.0)
        for c in spec.convs():
            cig = c.cin // c.groups
            std = (2.0 / (cig * c.k * c.k)) ** 0.5
            sl = slice(m * c.cout, (m + 1) * c.cout)
            p = params[c.name]
            _fill(p["w"][sl], g, 0.0, std)
            _fill(p["gamma"][sl], g, 1.0, 0.02)
            _fill(p["beta"][sl], g, 0.0, 0.02)
            _fill(p["mean"][sl], g, 0.0, 0.1)
            p["var"][sl].uniform_(0.5, 1.5, generator=g)
    return {"x": x, "params": params}
