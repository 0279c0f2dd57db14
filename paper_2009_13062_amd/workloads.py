"""The op sequences of the five workloads, expressed as calls into the merged-operator library.

Each class owns its weights (torch CUDA tensors in the merged layouts of include/netfuse.h) and
pre-allocates every activation buffer, so ``forward`` only enqueues kernels on the current
stream: it allocates nothing and can be captured into a HIP graph.  ``per_model()`` returns M
instances of the same class bound to model m's slices with M = 1 -- the same kernels launched
once per model, i.e. the "one model after the other" way of serving that merging replaces
(Section 5.1's Sequential baseline).
"""
from __future__ import annotations

from typing import Dict, List, Optional

import torch

import paper_2009_13062_amd as nf


def to_device(a, dtype: torch.dtype, device="cuda") -> torch.Tensor:
    """numpy float32 array -> contiguous device tensor of the storage dtype."""
    t = torch.from_numpy(a) if not isinstance(a, torch.Tensor) else a
    return t.to(device=device, dtype=dtype).contiguous()


class EncoderStack:
    """Post-LN encoder layers on X[M, batch*seq, hidden] (workloads 2 and 5):
    QKV = X Wqkv + b; A = attention(QKV); X1 = LN(A Wo + bo + X); X2 = LN(GELU(X1 W1 + b1) W2 + b2 + X1)."""

    MATS = ("Wqkv", "Wo", "W1", "W2", "Wr")

    def __init__(self, layers: List[Dict[str, torch.Tensor]], M: int, batch: int, seq: int, heads: int,
                 eps: float = 1e-5, buffers: Optional[Dict[str, torch.Tensor]] = None,
                 R: Optional[torch.Tensor] = None, packed: bool = False):
        """R[2*seq, hidden] (relative position encodings) switches the attention to the relative-position form
        (XLNet-shaped layers): per layer Kr = R Wr (one more merged matmul) and the query biases rwb, rrb.
        packed: re-lay the weight matrices out once (netfuse_linear_pack_weight) and run the matmuls that have a
        packed kernel through netfuse_linear_packed; the packed copies are kept beside the originals under
        the key + "_p"."""
        self.layers, self.M, self.batch, self.seq, self.heads, self.eps = layers, M, batch, seq, heads, eps
        self.R = R
        self.packed = packed
        if packed:
            for Lw in layers:
                for k in self.MATS:
                    if k in Lw and k + "_p" not in Lw:
                        rows = 2 * seq if k == "Wr" else batch * seq
                        if nf.linear_packed_supported(M, rows, Lw[k].shape[1], Lw[k].shape[2], Lw[k].dtype):
                            Lw[k + "_p"] = nf.linear_pack_weight(Lw[k])
        W = layers[0]
        self.hidden, self.ffn = W["Wqkv"].shape[1], W["W1"].shape[2]
        N, Hd, F = batch * seq, self.hidden, self.ffn
        dt, dev = W["Wqkv"].dtype, W["Wqkv"].device
        if buffers is None:
            e = lambda *s: torch.empty(s, dtype=dt, device=dev)
            buffers = dict(qkv=e(M, N, 3 * Hd), att=e(M, N, Hd), h=e(M, N, Hd), x1=e(M, N, Hd),
                           f1=e(M, N, F), f2=e(M, N, Hd), xa=e(M, N, Hd), xb=e(M, N, Hd))
            if R is not None:
                buffers["kr"] = e(M, 2 * seq, Hd)
                buffers["Rrep"] = R.unsqueeze(0).expand(M, -1, -1).contiguous()      # the shared encodings, once per model
        self.buf = buffers

    @classmethod
    def from_numpy(cls, inp, M, batch, seq, heads, dtype=torch.bfloat16, eps=1e-5, packed=False):
        layers = []
        for Lw in inp["layers"]:
            layers.append({k: to_device(v, dtype if k in cls.MATS else torch.float32) for k, v in Lw.items()})
        R = to_device(inp["R"], dtype) if "R" in inp else None
        return cls(layers, M, batch, seq, heads, eps, R=R, packed=packed)

    def _linear(self, X, Lw, key, **kw):
        if self.packed and key + "_p" in Lw:
            return nf.linear_packed(X, Lw[key + "_p"], **kw)
        return nf.linear(X, Lw[key], **kw)

    def layer(self, X, Lw, out, trace=None):
        b, M = self.buf, self.M
        self._linear(X, Lw, "Wqkv", bias=Lw["bqkv"], out=b["qkv"])
        if self.R is None:
            nf.attention_packed(b["qkv"], self.batch, self.seq, self.heads, out=b["att"])
        else:
            self._linear(b["Rrep"], Lw, "Wr", out=b["kr"])
            nf.attention_relpos_packed(b["qkv"], b["kr"], self.batch, self.seq, self.heads, bias_w=Lw["rwb"],
                                       bias_r=Lw["rrb"], out=b["att"])
        self._linear(b["att"], Lw, "Wo", bias=Lw["bo"], residual=X, out=b["h"])
        nf.layernorm(b["h"], Lw["ln1_g"], Lw["ln1_b"], M, eps=self.eps, out=b["x1"])
        self._linear(b["x1"], Lw, "W1", bias=Lw["b1"], act=nf.ACT_GELU, out=b["f1"])
        self._linear(b["f1"], Lw, "W2", bias=Lw["b2"], residual=b["x1"], out=b["f2"])
        nf.layernorm(b["f2"], Lw["ln2_g"], Lw["ln2_b"], M, eps=self.eps, out=out)
        if trace is not None:
            keys = ("qkv", "att", "h", "x1", "f1", "f2") + (("kr",) if self.R is not None else ())
            trace.append({k: b[k].clone() for k in keys} | {"x2": out.clone()})
        return out

    def forward(self, X, trace=None):
        outs = (self.buf["xa"], self.buf["xb"])
        for i, Lw in enumerate(self.layers):
            X = self.layer(X, Lw, outs[i % 2], trace)
        return X

    def per_model(self, packed: bool = False):
        """One single-model stack per model on slices of the same tensors.  By default they call netfuse_linear
        on the unpacked weights, whose tile rules know about single models."""
        Hd = self.hidden
        out = []
        for m in range(self.M):
            layers = []
            for Lw in self.layers:
                d = {}
                for k, v in Lw.items():
                    d[k] = v[m * Hd:(m + 1) * Hd] if k.startswith("ln") else v[m:m + 1]
                layers.append(d)
            bufs = {k: v[m:m + 1] for k, v in self.buf.items()}
            out.append(EncoderStack(layers, 1, self.batch, self.seq, self.heads, self.eps, bufs, R=self.R,
                                    packed=packed and self.packed))
        return out


def encoder_call_list(layers: int, rel: bool = False):
    """The calls of EncoderStack.forward as data: (entry point, operation, producer of the input, producer of
    the residual -- for the relative-position attention: of its second operand -- or None, activation),
    operations and producers named as in netfuse_inputs.graphs.  rel: the XLNet-shaped stack."""
    out, x = [], "x"
    for L in range(layers):
        p = "l%d." % L
        out += [("linear", p + "qkv", x, None, nf.ACT_NONE)]
        out += [("linear", p + "kr", "r", None, nf.ACT_NONE),
                ("attention_relpos", p + "attention", p + "qkv", p + "kr", nf.ACT_NONE)] if rel else [
                ("attention", p + "attention", p + "qkv", None, nf.ACT_NONE)]
        out += [
                ("linear", p + "o", p + "attention", x, nf.ACT_NONE),
                ("layernorm", p + "ln1", p + "o", None, nf.ACT_NONE),
                ("linear", p + "ffn1", p + "ln1", None, nf.ACT_GELU),
                ("linear", p + "ffn2", p + "ffn1", p + "ln1", nf.ACT_NONE),
                ("layernorm", p + "ln2", p + "ffn2", None, nf.ACT_NONE)]
        x = p + "ln2"
    return out


def resnet_call_list(spec):
    """The calls of ResNetForward.forward as data (see encoder_call_list); every conv2d carries its folded
    batch normalisation."""
    out = [("conv2d", "stem", "x", None, nf.ACT_RELU), ("maxpool2d", "maxpool", "stem", None, nf.ACT_NONE)]
    x = "maxpool"
    for blk in spec.blocks:
        out.append(("conv2d", blk.conv1.name, x, None, nf.ACT_RELU))
        out.append(("conv2d", blk.conv2.name, blk.conv1.name, None, nf.ACT_RELU))
        sc = x
        if blk.down is not None:
            out.append(("conv2d", blk.down.name, x, None, nf.ACT_NONE))
            sc = blk.down.name
        out.append(("conv2d", blk.conv3.name, blk.conv2.name, sc, nf.ACT_RELU))
        x = blk.conv3.name
    out.append(("avgpool_global", "avgpool", x, None, nf.ACT_NONE))
    return out


class ResNetForward:
    """Bottleneck ResNet / ResNeXt forward on x[batch, M*3, image, image] -> [batch, M*C_last]
    (workloads 3, 4; ``batch`` images per model, the models' channels concatenated in every tensor).
    Inference batch norm enters every convolution as its per-channel scale/shift epilogue."""

    def __init__(self, spec, params: Dict[str, Dict[str, torch.Tensor]], M: int, dtype=torch.bfloat16,
                 eps: float = 1e-5, device="cuda", batch: int = 1, _shared=None):
        self.spec, self.M, self.eps, self.batch = spec, M, eps, batch
        self.P = params
        if _shared is not None:
            self.fold, self.buf = _shared
            return
        self.fold = {}
        for c in spec.convs():
            p = params[c.name]
            self.fold[c.name] = nf.bn_fold(p["gamma"], p["beta"], p["mean"], p["var"], eps=eps)
        self.buf = self._buffers(M, batch, dtype, device)

    def _buffers(self, M, batch, dtype, device):
        """Activation buffers, one per op output."""
        spec = self.spec
        self.buf = {}
        e = lambda ch, hw: torch.empty((batch, M * ch, hw, hw), dtype=dtype, device=device)
        hw = nf.conv_out_size(spec.image, 7, 2, 3)
        self.buf["stem"] = e(spec.stem.cout, hw)
        hw = (hw + 2 - 3) // 2 + 1
        self.buf["maxpool"] = e(spec.stem.cout, hw)
        for blk in spec.blocks:
            self.buf[blk.conv1.name] = e(blk.conv1.cout, hw)
            hw2 = nf.conv_out_size(hw, 3, blk.conv2.stride, 1)
            self.buf[blk.conv2.name] = e(blk.conv2.cout, hw2)
            if blk.down is not None:
                self.buf[blk.down.name] = e(blk.down.cout, hw2)
            self.buf[blk.conv3.name] = e(blk.conv3.cout, hw2)
            hw = hw2
        self.buf["avgpool"] = torch.empty((batch, M * spec.out_channels), dtype=dtype, device=device)
        return self.buf

    @classmethod
    def from_numpy(cls, inp, spec, M, dtype=torch.bfloat16, eps=1e-5, batch=1):
        params = {}
        for name, p in inp["params"].items():
            params[name] = {k: to_device(v, dtype if k == "w" else torch.float32) for k, v in p.items()}
        return cls(spec, params, M, dtype, eps, batch=batch)

    def _conv(self, x, c, act, residual=None):
        scale, shift = self.fold[c.name]
        return nf.conv2d(x, self.P[c.name]["w"], self.M, g=c.groups, scale=scale, shift=shift,
                         residual=residual, stride=c.stride, pad=c.pad, act=act, out=self.buf[c.name])

    def forward(self, x):
        s = self.spec
        x = self._conv(x, s.stem, nf.ACT_RELU)
        x = nf.maxpool2d(x, 3, 2, 1, out=self.buf["maxpool"])
        for blk in s.blocks:
            a = self._conv(x, blk.conv1, nf.ACT_RELU)
            b = self._conv(a, blk.conv2, nf.ACT_RELU)
            sc = self._conv(x, blk.down, nf.ACT_NONE) if blk.down is not None else x
            x = self._conv(b, blk.conv3, nf.ACT_RELU, residual=sc)
        return nf.avgpool_global(x, out=self.buf["avgpool"])

    def per_model(self):
        """M single-model instances on model m's weight slices.  With one image per model a model's
        channels of every activation are one contiguous run, so the instances work in place on slices
        of the merged buffers; with more, the batch stride separates them and each instance gets
        buffers of its own."""
        out = []
        M = self.M
        any_buf = next(iter(self.buf.values()))
        for m in range(M):
            P, fold, buf = {}, {}, {}
            for c in self.spec.convs():
                sl = slice(m * c.cout, (m + 1) * c.cout)
                P[c.name] = {"w": self.P[c.name]["w"][sl]}
                fold[c.name] = (self.fold[c.name][0][sl], self.fold[c.name][1][sl])
            one = ResNetForward(self.spec, P, 1, eps=self.eps, batch=self.batch, _shared=(fold, buf))
            if self.batch == 1:
                for k, v in self.buf.items():
                    ch = v.shape[1] // M
                    buf[k] = v[:, m * ch:(m + 1) * ch]
            else:
                one.buf = one._buffers(1, self.batch, any_buf.dtype, any_buf.device)
            out.append(one)
        return out

    def slice_input(self, x, m):
        """Model m's images [batch, 3, H, W] (a copy when the batch stride makes the slice non-contiguous)."""
        return x[:, 3 * m:3 * (m + 1)].contiguous()


class TinyLayer:
    """Workload 1: batch-merged linear -> per-model LayerNorm (Section 3.2's two-layer example),
    and the merged 3x3 convolution on its own input."""

    def __init__(self, inp, M, dtype=torch.float32):
        self.M = M
        self.t = {k: to_device(v, dtype if k in ("X", "W", "conv_x", "conv_w") else torch.float32)
                  for k, v in inp.items()}

    def forward(self):
        t, M = self.t, self.M
        Y = nf.linear(t["X"], t["W"], bias=t["b"])
        Z = nf.layernorm(Y, t["gamma"], t["beta"], M, eps=1e-5)
        C = nf.conv2d(t["conv_x"], t["conv_w"], M, g=1, stride=1, pad=1)
        return {"linear": Y, "layernorm": Z, "conv": C}
