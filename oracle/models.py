"""Whole-workload oracles: the merged operators of ``oracle`` chained in the order the
workloads define.  TEST INFRASTRUCTURE ONLY (same rules as the package header).

Each function rounds to bf16 only where one operator call ends (``out_bf16``), which is
where a bf16-storage implementation writes an activation tensor.
"""
from __future__ import annotations

import numpy as np

import oracle as O


def tiny_layer(inp, M, out_bf16=False):
    """Workload 1: batch-merged linear -> per-model LayerNorm (the two-layer network of
    Section 3.2's example), plus the merged 3x3 convolution on its own input."""
    Y = O.linear(inp["X"], inp["W"], bias=inp["b"], out_bf16=out_bf16)
    Z = O.layernorm(Y, inp["gamma"], inp["beta"], M, eps=1e-5, out_bf16=out_bf16)
    C = O.conv2d(inp["conv_x"], inp["conv_w"], M, g=1, stride=1, pad=1, out_bf16=out_bf16)
    return {"linear": Y, "layernorm": Z, "conv": C}


def encoder_layer(X, Lw, M, batch, seq, heads, eps=1e-5, out_bf16=True, trace=None, R=None):
    """One post-LN encoder layer on X[M, batch*seq, hidden]:
    QKV = X Wqkv + b;  A = attention(QKV);  X1 = LN(A Wo + bo + X);
    F = GELU(X1 W1 + b1) W2 + b2;  X2 = LN(F + X1).
    With R (the relative position encodings [2 seq, hidden]) the attention is the relative-position one:
    Kr_m = R Wr_m, query biases rwb_m, rrb_m."""
    qkv = O.linear(X, Lw["Wqkv"], bias=Lw["bqkv"], out_bf16=out_bf16)
    if R is None:
        att = O.attention_packed(qkv, batch, seq, heads, out_bf16=out_bf16)
    else:
        kr = O.linear(np.broadcast_to(R, (M,) + R.shape).copy(), Lw["Wr"], out_bf16=out_bf16)
        att = O.attention_relpos_packed(qkv, kr, batch, seq, heads, bias_w=Lw["rwb"], bias_r=Lw["rrb"], out_bf16=out_bf16)
    h = O.linear(att, Lw["Wo"], bias=Lw["bo"], residual=X, out_bf16=out_bf16)
    x1 = O.layernorm(h, Lw["ln1_g"], Lw["ln1_b"], M, eps=eps, out_bf16=out_bf16)
    f1 = O.linear(x1, Lw["W1"], bias=Lw["b1"], act=O.ACT_GELU, out_bf16=out_bf16)
    f2 = O.linear(f1, Lw["W2"], bias=Lw["b2"], residual=x1, out_bf16=out_bf16)
    x2 = O.layernorm(f2, Lw["ln2_g"], Lw["ln2_b"], M, eps=eps, out_bf16=out_bf16)
    if trace is not None:
        trace.append(dict(qkv=qkv, att=att, h=h, x1=x1, f1=f1, f2=f2, x2=x2) | ({} if R is None else {"kr": kr}))
    return x2


def encoder_stack(inp, M, batch, seq, heads, eps=1e-5, out_bf16=True, trace=None):
    X = inp["X"]
    for Lw in inp["layers"]:
        X = encoder_layer(X, Lw, M, batch, seq, heads, eps=eps, out_bf16=out_bf16, trace=trace, R=inp.get("R"))
    return X


def _conv_bn(x, spec, p, M, act, residual=None, eps=1e-5, out_bf16=True):
    scale, shift = O.bn_fold(p["gamma"], p["beta"], p["mean"], p["var"], eps=eps)
    return O.conv2d(x, p["w"], M, g=spec.groups, scale=scale, shift=shift, residual=residual,
                    stride=spec.stride, pad=spec.pad, act=act, out_bf16=out_bf16)


def resnet_forward(inp, spec, M, eps=1e-5, out_bf16=True, trace=None):
    """Bottleneck ResNet / ResNeXt forward on x[1, M*3, image, image] -> [1, M*C_last]:
    stem conv+BN+ReLU, max-pool 3x3/2 pad 1, bottleneck blocks (conv+BN+ReLU, conv+BN+ReLU,
    conv+BN, + shortcut, ReLU), global average pool.  BatchNorm (inference) enters each conv call
    as its per-channel scale/shift; no classifier."""
    P = inp["params"]

    def rec(name, t):
        if trace is not None:
            trace[name] = t
        return t

    x = rec("stem", _conv_bn(inp["x"], spec.stem, P["stem"], M, O.ACT_RELU, eps=eps, out_bf16=out_bf16))
    x = rec("maxpool", O.maxpool2d(x, 3, 2, 1, out_bf16=out_bf16))
    for blk in spec.blocks:
        a = rec(blk.conv1.name, _conv_bn(x, blk.conv1, P[blk.conv1.name], M, O.ACT_RELU, eps=eps, out_bf16=out_bf16))
        b = rec(blk.conv2.name, _conv_bn(a, blk.conv2, P[blk.conv2.name], M, O.ACT_RELU, eps=eps, out_bf16=out_bf16))
        if blk.down is not None:
            sc = rec(blk.down.name, _conv_bn(x, blk.down, P[blk.down.name], M, O.ACT_NONE, eps=eps, out_bf16=out_bf16))
        else:
            sc = x
        x = rec(blk.conv3.name, _conv_bn(b, blk.conv3, P[blk.conv3.name], M, O.ACT_RELU, residual=sc, eps=eps, out_bf16=out_bf16))
    return rec("avgpool", O.avgpool_global(x, out_bf16=out_bf16))
