"""CPU oracle for the merged NetFuse operators -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``netfuse_oracle.c`` (plain C loops, double accumulation).
Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package; the GPU library never does, and this
package never imports the GPU library.

All arrays are C-contiguous ``float32`` numpy arrays.  A bf16-storage operator is
modelled by passing inputs that already lie on the bf16 grid and ``out_bf16=True``
(one nearest-even rounding of the result).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "netfuse_oracle.c")
_LIB = os.path.join(_HERE, "libnetfuse_oracle.so")

ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2
LAYOUT_BATCH, LAYOUT_CHANNEL = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (``-O2 -fopenmp``; no fast-math, no reordering flags)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-std=c11", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


_FP = ctypes.POINTER(ctypes.c_float)


def _p(a):
    if a is None:
        return ctypes.cast(None, _FP)
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"], "oracle takes contiguous float32"
    return a.ctypes.data_as(_FP)


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def conv_out_size(n, k, stride, pad, dil=1):
    return (n + 2 * pad - dil * (k - 1) - 1) // stride + 1


def linear(X, W, bias=None, residual=None, act=ACT_NONE, out_bf16=False):
    """Y[m] = act(X[m] @ W[m] + bias[m]) + residual[m];  X[M,N,K]  W[M,K,Nout]."""
    X, W, bias, residual = _f32(X), _f32(W), _f32(bias), _f32(residual)
    M, N, K = X.shape
    assert W.shape[0] == M and W.shape[1] == K
    Nout = W.shape[2]
    Y = np.empty((M, N, Nout), np.float32)
    _load().oracle_linear(_p(X), _p(W), _p(bias), _p(residual), _p(Y),
                          M, N, K, Nout, int(act), int(out_bf16))
    return Y


def linear_ragged(X, Ws, biases=None, act=ACT_NONE, out_bf16=False):
    """Per-model output widths (the unmerged per-task heads of Section 5.1): the plain definition, model by
    model -- Y_m = act(X[m] @ Ws[m] + biases[m]) with Ws[m] of shape [K, nout_m].  Returns the list of Y_m."""
    X = _f32(X)
    out = []
    for m, Wm in enumerate(Ws):
        b = None if biases is None else _f32(biases[m])[None]
        out.append(linear(X[m:m + 1], _f32(Wm)[None], bias=b, act=act, out_bf16=out_bf16)[0])
    return out


def conv2d(x, w, M, g=1, bias=None, scale=None, shift=None, residual=None, stride=1, pad=0,
           dil=1, act=ACT_NONE, out_bf16=False):
    """x[B, M*Cin, H, W], w[M*Cout, Cin/g, KH, KW] -> y[B, M*Cout, Ho, Wo]; groups = M*g."""
    x, w = _f32(x), _f32(w)
    bias, scale, shift, residual = _f32(bias), _f32(scale), _f32(shift), _f32(residual)
    B, Ct, H, Wd = x.shape
    assert Ct % M == 0 and w.shape[0] % M == 0
    Cin, Cout = Ct // M, w.shape[0] // M
    assert Cin % g == 0 and Cout % g == 0 and w.shape[1] == Cin // g
    KH, KW = w.shape[2], w.shape[3]
    Ho, Wo = conv_out_size(H, KH, stride, pad, dil), conv_out_size(Wd, KW, stride, pad, dil)
    assert (scale is None) == (shift is None)
    y = np.empty((B, M * Cout, Ho, Wo), np.float32)
    _load().oracle_conv2d(_p(x), _p(w), _p(bias), _p(scale), _p(shift), _p(residual), _p(y),
                          M, B, Cin, Cout, g, H, Wd, KH, KW, stride, pad, dil, int(act),
                          int(out_bf16))
    return y


def layernorm(x, gamma, beta, M, residual=None, eps=1e-5, layout=LAYOUT_BATCH, out_bf16=False):
    """layout BATCH: x[M, rows, H]; layout CHANNEL: x[rows, M*H].  gamma, beta[M*H]."""
    x, residual, gamma, beta = _f32(x), _f32(residual), _f32(gamma), _f32(beta)
    if layout == LAYOUT_BATCH:
        assert x.shape[0] == M
        rows, H = x.shape[1], x.shape[2]
    else:
        rows, H = x.shape[0], x.shape[1] // M
        assert x.shape[1] == M * H
    assert gamma.size == M * H and beta.size == M * H
    y = np.empty_like(x)
    f = _load().oracle_layernorm
    f.argtypes = [_FP, _FP, _FP, _FP, _FP, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                  ctypes.c_double, ctypes.c_int, ctypes.c_int]
    f(_p(x), _p(residual), _p(gamma), _p(beta), _p(y), M, rows, H, float(eps), int(layout),
      int(out_bf16))
    return y


def batchnorm(x, gamma, beta, mean, var, M, residual=None, eps=1e-5, act=ACT_NONE,
              out_bf16=False):
    """x[B, M*C, ...spatial]; per merged channel inference batch norm, + residual, activation."""
    x, residual = _f32(x), _f32(residual)
    gamma, beta, mean, var = _f32(gamma), _f32(beta), _f32(mean), _f32(var)
    B, Ct = x.shape[0], x.shape[1]
    HW = int(np.prod(x.shape[2:])) if x.ndim > 2 else 1
    y = np.empty_like(x)
    f = _load().oracle_batchnorm
    f.argtypes = [_FP] * 7 + [ctypes.c_int] * 4 + [ctypes.c_double, ctypes.c_int, ctypes.c_int]
    f(_p(x), _p(gamma), _p(beta), _p(mean), _p(var), _p(residual), _p(y), M, B, Ct // M, HW,
      float(eps), int(act), int(out_bf16))
    return y


def bn_fold(gamma, beta, mean, var, eps=1e-5):
    gamma, beta, mean, var = _f32(gamma), _f32(beta), _f32(mean), _f32(var)
    scale, shift = np.empty_like(gamma), np.empty_like(gamma)
    f = _load().oracle_bn_fold
    f.argtypes = [_FP] * 6 + [ctypes.c_int, ctypes.c_double]
    f(_p(gamma), _p(beta), _p(mean), _p(var), _p(scale), _p(shift), gamma.size, float(eps))
    return scale, shift


def attention(Q, K, V, M, B, S, heads, d, stride_m, stride_row, scale, mask=None, out_bf16=False):
    """Q, K, V: float32 arrays (possibly views into one packed buffer, see ``attention_packed``)."""
    assert all(a.dtype == np.float32 for a in (Q, K, V))
    mask = _f32(mask)
    O = np.empty((M, B * S, heads * d), np.float32)
    f = _load().oracle_attention
    f.argtypes = [_FP] * 5 + [ctypes.c_int] * 5 + [ctypes.c_long, ctypes.c_long, ctypes.c_double,
                                                   ctypes.c_int]
    f(Q.ctypes.data_as(_FP), K.ctypes.data_as(_FP), V.ctypes.data_as(_FP), _p(mask), _p(O),
      M, B, S, heads, d, int(stride_m), int(stride_row), float(scale), int(out_bf16))
    return O


def attention_packed(QKV, B, S, heads, scale=None, mask=None, out_bf16=False):
    """QKV[M, B*S, 3*heads*d] with column blocks [Q | K | V]; head h = columns h*d..h*d+d-1 of a block."""
    QKV = _f32(QKV)
    M, N, three_h = QKV.shape
    assert N == B * S and three_h % (3 * heads) == 0
    Hd = three_h // 3
    d = Hd // heads
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    flat = QKV.reshape(-1)
    return attention(flat, flat[Hd:], flat[2 * Hd:], M, B, S, heads, d, N * three_h, three_h,
                     scale, mask=mask, out_bf16=out_bf16)


def maxpool2d(x, k, stride, pad, out_bf16=False):
    x = _f32(x)
    B, Ct, H, Wd = x.shape
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (Wd + 2 * pad - k) // stride + 1
    y = np.empty((B, Ct, Ho, Wo), np.float32)
    _load().oracle_maxpool2d(_p(x), _p(y), B, Ct, H, Wd, k, stride, pad, int(out_bf16))
    return y


def avgpool_global(x, out_bf16=False):
    x = _f32(x)
    B, Ct = x.shape[0], x.shape[1]
    HW = int(np.prod(x.shape[2:]))
    y = np.empty((B, Ct), np.float32)
    _load().oracle_avgpool_global(_p(x), _p(y), B, Ct, HW, int(out_bf16))
    return y


def merge_transpose(src, M, to_channel):
    """to_channel: src[M, rows, H] -> dst[rows, M*H]; else the inverse."""
    src = _f32(src)
    if to_channel:
        _, rows, H = src.shape
        dst = np.empty((rows, M * H), np.float32)
    else:
        rows, H = src.shape[0], src.shape[1] // M
        dst = np.empty((M, rows, H), np.float32)
    _load().oracle_merge_transpose(_p(src), _p(dst), M, rows, H, int(bool(to_channel)))
    return dst


def attention_relpos_packed(qkv, Kr, B, S, heads, bias_w=None, bias_r=None, scale=None, mask=None, out_bf16=False):
    """Relative-position attention (Transformer-XL / XLNet form; the reference paper gives no equations for
    it, so no pin comes from there) written out per (model, sequence, head, query) in float64:
      s_ij = scale * ((q_i + bias_w) . k_j + (q_i + bias_r) . Kr[m, S - i + j]) + mask_j,  p = softmax_j,  o_i = sum_j p_ij v_j
    qkv[M, B*S, 3*heads*d] with column blocks [Q | K | V]; Kr[M, 2S, heads*d]; biases [M, heads*d]."""
    qkv, Kr = _f32(qkv).astype(np.float64), _f32(Kr).astype(np.float64)
    M, N, th = qkv.shape
    Hd = th // 3
    d = Hd // heads
    assert N == B * S and Kr.shape == (M, 2 * S, Hd)
    scale = d ** -0.5 if scale is None else scale
    out = np.zeros((M, N, Hd), np.float64)
    for m in range(M):
        for b in range(B):
            rows = slice(b * S, (b + 1) * S)
            for h in range(heads):
                c = slice(h * d, (h + 1) * d)
                q, k, v = qkv[m, rows, c], qkv[m, rows, Hd:][:, c], qkv[m, rows, 2 * Hd:][:, c]
                bw = 0.0 if bias_w is None else np.asarray(bias_w, np.float64)[m, c]
                br = 0.0 if bias_r is None else np.asarray(bias_r, np.float64)[m, c]
                for i in range(S):
                    s = np.empty(S)
                    for j in range(S):
                        s[j] = scale * (np.dot(q[i] + bw, k[j]) + np.dot(q[i] + br, Kr[m, S - i + j, c]))
                        if mask is not None:
                            s[j] += mask[m, b, j]
                    p = np.exp(s - s.max())
                    out[m, b * S + i, c] = (p / p.sum()) @ v
    out = out.astype(np.float32)
    return round_bf16(out) if out_bf16 else out


def round_bf16(a):
    """One round-to-nearest-even to the bf16 grid, by the C oracle's own routine (a 1x1 identity matmul)."""
    a = _f32(a)
    return linear(a.reshape(1, -1, 1), np.ones((1, 1, 1), np.float32), out_bf16=True).reshape(a.shape)
