"""Python binding of the NetFuse merged-operator library for MI355X (gfx950).

Argument marshalling only: every function here checks tensor types, takes ``data_ptr()`` and the
current torch stream, and calls the C entry point of the same name in ``libnetfuse.so``
(declared in ``include/netfuse.h``).  All arithmetic runs in the HIP kernels.  There is no
fallback: if the library has not been built, importing this package raises.

Tensors are torch CUDA tensors, contiguous, dtype float32 or bfloat16 (activations/weights);
per-feature vectors (bias, scale, shift, gamma, beta, mean, var) and masks are float32.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnetfuse.so")

NF_OK, NF_EINVAL, NF_EUNSUPPORTED, NF_ELAUNCH = 0, 1, 2, 3
NF_F32, NF_BF16 = 0, 1
ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2
MERGE_BATCH, MERGE_CHANNEL = 0, 1

EXPORTS = ("netfuse_linear", "netfuse_conv2d", "netfuse_layernorm", "netfuse_batchnorm",
           "netfuse_bn_fold", "netfuse_attention", "netfuse_maxpool2d", "netfuse_avgpool_global",
           "netfuse_merge_transpose", "netfuse_linear_pack_weight", "netfuse_linear_packed",
           "netfuse_time_next_launch", "netfuse_linear_packed_supported", "netfuse_linear_ragged",
           "netfuse_attention_relpos", "netfuse_probe_mfma", "netfuse_probe_hbm_read", "netfuse_strerror")


class NetFuseError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (fn, strerror(status), status))


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libnetfuse.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(or python paper_2009_13062_amd/build.py) first; there is no CPU fallback")
    lib = ctypes.CDLL(LIB_PATH)
    vp, fp, i, f, l = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_long
    lib.netfuse_linear.argtypes = [vp, vp, fp, vp, vp, i, i, i, i, i, i, vp]
    lib.netfuse_conv2d.argtypes = [vp, vp, fp, fp, fp, vp, vp] + [i] * 12 + [i, i, vp]
    lib.netfuse_layernorm.argtypes = [vp, vp, fp, fp, vp, i, i, i, f, i, i, vp]
    lib.netfuse_batchnorm.argtypes = [vp, fp, fp, fp, fp, vp, vp, i, i, i, i, f, i, i, vp]
    lib.netfuse_bn_fold.argtypes = [fp] * 6 + [i, f, vp]
    lib.netfuse_attention.argtypes = [vp, vp, vp, fp, vp, i, i, i, i, i, l, l, f, i, vp]
    lib.netfuse_maxpool2d.argtypes = [vp, vp, i, i, i, i, i, i, i, i, vp]
    lib.netfuse_avgpool_global.argtypes = [vp, vp, i, i, i, i, vp]
    lib.netfuse_merge_transpose.argtypes = [vp, vp, i, i, i, i, i, vp]
    lib.netfuse_linear_packed_supported.argtypes = [i, i, i, i, i]
    lib.netfuse_linear_pack_weight.argtypes = [vp, vp, i, i, i, i, vp]
    lib.netfuse_linear_packed.argtypes = [vp, vp, fp, vp, vp, i, i, i, i, i, i, vp]
    lib.netfuse_time_next_launch.argtypes = [vp, vp]
    lib.netfuse_attention_relpos.argtypes = [vp, vp, vp, vp, fp, fp, fp, vp, i, i, i, i, i, l, l, f, i, vp]
    lib.netfuse_linear_ragged.argtypes = [vp, vp, fp, vp, i, i, i, ctypes.POINTER(ctypes.c_int), i, i, vp]
    lib.netfuse_probe_mfma.argtypes = [vp, i, ctypes.POINTER(ctypes.c_double), vp]
    lib.netfuse_probe_hbm_read.argtypes = [vp, ctypes.c_longlong, vp, vp]
    for name in EXPORTS[:-1]:
        getattr(lib, name).restype = ctypes.c_int
    lib.netfuse_strerror.argtypes = [ctypes.c_int]
    lib.netfuse_strerror.restype = ctypes.c_char_p
    return lib


lib = _load()


def strerror(status: int) -> str:
    return lib.netfuse_strerror(int(status)).decode()


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return NF_F32
    if t.dtype == torch.bfloat16:
        return NF_BF16
    raise TypeError("netfuse tensors are float32 or bfloat16, got %s" % t.dtype)


def _ptr(t: Optional[torch.Tensor], like: Optional[torch.Tensor] = None, f32: bool = False):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("netfuse operands must be contiguous CUDA tensors")
    if f32 and t.dtype != torch.float32:
        raise TypeError("per-feature vectors and masks are float32")
    if like is not None and t.dtype != like.dtype:
        raise TypeError("operand dtype %s differs from %s" % (t.dtype, like.dtype))
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def _check(fn: str, st: int):
    if st != NF_OK:
        raise NetFuseError(fn, st)


def linear(X, W, bias=None, residual=None, act=ACT_NONE, out=None, stream=None):
    """Y[m] = act(X[m] @ W[m] + bias[m]) + residual[m];  X[M,N,K], W[M,K,Nout] -> Y[M,N,Nout]."""
    M, N, K = X.shape
    Nout = W.shape[2]
    if W.shape[0] != M or W.shape[1] != K:
        raise ValueError("W must be [M, K, Nout]")
    Y = torch.empty((M, N, Nout), dtype=X.dtype, device=X.device) if out is None else out
    _check("netfuse_linear", lib.netfuse_linear(
        _ptr(X), _ptr(W, X), _ptr(bias, f32=True), _ptr(residual, X), _ptr(Y, X), M, N, K, Nout,
        _dt(X), int(act), _stream(stream)))
    return Y


def linear_packed_supported(M, N, K, Nout, dtype=torch.bfloat16) -> bool:
    """True if linear_packed has a kernel for N rows per model of W[M,K,Nout]."""
    return bool(lib.netfuse_linear_packed_supported(M, N, K, Nout, NF_BF16 if dtype == torch.bfloat16 else NF_F32))


def linear_pack_weight(W, out=None, stream=None):
    """W[M,K,Nout] -> fragment-packed copy (same shape and dtype, layout of include/netfuse.h)."""
    M, K, Nout = W.shape
    Wp = torch.empty_like(W) if out is None else out
    _check("netfuse_linear_pack_weight", lib.netfuse_linear_pack_weight(
        _ptr(W), _ptr(Wp, W), M, K, Nout, _dt(W), _stream(stream)))
    return Wp


def linear_packed(X, Wp, bias=None, residual=None, act=ACT_NONE, out=None, stream=None):
    """netfuse_linear on weights packed by linear_pack_weight(W); Wp keeps W's shape [M,K,Nout]."""
    M, N, K = X.shape
    Nout = Wp.shape[2]
    if Wp.shape[0] != M or Wp.shape[1] != K:
        raise ValueError("Wp must be [M, K, Nout]")
    Y = torch.empty((M, N, Nout), dtype=X.dtype, device=X.device) if out is None else out
    _check("netfuse_linear_packed", lib.netfuse_linear_packed(
        _ptr(X), _ptr(Wp, X), _ptr(bias, f32=True), _ptr(residual, X), _ptr(Y, X), M, N, K, Nout,
        _dt(X), int(act), _stream(stream)))
    return Y


def linear_ragged(X, W, nout, bias=None, act=ACT_NONE, out=None, stream=None):
    """Per-model output widths: X[M,N,K]; W flat = concat of W_m[K, nout[m]]; bias flat float32 = concat of
    b_m[nout[m]] -> Y flat = concat of Y_m[N, nout[m]] (views: ragged_views)."""
    M, N, K = X.shape
    nout = [int(n) for n in nout]
    if len(nout) != M or W.numel() != K * sum(nout):
        raise ValueError("W must hold K * sum(nout) elements, nout one entry per model")
    Y = torch.empty(N * sum(nout), dtype=X.dtype, device=X.device) if out is None else out
    arr = (ctypes.c_int * M)(*nout)
    _check("netfuse_linear_ragged", lib.netfuse_linear_ragged(
        _ptr(X), _ptr(W, X), _ptr(bias, f32=True), _ptr(Y, X), M, N, K, arr, _dt(X), int(act), _stream(stream)))
    return Y


def ragged_views(flat, rows, nout):
    """The per-model [rows, nout[m]] views of a ragged concatenation."""
    out, o = [], 0
    for n in nout:
        out.append(flat[o:o + rows * n].view(rows, n))
        o += rows * n
    return out


def time_next_launch(start_event, stop_event):
    """Arm the next kernel launch of this thread with two raw hipEvent_t handles (ints or None)."""
    _check("netfuse_time_next_launch", lib.netfuse_time_next_launch(start_event, stop_event))


def probe_mfma(sink, iters, stream=None):
    """Launch the register-only matrix-instruction loop; returns the floating point operations it executes."""
    fl = ctypes.c_double()
    _check("netfuse_probe_mfma", lib.netfuse_probe_mfma(_ptr(sink), int(iters), ctypes.byref(fl), _stream(stream)))
    return fl.value


def probe_hbm_read(src, sink, stream=None):
    """Launch the read-only stream over the whole of `src`; returns the bytes it reads."""
    nbytes = src.numel() * src.element_size()
    _check("netfuse_probe_hbm_read", lib.netfuse_probe_hbm_read(_ptr(src), nbytes, _ptr(sink), _stream(stream)))
    return nbytes


def conv_out_size(n, k, stride, pad, dil=1):
    return (n + 2 * pad - dil * (k - 1) - 1) // stride + 1


def conv2d(x, w, M, g=1, bias=None, scale=None, shift=None, residual=None, stride=1, pad=0, dil=1,
           act=ACT_NONE, out=None, stream=None):
    """x[B, M*Cin, H, W], w[M*Cout, Cin/g, KH, KW] -> y[B, M*Cout, Ho, Wo]; merged groups = M*g."""
    B, Ct, H, Wd = x.shape
    Cin, Cout = Ct // M, w.shape[0] // M
    KH, KW = w.shape[2], w.shape[3]
    if Ct % M or w.shape[0] % M or w.shape[1] * g != Cin:
        raise ValueError("channel counts do not match M and g")
    Ho, Wo = conv_out_size(H, KH, stride, pad, dil), conv_out_size(Wd, KW, stride, pad, dil)
    y = torch.empty((B, M * Cout, Ho, Wo), dtype=x.dtype, device=x.device) if out is None else out
    _check("netfuse_conv2d", lib.netfuse_conv2d(
        _ptr(x), _ptr(w, x), _ptr(bias, f32=True), _ptr(scale, f32=True), _ptr(shift, f32=True),
        _ptr(residual, x), _ptr(y, x), M, B, Cin, Cout, g, H, Wd, KH, KW, stride, pad, dil, _dt(x),
        int(act), _stream(stream)))
    return y


def layernorm(x, gamma, beta, M, residual=None, eps=1e-5, layout=MERGE_BATCH, out=None, stream=None):
    """layout MERGE_BATCH: x[M, rows, H]; MERGE_CHANNEL: x[rows, M*H]; gamma, beta float32[M*H]."""
    if layout == MERGE_BATCH:
        rows, H = x.shape[1], x.shape[2]
    else:
        rows, H = x.shape[0], x.shape[1] // M
    y = torch.empty_like(x) if out is None else out
    _check("netfuse_layernorm", lib.netfuse_layernorm(
        _ptr(x), _ptr(residual, x), _ptr(gamma, f32=True), _ptr(beta, f32=True), _ptr(y, x), M, rows,
        H, float(eps), int(layout), _dt(x), _stream(stream)))
    return y


def batchnorm(x, gamma, beta, mean, var, M, residual=None, eps=1e-5, act=ACT_NONE, out=None,
              stream=None):
    """x[B, M*C, ...]: per merged channel inference batch norm, + residual, activation."""
    B, Ct = x.shape[0], x.shape[1]
    HW = 1
    for s in x.shape[2:]:
        HW *= s
    y = torch.empty_like(x) if out is None else out
    _check("netfuse_batchnorm", lib.netfuse_batchnorm(
        _ptr(x), _ptr(gamma, f32=True), _ptr(beta, f32=True), _ptr(mean, f32=True),
        _ptr(var, f32=True), _ptr(residual, x), _ptr(y, x), M, B, Ct // M, HW, float(eps), _dt(x),
        int(act), _stream(stream)))
    return y


def bn_fold(gamma, beta, mean, var, eps=1e-5, stream=None):
    """scale = gamma/sqrt(var+eps), shift = beta - mean*scale (float32[M*C] each)."""
    scale, shift = torch.empty_like(gamma), torch.empty_like(gamma)
    _check("netfuse_bn_fold", lib.netfuse_bn_fold(
        _ptr(gamma, f32=True), _ptr(beta, f32=True), _ptr(mean, f32=True), _ptr(var, f32=True),
        _ptr(scale, f32=True), _ptr(shift, f32=True), gamma.numel(), float(eps), _stream(stream)))
    return scale, shift


def attention_packed(QKV, B, S, heads, scale=None, mask=None, out=None, stream=None):
    """QKV[M, B*S, 3*heads*d] with column blocks [Q | K | V] -> O[M, B*S, heads*d]."""
    M, N, three_h = QKV.shape
    Hd = three_h // 3
    d = Hd // heads
    if N != B * S or three_h != 3 * heads * d:
        raise ValueError("QKV must be [M, B*S, 3*heads*d]")
    if scale is None:
        scale = d ** -0.5
    O = torch.empty((M, N, Hd), dtype=QKV.dtype, device=QKV.device) if out is None else out
    base, esz = _ptr(QKV), QKV.element_size()
    _check("netfuse_attention", lib.netfuse_attention(
        base, base + Hd * esz, base + 2 * Hd * esz, _ptr(mask, f32=True), _ptr(O, QKV), M, B, S,
        heads, d, N * three_h, three_h, float(scale), _dt(QKV), _stream(stream)))
    return O


def attention(Q, K, V, B, S, heads, scale=None, mask=None, out=None, stream=None):
    """Separate dense Q, K, V of shape [M, B*S, heads*d]."""
    M, N, Hd = Q.shape
    d = Hd // heads
    if scale is None:
        scale = d ** -0.5
    O = torch.empty((M, N, Hd), dtype=Q.dtype, device=Q.device) if out is None else out
    _check("netfuse_attention", lib.netfuse_attention(
        _ptr(Q), _ptr(K, Q), _ptr(V, Q), _ptr(mask, f32=True), _ptr(O, Q), M, B, S, heads, d, N * Hd,
        Hd, float(scale), _dt(Q), _stream(stream)))
    return O


def attention_relpos_packed(QKV, Kr, B, S, heads, bias_w=None, bias_r=None, scale=None, mask=None, out=None,
                            stream=None):
    """Relative-position attention on QKV[M, B*S, 3*heads*d] (column blocks [Q | K | V]) and the projected
    position encodings Kr[M, 2*S, heads*d]; bias_w, bias_r float32 [M, heads*d]."""
    M, N, three_h = QKV.shape
    Hd = three_h // 3
    d = Hd // heads
    if N != B * S or three_h != 3 * heads * d or tuple(Kr.shape) != (M, 2 * S, Hd):
        raise ValueError("QKV must be [M, B*S, 3*heads*d] and Kr [M, 2*S, heads*d]")
    if scale is None:
        scale = d ** -0.5
    O = torch.empty((M, N, Hd), dtype=QKV.dtype, device=QKV.device) if out is None else out
    base, esz = _ptr(QKV), QKV.element_size()
    _check("netfuse_attention_relpos", lib.netfuse_attention_relpos(
        base, base + Hd * esz, base + 2 * Hd * esz, _ptr(Kr, QKV), _ptr(bias_w, f32=True), _ptr(bias_r, f32=True),
        _ptr(mask, f32=True), _ptr(O, QKV), M, B, S, heads, d, N * three_h, three_h, float(scale), _dt(QKV),
        _stream(stream)))
    return O


def maxpool2d(x, k, stride, pad, out=None, stream=None):
    B, Ct, H, Wd = x.shape
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (Wd + 2 * pad - k) // stride + 1
    y = torch.empty((B, Ct, Ho, Wo), dtype=x.dtype, device=x.device) if out is None else out
    _check("netfuse_maxpool2d", lib.netfuse_maxpool2d(_ptr(x), _ptr(y, x), B, Ct, H, Wd, k, stride,
                                                      pad, _dt(x), _stream(stream)))
    return y


def avgpool_global(x, out=None, stream=None):
    B, Ct = x.shape[0], x.shape[1]
    HW = 1
    for s in x.shape[2:]:
        HW *= s
    y = torch.empty((B, Ct), dtype=x.dtype, device=x.device) if out is None else out
    _check("netfuse_avgpool_global", lib.netfuse_avgpool_global(_ptr(x), _ptr(y, x), B, Ct, HW,
                                                                _dt(x), _stream(stream)))
    return y


def merge_transpose(src, M, to_channel, out=None, stream=None):
    """to_channel: src[M, rows, H] -> [rows, M*H]; else src[rows, M*H] -> [M, rows, H]."""
    if to_channel:
        _, rows, H = src.shape
        shape = (rows, M * H)
    else:
        rows, H = src.shape[0], src.shape[1] // M
        shape = (M, rows, H)
    dst = torch.empty(shape, dtype=src.dtype, device=src.device) if out is None else out
    _check("netfuse_merge_transpose", lib.netfuse_merge_transpose(
        _ptr(src), _ptr(dst, src), M, rows, H, int(bool(to_channel)), _dt(src), _stream(stream)))
    return dst
