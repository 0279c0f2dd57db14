"""Pins for the CPU oracle: it is checked against things other than itself.

* brute force: the merged call equals M independent evaluations of a second, simpler
  single-model definition written here in numpy float64 / python loops (Appendix A, Eq. 3-6:
  y_m = Conv(x_m, w_m); Section 3.1 for the other operators);
* library special case: at M = 1 every merged operator is the ordinary operator, taken from
  torch's CPU routines (Appendix A: GroupConv(x, w, 1) = Conv(x, w));
* closed forms and invariants that a dropped term, wrong index, sign or transposed operand breaks.
"""
import itertools
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import netfuse_inputs as NI

GOLD = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(1234)


def rnd(*shape, std=1.0):
    return (std * rng.standard_normal(shape)).astype(np.float32)


def close(a, b, tol=2e-6):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    assert a.shape == b.shape
    scale = max(1.0, float(np.abs(b).max()))
    assert np.abs(a - b).max() <= tol * scale, float(np.abs(a - b).max())


def gelu_erf64(v):
    from math import erf, sqrt
    return np.vectorize(lambda t: 0.5 * t * (1.0 + erf(t / sqrt(2.0))))(np.asarray(v, np.float64))


# ------------------------------------------------------------------ single-model definitions
def conv_single_loops(x, w, stride, pad, dil):
    """Plain convolution of ONE model with python loops: x[C,H,W], w[Co,C,KH,KW] (Appendix A Eq. 1)."""
    C, H, Wd = x.shape
    Co, _, KH, KW = w.shape
    xp = np.zeros((C, H + 2 * pad, Wd + 2 * pad))
    xp[:, pad:pad + H, pad:pad + Wd] = x
    Ho = (H + 2 * pad - dil * (KH - 1) - 1) // stride + 1
    Wo = (Wd + 2 * pad - dil * (KW - 1) - 1) // stride + 1
    y = np.zeros((Co, Ho, Wo))
    for co, oy, ox in itertools.product(range(Co), range(Ho), range(Wo)):
        s = 0.0
        for ci, ky, kx in itertools.product(range(C), range(KH), range(KW)):
            s += float(w[co, ci, ky, kx]) * xp[ci, oy * stride + ky * dil, ox * stride + kx * dil]
        y[co, oy, ox] = s
    return y


def attention_single(q, k, v, scale, mask=None):
    s = scale * (q.astype(np.float64) @ k.astype(np.float64).T)
    if mask is not None:
        s = s + mask[None, :]
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    p /= p.sum(axis=1, keepdims=True)
    return p @ v.astype(np.float64)


# ------------------------------------------------------------------ bf16 rounding
def test_bf16_rounding_matches_torch_and_ties(oracle):
    vals = np.concatenate([rnd(4096), rnd(512, std=1e-3), rnd(512, std=1e4),
                           np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 0.0, 65280.0], np.float32)])
    # 1.00390625 = 1 + 2^-8 is an exact tie between 1.0 and 1.0078125 -> even mantissa (1.0);
    # 1.01171875 = 1 + 3*2^-8 is a tie between 1.0078125 and 1.015625 -> 1.015625.
    ident = np.stack([np.eye(1, dtype=np.float32)])                      # W = [[1]]: Y = X
    got = oracle.linear(vals.reshape(1, -1, 1), ident, out_bf16=True).reshape(-1)
    want = torch.from_numpy(vals).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got, want)
    assert got[5120] == 1.0 and got[5121] == 1.0 and got[5122] == 1.015625 and got[5123] == -1.0
    # the input generator's storage conversion agrees with the same library routine
    assert np.array_equal(NI.on_bf16_grid(vals), want)
    assert np.array_equal(NI.bf16_to_f32(NI.bf16_bits(vals)), want)


# ------------------------------------------------------------------ linear
@pytest.mark.parametrize("M,N,K,Nout", [(1, 3, 5, 7), (3, 4, 6, 2), (5, 1, 9, 4)])
def test_linear_bruteforce_per_model(oracle, M, N, K, Nout):
    X, W, b, R = rnd(M, N, K), rnd(M, K, Nout), rnd(M, Nout), rnd(M, N, Nout)
    got = oracle.linear(X, W, bias=b, residual=R, act=oracle.ACT_GELU)
    for m in range(M):
        z = X[m].astype(np.float64) @ W[m].astype(np.float64) + b[m]
        close(got[m], gelu_erf64(z) + R[m])
    got = oracle.linear(X, W, bias=b, act=oracle.ACT_RELU)
    for m in range(M):
        close(got[m], np.maximum(X[m].astype(np.float64) @ W[m].astype(np.float64) + b[m], 0))


def test_linear_m1_is_torch_linear(oracle):
    X, W, b = rnd(1, 6, 10), rnd(1, 10, 4), rnd(1, 4)
    want = F.linear(torch.from_numpy(X[0]).double(), torch.from_numpy(W[0]).double().t(),
                    torch.from_numpy(b[0]).double())
    close(oracle.linear(X, W, bias=b)[0], want.numpy())
    want_g = F.gelu(want)            # torch's default GELU is the erf form
    close(oracle.linear(X, W, bias=b, act=oracle.ACT_GELU)[0], want_g.numpy())


def test_linear_closed_forms(oracle):
    M, N, K = 4, 3, 5
    X, b = rnd(M, N, K), rnd(M, K)
    eye = np.stack([np.eye(K, dtype=np.float32)] * M)
    close(oracle.linear(X, eye, bias=b), X + b[:, None, :])
    scaled = np.stack([(m + 1) * np.eye(K, dtype=np.float32) for m in range(M)])
    got = oracle.linear(X, scaled)
    for m in range(M):                       # a model mix-up would use the wrong multiple
        close(got[m], (m + 1) * X[m])
    # orientation: W[m] is [K, Nout], Y = X W (one-hot column picks one input feature)
    W = np.zeros((1, K, 2), np.float32)
    W[0, 3, 1] = 1.0
    got = oracle.linear(X[:1], W)
    close(got[0, :, 1], X[0, :, 3])
    close(got[0, :, 0], np.zeros(N))


def test_linear_equals_1x1_conv(oracle):
    """A matrix multiplication is a 1x1 convolution (Section 3.1)."""
    M, N, K, Nout = 3, 6, 4, 5
    X, W, b = rnd(M, N, K), rnd(M, K, Nout), rnd(M, Nout)
    lin = oracle.linear(X, W, bias=b)
    # rows become the 1 x N spatial positions; channels are features
    x = np.concatenate([X[m].T for m in range(M)]).reshape(1, M * K, 1, N)
    w = np.concatenate([W[m].T for m in range(M)]).reshape(M * Nout, K, 1, 1)
    y = oracle.conv2d(x, w, M, bias=b.reshape(-1))
    for m in range(M):
        close(y[0, m * Nout:(m + 1) * Nout, 0, :].T, lin[m])


# ------------------------------------------------------------------ convolution
@pytest.mark.parametrize("M,g,Cin,Cout,H,W,KH,KW,stride,pad,dil", [
    (1, 1, 2, 3, 5, 4, 3, 3, 1, 1, 1),
    (3, 1, 2, 2, 5, 6, 3, 2, 2, 1, 1),
    (2, 2, 4, 6, 6, 5, 3, 3, 1, 2, 2),
    (2, 1, 3, 2, 7, 7, 1, 1, 2, 0, 1),
])
def test_conv_bruteforce_per_model(oracle, M, g, Cin, Cout, H, W, KH, KW, stride, pad, dil):
    B = 2
    cig, cog = Cin // g, Cout // g
    x, w = rnd(B, M * Cin, H, W), rnd(M * Cout, cig, KH, KW)
    got = oracle.conv2d(x, w, M, g=g, stride=stride, pad=pad, dil=dil)
    for b, m, gi in itertools.product(range(B), range(M), range(g)):
        xs = x[b, m * Cin + gi * cig: m * Cin + (gi + 1) * cig]
        ws = w[m * Cout + gi * cog: m * Cout + (gi + 1) * cog]
        want = conv_single_loops(xs, ws, stride, pad, dil)
        close(got[b, m * Cout + gi * cog: m * Cout + (gi + 1) * cog], want)


@pytest.mark.parametrize("g", [1, 2, 4])
def test_conv_m1_is_torch_conv(oracle, g):
    x, w, bias = rnd(2, 8, 9, 7), rnd(12, 8 // g, 3, 3), rnd(12)
    for stride, pad, dil in [(1, 1, 1), (2, 0, 1), (2, 3, 2)]:
        want = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                        torch.from_numpy(bias).double(), stride=stride, padding=pad, dilation=dil,
                        groups=g).numpy()
        close(oracle.conv2d(x, w, 1, g=g, bias=bias, stride=stride, pad=pad, dil=dil), want)


def test_conv_four_models_of_two_groups_is_eight_groups(oracle):
    """Merging 4 grouped convolutions of 2 groups each gives one of 4 x 2 = 8 groups (Section 3.1)."""
    M, g, Cin, Cout = 4, 2, 6, 4
    x, w = rnd(1, M * Cin, 6, 6), rnd(M * Cout, Cin // g, 3, 3)
    got = oracle.conv2d(x, w, M, g=g, pad=1)
    want8 = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), padding=1,
                     groups=8).numpy()
    close(got, want8)
    for m in range(M):
        wm = F.conv2d(torch.from_numpy(x[:, m * Cin:(m + 1) * Cin]).double(),
                      torch.from_numpy(w[m * Cout:(m + 1) * Cout]).double(), padding=1, groups=2)
        close(got[:, m * Cout:(m + 1) * Cout], wm.numpy())


def test_group_offset_identity_exhaustive():
    """Appendix A Eq. 5: C_in * floor((C_out*m + c_out)/C_out) = C_in*m for 0 <= c_out < C_out."""
    for Cin, Cout, M in itertools.product(range(1, 7), range(1, 7), range(1, 6)):
        for m, co in itertools.product(range(M), range(Cout)):
            assert Cin * ((Cout * m + co) // Cout) == Cin * m


def test_conv_closed_forms(oracle):
    M, C = 3, 4
    x = rnd(1, M * C, 5, 6)
    # centre-tap delta on the matching channel: identity
    w = np.zeros((M * C, C, 3, 3), np.float32)
    for c in range(M * C):
        w[c, c % C, 1, 1] = 1.0
    close(oracle.conv2d(x, w, M, pad=1), x)
    # all-ones 3x3 on all-ones input, pad 1: 9*cig inside, 6*cig on edges, 4*cig in corners
    with open(os.path.join(GOLD, "conv_ones_3x3_pad1.txt")) as f:
        rows = [list(map(float, ln.split())) for ln in f if ln.strip() and not ln.startswith("#")]
    per_cig = np.array(rows)                                    # 5 x 6 table for cig = 1
    y = oracle.conv2d(np.ones((1, M * C, 5, 6), np.float32), np.ones((M * 2, C, 3, 3), np.float32),
                      M, pad=1)
    for c in range(M * 2):
        close(y[0, c], C * per_cig)
    # which input channel is read: x = its merged channel index, one-hot weights
    xi = np.broadcast_to(np.arange(M * C, dtype=np.float32)[None, :, None, None], (1, M * C, 3, 3)).copy()
    Cout = 5
    w = np.zeros((M * Cout, C, 1, 1), np.float32)
    pick = rng.integers(0, C, size=M * Cout)
    for c in range(M * Cout):
        w[c, pick[c], 0, 0] = 1.0
    y = oracle.conv2d(xi, w, M)
    for c in range(M * Cout):
        m = c // Cout                                           # Eq. 3: y_m[c_out] = y[Cout*m + c_out]
        assert np.all(y[0, c] == C * m + pick[c])               # x[Cin*m + c_in] = x_m[c_in]
    # kernel orientation: cross-correlation, no flip, and (ky, kx) not transposed
    x1 = np.zeros((1, 1, 4, 5), np.float32)
    x1[0, 0, 2, 3] = 1.0
    w1 = np.arange(6, dtype=np.float32).reshape(1, 1, 2, 3)
    y1 = oracle.conv2d(x1, w1, 1)                               # valid: 3 x 3 output
    want = np.zeros((3, 3))
    for ky, kx in itertools.product(range(2), range(3)):
        oy, ox = 2 - ky, 3 - kx
        if 0 <= oy < 3 and 0 <= ox < 3:
            want[oy, ox] = w1[0, 0, ky, kx]
    close(y1[0, 0], want)


def test_conv_epilogue_order(oracle):
    M, C = 2, 3
    x, w = rnd(1, M * C, 4, 4), rnd(M * C, C, 3, 3)
    bias, scale, shift, res = rnd(M * C), rnd(M * C), rnd(M * C), rnd(1, M * C, 4, 4)
    raw = oracle.conv2d(x, w, M, pad=1).astype(np.float64)
    v = (raw + bias[None, :, None, None]) * scale[None, :, None, None] + shift[None, :, None, None] + res
    close(oracle.conv2d(x, w, M, pad=1, bias=bias, scale=scale, shift=shift, residual=res,
                        act=oracle.ACT_RELU), np.maximum(v, 0))


# ------------------------------------------------------------------ layer norm
def test_layernorm_m_models_is_groupnorm_not_big_layernorm(oracle):
    """M LayerNorms = GroupNorm with M groups on the channel concatenation; one LayerNorm over the
    concatenation is a different function (Section 3.1)."""
    M, rows, H = 3, 5, 8
    xs = [rnd(rows, H) + 3.0 * m for m in range(M)]
    gam, bet = rnd(M * H), rnd(M * H)
    xc = np.concatenate(xs, axis=1)                                        # [rows, M*H]
    got = oracle.layernorm(xc, gam, bet, M, eps=1e-5, layout=oracle.LAYOUT_CHANNEL)
    want = F.group_norm(torch.from_numpy(xc).double(), M, torch.from_numpy(gam).double(),
                        torch.from_numpy(bet).double(), eps=1e-5).numpy()
    close(got, want)
    for m in range(M):
        wm = F.layer_norm(torch.from_numpy(xs[m]).double(), (H,), torch.from_numpy(gam[m * H:(m + 1) * H]).double(),
                          torch.from_numpy(bet[m * H:(m + 1) * H]).double(), eps=1e-5).numpy()
        close(got[:, m * H:(m + 1) * H], wm)
    big = F.layer_norm(torch.from_numpy(xc).double(), (M * H,), torch.from_numpy(gam).double(),
                       torch.from_numpy(bet).double(), eps=1e-5).numpy()
    assert np.abs(big - got).max() > 0.1                                  # negative control
    # both merge layouts hold the same numbers (Section 3.2's reshape between bmm and group norm)
    xb = np.stack(xs)                                                      # [M, rows, H]
    gb = oracle.layernorm(xb, gam, bet, M, eps=1e-5, layout=oracle.LAYOUT_BATCH)
    assert np.array_equal(oracle.merge_transpose(gb, M, True), got)


def test_layernorm_closed_forms(oracle):
    M, rows, H, eps = 2, 4, 16, 1e-3
    x = rnd(M, rows, H) * 2.0 + 1.0
    y = oracle.layernorm(x, np.ones(M * H, np.float32), np.zeros(M * H, np.float32), M, eps=eps)
    var = x.astype(np.float64).var(axis=2)
    close(y.astype(np.float64).mean(axis=2), np.zeros((M, rows)), tol=1e-6)
    close(y.astype(np.float64).var(axis=2), var / (var + eps), tol=1e-5)
    beta = rnd(M * H)
    const = np.full((M, rows, H), 2.5, np.float32)
    close(oracle.layernorm(const, rnd(M * H), beta, M), np.broadcast_to(beta.reshape(M, 1, H), (M, rows, H)))
    # residual is added before the statistics
    r = rnd(M, rows, H)
    g, b = rnd(M * H), rnd(M * H)
    close(oracle.layernorm(x, g, b, M, residual=r), oracle.layernorm(x + r, g, b, M), tol=1e-5)


# ------------------------------------------------------------------ batch norm
def test_batchnorm_vs_torch_and_identity(oracle):
    M, C, B = 3, 4, 2
    x = rnd(B, M * C, 3, 5)
    g, b, mu = rnd(M * C), rnd(M * C), rnd(M * C)
    var = rng.uniform(0.5, 1.5, M * C).astype(np.float32)
    want = F.batch_norm(torch.from_numpy(x).double(), torch.from_numpy(mu).double(),
                        torch.from_numpy(var).double(), torch.from_numpy(g).double(),
                        torch.from_numpy(b).double(), training=False, eps=1e-5).numpy()
    close(oracle.batchnorm(x, g, b, mu, var, M), want)
    res = rnd(B, M * C, 3, 5)
    close(oracle.batchnorm(x, g, b, mu, var, M, residual=res, act=oracle.ACT_RELU), np.maximum(want + res, 0))
    ones, zeros = np.ones(M * C, np.float32), np.zeros(M * C, np.float32)
    close(oracle.batchnorm(x, ones, zeros, zeros, np.full(M * C, 1 - 1e-5, np.float32), M), x)
    # folded form used as a convolution epilogue gives the same function
    scale, shift = oracle.bn_fold(g, b, mu, var)
    close(x * scale[None, :, None, None] + shift[None, :, None, None], want, tol=1e-5)


# ------------------------------------------------------------------ attention
def test_attention_bruteforce_and_strides(oracle):
    M, B, S, heads, d = 2, 2, 5, 3, 4
    Hd = heads * d
    qkv = rnd(M, B * S, 3 * Hd)
    mask = rnd(M, B, S)
    got = oracle.attention_packed(qkv, B, S, heads, mask=mask)
    for m, b, h in itertools.product(range(M), range(B), range(heads)):
        rows = slice(b * S, (b + 1) * S)
        q = qkv[m, rows, h * d:(h + 1) * d]
        k = qkv[m, rows, Hd + h * d: Hd + (h + 1) * d]
        v = qkv[m, rows, 2 * Hd + h * d: 2 * Hd + (h + 1) * d]
        close(got[m, rows, h * d:(h + 1) * d], attention_single(q, k, v, 1 / np.sqrt(d), mask[m, b]))
    # separate contiguous Q, K, V give the same answer as the packed view
    Q, K, V = (np.ascontiguousarray(qkv[:, :, i * Hd:(i + 1) * Hd]) for i in range(3))
    sep = oracle.attention(Q.reshape(-1), K.reshape(-1), V.reshape(-1), M, B, S, heads, d,
                           B * S * Hd, Hd, 1 / np.sqrt(d), mask=mask)
    assert np.array_equal(sep, got)


def test_attention_m1_is_torch_sdpa(oracle):
    S, heads, d = 7, 2, 8
    Hd = heads * d
    qkv = rnd(1, S, 3 * Hd)
    got = oracle.attention_packed(qkv, 1, S, heads)
    t = torch.from_numpy(qkv[0]).double()
    q, k, v = (t[:, i * Hd:(i + 1) * Hd].reshape(S, heads, d).transpose(0, 1) for i in range(3))
    want = F.scaled_dot_product_attention(q, k, v).transpose(0, 1).reshape(S, Hd).numpy()
    close(got[0], want)


def test_attention_closed_forms(oracle):
    M, S, heads, d = 2, 6, 2, 4
    Hd = heads * d
    qkv = rnd(M, S, 3 * Hd)
    zero_q = qkv.copy()
    zero_q[:, :, :Hd] = 0.0                                    # uniform weights: O_i = mean_j V_j
    got = oracle.attention_packed(zero_q, 1, S, heads)
    for m in range(M):
        close(got[m], np.broadcast_to(qkv[m, :, 2 * Hd:].astype(np.float64).mean(axis=0), (S, Hd)))
    # a mask of -1e9 on all keys but one selects that key's V row
    mask = np.full((M, 1, S), -1e9, np.float32)
    mask[:, 0, 4] = 0.0
    got = oracle.attention_packed(qkv, 1, S, heads, mask=mask)
    for m in range(M):
        close(got[m], np.broadcast_to(qkv[m, 4, 2 * Hd:], (S, Hd)))
    # one-hot-dominant keys: query i matches key perm[i] only
    big = np.zeros((1, S, 3 * S), np.float32)                  # heads = 1, d = S
    perm = rng.permutation(S)
    for i in range(S):
        big[0, i, perm[i]] = 30.0                              # Q_i = 30 e_perm[i]
        big[0, i, S + i] = 30.0                                # K_j = 30 e_j
    big[0, :, 2 * S:] = rnd(S, S)
    got = oracle.attention_packed(big, 1, S, 1, scale=1.0)
    close(got[0], big[0, perm, 2 * S:], tol=1e-6)


# ------------------------------------------------------------------ non-trainable glue
def test_pools_and_transpose_vs_library(oracle):
    x = rnd(2, 6, 9, 8)
    want = F.max_pool2d(torch.from_numpy(x), 3, 2, 1).numpy()
    assert np.array_equal(oracle.maxpool2d(x, 3, 2, 1), want)
    neg = -np.abs(x) - 1.0                                      # padding must never win
    assert np.array_equal(oracle.maxpool2d(neg, 3, 2, 1), F.max_pool2d(torch.from_numpy(neg), 3, 2, 1).numpy())
    close(oracle.avgpool_global(x), x.astype(np.float64).mean(axis=(2, 3)))
    M, rows, H = 3, 4, 5
    s = rnd(M, rows, H)
    t = oracle.merge_transpose(s, M, True)
    assert np.array_equal(t, s.transpose(1, 0, 2).reshape(rows, M * H))
    assert np.array_equal(oracle.merge_transpose(t, M, False), s)


# ------------------------------------------------------------------ invariants over all operators
def _all_ops(oracle, inp, M, enc, Menc, spec, rn):
    from oracle import models as OM
    out = dict(OM.tiny_layer(inp, M))
    out["encoder"] = OM.encoder_stack(enc, Menc, 1, 6, 2, out_bf16=False)
    out["resnet"] = OM.resnet_forward(rn, spec, Menc, out_bf16=False)
    return out


def test_permuting_models_permutes_outputs(oracle):
    """Merging is concatenation in an arbitrary model order (Section 3.1)."""
    M = 4
    perm = [2, 0, 3, 1]
    shape = NI.EncoderShape(hidden=16, heads=2, ffn=32, layers=2, seq=6)
    spec = NI.resnet_spec(image=32, width_div=16, depths=(1, 1, 1, 1))
    a = _all_ops(oracle, NI.tiny_layer(M), M, NI.encoder_stack(M, shape, bf16=False), M, spec,
                 NI.resnet_params(spec, M, bf16=False))
    b = _all_ops(oracle, NI.tiny_layer(M, order=perm), M,
                 NI.encoder_stack(M, shape, bf16=False, order=perm), M, spec,
                 NI.resnet_params(spec, M, bf16=False, order=perm))
    for i, src in enumerate(perm):
        for key in ("linear", "layernorm", "encoder"):
            assert np.array_equal(b[key][i], a[key][src]), key
        assert np.array_equal(b["conv"][0, 16 * i:16 * (i + 1)], a["conv"][0, 16 * src:16 * (src + 1)])
        C = spec.out_channels
        assert np.array_equal(b["resnet"][0, C * i:C * (i + 1)], a["resnet"][0, C * src:C * (src + 1)])


def test_other_models_cannot_influence_model_m(oracle):
    """Each weight set touches only its own input: poisoning every other model leaves y_m bit-identical."""
    M, keep = 3, 1
    inp = NI.tiny_layer(M)
    from oracle import models as OM
    clean = OM.tiny_layer(inp, M)
    bad = {k: v.copy() for k, v in inp.items()}
    for m in range(M):
        if m == keep:
            continue
        bad["X"][m] = np.nan
        bad["W"][m] = 1e30
        bad["b"][m] = np.nan
        bad["gamma"][64 * m:64 * (m + 1)] = np.nan
        bad["conv_x"][0, 16 * m:16 * (m + 1)] = np.nan
        bad["conv_w"][16 * m:16 * (m + 1)] = np.inf
    dirty = OM.tiny_layer(bad, M)
    assert np.array_equal(dirty["linear"][keep], clean["linear"][keep])
    assert np.array_equal(dirty["layernorm"][keep], clean["layernorm"][keep])
    assert np.array_equal(dirty["conv"][0, 16 * keep:16 * (keep + 1)], clean["conv"][0, 16 * keep:16 * (keep + 1)])
    assert np.isnan(dirty["linear"][0]).all()
    qkv = rnd(M, 5, 3 * 8)
    a = oracle.attention_packed(qkv, 1, 5, 2)
    qkv2 = qkv.copy()
    qkv2[[0, 2]] = np.nan
    assert np.array_equal(oracle.attention_packed(qkv2, 1, 5, 2)[keep], a[keep])


# ------------------------------------------------------------------ whole-workload chains
def test_encoder_layer_matches_torch_modules(oracle):
    """The post-LN encoder layer chain equals torch's own TransformerEncoderLayer (norm_first=False,
    erf GELU) at M = 1 and, model by model, at M = 3."""
    from oracle import models as OM
    M = 3
    shape = NI.EncoderShape(hidden=16, heads=4, ffn=40, layers=1, seq=7)
    inp = NI.encoder_stack(M, shape, bf16=False)
    got = OM.encoder_stack(inp, M, 1, shape.seq, shape.heads, eps=1e-5, out_bf16=False)
    Lw = inp["layers"][0]
    Hd = shape.hidden
    for m in range(M):
        layer = torch.nn.TransformerEncoderLayer(Hd, shape.heads, shape.ffn, dropout=0.0,
                                                 activation="gelu", batch_first=True, norm_first=False).double().eval()
        with torch.no_grad():
            t = lambda a: torch.from_numpy(np.asarray(a)).double()
            layer.self_attn.in_proj_weight.copy_(t(Lw["Wqkv"][m]).t())
            layer.self_attn.in_proj_bias.copy_(t(Lw["bqkv"][m]))
            layer.self_attn.out_proj.weight.copy_(t(Lw["Wo"][m]).t())
            layer.self_attn.out_proj.bias.copy_(t(Lw["bo"][m]))
            layer.linear1.weight.copy_(t(Lw["W1"][m]).t()); layer.linear1.bias.copy_(t(Lw["b1"][m]))
            layer.linear2.weight.copy_(t(Lw["W2"][m]).t()); layer.linear2.bias.copy_(t(Lw["b2"][m]))
            layer.norm1.weight.copy_(t(Lw["ln1_g"][m * Hd:(m + 1) * Hd])); layer.norm1.bias.copy_(t(Lw["ln1_b"][m * Hd:(m + 1) * Hd]))
            layer.norm2.weight.copy_(t(Lw["ln2_g"][m * Hd:(m + 1) * Hd])); layer.norm2.bias.copy_(t(Lw["ln2_b"][m * Hd:(m + 1) * Hd]))
            want = layer(t(inp["X"][m])[None])[0].numpy()
        close(got[m], want, tol=1e-5)


def test_resnet_chain_matches_torch_functional(oracle):
    """The bottleneck forward (stem, max-pool, blocks with projection shortcuts, average pool) equals
    the same network evaluated model by model with torch's conv2d / batch_norm / pools."""
    from oracle import models as OM
    M = 2
    for card, bw in [(1, 64), (4, 16)]:
        spec = NI.resnet_spec(cardinality=card, base_width=bw, image=32, width_div=8, depths=(2, 1, 1, 1))
        inp = NI.resnet_params(spec, M, bf16=False)
        got = OM.resnet_forward(inp, spec, M, out_bf16=False)
        P = inp["params"]
        for m in range(M):
            def cb(x, c, relu):
                p = P[c.name]
                sl = slice(m * c.cout, (m + 1) * c.cout)
                t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).double()
                y = F.conv2d(x, t(p["w"][sl]), stride=c.stride, padding=c.pad, groups=c.groups)
                y = F.batch_norm(y, t(p["mean"][sl]), t(p["var"][sl]), t(p["gamma"][sl]), t(p["beta"][sl]),
                                 training=False, eps=1e-5)
                return F.relu(y) if relu else y
            x = torch.from_numpy(inp["x"][:, 3 * m:3 * (m + 1)]).double()
            x = F.max_pool2d(cb(x, spec.stem, True), 3, 2, 1)
            for blk in spec.blocks:
                y = cb(cb(cb(x, blk.conv1, True), blk.conv2, True), blk.conv3, False)
                sc = cb(x, blk.down, False) if blk.down else x
                x = F.relu(y + sc)
            want = x.mean(dim=(2, 3)).numpy()
            C = spec.out_channels
            close(got[:, C * m:C * (m + 1)], want, tol=1e-5)


def test_network_shape_tables():
    """ResNet-50 has 53 convolutions; ResNeXt-50 32x4d has 3x3 widths 128/256/512/1024 with 32 groups."""
    r50 = NI.resnet_spec()
    assert len(r50.convs()) == 53 and r50.out_channels == 2048
    assert sum(c.cout * (c.cin // c.groups) * c.k * c.k for c in r50.convs()) == 23454912
    x50 = NI.resnet_spec(cardinality=32, base_width=4)
    widths = sorted({c.cin for c in x50.convs() if c.k == 3})
    assert widths == [128, 256, 512, 1024]
    assert all(c.groups == 32 for c in x50.convs() if c.k == 3)
    assert sorted({c.cin // c.groups for c in x50.convs() if c.k == 3}) == [4, 8, 16, 32]


# ------------------------------------------------------------------ ragged per-task heads
def test_linear_ragged_is_the_per_model_definition(oracle):
    """Per-model output widths: against a numpy float64 product per model, and against the uniform-width
    operator when all widths agree."""
    r = np.random.default_rng(5)
    M, N, K = 4, 3, 37
    nout = [1, 10, 65, 7]
    X = r.standard_normal((M, N, K)).astype(np.float32)
    Ws = [r.standard_normal((K, n)).astype(np.float32) for n in nout]
    bs = [r.standard_normal(n).astype(np.float32) for n in nout]
    got = oracle.linear_ragged(X, Ws, bs, act=oracle.ACT_RELU)
    for m in range(M):
        want = np.maximum(X[m].astype(np.float64) @ Ws[m].astype(np.float64) + bs[m], 0.0)
        assert got[m].shape == (N, nout[m])
        np.testing.assert_allclose(got[m], want, rtol=1e-6, atol=1e-6)
    same = [r.standard_normal((K, 6)).astype(np.float32) for _ in range(M)]
    uni = oracle.linear(X, np.stack(same))
    for m, y in enumerate(oracle.linear_ragged(X, same)):
        assert np.array_equal(y, uni[m])


# ------------------------------------------------------------------ relative-position attention
def _rel_shift_reference(qkv, Kr, S, heads, bias_w, bias_r, scale, mask):
    """The same operator by the published procedure instead of the closed-form index: the raw position
    scores against ALL 2S encodings (distances S, S-1, ..., -S+1), then XLNet's "relative shift": view the
    [S, 2S] block as [2S, S], drop the first row, view the rest as [S, 2S-1], keep the first S columns."""
    M, N, th = qkv.shape
    Hd = th // 3
    d = Hd // heads
    out = np.zeros((M, N, Hd))
    for m in range(M):
        for h in range(heads):
            c = slice(h * d, (h + 1) * d)
            q, k, v = (qkv[m, :, i * Hd:(i + 1) * Hd][:, c].astype(np.float64) for i in range(3))
            ac = (q + bias_w[m, c]) @ k.T
            raw = (q + bias_r[m, c]) @ Kr[m, :, c].astype(np.float64).T                    # [S, 2S]
            bd = raw.reshape(2 * S, S)[1:].reshape(S, 2 * S - 1)[:, :S]
            s = scale * (ac + bd) + mask[m, 0][None, :]
            p = np.exp(s - s.max(axis=1, keepdims=True))
            out[m, :, c] = (p / p.sum(axis=1, keepdims=True)) @ v
    return out


def test_attention_relpos_against_the_relative_shift_procedure_and_special_cases(oracle):
    """No number for this operator exists in the reference paper (it only says XLNet has extra computations):
    the oracle is pinned to the Transformer-XL relative-shift procedure, to plain attention when the position
    term vanishes, and to a distance-only closed form."""
    M, S, heads, d = 2, 7, 2, 4
    Hd = heads * d
    qkv, Kr = rnd(M, S, 3 * Hd), rnd(M, 2 * S, Hd)
    bw, br, mask = rnd(M, Hd), rnd(M, Hd), rnd(M, 1, S)
    got = oracle.attention_relpos_packed(qkv, Kr, 1, S, heads, bias_w=bw, bias_r=br, scale=0.37, mask=mask)
    close(got, _rel_shift_reference(qkv, Kr, S, heads, bw, br, 0.37, mask))
    # no position term, no biases: the plain merged attention (pinned above against torch)
    zero = np.zeros_like(Kr)
    close(oracle.attention_relpos_packed(qkv, zero, 1, S, heads), oracle.attention_packed(qkv, 1, S, heads))
    # bias_w alone adds bw.k_j to every row of scores; with identical keys that is a constant: no effect
    same_k = qkv.copy()
    same_k[:, :, Hd:2 * Hd] = same_k[:, :1, Hd:2 * Hd]
    close(oracle.attention_relpos_packed(same_k, zero, 1, S, heads, bias_w=bw), oracle.attention_packed(same_k, 1, S, heads))
    # Q = 0, K = 0, bias_r = e_0, Kr[p] = g(S - p) e_0: the weights depend on the distance i - j only
    q0 = np.zeros_like(qkv)
    q0[:, :, 2 * Hd:] = qkv[:, :, 2 * Hd:]
    g = rnd(2 * S)
    Krd = np.zeros_like(Kr)
    Krd[:, :, 0::d] = g[None, :, None]
    e0 = np.zeros((M, Hd), np.float32)
    e0[:, 0::d] = 1.0
    got = oracle.attention_relpos_packed(q0, Krd, 1, S, heads, bias_r=e0, scale=1.0)
    for i in range(S):
        w = np.exp(np.array([g[S - i + j] for j in range(S)], np.float64))
        w /= w.sum()
        close(got[0, i, :d], w @ q0[0, :, 2 * Hd:2 * Hd + d].astype(np.float64))
    # two sequences per model are independent problems
    two = np.concatenate([qkv, qkv[:, ::-1]], axis=1)
    both = oracle.attention_relpos_packed(two, Kr, 2, S, heads, bias_w=bw, bias_r=br)
    close(both[:, :S], oracle.attention_relpos_packed(qkv, Kr, 1, S, heads, bias_w=bw, bias_r=br))
