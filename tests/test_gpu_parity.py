"""GPU parity: every entry point of the C ABI (through the thin binding) against the CPU oracle,
element by element, on the same seeded inputs.

Bar: layout/indexing exact (index-coded and poison tests compare bit patterns); floating point
within   |gpu - ref| <= tol*|ref| + tol*rms(ref)   with tol = 1e-4 for float32 storage and 2e-2 for
bf16 storage with fp32 accumulation.
"""
import numpy as np
import pytest
import torch

import netfuse_inputs as NI

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}


@pytest.fixture(scope="module")
def nf():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2009_13062_amd as nf_
    return nf_


def dev(a, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda", dtype).contiguous()


def host(t):
    torch.cuda.synchronize()
    return t.detach().float().cpu().numpy()


def grid(a, dtype):
    """Host copy of what the device holds: bf16 storage rounds the inputs once."""
    return NI.on_bf16_grid(a) if dtype == torch.bfloat16 else np.ascontiguousarray(a, np.float32)


def check(got, ref, dtype, what=""):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), what + ": non-finite output"
    tol = TOL[dtype]
    rms = float(np.sqrt(np.mean(ref * ref)))
    bound = tol * np.abs(ref) + tol * rms
    err = np.abs(got - ref)
    bad = err > bound
    assert not bad.any(), "%s: %d/%d outside tolerance, worst err %.3e at %s (ref %.4e, rms %.3e)" % (
        what, int(bad.sum()), bad.size, float(err.max()), np.unravel_index(int(err.argmax()), err.shape),
        float(ref.flat[int(err.argmax())]), rms)


rng = np.random.default_rng(77)


def rnd(*shape, std=1.0, mean=0.0):
    return (mean + std * rng.standard_normal(shape)).astype(np.float32)


DTYPES = [torch.float32, torch.bfloat16]
ids = lambda d: "f32" if d == torch.float32 else "bf16"


# ------------------------------------------------------------------ workload 1 at M in {1,2,8,32}
@pytest.mark.parametrize("dtype", DTYPES, ids=ids)
@pytest.mark.parametrize("M", [1, 2, 8, 32])
def test_tiny_layer(nf, oracle, M, dtype):
    from oracle import models as OM
    from paper_2009_13062_amd.workloads import TinyLayer
    bf = dtype == torch.bfloat16
    inp = NI.tiny_layer(M, bf16=bf)
    ref = OM.tiny_layer(inp, M, out_bf16=bf)
    got = TinyLayer(inp, M, dtype).forward()
    check(host(got["linear"]), ref["linear"], dtype, "linear")
    # per call on identical inputs: LN is fed the GPU's own linear output
    ref_ln = oracle.layernorm(host(got["linear"]), inp["gamma"], inp["beta"], M, eps=1e-5, out_bf16=bf)
    check(host(got["layernorm"]), ref_ln, dtype, "layernorm")
    check(host(got["conv"]), ref["conv"], dtype, "conv")
    check(host(got["layernorm"]), ref["layernorm"], dtype, "linear->layernorm chain")


# ------------------------------------------------------------------ linear
LIN_CASES = [
    # M, N, K, Nout, bias, residual, act
    (3, 200, 264, 328, True, True, 2),       # several tiles + ragged tails, GELU, residual
    (2, 128, 768, 2304, True, False, 0),     # the QKV projection of one encoder layer
    (2, 512, 768, 768, True, True, 0),       # 4 row tiles
    (1, 130, 3072, 768, True, True, 0),      # long K
    (5, 33, 100, 50, True, False, 1),        # rows of 200/100 bytes: 8-byte / 4-byte aligned loaders
    (4, 7, 9, 11, False, True, 0),           # odd everything: element-wise loaders
    (2, 300, 72, 136, False, False, 0),      # K not a multiple of 64
    (32, 8, 64, 64, True, False, 0),
    (3, 70, 256, 100, True, True, 0),        # deep load pipeline, weight rows at odd 4-byte addresses, last chunk crosses the operand end
    (2, 200, 512, 77, True, False, 2),       # the same with rows at 2-byte addresses and the 8-wave tile
    (2, 96, 256, 256, True, True, 0),        # deep pipeline, aligned
    (64, 128, 2048, 256, True, False, 0),    # direct-to-LDS 128 x 128 tile with k-steps of 64 (long K, narrow layer)
    (40, 256, 96, 384, False, True, 1),      # direct-to-LDS 128 x 128 tile with k-steps of 32; fewer k-steps than stages
]


@pytest.mark.parametrize("dtype", DTYPES, ids=ids)
@pytest.mark.parametrize("case", LIN_CASES, ids=lambda c: "x".join(map(str, c[:4])))
def test_linear(nf, oracle, case, dtype):
    M, N, K, Nout, use_b, use_r, act = case
    bf = dtype == torch.bfloat16
    X, W = grid(rnd(M, N, K), dtype), grid(rnd(M, K, Nout, std=K ** -0.5), dtype)
    b = rnd(M, Nout, std=0.5) if use_b else None
    R = grid(rnd(M, N, Nout), dtype) if use_r else None
    ref = oracle.linear(X, W, bias=b, residual=R, act=act, out_bf16=bf)
    got = nf.linear(dev(X, dtype), dev(W, dtype), bias=None if b is None else dev(b),
                    residual=None if R is None else dev(R, dtype), act=act)
    check(host(got), ref, dtype, "linear %s" % (case,))


@pytest.mark.parametrize("dtype", DTYPES, ids=ids)
@pytest.mark.parametrize("M,N,K,nout", [
    (5, 3, 100, [10, 1000, 2, 65, 64]),            # widths around the 64-column tile, a one-tile and a 16-tile model
    (32, 1, 768, None),                            # one sequence per model, encoder heads of 2..20 classes
    (16, 9, 2048, [1000, 10, 100, 1] * 4),         # ResNet heads, two row tiles, a single-output model
    (1, 8, 33, [7]),                               # one model
], ids=["mixed", "encoder-heads", "resnet-heads", "single"])
def test_linear_ragged(nf, oracle, M, N, K, nout, dtype):
    """The per-task output layers (a different width per model) as one launch: every model against the
    oracle's per-model definition, and nothing written outside a model's block."""
    bf = dtype == torch.bfloat16
    if nout is None:
        nout = [int(v) for v in rng.integers(2, 21, M)]
    X = grid(rnd(M, N, K), dtype)
    Ws = [grid(rnd(K, n, std=K ** -0.5), dtype) for n in nout]
    bs = [rnd(n, std=0.5) for n in nout]
    ref = oracle.linear_ragged(X, Ws, bs, act=1, out_bf16=bf)
    Wd = dev(np.concatenate([w.ravel() for w in Ws]), dtype)
    bd = dev(np.concatenate(bs))
    Y = nf.linear_ragged(dev(X, dtype), Wd, nout, bias=bd, act=1)
    for m, y in enumerate(nf.ragged_views(Y, N, nout)):
        check(host(y), ref[m], dtype, "ragged model %d (%d outputs)" % (m, nout[m]))
    # without bias and activation, poisoned neighbours: model 1 (or 0) stays bit-identical
    keep = min(1, M - 1)
    clean = nf.linear_ragged(dev(X, dtype), Wd, nout)
    Xp = X.copy()
    Xp[[m for m in range(M) if m != keep]] = np.nan
    dirty = nf.linear_ragged(dev(Xp, dtype), Wd, nout)
    assert torch.equal(nf.ragged_views(clean, N, nout)[keep], nf.ragged_views(dirty, N, nout)[keep])


def test_linear_residual_may_alias_output(nf, oracle):
    M, N, K, Nout = 2, 150, 128, 256
    X, W, R = (NI.on_bf16_grid(a) for a in (rnd(M, N, K), rnd(M, K, Nout, std=0.1), rnd(M, N, Nout)))
    ref = oracle.linear(X, W, residual=R, out_bf16=True)
    buf = dev(R, torch.bfloat16)
    nf.linear(dev(X, torch.bfloat16), dev(W, torch.bfloat16), residual=buf, out=buf)
    check(host(buf), ref, torch.bfloat16, "in-place residual")


@pytest.mark.parametrize("dtype", DTYPES, ids=ids)
def test_linear_output_rounding_and_indexing_exact(nf, oracle, dtype):
    """Integer-coded inputs: every product and sum is exact in fp32, so the output must match the
    oracle bit for bit -- any wrong index, model mix-up or double rounding shows."""
    M, N, K, Nout = 3, 70, 40, 136
    X = rng.integers(-4, 5, (M, N, K)).astype(np.float32)
    W = rng.integers(-3, 4, (M, K, Nout)).astype(np.float32)
    b = rng.integers(-8, 9, (M, Nout)).astype(np.float32)
    ref = oracle.linear(X, W, bias=b, out_bf16=dtype == torch.bfloat16)
    got = host(nf.linear(dev(X, dtype), dev(W, dtype), bias=dev(b)))
    assert np.array_equal(got, ref)


# ------------------------------------------------------------------ convolution
CONV_CASES = [
    # M, B, Cin, Cout, g, H, W, KH, KW, stride, pad, dil
    (2, 1, 64, 64, 1, 14, 14, 3, 3, 1, 1, 1),      # ResNet 3x3
    (2, 1, 64, 128, 1, 28, 28, 1, 1, 1, 0, 1),     # pointwise, HW % 8 == 0
    (3, 1, 64, 256, 1, 14, 14, 1, 1, 1, 0, 1),     # pointwise, HW = 196 (8-byte rows)
    (2, 1, 128, 96, 1, 7, 7, 1, 1, 1, 0, 1),       # pointwise, HW = 49 (2-byte rows)
    (3, 2, 256, 96, 1, 7, 7, 1, 1, 1, 0, 1),       # the same through the deep load pipeline (K % 256 == 0): last chunk of the last plane
    (2, 1, 512, 192, 1, 14, 14, 1, 1, 1, 0, 1),    # deep pipeline, HW = 196, two column tiles
    (2, 1, 256, 64, 1, 3, 3, 1, 1, 1, 0, 1),       # deep pipeline, rows of 9 elements
    (2, 1, 256, 64, 1, 2, 3, 1, 1, 1, 0, 1),       # rows shorter than a chunk: the deep pipeline does not apply
    (2, 1, 3, 64, 1, 32, 32, 7, 7, 2, 3, 1),       # stem: Cin 3, K = 147 (odd rows of weights)
    (2, 1, 128, 256, 1, 16, 16, 1, 1, 2, 0, 1),    # strided projection shortcut, Wo % 4 == 0: 4 pixel pairs per load
    (2, 2, 72, 96, 1, 24, 40, 1, 1, 2, 0, 1),      # the same, non-square, K not a multiple of the k step, ragged columns
    (3, 1, 64, 128, 1, 14, 28, 1, 1, 2, 0, 1),     # strided projection, Wo = 14: 2 pixel pairs per load
    (2, 1, 64, 128, 1, 14, 14, 1, 1, 2, 0, 1),     # strided projection, Wo = 7: element gather
    (2, 2, 128, 256, 1, 14, 14, 1, 1, 2, 0, 1),    # strided projection, Wo = 7: one input row per task, 8-wave tile
    (3, 1, 256, 64, 1, 14, 14, 1, 1, 2, 0, 1),     # the same on the 64x64 tile (two tasks per thread)
    (2, 1, 128, 256, 1, 10, 14, 1, 1, 2, 0, 1),    # the same with 5 output rows
    (2, 1, 128, 256, 1, 10, 10, 1, 1, 2, 0, 1),    # strided projection, Wo = 5: one pixel pair per load through the deep pipeline
    (2, 1, 128, 256, 1, 12, 12, 1, 1, 2, 0, 1),    # strided projection, Wo = 6: two pixel pairs per load through the deep pipeline
    (2, 1, 64, 128, 1, 15, 15, 1, 1, 2, 0, 1),     # strided projection, odd width
    (2, 1, 64, 64, 1, 12, 12, 1, 1, 3, 0, 1),      # pointwise, stride 3
    (2, 1, 64, 64, 1, 16, 16, 3, 3, 2, 1, 1),      # strided 3x3
    (2, 1, 128, 128, 32, 14, 14, 3, 3, 1, 1, 1),   # ResNeXt: 4 channels per group, 64 groups merged
    (2, 2, 32, 64, 4, 9, 11, 3, 3, 1, 1, 1),       # batch 2 per model, non-square image
    (1, 1, 16, 24, 1, 10, 10, 3, 3, 1, 2, 2),      # dilation 2
    (3, 1, 8, 200, 2, 5, 5, 2, 3, 1, 1, 1),        # non-square kernel, 100 outputs per group
    (2, 1, 128, 256, 1, 28, 28, 3, 3, 1, 1, 1),    # patch-gather 3x3: two 128-channel row tiles, 7 position tiles
    (3, 2, 32, 32, 2, 7, 7, 3, 3, 1, 1, 1),        # patch-gather, 16 channels per group, image smaller than a tile
    (1, 1, 64, 64, 1, 56, 56, 3, 3, 1, 1, 1),      # patch-gather, 58-wide patch, tiles that start mid-row
    (2, 1, 64, 128, 1, 30, 30, 3, 3, 2, 1, 1),     # patch-gather, stride 2, odd output width 15
    (2, 1, 48, 64, 1, 12, 12, 3, 3, 1, 0, 1),      # patch-gather, no padding, 3 channel blocks
    (2, 2, 64, 80, 1, 7, 7, 3, 3, 1, 1, 1),        # tap-major 3x3: 1-pixel chunks, ragged row tile, batch 2
    (2, 1, 96, 64, 1, 12, 20, 3, 3, 1, 0, 1),      # tap-major 3x3: 3 channel blocks, no padding, non-square, 4-pixel chunks
    (1, 1, 32, 32, 1, 28, 28, 3, 3, 2, 1, 1),      # tap-major 3x3: stride 2, three patch tasks per thread
    (1, 1, 32, 64, 1, 56, 56, 3, 3, 2, 1, 1),      # tap-major 3x3: stride 2, 8-pixel chunks, two patch tasks per thread
    (3, 1, 64, 64, 8, 28, 28, 3, 3, 1, 1, 1),      # fused narrow groups: 8 channels per group, 4 groups per block
    (2, 2, 64, 64, 4, 16, 16, 3, 3, 2, 1, 1),      # fused narrow groups: 16 per group, stride 2, batch 2
    (1, 1, 32, 32, 8, 56, 56, 3, 3, 1, 1, 1),      # fused narrow groups: 4 per group on a 56x56 image
    (3, 1, 3, 64, 1, 56, 56, 7, 7, 2, 3, 1),       # stem kernel: 28-wide output, tiles that start mid-row
    (2, 2, 3, 96, 1, 24, 40, 7, 7, 2, 3, 1),       # stem kernel: batch 2, non-square image, a partial second row tile
    (2, 1, 3, 64, 1, 30, 30, 7, 7, 2, 3, 1),       # stem shape whose rows are not whole 16-byte chunks (gathering loader)
]


@pytest.mark.parametrize("dtype", DTYPES, ids=ids)
@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: "-".join(map(str, c)))
def test_conv2d(nf, oracle, case, dtype):
    M, B, Cin, Cout, g, H, W, KH, KW, stride, pad, dil = case
    bf = dtype == torch.bfloat16
    cig = Cin // g
    x = grid(rnd(B, M * Cin, H, W), dtype)
    w = grid(rnd(M * Cout, cig, KH, KW, std=(cig * KH * KW) ** -0.5), dtype)
    scale, shift = rnd(M * Cout, std=0.1, mean=1.0), rnd(M * Cout, std=0.1)
    Ho, Wo = oracle.conv_out_size(H, KH, stride, pad, dil), oracle.conv_out_size(W, KW, stride, pad, dil)
    res = grid(rnd(B, M * Cout, Ho, Wo), dtype)
    ref = oracle.conv2d(x, w, M, g=g, scale=scale, shift=shift, residual=res, stride=stride, pad=pad,
                        dil=dil, act=1, out_bf16=bf)
    got = nf.conv2d(dev(x, dtype), dev(w, dtype), M, g=g, scale=dev(scale), shift=dev(shift),
                    residual=dev(res, dtype), stride=stride, pad=pad, dil=dil, act=1)
    check(host(got), ref, dtype, "conv %s" % (case,))
    bias = rnd(M * Cout)
    ref = oracle.conv2d(x, w, M, g=g, bias=bias, stride=stride, pad=pad, dil=dil, out_bf16=bf)
    got = nf.conv2d(dev(x, dtype), dev(w, dtype), M, g=g, bias=dev(bias), stride=stride, pad=pad, dil=dil)
    check(host(got), ref, dtype, "conv+bias %s" % (case,))


@pytest.mark.parametrize("dtype", DTYPES, ids=ids)
def test_conv_reads_exactly_its_group(nf, oracle, dtype):
    """x = merged channel index, one-hot weights: the output names the input channel that was read
    (Appendix A: x[Cin*m + ci] = x_m[ci], y_m[co] = y[Cout*m + co], group = c / (Cout/g))."""
    M, g, Cin, Cout, H = 4, 2, 64, 64, 6
    cig, cog = Cin // g, Cout // g
    x = np.broadcast_to(np.arange(M * Cin, dtype=np.float32)[None, :, None, None], (1, M * Cin, H, H)).copy()
    for k, pad in ((1, 0), (3, 1)):
        w = np.zeros((M * Cout, cig, k, k), np.float32)
        pick = rng.integers(0, cig, M * Cout)
        w[np.arange(M * Cout), pick, k // 2, k // 2] = 1.0
        got = host(nf.conv2d(dev(x, dtype), dev(w, dtype), M, g=g, pad=pad))
        want = ((np.arange(M * Cout) // cog) * cig + pick).astype(np.float32)
        assert np.array_equal(got, np.broadcast_to(want[None, :, None, None], got.shape))
        assert np.array_equal(got, oracle.conv2d(x, w, M, g=g, pad=pad))


def test_maxpool_stem_shape_bf16(nf, oracle):
    """3x3 / stride 2 / pad 1 on rows of 8k pixels takes the four-outputs-per-thread kernel: exact, edges
    (odd height, first and last columns), all-negative windows and NaN inputs included."""
    dtype = torch.bfloat16
    for (B, C, H, W) in ((1, 6, 16, 24), (2, 3, 15, 8), (1, 2, 112, 112)):
        x = rnd(B, C, H, W)
        x[0, 0] = -np.abs(x[0, 0]) - 1.0
        x = grid(x, dtype)
        x[0, 1, 3, 5] = np.nan
        x[0, 1, 0, 0] = np.nan
        got, ref = host(nf.maxpool2d(dev(x, dtype), 3, 2, 1)), oracle.maxpool2d(x, 3, 2, 1)
        assert got.shape == ref.shape and np.array_equal(got, ref, equal_nan=True), (B, C, H, W)


def test_linear_equals_pointwise_conv_on_gpu(nf):
    """Section 3.1: a matmul is a 1x1 convolution -- both entry points, same numbers."""
    M, N, K, Nout = 3, 64, 128, 96
    X, W = NI.on_bf16_grid(rnd(M, N, K)), NI.on_bf16_grid(rnd(M, K, Nout, std=0.1))
    lin = host(nf.linear(dev(X, torch.bfloat16), dev(W, torch.bfloat16)))
    x = np.concatenate([X[m].T for m in range(M)]).reshape(1, M * K, 8, 8)
    w = np.concatenate([W[m].T for m in range(M)]).reshape(M * Nout, K, 1, 1)
    y = host(nf.conv2d(dev(x, torch.bfloat16), dev(w, torch.bfloat16), M))
    for m in range(M):
        check(y[0, m * Nout:(m + 1) * Nout].reshape(Nout, N).T, lin[m], torch.bfloat16, "1x1 conv vs linear")


# ------------------------------------------------------------------ norms
@pytest.mark.parametrize("dtype", DTYPES, ids=ids)
@pytest.mark.parametrize("M,rows,H", [(8, 128, 768), (3, 5, 50), (2, 3, 3000), (2, 4, 1028), (32, 8, 64), (32, 512, 64)])
def test_layernorm_both_layouts(nf, oracle, M, rows, H, dtype):
    bf = dtype == torch.bfloat16
    x, r = grid(rnd(M, rows, H, std=2.0, mean=0.5), dtype), grid(rnd(M, rows, H), dtype)
    gam, bet = rnd(M * H, std=0.1, mean=1.0), rnd(M * H, std=0.1)
    for res in (None, r):
        ref = oracle.layernorm(x, gam, bet, M, residual=res, eps=1e-5, out_bf16=bf)
        got = nf.layernorm(dev(x, dtype), dev(gam), dev(bet), M, residual=None if res is None else dev(res, dtype))
        check(host(got), ref, dtype, "layernorm batch layout")
        xc = oracle.merge_transpose(x, M, True)
        rc = None if res is None else oracle.merge_transpose(res, M, True)
        refc = oracle.layernorm(xc, gam, bet, M, residual=rc, eps=1e-5, layout=oracle.LAYOUT_CHANNEL, out_bf16=bf)
        gotc = nf.layernorm(dev(xc, dtype), dev(gam), dev(bet), M, residual=None if rc is None else dev(rc, dtype),
                            layout=nf.MERGE_CHANNEL)
        check(host(gotc), refc, dtype, "layernorm channel layout")
        # the two layouts hold the same numbers (Section 3.2's reshape between bmm and group norm)
        assert torch.equal(nf.merge_transpose(got, M, True), gotc)
    xd = dev(x, dtype)
    inplace = nf.layernorm(xd, dev(gam), dev(bet), M, out=xd)
    check(host(inplace), oracle.layernorm(x, gam, bet, M, out_bf16=bf), dtype, "in-place")


@pytest.mark.parametrize("dtype", DTYPES, ids=ids)
def test_batchnorm_fold_pools_transpose(nf, oracle, dtype):
    bf = dtype == torch.bfloat16
    M, C, B, H, W = 3, 20, 2, 9, 7
    x, res = grid(rnd(B, M * C, H, W), dtype), grid(rnd(B, M * C, H, W), dtype)
    g, b, mu = rnd(M * C, std=0.1, mean=1.0), rnd(M * C, std=0.1), rnd(M * C, std=0.1)
    var = rng.uniform(0.5, 1.5, M * C).astype(np.float32)
    ref = oracle.batchnorm(x, g, b, mu, var, M, residual=res, act=1, out_bf16=bf)
    got = nf.batchnorm(dev(x, dtype), dev(g), dev(b), dev(mu), dev(var), M, residual=dev(res, dtype), act=1)
    check(host(got), ref, dtype, "batchnorm")
    s_ref, t_ref = oracle.bn_fold(g, b, mu, var)
    s_got, t_got = nf.bn_fold(dev(g), dev(b), dev(mu), dev(var))
    check(host(s_got), s_ref, torch.float32, "bn_fold scale")
    check(host(t_got), t_ref, torch.float32, "bn_fold shift")
    for (k, s, p) in ((3, 2, 1), (2, 2, 0), (3, 1, 1)):
        assert np.array_equal(host(nf.maxpool2d(dev(x, dtype), k, s, p)), oracle.maxpool2d(x, k, s, p)), (k, s, p)
    neg = grid(-np.abs(x) - 1.0, dtype)
    assert np.array_equal(host(nf.maxpool2d(dev(neg, dtype), 3, 2, 1)), oracle.maxpool2d(neg, 3, 2, 1))
    check(host(nf.avgpool_global(dev(x, dtype))), oracle.avgpool_global(x, out_bf16=bf), dtype, "avgpool")
    src = grid(rnd(4, 6, 10), dtype)
    t = nf.merge_transpose(dev(src, dtype), 4, True)
    assert np.array_equal(host(t), oracle.merge_transpose(src, 4, True))
    assert np.array_equal(host(nf.merge_transpose(t, 4, False)), src)


@pytest.mark.parametrize("dtype", DTYPES, ids=ids)
@pytest.mark.parametrize("M,C,B,H,W", [(2, 3, 1, 40, 40), (3, 5, 2, 7, 7), (2, 4, 1, 14, 14), (2, 3, 1, 1, 3), (2, 8, 1, 56, 56)],
                         ids=["1600", "49", "196", "3-unaligned", "3136"])
def test_batchnorm_plane_sizes(nf, oracle, M, C, B, H, W, dtype):
    """Planes longer than a workgroup pass (HW > 1024), planes that end inside a 16-byte chunk (49, 196), a tensor
    whose size is no multiple of the chunk (the per-plane kernel), with and without residual, in place."""
    bf = dtype == torch.bfloat16
    x, res = grid(rnd(B, M * C, H, W), dtype), grid(rnd(B, M * C, H, W), dtype)
    g, b, mu = rnd(M * C, std=0.1, mean=1.0), rnd(M * C, std=0.1), rnd(M * C, std=0.1)
    var = rng.uniform(0.5, 1.5, M * C).astype(np.float32)
    for r in (None, res):
        ref = oracle.batchnorm(x, g, b, mu, var, M, residual=r, act=1, out_bf16=bf)
        got = nf.batchnorm(dev(x, dtype), dev(g), dev(b), dev(mu), dev(var), M, residual=None if r is None else dev(r, dtype), act=1)
        check(host(got), ref, dtype, "batchnorm %s" % ((M, C, B, H, W),))
    xd = dev(x, dtype)
    nf.batchnorm(xd, dev(g), dev(b), dev(mu), dev(var), M, out=xd)
    check(host(xd), oracle.batchnorm(x, g, b, mu, var, M, out_bf16=bf), dtype, "in place")


# ------------------------------------------------------------------ attention
@pytest.mark.parametrize("dtype,M,B,S,heads,d,use_mask", [
    (torch.bfloat16, 2, 1, 128, 12, 64, False),     # workload 2/5 shape
    (torch.bfloat16, 2, 2, 200, 3, 64, True),       # ragged keys and queries, two sequences, mask
    (torch.bfloat16, 1, 1, 512, 2, 64, False),      # several query blocks, 8 key stages
    (torch.bfloat16, 2, 1, 37, 2, 64, True),        # shorter than one stage
    (torch.bfloat16, 2, 1, 70, 3, 32, True),        # head dim without an MFMA kernel: general path
    (torch.float32, 2, 2, 75, 3, 16, True),
    (torch.float32, 1, 1, 130, 2, 80, False),
], ids=lambda v: str(v).replace("torch.", ""))
def test_attention(nf, oracle, dtype, M, B, S, heads, d, use_mask):
    bf = dtype == torch.bfloat16
    qkv = grid(rnd(M, B * S, 3 * heads * d), dtype)
    mask = rnd(M, B, S, std=2.0) if use_mask else None
    ref = oracle.attention_packed(qkv, B, S, heads, mask=mask, out_bf16=bf)
    got = nf.attention_packed(dev(qkv, dtype), B, S, heads, mask=None if mask is None else dev(mask))
    check(host(got), ref, dtype, "attention packed")
    Hd = heads * d
    Q, K, V = (np.ascontiguousarray(qkv[:, :, i * Hd:(i + 1) * Hd]) for i in range(3))
    got2 = nf.attention(dev(Q, dtype), dev(K, dtype), dev(V, dtype), B, S, heads, mask=None if mask is None else dev(mask))
    assert torch.equal(got, got2), "packed and separate Q/K/V must agree bit for bit"


@pytest.mark.parametrize("dtype,M,B,S,heads,d", [(torch.bfloat16, 2, 1, 48, 3, 64), (torch.bfloat16, 3, 2, 70, 2, 32),
                                               (torch.bfloat16, 2, 1, 128, 2, 64),      # one full query block, two key blocks
                                               (torch.bfloat16, 1, 2, 200, 1, 64),      # ragged second query block, four key blocks
                                               (torch.bfloat16, 1, 1, 300, 1, 64),      # three query blocks: bands that start below row 0
                                               (torch.float32, 2, 1, 33, 2, 16), (torch.float32, 1, 1, 5, 1, 80)],
                         ids=lambda v: str(v).replace("torch.", ""))
def test_attention_relpos(nf, oracle, dtype, M, B, S, heads, d):
    """Relative-position attention (the XLNet / Transformer-XL score) per (model, sequence, head); with a zero
    position term it is the plain merged attention; NaN in another model stays there."""
    bf = dtype == torch.bfloat16
    Hd = heads * d
    qkv, Kr = grid(rnd(M, B * S, 3 * Hd), dtype), grid(rnd(M, 2 * S, Hd), dtype)
    bw, br, mask = rnd(M, Hd, std=0.5), rnd(M, Hd, std=0.5), rnd(M, B, S, std=2.0)
    ref = oracle.attention_relpos_packed(qkv, Kr, B, S, heads, bias_w=bw, bias_r=br, mask=mask, out_bf16=bf)
    got = nf.attention_relpos_packed(dev(qkv, dtype), dev(Kr, dtype), B, S, heads, bias_w=dev(bw), bias_r=dev(br), mask=dev(mask))
    check(host(got), ref, dtype, "relative-position attention")
    nobias = nf.attention_relpos_packed(dev(qkv, dtype), dev(Kr, dtype), B, S, heads)
    check(host(nobias), oracle.attention_relpos_packed(qkv, Kr, B, S, heads, out_bf16=bf), dtype, "no biases, no mask")
    plain = nf.attention_packed(dev(qkv, dtype), B, S, heads)
    zero = nf.attention_relpos_packed(dev(qkv, dtype), dev(np.zeros_like(Kr), dtype), B, S, heads)
    check(host(zero), host(plain), dtype, "zero position term")
    if M > 1:
        qp, kp = qkv.copy(), Kr.copy()
        qp[1:], kp[1:] = np.nan, np.nan
        dirty = nf.attention_relpos_packed(dev(qp, dtype), dev(kp, dtype), B, S, heads, bias_w=dev(bw), bias_r=dev(br), mask=dev(mask))
        assert torch.equal(dirty[0], got[0]) and not torch.isfinite(dirty[1].float()).any()


def test_attention_sharp_softmax(nf, oracle):
    """Large logits: the row maximum must be subtracted, and one key must win exactly."""
    M, S, heads, d = 2, 96, 2, 64
    qkv = rnd(M, S, 3 * heads * d)
    qkv[:, :, :2 * heads * d] *= 6.0
    qkv = NI.on_bf16_grid(qkv)
    ref = oracle.attention_packed(qkv, 1, S, heads, out_bf16=True)
    got = nf.attention_packed(dev(qkv, torch.bfloat16), 1, S, heads)
    check(host(got), ref, torch.bfloat16, "sharp softmax")


# ------------------------------------------------------------------ invariants on the GPU
@pytest.mark.parametrize("dtype", DTYPES, ids=ids)
def test_models_are_isolated_and_order_is_free(nf, dtype):
    """Poisoning every other model leaves model m's output bit-identical; permuting the models
    permutes the outputs (each weight set touches only its own input: Section 3, Appendix A)."""
    M, keep = 4, 2
    N, K, Nout, heads, d = 70, 128, 192, 3, 64
    X, W = rnd(M, N, K), rnd(M, K, Nout, std=0.1)
    gam, bet = rnd(M * Nout, mean=1.0, std=0.1), rnd(M * Nout, std=0.1)
    cx, cw = rnd(1, M * 64, 10, 10), rnd(M * 64, 64, 3, 3, std=0.05)
    qkv = rnd(M, 80, 3 * heads * d)

    def run(X, W, gam, bet, cx, cw, qkv):
        y = nf.linear(dev(X, dtype), dev(W, dtype))
        z = nf.layernorm(y, dev(gam), dev(bet), M)
        c = nf.conv2d(dev(cx, dtype), dev(cw, dtype), M, pad=1)
        p = nf.conv2d(dev(cx, dtype), dev(cw[:, :, 1:2, 1:2].copy(), dtype), M)
        a = nf.attention_packed(dev(qkv, dtype), 1, 80, heads)
        torch.cuda.synchronize()
        return y, z, c, p, a

    clean = run(X, W, gam, bet, cx, cw, qkv)
    Xp, Wp, gp, cxp, cwp, qp = X.copy(), W.copy(), gam.copy(), cx.copy(), cw.copy(), qkv.copy()
    for m in range(M):
        if m != keep:
            Xp[m], Wp[m], qp[m] = np.nan, np.inf, np.nan
            gp[m * Nout:(m + 1) * Nout] = np.nan
            cxp[0, m * 64:(m + 1) * 64] = np.nan
            cwp[m * 64:(m + 1) * 64] = np.inf
    dirty = run(Xp, Wp, gp, bet, cxp, cwp, qp)
    for a, b in zip(clean[:2] + clean[4:], dirty[:2] + dirty[4:]):
        assert torch.equal(a[keep], b[keep])
        assert not torch.isfinite(b[(keep + 1) % M].float()).any()
    for a, b in zip(clean[2:4], dirty[2:4]):
        assert torch.equal(a[0, keep * 64:(keep + 1) * 64], b[0, keep * 64:(keep + 1) * 64])
    perm = [3, 0, 2, 1]
    gperm = np.concatenate([gam[p * Nout:(p + 1) * Nout] for p in perm])
    bperm = np.concatenate([bet[p * Nout:(p + 1) * Nout] for p in perm])
    cxperm = np.concatenate([cx[:, p * 64:(p + 1) * 64] for p in perm], axis=1)
    cwperm = np.concatenate([cw[p * 64:(p + 1) * 64] for p in perm])
    permd = run(X[perm], W[perm], gperm, bperm, cxperm, cwperm, qkv[perm])
    for i, p in enumerate(perm):
        for a, b in zip(clean[:2] + clean[4:], permd[:2] + permd[4:]):
            assert torch.equal(b[i], a[p])
        for a, b in zip(clean[2:4], permd[2:4]):
            assert torch.equal(b[0, i * 64:(i + 1) * 64], a[0, p * 64:(p + 1) * 64])


@pytest.mark.parametrize("Cin,g", [(16, 1), (16, 2), (32, 4), (32, 8), (24, 3)], ids=lambda v: str(v))
def test_narrow_group_convs_isolate_models(nf, Cin, g):
    """3x3 convolutions with fewer than 32 channels per group (the block-diagonal fused kernels and what
    replaces them when a fused block would span two models): NaN / infinity in every other model's input
    and weights leaves model m's output bit-identical and finite (Section 3: a weight set meets only its
    own input)."""
    M, keep, H = 3, 1, 12
    x, w = rnd(1, M * Cin, H, H), rnd(M * Cin, Cin // g, 3, 3, std=0.1)
    clean = nf.conv2d(dev(x, torch.bfloat16), dev(w, torch.bfloat16), M, g=g, pad=1)
    xp, wp = x.copy(), w.copy()
    for m in range(M):
        if m != keep:
            xp[0, m * Cin:(m + 1) * Cin] = np.nan
            wp[m * Cin:(m + 1) * Cin] = np.inf
    dirty = nf.conv2d(dev(xp, torch.bfloat16), dev(wp, torch.bfloat16), M, g=g, pad=1)
    torch.cuda.synchronize()
    sl = slice(keep * Cin, (keep + 1) * Cin)
    assert torch.isfinite(dirty[0, sl].float()).all()
    assert torch.equal(clean[0, sl], dirty[0, sl])
    assert not torch.isfinite(dirty[0, :Cin].float()).any()


def test_merged_equals_m_separate_launches_bitwise(nf):
    """The merged call and M calls with M = 1 on the slices run the same arithmetic per model."""
    from paper_2009_13062_amd.workloads import EncoderStack
    M = 3
    shape = NI.EncoderShape(hidden=128, heads=2, ffn=256, layers=2, seq=96)
    inp = NI.encoder_stack(M, shape, bf16=True)
    enc = EncoderStack.from_numpy(inp, M, 1, shape.seq, shape.heads)
    X = dev(inp["X"], torch.bfloat16)
    merged = enc.forward(X).clone()
    for m, one in enumerate(enc.per_model()):
        out = one.forward(X[m:m + 1])
        assert torch.equal(out[0], merged[m])


def test_graph_replay_equals_eager_forward(nf):
    """What bench.py times is a captured HIP graph of the forward: its replays (several, with eager work and
    synchronisations between them, on fresh inputs) give the eager result bit for bit."""
    from paper_2009_13062_amd.workloads import EncoderStack, ResNetForward
    M = 4
    shape = NI.EncoderShape(hidden=256, heads=4, ffn=1024, layers=2, seq=128)
    inp = NI.encoder_stack(M, shape, bf16=True)
    enc = EncoderStack.from_numpy(inp, M, 1, shape.seq, shape.heads)
    spec = NI.resnet_spec(cardinality=8, base_width=8, image=64, width_div=2, depths=(1, 1, 1, 1))
    rinp = NI.resnet_params(spec, M, bf16=True)
    net = ResNetForward.from_numpy(rinp, spec, M)
    # and the configuration bench.py times: packed weights, 32 models, one full-size layer
    from netfuse_inputs.device import encoder_stack_device
    pshape = NI.EncoderShape(layers=1, seq=128)
    pinp = encoder_stack_device(32, pshape, cfg=5)
    penc = EncoderStack(pinp["layers"], 32, 1, pshape.seq, pshape.heads, packed=True)
    assert all(k + "_p" in penc.layers[0] for k in ("Wqkv", "Wo", "W1", "W2"))
    for fwd, x0 in ((enc.forward, dev(inp["X"], torch.bfloat16)), (net.forward, dev(rinp["x"], torch.bfloat16)),
                    (penc.forward, pinp["X"])):
        x = x0.clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fwd(x)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            out = fwd(x)
        for rep in range(4):
            x.copy_(x0 * (1.0 + 0.25 * rep))              # new input values in the captured buffer
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            replayed = out.clone()
            eager = fwd(x).clone()                        # the program's own eager work between replays
            torch.cuda.synchronize()
            assert torch.equal(replayed, eager), "replay %d differs from the eager forward" % rep
            assert torch.isfinite(eager.float()).all()


def test_runs_are_bit_reproducible(nf):
    X, W = dev(rnd(4, 256, 512), torch.bfloat16), dev(rnd(4, 512, 384, std=0.05), torch.bfloat16)
    a = nf.linear(X, W, act=2).clone()
    for _ in range(3):
        assert torch.equal(nf.linear(X, W, act=2), a)


# ------------------------------------------------------------------ whole workloads, reduced and full size
def _encoder_per_call_parity(oracle, trace_layer, X_in, Lw_host, m_list, batch, seq, heads, dtype, R=None):
    """Each call of one layer against the oracle on the GPU's own input to that call.  R: the relative position
    encodings of an XLNet-shaped layer (position projection, then attention with the position term)."""
    bf = dtype == torch.bfloat16
    t = {k: host(v[m_list]) for k, v in trace_layer.items()}
    X = host(X_in[m_list])
    M = len(m_list)
    L = Lw_host
    check(t["qkv"], oracle.linear(X, L["Wqkv"], bias=L["bqkv"], out_bf16=bf), dtype, "qkv")
    if R is None:
        check(t["att"], oracle.attention_packed(t["qkv"], batch, seq, heads, out_bf16=bf), dtype, "attention")
    else:
        Rrep = np.broadcast_to(R, (M,) + R.shape).copy()
        check(t["kr"], oracle.linear(Rrep, L["Wr"], out_bf16=bf), dtype, "position projection")
        check(t["att"], oracle.attention_relpos_packed(t["qkv"], t["kr"], batch, seq, heads, bias_w=L["rwb"], bias_r=L["rrb"],
                                                       out_bf16=bf), dtype, "relative attention")
    check(t["h"], oracle.linear(t["att"], L["Wo"], bias=L["bo"], residual=X, out_bf16=bf), dtype, "o-proj")
    check(t["x1"], oracle.layernorm(t["h"], L["ln1_g"], L["ln1_b"], M, out_bf16=bf), dtype, "ln1")
    check(t["f1"], oracle.linear(t["x1"], L["W1"], bias=L["b1"], act=2, out_bf16=bf), dtype, "ffn1+gelu")
    check(t["f2"], oracle.linear(t["f1"], L["W2"], bias=L["b2"], residual=t["x1"], out_bf16=bf), dtype, "ffn2")
    check(t["x2"], oracle.layernorm(t["f2"], L["ln2_g"], L["ln2_b"], M, out_bf16=bf), dtype, "ln2")


def _slice_layer(Lw, m_list, Hd):
    out = {}
    for k, v in Lw.items():
        if k.endswith("_p"):
            continue                                   # packed weight copies: the oracle takes the originals
        if k.startswith("ln"):
            v = torch.cat([v[m * Hd:(m + 1) * Hd] for m in m_list])
        else:
            v = v[m_list]
        out[k] = host(v)
    return out


def test_encoder_layer_workload2_full_size(nf, oracle):
    """Workload 2 as specified: M = 8, one sequence of 128 per model, hidden 768, 12 heads, FFN 3072,
    bf16: every call of the layer checked for all 8 models, then the chain end to end."""
    from oracle import models as OM
    from paper_2009_13062_amd.workloads import EncoderStack
    M, shape = 8, NI.EncoderShape(layers=1, seq=128)
    inp = NI.encoder_stack(M, shape, cfg=2, bf16=True)
    enc = EncoderStack.from_numpy(inp, M, 1, shape.seq, shape.heads)
    X = dev(inp["X"], torch.bfloat16)
    trace = []
    out = enc.forward(X, trace)
    _encoder_per_call_parity(oracle, trace[0], X, _slice_layer(enc.layers[0], list(range(M)), shape.hidden),
                             list(range(M)), 1, shape.seq, shape.heads, torch.bfloat16)
    ref = OM.encoder_stack(inp, M, 1, shape.seq, shape.heads, out_bf16=True)
    err = np.abs(host(out) - ref)
    # end to end the two chains round differently at every call; LN output is O(1)
    print("end-to-end max abs err %.4f mean %.5f" % (float(err.max()), float(err.mean())))
    assert float(err.max()) < 0.15 and float(err.mean()) < 0.01, (float(err.max()), float(err.mean()))


@pytest.mark.parametrize("seq,packed,rel", [(128, False, False), (128, True, False), (512, False, False), (512, True, False),
                                            (128, True, True)])
def test_encoder_stack_workload5_full_size_sampled(nf, oracle, seq, packed, rel):
    """Workload 5 in the configurations bench.py times: M = 32, 12 layers, hidden 768, bf16, on row-major and
    on packed weights (bench.py's default), and the XLNet-shaped stack.  The first and last layers are checked
    call by call for sampled models on the GPU's own inputs; then the whole 12-layer chain of sampled models
    against the oracle run on the seeded inputs alone."""
    from netfuse_inputs.device import encoder_stack_device
    from oracle import models as OM
    from paper_2009_13062_amd.workloads import EncoderStack
    M, shape = 32, NI.EncoderShape(layers=12, seq=seq)
    inp = encoder_stack_device(M, shape, cfg=5, rel=rel)
    enc = EncoderStack(inp["layers"], M, 1, seq, shape.heads, packed=packed, R=inp.get("R"))
    assert not packed or all(k + "_p" in enc.layers[0] for k in ("Wqkv", "Wo", "W1", "W2"))
    Rh = host(inp["R"]) if rel else None
    trace = []
    out = enc.forward(inp["X"], trace)
    assert torch.isfinite(out.float()).all()
    sample = [0, 13, 31]
    for li in (0, 11):
        X_in = inp["X"] if li == 0 else trace[li - 1]["x2"]
        _encoder_per_call_parity(oracle, trace[li], X_in, _slice_layer(enc.layers[li], sample, shape.hidden),
                                 sample, 1, seq, shape.heads, torch.bfloat16, R=Rh)
    # end to end: nothing of the expected value comes from the GPU path
    e2e = [0, 31] if seq == 128 else [13]
    sub = dict(X=host(inp["X"][e2e]), layers=[_slice_layer(Lw, e2e, shape.hidden) for Lw in enc.layers])
    if rel:
        sub["R"] = Rh
    ref = OM.encoder_stack(sub, len(e2e), 1, seq, shape.heads, out_bf16=True)
    err = np.abs(host(out[e2e]) - ref)
    print("end-to-end over 12 layers: max abs err %.4f mean %.5f" % (float(err.max()), float(err.mean())))
    assert float(err.max()) < 0.15 and float(err.mean()) < 0.012, (float(err.max()), float(err.mean()))
    # merged == one model at a time, bit for bit, on a sampled model
    # (row-major weights only: every kernel of that path sums k in the same order whatever tile it picks, while
    # the packed kernels split k over wavefronts for some model counts and not for others)
    if not packed:
        one = enc.per_model()[17]
        ref17 = out[17].clone()
        assert torch.equal(one.forward(inp["X"][17:18])[0], ref17)


def _resnet_per_call_parity(oracle, net, x, spec, m_list, dtype=torch.bfloat16):
    """Each op of the forward against the oracle on the GPU's own input to that op, model by model
    (model m's slice run alone through the oracle with M = 1)."""
    M = net.M

    def sl(t, m):
        ch = t.shape[1] // M
        return host(t[:, m * ch:(m + 1) * ch])

    def conv(c, xin, m, act, res=None):
        p = net.P[c.name]
        s = slice(m * c.cout, (m + 1) * c.cout)
        scale, shift = oracle.bn_fold(host(p["gamma"][s]), host(p["beta"][s]), host(p["mean"][s]), host(p["var"][s]))
        ref = oracle.conv2d(sl(xin, m), host(p["w"][s]), 1, g=c.groups, scale=scale, shift=shift,
                            residual=None if res is None else sl(res, m), stride=c.stride, pad=c.pad,
                            act=act, out_bf16=True)
        check(sl(net.buf[c.name], m), ref, dtype, "%s model %d" % (c.name, m))

    for m in m_list:
        conv(spec.stem, x, m, 1)
        assert np.array_equal(sl(net.buf["maxpool"], m), oracle.maxpool2d(sl(net.buf["stem"], m), 3, 2, 1))
        cur = net.buf["maxpool"]
        for blk in spec.blocks:
            conv(blk.conv1, cur, m, 1)
            conv(blk.conv2, net.buf[blk.conv1.name], m, 1)
            if blk.down is not None:
                conv(blk.down, cur, m, 0)
                scb = net.buf[blk.down.name]
            else:
                scb = cur
            conv(blk.conv3, net.buf[blk.conv2.name], m, 1, res=scb)
            cur = net.buf[blk.conv3.name]
        C = spec.out_channels
        check(host(net.buf["avgpool"][:, m * C:(m + 1) * C]), oracle.avgpool_global(sl(cur, m), out_bf16=True),
              dtype, "avgpool")


@pytest.mark.parametrize("card,bw", [(1, 64), (8, 8)], ids=["resnet", "resnext"])
def test_resnet_reduced(nf, oracle, card, bw):
    """A narrow, shallow bottleneck network (all op kinds of workloads 3/4) for every model, plus
    the end-to-end chain against the oracle's own chain."""
    from oracle import models as OM
    from paper_2009_13062_amd.workloads import ResNetForward
    M = 3
    spec = NI.resnet_spec(cardinality=card, base_width=bw, image=64, width_div=2, depths=(2, 1, 1, 1))
    inp = NI.resnet_params(spec, M, bf16=True)
    net = ResNetForward.from_numpy(inp, spec, M)
    x = dev(inp["x"], torch.bfloat16)
    out = net.forward(x)
    _resnet_per_call_parity(oracle, net, x, spec, list(range(M)))
    ref = OM.resnet_forward(inp, spec, M, out_bf16=True)
    err = np.abs(host(out) - ref)
    assert float(err.max()) < 0.1 * max(1.0, float(np.abs(ref).max())), float(err.max())
    for m, one in enumerate(net.per_model()):
        assert torch.equal(one.forward(net.slice_input(x, m)), out[:, m * spec.out_channels:(m + 1) * spec.out_channels])


@pytest.mark.parametrize("batch", [2, 4])
@pytest.mark.parametrize("card,bw", [(1, 64), (8, 8)], ids=["resnet", "resnext"])
def test_resnet_reduced_batch_per_model(nf, oracle, card, bw, batch):
    """Several images per model (Section 5.2's batch-size experiment): tensors are [batch, M*C, H, W], so a
    model's channels are no longer one contiguous run.  Every op for every model against the oracle, the
    chain end to end, and merged == one model at a time bit for bit."""
    from oracle import models as OM
    from paper_2009_13062_amd.workloads import ResNetForward
    M = 3
    spec = NI.resnet_spec(cardinality=card, base_width=bw, image=64, width_div=2, depths=(1, 1, 1, 1))
    inp = NI.resnet_params(spec, M, bf16=True, batch=batch)
    net = ResNetForward.from_numpy(inp, spec, M, batch=batch)
    x = dev(inp["x"], torch.bfloat16)
    out = net.forward(x)
    assert out.shape == (batch, M * spec.out_channels)
    _resnet_per_call_parity(oracle, net, x, spec, list(range(M)))
    ref = OM.resnet_forward(inp, spec, M, out_bf16=True)
    err = np.abs(host(out) - ref)
    print("end-to-end max abs err %.4f (max |ref| %.3f)" % (float(err.max()), float(np.abs(ref).max())))
    assert float(err.max()) < 0.1 * max(1.0, float(np.abs(ref).max())), float(err.max())
    for m, one in enumerate(net.per_model()):
        assert torch.equal(one.forward(net.slice_input(x, m)), out[:, m * spec.out_channels:(m + 1) * spec.out_channels])


@pytest.mark.parametrize("batch", [2, 4])
def test_encoder_reduced_batch_per_model(nf, oracle, batch):
    """Several sequences per model: N = batch * seq rows per matmul, attention per (model, sequence, head)."""
    from oracle import models as OM
    from paper_2009_13062_amd.workloads import EncoderStack
    M = 3
    shape = NI.EncoderShape(hidden=256, heads=4, ffn=512, layers=2, seq=96, batch=batch)
    inp = NI.encoder_stack(M, shape, bf16=True)
    enc = EncoderStack.from_numpy(inp, M, batch, shape.seq, shape.heads)
    X = dev(inp["X"], torch.bfloat16)
    trace = []
    out = enc.forward(X, trace)
    for li in range(shape.layers):
        X_in = X if li == 0 else trace[li - 1]["x2"]
        _encoder_per_call_parity(oracle, trace[li], X_in, _slice_layer(enc.layers[li], list(range(M)), shape.hidden),
                                 list(range(M)), batch, shape.seq, shape.heads, torch.bfloat16)
    ref = OM.encoder_stack(inp, M, batch, shape.seq, shape.heads, out_bf16=True)
    err = np.abs(host(out) - ref)
    print("end-to-end max abs err %.4f mean %.5f" % (float(err.max()), float(err.mean())))
    assert float(err.max()) < 0.15 and float(err.mean()) < 0.01
    for m, one in enumerate(enc.per_model()):
        assert torch.equal(one.forward(X[m:m + 1])[0], out[m])


def test_encoder_with_relative_position_attention(nf, oracle):
    """XLNet-shaped layers: the position projection as one more merged matmul, then the relative-position
    attention; every call against the oracle, the chain end to end, merged == one model at a time."""
    from oracle import models as OM
    from paper_2009_13062_amd.workloads import EncoderStack
    M = 3
    shape = NI.EncoderShape(hidden=128, heads=2, ffn=256, layers=2, seq=40)
    inp = NI.encoder_stack(M, shape, bf16=True, rel=True)
    enc = EncoderStack.from_numpy(inp, M, 1, shape.seq, shape.heads)
    X = dev(inp["X"], torch.bfloat16)
    trace = []
    out = enc.forward(X, trace)
    bf = torch.bfloat16
    for li, Lw in enumerate(inp["layers"]):
        t = {k: host(v) for k, v in trace[li].items()}
        Rrep = np.broadcast_to(inp["R"], (M,) + inp["R"].shape).copy()
        check(t["kr"], oracle.linear(Rrep, Lw["Wr"], out_bf16=True), bf, "position projection")
        check(t["att"], oracle.attention_relpos_packed(t["qkv"], t["kr"], 1, shape.seq, shape.heads, bias_w=Lw["rwb"],
                                                       bias_r=Lw["rrb"], out_bf16=True), bf, "relative attention")
    ref = OM.encoder_stack(inp, M, 1, shape.seq, shape.heads, out_bf16=True)
    err = np.abs(host(out) - ref)
    print("end-to-end max abs err %.4f mean %.5f" % (float(err.max()), float(err.mean())))
    assert float(err.max()) < 0.15 and float(err.mean()) < 0.01
    for m, one in enumerate(enc.per_model()):
        assert torch.equal(one.forward(X[m:m + 1])[0], out[m])


@pytest.mark.parametrize("name,M,card,bw,cfg", [("resnet50", 32, 1, 64, 3), ("resnext50_32x4d", 16, 32, 4, 4)])
def test_resnet_full_size_sampled(nf, oracle, name, M, card, bw, cfg):
    """Workloads 3 and 4 at full size (224x224, M = 32 / 16, merged groups 32 / 512 on the 3x3 convs):
    every op checked for a sampled model on the GPU's own inputs."""
    from netfuse_inputs.device import resnet_params_device
    from paper_2009_13062_amd.workloads import ResNetForward
    spec = NI.resnet_spec(cardinality=card, base_width=bw)
    inp = resnet_params_device(spec, M, cfg=cfg)
    net = ResNetForward(spec, inp["params"], M)
    out = net.forward(inp["x"])
    assert torch.isfinite(out.float()).all()
    _resnet_per_call_parity(oracle, net, inp["x"], spec, [0, M // 2, M - 1])
    # end to end for one model: nothing of the expected value comes from the GPU path
    from oracle import models as OM
    m = M // 2
    P = {}
    for c in spec.convs():
        sl = slice(m * c.cout, (m + 1) * c.cout)
        P[c.name] = {k: host(v[sl]) for k, v in inp["params"][c.name].items()}
    ref = OM.resnet_forward(dict(x=host(inp["x"][:, 3 * m:3 * m + 3]), params=P), spec, 1, out_bf16=True)
    C = spec.out_channels
    err = np.abs(host(out[:, m * C:(m + 1) * C]) - ref)
    print("end-to-end over %d convolutions: max abs err %.4f, max |ref| %.3f" % (len(spec.convs()), float(err.max()), float(np.abs(ref).max())))
    assert float(err.max()) < 0.1 * max(1.0, float(np.abs(ref).max())), float(err.max())


# ------------------------------------------------------------------ degenerate and extreme shapes
@pytest.mark.parametrize("dtype", DTYPES, ids=ids)
def test_degenerate_shapes(nf, oracle, dtype):
    """Single rows, single features, single keys, one-pixel images, depthwise groups."""
    bf = dtype == torch.bfloat16
    for (M, N, K, Nout) in [(1, 1, 1, 1), (3, 1, 8, 8), (2, 9, 1, 16), (2, 16, 64, 1)]:
        X, W, b = grid(rnd(M, N, K), dtype), grid(rnd(M, K, Nout), dtype), rnd(M, Nout)
        check(host(nf.linear(dev(X, dtype), dev(W, dtype), bias=dev(b))),
              oracle.linear(X, W, bias=b, out_bf16=bf), dtype, "linear %s" % ((M, N, K, Nout),))
    # H = 1: the variance is zero, the output is beta; rows = 1
    x, g, b = grid(rnd(3, 1, 1), dtype), rnd(3), rnd(3)
    check(host(nf.layernorm(dev(x, dtype), dev(g), dev(b), 3)), oracle.layernorm(x, g, b, 3, out_bf16=bf), dtype, "LN H=1")
    # one key: softmax is 1, O = V; head dim 1
    for (S, heads, d) in [(1, 2, 64), (1, 1, 1), (5, 2, 1)]:
        qkv = grid(rnd(2, S, 3 * heads * d), dtype)
        check(host(nf.attention_packed(dev(qkv, dtype), 1, S, heads)),
              oracle.attention_packed(qkv, 1, S, heads, out_bf16=bf), dtype, "attention S=%d d=%d" % (S, d))
    # 1x1 image with a 3x3 kernel and padding; depthwise (one channel per group); 1x1 image pointwise
    for (M, Cin, Cout, g_, H, k, pad) in [(2, 16, 16, 1, 1, 3, 1), (2, 8, 8, 8, 5, 3, 1), (3, 4, 6, 2, 1, 1, 0)]:
        x = grid(rnd(1, M * Cin, H, H), dtype)
        w = grid(rnd(M * Cout, Cin // g_, k, k, std=0.3), dtype)
        check(host(nf.conv2d(dev(x, dtype), dev(w, dtype), M, g=g_, pad=pad)),
              oracle.conv2d(x, w, M, g=g_, pad=pad, out_bf16=bf), dtype, "conv %s" % ((M, Cin, Cout, g_, H, k),))
    x = grid(rnd(1, 6, 1, 1), dtype)
    assert np.array_equal(host(nf.maxpool2d(dev(x, dtype), 3, 2, 1)), oracle.maxpool2d(x, 3, 2, 1))
    check(host(nf.avgpool_global(dev(x, dtype))), oracle.avgpool_global(x, out_bf16=bf), dtype, "avgpool HW=1")


def test_many_small_problems_and_long_rows(nf, oracle):
    """Grid-size extremes: 4096 models of a tiny matmul; one LayerNorm row of 65536 features."""
    M = 4096
    X, W = NI.on_bf16_grid(rnd(M, 4, 16)), NI.on_bf16_grid(rnd(M, 16, 8, std=0.25))
    check(host(nf.linear(dev(X, torch.bfloat16), dev(W, torch.bfloat16))), oracle.linear(X, W, out_bf16=True),
          torch.bfloat16, "4096 models")
    H = 65536
    x, g, b = rnd(1, 2, H), rnd(H, mean=1.0, std=0.1), rnd(H, std=0.1)
    check(host(nf.layernorm(dev(x), dev(g), dev(b), 1)), oracle.layernorm(x, g, b, 1), torch.float32, "LN H=65536")


def test_errors_leave_outputs_untouched(nf):
    """A rejected call enqueues nothing."""
    X = torch.zeros(2, 4, 8, device="cuda", dtype=torch.bfloat16)
    W = torch.zeros(2, 8, 8, device="cuda", dtype=torch.bfloat16)
    Y = torch.full((2, 4, 8), 7.0, device="cuda", dtype=torch.bfloat16)
    st = nf.lib.netfuse_linear(X.data_ptr(), W.data_ptr(), None, None, Y.data_ptr(), 2, 4, 8, 8, 1, 99, None)
    assert st == nf.NF_EINVAL
    with pytest.raises(nf.NetFuseError):
        nf.conv2d(torch.zeros(1, 6, 4, 4, device="cuda"), torch.zeros(6, 3, 3, 3, device="cuda"), 2, dil=0)
    torch.cuda.synchronize()
    assert torch.all(Y == 7.0)
