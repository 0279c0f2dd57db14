"""GPU parity of the packed-weight merged matmul: the packed layout is what include/netfuse.h states
(checked byte for byte against an index formula written here), and netfuse_linear_packed agrees with the
oracle (on the unpacked weights) and, up to the fp32 summation order, with netfuse_linear."""
import numpy as np
import pytest
import torch

import netfuse_inputs as NI
from test_gpu_parity import check, dev, host, nf, rnd  # noqa: F401  (nf is a fixture)

pytestmark = pytest.mark.gpu
BF = torch.bfloat16


def packed_reference(W):
    """Wp[m][j][s][l][e] = W[m][16 s + 8 (l / 32) + e][32 j + l % 32], written with numpy reshapes."""
    M, K, Nout = W.shape
    v = W.reshape(M, K // 16, 2, 8, Nout // 32, 32)                     # m s h e j c   (lane l = 32 h + c)
    return np.ascontiguousarray(v.transpose(0, 4, 1, 2, 5, 3)).reshape(M, K, Nout)


@pytest.mark.parametrize("M,K,Nout", [(2, 64, 96), (3, 96, 384), (1, 16, 32), (2, 128, 768)])
def test_pack_layout_is_the_documented_one(nf, M, K, Nout):
    W = NI.on_bf16_grid(rnd(M, K, Nout))
    got = host(nf.linear_pack_weight(dev(W, BF)))
    assert np.array_equal(got, packed_reference(W))
    # and element by element from the formula itself, on a few entries
    flat = got.reshape(M, Nout // 32, K // 16, 64, 8)
    for (m, j, s, l, e) in [(0, 0, 0, 0, 0), (M - 1, Nout // 32 - 1, K // 16 - 1, 63, 7), (0, 1 % (Nout // 32), 0, 37, 3)]:
        assert flat[m, j, s, l, e] == W[m, 16 * s + 8 * (l // 32) + e, 32 * j + l % 32]


PACKED_CASES = [
    # M, N, K, Nout, bias, residual, act; the tile each shape is routed to is named beside it
    (32, 128, 768, 2304, True, False, 0),     # QKV projection: 128 x 288 tiles, 9 waves
    (32, 128, 768, 3072, True, False, 2),     # FFN1 + GELU: 128 x 384 tiles, 12 waves
    (32, 128, 3072, 768, True, True, 0),      # FFN2 + residual: 128 x 96 tiles, four k-groups reduced through LDS
    (32, 128, 768, 768, True, True, 0),       # output projection: 128 x 96 tiles
    (32, 512, 768, 768, True, True, 0),       # four row tiles per model
    (8, 512, 768, 3072, True, False, 2),
    (3, 256, 256, 96, False, True, 1),        # K = one round of the four-stage pipeline (k-steps of 64), ReLU
    (3, 128, 128, 288, False, False, 0),      # K = one round at k-steps of 32
    (5, 128, 512, 384, True, True, 2),
    (2, 128, 768, 2304, True, False, 0),      # few models
    # 256 rows per model and more, 256-column multiples: 256 x 256 tiles with the packed fragments staged through LDS
    (32, 512, 768, 3072, True, False, 2),     # three column tiles per workgroup, GELU
    (32, 512, 768, 2304, True, False, 0),     # three column tiles per workgroup
    (32, 512, 3072, 768, True, True, 0),      # one tile per workgroup, long k, residual
    (2, 256, 64, 512, True, True, 1),         # only this kernel fits 512 columns; K shorter than the pipeline
    (3, 256, 96, 1024, False, True, 2),
    (1, 768, 160, 256, True, False, 0),       # three row tiles of one model
    # widths that only the 128- and 256-column fragment tiles divide (a BERT-large-shaped layer)
    (16, 128, 1024, 1024, True, True, 0),
    (8, 128, 1024, 4096, True, False, 2),
    (3, 128, 256, 640, False, True, 1),       # five tiles of 128
    # 64-row tiles (fewer models: one round of 129 ... 256 workgroups instead of half a round of 128-row tiles)
    (16, 128, 768, 2304, True, False, 0),     # 64 x 288
    (16, 128, 768, 3072, True, False, 2),     # 64 x 384, GELU
    (16, 128, 3072, 768, True, True, 0),      # 64 x 96, two k-groups reduced through LDS, residual
    (16, 128, 768, 768, True, True, 1),       # 64 x 96, ReLU before the residual
    (8, 256, 768, 768, False, True, 0),       # four 64-row tiles per model
    (43, 192, 256, 96, True, False, 0),       # three 64-row tiles per model: rows no 128-row tile divides
]


@pytest.mark.parametrize("case", PACKED_CASES, ids=lambda c: "x".join(map(str, c[:4])))
def test_linear_packed(nf, oracle, case):
    M, N, K, Nout, use_b, use_r, act = case
    X, W = NI.on_bf16_grid(rnd(M, N, K)), NI.on_bf16_grid(rnd(M, K, Nout, std=K ** -0.5))
    b = rnd(M, Nout, std=0.5) if use_b else None
    R = NI.on_bf16_grid(rnd(M, N, Nout)) if use_r else None
    sample = sorted({0, M // 3, M - 1})                       # models the oracle evaluates
    ref = oracle.linear(X[sample], W[sample], bias=None if b is None else b[sample],
                        residual=None if R is None else R[sample], act=act, out_bf16=True)
    Xd, Wd = dev(X, BF), dev(W, BF)
    bd, Rd = (None if b is None else dev(b)), (None if R is None else dev(R, BF))
    Wp = nf.linear_pack_weight(Wd)
    got = nf.linear_packed(Xd, Wp, bias=bd, residual=Rd, act=act)
    check(host(got[sample]), ref, BF, "linear_packed %s" % (case[:4],))
    # against the unpacked entry point over ALL models: the same products summed in another order in fp32
    # (error of a few 1e-7 of the largest partial sum), so a bf16 result may differ by one unit in the last
    # place, and only rarely
    plain = nf.linear(Xd, Wd, bias=bd, residual=Rd, act=act).float()
    diff = (got.float() - plain).abs()
    assert float((diff > 0).float().mean()) < 0.02
    assert bool((diff <= 2.0 ** -7 * plain.abs() + 4e-6 * float(plain.abs().max())).all())


def test_linear_packed_isolates_models(nf):
    """NaN weights and inputs of every other model leave model m's packed result bit-identical."""
    M, N, K, Nout, keep = 4, 128, 256, 384, 1
    X, W = NI.on_bf16_grid(rnd(M, N, K)), NI.on_bf16_grid(rnd(M, K, Nout, std=0.1))
    clean = nf.linear_packed(dev(X, BF), nf.linear_pack_weight(dev(W, BF)))
    Xp, Wp = X.copy(), W.copy()
    for m in range(M):
        if m != keep:
            Xp[m], Wp[m] = np.nan, np.inf
    dirty = nf.linear_packed(dev(Xp, BF), nf.linear_pack_weight(dev(Wp, BF)))
    assert torch.equal(clean[keep], dirty[keep])
    assert not torch.isfinite(dirty[(keep + 1) % M].float()).any()


def test_linear_packed_refuses_what_it_cannot_run(nf):
    X = torch.zeros(2, 100, 64, device="cuda", dtype=BF)
    Wp = torch.zeros(2, 64, 96, device="cuda", dtype=BF)
    with pytest.raises(nf.NetFuseError) as e:
        nf.linear_packed(X, Wp)
    assert e.value.status == nf.NF_EUNSUPPORTED
    assert not nf.linear_packed_supported(2, 100, 64, 96)
    assert not nf.linear_packed_supported(2, 128, 64, 96)             # K shorter than one pipeline round
