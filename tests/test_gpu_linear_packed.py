"""GPU parity of the packed-weight merged matmul: the packed layout is what include/netfuse.h states
(checked byte for byte against an index formula written here), and netfuse_linear_packed equals both the
oracle (on the unpacked weights) and netfuse_linear bit for bit."""
import numpy as np
import pytest
import torch

import netfuse_inputs as NI
from test_gpu_parity import check, dev, host, nf, rnd  # noqa: F401  (nf is a fixture)

pytestmark = pytest.mark.gpu
BF = torch.bfloat16


def packed_reference(W, panel):
    """Wp[m][p][kb][j][r][c] = W[m][32 kb + r][panel p + 32 j + c], written with numpy reshapes."""
    M, K, Nout = W.shape
    v = W.reshape(M, K // 32, 32, Nout // panel, panel // 32, 32)       # m kb r p j c
    return np.ascontiguousarray(v.transpose(0, 3, 1, 4, 2, 5)).reshape(M, K, Nout)


@pytest.mark.parametrize("M,K,Nout,panel", [(2, 64, 96, 96), (3, 96, 384, 128), (1, 32, 32, 32), (2, 128, 768, 768)])
def test_pack_layout_is_the_documented_one(nf, M, K, Nout, panel):
    W = NI.on_bf16_grid(rnd(M, K, Nout))
    got = host(nf.linear_pack_weight(dev(W, BF), panel))
    assert np.array_equal(got, packed_reference(W, panel))


PACKED_CASES = [
    # M, N, K, Nout, bias, residual, act, panels to try (0 = the library's own choice); the tile each shape
    # is routed to is named beside it (M = 32 so that the cost model takes the wide tiles, as in the workloads)
    (32, 128, 768, 2304, True, False, 0, (0, 2304)),    # QKV projection: 128 x 288 tiles
    (32, 128, 768, 3072, True, False, 2, (0, 3072)),    # FFN1 + GELU: 128 x 384 tiles
    (32, 128, 3072, 768, True, True, 0, (0, 768)),      # FFN2 + residual: 128 x 96 tiles, k-steps of 64
    (32, 128, 768, 768, True, True, 0, (0, 384)),       # output projection: 128 x 96 tiles
    (32, 512, 768, 768, True, True, 0, (0, 768)),       # 256 x 256 tiles
    (8, 512, 768, 3072, True, False, 2, (0,)),          # 256 x 256 tiles, GELU: register epilogue, one tile per workgroup
    (32, 512, 768, 3072, True, False, 2, (0, 768)),     # the same at 32 models: three tiles per workgroup through one pipeline
    (32, 512, 768, 2304, True, True, 0, (0, 2304)),     # 576 tiles of 256 x 256: runs as three 128 x 384 tiles per workgroup
    (64, 128, 2048, 256, False, False, 0, (0,)),        # long K, narrow: the 128 x 128 tile with k-steps of 64
    (40, 256, 96, 384, True, False, 1, (0, 128)),       # 128 x 128 tiles, k-steps of 32, K = 3 k-blocks (fewer than stages)
    (2, 128, 32, 128, False, True, 0, (128,)),          # a single k-block
    (2, 128, 64, 96, False, True, 0, (96,)),            # a single k-step of 64
    (2, 128, 768, 2304, True, False, 0, (2304,)),       # few models
]


@pytest.mark.parametrize("case", PACKED_CASES, ids=lambda c: "x".join(map(str, c[:4])))
def test_linear_packed(nf, oracle, case):
    M, N, K, Nout, use_b, use_r, act, panels = case
    X, W = NI.on_bf16_grid(rnd(M, N, K)), NI.on_bf16_grid(rnd(M, K, Nout, std=K ** -0.5))
    b = rnd(M, Nout, std=0.5) if use_b else None
    R = NI.on_bf16_grid(rnd(M, N, Nout)) if use_r else None
    sample = sorted({0, M // 3, M - 1})                       # models the oracle evaluates
    ref = oracle.linear(X[sample], W[sample], bias=None if b is None else b[sample],
                        residual=None if R is None else R[sample], act=act, out_bf16=True)
    Xd, Wd = dev(X, BF), dev(W, BF)
    bd, Rd = (None if b is None else dev(b)), (None if R is None else dev(R, BF))
    plain = nf.linear(Xd, Wd, bias=bd, residual=Rd, act=act)
    for panel in panels:
        if panel == 0:
            # 0 from the library = it prefers its small-tile kernel for the unpacked call at this model count;
            # any whole-tile width is still accepted by the packed entry
            panel = nf.linear_packed_panel(M, N, K, Nout) or Nout
        Wp = nf.linear_pack_weight(Wd, panel)
        got = nf.linear_packed(Xd, Wp, panel, bias=bd, residual=Rd, act=act)
        check(host(got[sample]), ref, BF, "linear_packed %s panel %d" % (case[:4], panel))
        assert torch.equal(got, plain), "packed and unpacked weights must give the same bits"


def test_linear_packed_isolates_models(nf):
    """NaN weights and inputs of every other model leave model m's packed result bit-identical."""
    M, N, K, Nout, keep = 4, 128, 256, 384, 1
    X, W = NI.on_bf16_grid(rnd(M, N, K)), NI.on_bf16_grid(rnd(M, K, Nout, std=0.1))
    panel = nf.linear_packed_panel(M, N, K, Nout) or Nout
    clean = nf.linear_packed(dev(X, BF), nf.linear_pack_weight(dev(W, BF), panel), panel)
    Xp, Wp = X.copy(), W.copy()
    for m in range(M):
        if m != keep:
            Xp[m], Wp[m] = np.nan, np.inf
    dirty = nf.linear_packed(dev(Xp, BF), nf.linear_pack_weight(dev(Wp, BF), panel), panel)
    assert torch.equal(clean[keep], dirty[keep])
    assert not torch.isfinite(dirty[(keep + 1) % M].float()).any()


def test_linear_packed_refuses_what_it_cannot_run(nf):
    X = torch.zeros(2, 100, 64, device="cuda", dtype=BF)
    Wp = torch.zeros(2, 64, 96, device="cuda", dtype=BF)
    with pytest.raises(nf.NetFuseError) as e:
        nf.linear_packed(X, Wp, 96)
    assert e.value.status == nf.NF_EUNSUPPORTED
