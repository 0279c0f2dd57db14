"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol that
include/netfuse.h declares, and rejects bad arguments before any HIP call is made."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "netfuse.h")
LIB = os.path.join(ROOT, "paper_2009_13062_amd", "libnetfuse.so")

EINVAL = 1
P = 4096          # a non-null, well-aligned fake device address; never dereferenced on the host


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import sys
        sys.path.insert(0, ROOT)
        import __graft_entry__ as g
        g.build()
    import paper_2009_13062_amd as nf
    return nf.lib


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(netfuse_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_symbols()
    assert len(names) >= 10
    for n in names:
        assert hasattr(lib, n), n
    import paper_2009_13062_amd as nf
    assert sorted(nf.EXPORTS) == names


def test_strerror_is_total(lib):
    for st in range(-1, 6):
        s = lib.netfuse_strerror(st)
        assert s and len(s) > 1


def test_linear_rejects_bad_arguments(lib):
    f = lib.netfuse_linear
    ok = dict(X=P, W=P, bias=None, res=None, Y=P, M=2, N=4, K=8, Nout=8, dt=1, act=0)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["X"], a["W"], a["bias"], a["res"], a["Y"], a["M"], a["N"], a["K"], a["Nout"], a["dt"], a["act"], None)

    for bad in (dict(X=None), dict(W=None), dict(Y=None), dict(M=0), dict(N=-1), dict(K=0), dict(Nout=0),
                dict(dt=7), dict(act=9), dict(X=P + 1), dict(bias=P + 2),
                dict(M=2 ** 31 - 1, N=2 ** 31 - 1, K=2 ** 31 - 1)):
        assert call(**bad) == EINVAL, bad


def test_packed_linear_rejects_bad_arguments(lib):
    pk, run, can = lib.netfuse_linear_pack_weight, lib.netfuse_linear_packed, lib.netfuse_linear_packed_supported
    for bad in ((None, 2 * P, 2, 64, 96, 1), (P, None, 2, 64, 96, 1), (P, P, 2, 64, 96, 1),
                (P, 2 * P, 0, 64, 96, 1), (P, 2 * P, 2, 60, 96, 1), (P, 2 * P, 2, 64, 80, 1),
                (P, 2 * P, 2, 64, 96, 5), (P + 1, 2 * P, 2, 64, 96, 1), (P, 2 * P + 8, 2, 64, 96, 1)):
        assert pk(*bad, None) == EINVAL, bad
    assert pk(P, 2 * P, 2, 64, 96, 0, None) == 2                       # float storage: no packed kernel
    ok = dict(X=P, W=P, bias=None, res=None, Y=P, M=2, N=128, K=256, Nout=96, dt=1, act=0)

    def call(**kw):
        a = dict(ok, **kw)
        return run(a["X"], a["W"], a["bias"], a["res"], a["Y"], a["M"], a["N"], a["K"], a["Nout"],
                   a["dt"], a["act"], None)

    for bad in (dict(X=None), dict(W=None), dict(Y=None), dict(M=0), dict(N=0), dict(K=40), dict(Nout=80),
                dict(dt=3), dict(act=7), dict(W=P + 2), dict(bias=P + 1)):
        assert call(**bad) == EINVAL, bad
    assert call(dt=0) == 2
    assert call(N=100) == 2                                             # not whole tiles: NF_EUNSUPPORTED
    assert call(K=64) == 2                                              # shorter than one round of the pipeline
    assert call(Nout=160) == 2                                          # no tile width divides it
    # the query agrees with what the call accepts
    assert can(32, 128, 768, 3072, 1) == 1 and can(32, 128, 3072, 768, 1) == 1 and can(64, 256, 128, 288, 1) == 1
    assert can(32, 128, 768, 3072, 0) == 0 and can(32, 100, 768, 3072, 1) == 0 and can(0, 128, 768, 768, 1) == 0
    assert can(2, 128, 64, 96, 1) == 0 and can(2, 128, 256, 160, 1) == 0 and can(128, 128, 256, 128, 1) == 1
    assert can(2, 256, 128, 288, 1) == 0 and can(8, 128, 3072, 768, 1) == 0      # a kernel exists, but too few tiles for it to pay
    assert can(2, 256, 64, 512, 1) == 1 and can(2, 256, 48, 512, 1) == 0    # 256 x 256 tiles: K in steps of 32


def test_ragged_linear_rejects_bad_arguments(lib):
    import ctypes
    f = lib.netfuse_linear_ragged
    arr = lambda *v: (ctypes.c_int * len(v))(*v)
    assert f(None, P, None, P, 2, 4, 8, arr(3, 5), 1, 0, None) == EINVAL
    assert f(P, P, None, P, 2, 4, 8, None, 1, 0, None) == EINVAL
    assert f(P, P, None, P, 2, 4, 8, arr(3, 0), 1, 0, None) == EINVAL          # a model without outputs
    assert f(P, P, None, P, 2, 0, 8, arr(3, 5), 1, 0, None) == EINVAL
    assert f(P, P, None, P, 2, 4, 8, arr(3, 5), 4, 0, None) == EINVAL
    assert f(P, P, None, P, 2, 4, 8, arr(3, 5), 1, 9, None) == EINVAL
    assert f(P, P + 1, None, P, 2, 4, 8, arr(3, 5), 1, 0, None) == EINVAL
    assert f(P, P, None, P, 300, 4, 8, arr(*([3] * 300)), 1, 0, None) == 2     # more models than the table holds


def test_conv_rejects_bad_arguments(lib):
    f = lib.netfuse_conv2d
    ok = dict(x=P, w=P, bias=None, scale=None, shift=None, res=None, y=P, M=2, B=1, Cin=8, Cout=8, g=2, H=8,
              W=8, KH=3, KW=3, stride=1, pad=1, dil=1, dt=1, act=0)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["x"], a["w"], a["bias"], a["scale"], a["shift"], a["res"], a["y"], a["M"], a["B"], a["Cin"],
                 a["Cout"], a["g"], a["H"], a["W"], a["KH"], a["KW"], a["stride"], a["pad"], a["dil"], a["dt"],
                 a["act"], None)

    for bad in (dict(x=None), dict(w=None), dict(y=None), dict(M=0), dict(B=0), dict(Cin=0), dict(g=0),
                dict(g=3), dict(Cout=9), dict(stride=0), dict(pad=-1), dict(dil=0), dict(dt=2), dict(act=-1),
                dict(scale=P), dict(shift=P), dict(H=1, W=1, pad=0), dict(KH=0), dict(x=P + 1),
                dict(M=2 ** 30, Cin=2 ** 10, g=1, Cout=8)):
        assert call(**bad) == EINVAL, bad


def test_norms_reject_bad_arguments(lib):
    ln = lib.netfuse_layernorm
    assert ln(None, None, P, P, P, 1, 1, 4, 1e-5, 0, 0, None) == EINVAL
    assert ln(P, None, None, P, P, 1, 1, 4, 1e-5, 0, 0, None) == EINVAL
    assert ln(P, None, P, P, P, 0, 1, 4, 1e-5, 0, 0, None) == EINVAL
    assert ln(P, None, P, P, P, 1, 1, 4, -1.0, 0, 0, None) == EINVAL
    assert ln(P, None, P, P, P, 1, 1, 4, 1e-5, 2, 0, None) == EINVAL
    assert ln(P, None, P, P, P, 1, 1, 4, 1e-5, 0, 3, None) == EINVAL
    bn = lib.netfuse_batchnorm
    assert bn(P, P, P, P, None, None, P, 1, 1, 4, 4, 1e-5, 0, 0, None) == EINVAL
    assert bn(P, P, P, P, P, None, P, 1, 1, 0, 4, 1e-5, 0, 0, None) == EINVAL
    assert bn(P, P, P, P, P, None, P, 1, 1, 4, 4, float("nan"), 0, 0, None) == EINVAL
    assert lib.netfuse_bn_fold(P, P, P, P, P, None, 4, 1e-5, None) == EINVAL
    assert lib.netfuse_bn_fold(P, P, P, P, P, P, 0, 1e-5, None) == EINVAL


def test_attention_and_glue_reject_bad_arguments(lib):
    at = lib.netfuse_attention
    assert at(None, P, P, None, P, 1, 1, 8, 2, 64, 8 * 128, 128, 0.125, 1, None) == EINVAL
    assert at(P, P, P, None, P, 1, 1, 0, 2, 64, 8 * 128, 128, 0.125, 1, None) == EINVAL
    assert at(P, P, P, None, P, 1, 1, 8, 2, 64, 8 * 128, 100, 0.125, 1, None) == EINVAL     # row stride < heads*d
    assert at(P, P, P, None, P, 2, 1, 8, 2, 64, 100, 128, 0.125, 1, None) == EINVAL         # models overlap
    assert at(P, P, P, None, P, 1, 1, 8, 2, 64, 8 * 128, 128, float("nan"), 1, None) == EINVAL
    mp = lib.netfuse_maxpool2d
    assert mp(P, P, 1, 4, 8, 8, 3, 2, 3, 1, None) == EINVAL          # pad >= k
    assert mp(P, None, 1, 4, 8, 8, 3, 2, 1, 1, None) == EINVAL
    assert mp(P, P, 1, 4, 1, 1, 3, 2, 0, 1, None) == EINVAL          # window larger than padded input
    assert lib.netfuse_avgpool_global(P, P, 1, 0, 4, 1, None) == EINVAL
    mt = lib.netfuse_merge_transpose
    assert mt(P, P, 2, 2, 2, 1, 1, None) == EINVAL                   # in place is not supported
    assert mt(P, 2 * P, 2, 0, 2, 1, 1, None) == EINVAL


def test_binding_has_no_cpu_fallback():
    """The product path never imports the oracle."""
    import paper_2009_13062_amd as nf
    import paper_2009_13062_amd.workloads as wl
    for mod in (nf, wl):
        src = open(mod.__file__).read()
        assert "import oracle" not in src and "from oracle" not in src
