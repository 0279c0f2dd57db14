"""Algorithm 1 (Section 3.2): the oracle against what the paper states, the C++ merger against the oracle,
and the lowered call lists against the hand-written op sequences of the workloads.  No GPU needed: the
merger is host code (the one test that executes a generated call list is marked gpu)."""
import ctypes
import os
import re
import time

import numpy as np
import pytest

import netfuse_inputs as NI
from netfuse_inputs import graphs as G
from oracle import graph_merge as OG

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def node(kind, parents=(), **attrs):
    return dict(kind=kind, parents=list(parents), attrs=attrs, name=kind)


# ------------------------------------------------------------------ the oracle against the paper
def test_oracle_section_3_2_example():
    """A fully connected layer followed by a layer normalisation: batch matmul, then a reshape, then a group
    normalisation with one group per model (Section 3.2, the two feed-forward networks of its example)."""
    m = OG.merge_graph(G.ffnn_example(), 2)
    assert [n["kind"] for n in m] == ["input", "matmul", "reshape_transpose", "layernorm"]
    assert [n["dim"] for n in m] == ["DontCare", "Batch", "Channel", "Channel"]
    assert m[1]["attrs"]["batch"] == 2 and m[3]["attrs"]["groups"] == 2
    assert m[2]["attrs"] == {"from": "Batch", "to": "Channel"}
    assert m[1]["parents"] == [0] and m[2]["parents"] == [1] and m[3]["parents"] == [2]


def test_oracle_four_grouped_convolutions_of_two_groups_give_eight():
    """Section 3.1: merging 4 grouped convolutions that use 2 groups each gives one of 4 x 2 = 8 groups."""
    g = [node("input"), node("conv2d", [0], cin=8, cout=16, k=3, stride=1, pad=1, groups=2, bias=0)]
    m = OG.merge_graph(g, 4)
    assert m[1]["attrs"]["groups"] == 8 and m[1]["attrs"]["cin"] == 32 and m[1]["attrs"]["cout"] == 64
    assert m[1]["dim"] == "Channel" and len(m) == 2          # the network input needs no reshape


def test_oracle_dontcare_takes_the_majority_and_the_first_parent_on_a_tie():
    conv = dict(cin=4, cout=4, k=1, stride=1, pad=0, groups=1, bias=0)
    g = [node("input"), node("conv2d", [0], **conv), node("conv2d", [0], **conv), node("matmul", [0], K=4, Nout=4, bias=0),
         node("add", [3, 1, 2]),            # Batch, Channel, Channel -> Channel; the matmul edge gets a reshape
         node("add", [3, 1]),               # tie -> the first parent: Batch
         node("add", [1, 3]),               # tie -> the first parent: Channel
         node("relu", [0])]                 # only a DontCare parent: stays DontCare
    m = OG.merge_graph(g, 3)
    by_src = {n["source"]: n for n in m if n["source"] is not None}
    assert by_src[4]["dim"] == "Channel" and by_src[5]["dim"] == "Batch" and by_src[6]["dim"] == "Channel"
    assert by_src[7]["dim"] == "DontCare"
    kinds = [m[p]["kind"] for p in by_src[4]["parents"]]
    assert kinds == ["reshape_transpose", "conv2d", "conv2d"]
    assert sum(n["kind"] == "reshape_transpose" for n in m) == 3          # one per conflicting edge


def test_oracle_waits_for_all_parents():
    """A residual addition is reached through the short branch first; it is merged after its long branch."""
    conv = dict(cin=4, cout=4, k=3, stride=1, pad=1, groups=1, bias=0)
    g = [node("input"), node("conv2d", [0], **conv), node("conv2d", [1], **conv), node("conv2d", [2], **conv),
         node("add", [0, 3])]
    m = OG.merge_graph(g, 2)
    assert [n["source"] for n in m] == [0, 1, 2, 3, 4]
    assert m[4]["parents"] == [0, 3] and m[4]["dim"] == "Channel"


def test_oracle_merges_the_common_backbone_only():
    """Section 3.2 (paragraph after the listing) and Section 6: networks that share a backbone are merged up to
    their own layers, which are left as they are.  Example: the two-layer network of Section 3.2 as the
    backbone, then one fully connected layer per network."""
    g = G.ffnn_example(K=16, Nout=16) + [node("task_head", [2], K=16, bias=1)]
    m = OG.merge_graph(g, 5)
    assert [n["kind"] for n in m] == ["input", "matmul", "reshape_transpose", "layernorm", "reshape_transpose", "task_head"]
    head = m[-1]
    # not merged: its own attributes are untouched (no batch matmul over a common width, K is not multiplied),
    # it only records that there are M of it ...
    assert head["attrs"] == {"K": 16, "bias": 1, "instances": 5} and head["source"] == 3
    # ... and each reads its own network's rows: the batch form, so the channel-merged normalisation's output
    # is reshaped back
    assert head["dim"] == "Batch" and m[4]["attrs"] == {"from": "Channel", "to": "Batch"} and head["parents"] == [4]
    # the backbone is merged exactly as without the heads
    assert m[:4] == OG.merge_graph(G.ffnn_example(K=16, Nout=16), 5)
    # a batch-merged backbone output needs no reshape; several heads on one backbone are all left alone
    g2 = [node("input"), node("matmul", [0], K=8, Nout=8, bias=0), node("task_head", [1], K=8, bias=0), node("task_head", [1], K=8, bias=1)]
    m2 = OG.merge_graph(g2, 3)
    assert [n["kind"] for n in m2] == ["input", "matmul", "task_head", "task_head"] and m2[1]["attrs"]["batch"] == 3
    # nothing past the backbone is merged, so nothing may follow a head
    with pytest.raises(ValueError):
        OG.merge_graph(g2 + [node("relu", [2])], 3)


def check_invariants(common, merged, M):
    """What must hold for any input: every operation merged exactly once, parents before children, the
    original edges recovered when the reshapes are contracted, a reshape on exactly the Batch/Channel edges."""
    srcs = [n["source"] for n in merged if n["source"] is not None]
    assert sorted(srcs) == list(range(len(common)))
    pos = {n["source"]: i for i, n in enumerate(merged) if n["source"] is not None}
    for i, n in enumerate(merged):
        assert all(p < i for p in n["parents"])
        if n["kind"] == "reshape_transpose":
            (p,) = n["parents"]
            assert {merged[p]["dim"], n["dim"]} == {"Batch", "Channel"}
            assert n["attrs"] == {"from": merged[p]["dim"], "to": n["dim"]}
            continue
        contracted = [merged[p]["parents"][0] if merged[p]["kind"] == "reshape_transpose" else p for p in n["parents"]]
        assert contracted == [pos[q] for q in common[n["source"]]["parents"]]
        for p in n["parents"]:
            assert {merged[p]["dim"], n["dim"]} != {"Batch", "Channel"}
            if merged[p]["kind"] == "reshape_transpose":
                assert merged[p]["dim"] == n["dim"]
        if n["kind"] in ("matmul", "attention", "attention_relpos"):
            assert n["dim"] == "Batch" and n["attrs"]["batch"] == M * common[n["source"]]["attrs"].get("batch", 1)
        if n["kind"] == "conv2d":
            assert n["dim"] == "Channel" and n["attrs"]["groups"] == M * common[n["source"]]["attrs"]["groups"]
        if n["kind"] == "layernorm":
            assert n["dim"] == "Channel" and n["attrs"]["groups"] == M
        if n["kind"] == "task_head":
            src = common[n["source"]]["attrs"]
            assert n["dim"] == "Batch" and n["attrs"]["instances"] == M
            assert {k: v for k, v in n["attrs"].items() if k != "instances"} == src


def random_dag(rng, n):
    nodes = [node("input")]
    for i in range(1, n):
        kind = rng.choice(["matmul", "conv2d", "layernorm", "batchnorm", "attention", "relu", "gelu", "add", "maxpool", "input"],
                          p=[.15, .15, .1, .1, .05, .1, .05, .2, .05, .05])
        if kind == "input":
            nodes.append(node("input"))
            continue
        k = int(rng.integers(2, 4)) if kind == "add" else 1
        parents = [int(p) for p in rng.integers(0, i, k)]
        attrs = {"matmul": dict(K=8, Nout=8, bias=1), "conv2d": dict(cin=8, cout=8, k=3, stride=1, pad=1, groups=int(rng.choice([1, 2, 4])), bias=0),
                 "layernorm": dict(H=8), "batchnorm": dict(C=8), "attention": dict(heads=2, d=4), "maxpool": dict(k=3, stride=2, pad=1)}.get(kind, {})
        nodes.append(node(kind, parents, **attrs))
    for _ in range(int(rng.integers(0, 3))):          # per-network layers hang off the backbone as leaves
        nodes.append(node("task_head", [int(rng.integers(0, n))], K=8, bias=int(rng.integers(0, 2))))
    return nodes


def test_oracle_invariants_on_random_graphs_and_workloads():
    rng = np.random.default_rng(11)
    for _ in range(60):
        g = random_dag(rng, int(rng.integers(2, 40)))
        M = int(rng.integers(1, 6))
        check_invariants(g, OG.merge_graph(g, M), M)
    for g in (G.encoder_stack_graph(NI.EncoderShape(layers=3)), G.resnet_graph(NI.resnet_spec()), G.resnet_graph(NI.resnet_spec(32, 4)),
              G.xlnet_stack_graph(NI.EncoderShape(layers=3)), G.encoder_with_task_heads_graph(NI.EncoderShape(layers=2))):
        check_invariants(g, OG.merge_graph(g, 32), 32)
    # a ResNet is channel-merged throughout: no reshape at all; M = 1 changes nothing but the tags
    assert not any(n["kind"] == "reshape_transpose" for n in OG.merge_graph(G.resnet_graph(NI.resnet_spec()), 32))
    one = OG.merge_graph(G.resnet_graph(NI.resnet_spec()), 1)
    base = G.resnet_graph(NI.resnet_spec())
    assert all(n["attrs"] == base[n["source"]]["attrs"] for n in one) and len(one) == len(base)


# ------------------------------------------------------------------ the C++ merger against the oracle
@pytest.fixture(scope="module")
def NG():
    if not os.path.exists(os.path.join(ROOT, "paper_2009_13062_amd", "libnetfuse.so")):
        import __graft_entry__ as g
        g.build()
    from paper_2009_13062_amd import graph
    return graph


def canon(nodes):
    out = []
    for n in nodes:
        a = {k: v for k, v in n["attrs"].items()}
        out.append((n["kind"], tuple(n["parents"]), n["dim"], n["source"], tuple(sorted(a.items()))))
    return out


def oracle_canon(common, M):
    """The oracle's result with the attribute slots the C ABI carries (defaults filled in)."""
    from paper_2009_13062_amd.graph import SLOTS
    out = []
    for n in OG.merge_graph(common, M):
        slots = SLOTS.get(n["kind"], ())
        if n["kind"] == "reshape_transpose":
            a = dict(n["attrs"])
        else:
            a = {s: int(n["attrs"].get(s, M if s in ("batch", "groups", "instances") and n["kind"] in ("matmul", "layernorm", "attention", "task_head", "attention_relpos") else 0))
                 for s in slots}
        out.append((n["kind"], tuple(n["parents"]), n["dim"], n["source"], tuple(sorted(a.items()))))
    return out


def test_header_symbols_are_exported(NG):
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "netfuse_graph.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(netfuse_graph_[a-z0-9_]+)\s*\(", text)))
    assert len(names) == 7
    import paper_2009_13062_amd as nf
    for n in names:
        assert hasattr(nf.lib, n), n


def test_merger_equals_oracle(NG):
    rng = np.random.default_rng(12)
    cases = [(G.ffnn_example(), 2), (G.encoder_stack_graph(NI.EncoderShape(layers=2)), 8),
             (G.encoder_with_task_heads_graph(NI.EncoderShape(layers=2)), 8),
             (G.xlnet_stack_graph(NI.EncoderShape(layers=3)), 32),
             (G.resnet_graph(NI.resnet_spec()), 32), (G.resnet_graph(NI.resnet_spec(32, 4)), 16)]
    cases += [(random_dag(rng, int(rng.integers(2, 60))), int(rng.integers(1, 9))) for _ in range(80)]
    for common, M in cases:
        got = NG.Graph.from_nodes(common).merge(M).nodes()
        assert canon(got) == oracle_canon(common, M)


def test_merger_rejects_bad_arguments(NG):
    import paper_2009_13062_amd as nf
    L = nf.lib
    g = NG.Graph()
    zero = (ctypes.c_int * 1)(0)
    assert L.netfuse_graph_add_op(g.h, 1, zero, 1, None, 0) < 0          # parent 0 does not exist yet
    assert L.netfuse_graph_add_op(g.h, 0, None, 0, None, 0) == 0
    assert L.netfuse_graph_add_op(g.h, 0, zero, 1, None, 0) < 0          # an input with a parent
    assert L.netfuse_graph_add_op(g.h, 6, None, 0, None, 0) < 0          # an operation without one
    assert L.netfuse_graph_add_op(g.h, 11, zero, 1, None, 0) < 0         # reshapes are the merger's to insert
    assert L.netfuse_graph_add_op(g.h, 99, zero, 1, None, 0) < 0
    head = L.netfuse_graph_add_op(g.h, 12, zero, 1, None, 0)             # a task head on the input ...
    assert head == 1 and L.netfuse_graph_merge(g.h, 2)
    assert L.netfuse_graph_add_op(g.h, 6, (ctypes.c_int * 1)(head), 1, None, 0) == 2
    assert not L.netfuse_graph_merge(g.h, 2)                             # ... must stay a leaf
    assert L.netfuse_graph_add_op(None, 0, None, 0, None, 0) < 0
    assert not L.netfuse_graph_merge(g.h, 0) and not L.netfuse_graph_merge(None, 2)
    assert L.netfuse_graph_size(None) < 0 and L.netfuse_graph_lower(None, None, 0) < 0


# ------------------------------------------------------------------ lowering to library calls
def named_calls(NG, common, M):
    merged = NG.Graph.from_nodes(common).merge(M)
    nodes, calls = merged.nodes(), merged.lower()
    name = lambda op: "x" if op < 0 else common[nodes[op]["source"]]["name"]
    produced = {}                         # merged op id -> name of the call that produced its tensor
    for i, n in enumerate(nodes):
        if n["kind"] == "input":
            produced[i] = common[n["source"]]["name"]
    out = []
    for c in calls:
        assert c["input"] in produced and (c["residual"] < 0 or c["residual"] in produced), "operand used before it exists"
        out.append((c["call"], name(c["op"]), produced[c["input"]], None if c["residual"] < 0 else produced[c["residual"]], c["act"]))
        produced[c["output"]] = name(c["op"])
        produced[c["op"]] = name(c["op"])
    return out, calls, nodes


def test_lowered_encoder_equals_the_hand_written_sequence(NG):
    from paper_2009_13062_amd.workloads import encoder_call_list
    shape = NI.EncoderShape(layers=3)
    got, calls, nodes = named_calls(NG, G.encoder_stack_graph(shape), 32)
    assert got == encoder_call_list(3)
    # the reshapes Algorithm 1 inserts around the layer normalisations are there, and none is materialised
    # (per layer: one into each normalisation, one out of it per consumer -- the next matmul and the next addition)
    assert sum(n["kind"] == "reshape_transpose" for n in nodes) == 3 * 6 - 2
    assert all(c["layout"] == 0 for c in calls if c["call"] == "layernorm")


@pytest.mark.parametrize("card,bw,M", [(1, 64, 32), (32, 4, 16)], ids=["resnet50", "resnext50"])
def test_lowered_resnet_equals_the_hand_written_sequence(NG, card, bw, M):
    from paper_2009_13062_amd.workloads import resnet_call_list
    spec = NI.resnet_spec(card, bw)
    got, calls, nodes = named_calls(NG, G.resnet_graph(spec), M)
    want = resnet_call_list(spec)
    assert sorted(got, key=str) == sorted(want, key=str)          # same calls with the same operands ...
    assert len(got) == len(spec.convs()) + 2                      # ... one per convolution plus the two pools
    assert all(c["batchnorm"] >= 0 for c in calls if c["call"] == "conv2d")
    merged_groups = {nodes[c["op"]]["attrs"]["groups"] for c in calls if c["call"] == "conv2d"}
    assert merged_groups == ({M} if card == 1 else {M, M * card})


def test_lowered_xlnet_stack_equals_the_hand_written_sequence(NG):
    """Two inputs: the breadth-first traversal reaches every layer's position projection from the encodings
    early, so the calls come in another (valid: named_calls checks every operand exists) order than the
    hand-written forward issues them; call by call they are the same."""
    from paper_2009_13062_amd.workloads import encoder_call_list
    got, calls, nodes = named_calls(NG, G.xlnet_stack_graph(NI.EncoderShape(layers=3)), 32)
    want = encoder_call_list(3, rel=True)
    assert sorted(got, key=str) == sorted(want, key=str) and len(got) == 3 * 8
    rel = [nodes[c["op"]] for c in calls if c["call"] == "attention_relpos"]
    assert len(rel) == 3 and all(n["attrs"]["batch"] == 32 and n["dim"] == "Batch" for n in rel)
    assert not any(c["call"] in ("merge_transpose", "unfused") for c in calls)


def test_lowered_backbone_with_task_heads(NG):
    """The encoder as a common backbone: the same calls as without heads, then ONE ragged launch for the M
    unmerged layers, reading the last normalisation's output in the batch form (no reshape materialised)."""
    from paper_2009_13062_amd.workloads import encoder_call_list
    shape = NI.EncoderShape(layers=2)
    got, calls, nodes = named_calls(NG, G.encoder_with_task_heads_graph(shape), 8)
    assert got[:-1] == encoder_call_list(2)
    assert got[-1] == ("linear_ragged", "head", "l1.ln2", None, 0)
    assert all(c["layout"] == 0 for c in calls if c["call"] == "layernorm")
    assert not any(c["call"] == "merge_transpose" for c in calls)
    assert nodes[calls[-1]["op"]]["attrs"] == {"K": shape.hidden, "bias": 1, "instances": 8}


def test_lowering_keeps_what_it_cannot_fold(NG):
    """A batch matmul feeding a group normalisation AND a convolution-side consumer: the reshape is real."""
    g = [node("input"), node("matmul", [0], K=8, Nout=8, bias=0), node("layernorm", [1], H=8), node("batchnorm", [2], C=8),
         node("relu", [0])]
    merged = NG.Graph.from_nodes(g).merge(2)
    kinds = [c["call"] for c in merged.lower()]
    assert kinds == ["linear", "unfused", "merge_transpose", "layernorm", "unfused"]          # breadth-first order


def test_merging_32_resnext50_takes_far_less_than_the_papers_600_ms(NG):
    """Section 4 reports at most 600 ms of merging overhead (32 ResNeXt-50 instances)."""
    common = G.resnet_graph(NI.resnet_spec(32, 4))
    t0 = time.perf_counter()
    merged = NG.Graph.from_nodes(common).merge(32)
    calls = merged.lower()
    dt = time.perf_counter() - t0
    assert len(calls) == 55 and dt < 0.6, dt
    # the traversal itself, without the Python marshalling
    g = NG.Graph.from_nodes(common)
    import paper_2009_13062_amd as nf
    t0 = time.perf_counter()
    for _ in range(100):
        nf.lib.netfuse_graph_destroy(nf.lib.netfuse_graph_merge(g.h, 32))
    per = (time.perf_counter() - t0) / 100
    print("merge of 32 x ResNeXt-50 (%d operations): %.1f us in the library, %.1f ms with graph construction" % (len(common), per * 1e6, dt * 1e3))
    assert per < 0.01


# ------------------------------------------------------------------ a generated call list on the GPU
@pytest.mark.gpu
@pytest.mark.parametrize("which", ["encoder", "resnext", "encoder_heads", "xlnet"])
def test_generated_call_list_runs_like_the_hand_written_forward(NG, oracle, which):
    import torch
    from oracle import models as OM
    from paper_2009_13062_amd.workloads import EncoderStack, ResNetForward
    M = 3
    heads = None
    if which in ("encoder", "encoder_heads", "xlnet"):
        shape = NI.EncoderShape(hidden=128, heads=2, ffn=256, layers=2, seq=64)
        inp = NI.encoder_stack(M, shape, bf16=True, rel=which == "xlnet")
        net = EncoderStack.from_numpy(inp, M, 1, shape.seq, shape.heads)
        x = torch.from_numpy(inp["X"]).to("cuda", torch.bfloat16)
        want = net.forward(x).clone()
        common = G.xlnet_stack_graph(shape) if which == "xlnet" else G.encoder_stack_graph(shape)
        if which == "xlnet":
            x = {"x": x, "r": net.buf["Rrep"]}
        weights = {}
        for L, Lw in enumerate(net.layers):
            p = "l%d." % L
            weights.update({p + "qkv": dict(W=Lw["Wqkv"], b=Lw["bqkv"]), p + "o": dict(W=Lw["Wo"], b=Lw["bo"]),
                            p + "ffn1": dict(W=Lw["W1"], b=Lw["b1"]), p + "ffn2": dict(W=Lw["W2"], b=Lw["b2"]),
                            p + "ln1": dict(gamma=Lw["ln1_g"], beta=Lw["ln1_b"]), p + "ln2": dict(gamma=Lw["ln2_g"], beta=Lw["ln2_b"])})
            if which == "xlnet":
                weights.update({p + "kr": dict(W=Lw["Wr"]), p + "attention": dict(rwb=Lw["rwb"], rrb=Lw["rrb"])})
        ref = OM.encoder_stack(inp, M, 1, shape.seq, shape.heads, out_bf16=True)
        last, seq = "l%d.ln2" % (shape.layers - 1), shape.seq
        if which == "encoder_heads":
            # networks fine-tuned for tasks with 2, 5 and 3 classes: one fully connected layer each on the backbone
            common = G.encoder_with_task_heads_graph(shape)
            nout = [2, 5, 3]
            rng = np.random.default_rng(5)
            Wh = [NI.on_bf16_grid((rng.standard_normal((shape.hidden, n)) * 0.05).astype(np.float32)) for n in nout]
            bh = [(rng.standard_normal(n) * 0.05).astype(np.float32) for n in nout]
            weights["head"] = dict(W=torch.from_numpy(np.concatenate([w.ravel() for w in Wh])).to("cuda", torch.bfloat16),
                                   b=torch.from_numpy(np.concatenate(bh)).cuda(), nout=nout)
            heads = (Wh, bh, nout)
    else:
        spec = NI.resnet_spec(cardinality=8, base_width=8, image=64, width_div=2, depths=(1, 1, 1, 1))
        inp = NI.resnet_params(spec, M, bf16=True)
        net = ResNetForward.from_numpy(inp, spec, M)
        x = torch.from_numpy(inp["x"]).to("cuda", torch.bfloat16)
        want = net.forward(x).clone()
        common = G.resnet_graph(spec)
        weights = {}
        for c in spec.convs():
            weights[c.name] = dict(w=net.P[c.name]["w"])
            weights[c.name + ".bn"] = dict(scale=net.fold[c.name][0], shift=net.fold[c.name][1])
        ref = OM.resnet_forward(inp, spec, M, out_bf16=True)
        last, seq = "avgpool", None
    merged = NG.Graph.from_nodes(common).merge(M)
    nodes = merged.nodes()
    T = NG.run_calls(merged.lower(), nodes, common, M, x, weights, batch=1, seq=seq)
    out_id = [i for i, n in enumerate(nodes) if n["source"] is not None and common[n["source"]]["name"] == last][0]
    got = T[out_id]
    torch.cuda.synchronize()
    assert torch.equal(got, want), "the generated call list and the hand-written forward run the same calls"
    err = np.abs(got.float().cpu().numpy() - ref)
    assert float(err.max()) < 0.15 * max(1.0, float(np.abs(ref).max()))
    if heads is not None:
        import paper_2009_13062_amd as nf
        Wh, bh, nout = heads
        head_id = [i for i, n in enumerate(nodes) if n["kind"] == "task_head"][0]
        ys = nf.ragged_views(T[head_id], shape.seq, nout)
        # the oracle's per-network layers on the oracle's own backbone output (end-to-end bound as above; the
        # ragged launch has its per-operator parity tests of its own)
        want_h = oracle.linear_ragged(ref, Wh, bh, out_bf16=True)
        for m in range(M):
            assert tuple(ys[m].shape) == want_h[m].shape == (shape.seq, nout[m])
            e = np.abs(ys[m].float().cpu().numpy() - want_h[m])
            assert float(e.max()) <= 0.15 * max(1.0, float(np.abs(want_h[m]).max())), (m, float(e.max()))
