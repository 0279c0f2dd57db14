"""Binding of the host-side DNN merger (include/netfuse_graph.h: Section 3.2, Algorithm 1) and an executor
for the call lists it lowers merged graphs to.

Marshalling only: node lists go in through netfuse_graph_add_op, the merged graph and the calls are read
back into plain Python structures, and ``run_calls`` hands each call to the entry point of the same name
in the merged-operator library.
"""
from __future__ import annotations

import ctypes
from typing import Dict, List, Sequence

from . import lib as _lib

KINDS = ("input", "matmul", "conv2d", "layernorm", "batchnorm", "attention", "relu", "gelu", "add", "maxpool",
         "avgpool_global", "reshape_transpose", "task_head", "attention_relpos")
DIMS = ("Batch", "Channel", "DontCare")
CALLS = ("linear", "conv2d", "layernorm", "attention", "maxpool2d", "avgpool_global", "merge_transpose", "unfused",
         "linear_ragged", "attention_relpos")
# attribute slots per kind (include/netfuse_graph.h)
SLOTS = {
    "matmul": ("K", "Nout", "bias", "batch"),
    "conv2d": ("cin", "cout", "k", "stride", "pad", "groups", "bias"),
    "layernorm": ("H", "groups"),
    "batchnorm": ("C",),
    "attention": ("heads", "d", "batch"),
    "maxpool": ("k", "stride", "pad"),
    "reshape_transpose": ("from", "to"),
    "task_head": ("K", "bias", "instances"),
    "attention_relpos": ("heads", "d", "batch"),
}
_DEFAULT_ONE = ("batch", "groups", "instances")
MAX_ATTRS = 8


class NfCall(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("call", "op", "input", "residual", "output", "act", "batchnorm", "layout")]


_lib.netfuse_graph_create.restype = ctypes.c_void_p
_lib.netfuse_graph_destroy.argtypes = [ctypes.c_void_p]
_lib.netfuse_graph_destroy.restype = None
_lib.netfuse_graph_add_op.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_int), ctypes.c_int,
                                      ctypes.POINTER(ctypes.c_long), ctypes.c_int]
_lib.netfuse_graph_size.argtypes = [ctypes.c_void_p]
_lib.netfuse_graph_merge.argtypes = [ctypes.c_void_p, ctypes.c_int]
_lib.netfuse_graph_merge.restype = ctypes.c_void_p
_lib.netfuse_graph_get_op.argtypes = [ctypes.c_void_p, ctypes.c_int] + [ctypes.POINTER(ctypes.c_int)] * 4 + [
    ctypes.c_int, ctypes.POINTER(ctypes.c_long)]
_lib.netfuse_graph_lower.argtypes = [ctypes.c_void_p, ctypes.POINTER(NfCall), ctypes.c_int]


class Graph:
    """Owns one nf_graph handle."""

    def __init__(self, handle=None):
        self.h = handle if handle is not None else _lib.netfuse_graph_create()
        if not self.h:
            raise MemoryError("netfuse_graph_create failed")

    def __del__(self):
        if getattr(self, "h", None):
            _lib.netfuse_graph_destroy(self.h)
            self.h = None

    @classmethod
    def from_nodes(cls, nodes: Sequence[Dict]) -> "Graph":
        g = cls()
        for nd in nodes:
            slots = SLOTS.get(nd["kind"], ())
            vals = [int(nd["attrs"].get(s, 1 if s in _DEFAULT_ONE else 0)) for s in slots]
            par = nd["parents"]
            rc = _lib.netfuse_graph_add_op(g.h, KINDS.index(nd["kind"]), (ctypes.c_int * len(par))(*par), len(par),
                                           (ctypes.c_long * len(vals))(*vals), len(vals))
            if rc < 0:
                raise ValueError("netfuse_graph_add_op rejected node %r (status %d)" % (nd.get("name"), -rc))
        return g

    def __len__(self):
        return _lib.netfuse_graph_size(self.h)

    def merge(self, M: int) -> "Graph":
        h = _lib.netfuse_graph_merge(self.h, int(M))
        if not h:
            raise ValueError("netfuse_graph_merge failed (M <= 0 or a malformed graph)")
        return Graph(h)

    def nodes(self) -> List[Dict]:
        out = []
        for i in range(len(self)):
            kind, dim, src = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
            par = (ctypes.c_int * 8)()
            attrs = (ctypes.c_long * MAX_ATTRS)()
            n = _lib.netfuse_graph_get_op(self.h, i, ctypes.byref(kind), ctypes.byref(dim), ctypes.byref(src), par, 8, attrs)
            k = KINDS[kind.value]
            a = {s: int(attrs[j]) for j, s in enumerate(SLOTS.get(k, ()))}
            if k == "reshape_transpose":
                a = {"from": DIMS[a["from"]], "to": DIMS[a["to"]]}
            out.append(dict(kind=k, parents=[par[j] for j in range(n)], attrs=a, dim=DIMS[dim.value],
                            source=None if src.value < 0 else src.value))
        return out

    def lower(self) -> List[Dict]:
        n = _lib.netfuse_graph_lower(self.h, None, 0)
        if n < 0:
            raise ValueError("netfuse_graph_lower failed")
        buf = (NfCall * max(n, 1))()
        n = _lib.netfuse_graph_lower(self.h, buf, n)
        return [dict(call=CALLS[c.call], op=c.op, input=c.input, residual=c.residual, output=c.output, act=c.act,
                     batchnorm=c.batchnorm, layout=c.layout) for c in buf[:n]]


def run_calls(calls, merged_nodes, common_nodes, M, graph_input, weights, batch=1, seq=None, eps=1e-5):
    """Executes a lowered call list.  ``weights[name]`` holds the merged parameters of the operation of the
    common subgraph called ``name``: matmul {"W", "b"}, layernorm {"gamma", "beta"}, conv2d {"w"} and, for the
    batch normalisation folded into it, {"scale", "shift"} under the batch norm's own name; a task head
    {"W", "b", "nout"}: the M unmerged layers' weights and biases one after another and their output widths; a
    relative-position attention {"rwb", "rrb"}.  ``graph_input``: the tensor of the graph's input, or
    {input name: tensor} when it has several.
    Returns {merged operation id: output tensor}."""
    import paper_2009_13062_amd as nf
    T = {}
    for i, nd in enumerate(merged_nodes):
        if nd["kind"] == "input":
            T[i] = graph_input[common_nodes[nd["source"]]["name"]] if isinstance(graph_input, dict) else graph_input
    name_of = lambda op: common_nodes[merged_nodes[op]["source"]]["name"]
    for c in calls:
        nd = merged_nodes[c["op"]]
        x = T[c["input"]]
        res = T[c["residual"]] if c["residual"] >= 0 else None
        if c["call"] == "linear":
            w = weights[name_of(c["op"])]
            y = nf.linear(x, w["W"], bias=w.get("b"), residual=res, act=c["act"])
        elif c["call"] == "conv2d":
            w = weights[name_of(c["op"])]
            bn = weights[name_of(c["batchnorm"])] if c["batchnorm"] >= 0 else {}
            a = nd["attrs"]
            y = nf.conv2d(x, w["w"], M, g=a["groups"] // M, scale=bn.get("scale"), shift=bn.get("shift"), residual=res,
                          stride=a["stride"], pad=a["pad"], act=c["act"])
        elif c["call"] == "layernorm":
            w = weights[name_of(c["op"])]
            y = nf.layernorm(x, w["gamma"], w["beta"], M, eps=eps, layout=c["layout"])
        elif c["call"] == "attention":
            y = nf.attention_packed(x, batch, seq, nd["attrs"]["heads"])
        elif c["call"] == "attention_relpos":
            w = weights[name_of(c["op"])]
            y = nf.attention_relpos_packed(x, res, batch, seq, nd["attrs"]["heads"], bias_w=w.get("rwb"), bias_r=w.get("rrb"))
        elif c["call"] == "maxpool2d":
            a = nd["attrs"]
            y = nf.maxpool2d(x, a["k"], a["stride"], a["pad"])
        elif c["call"] == "avgpool_global":
            y = nf.avgpool_global(x)
        elif c["call"] == "linear_ragged":
            w = weights[name_of(c["op"])]
            y = nf.linear_ragged(x, w["W"], w["nout"], bias=w.get("b"))
        elif c["call"] == "merge_transpose":
            y = nf.merge_transpose(x, M, bool(c["layout"]))
        else:
            raise NotImplementedError("operation %r was not folded into a library call" % nd["kind"])
        T[c["output"]] = y
        T[c["op"]] = y if c["op"] not in T else T[c["op"]]
    return T
