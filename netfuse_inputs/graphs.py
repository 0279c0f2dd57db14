"""Single-model operator graphs of the workloads, as plain data.

Section 3.2's merging algorithm takes "a common subgraph (V, E) of M DNNs".  These builders write that
subgraph down for the architectures of the workloads: a list of nodes, each a dict
``{"kind": str, "parents": [node indices], "attrs": {...}, "name": str}`` in construction order
(parents always precede children).  No merging logic lives here: the C++ merger of the library and the
Python oracle both take these lists as their input.

kinds: input, matmul, conv2d, layernorm, batchnorm, attention, attention_relpos, relu, gelu, add, maxpool,
avgpool_global,
task_head (a fully connected layer outside the common backbone: Section 3.2, last paragraph; Section 6)
"""
from __future__ import annotations

from typing import Dict, List

from . import EncoderShape, ResNetSpec

Node = Dict[str, object]


class GraphBuilder:
    def __init__(self):
        self.nodes: List[Node] = []

    def add(self, kind: str, parents=(), name: str = "", **attrs) -> int:
        self.nodes.append(dict(kind=kind, parents=list(parents), attrs=dict(attrs), name=name or "%s%d" % (kind, len(self.nodes))))
        return len(self.nodes) - 1


def ffnn_example(K: int = 64, Nout: int = 64) -> List[Node]:
    """The two-layer network of Section 3.2: a fully connected layer followed by a layer normalisation."""
    g = GraphBuilder()
    x = g.add("input", name="x")
    y = g.add("matmul", [x], name="fc", K=K, Nout=Nout, bias=1)
    g.add("layernorm", [y], name="ln", H=Nout)
    return g.nodes


def encoder_layer(g: GraphBuilder, x: int, shape: EncoderShape, prefix: str, r: int = -1) -> int:
    """The residual additions name the matmul branch first: where the two operands of an addition disagree on
    the concatenation dimension one against one, Algorithm 1's vote goes to the first parent.
    r: the node of the relative position encodings; with it the layer is XLNet-shaped (its own projection of the
    encodings, attention with the relative-position term)."""
    Hd, F = shape.hidden, shape.ffn
    qkv = g.add("matmul", [x], name=prefix + "qkv", K=Hd, Nout=3 * Hd, bias=1)
    if r < 0:
        att = g.add("attention", [qkv], name=prefix + "attention", heads=shape.heads, d=shape.head_dim)
    else:
        kr = g.add("matmul", [r], name=prefix + "kr", K=Hd, Nout=Hd, bias=0)
        att = g.add("attention_relpos", [qkv, kr], name=prefix + "attention", heads=shape.heads, d=shape.head_dim)
    o = g.add("matmul", [att], name=prefix + "o", K=Hd, Nout=Hd, bias=1)
    h = g.add("add", [o, x], name=prefix + "add1")
    x1 = g.add("layernorm", [h], name=prefix + "ln1", H=Hd)
    f1 = g.add("matmul", [x1], name=prefix + "ffn1", K=Hd, Nout=F, bias=1)
    a1 = g.add("gelu", [f1], name=prefix + "gelu")
    f2 = g.add("matmul", [a1], name=prefix + "ffn2", K=F, Nout=Hd, bias=1)
    h2 = g.add("add", [f2, x1], name=prefix + "add2")
    return g.add("layernorm", [h2], name=prefix + "ln2", H=Hd)


def encoder_stack_graph(shape: EncoderShape) -> List[Node]:
    """Post-LN encoder layers (workloads 2 and 5)."""
    g = GraphBuilder()
    x = g.add("input", name="x")
    for L in range(shape.layers):
        x = encoder_layer(g, x, shape, "l%d." % L)
    return g.nodes


def xlnet_stack_graph(shape: EncoderShape) -> List[Node]:
    """The XLNet-shaped stack: two inputs (the token embeddings and the relative position encodings)."""
    g = GraphBuilder()
    x = g.add("input", name="x")
    r = g.add("input", name="r")
    for L in range(shape.layers):
        x = encoder_layer(g, x, shape, "l%d." % L, r)
    return g.nodes


def encoder_with_task_heads_graph(shape: EncoderShape) -> List[Node]:
    """The encoder stack as the common backbone of networks fine-tuned for different tasks (Section 6): every
    network ends in a fully connected layer of its own width on the backbone's output."""
    nodes = encoder_stack_graph(shape)
    nodes.append(dict(kind="task_head", parents=[len(nodes) - 1], attrs=dict(K=shape.hidden, bias=1), name="head"))
    return nodes


def resnet_graph(spec: ResNetSpec) -> List[Node]:
    """Bottleneck ResNet / ResNeXt (workloads 3 and 4): conv -> batch norm -> ReLU, max-pool, bottleneck blocks
    with the shortcut added before the last ReLU, global average pool."""
    g = GraphBuilder()

    def conv_bn(x, c, relu):
        y = g.add("conv2d", [x], name=c.name, cin=c.cin, cout=c.cout, k=c.k, stride=c.stride, pad=c.pad, groups=c.groups, bias=0)
        y = g.add("batchnorm", [y], name=c.name + ".bn", C=c.cout)
        return g.add("relu", [y], name=c.name + ".relu") if relu else y

    x = g.add("input", name="x")
    x = conv_bn(x, spec.stem, True)
    x = g.add("maxpool", [x], name="maxpool", k=3, stride=2, pad=1)
    for blk in spec.blocks:
        a = conv_bn(x, blk.conv1, True)
        b = conv_bn(a, blk.conv2, True)
        sc = conv_bn(x, blk.down, False) if blk.down is not None else x
        c = conv_bn(b, blk.conv3, False)
        s = g.add("add", [sc, c], name=blk.conv3.name + ".add")
        x = g.add("relu", [s], name=blk.conv3.name + ".relu")
    g.add("avgpool_global", [x], name="avgpool")
    return g.nodes
