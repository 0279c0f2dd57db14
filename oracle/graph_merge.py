"""Oracle for the DNN merging algorithm (Section 3.2, Algorithm 1) -- TEST INFRASTRUCTURE ONLY.

A plain Python rendering of the algorithm's steps in the paper's order and notation: a queue of
operations starting from the roots, Merge(op, weights) per Section 3.1 / Table 1 giving the merged
operation m_i and its concatenation dimension d_i, the copied dependencies, the majority vote for
DontCare operations, and the reshape-and-transpose operation inserted where a parent's dimension
conflicts.  It shares nothing with the C++ merger of the library.

Input: the common subgraph as a list of nodes {"kind", "parents", "attrs", "name"} (parents precede
children); M = the number of DNNs.  Output: the merged graph as a list of nodes
{"kind", "parents", "attrs", "dim", "source"} where ``source`` is the index of the operation of the
common subgraph a merged operation came from (None for an inserted reshape) and ``parents`` index
the merged list.  Order: operations in the order they are visited, each preceded by the reshapes
inserted on its incoming edges (so parents always precede children).

Readings of the paper recorded here (where the printed algorithm is silent):
  * An operation is processed once all its parents have been processed: an operation that is dequeued
    earlier (a residual addition reached through the short branch first) waits in the queue.  The
    printed listing would otherwise copy an edge from a parent that has no merged operation yet.
  * Batch and Channel conflict with each other only; DontCare is compatible with both (the text after the
    listing names exactly these two conflicts), so the inputs of the network need no reshape.
  * Common backbones (the paragraph after the listing): the layers a network does not share are not part of
    (V, E); here the one kind the paper names -- the per-task fully connected layer -- may be written down as a
    leaf "task_head" so that the merged graph says where the M unmerged layers attach and in which form they
    read the backbone's output.
  * MostFrequent ignores parents that are themselves still DontCare, and on a tie takes the dimension
    of the first parent among the tied ones; with no parent of a definite dimension the operation
    stays DontCare.
"""
from __future__ import annotations

from collections import deque
from typing import Dict, List, Optional

BATCH, CHANNEL, DONTCARE = "Batch", "Channel", "DontCare"


def merge_op(node: Dict, M: int):
    """Merge(op_i, {w_ij}): the merged operation's attributes and required concatenation dimension.
    matmul -> batch matmul over M weight sets (Batch); convolution -> grouped convolution with M times the
    groups and channels (Channel); layer normalisation -> group normalisation with M groups (Channel); batch
    normalisation -> M times the channels (Channel); attention (plain or with the relative-position term), already
    a batch of independent problems, -> M times the problems (Batch); operations without weights are unchanged (DontCare)."""
    kind, a = node["kind"], dict(node["attrs"])
    if kind == "matmul":
        a["batch"] = a.get("batch", 1) * M
        return a, BATCH
    if kind == "conv2d":
        a["cin"], a["cout"], a["groups"] = a["cin"] * M, a["cout"] * M, a["groups"] * M
        return a, CHANNEL
    if kind == "layernorm":
        a["groups"] = a.get("groups", 1) * M
        return a, CHANNEL
    if kind == "batchnorm":
        a["C"] = a["C"] * M
        return a, CHANNEL
    if kind in ("attention", "attention_relpos"):
        a["batch"] = a.get("batch", 1) * M
        return a, BATCH
    if kind == "task_head":
        # Section 3.2, last paragraph / Section 6: only the common backbone is merged; a layer of a network's
        # own (the fully connected layer of its downstream task) stays as it is -- M instances of it, each
        # reading its own network's rows, which only the batch concatenation keeps together
        a["instances"] = a.get("instances", 1) * M
        return a, BATCH
    if kind in ("input", "relu", "gelu", "add", "maxpool", "avgpool_global"):
        return a, DONTCARE
    raise ValueError("no merge rule for operation kind %r" % kind)


def most_frequent(dims: List[str]) -> str:
    definite = [d for d in dims if d != DONTCARE]
    if not definite:
        return DONTCARE
    nb, nc = definite.count(BATCH), definite.count(CHANNEL)
    if nb != nc:
        return BATCH if nb > nc else CHANNEL
    return definite[0]


def merge_graph(nodes: List[Dict], M: int) -> List[Dict]:
    n = len(nodes)
    children: List[List[int]] = [[] for _ in range(n)]
    for i, nd in enumerate(nodes):
        for p in nd["parents"]:
            if nodes[p]["kind"] == "task_head":
                raise ValueError("a task head lies outside the common backbone: nothing after it is merged")
            children[p].append(i)
    merged: List[Dict] = []
    m_of: List[Optional[int]] = [None] * n          # index of m_i in the merged list
    visited = [False] * n
    Q = deque(i for i in range(n) if not nodes[i]["parents"])
    while Q:
        i = Q.popleft()
        if visited[i]:
            continue
        if any(not visited[p] for p in nodes[i]["parents"]):
            continue                                  # its last parent will enqueue it again
        visited[i] = True
        attrs, d_i = merge_op(nodes[i], M)
        parent_ms = [m_of[p] for p in nodes[i]["parents"]]          # copied dependencies (m_j, m_i)
        if d_i == DONTCARE:
            d_i = most_frequent([merged[mj]["dim"] for mj in parent_ms])
        edges = []
        for mj in parent_ms:
            d_j = merged[mj]["dim"]
            if {d_j, d_i} == {BATCH, CHANNEL}:
                merged.append(dict(kind="reshape_transpose", parents=[mj], attrs={"from": d_j, "to": d_i},
                                   dim=d_i, source=None))
                edges.append(len(merged) - 1)
            else:
                edges.append(mj)
        merged.append(dict(kind=nodes[i]["kind"], parents=edges, attrs=attrs, dim=d_i, source=i))
        m_of[i] = len(merged) - 1
        for c in children[i]:
            if not visited[c]:
                Q.append(c)
    assert all(visited), "the common subgraph has a cycle or an unreachable operation"
    return merged
