// DNN merging (Section 3.2, Algorithm 1) and its lowering to library calls.  Host code only.
//
// Data structure: a graph is a vector of operations in insertion order (parents before children); each
// operation keeps its parent ids, so the copied dependencies of Algorithm 1 are index translations.  The
// traversal is the algorithm's queue of operations; an operation whose parents are not all merged yet
// when it is dequeued is dropped and comes back when its last parent enqueues its children, which keeps the
// total work at O(|V| + |E|) queue entries.
#include <deque>
#include <new>
#include <vector>

#include "../../include/netfuse.h"
#include "../../include/netfuse_graph.h"

namespace {

struct Op {
  int kind;
  int dim;                      // nf_concat_dim
  int source;                   // operation of the common subgraph, -1 for an inserted reshape
  std::vector<int> parents;
  long attrs[NF_GRAPH_MAX_ATTRS];
};

bool valid_kind(int k) { return k >= NF_OP_INPUT && k <= NF_OP_ATTENTION_RELPOS; }

// slot of the "how many independent weight sets" attribute, or -1
int count_slot(int kind) {
  switch (kind) {
    case NF_OP_MATMUL: return 3;
    case NF_OP_LAYERNORM: return 1;
    case NF_OP_ATTENTION: return 2;
    case NF_OP_TASK_HEAD: return 2;
    case NF_OP_ATTENTION_RELPOS: return 2;
  }
  return -1;
}

// Merge(op_i, {w_ij}) of Algorithm 1: Section 3.1, Table 1
int merge_op(Op& m, int M) {
  switch (m.kind) {
    case NF_OP_MATMUL: m.attrs[3] *= M; return NF_DIM_BATCH;             // batch matrix multiplication
    case NF_OP_CONV2D:                                                   // grouped convolution, M times the groups
      m.attrs[0] *= M; m.attrs[1] *= M; m.attrs[5] *= M;
      return NF_DIM_CHANNEL;
    case NF_OP_LAYERNORM: m.attrs[1] *= M; return NF_DIM_CHANNEL;        // group normalisation with M groups
    case NF_OP_BATCHNORM: m.attrs[0] *= M; return NF_DIM_CHANNEL;        // per channel: concatenated channels
    case NF_OP_ATTENTION:                                                // M times the independent problems
    case NF_OP_ATTENTION_RELPOS: m.attrs[2] *= M; return NF_DIM_BATCH;   // (its two query biases: one pair per model)
    // outside the common backbone (Section 3.2, last paragraph): not merged -- M instances of the layer as it
    // is, each on its own network's rows, which are contiguous in the batch-concatenated form
    case NF_OP_TASK_HEAD: m.attrs[2] *= M; return NF_DIM_BATCH;
    default: return NF_DIM_DONTCARE;                                     // no weights
  }
}

bool conflict(int a, int b) {
  return (a == NF_DIM_BATCH && b == NF_DIM_CHANNEL) || (a == NF_DIM_CHANNEL && b == NF_DIM_BATCH);
}

}  // namespace

struct nf_graph {
  std::vector<Op> ops;
};

extern "C" {

nf_graph* netfuse_graph_create(void) { return new (std::nothrow) nf_graph(); }

void netfuse_graph_destroy(nf_graph* g) { delete g; }

int netfuse_graph_size(const nf_graph* g) { return g ? (int)g->ops.size() : -(int)NF_EINVAL; }

int netfuse_graph_add_op(nf_graph* g, int kind, const int* parents, int n_parents, const long* attrs, int n_attrs) {
  if (!g || !valid_kind(kind) || kind == NF_OP_RESHAPE_TRANSPOSE) return -(int)NF_EINVAL;
  if (n_parents < 0 || n_attrs < 0 || n_attrs > NF_GRAPH_MAX_ATTRS) return -(int)NF_EINVAL;
  if ((n_parents > 0 && !parents) || (n_attrs > 0 && !attrs)) return -(int)NF_EINVAL;
  if ((kind == NF_OP_INPUT) != (n_parents == 0)) return -(int)NF_EINVAL;
  const int id = (int)g->ops.size();
  Op op;
  op.kind = kind; op.dim = NF_DIM_DONTCARE; op.source = id;
  for (int i = 0; i < n_parents; ++i) {
    if (parents[i] < 0 || parents[i] >= id) return -(int)NF_EINVAL;
    op.parents.push_back(parents[i]);
  }
  for (int i = 0; i < NF_GRAPH_MAX_ATTRS; ++i) op.attrs[i] = i < n_attrs ? attrs[i] : 0;
  const int cs = count_slot(kind);
  if (cs >= 0 && cs >= n_attrs) op.attrs[cs] = 1;
  if (kind == NF_OP_CONV2D && n_attrs <= 5) op.attrs[5] = 1;
  g->ops.push_back(op);
  return id;
}

int netfuse_graph_get_op(const nf_graph* g, int id, int* kind, int* concat_dim, int* source, int* parents,
                         int parents_cap, long* attrs) {
  if (!g || id < 0 || id >= (int)g->ops.size() || parents_cap < 0) return -(int)NF_EINVAL;
  const Op& op = g->ops[id];
  if (kind) *kind = op.kind;
  if (concat_dim) *concat_dim = op.dim;
  if (source) *source = op.source;
  if (parents)
    for (int i = 0; i < (int)op.parents.size() && i < parents_cap; ++i) parents[i] = op.parents[i];
  if (attrs)
    for (int i = 0; i < NF_GRAPH_MAX_ATTRS; ++i) attrs[i] = op.attrs[i];
  return (int)op.parents.size();
}

nf_graph* netfuse_graph_merge(const nf_graph* common, int M) {
  if (!common || M <= 0) return nullptr;
  const std::vector<Op>& V = common->ops;
  const int n = (int)V.size();
  std::vector<std::vector<int>> children(n);
  for (int i = 0; i < n; ++i)
    for (int p : V[i].parents) {
      if (V[p].kind == NF_OP_TASK_HEAD) return nullptr;   // nothing past the backbone is merged or described
      children[p].push_back(i);
    }

  nf_graph* out = new (std::nothrow) nf_graph();
  if (!out) return nullptr;
  std::vector<Op>& Vm = out->ops;
  Vm.reserve(n + n / 4);
  std::vector<int> m_of(n, -1);                       // merged operation of op_i; -1 = not visited
  std::deque<int> Q;
  for (int i = 0; i < n; ++i)
    if (V[i].parents.empty()) Q.push_back(i);         // root operations
  int visited = 0;
  while (!Q.empty()) {
    const int i = Q.front();
    Q.pop_front();
    if (m_of[i] >= 0) continue;
    bool ready = true;
    for (int p : V[i].parents) ready = ready && m_of[p] >= 0;
    if (!ready) continue;                             // comes back with its last parent
    Op m = V[i];
    m.source = i;
    m.dim = merge_op(m, M);
    for (int& p : m.parents) p = m_of[p];             // copied dependencies (m_j, m_i)
    if (m.dim == NF_DIM_DONTCARE) {
      // the concatenation dimension of the parents; the majority if they disagree, the first on a tie
      int nb = 0, nc = 0, first = NF_DIM_DONTCARE;
      for (int p : m.parents) {
        const int d = Vm[p].dim;
        if (d == NF_DIM_DONTCARE) continue;
        if (first == NF_DIM_DONTCARE) first = d;
        (d == NF_DIM_BATCH ? nb : nc)++;
      }
      m.dim = nb == nc ? first : (nb > nc ? NF_DIM_BATCH : NF_DIM_CHANNEL);
    }
    for (int& p : m.parents) {
      if (!conflict(Vm[p].dim, m.dim)) continue;
      Op r;                                            // ReshapeAndTransposeOp(d_j, d_i) on the edge (m_j, m_i)
      r.kind = NF_OP_RESHAPE_TRANSPOSE; r.dim = m.dim; r.source = -1;
      r.parents.push_back(p);
      for (long& a : r.attrs) a = 0;
      r.attrs[0] = Vm[p].dim; r.attrs[1] = m.dim;
      Vm.push_back(r);
      p = (int)Vm.size() - 1;
    }
    Vm.push_back(m);
    m_of[i] = (int)Vm.size() - 1;
    ++visited;
    for (int c : children[i])
      if (m_of[c] < 0) Q.push_back(c);
  }
  if (visited != n) {                                 // unreachable operations: not a well-formed subgraph
    delete out;
    return nullptr;
  }
  return out;
}

int netfuse_graph_lower(const nf_graph* merged, nf_call* calls, int cap) {
  if (!merged || cap < 0 || (cap > 0 && !calls)) return -(int)NF_EINVAL;
  const std::vector<Op>& V = merged->ops;
  const int n = (int)V.size();
  std::vector<std::vector<int>> consumers(n);
  for (int i = 0; i < n; ++i)
    for (int p : V[i].parents) consumers[p].push_back(i);
  std::vector<char> folded(n, 0);
  // the single consumer of `id` if it has exactly one and that one is of `kind`, else -1
  auto sole = [&](int id, int kind) {
    return consumers[id].size() == 1 && V[consumers[id][0]].kind == kind ? consumers[id][0] : -1;
  };
  // alias[q] = the operation whose output tensor stands for q's (a reshape that was not materialised)
  std::vector<int> alias(n);
  for (int i = 0; i < n; ++i) alias[i] = i;
  int count = 0;
  auto emit = [&](nf_call c) {
    if (c.input >= 0) c.input = alias[c.input];
    if (c.residual >= 0) c.residual = alias[c.residual];
    if (count < cap) calls[count] = c;
    ++count;
  };
  for (int i = 0; i < n; ++i) {
    if (folded[i]) continue;
    const Op& op = V[i];
    nf_call c;
    c.call = NF_CALL_UNFUSED; c.op = i; c.input = op.parents.empty() ? -1 : op.parents[0];
    c.residual = -1; c.output = i; c.act = NF_ACT_NONE; c.batchnorm = -1; c.layout = 0;
    switch (op.kind) {
      case NF_OP_INPUT: continue;
      case NF_OP_CONV2D: {
        c.call = NF_CALL_CONV2D;
        int cur = i, nx;
        if ((nx = sole(cur, NF_OP_BATCHNORM)) >= 0) { c.batchnorm = nx; folded[nx] = 1; cur = nx; }
        // the addition is folded when this chain is its LATER operand (the other one, or what stands for it when
        // it is a reshape that is not materialised, is computed by then)
        if ((nx = sole(cur, NF_OP_ADD)) >= 0 && V[nx].parents.size() == 2) {
          const int other = V[nx].parents[0] == cur ? V[nx].parents[1] : V[nx].parents[0];
          if (alias[other] < i) { c.residual = other; folded[nx] = 1; cur = nx; }
        }
        if ((nx = sole(cur, NF_OP_RELU)) >= 0) { c.act = NF_ACT_RELU; folded[nx] = 1; cur = nx; }
        c.output = cur;
        break;
      }
      case NF_OP_MATMUL: {
        c.call = NF_CALL_LINEAR;
        int cur = i, nx;
        if ((nx = sole(cur, NF_OP_GELU)) >= 0) { c.act = NF_ACT_GELU; folded[nx] = 1; cur = nx; }
        else if ((nx = sole(cur, NF_OP_RELU)) >= 0) { c.act = NF_ACT_RELU; folded[nx] = 1; cur = nx; }
        if ((nx = sole(cur, NF_OP_ADD)) >= 0 && V[nx].parents.size() == 2) {
          const int other = V[nx].parents[0] == cur ? V[nx].parents[1] : V[nx].parents[0];
          if (alias[other] < i) { c.residual = other; folded[nx] = 1; cur = nx; }
        }
        c.output = cur;
        break;
      }
      case NF_OP_RESHAPE_TRANSPOSE: {
        // a reshape whose only consumer is a layer normalisation is absorbed by it (below)
        const int nx = sole(i, NF_OP_LAYERNORM);
        if (nx >= 0 && V[nx].parents.size() == 1) continue;
        c.call = NF_CALL_MERGE_TRANSPOSE;
        c.layout = op.attrs[1] == NF_DIM_CHANNEL;
        break;
      }
      case NF_OP_LAYERNORM: {
        c.call = NF_CALL_LAYERNORM;
        c.layout = NF_MERGE_CHANNEL;
        const int p = op.parents.empty() ? -1 : op.parents[0];
        if (p >= 0 && V[p].kind == NF_OP_RESHAPE_TRANSPOSE && consumers[p].size() == 1 && V[p].attrs[1] == NF_DIM_CHANNEL) {
          // batch-merged producer behind a reshape that only this normalisation reads
          bool all_back = true;
          for (int q : consumers[i])
            all_back = all_back && V[q].kind == NF_OP_RESHAPE_TRANSPOSE && V[q].attrs[1] == NF_DIM_BATCH;
          if (all_back) {
            // every consumer wants the batch-merged form back (or there is none): the normalisation reads and
            // writes the producer's layout and the reshapes on both sides disappear
            c.input = V[p].parents[0];
            c.layout = NF_MERGE_BATCH;
            for (int q : consumers[i]) { folded[q] = 1; alias[q] = i; }
          } else {
            // someone needs the channel-merged form: the reshape in front of the normalisation is materialised
            nf_call t;
            t.call = NF_CALL_MERGE_TRANSPOSE; t.op = p; t.input = alias[V[p].parents[0]]; t.residual = -1; t.output = p;
            t.act = NF_ACT_NONE; t.batchnorm = -1; t.layout = 1;
            emit(t);
          }
        }
        break;
      }
      case NF_OP_TASK_HEAD: c.call = NF_CALL_LINEAR_RAGGED; break;
      case NF_OP_ATTENTION: c.call = NF_CALL_ATTENTION; break;
      case NF_OP_ATTENTION_RELPOS:
        if (op.parents.size() != 2) break;                 // NF_CALL_UNFUSED: not the two-operand form
        c.call = NF_CALL_ATTENTION_RELPOS;
        c.residual = op.parents[1];
        break;
      case NF_OP_MAXPOOL: c.call = NF_CALL_MAXPOOL; break;
      case NF_OP_AVGPOOL_GLOBAL: c.call = NF_CALL_AVGPOOL_GLOBAL; break;
      case NF_OP_BATCHNORM: case NF_OP_RELU: case NF_OP_GELU: case NF_OP_ADD: break;       // NF_CALL_UNFUSED
    }
    emit(c);
  }
  return count;
}

}  // extern "C"
