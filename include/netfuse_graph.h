/*
 * netfuse_graph.h -- host-side C ABI of the DNN merging algorithm of NetFuse (Section 3.2, Algorithm 1)
 * and of its lowering to calls of netfuse.h.  Pure host code: nothing here touches the GPU.
 *
 * The caller describes the COMMON SUBGRAPH (V, E) of the M networks -- one architecture, one node per
 * operation -- with netfuse_graph_add_op, parents before children.  netfuse_graph_merge runs Algorithm 1:
 * a breadth-first traversal from the root operations in which every operation is merged per Section 3.1
 * (Table 1), receives the dimension its M instances are concatenated along (Batch, Channel or, for
 * operations without weights, DontCare = the majority of its parents), and gets a reshape-and-transpose
 * operation on every incoming edge whose dimension conflicts (Batch against Channel).  Time O(|V| + |E|).
 *
 * Common backbones (Section 3.2, last paragraph; Section 6): networks that share a backbone but end in layers
 * of their own -- the fully connected layers of different downstream tasks -- are merged up to those layers,
 * which stay as they are.  Such a layer is described once, as NF_OP_TASK_HEAD (a fully connected layer whose
 * output width differs from network to network, so it carries no width): netfuse_graph_merge does NOT merge it
 * -- its K is unchanged -- but records that M instances of it follow, each reading its own network's rows of
 * the backbone's output, i.e. the batch-concatenated form (a reshape is inserted if the backbone ends channel-
 * concatenated).  It must be a leaf: nothing past the backbone is merged, so nothing past it is described.
 *
 * Attribute slots per kind (netfuse_graph_add_op's attrs, and what netfuse_graph_get_op returns):
 *   NF_OP_MATMUL       { K, Nout, has_bias, batch }              batch: 1 in a single model, M after merging
 *   NF_OP_CONV2D       { Cin, Cout, k, stride, pad, groups, has_bias }   Cin, Cout, groups are multiplied by M
 *   NF_OP_LAYERNORM    { H, groups }                             groups: 1 -> M (a group normalisation)
 *   NF_OP_BATCHNORM    { C }                                     C -> M * C
 *   NF_OP_ATTENTION    { heads, d, batch }                       batch: 1 -> M
 *   NF_OP_MAXPOOL      { k, stride, pad }
 *   NF_OP_RESHAPE_TRANSPOSE { from_dim, to_dim }                 merged graphs only
 *   NF_OP_TASK_HEAD    { K, has_bias, instances }                instances: 1 -> M (M unmerged layers)
 *   NF_OP_ATTENTION_RELPOS { heads, d, batch }                   batch: 1 -> M; parents: the packed Q|K|V tensor,
 *                                                                then the projected position encodings
 *   others             none
 * Trailing slots that are not passed default to 1 for batch / groups / instances and to 0 otherwise.
 *
 * Readings where the printed algorithm is silent: an operation is processed once all its parents are
 * (one reached early through a short branch waits); DontCare is compatible with both definite
 * dimensions; the majority vote ignores DontCare parents and a tie goes to the first parent.
 *
 * Errors: functions returning int return a negative value (the negated nf_status of netfuse.h) on
 * invalid arguments; functions returning a graph return NULL.  Graphs are owned by the caller and freed
 * with netfuse_graph_destroy.  A graph is not thread-safe; different graphs are independent.
 */
#ifndef NETFUSE_GRAPH_H
#define NETFUSE_GRAPH_H

#ifdef __cplusplus
extern "C" {
#endif

typedef struct nf_graph nf_graph;

typedef enum {
  NF_OP_INPUT = 0, NF_OP_MATMUL = 1, NF_OP_CONV2D = 2, NF_OP_LAYERNORM = 3, NF_OP_BATCHNORM = 4,
  NF_OP_ATTENTION = 5, NF_OP_RELU = 6, NF_OP_GELU = 7, NF_OP_ADD = 8, NF_OP_MAXPOOL = 9,
  NF_OP_AVGPOOL_GLOBAL = 10, NF_OP_RESHAPE_TRANSPOSE = 11, NF_OP_TASK_HEAD = 12,
  NF_OP_ATTENTION_RELPOS = 13
} nf_op_kind;

/* d_i of Algorithm 1: the dimension along which the tensors of the M instances are concatenated */
typedef enum { NF_DIM_BATCH = 0, NF_DIM_CHANNEL = 1, NF_DIM_DONTCARE = 2 } nf_concat_dim;

#define NF_GRAPH_MAX_ATTRS 8

nf_graph* netfuse_graph_create(void);
void netfuse_graph_destroy(nf_graph* g);

/* Appends an operation; parents are ids returned by earlier calls.  Returns the new id (>= 0). */
int netfuse_graph_add_op(nf_graph* g, int kind, const int* parents, int n_parents, const long* attrs,
                         int n_attrs);
int netfuse_graph_size(const nf_graph* g);

/* Algorithm 1.  The result lists every merged operation in the order it was visited, each preceded by the
 * reshape operations inserted on its incoming edges, so parents always precede children.  NULL for M <= 0, a
 * graph with unreachable operations, or a task head that has a consumer. */
nf_graph* netfuse_graph_merge(const nf_graph* common, int M);

/* Reads operation `id`: kind, concatenation dimension (NF_DIM_DONTCARE in an un-merged graph), the id of the
 * operation of the common subgraph it was merged from (-1 for an inserted reshape, its own id in an
 * un-merged graph), up to parents_cap parent ids and NF_GRAPH_MAX_ATTRS attributes.  Returns the number
 * of parents. */
int netfuse_graph_get_op(const nf_graph* g, int id, int* kind, int* concat_dim, int* source, int* parents,
                         int parents_cap, long* attrs);

/*
 * Lowering of a merged graph to library calls.  Operations without weights are folded into the epilogue
 * of the producing call where netfuse.h offers one, and a reshape between a batch matmul and a group
 * normalisation is not materialised (netfuse_layernorm reads either layout):
 *   conv2d [-> batchnorm] [-> add(residual)] [-> relu]      one netfuse_conv2d (scale/shift, residual, act)
 *   matmul [-> gelu | relu] [-> add(residual)]              one netfuse_linear (act before the residual)
 *   [reshape ->] layernorm [-> reshape]                     one netfuse_layernorm in the producer's layout
 *   attention, maxpool, avgpool_global                      one call each
 *   relative-position attention                             one netfuse_attention_relpos; the call's `residual`
 *                                                            field names its second operand (the positions)
 *   any other reshape                                       netfuse_merge_transpose
 *   task head (M unmerged fully connected layers)           one netfuse_linear_ragged: the M layers in one
 *                                                            launch, each with its own output width (the
 *                                                            caller holds the widths and the weights)
 *   relu / gelu / add that could not be folded              NF_CALL_UNFUSED (the caller has no entry point for
 *                                                            them; none of the workloads produces one)
 * A producer is folded into only when the folded operation is its single consumer.
 */
typedef enum {
  NF_CALL_LINEAR = 0, NF_CALL_CONV2D = 1, NF_CALL_LAYERNORM = 2, NF_CALL_ATTENTION = 3, NF_CALL_MAXPOOL = 4,
  NF_CALL_AVGPOOL_GLOBAL = 5, NF_CALL_MERGE_TRANSPOSE = 6, NF_CALL_UNFUSED = 7, NF_CALL_LINEAR_RAGGED = 8,
  NF_CALL_ATTENTION_RELPOS = 9
} nf_call_kind;

typedef struct {
  int call;       /* nf_call_kind */
  int op;         /* merged operation that carries the weights / attributes (matmul, conv2d, layernorm, ...) */
  int input;      /* merged operation whose output tensor is this call's input */
  int residual;   /* merged operation whose output is added in the epilogue, or -1
                     (NF_CALL_ATTENTION_RELPOS: the operation that produces the projected position encodings) */
  int output;     /* last merged operation folded into the call: its output tensor is the call's output */
  int act;        /* nf_act of the epilogue */
  int batchnorm;  /* folded batch normalisation operation (conv2d), or -1 */
  int layout;     /* NF_CALL_LAYERNORM: nf_merge_dim of the tensors it reads and writes;
                     NF_CALL_MERGE_TRANSPOSE: 1 = to the channel-merged form */
} nf_call;

/* Writes up to `cap` calls in execution order; returns how many the graph needs (call again with a larger
 * buffer if that exceeds cap). */
int netfuse_graph_lower(const nf_graph* merged, nf_call* calls, int cap);

#ifdef __cplusplus
}
#endif
#endif /* NETFUSE_GRAPH_H */
