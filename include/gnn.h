/*
 * gnn.h -- C ABI of the MI355X (gfx950) message-passing library.
 *
 * The library implements the forward hot path of graph message passing as the
 * paper describes it (section 3, "Message Passing"): for every edge j -> i a
 * message is built from the source node's features x_j and the edge's own data
 * e_(j->i) (apply_edges), and the messages are reduced over each destination
 * node's neighbourhood (aggregate_neighbors); `propagate` fuses the two, and
 * particular (message, reduction) pairs are sparse-times-dense products.
 *
 * Conventions (all entry points):
 *   - nodes are 0..N-1, edges 0..E-1, indices are int32_t; edge k carries a
 *     message from src[k] (j) to dst[k] (i) and is reduced at i;
 *   - features are float, row-major [N x F] (one node's F values contiguous);
 *     this is byte-identical to the paper's column-major [F x N] Julia arrays;
 *   - multi-edges and self-loops are legal and count with multiplicity;
 *   - a node without incoming edges receives 0 for sum, mean and max alike;
 *   - every pointer named d_* is DEVICE memory owned by the caller; the library
 *     neither frees nor keeps it after the call returns (the call only enqueues
 *     work: the memory must stay valid until that work has run);
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream);
 *     compute calls enqueue kernels and return without synchronising;
 *   - outputs must not alias inputs;
 *   - errors are reported by return code only.  Argument errors are found on the
 *     host before anything is launched.  Inputs are finite by contract.
 *
 * All device work runs on the device that is current when gnn_build_csr is
 * called; the caller keeps that device current for later calls on the graph.
 *
 * Which calls allocate or synchronise: the graph builders (gnn_build_csr*, which read back a flag and the list
 * sizes), gnn_graph_reserve, gnn_graph_build_edge_route, gnn_graph_destroy, gnn_release_cached_memory and
 * gnn_check_graph_indicator.
 * Every other call only enqueues kernels on `stream`: it never allocates, frees or synchronises, so it may be
 * recorded into a HIP graph from its first use on.
 *
 * Concurrency: a graph handle carries scratch memory for rows that are split over several wavefronts and for
 * per-row softmax statistics (a part of the graph's one allocation, sized when the graph is built; see
 * gnn_graph_reserve) and, after gnn_graph_build_edge_route, the route's buffers, so compute calls on ONE handle
 * must not overlap: issue them on one stream, or order them
 * with events.  Calls on different handles are independent and may come from different host threads; the
 * process-wide buffer that graph builds share is handed to one build at a time (a concurrent build allocates
 * its own temporaries).  Caller-provided workspaces follow the same rule as the handle: one call at a time
 * per workspace.
 */
#ifndef GNN_MI355X_H
#define GNN_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gnn_graph gnn_graph; /* opaque: owns device rowptr/colidx/perm/in-degree + work lists */

typedef enum {
    GNN_OK = 0,
    GNN_ERR_NULL = 1,        /* a required pointer is NULL */
    GNN_ERR_BAD_SIZE = 2,    /* N <= 0, E < 0, E >= 2^31, a dimension <= 0, unknown enum, short workspace */
    GNN_ERR_INDEX_RANGE = 3, /* a node id outside [0, N) (or a graph id outside [0, G)) */
    GNN_ERR_UNSUPPORTED = 4, /* combination not implemented */
    GNN_ERR_ALLOC = 5,       /* device allocation failed */
    GNN_ERR_DEVICE = 6,      /* a HIP call or launch failed */
    GNN_ERR_NOT_SORTED = 7,  /* graph_indicator is not non-decreasing (gnn_check_graph_indicator) */
    GNN_ERR_NOT_RESERVED = 8,/* the graph's scratch memory is too small for this call: gnn_graph_reserve first */
    GNN_ERR_SCRATCH_LIMIT = 9/* gnn_propagate_noalloc: the call needs more than the fixed scratch array holds */
} gnn_status;

/*
 * Message of edge k = (j -> i) built from the target's features x_i, the source's features x_j and the
 * edge's data e (paper section 3, "Message Passing": the message function takes xi, xj, e):
 *   COPY_XJ   m = x_j                       E_MUL_XJ  m = e * x_j (e_dim = 1 broadcasts, e_dim = F element-wise)
 *   XJ_SUB_XI m = x_j - x_i                 XI_DOT_XJ m = <x_i, x_j>, one scalar per edge (gnn_apply_edges only)
 * Reductions over a node's incoming edges; a node without incoming edges gets 0 under every one of
 * them; MIN puts -0 below +0 as MAX puts +0 above -0; PROD multiplies in a fixed order.
 */
typedef enum { GNN_MSG_COPY_XJ = 0, GNN_MSG_E_MUL_XJ = 1, GNN_MSG_XJ_SUB_XI = 2, GNN_MSG_XI_DOT_XJ = 3 } gnn_msg_op;
typedef enum { GNN_AGGR_SUM = 0, GNN_AGGR_MEAN = 1, GNN_AGGR_MAX = 2, GNN_AGGR_MIN = 3, GNN_AGGR_PROD = 4 } gnn_aggr;
typedef enum { GNN_EDGE_ORDER_COO = 0, GNN_EDGE_ORDER_CSR = 1 } gnn_edge_order;
typedef enum { GNN_ACT_NONE = 0, GNN_ACT_RELU = 1 } gnn_activation;

/* Static text for a status code (spec boundary: errors are reported by return code only). */
const char *gnn_status_string(gnn_status s);

/*
 * COO -> CSR by destination (paper section 3, "Graph Data Structures": COO is
 * the default topology encoding and a sparse adjacency encodes the same graph).
 *
 * d_src, d_dst : device, [num_edges] each (may be NULL only if num_edges == 0).
 * On success *out_graph owns device arrays
 *   rowptr[N+1] (exclusive prefix sum of the in-degrees), in-degree[N],
 *   perm[E]   = the STABLE permutation that sorts the edges by destination
 *               (a row lists its edges in increasing original edge index),
 *   colidx[E] = src[perm[p]],
 * plus the degree-bucketed work lists the compute calls use.  The sort is a
 * least-significant-digit radix sort on the destination id.
 * Synchronises the stream (it reads back the range-check flag and list sizes).
 * Errors: GNN_ERR_NULL, GNN_ERR_BAD_SIZE, GNN_ERR_INDEX_RANGE (no graph is
 * returned), GNN_ERR_ALLOC, GNN_ERR_DEVICE.  num_edges == 0 is valid.
 */
gnn_status gnn_build_csr(const int32_t *d_src, const int32_t *d_dst, int64_t num_edges,
                         int32_t num_nodes, void *stream, gnn_graph **out_graph);

/*
 * Same, with the two scheduling thresholds exposed.  Both 0: the library defaults (16, and 256 / 512 / 1024
 * edges per piece growing with the number of edges).  chunk_edges alone 0: its default, with small_max_degree
 * taken as given (0 then means that every non-empty row is cut into wavefront pieces).
 * rows with in-degree <= small_max_degree are reduced by a sub-group of a
 * wavefront; longer rows are cut into pieces of at most chunk_edges edges, one
 * wavefront each (pieces of one row are combined in a fixed order afterwards).
 * The thresholds change scheduling only, never which edges a row holds.
 * small_max_degree in [0, 64], chunk_edges a multiple of 64 in [64, 65536].
 */
gnn_status gnn_build_csr_ex(const int32_t *d_src, const int32_t *d_dst, int64_t num_edges,
                            int32_t num_nodes, int32_t small_max_degree, int32_t chunk_edges,
                            void *stream, gnn_graph **out_graph);

/*
 * Temporal graphs (paper section 3, "Graph Data Structures": a temporal graph is a sequence of snapshot
 * graphs over time): num_snapshots edge lists over ONE node set of num_nodes nodes are turned into
 * num_snapshots handles with one device allocation (shared by the handles and freed with the last of
 * them), one stream synchronisation and ONE set of kernel launches -- every kernel of the build takes the
 * snapshot as a grid dimension, so the launch count does not grow with the number of snapshots (256 snapshots
 * of 20 000 edges: 1.4 ms against 48 ms for 256 separate builds).
 * d_src, d_dst : HOST arrays of num_snapshots DEVICE pointers, snapshot t holding num_edges[t] edges
 * (num_edges is a HOST array; an entry may be 0, its pointers then may be NULL).
 * out_graphs   : HOST array of num_snapshots handle slots.  Every handle is an ordinary graph (same CSR,
 * same work lists, bit for bit, as gnn_build_csr on that snapshot alone) and is destroyed on its own with
 * gnn_graph_destroy.  Errors as gnn_build_csr; on any error no handle is returned (all slots NULL), and
 * GNN_ERR_INDEX_RANGE means that at least one snapshot holds a node id outside [0, num_nodes).
 */
gnn_status gnn_build_csr_batch(int32_t num_snapshots, const int32_t *const *d_src, const int32_t *const *d_dst,
                               const int64_t *num_edges, int32_t num_nodes, void *stream, gnn_graph **out_graphs);

/*
 * One relation of a heterogeneous graph (paper section 3, "Graph Data Structures": graphs with several
 * node and edge types): edges from a source node set of num_src_nodes nodes to a destination node set of
 * num_dst_nodes nodes.  d_src[k] in [0, num_src_nodes), d_dst[k] in [0, num_dst_nodes); the CSR has one
 * row per destination node.  Such a handle is accepted by gnn_propagate (x has num_src_nodes rows, the
 * result num_dst_nodes), gnn_apply_edges / gnn_aggregate_neighbors, gnn_segment_softmax and
 * gnn_hetero_propagate; what needs a node's own features next to its neighbours' (self-loops, x_j - x_i,
 * the layers, the backward passes) returns GNN_ERR_UNSUPPORTED.
 */
gnn_status gnn_build_csr_bipartite(const int32_t *d_src, const int32_t *d_dst, int64_t num_edges,
                                   int32_t num_src_nodes, int32_t num_dst_nodes, void *stream,
                                   gnn_graph **out_graph);

/*
 * gnn_build_csr keeps its temporaries (about 16 bytes per edge) in one device buffer per process between
 * calls, and gnn_graph_destroy keeps the arrays of one destroyed graph, or of one batch of graphs once its last
 * handle is destroyed (the largest block it has seen), for the next build or batch build of a similar size, so that building and destroying graph after graph -- one per mini-batch -- does not
 * allocate and free each time.  This call frees both (GNN_ERR_UNSUPPORTED, with the graph arrays already
 * freed, if a build is using the temporaries on another thread); the next build allocates again.
 */
gnn_status gnn_release_cached_memory(void);

/*
 * Sizes the graph's scratch memory (partial rows of nodes whose edges are split over several wavefronts --
 * section 3 "Message Passing": the reduction over a neighbourhood, here cut into pieces for hub nodes -- and the
 * per-node softmax statistics).  After it returns GNN_OK, on this graph
 *   gnn_propagate / gnn_aggregate_neighbors / gnn_gin_update / gnn_gcnconv / their backward calls accept
 *     feat_dim (f_in, f_out) up to 3 * max_feat_dim,
 *   gnn_gatconv / gnn_gatconv_backward accept heads * ch up to max_feat_dim,
 *   gnn_segment_softmax / gnn_segment_softmax_backward accept up to max_heads heads.
 * A freshly built graph is reserved for max_feat_dim = 128 (384 floats for every partial row its edge count
 * could give rise to): wider features need this call, and so does the segment softmax on all but small graphs
 * (it keeps two floats per node and head: call gnn_graph_reserve(g, 0, heads) once before using it).  A
 * compute call beyond what is reserved returns GNN_ERR_NOT_RESERVED and launches nothing.  The reservation
 * only grows.
 * This call may allocate and then synchronises the DEVICE (kernels enqueued earlier may use the buffer it
 * replaces): call it when the graph is set up, not between enqueued work and not during stream capture.
 * Errors: GNN_ERR_NULL, GNN_ERR_BAD_SIZE (a negative size), GNN_ERR_ALLOC, GNN_ERR_DEVICE.
 */
gnn_status gnn_graph_reserve(gnn_graph *g, int32_t max_feat_dim, int32_t max_heads);

/*
 * Destroys the graph.  The caller makes sure no enqueued work still uses it: its device arrays are freed or
 * handed to a later gnn_build_csr call (see gnn_release_cached_memory).
 */
gnn_status gnn_graph_destroy(gnn_graph *g);

/*
 * The sparse (by-destination) encoding of the topology that section 3, "Graph Data Structures", names next to
 * COO, as borrowed device pointers / sizes, valid until gnn_graph_destroy.  NULL / 0 for a NULL graph.
 */
const int32_t *gnn_graph_rowptr(const gnn_graph *g);   /* [N+1] */
const int32_t *gnn_graph_colidx(const gnn_graph *g);   /* [E]   */
const int32_t *gnn_graph_perm(const gnn_graph *g);     /* [E]   */
const int32_t *gnn_graph_indegree(const gnn_graph *g); /* [N]   */
int32_t gnn_graph_num_nodes(const gnn_graph *g);       /* rows = destination nodes */
int32_t gnn_graph_num_src_nodes(const gnn_graph *g);   /* differs only for gnn_build_csr_bipartite */
int64_t gnn_graph_num_edges(const gnn_graph *g);
/*
 * Host-side sizes of the work lists that schedule the reduction over each neighbourhood (section 3, "Message
 * Passing") by in-degree: rows reduced by a sub-group, wavefront work items, split rows.
 */
void gnn_graph_work_sizes(const gnn_graph *g, int32_t *n_small_rows, int32_t *n_items, int32_t *n_split_rows);
/*
 * Borrowed device pointers to the work lists themselves (introspection and tests; any argument may be NULL):
 *   small_rows[n_small_rows]   the short rows, ascending;
 *   item_row / item_start / item_slot [n_items]   one entry per piece of a longer row, rows ascending and a row's
 *     pieces in order: the row, the piece's first CSR position, and its partial-result slot (-1 when the row is one
 *     piece; a split row's pieces have consecutive slots);
 *   split_rows / split_slot0 [n_split_rows]   the rows made of several pieces, ascending, and their first slot.
 */
void gnn_graph_work_lists(const gnn_graph *g, const int32_t **small_rows, const int32_t **item_row,
                          const int32_t **item_start, const int32_t **item_slot, const int32_t **split_rows,
                          const int32_t **split_slot0);

/*
 * Per-edge data (the edge features e of section 3, "Message Passing", stored per edge of the COO list) from
 * the caller's COO order into CSR order:
 *   d_e_csr[p, :] = d_e[perm[p], :],  both [E x e_dim] float.
 * Done once per graph and edge tensor so that compute calls stream edge data.
 */
gnn_status gnn_edge_data_to_csr(const gnn_graph *g, const float *d_e, int32_t e_dim,
                                float *d_e_csr, void *stream);

/*
 * The way back (gradients with respect to per-edge data come out of the kernels in CSR order, section 3,
 * "Message Passing"):  d_e[perm[p], :] = d_e_csr[p, :],  both [E x e_dim] float.  Only enqueues kernels.
 */
gnn_status gnn_edge_data_to_coo(const gnn_graph *g, const float *d_e_csr, int32_t e_dim,
                                float *d_e, void *stream);

/*
 * Optional set-up call for graphs whose per-edge scalars change every step (learned or recomputed edge weights of
 * section 3's e_mul_xj message): moving ONE float per edge between the caller's order and CSR order by perm is a
 * random 4-byte access per edge, and each costs a whole 128-byte memory line.  This call splits the permutation,
 * once, into two passes that only move data inside 16 384-entry ranges held in on-chip memory or in contiguous
 * runs; afterwards gnn_edge_data_to_csr / gnn_edge_data_to_coo with e_dim == 1, gnn_propagate, gnn_apply_edges
 * and gnn_propagate_backward with one weight per edge in COO order, the per-edge dot product of gnn_apply_edges,
 * the edge gradient of gnn_propagate_backward and gnn_segment_softmax(_backward) with one head in COO order
 * take the route (16-byte aligned buffers; anything else keeps the direct path).  Results are bit-identical: the
 * route only moves values.
 * Cost: 16 bytes of device memory per edge, owned by the graph (three index arrays, an intermediate buffer and a
 * CSR-ordered staging buffer for the compute calls; like the scratch memory it is shared by all calls on the graph,
 * so those must not overlap in time), and two sorting kernels of about three times a build's duration.
 * Allocates, enqueues on `stream` and waits for it; a second call is a no-op.
 * Errors: GNN_ERR_NULL, GNN_ERR_ALLOC, GNN_ERR_DEVICE.
 */
gnn_status gnn_graph_build_edge_route(gnn_graph *g, void *stream);

/*
 * propagate (paper section 3, "Message Passing"): for every node i
 *   out[i,:] = AGGR over edges k with dst[k] = i of  msg(x[dst[k],:], x[src[k],:], e[k,:])
 * msg  = COPY_XJ: x_j;   E_MUL_XJ: float(e * x_j) with e_dim == 1 (one weight per edge,
 *        broadcast over features) or e_dim == feat_dim (element-wise);   XJ_SUB_XI: float(x_j - x_i).
 * aggr = SUM, MEAN (divides by the number of incoming edges, not by a weight sum), MAX
 *        (the larger value; +0 beats -0), MIN (the smaller; -0 below +0), PROD.  No incoming edge -> 0.
 * d_x [N x feat_dim], d_out [N x feat_dim]; d_e [E x e_dim] in the order e_order names
 * (COO = the order the edges were given in, CSR = after gnn_edge_data_to_csr), NULL for COPY_XJ.
 * Any feat_dim > 0 is accepted; 16-byte aligned pointers with feat_dim % 4 == 0 take the
 * 128-bit path.  Calls on one graph must not overlap in time (they share the graph's
 * scratch buffer for rows that are split across wavefronts).  Only enqueues kernels.
 * Errors: GNN_ERR_NULL, GNN_ERR_BAD_SIZE, GNN_ERR_NOT_RESERVED (feat_dim beyond what the graph is
 * reserved for, see gnn_graph_reserve), GNN_ERR_DEVICE.
 */
gnn_status gnn_propagate(const gnn_graph *g, const float *d_x, int32_t feat_dim,
                         const float *d_e, int32_t e_dim, gnn_edge_order e_order,
                         gnn_msg_op msg, gnn_aggr aggr, float *d_out, void *stream);

/*
 * gnn_propagate for callers that cannot call the allocator at all -- code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc: same arguments, same kernels and bit-identical results, but the partial
 * rows of nodes whose edges are split over several wavefronts go to a fixed 16 MiB array inside the library's
 * device image instead of memory owned by the graph.  The call makes no allocation of any kind (its first call on
 * a device only asks the runtime for the address of that device's copy of the array).
 * Limit: (number of partial-row slots of the graph) * feat_dim <= 4 194 304 floats; beyond it the call returns
 * GNN_ERR_SCRATCH_LIMIT and launches nothing (the headline graph, 1 M nodes / 20 M edges, has 9 473 slots: 0.6 M
 * floats at feat_dim = 64).  All calls on one GPU share that GPU's array, whatever the graph: calls that overlap in time on
 * one GPU race, so keep them on one stream or order them with events.  The array keeps the last call's partial
 * rows; nothing in it has to be cleared, since a launch only reads partial rows it has written itself.
 */
gnn_status gnn_propagate_noalloc(const gnn_graph *g, const float *d_x, int32_t feat_dim, const float *d_e,
                                 int32_t e_dim, gnn_edge_order e_order, gnn_msg_op msg, gnn_aggr aggr,
                                 float *d_out, void *stream);

/*
 * Message passing on a heterogeneous graph, for one destination node type: the relations that end in it
 * are propagated one after the other and their results are summed,
 *   out[i,:] = sum over relations r of  AGGR over edges k of r with dst[k] = i of msg(x_r[src[k],:], e_r[k,:]).
 * graphs, d_x and d_e are HOST arrays of num_relations entries: graphs[r] a handle whose rows are the
 * destination type's nodes (all with the same gnn_graph_num_nodes), d_x[r] the DEVICE features of relation
 * r's source type [gnn_graph_num_src_nodes(graphs[r]) x feat_dim], d_e[r] its DEVICE edge data [E_r x e_dim]
 * (d_e may be NULL for COPY_XJ).  msg = COPY_XJ or E_MUL_XJ; aggr applies inside a relation.
 * Temporal snapshot graphs: gnn_build_csr_batch gives one handle per snapshot, then one gnn_propagate each.
 */
gnn_status gnn_hetero_propagate(int32_t num_relations, const gnn_graph *const *graphs,
                                const float *const *d_x, const float *const *d_e, int32_t feat_dim,
                                int32_t e_dim, gnn_edge_order e_order, gnn_msg_op msg, gnn_aggr aggr,
                                float *d_out, void *stream);

/*
 * propagate over node features stored as bfloat16 (the upper 16 bits of a float; half the gather
 * bytes of the float path).  Values are widened exactly, messages, sums and the result are float:
 * the result equals gnn_propagate on the widened features up to summation order.
 * msg = COPY_XJ or E_MUL_XJ with one float weight per edge (d_e [E], e_order as above), aggr = SUM,
 * MEAN or MAX; anything else GNN_ERR_UNSUPPORTED, as are feat_dim % 8 != 0 or pointers that are not
 * 16-byte aligned.  d_x_bf16 [N x feat_dim] uint16, d_out [N x feat_dim] float.
 * gnn_f32_to_bf16 converts finite floats with round-to-nearest-even (ties to the even 16-bit code).
 *
 * gnn_propagate_f16 / gnn_f32_to_f16: the same with IEEE binary16 storage (1 sign, 5 exponent, 10 fraction
 * bits; subnormals kept, |x| >= 65520 becomes infinity in the conversion -- features are expected to lie
 * inside the format's range, and propagate itself takes finite values only).
 */
gnn_status gnn_propagate_bf16(const gnn_graph *g, const uint16_t *d_x_bf16, int32_t feat_dim,
                              const float *d_e, gnn_edge_order e_order, gnn_msg_op msg, gnn_aggr aggr,
                              float *d_out, void *stream);
gnn_status gnn_f32_to_bf16(const float *d_in, int64_t count, uint16_t *d_out, void *stream);
gnn_status gnn_propagate_f16(const gnn_graph *g, const uint16_t *d_x_f16, int32_t feat_dim,
                             const float *d_e, gnn_edge_order e_order, gnn_msg_op msg, gnn_aggr aggr,
                             float *d_out, void *stream);
gnn_status gnn_f32_to_f16(const float *d_in, int64_t count, uint16_t *d_out, void *stream);

/*
 * The two un-fused primitives of the paper's listing (section 3, "Message Passing"):
 *
 * apply_edges: one message row per edge,  m[k,:] = msg(x[dst[k],:], x[src[k],:], e[k,:])  with the
 * message ops of gnn_propagate, plus XI_DOT_XJ (one scalar per edge: d_m is then [E x 1]).
 * d_m is [E x feat_dim], written in the order m_order names (COO = the
 * order the edges were given in, CSR = by destination, stable); d_e is read in e_order.
 *
 * aggregate_neighbors: reduces message rows onto their destinations,
 *   out[i,:] = AGGR over edges k with dst[k] = i of m[k,:]      (sum, mean over the edge count, max, min, prod)
 * with d_m [E x feat_dim] stored in m_order.  gnn_propagate gives the same result as the two
 * calls in a row without ever storing the messages.
 */
gnn_status gnn_apply_edges(const gnn_graph *g, const float *d_x, int32_t feat_dim, const float *d_e,
                           int32_t e_dim, gnn_edge_order e_order, gnn_msg_op msg, float *d_m,
                           gnn_edge_order m_order, void *stream);
gnn_status gnn_aggregate_neighbors(const gnn_graph *g, const float *d_m, int32_t feat_dim,
                                   gnn_edge_order m_order, gnn_aggr aggr, float *d_out, void *stream);

/*
 * Winners of a max aggregation (what the gradient of propagate with the max reduction routes along; the
 * paper's training example, section 3 "Training Example", differentiates through its layers): d_argmax[i,f] = the edge (id in the caller's numbering) whose message
 * is out[i,f], the FIRST such edge in increasing edge id on ties, -1 where node i has no incoming
 * edge.  d_out_max must be the result of gnn_propagate(..., GNN_AGGR_MAX, ...) on the same inputs.
 * d_argmax is [N x feat_dim] int32.
 */
gnn_status gnn_propagate_argmax(const gnn_graph *g, const float *d_x, int32_t feat_dim, const float *d_e,
                                int32_t e_dim, gnn_edge_order e_order, gnn_msg_op msg,
                                const float *d_out_max, int32_t *d_argmax, void *stream);

/*
 * Backward of gnn_propagate: given d_grad_out = dL/d out [N x feat_dim],
 *   d_grad_x [N x feat_dim]  = dL/dx:  row j = sum over edges k with src[k] = j of w[k,:] * g'[dst[k],:]
 *   d_grad_e [E x e_dim]     = dL/de in the caller's edge order (E_MUL_XJ only):
 *                              <x[src[k],:], g'[dst[k],:]> for e_dim == 1, the element-wise product otherwise
 * with w = 1 (COPY_XJ) or e, and g' = grad_out (SUM), grad_out[i,:] / in-degree(i) (MEAN), or
 * grad_out masked to the elements this edge won (MAX; d_argmax from gnn_propagate_argmax, else NULL).
 * g is the graph the forward call used; g_by_source is the same edge list sorted by source, i.e.
 * gnn_build_csr(d_dst, d_src, ...) with the two arrays exchanged (needed for d_grad_x only).
 * d_e is in the caller's edge order (both graphs share it through their perm arrays).
 * Either output may be NULL.  d_workspace: gnn_propagate_backward_workspace_bytes() bytes of device
 * scratch, 16-byte aligned (0 bytes unless MEAN).
 * Only COPY_XJ / E_MUL_XJ with SUM / MEAN / MAX are differentiated here; XJ_SUB_XI, MIN and PROD
 * return GNN_ERR_UNSUPPORTED.
 */
size_t gnn_propagate_backward_workspace_bytes(int32_t num_nodes, int32_t feat_dim, gnn_aggr aggr);
gnn_status gnn_propagate_backward(const gnn_graph *g, const gnn_graph *g_by_source, const float *d_x,
                                  int32_t feat_dim, const float *d_e, int32_t e_dim, gnn_msg_op msg,
                                  gnn_aggr aggr, const float *d_grad_out, const int32_t *d_argmax,
                                  float *d_grad_x, float *d_grad_e, void *d_workspace,
                                  size_t workspace_bytes, void *stream);

/*
 * GCNConv forward (layer named in the paper's training example; fused form of
 * propagate per section 3):   out = D^-1/2 (A [+ I]) D^-1/2 X W + b
 * with d_i = in-degree of i (+1 when add_self_loops != 0; one loop per node is
 * added without looking for loops already present); an edge j -> i carries
 * 1/sqrt(d_i d_j); a node with d = 0 contributes the coefficient 0.  act = GNN_ACT_RELU applies
 * max(., 0) to the result (the second graph convolution of the example model in section 3, "Training Example", has one), GNN_ACT_NONE leaves it.
 * d_x [N x f_in], d_w [f_in x f_out] row-major, d_bias [f_out] or NULL, d_out [N x f_out].
 * d_workspace: device scratch of at least gnn_gcnconv_workspace_bytes(N, f_out) bytes.
 * The two products are taken in the order that gathers the narrower rows: (Ahat X) W when f_in < f_out,
 * Ahat (X W) otherwise; results of the two orders differ by rounding only.  A handle built by
 * gnn_build_csr_bipartite is refused (GNN_ERR_UNSUPPORTED).
 */
size_t gnn_gcnconv_workspace_bytes(int32_t num_nodes, int32_t f_out);
gnn_status gnn_gcnconv(const gnn_graph *g, const float *d_x, int32_t f_in, const float *d_w,
                       const float *d_bias, int32_t f_out, int32_t add_self_loops, gnn_activation act,
                       float *d_out, void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Backward of gnn_gcnconv: with Ahat the normalised (self-looped) adjacency of the forward call and
 * G = d_grad_out [N x f_out]:   T = Ahat^T G;
 *   d_grad_x [N x f_in] = T W^T,   d_grad_w [f_in x f_out] = X^T T,   d_grad_b [f_out] = column sums of G.
 * Each output may be NULL.  g is the forward graph, g_by_source the same edges sorted by source
 * (gnn_build_csr with d_src and d_dst exchanged).  d_workspace: 256-byte aligned device scratch of
 * gnn_gcnconv_backward_workspace_bytes(N, f_in, f_out) bytes.
 */
size_t gnn_gcnconv_backward_workspace_bytes(int32_t num_nodes, int32_t f_in, int32_t f_out);
gnn_status gnn_gcnconv_backward(const gnn_graph *g, const gnn_graph *g_by_source, const float *d_x, int32_t f_in,
                                const float *d_w, int32_t f_out, int32_t add_self_loops,
                                const float *d_grad_out, float *d_grad_x, float *d_grad_w, float *d_grad_b,
                                void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Segment softmax over each destination's incoming edges, independently per head -- the normalisation of
 * per-edge attention scores in the attention layers section 3, "Graph Convolutional Layers", names (GAT): a
 * reduction over each neighbourhood followed by a per-edge rescale:
 *   out[k,h] = exp(s[k,h] - m[i,h]) / sum_{q: dst[q] = i} exp(s[q,h] - m[i,h]),  i = dst[k],
 * m = the segment maximum.  d_scores and d_out are [E x heads], both in the order `order` names.
 * Scores must be finite.  float arithmetic; the terms of the denominator are formed with the hardware's 2^x
 * (each within about (1 + |s - m|) * 2^-23 of its value), the numerator with the accurate exponential.
 * Needs gnn_graph_reserve(g, ., heads) once beforehand (else GNN_ERR_NOT_RESERVED); only enqueues kernels.
 */
gnn_status gnn_segment_softmax(const gnn_graph *g, const float *d_scores, int32_t heads,
                               gnn_edge_order order, float *d_out, void *stream);

/*
 * Backward of gnn_segment_softmax (training is the paper's purpose, section 3 "Training Example"):
 * the Jacobian of a softmax applied per destination segment and head,
 *   grad_scores[k,h] = alpha[k,h] * (grad_alpha[k,h] - sum_{q: dst[q] = dst[k]} alpha[q,h] grad_alpha[q,h]).
 * d_alpha is the forward result, d_grad_alpha = dL/d alpha, all three arrays [E x heads] in the order
 * `order` names.  No atomics: bitwise reproducible.  d_grad_scores must not alias the inputs.
 */
gnn_status gnn_segment_softmax_backward(const gnn_graph *g, const float *d_alpha, const float *d_grad_alpha,
                                        int32_t heads, gnn_edge_order order, float *d_grad_scores,
                                        void *stream);

/*
 * GAT-style attention layer (layer named in the paper, section 3 "Graph Convolutional Layers"):
 *   h = X W  [N x heads*ch];  sl[j,hd] = <a_src[hd,:], h[j,hd,:]>;  sr[i,hd] = <a_dst[hd,:], h[i,hd,:]>
 *   s[k,hd] = lrelu(sl[src[k],hd] + sr[dst[k],hd]),  lrelu(v) = v > 0 ? v : negative_slope * v
 *   out[i,hd,:] = sum_k softmax_i(s)[k,hd] * h[src[k],hd,:]      (heads concatenated)
 * No bias, no activation; self-loops only if the edge list holds them.  The softmax weights are formed with the
 * hardware's 2^x (each within about (1 + |s - m|) * 2^-23 of its value; they enter the result only as ratios).
 * d_w [f_in x heads*ch] row-major, d_a_src / d_a_dst [heads x ch], d_out [N x heads*ch].
 * d_softmax_stats (optional, may be NULL): [N x heads x 2] floats that receive, per destination and
 * head, the segment maximum of the scores and the softmax denominator relative to it (-inf and 0
 * for a node without incoming edges) -- what gnn_gatconv_backward needs from the forward pass.
 * d_workspace: at least gnn_gatconv_workspace_bytes(N, heads, ch) bytes of device scratch.
 */
size_t gnn_gatconv_workspace_bytes(int32_t num_nodes, int32_t heads, int32_t ch);
gnn_status gnn_gatconv(const gnn_graph *g, const float *d_x, int32_t f_in, const float *d_w,
                       const float *d_a_src, const float *d_a_dst, int32_t heads, int32_t ch,
                       float negative_slope, float *d_out, float *d_softmax_stats, void *d_workspace,
                       size_t workspace_bytes, void *stream);

/*
 * Backward of gnn_gatconv (training is the paper's purpose, section 3 "Training Example"): given
 * d_grad_out = dL/d out [N x heads*ch], the forward result d_out and the statistics the forward call
 * wrote to d_softmax_stats, computes
 *   d_grad_x [N x f_in], d_grad_w [f_in x heads*ch], d_grad_a_src, d_grad_a_dst [heads x ch]
 * (each may be NULL to skip it).  The attention weights are recomputed from per-node records, so no
 * [E x heads] tensor is stored.  g_by_source is a second handle built from the same edge list with
 * the roles of src and dst exchanged: gnn_build_csr(dst, src, ...).  The derivative of the leaky
 * ReLU at exactly 0 is negative_slope (the branch the forward takes).  No atomics: results are
 * bitwise reproducible.
 * Restriction: with L = ch / 4 when ch is a multiple of 4, else ch (the lanes a head occupies): L <= 64,
 * otherwise GNN_ERR_UNSUPPORTED (e.g. heads of 65 channels).
 * d_workspace: at least gnn_gatconv_backward_workspace_bytes(N, f_in, heads, ch) bytes, 256-byte aligned.
 */
size_t gnn_gatconv_backward_workspace_bytes(int32_t num_nodes, int32_t f_in, int32_t heads, int32_t ch);
gnn_status gnn_gatconv_backward(const gnn_graph *g, const gnn_graph *g_by_source, const float *d_x, int32_t f_in,
                                const float *d_w, const float *d_a_src, const float *d_a_dst, int32_t heads,
                                int32_t ch, float negative_slope, const float *d_out,
                                const float *d_softmax_stats, const float *d_grad_out, float *d_grad_x,
                                float *d_grad_w, float *d_grad_a_src, float *d_grad_a_dst, void *d_workspace,
                                size_t workspace_bytes, void *stream);

/*
 * Graph-level readout of a batch of graphs (GlobalPool in the paper's example):
 *   out[g,:] = AGGR over nodes i with graph_indicator[i] = g of x[i,:]
 * d_graph_indicator [num_nodes] must be non-decreasing with values in [0, num_graphs)
 * (what batching produces); a graph without nodes gets a zero row.  Sortedness and range
 * are the caller's contract; this call does not check them (gnn_check_graph_indicator does).
 */
gnn_status gnn_graph_pool(const int32_t *d_graph_indicator, int32_t num_nodes, int32_t num_graphs,
                          const float *d_x, int32_t feat_dim, gnn_aggr aggr, float *d_out,
                          void *stream);

/*
 * The same readout (GlobalPool of section 3, "Training Example") for batches of FEW, LARGE graphs -- 8 192 nodes
 * per graph or more on average, down to one graph that is the whole node set: gnn_graph_pool gives a graph one
 * thread block, which is slow when a graph has a million nodes.  With a workspace a graph is cut into parts of
 * about 2 048 nodes, one block each, and the parts are combined in a fixed order (no atomics; sums may differ
 * from gnn_graph_pool's by rounding order, max is identical).
 * gnn_graph_pool_workspace_bytes: bytes this needs, 0 when the batch is not of that kind (then gnn_graph_pool_ws
 * is gnn_graph_pool and d_workspace may be NULL).  d_workspace: 256-byte aligned.  Only enqueues kernels.
 * Errors: as gnn_graph_pool; GNN_ERR_NULL / GNN_ERR_BAD_SIZE for a missing, small or misaligned workspace.
 */
size_t gnn_graph_pool_workspace_bytes(int32_t num_nodes, int32_t num_graphs, int32_t feat_dim);
gnn_status gnn_graph_pool_ws(const int32_t *d_graph_indicator, int32_t num_nodes, int32_t num_graphs,
                             const float *d_x, int32_t feat_dim, gnn_aggr aggr, float *d_out,
                             void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Debug check of a graph_indicator (section 3, "Graph Data Structures": batching collates small graphs into
 * one graph whose nodes carry the index of their graph): GNN_OK if d_graph_indicator [num_nodes] is
 * non-decreasing with every value in [0, num_graphs), GNN_ERR_INDEX_RANGE for a value outside that range,
 * else GNN_ERR_NOT_SORTED.  Reads a flag back: it synchronises the stream (and allocates the flag).
 */
gnn_status gnn_check_graph_indicator(const int32_t *d_graph_indicator, int32_t num_nodes, int32_t num_graphs,
                                     void *stream);

/*
 * GIN-style node update without the MLP (layer named in the paper, section 3):
 *   out[i,:] = (1 + eps) * x[i,:] + sum_{j -> i} x[j,:]
 */
gnn_status gnn_gin_update(const gnn_graph *g, const float *d_x, int32_t feat_dim, float eps,
                          float *d_out, void *stream);

/*
 * The remaining layers of the paper's example model (section 3, "Training Example": a chain of two graph
 * convolutions with a batch normalisation and a relu in between, a mean readout per graph and a dense head).
 *
 * gnn_batchnorm: normalisation across the row (node) dimension,
 *   out[i,f] = act(gamma[f] * (x[i,f] - mean[f]) / sqrt(var[f] + eps) + beta[f]),
 * with mean / biased variance computed from the num_rows rows and WRITTEN to d_mean / d_var [feat_dim]
 * (use_given_stats == 0), or READ from them (use_given_stats != 0: stored statistics; no workspace
 * needed).  d_gamma / d_beta [feat_dim] may be NULL (1 and 0).  d_out may alias d_x.
 *
 * gnn_dense: out = act(X W + b), X [rows x k], W [k x n] row-major, b [n] or NULL.
 *
 * gnn_example_model_forward: the chain above on a collated batch: GCNConv(f0 => f1) with self-loops and
 * bias, batch norm over all nodes of the batch (batch statistics) + relu, GCNConv(f1 => f2) + relu, mean
 * pooling per graph (d_graph_indicator as for gnn_graph_pool), Dense(f2, f3).  d_y is [num_graphs x f3].
 * It runs the kernels of those entry points on the caller's stream, with one fusion: the normalised
 * activations are not written -- the second convolution's projection applies the normalisation and relu to the
 * rows of the first one's output as it reads them (the same arithmetic: results equal the call-by-call chain
 * bit for bit).
 * Workspaces: at least the matching *_workspace_bytes(), 256-byte aligned.
 */
size_t gnn_batchnorm_workspace_bytes(int32_t num_rows, int32_t feat_dim);
gnn_status gnn_batchnorm(const float *d_x, int32_t num_rows, int32_t feat_dim, const float *d_gamma,
                         const float *d_beta, float eps, gnn_activation act, int32_t use_given_stats,
                         float *d_mean, float *d_var, float *d_out, void *d_workspace,
                         size_t workspace_bytes, void *stream);
gnn_status gnn_dense(const float *d_x, int64_t rows, int32_t k, const float *d_w, int32_t n,
                     const float *d_bias, gnn_activation act, float *d_out, void *stream);
size_t gnn_example_model_workspace_bytes(int32_t num_nodes, int32_t num_graphs, int32_t f1, int32_t f2);
gnn_status gnn_example_model_forward(const gnn_graph *g, const int32_t *d_graph_indicator,
                                     int32_t num_graphs, const float *d_x, int32_t f0, const float *d_w1,
                                     const float *d_b1, int32_t f1, const float *d_gamma,
                                     const float *d_beta, float eps, const float *d_w2, const float *d_b2,
                                     int32_t f2, const float *d_w3, const float *d_b3, int32_t f3,
                                     float *d_y, void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Training-side pieces of the paper's example (section 3, "Training Example": mean-squared-error loss,
 * gradients of the whole chain, Adam update).  No atomics anywhere: a step is bitwise reproducible.
 *
 * gnn_mse_loss: *d_loss = mean (pred - target)^2 over `count` values, d_grad = 2 (pred - target) / count
 *   (either output may be NULL).  d_loss is a DEVICE scalar.
 * gnn_relu_backward: d_grad_x = d_y > 0 ? d_grad_y : 0, d_y being the relu's OUTPUT; d_grad_x may alias d_grad_y.
 * gnn_graph_pool_backward: every node of graph g receives d_grad_out[g,:] (SUM) or that divided by the
 *   graph's node count (MEAN); d_graph_indicator as for gnn_graph_pool (every node lies in a graph, so every
 *   row of d_grad_x is written).
 * gnn_dense_backward: for out = X W + b:  d_grad_x = gy W^T, d_grad_w = X^T gy, d_grad_b = column sums of gy
 *   (each may be NULL; an activation is differentiated by masking gy first).
 * gnn_batchnorm_backward: for y = gamma * xhat + beta with batch statistics (d_mean / d_var as written by
 *   gnn_batchnorm): d_grad_beta = sum_i g, d_grad_gamma = sum_i g xhat,
 *   d_grad_x = gamma / sqrt(var + eps) * (g - grad_beta / N - xhat * grad_gamma / N) (may be NULL), where
 *   g = d_grad_y, masked by d_y_relu > 0 when d_y_relu (the output of a fused relu) is not NULL.
 * gnn_adam_step: m = b1 m + (1 - b1) g;  v = b2 v + (1 - b2) g^2;
 *   p -= lr * (m / (1 - b1^step)) / (sqrt(v / (1 - b2^step)) + eps);   step counts from 1; p, m, v in place.
 * gnn_example_model_train_step: forward of gnn_example_model_forward, MSE loss against d_target
 *   [num_graphs x f3], gradients of all parameters and one Adam step on them.  d_params, d_adam_m, d_adam_v
 *   are HOST arrays of 8 DEVICE pointers in the order w1 [f0 x f1], b1 [f1], gamma [f1], beta [f1],
 *   w2 [f1 x f2], b2 [f2], w3 [f2 x f3], b3 [f3]; parameters and optimiser state are updated in place.
 *   g_by_source = gnn_build_csr(dst, src, ...).  d_loss (DEVICE scalar, may be NULL) receives the loss of
 *   the forward pass, i.e. before the update.
 * Workspaces: at least the matching *_workspace_bytes(), 256-byte aligned.
 */
gnn_status gnn_mse_loss(const float *d_pred, const float *d_target, int64_t count, float *d_loss,
                        float *d_grad, void *stream);
gnn_status gnn_relu_backward(const float *d_y, const float *d_grad_y, int64_t count, float *d_grad_x,
                             void *stream);
gnn_status gnn_graph_pool_backward(const int32_t *d_graph_indicator, int32_t num_nodes, int32_t num_graphs,
                                   const float *d_grad_out, int32_t feat_dim, gnn_aggr aggr,
                                   float *d_grad_x, void *stream);
size_t gnn_dense_backward_workspace_bytes(int64_t rows, int32_t k, int32_t n);
gnn_status gnn_dense_backward(const float *d_x, int64_t rows, int32_t k, const float *d_w, int32_t n,
                              const float *d_grad_y, float *d_grad_x, float *d_grad_w, float *d_grad_b,
                              void *d_workspace, size_t workspace_bytes, void *stream);
size_t gnn_batchnorm_backward_workspace_bytes(int32_t num_rows, int32_t feat_dim);
gnn_status gnn_batchnorm_backward(const float *d_x, int32_t num_rows, int32_t feat_dim, const float *d_gamma,
                                  const float *d_mean, const float *d_var, float eps,
                                  const float *d_grad_y, const float *d_y_relu, float *d_grad_x,
                                  float *d_grad_gamma, float *d_grad_beta, void *d_workspace,
                                  size_t workspace_bytes, void *stream);
gnn_status gnn_adam_step(float *d_param, float *d_m, float *d_v, const float *d_grad, int64_t count, float lr,
                         float beta1, float beta2, float eps, int32_t step, void *stream);
size_t gnn_example_model_train_workspace_bytes(int32_t num_nodes, int32_t num_graphs, int32_t f0, int32_t f1,
                                               int32_t f2, int32_t f3);
gnn_status gnn_example_model_train_step(const gnn_graph *g, const gnn_graph *g_by_source,
                                        const int32_t *d_graph_indicator, int32_t num_graphs,
                                        const float *d_x, int32_t f0, int32_t f1, int32_t f2, int32_t f3,
                                        const float *d_target, float *const *d_params,
                                        float *const *d_adam_m, float *const *d_adam_v, float bn_eps,
                                        float lr, float beta1, float beta2, float adam_eps, int32_t step,
                                        float *d_loss, void *d_workspace, size_t workspace_bytes,
                                        void *stream);

/*
 * Dense projection Z = X W on the matrix cores (fp32 MFMA, fp32 accumulate), the
 * contraction inside GCNConv and the GAT layer (the layers of section 3, "Graph Convolutional Layers" and
 * "Training Example", apply a learned weight matrix to the node features).  d_x [rows x k], d_w [k x n] row-major,
 * d_z [rows x n].  d_row_scale [rows] or NULL: Z[r,:] is multiplied by d_row_scale[r].
 */
gnn_status gnn_dense_xw(const float *d_x, int64_t rows, int32_t k, const float *d_w, int32_t n,
                        const float *d_row_scale, float *d_z, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* GNN_MI355X_H */
