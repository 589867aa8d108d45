/*
 * omega_srpe.h - C ABI of the single-GPU SRPE serving path (Omega, arXiv 2501.08547).
 *
 * What the library does: for one batch of query nodes it builds the batch's computation
 * graph under selective recomputation of precomputed embeddings (Sec. 5, Sec. 6.1) and
 * executes the GNN layers over it (Sec. 2, Eq. 1), reading most neighbour embeddings from
 * per-layer tables that stay resident in device memory and the recomputed few from a
 * buffer of freshly computed rows.  One GPU.  Of the paper's computation graph parallelism
 * (Sec. 6) the part one GPU can show is here as well: one partition's share of a computation
 * graph, its local aggregations and the merge functions (omg_cgp_*); request splitting across
 * machines and the all-to-all exchange of the records are not.
 *
 * Conventions
 *   - Every function returns OMG_OK (0) or a negative error code; nothing throws.
 *   - "DEVICE" pointers are HIP device memory owned by the caller.  The library borrows
 *     them for the duration of a call and never frees them.  "HOST" pointers are ordinary
 *     host memory.  Where a `where` argument is given it says which of the two the edge
 *     arrays are (OMG_HOST / OMG_DEVICE).
 *   - Work is enqueued on the HIP stream given to omg_create.  Functions that return sizes
 *     or copy to host memory synchronise that stream; omg_run_layer / omg_init_buffer /
 *     omg_gat_src_logits only enqueue.  Outputs are valid once the stream is synchronised.
 *   - Node ids are int32 (omg_node_t); offsets into edge arrays are int64.
 *   - Dense matrices are row-major fp32; `ld` arguments count elements, not bytes.
 *   - A context and the graphs built from it must be used from one host thread at a time.
 *
 * Canonical computation graph (omg_graph_export).  Rows: the B queries in index order, then
 * the recompute targets in ascending node id.  Columns of a query row: its neighbours in
 * ascending node id.  Columns of a target row: its base in-neighbours in base-CSR order,
 * then the queries attached to it in ascending query index.  A column c >= 0 reads row c of
 * the layer's table; c < 0 reads row ~c of the buffer of freshly computed rows.  The last
 * layer uses the first B rows only (Sec. 6.1: edges whose destination is a query node).
 */
#ifndef OMEGA_SRPE_H
#define OMEGA_SRPE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t omg_node_t;
typedef struct omg_ctx omg_ctx;
typedef struct omg_graph omg_graph;

enum {
    OMG_OK = 0,
    OMG_EINVAL = -1,       /* null pointer, bad enum, misaligned ld, dimension mismatch, gamma > 10^6 */
    OMG_ERANGE = -2,       /* node id >= n_nodes, query index >= n_query, recompute set not within the candidates */
    OMG_ENOMEM = -3,       /* device or host allocation failed */
    OMG_ESTATE = -4,       /* graph belongs to another context, or is empty */
    OMG_EHIP = -5,         /* a HIP runtime call failed */
    OMG_EUNSUPPORTED = -6, /* a shape outside what the kernels are built for: rows of more than 256 sixteen-byte
                              pieces (1,024 fp32 or 2,048 bf16 values), GAT with other than 1, 2, 4 or 8 heads
                              (8 heads: rows of more than 1,024 values), moments of odd order */
    OMG_ESCRATCH = -7      /* omg_run_layer_static: the layer needs more scratch than OMG_STATIC_SCRATCH_MIB holds */
};

enum { OMG_HOST = 0, OMG_DEVICE = 1 };
enum { OMG_F32 = 0, OMG_BF16 = 1 };                         /* storage type of a table */
enum { OMG_SAGE_MEAN = 0, OMG_GCN_SYM = 1, OMG_GAT = 2, OMG_GCNII = 3 };   /* layer type */
/* Aggregation function of a SAGE-type layer (Sec. 6.2 names the forms beyond the mean).  N = number of
 * edges of the row; an empty row aggregates to zeros in every case.
 *   MEAN    (1/N) sum_u h_u
 *   SUM     sum_u h_u
 *   MAX     element-wise maximum
 *   POWER   ((1/N) sum_u m_u^p)^(1/p) with positive messages m_u = max(h_u, 0) + agg_eps; p = agg_p > 0
 *   MOMENT  ((1/N) sum_u (h_u - mean)^n)^(1/n), n = agg_p an even integer 2..8 (two passes over the row).
 *           Odd orders are refused: an odd central moment is zero on every symmetric neighbourhood (any two
 *           neighbours), where the root's derivative is unbounded and rounding decides the result. */
enum { OMG_AGG_MEAN = 0, OMG_AGG_SUM = 1, OMG_AGG_MAX = 2, OMG_AGG_POWER = 3, OMG_AGG_MOMENT = 4 };
enum { OMG_ACT_NONE = 0, OMG_ACT_RELU = 1, OMG_ACT_ELU = 2 };

/* Training graph: CSR of in-neighbours.  DEVICE pointers, borrowed for the context's life. */
typedef struct {
    int64_t n_nodes;
    const int64_t* indptr;        /* [n_nodes + 1], non-decreasing, indptr[0] == 0 */
    const omg_node_t* indices;    /* [indptr[n_nodes]] */
} omg_base_csr;

/* One stored table: node features (layer 0) or the precomputed embeddings p^(l) of one
 * layer (Sec. 5).  DEVICE, row-major, n_rows x ld elements of which the first `dim` are
 * used.  ld * element size must be a multiple of 16 bytes and data 16-byte aligned. */
typedef struct {
    const void* data;
    int32_t dtype;                /* OMG_F32 | OMG_BF16 */
    int32_t dim;
    int64_t n_rows;
    int64_t ld;
} omg_table;

/* One GNN layer (update function of Eq. 1).  All pointers DEVICE fp32, borrowed.
 *   SAGE-mean: out = act(h_v W_self + mean_{u in N'(v)} h_u W_nb + bias); empty mean = 0.  `aggregator`
 *              replaces the mean by another OMG_AGG_* function (0 = mean; must be 0 for the other models)
 *   GCN-sym  : out = act((h_v / d_v + sum_u h_u / sqrt(d_u d_v)) W_nb + bias), d = in-degree in
 *              the graph that includes the batch's query edges, plus one
 *   GCNII    : the deep convolution of the paper's appendix on the number of layers (initial residual and
 *              identity mapping): out = act(((1 - alpha) g_v + alpha h0_v) W_nb + bias), g_v = GCN-sym's
 *              normalised sum above, h0_v = the row's layer-0 value, W_nb = (1 - beta) I + beta W handed
 *              over as one d x d matrix (d_in == d_out), 0 <= alpha <= 1
 *   GAT      : z = h W_nb split into `heads` blocks of d_out / heads columns;
 *              e_uv = LeakyReLU(a_src[h] . z_u[h] + a_dst[h] . z_v[h]); alpha = softmax_u e_uv;
 *              out = act(concat_h sum_u alpha z_u[h] + bias), or with head_mean != 0 the mean
 *              over heads of (sum_u alpha z_u[h] + bias[h]) with no concatenation.
 *   W_self, W_nb: d_in x d_out.  a_src, a_dst: heads x (d_out / heads).  bias: d_out. */
typedef struct {
    int32_t model;                /* OMG_SAGE_MEAN | OMG_GCN_SYM | OMG_GAT | OMG_GCNII */
    int32_t d_in, d_out, heads;
    int32_t act;                  /* OMG_ACT_* */
    int32_t head_mean;
    float leaky_slope;
    int32_t aggregator;           /* OMG_AGG_*, SAGE-type layers only */
    const float* W_self;
    const float* W_nb;
    const float* a_src;
    const float* a_dst;
    const float* bias;
    const float* src_logits;      /* GAT only, optional: output of omg_gat_src_logits for this layer's table */
    float agg_p;                  /* OMG_AGG_POWER: exponent p; OMG_AGG_MOMENT: order n */
    float agg_eps;                /* OMG_AGG_POWER: added to the clamped messages */
    float alpha;                  /* OMG_GCNII: weight of the initial residual */
    const float* init_rows;       /* OMG_GCNII, omg_run_layer only: DEVICE rows_in x init_ld fp32, the layer-0 values of
                                     the freshly computed rows (the buffer omg_init_buffer filled); omg_serve_batch and
                                     omg_precompute_embeddings use their own and ignore this field */
    int64_t init_ld;
    const float* fold;            /* GAT only, optional: output of omg_gat_fold for this layer's weights; without it the
                                     two folded score vectors are recomputed by every call that runs the layer */
} omg_layer;

#define OMG_MAX_LAYERS 8
/* Durations measured with HIP events on the context's stream, in milliseconds. */
typedef struct {
    float build_ms;
    float gather_ms[OMG_MAX_LAYERS];   /* layer l (index l - 1): the gather-reduce kernel over all work items */
    float combine_ms[OMG_MAX_LAYERS];  /* layer l: adding up the parts of rows that were cut */
    float update_ms[OMG_MAX_LAYERS];   /* layer l: dense update */
    float total_ms;
} omg_timing;

/* Creates a context bound to the current HIP device and to `hip_stream` (a hipStream_t, or NULL
 * for the default stream).  Checks the CSR header on the host (n_nodes > 0 and < 2^31).  The context
 * allocates about 16.2 bytes of device memory per node of the graph for the lifetime of the context (the
 * builder's per-node records and bitmaps), beyond the buffers that grow with the batches it serves.
 * Errors: OMG_EINVAL, OMG_ENOMEM, OMG_EHIP. */
int omg_create(omg_ctx** ctx, const omg_base_csr* graph, void* hip_stream);
void omg_destroy(omg_ctx* ctx);
const char* omg_strerror(int code);

/* With profiling on, omg_build_computation_graph / omg_run_layer / omg_serve_batch record HIP
 * events around their phases; omg_get_timing synchronises and reports the last call's phases.
 * on = 1: every phase.  on = 2: as 1, but from the second layer of a call on, the gather-reduce kernel and
 * the adding up of cut rows are timed together (gather_ms holds both, combine_ms is 0): one event less per
 * layer on the stream (an event costs it 3-4 us).  on = 0: no events. */
int omg_set_profiling(omg_ctx* ctx, int on);
int omg_get_timing(omg_ctx* ctx, omg_timing* out);

/* Which candidates are recomputed when no explicit set is given (Sec. 5.2.2).  The budget, the tie rule
 * (smaller node id) and everything downstream are the same for all three.
 *   OMG_POLICY_RATIO   (default) largest query-edge ratio, the paper's policy
 *   OMG_POLICY_RANDOM  largest random key; key(u) = top 39 bits of the splitmix64 finaliser
 *                      (z ^= z >> 30, *= 0xBF58476D1CE4E5B9, z ^= z >> 27, *= 0x94D049BB133111EB, z ^= z >> 31)
 *                      of z = u + seed * 0x9E3779B97F4A7C15 mod 2^64
 *   OMG_POLICY_SCORE   largest node_scores[u]: DEVICE fp32 [n_nodes], finite, borrowed until the policy is set
 *                      again or the context is destroyed (e.g. node importance scores, or measured
 *                      approximation errors); -0 counts as +0
 * Takes effect from the next graph construction.  Errors: OMG_EINVAL. */
enum { OMG_POLICY_RATIO = 0, OMG_POLICY_RANDOM = 1, OMG_POLICY_SCORE = 2 };
int omg_set_policy(omg_ctx* ctx, int policy, uint64_t seed, const float* node_scores);

/* Computation-graph construction for one batch (Sec. 5.2.1 candidates; Sec. 5.2.2 policy;
 * Sec. 6.1 layers).  The request is n_qedges pairs (qe_query[i] in [0, n_query), qe_node[i] in
 * [0, n_nodes)), in any order; duplicates count with multiplicity.
 *   recompute_set == NULL: the top-query-edges-ratio policy picks floor(gamma_ppm * |R| / 10^6)
 *     of the candidates R, ranked by (query edges at u) / (in-degree of u + query edges at u),
 *     compared exactly; equal ratios go to the smaller node id.  gamma_ppm <= 10^6.
 *   recompute_set != NULL: that set is used as given (ascending, unique, within R; same memory
 *     space as the edge arrays) and gamma_ppm is ignored.
 * *graph == NULL allocates a new graph object; otherwise the given one is rebuilt in place and
 * keeps its device buffers when they are large enough.  Synchronises the stream once.
 * Errors: OMG_EINVAL, OMG_ERANGE (nothing is built), OMG_ENOMEM, OMG_EHIP. */
int omg_build_computation_graph(omg_ctx* ctx, int32_t n_query, int64_t n_qedges,
                                const int32_t* qe_query, const omg_node_t* qe_node, int where,
                                uint32_t gamma_ppm,
                                const omg_node_t* recompute_set, int64_t n_recompute,
                                omg_graph** graph);

/* sizes[0..3] = |R| candidates, |T| targets, rows_in = n_query + |T|, nnz_in. */
int omg_graph_sizes(const omg_graph* graph, int64_t sizes[4]);

/* Copies the canonical graph to HOST arrays (any may be NULL): cand[|R|], qdeg[|R|],
 * targets[|T|], indptr[rows_in + 1], cols[nnz_in] (tagged), cdeg[nnz_in] = in-degree of each
 * column's source in the graph that includes the batch.  Synchronises. */
int omg_graph_export(const omg_graph* graph, omg_node_t* cand, int32_t* qdeg, omg_node_t* targets,
                     int64_t* indptr, int32_t* cols, int32_t* cdeg);
void omg_graph_destroy(omg_graph* graph);

/* Layer-0 values of the freshly computed rows (Sec. 2: h^(0) is the feature vector):
 * buf0[0..B) = query_feats, buf0[B + t] = feature-table row of target t, converted to fp32.
 * query_feats: DEVICE B x ld_q.  buf0: DEVICE rows_in x ld0, ld0 >= features->dim. */
int omg_init_buffer(omg_ctx* ctx, const omg_graph* graph, const omg_table* features,
                    const float* query_feats, int64_t ld_q, float* buf0, int64_t ld0);

/* One GNN layer over the batch's computation graph (Sec. 6.1, layer-wise execution with a
 * single partition; Eq. 1).  table_prev holds h^(l-1) of every training node (features for
 * l = 1, else p^(l-1)); buf_prev (DEVICE, rows_in x ld_prev) holds h^(l-1) of the freshly
 * computed rows.  Writes buf_out (DEVICE): rows_in rows, or only the n_query query rows when
 * is_last != 0, each of width d_out (d_out / heads with head_mean).  Enqueues only. */
int omg_run_layer(omg_ctx* ctx, const omg_graph* graph, int is_last,
                  const omg_table* table_prev, const float* buf_prev, int64_t ld_prev,
                  const omg_layer* layer, float* buf_out, int64_t ld_out);

/* omg_run_layer for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical results; what
 * omg_run_layer keeps in growable buffers of the context (aggregated rows, partial sums of rows cut into parts,
 * GAT's folded score vectors and the fresh rows' score halves, the raw sums of a split update) lives here in a
 * device array of OMG_STATIC_SCRATCH_MIB MiB that is part of the library's image (every GPU the library runs on
 * holds its copy until the process ends).  The call makes no hipMalloc / hipFree and no other allocating call.
 *   - A layer that needs more returns OMG_ESCRATCH and launches nothing; omg_static_scratch_bytes() is the limit.
 *     Need, in floats, each piece rounded up to 256 bytes: rows x w (rows = rows_in, or n_query with is_last;
 *     w = d_in rounded up to 8, times heads for GAT; twice for the normalised moments) + work items x w (+ 20 per
 *     work item for GAT) if any row is cut into parts + 2 x heads x d_in + 2 x (rows_in x heads + 4) for GAT
 *     + 2 Mi floats for the update of up to 8,192 rows.
 *   - A GAT layer must bring src_logits (OMG_EINVAL otherwise: the side table would be an allocation).
 *   - Work items are walked in table-region order only if an earlier omg_run_layer on this graph built that
 *     order; the results do not depend on it.
 *   - All calls on one GPU share the array, whatever their context or stream: calls that overlap on one GPU
 *     race.  Nothing in it has to start at zero (every value is written before it is read).
 * Errors: as omg_run_layer, plus OMG_ESCRATCH. */
#define OMG_STATIC_SCRATCH_MIB 32
int omg_run_layer_static(omg_ctx* ctx, const omg_graph* graph, int is_last,
                         const omg_table* table_prev, const float* buf_prev, int64_t ld_prev,
                         const omg_layer* layer, float* buf_out, int64_t ld_out);
int64_t omg_static_scratch_bytes(void);

/* GAT helper, run once per (table, layer) when the model is loaded: logits[u * heads + h] =
 * a_src[h] . (row u of table x W_nb[:, head h]), the source half of the attention score of
 * every stored row.  Passing the result as omg_layer.src_logits lets omg_run_layer skip the
 * per-edge projection of stored rows.  logits: DEVICE n_rows x heads fp32. */
int omg_gat_src_logits(omg_ctx* ctx, const omg_table* table, const omg_layer* layer, float* logits);

/* GAT helper, run once per layer when the model is loaded (and again whenever W_nb, a_src or a_dst change): the
 * folded score vectors fold[h * d_in + k] = sum_j W_nb[k][h * dh + j] * a_src[h][j] and, at offset heads * d_in, the
 * same with a_dst, so that a score half is a dot product of an input row with a vector (a . (h W) = (W a) . h).
 * Passing the result as omg_layer.fold saves every later call that runs the layer this step.
 * fold: DEVICE 2 x heads x d_in fp32, 16-byte aligned.  Enqueues only. */
int omg_gat_fold(omg_ctx* ctx, const omg_layer* layer, float* fold);

/* Whole path for one batch: graph construction, layer-0 buffer, k layers (Sec. 4 workflow
 * restricted to one GPU).  tables[0] = features, tables[l] = p^(l) for l = 1..k-1.
 * query_feats: DEVICE n_query x ld_q.  out: DEVICE n_query x ld_o.  Edge arrays as in
 * omg_build_computation_graph.  Intermediate buffers live in the context and are reused
 * between calls; the two buffers of freshly computed rows are sized for the most rows the budget
 * allows, n_query + floor(gamma_ppm * min(n_qedges, n_nodes) / 10^6), times the widest layer input.
 * Synchronises once (inside graph construction: the host waits for the sizes while the layer-0
 * values are already being written); the layers are enqueued. */
int omg_serve_batch(omg_ctx* ctx, int32_t k, const omg_table* tables, const omg_layer* layers,
                    const float* query_feats, int64_t ld_q,
                    int32_t n_query, int64_t n_qedges,
                    const int32_t* qe_query, const omg_node_t* qe_node, int where,
                    uint32_t gamma_ppm, float* out, int64_t ld_o);

/* Precomputed embeddings (Sec. 5): applies layers 1..k-1 of the model to EVERY node of the training
 * graph, on the training graph alone, and stores layer l's output as out_tables[l - 1], the table that
 * serving reads as p^(l).  Layer l reads `features` (l = 1) or out_tables[l - 2].  out_tables[l - 1]:
 * DEVICE n_nodes x ld, caller-allocated and WRITTEN here (the data pointer is const only because
 * omg_table is shared with the reading calls); dtype OMG_F32, or OMG_BF16 (rounded to nearest even from
 * the fp32 result; padding columns are set to zero).  Same kernels and the same layer definitions as
 * serving.  layers[l].src_logits must be NULL.  Not a serving-time call: it synchronises several times.
 * Errors: OMG_EINVAL, OMG_EUNSUPPORTED, OMG_ENOMEM, OMG_EHIP. */
int omg_precompute_embeddings(omg_ctx* ctx, int32_t k, const omg_table* features, const omg_layer* layers,
                              const omg_table* out_tables);

/* Sizes of the graph built by the last omg_serve_batch on this context (as omg_graph_sizes). */
int omg_last_graph_sizes(const omg_ctx* ctx, int64_t sizes[4]);

/* ---- Computation graph parallelism (Sec. 6), as far as one GPU shows it ---------------------------------
 * When the tables are spread over P partitions (GPUs), every partition executes the share of the batch's
 * computation graph whose SOURCES it holds, and the local aggregations of a destination are merged (Eq. 3).
 * The three steps below are one partition's work for one layer; between omg_cgp_local_aggregate and
 * omg_cgp_merge_* lies, on several GPUs, one all-to-all of the records, which this library does not do: the
 * caller places the records of partition p at wire + p * n_rows * ld_wire (what the exchange leaves at the
 * receiver).  On one GPU the P shares are run one after the other into one such buffer.
 *
 * Record of one destination from one partition (fp32, ld_wire >= omg_cgp_wire_width(layer) floats, ld_wire a
 * multiple of 4, 16-byte aligned), with w = d_in rounded up to a multiple of 8:
 *   SAGE-type, GCN, GCNII : [0, w) the local aggregation - mean, sum, moments' first step: sum of the sources;
 *                           max: their maximum (-inf where the partition holds none); power mean: sum of
 *                           (max(h, 0) + eps)^p; moments' second step: sum of (h - row mean)^n; GCN / GCNII: sum of
 *                           h_u / sqrt(d_u + 1) (the destination's factor and the self term belong to the merge) -
 *                           then at [w] the number of local sources as an int32 bit pattern
 *   GAT                   : per head h, [h w, (h + 1) w) the sum of the sources weighted by exp(score - m_h), m_h the
 *                           largest local score; then at [H w + h] m_h (-inf: none), at [H w + 8 + h] the sum of
 *                           those exponentials, at [H w + 16] the number of local sources (int32 bit pattern):
 *                           the two-step softmax of Sec. 6.2.  The record is H w + 20 floats wide.
 * Columns between d_in (rounded up to 4) and w are not defined. */

/* Floats per record for this layer (see above); 0 if the layer is not valid. */
int64_t omg_cgp_wire_width(const omg_layer* layer);

/* Partition p's computation graph (Sec. 6.1): the rows of `graph` (all queries, all recompute targets), each
 * with only the edges whose source belongs to partition p, in the order they have in `graph`.  A stored row
 * u belongs to node_part[u]; a freshly computed row to the partition that computes it: query q to q mod
 * n_part, a recompute target to its node's partition.  node_part: DEVICE int32 [n_nodes], values in
 * [0, n_part) (else OMG_ERANGE); 1 <= n_part <= 64.  *part_graph: NULL (a new handle is made) or a handle
 * from an earlier call (re-filled); it works with omg_graph_sizes, omg_graph_export, omg_cgp_local_aggregate
 * and omg_graph_destroy.  Synchronises once.  Errors: OMG_EINVAL, OMG_ESTATE, OMG_ERANGE, OMG_ENOMEM, OMG_EHIP. */
int omg_cgp_partition_graph(omg_ctx* ctx, const omg_graph* graph, const int32_t* node_part, int32_t n_part, int32_t p,
                            omg_graph** part_graph);

/* Local aggregation a_{v,p} of one layer (Eq. 3) over a partition's graph: one record per row (all rows, or the
 * query rows with is_last != 0) at wire + v * ld_wire.  table_prev / buf_prev as in omg_run_layer (buf_prev
 * holds the previous layer's value of EVERY fresh row: GAT's scores need the destinations', which Sec. 6.2
 * all-gathers).  row_mean: NULL, except for the second step of the normalised moments: DEVICE n_rows x ld_mean
 * fp32, the rows' overall means (omg_cgp_merge_mean); with NULL a moments layer does its first step.
 * Enqueues only. */
int omg_cgp_local_aggregate(omg_ctx* ctx, const omg_graph* part_graph, int is_last, const omg_table* table_prev,
                            const float* buf_prev, int64_t ld_prev, const omg_layer* layer, const float* row_mean,
                            int64_t ld_mean, float* wire, int64_t ld_wire);

/* Normalised moments, between the two steps (Sec. 6.2): the mean of all messages of every row from the n_part
 * first-step records, row_mean: DEVICE n_rows x ld_mean (ld_mean >= d_in rounded up to 8, a multiple of 4).
 * On several GPUs the result is what the all-gather distributes.  Enqueues only. */
int omg_cgp_merge_mean(omg_ctx* ctx, int64_t n_rows, int32_t n_part, const float* wire, int64_t ld_wire,
                       const omg_layer* layer, float* row_mean, int64_t ld_mean);

/* Merge function and update (Eq. 3): from the n_part records of each of n_rows rows to the layer's output,
 * buf_out: DEVICE n_rows x ld_out.  The merge adds sums (then divides by the total count / takes the root),
 * maximises maxima, rescales and adds softmax records, and for GCN / GCNII applies 1 / sqrt(d_v + 1) and adds
 * h_v / (d_v + 1), d_v = the total count.  buf_prev: the rows' own previous values (DEVICE n_rows x ld_prev);
 * GCNII reads layer->init_rows as omg_run_layer does.  Partitions are merged in ascending order: reruns are
 * bit-identical.  Enqueues only. */
int omg_cgp_merge_update(omg_ctx* ctx, int64_t n_rows, int32_t n_part, const float* wire, int64_t ld_wire,
                         const omg_layer* layer, const float* buf_prev, int64_t ld_prev, float* buf_out, int64_t ld_out);

/* Measurement aid, not a step of the method (for bench.py and whoever prices the gather of Sec. 6.2
 * against this GPU): reads `bytes` of DEVICE memory at `buffer` (16-byte aligned, at least 1 MiB and at
 * least blocks x 16 KiB) `reps` times with `blocks` workgroups of 256 lanes, four 16-byte loads in
 * flight per lane, on the context's stream, after one untimed pass.  *bytes_read = bytes the timed
 * launch loaded, *ms = its duration by HIP events.  A buffer of up to 256 MB is served by the
 * memory-side cache, a larger one by HBM.  Synchronises.  Errors: OMG_EINVAL, OMG_ENOMEM, OMG_EHIP. */
int omg_measure_read_rate(omg_ctx* ctx, const void* buffer, int64_t bytes, int32_t reps, int32_t blocks,
                          double* bytes_read, float* ms);

/* Testing aid, not a step of the method: the nth growing device allocation the library makes from now on
 * (counted from 0, over all contexts) fails with OMG_ENOMEM; a negative nth switches the injection off.
 * Lets a test walk every allocation of a call and check that the call leaves the context usable. */
void omg_debug_fail_allocation(int64_t nth);

/* Testing aid: the graph construction finishes its prefix sums inside the kernels that consume them as long as
 * there are at most `limit` chunk or block totals to add up (4,096 by default) and has one block scan the totals
 * first beyond that.  A small limit makes small requests take the second route.  limit >= 1. */
int omg_debug_set_fused_sum_limit(omg_ctx* ctx, int32_t limit);

/* Testing aid: a request of up to 2,048 edges and 2,048 queries (and no explicit recompute set) is normally built
 * by one block (the first half of the construction in one kernel; the second half in one more when the graph has
 * at most 2,048 work items and 16,384 edges); on == 0 sends such requests down the general route as well, on == 2
 * only their second half, so that a test can compare the routes on the same input. */
int omg_debug_set_small_path(omg_ctx* ctx, int32_t on);

/* Testing aid: launches of at least 32,768 work items that are short (on average at most half the part size, rows
 * of at most 32 sixteen-byte pieces) are normally aggregated several work items per wavefront; on == 0 sends them
 * through the one-work-item-per-wavefront kernel as well, on == 2 drops the lower bound on the number of work
 * items (small test batches then take the several-per-wavefront kernel), on == 1 is the default. */
int omg_debug_set_gather_multi(omg_ctx* ctx, int32_t on);

#ifdef __cplusplus
}
#endif
#endif /* OMEGA_SRPE_H */
