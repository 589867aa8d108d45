// Internal declarations shared by the translation units of libomega_srpe.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "omega_srpe.h"

#define OMG_HIP(expr)                                   \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) {                         \
            omg_note_hip_error(e_, #expr, __LINE__);    \
            return (e_ == hipErrorOutOfMemory) ? OMG_ENOMEM : OMG_EHIP; \
        }                                               \
    } while (0)

#define OMG_TRY(expr)                 \
    do {                              \
        int rc_ = (expr);             \
        if (rc_ != OMG_OK) return rc_; \
    } while (0)

void omg_note_hip_error(hipError_t e, const char* what, int line);

// Edges of one wavefront's work item: long rows are cut into parts of at most this many edges
// (the actual part size of a graph is chosen per batch, a power of two between 32 and this).
constexpr int OMG_PART_EDGES = 256;
constexpr int OMG_WAVE = 64;
// tables larger than this (most of the 256 MB memory-side cache) get their inner-layer work items walked
// region by region when a batch reads their rows more than twice over
constexpr int64_t OMG_ORDER_MIN_TABLE_BYTES = (int64_t)192 << 20;
// Whether walking an inner layer's work items by table region pays (the table is already known to be larger
// than OMG_ORDER_MIN_TABLE_BYTES): the launch reads the table more than twice over (rows then meet in L2), or
// the table is far beyond what the address translation caches cover and the launch reads a few hundred MB at
// random (a 61 GB table, 2 GB gathered: 7 % off the gather).
inline bool omg_order_pays(int64_t gathered_bytes, int64_t table_bytes) {
    return gathered_bytes > 2 * table_bytes || (table_bytes > ((int64_t)8 << 30) && gathered_bytes > ((int64_t)256 << 20));
}
constexpr int OMG_MANY_PARTS = 16;   // rows with more parts than this are combined by a wider scheme

// Part size of one row: one place, used by the builder and by every kernel that walks parts.
// Uniform parts measured best: larger parts for very long rows shorten the combine step but lengthen
// the gather's tail by more.
__host__ __device__ inline int omg_row_part(int64_t len, int part_edges) {
    (void)len;
    return part_edges;
}

// eight bf16 values of a 16-byte piece -> fp32 (a bf16 is the top half of an fp32)
__device__ inline void unpack_bf16x8(const uint4& r, float* o) {
    o[0] = __uint_as_float(r.x << 16); o[1] = __uint_as_float(r.x & 0xffff0000u);
    o[2] = __uint_as_float(r.y << 16); o[3] = __uint_as_float(r.y & 0xffff0000u);
    o[4] = __uint_as_float(r.z << 16); o[5] = __uint_as_float(r.z & 0xffff0000u);
    o[6] = __uint_as_float(r.w << 16); o[7] = __uint_as_float(r.w & 0xffff0000u);
}

// Growable device allocation (never shrinks).
struct DevBuf {
    void* p = nullptr;
    size_t cap = 0;
    int ensure(size_t bytes);
    void release();
    template <typename T> T* as() const { return static_cast<T*>(p); }
};

// Counters a graph build reads back in one copy.
struct BuildCounts {
    int64_t n_cand;
    int64_t n_target;
    int64_t nnz_in;
    int64_t n_parts;        // work items over all rows_in rows
    int64_t n_parts_last;   // work items of the first n_query rows
    int64_t n_split;        // rows cut into 2..OMG_MANY_PARTS parts
    int64_t n_split_last;
    int64_t n_split_big;    // rows cut into more than OMG_MANY_PARTS parts
    int64_t n_split_big_last;
    int64_t n_small;        // rows whose unsorted segment has 1..64 keys
    int64_t n_med;          // ... 65..4096 keys
    int64_t n_big;          // ... more
    int32_t err;            // bit 0: index out of range, bit 1: bad recompute set
    int32_t pad;
};

// Layer-0 buffer (Sec. 6.1): row r < n_query is query r's feature row, row n_query + t the stored feature row of
// target t widened to fp32; columns dim .. ld0 are zero.  Thread `t` of a group of `nt` threads fills the columns
// t, t + nt, ... of the rows group, group + n_groups, ...
struct InitBufferArgs {
    const void* table;             // feature table
    int dtype;
    int64_t table_ld;
    int dim;
    const float* qf;
    int64_t ld_q;
    const int32_t* targets;
    int32_t n_query;
    int64_t n_rows;                // rows to fill (an upper bound when `counts` is given)
    const BuildCounts* counts;     // not null: the number of targets is read on the device
    float* buf0;
    int64_t ld0;
};

__device__ inline void omg_init_buffer_rows(const InitBufferArgs& a, int64_t group, int64_t n_groups, int t, int nt) {
    int64_t n_rows = a.n_rows;
    if (a.counts != nullptr) {
        const int64_t have = (int64_t)a.n_query + a.counts->n_target;
        n_rows = have < n_rows ? have : n_rows;
    }
    for (int64_t row = group; row < n_rows; row += n_groups)
        for (int c = t; c < a.ld0; c += nt) {
            float x = 0.f;
            if (c < a.dim) {
                if (row < a.n_query) {
                    x = a.qf[row * a.ld_q + c];
                } else {
                    const int64_t u = a.targets[row - a.n_query];
                    if (a.dtype == OMG_F32) x = static_cast<const float*>(a.table)[u * a.table_ld + c];
                    else x = __uint_as_float((uint32_t) static_cast<const uint16_t*>(a.table)[u * a.table_ld + c] << 16);
                }
            }
            a.buf0[row * a.ld0 + c] = x;
        }
}

// What the builder's kernels leave for the host in pinned, coherent host memory: the sizes, then the number of
// the build they belong to.  The host spins on the number instead of sleeping on an event: it sees the store a
// microsecond or two after it is made, where a wake-up takes ten to twenty.
struct HostMailbox {
    BuildCounts counts;
    unsigned long long seq;
};

struct omg_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    omg_base_csr base{};
    int64_t max_base_deg = 0;
    int policy = OMG_POLICY_RATIO;     // how the recompute set is chosen (omg_set_policy)
    uint64_t policy_seed = 0;
    const float* node_scores = nullptr;   // borrowed
    // Per-node state of the builder, one 16-byte record per node so that a kernel that needs two or three of the
    // fields for a node pays one memory transaction (on a 10^8-node graph every such access is a trip to HBM):
    // slot = the node's place in R during a build (-1 outside), cnt = request edges counted at it beyond the first
    // in this build (0 outside; the first one sets the node's bit in the bitmap), deg = its degree in the training
    // graph (never changes).
    struct NodeRec {
        int32_t slot;
        int32_t cnt;
        int32_t deg;
        int32_t pad;
    };
    NodeRec* node = nullptr;           // [n_nodes]
    bool slots_dirty = false;          // a build has written the nodes' slots and not yet returned them to -1
    BuildCounts* counts_host = nullptr;   // pinned: the counts of a HostMailbox
    HostMailbox* mailbox = nullptr;       // the same memory
    HostMailbox* mailbox_dev = nullptr;   // ... as the device addresses it
    unsigned long long build_seq = 0;     // number of the last build whose sizes were asked for
    bool gather_multi = true;          // short work items are aggregated several per wavefront (k_gather_multi)
    int64_t gather_multi_min_parts = 32768;
    int small_path = 1;                // requests that fit one compute unit's LDS are built by one block (k_build_small);
                                       // 2: as 1, but their second half takes the general route's launches (testing aid)
    int fused_sum_max = 4096;          // chunk / block totals a consumer's block adds up by itself; beyond, one block scans them first
    BuildCounts* counts_dev = nullptr;    // inside devState
    // per-node scratch that is idle (all zero) between builds
    DevBuf devState, bitmap, bitmap1, wordList, wordCnt;
    // build scratch (sized by the request)
    DevBuf smallRaw, chunkTot, flagTot, rowTot, qcnt, qcur, tcur, skey, flag, tLen, tOff, nParts, listSmall, listMed, listBig, sortTmp, subSeg,
        edges_in, rset_in;
    // layer scratch
    DevBuf agg, agg2, partial, foldv, dstlog, srclog, gemmSplit;
    // precomputation of the embedding tables
    DevBuf rowOff;
    // the caller's largest inner-layer table that is gathered by rows (bytes, bytes per row): decides whether a
    // build also orders the work items by table region
    int64_t hint_table_bytes = 0, hint_row_bytes = 0;
    int hint_min_part_edges = 0;       // lower bound for the next build's work-item size (0: none)
    // Work the caller wants queued right behind the builder's read-back of the sizes: the host then waits for the
    // read-back alone (an event) while the GPU goes on, instead of idling until the host has woken up and
    // launched again.  omg_serve_batch fills the layer-0 buffer this way; the row count is read on the device.
    struct {
        bool armed = false, done = false;
        const omg_table* features = nullptr;
        const float* query_feats = nullptr;
        int64_t ld_q = 0;
        float* buf0 = nullptr;
        int64_t ld0 = 0, max_rows = 0;
    } early;
    DevBuf preIds, preNparts, preCounts, preCdeg, preSelf, preInit, preStage;
    // partitioned execution (Sec. 6): per-row scratch of a partition's graph
    DevBuf cgpLen, cgpOff, cgpNp, cgpCounts;
    // serve_batch state
    omg_graph* serve_graph = nullptr;
    DevBuf buf[2], bufInit;
    // profiling
    int profiling = 0;
    hipEvent_t ev[2 + 4 * OMG_MAX_LAYERS] = {};
    int ev_ready = 0;
    int n_layers_timed = 0;
    int layer_cursor = 0;
    int build_timed = 0;
    // which event marks the start of layer l's first phase: its own, or (omg_serve_batch, where nothing is launched
    // in between) the event that ended the phase before it - every event costs the stream a few microseconds
    int start_idx[OMG_MAX_LAYERS] = {};
    bool main_timed[OMG_MAX_LAYERS] = {};    // the layer's main kernel has an event of its own (omg_set_profiling)
    bool chain_events = false;
};

struct omg_graph {
    omg_ctx* ctx = nullptr;
    int32_t n_query = 0;
    int64_t n_qedges = 0;
    BuildCounts c{};
    int64_t rows_in = 0;
    int part_edges = OMG_PART_EDGES;
    DevBuf cand, qdeg, cand_row, targets, target_slot, indptr, cols, cdeg;
    DevBuf part_ptr, part_row, split_rows, split_rows_q, split_big, split_big_q;   // split lists: rows cut into parts (all / query rows)
    DevBuf order;             // inner layers: work items in the order they are walked (see omg_graph_order)
    bool order_ready = false;
    bool built = false;
};

// graph_build.hip
int omg_build_impl(omg_ctx* ctx, omg_graph* g, int32_t n_query, int64_t n_qedges,
                   const int32_t* qe_query_dev, const omg_node_t* qe_node_dev, uint32_t gamma_ppm,
                   const omg_node_t* rset_dev, int64_t n_rset);
int omg_init_state(omg_ctx* ctx);
// Work items of the inner layers ordered by the part of the table they read (built on first use, on the
// context's stream).  OMG_EUNSUPPORTED when there are too many work items for the packed counters.
int omg_graph_order(omg_ctx* ctx, omg_graph* g);

// precompute.hip
int omg_precompute_layer(omg_ctx* ctx, const omg_table* first, const omg_table* prev, const omg_layer* layer,
                         const omg_table* out);
int omg_validate_base(omg_ctx* ctx);

// gather.hip
struct GatherArgs {
    const int64_t* indptr;
    const int32_t* cols;
    const int32_t* cdeg;
    const int32_t* part_ptr;
    const int32_t* part_row;
    const int32_t* order;     // optional: wavefront i takes work item order[i] instead of i
    const int32_t* split_rows;
    const int32_t* split_big;
    int64_t n_parts, n_split, n_split_big, n_rows;
    int64_t nnz;              // edges of the launch (decides between a work item and several per wavefront)
    int multi_ok;             // several short work items per wavefront allowed (a switch for comparisons)
    int64_t multi_min_parts;  // ... from this many work items on
    int part_edges;
    const void* table;
    int table_dtype;
    int64_t table_ld;
    const float* buf;
    int64_t buf_ld;
    int dim;
    int op;                   // OMG_OP_*: what is reduced and how a row is finished
    float agg_p;              // OMG_OP_POW: the exponent; OMG_OP_MOM: the (even) order
    float agg_eps;            // OMG_OP_POW: messages are max(h, 0) + agg_eps
    const float* mean;        // OMG_OP_MOM: the rows' means [n_rows x agg_ld] (a first pass with OMG_OP_MEAN)
    const float* h0;          // OMG_OP_GCN, optional (GCNII): rows' layer-0 values; the finished row is
    int64_t h0_ld;            //   (1 - alpha) * aggregate + alpha * h0
    float alpha;
    int64_t mean_ld;          //   row stride of `mean` (0: agg_ld)
    float* agg;
    int64_t agg_ld;
    int64_t agg_stride;       // row stride of agg (0: agg_ld)
    int raw;                  // local aggregation of a partition (Sec. 6): rows are stored unfinished (plain sum, sum of
                              //   powers, maximum with -inf for "no edge"; GCN: sources weighted by 1 / sqrt(d_u + 1) only)
                              //   and followed, at column agg_ld, by the row's edge count as an int
    float* partial;           // [n_parts x agg_ld]
};
enum { OMG_OP_MEAN = 0, OMG_OP_GCN = 1, OMG_OP_SUM = 2, OMG_OP_MAX = 3, OMG_OP_POW = 4, OMG_OP_MOM = 5 };
int omg_launch_gather(const GatherArgs& a, hipStream_t s, hipEvent_t after_main);
int omg_launch_init_buffer(const omg_table* feat, const float* qf, int64_t ld_q, const omg_node_t* targets,
                           int32_t n_query, int64_t n_target, float* buf0, int64_t ld0, hipStream_t s);
// the same with the number of targets read on the device (counts->n_target), at most max_rows rows in all
int omg_launch_init_buffer_dev(const omg_table* feat, const float* qf, int64_t ld_q, const omg_node_t* targets,
                               int32_t n_query, const BuildCounts* counts, int64_t max_rows, float* buf0, int64_t ld0,
                               hipStream_t s);

// gat.hip
// Softmax statistics that follow the heads x agg_ld sums of a partial row (a row cut into parts) and of a
// partition's record: local maximum score of head h at [h], sum of exp(score - maximum) at [OMG_GAT_STAT_SUM + h],
// number of edges (int32 bit pattern, records only) at [OMG_GAT_STAT_COUNT].
constexpr int OMG_GAT_MAX_HEADS = 8;
constexpr int OMG_GAT_STAT_SUM = OMG_GAT_MAX_HEADS;
constexpr int OMG_GAT_STAT_COUNT = 2 * OMG_GAT_MAX_HEADS;
constexpr int OMG_GAT_STAT_PAD = 2 * OMG_GAT_MAX_HEADS + 4;      // keeps rows 16-byte aligned

struct GatArgs {
    const int64_t* indptr;
    const int32_t* cols;
    const int32_t* part_ptr;
    const int32_t* part_row;
    const int32_t* split_rows;
    const int32_t* split_big;
    int64_t n_parts, n_split, n_split_big, n_rows;
    int part_edges;
    const void* table;
    int table_dtype;
    int64_t table_ld;
    const float* buf;
    int64_t buf_ld;
    int dim, heads;
    float leaky;
    const float* fold_src;    // [heads x dim]  W_h a_src,h
    const float* fold_dst;    // [heads x dim]
    const float* src_logits;  // optional [n_table_rows x heads]
    float* buf_logits;        // scratch [rows_in x heads]: source logits of the buffer rows
    float* dst_logits;        // scratch [n_rows x heads]
    int64_t n_buf_rows;
    float* agg;               // [n_rows x heads x agg_ld]
    int64_t agg_ld;
    int64_t agg_stride;       // row stride of agg (0: heads x agg_ld)
    int raw;                  // local aggregation of a partition (Sec. 6.2): a row holds, per head, the sum of the sources
                              //   weighted by exp(score - local maximum), not normalised; then at column heads x agg_ld
                              //   the softmax statistics laid out as the OMG_GAT_STAT_* constants say
    float* partial;           // [n_parts x (heads x agg_ld + OMG_GAT_STAT_PAD)]
};
int omg_launch_gat(const GatArgs& a, hipStream_t s, hipEvent_t after_main);
int omg_launch_gat_fold(const omg_layer* L, float* fold_src, float* fold_dst, hipStream_t s);
int omg_launch_table_logits(const omg_table* t, const float* fold_src, int heads, float* logits, hipStream_t s);

// cgp.hip: one partition's share of a computation graph, and the merge of the partitions' local aggregations (Sec. 6)
constexpr int OMG_CGP_MAX_PARTS = 64;
int omg_cgp_partition_impl(omg_ctx* ctx, const omg_graph* whole, const int32_t* node_part, int n_part, int p, omg_graph* out);
struct CgpMergeArgs {
    const float* wire;        // [n_part][n_rows] records of ld_wire floats (see GatherArgs::raw / GatArgs::raw)
    int64_t ld_wire;
    int64_t n_rows;
    int n_part;
    int op;                   // OMG_OP_*; for OMG_OP_GCN the destination's factor and the self term are applied here
    int heads;                // > 0: softmax merge of a GAT layer (op ignored)
    float agg_p;
    int dim;
    int64_t agg_ld;
    float* out;               // [n_rows x out_ld] (GAT: [n_rows x heads x agg_ld], out_ld ignored)
    int64_t out_ld;
    const float* self;        // OMG_OP_GCN: the rows' own inputs
    int64_t self_ld;
    const float* h0;          // GCNII, optional
    int64_t h0_ld;
    float alpha;
};
int omg_launch_cgp_merge(const CgpMergeArgs& a, hipStream_t s);

// update_gemm.hip
constexpr int OMG_MAX_SEG = 8;
struct GemmSeg {
    const float* A;   // rows x k, row stride lda
    int64_t lda;
    const float* W;   // k x n, row stride ldw
    int64_t ldw;
    int k;
};
struct GemmArgs {
    GemmSeg seg[OMG_MAX_SEG];
    int n_seg;
    int64_t m;
    int n;                    // output columns produced by one z-slice
    int n_z;                  // grid z: independent column blocks (GAT heads)
    int64_t a_z_stride;       // added to every A pointer per z
    int64_t w_z_stride;       // added to every W pointer per z (column offset)
    int out_z_stride;         // column offset of the output per z
    const float* bias;        // indexed by output column (incl. z offset); see bias_sum
    int bias_sum;             // >1: bias of column c = mean of bias[c + j * n], j < bias_sum
    float scale;              // applied to the accumulated product before the bias
    int act;
    float* out;
    int64_t ldo;
    float* split_buf;         // optional scratch for launches of few blocks (raw sums of the blocks that share a tile)
    int64_t split_floats;     // its size in floats
    int k_split;              // set by the launcher
};
constexpr size_t OMG_GEMM_SPLIT_BYTES = sizeof(float) * 4 * 128 * 64 * 64;   // four shares of 128 output tiles
int omg_launch_update(const GemmArgs& a, hipStream_t s);
