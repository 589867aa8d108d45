// C ABI of libomega_srpe: argument checks, context / graph lifetime, and the sequencing of
// the kernels of one layer and of one batch.  See include/omega_srpe.h for the contract.
#include "internal.h"

#include <stdio.h>
#include <string.h>
#include <atomic>
#include <mutex>
#include <new>

// Scratch memory that is part of the library's image, for omg_run_layer_static (callers that must not allocate).
// Every GPU the library runs on holds its own copy until the process ends.  In host code the name is only a
// stand-in for the symbol: the array's device address is asked from the runtime once per device
// (static_scratch_init) and that pointer is what the kernels get.
constexpr size_t OMG_STATIC_SCRATCH_BYTES = (size_t)OMG_STATIC_SCRATCH_MIB << 20;
static __device__ __align__(256) unsigned char scratch[OMG_STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_hip_msg[256] = "";

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_table(const omg_table* t) {
    if (t == nullptr || t->data == nullptr) return OMG_EINVAL;
    if (t->dtype != OMG_F32 && t->dtype != OMG_BF16) return OMG_EINVAL;
    const int64_t es = t->dtype == OMG_F32 ? 4 : 2;
    if (t->dim <= 0 || t->ld < t->dim || (t->ld * es) % 16 != 0 || !aligned16(t->data) || t->n_rows < 0)
        return OMG_EINVAL;
    return OMG_OK;
}

int check_layer(const omg_layer* L) {
    if (L == nullptr || L->W_nb == nullptr || L->d_in <= 0 || L->d_out <= 0) return OMG_EINVAL;
    if (L->act != OMG_ACT_NONE && L->act != OMG_ACT_RELU && L->act != OMG_ACT_ELU) return OMG_EINVAL;
    if (L->model != OMG_SAGE_MEAN && L->aggregator != OMG_AGG_MEAN) return OMG_EINVAL;
    switch (L->model) {
        case OMG_SAGE_MEAN:
            if (L->W_self == nullptr) return OMG_EINVAL;
            if (L->aggregator < OMG_AGG_MEAN || L->aggregator > OMG_AGG_MOMENT) return OMG_EINVAL;
            if (L->aggregator == OMG_AGG_POWER && !(L->agg_p > 0.f && L->agg_p <= 64.f && L->agg_eps >= 0.f)) return OMG_EINVAL;
            if (L->aggregator == OMG_AGG_MOMENT) {
                const int n = (int)L->agg_p;
                if ((float)n != L->agg_p || n < 2 || n > 8) return OMG_EINVAL;
                if (n % 2 != 0) return OMG_EUNSUPPORTED;         // odd orders: see omega_srpe.h
            }
            break;
        case OMG_GCN_SYM:
            break;
        case OMG_GCNII:
            if (L->d_in != L->d_out || !(L->alpha >= 0.f && L->alpha <= 1.f)) return OMG_EINVAL;
            break;
        case OMG_GAT:
            if (L->heads <= 0 || L->d_out % L->heads != 0 || L->a_src == nullptr || L->a_dst == nullptr)
                return OMG_EINVAL;
            if (L->heads != 1 && L->heads != 2 && L->heads != 4 && L->heads != 8) return OMG_EUNSUPPORTED;
            break;
        default:
            return OMG_EINVAL;
    }
    return OMG_OK;
}

int layer_out_width(const omg_layer* L) {
    return (L->model == OMG_GAT && L->head_mean) ? L->d_out / L->heads : L->d_out;
}

int ensure_events(omg_ctx* ctx) {
    if (ctx->ev_ready) return OMG_OK;
    for (auto& e : ctx->ev) OMG_HIP(hipEventCreate(&e));
    ctx->ev_ready = 1;
    return OMG_OK;
}

int stage_edges(omg_ctx* ctx, int64_t n_e, const int32_t* qe_query, const omg_node_t* qe_node, int where,
                const omg_node_t* rset, int64_t n_rset, const int32_t** q_dev, const omg_node_t** u_dev,
                const omg_node_t** rset_dev) {
    if (where == OMG_DEVICE) {
        *q_dev = qe_query;
        *u_dev = qe_node;
        *rset_dev = rset;
        return OMG_OK;
    }
    OMG_TRY(ctx->edges_in.ensure(sizeof(int32_t) * (size_t)(2 * n_e + 2)));
    int32_t* d = ctx->edges_in.as<int32_t>();
    if (n_e > 0) {
        OMG_HIP(hipMemcpyAsync(d, qe_query, sizeof(int32_t) * (size_t)n_e, hipMemcpyHostToDevice, ctx->stream));
        OMG_HIP(hipMemcpyAsync(d + n_e, qe_node, sizeof(int32_t) * (size_t)n_e, hipMemcpyHostToDevice, ctx->stream));
    }
    *q_dev = d;
    *u_dev = d + n_e;
    *rset_dev = nullptr;
    if (rset != nullptr) {
        OMG_TRY(ctx->rset_in.ensure(sizeof(int32_t) * (size_t)(n_rset + 1)));
        if (n_rset > 0)
            OMG_HIP(hipMemcpyAsync(ctx->rset_in.p, rset, sizeof(int32_t) * (size_t)n_rset, hipMemcpyHostToDevice,
                                   ctx->stream));
        *rset_dev = ctx->rset_in.as<omg_node_t>();
    }
    return OMG_OK;
}

int check_request(const omg_ctx* ctx, int32_t n_query, int64_t n_e, const int32_t* qe_query, const omg_node_t* qe_node,
                  int where, uint32_t gamma_ppm, const omg_node_t* rset, int64_t n_rset) {
    if (ctx == nullptr || n_query < 0 || n_e < 0 || n_e >= (int64_t)1 << 31) return OMG_EINVAL;
    if (n_e > 0 && (qe_query == nullptr || qe_node == nullptr)) return OMG_EINVAL;
    if (where != OMG_HOST && where != OMG_DEVICE) return OMG_EINVAL;
    if (rset == nullptr && gamma_ppm > 1000000u) return OMG_EINVAL;
    if (n_rset < 0 || (rset == nullptr && n_rset != 0)) return OMG_EINVAL;
    if (n_e > 0 && n_query == 0) return OMG_ERANGE;
    return OMG_OK;
}

// Device memory one layer needs beyond its inputs and outputs, in floats (0: not needed).
struct LayerScratchSizes {
    size_t agg = 0, agg2 = 0, partial = 0, fold = 0, logits = 0, split = 0;
};
struct LayerScratch {
    float* agg = nullptr;       // aggregated rows, the update's input
    float* agg2 = nullptr;      // normalised moments: the second pass's sums
    float* partial = nullptr;   // partial sums of rows cut into parts
    float* fold = nullptr;      // GAT: folded score vectors
    float* logits = nullptr;    // GAT: both score halves of the freshly computed rows
    float* split = nullptr;     // update of few rows: raw sums of the blocks that share an output tile
    size_t split_floats = 0;
};

LayerScratchSizes layer_scratch_sizes(const omg_graph* g, int is_last, const omg_layer* L) {
    LayerScratchSizes z;
    const int64_t n_rows = is_last ? g->n_query : g->rows_in;
    const int64_t n_parts = is_last ? g->c.n_parts_last : g->c.n_parts;
    const int64_t n_cut = is_last ? g->c.n_split_last + g->c.n_split_big_last : g->c.n_split + g->c.n_split_big;
    const int64_t agg_ld = round_up(L->d_in, 8);
    if (L->model == OMG_GAT) {
        const int H = L->heads;
        z.agg = (size_t)(n_rows * H * agg_ld);
        z.partial = (size_t)((n_cut > 0 ? n_parts : 0) * (H * agg_ld + OMG_GAT_STAT_PAD) + 4);
        z.fold = 2 * (size_t)H * L->d_in;
        z.logits = 2 * (size_t)(g->rows_in * H + 4);
    } else {
        z.agg = (size_t)(n_rows * agg_ld);
        z.partial = (size_t)((n_cut > 0 ? n_parts : 0) * agg_ld + 4);
        if (L->model == OMG_SAGE_MEAN && L->aggregator == OMG_AGG_MOMENT) z.agg2 = z.agg;
    }
    if (n_rows <= 128 * 64) z.split = OMG_GEMM_SPLIT_BYTES / sizeof(float);
    return z;
}

// the context's own growable buffers
int scratch_from_context(omg_ctx* ctx, const LayerScratchSizes& z, LayerScratch* out) {
    struct { DevBuf* b; size_t n; float** p; } want[] = {
        {&ctx->agg, z.agg, &out->agg}, {&ctx->agg2, z.agg2, &out->agg2}, {&ctx->partial, z.partial, &out->partial},
        {&ctx->foldv, z.fold, &out->fold}, {&ctx->dstlog, z.logits, &out->logits}, {&ctx->gemmSplit, z.split, &out->split}};
    for (auto& w : want) {
        if (w.n == 0) continue;
        OMG_TRY(w.b->ensure(sizeof(float) * w.n));
        *w.p = w.b->as<float>();
    }
    out->split_floats = z.split;
    return OMG_OK;
}

// ---- scratch that is part of the library's image: for callers that must not allocate (omg_run_layer_static)
constexpr int OMG_MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[OMG_MAX_DEVICES] = {};      // the array's address on each device (every GPU has its own copy)

// Called with `device` current.  The array's name is a host-side stand-in; its device address comes from the runtime.
int static_scratch_init(int device) {
    if (device < 0 || device >= OMG_MAX_DEVICES) return OMG_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device] != nullptr) return OMG_OK;
    void* p = nullptr;
    OMG_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr || (reinterpret_cast<uintptr_t>(p) & 255u) != 0) return OMG_EHIP;
    g_scratch_ptr[device] = static_cast<unsigned char*>(p);
    return OMG_OK;
}

// carves the layer's scratch out of the static array: 256-byte aligned pieces, one after the other
int scratch_from_static(const omg_ctx* ctx, const LayerScratchSizes& z, LayerScratch* out) {
    unsigned char* base = (ctx->device >= 0 && ctx->device < OMG_MAX_DEVICES) ? g_scratch_ptr[ctx->device] : nullptr;
    if (base == nullptr) return OMG_ESTATE;
    size_t at = 0;
    struct { size_t n; float** p; } want[] = {{z.agg, &out->agg}, {z.agg2, &out->agg2}, {z.partial, &out->partial},
                                              {z.fold, &out->fold}, {z.logits, &out->logits}, {z.split, &out->split}};
    for (auto& w : want) {
        if (w.n == 0) continue;
        const size_t bytes = (sizeof(float) * w.n + 255) & ~(size_t)255;
        if (bytes > OMG_STATIC_SCRATCH_BYTES - at) return OMG_ESCRATCH;
        *w.p = reinterpret_cast<float*>(base + at);
        at += bytes;
    }
    out->split_floats = z.split;
    return OMG_OK;
}

}  // namespace

void omg_note_hip_error(hipError_t e, const char* what, int line) {
    snprintf(g_hip_msg, sizeof(g_hip_msg), "%s at line %d: %s", hipGetErrorString(e), line, what);
    fprintf(stderr, "omega_srpe: HIP error: %s\n", g_hip_msg);
}

// fault injection for tests of the error paths: the allocation that finds this counter at zero fails
static std::atomic<long long> g_fail_allocation{-1};

int DevBuf::ensure(size_t bytes) {
    if (bytes <= cap && p != nullptr) return OMG_OK;
    if (g_fail_allocation.load() >= 0 && g_fail_allocation.fetch_sub(1) == 0) return OMG_ENOMEM;
    if (bytes == 0) bytes = 16;
    size_t want = bytes + bytes / 4;                 // head room so that slightly larger batches do not reallocate
    want = (want + 255) & ~(size_t)255;
    void* np = nullptr;
    hipError_t e = hipMalloc(&np, want);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return OMG_ENOMEM;
    }
    if (p != nullptr) (void)hipFree(p);              // synchronises with work that still uses the old block
    p = np;
    cap = want;
    return OMG_OK;
}

void DevBuf::release() {
    if (p != nullptr) (void)hipFree(p);
    p = nullptr;
    cap = 0;
}

extern "C" {

const char* omg_strerror(int code) {
    switch (code) {
        case OMG_OK: return "ok";
        case OMG_EINVAL: return "invalid argument";
        case OMG_ERANGE: return "index out of range";
        case OMG_ENOMEM: return "out of memory";
        case OMG_ESTATE: return "object in the wrong state";
        case OMG_EHIP: return g_hip_msg[0] ? g_hip_msg : "HIP runtime error";
        case OMG_EUNSUPPORTED: return "shape not supported by the kernels";
        case OMG_ESCRATCH: return "the layer needs more scratch memory than the library's static buffer holds";
        default: return "unknown error";
    }
}

void omg_debug_fail_allocation(int64_t nth) { g_fail_allocation.store(nth); }

int omg_debug_set_small_path(omg_ctx* ctx, int32_t on) {
    if (ctx == nullptr) return OMG_EINVAL;
    ctx->small_path = on == 2 ? 2 : on != 0 ? 1 : 0;
    return OMG_OK;
}

int omg_debug_set_gather_multi(omg_ctx* ctx, int32_t on) {
    if (ctx == nullptr) return OMG_EINVAL;
    ctx->gather_multi = on != 0;
    ctx->gather_multi_min_parts = on > 1 ? 0 : 32768;      // on > 1: also for launches of few work items
    return OMG_OK;
}

int omg_debug_set_fused_sum_limit(omg_ctx* ctx, int32_t limit) {
    if (ctx == nullptr || limit < 1) return OMG_EINVAL;
    ctx->fused_sum_max = limit;
    return OMG_OK;
}

int omg_create(omg_ctx** out, const omg_base_csr* graph, void* hip_stream) {
    if (out == nullptr || graph == nullptr) return OMG_EINVAL;
    *out = nullptr;
    if (graph->n_nodes <= 0 || graph->n_nodes >= ((int64_t)1 << 31) || graph->indptr == nullptr) return OMG_EINVAL;
    omg_ctx* ctx = new (std::nothrow) omg_ctx();
    if (ctx == nullptr) return OMG_ENOMEM;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    ctx->base = *graph;
    int rc = OMG_OK;
    do {
        if (hipGetDevice(&ctx->device) != hipSuccess) { rc = OMG_EHIP; break; }
        rc = static_scratch_init(ctx->device);
        if (rc != OMG_OK) break;
        if (hipMalloc(reinterpret_cast<void**>(&ctx->node), sizeof(omg_ctx::NodeRec) * (size_t)graph->n_nodes) != hipSuccess) { rc = OMG_ENOMEM; break; }
        // pinned and coherent: the builder's last kernel of the first half writes the batch's sizes here
        if (hipHostMalloc(reinterpret_cast<void**>(&ctx->mailbox), sizeof(HostMailbox), hipHostMallocMapped | hipHostMallocCoherent) != hipSuccess) { rc = OMG_ENOMEM; break; }
        memset(ctx->mailbox, 0, sizeof(HostMailbox));
        ctx->counts_host = &ctx->mailbox->counts;
        if (hipHostGetDevicePointer(reinterpret_cast<void**>(&ctx->mailbox_dev), ctx->mailbox, 0) != hipSuccess) { rc = OMG_EHIP; break; }
        rc = omg_init_state(ctx);
        if (rc == OMG_OK) rc = omg_validate_base(ctx);
    } while (0);
    if (rc != OMG_OK) {
        omg_destroy(ctx);
        return rc;
    }
    *out = ctx;
    return OMG_OK;
}

void omg_destroy(omg_ctx* ctx) {
    if (ctx == nullptr) return;
    (void)hipStreamSynchronize(ctx->stream);
    if (ctx->serve_graph != nullptr) omg_graph_destroy(ctx->serve_graph);
    DevBuf* bufs[] = {&ctx->devState, &ctx->bitmap, &ctx->bitmap1,
                      &ctx->wordList, &ctx->wordCnt, &ctx->smallRaw, &ctx->chunkTot, &ctx->flagTot, &ctx->rowTot, &ctx->qcnt, &ctx->qcur,
                      &ctx->tcur, &ctx->skey, &ctx->flag, &ctx->tLen, &ctx->tOff, &ctx->nParts,
                      &ctx->listSmall, &ctx->listMed, &ctx->listBig, &ctx->sortTmp, &ctx->subSeg, &ctx->edges_in, &ctx->rset_in,
                      &ctx->agg, &ctx->agg2, &ctx->partial, &ctx->gemmSplit, &ctx->preIds, &ctx->preNparts, &ctx->preCounts, &ctx->preCdeg,
                      &ctx->preSelf, &ctx->preStage, &ctx->foldv, &ctx->dstlog, &ctx->srclog, &ctx->buf[0], &ctx->buf[1],
                      &ctx->bufInit, &ctx->preInit, &ctx->rowOff, &ctx->cgpLen, &ctx->cgpOff, &ctx->cgpNp, &ctx->cgpCounts};
    for (DevBuf* b : bufs) b->release();
    if (ctx->node) (void)hipFree(ctx->node);
    if (ctx->mailbox) (void)hipHostFree(ctx->mailbox);
    if (ctx->ev_ready)
        for (auto& e : ctx->ev) (void)hipEventDestroy(e);
    delete ctx;
}

int omg_set_policy(omg_ctx* ctx, int policy, uint64_t seed, const float* node_scores) {
    if (ctx == nullptr || policy < OMG_POLICY_RATIO || policy > OMG_POLICY_SCORE) return OMG_EINVAL;
    if (policy == OMG_POLICY_SCORE && node_scores == nullptr) return OMG_EINVAL;
    ctx->policy = policy;
    ctx->policy_seed = seed;
    ctx->node_scores = policy == OMG_POLICY_SCORE ? node_scores : nullptr;
    return OMG_OK;
}

int omg_set_profiling(omg_ctx* ctx, int on) {
    if (ctx == nullptr) return OMG_EINVAL;
    if (on) OMG_TRY(ensure_events(ctx));
    ctx->profiling = on == 2 ? 2 : on ? 1 : 0;
    ctx->layer_cursor = 0;
    ctx->build_timed = 0;
    return OMG_OK;
}

int omg_get_timing(omg_ctx* ctx, omg_timing* out) {
    if (ctx == nullptr || out == nullptr) return OMG_EINVAL;
    if (!ctx->profiling || !ctx->ev_ready) return OMG_ESTATE;
    memset(out, 0, sizeof(*out));
    OMG_HIP(hipStreamSynchronize(ctx->stream));
    float total = 0.f;
    if (ctx->build_timed) {
        OMG_HIP(hipEventElapsedTime(&out->build_ms, ctx->ev[0], ctx->ev[1]));
        total += out->build_ms;
    }
    for (int l = 0; l < ctx->layer_cursor && l < OMG_MAX_LAYERS; ++l) {
        if (ctx->main_timed[l]) {
            OMG_HIP(hipEventElapsedTime(&out->gather_ms[l], ctx->ev[ctx->start_idx[l]], ctx->ev[3 + 4 * l]));
            OMG_HIP(hipEventElapsedTime(&out->combine_ms[l], ctx->ev[3 + 4 * l], ctx->ev[4 + 4 * l]));
        } else {
            OMG_HIP(hipEventElapsedTime(&out->gather_ms[l], ctx->ev[ctx->start_idx[l]], ctx->ev[4 + 4 * l]));
        }
        OMG_HIP(hipEventElapsedTime(&out->update_ms[l], ctx->ev[4 + 4 * l], ctx->ev[5 + 4 * l]));
        total += out->gather_ms[l] + out->combine_ms[l] + out->update_ms[l];
    }
    out->total_ms = total;
    return OMG_OK;
}

int omg_build_computation_graph(omg_ctx* ctx, int32_t n_query, int64_t n_qedges, const int32_t* qe_query,
                                const omg_node_t* qe_node, int where, uint32_t gamma_ppm,
                                const omg_node_t* recompute_set, int64_t n_recompute, omg_graph** graph) {
    if (graph == nullptr) return OMG_EINVAL;
    OMG_TRY(check_request(ctx, n_query, n_qedges, qe_query, qe_node, where, gamma_ppm, recompute_set, n_recompute));
    omg_graph* g = *graph;
    bool fresh = false;
    if (g == nullptr) {
        g = new (std::nothrow) omg_graph();
        if (g == nullptr) return OMG_ENOMEM;
        g->ctx = ctx;
        fresh = true;
    } else if (g->ctx != ctx) {
        return OMG_ESTATE;
    }
    const int32_t* q_dev = nullptr;
    const omg_node_t* u_dev = nullptr;
    const omg_node_t* r_dev = nullptr;
    int rc = OMG_OK;
    if (ctx->profiling) {
        ctx->layer_cursor = 0;
        ctx->build_timed = 0;
        if (hipEventRecord(ctx->ev[0], ctx->stream) != hipSuccess) rc = OMG_EHIP;
    }
    if (rc == OMG_OK) rc = stage_edges(ctx, n_qedges, qe_query, qe_node, where, recompute_set, n_recompute, &q_dev, &u_dev, &r_dev);
    if (rc == OMG_OK) rc = omg_build_impl(ctx, g, n_query, n_qedges, q_dev, u_dev, gamma_ppm, r_dev, n_recompute);
    if (rc == OMG_OK && ctx->profiling) {
        if (hipEventRecord(ctx->ev[1], ctx->stream) != hipSuccess) rc = OMG_EHIP;
        else ctx->build_timed = 1;
    }
    if (rc != OMG_OK) {
        if (fresh) omg_graph_destroy(g);
        return rc;
    }
    *graph = g;
    return OMG_OK;
}

int omg_graph_sizes(const omg_graph* g, int64_t sizes[4]) {
    if (g == nullptr || sizes == nullptr) return OMG_EINVAL;
    if (!g->built) return OMG_ESTATE;
    sizes[0] = g->c.n_cand;
    sizes[1] = g->c.n_target;
    sizes[2] = g->rows_in;
    sizes[3] = g->c.nnz_in;
    return OMG_OK;
}

int omg_graph_export(const omg_graph* g, omg_node_t* cand, int32_t* qdeg, omg_node_t* targets, int64_t* indptr,
                     int32_t* cols, int32_t* cdeg) {
    if (g == nullptr) return OMG_EINVAL;
    if (!g->built) return OMG_ESTATE;
    OMG_HIP(hipStreamSynchronize(g->ctx->stream));
    const size_t nc = (size_t)g->c.n_cand, nt = (size_t)g->c.n_target, nz = (size_t)g->c.nnz_in;
    if (cand && nc) OMG_HIP(hipMemcpy(cand, g->cand.p, nc * sizeof(int32_t), hipMemcpyDeviceToHost));
    if (qdeg && nc) OMG_HIP(hipMemcpy(qdeg, g->qdeg.p, nc * sizeof(int32_t), hipMemcpyDeviceToHost));
    if (targets && nt) OMG_HIP(hipMemcpy(targets, g->targets.p, nt * sizeof(int32_t), hipMemcpyDeviceToHost));
    if (indptr) OMG_HIP(hipMemcpy(indptr, g->indptr.p, (size_t)(g->rows_in + 1) * sizeof(int64_t), hipMemcpyDeviceToHost));
    if (cols && nz) OMG_HIP(hipMemcpy(cols, g->cols.p, nz * sizeof(int32_t), hipMemcpyDeviceToHost));
    if (cdeg && nz) OMG_HIP(hipMemcpy(cdeg, g->cdeg.p, nz * sizeof(int32_t), hipMemcpyDeviceToHost));
    return OMG_OK;
}

void omg_graph_destroy(omg_graph* g) {
    if (g == nullptr) return;
    if (g->ctx != nullptr) {
        (void)hipStreamSynchronize(g->ctx->stream);
        if (g->ctx->serve_graph == g) g->ctx->serve_graph = nullptr;
    }
    DevBuf* bufs[] = {&g->cand, &g->qdeg, &g->cand_row, &g->targets, &g->target_slot, &g->indptr, &g->cols,
                      &g->cdeg, &g->order, &g->part_ptr, &g->part_row, &g->split_rows, &g->split_rows_q, &g->split_big, &g->split_big_q};
    for (DevBuf* b : bufs) b->release();
    delete g;
}

int omg_init_buffer(omg_ctx* ctx, const omg_graph* g, const omg_table* features, const float* query_feats,
                    int64_t ld_q, float* buf0, int64_t ld0) {
    if (ctx == nullptr || g == nullptr || buf0 == nullptr) return OMG_EINVAL;
    if (!g->built || g->ctx != ctx) return OMG_ESTATE;
    OMG_TRY(check_table(features));
    if (g->n_query > 0 && (query_feats == nullptr || ld_q < features->dim)) return OMG_EINVAL;
    if (ld0 < features->dim) return OMG_EINVAL;
    return omg_launch_init_buffer(features, query_feats, ld_q, g->targets.as<omg_node_t>(), g->n_query,
                                  g->c.n_target, buf0, ld0, ctx->stream);
}

int omg_gat_fold(omg_ctx* ctx, const omg_layer* layer, float* fold) {
    if (ctx == nullptr || fold == nullptr || !aligned16(fold)) return OMG_EINVAL;
    OMG_TRY(check_layer(layer));
    if (layer->model != OMG_GAT) return OMG_EINVAL;
    return omg_launch_gat_fold(layer, fold, fold + (size_t)layer->heads * layer->d_in, ctx->stream);
}

int omg_gat_src_logits(omg_ctx* ctx, const omg_table* table, const omg_layer* layer, float* logits) {
    if (ctx == nullptr || logits == nullptr) return OMG_EINVAL;
    OMG_TRY(check_table(table));
    OMG_TRY(check_layer(layer));
    if (layer->model != OMG_GAT || table->dim != layer->d_in) return OMG_EINVAL;
    const size_t fold = sizeof(float) * (size_t)layer->heads * layer->d_in;
    OMG_TRY(ctx->foldv.ensure(2 * fold));
    float* fs = ctx->foldv.as<float>();
    OMG_TRY(omg_launch_gat_fold(layer, fs, fs + (size_t)layer->heads * layer->d_in, ctx->stream));
    return omg_launch_table_logits(table, fs, layer->heads, logits, ctx->stream);
}

// Where a partition's local aggregations go instead of into the layer's update (Sec. 6, Eq. 3).
struct LocalOut {
    float* wire;
    int64_t ld_wire;
    const float* row_mean;    // normalised moments, second step: the rows' overall means
    int64_t ld_mean;
};

// the layer's update (the U of Eq. 1 / Eq. 3) from aggregated rows
static int launch_layer_update(omg_ctx* ctx, const omg_layer* L, int64_t n_rows, const float* agg, int64_t agg_ld,
                               const float* buf_prev, int64_t ld_prev, float* buf_out, int64_t ld_out,
                               float* split_buf, size_t split_floats) {
    GemmArgs ga{};
    ga.m = n_rows;
    ga.n_z = 1;
    ga.scale = 1.f;
    ga.bias = L->bias;
    ga.bias_sum = 1;
    ga.act = L->act;
    ga.out = buf_out;
    ga.ldo = ld_out;
    const int d_in = L->d_in;
    if (L->model == OMG_GAT) {
        const int H = L->heads, dh = L->d_out / H;
        ga.n = dh;
        if (L->head_mean) {
            ga.n_seg = H;
            for (int h = 0; h < H; ++h)
                ga.seg[h] = GemmSeg{agg + (int64_t)h * agg_ld, (int64_t)H * agg_ld, L->W_nb + h * dh, L->d_out, d_in};
            ga.scale = 1.f / (float)H;
            ga.bias_sum = H;
        } else {
            ga.n_seg = 1;
            ga.seg[0] = GemmSeg{agg, (int64_t)H * agg_ld, L->W_nb, L->d_out, d_in};
            ga.n_z = H;
            ga.a_z_stride = agg_ld;
            ga.w_z_stride = dh;
            ga.out_z_stride = dh;
        }
    } else {
        ga.n = L->d_out;
        if (L->model == OMG_SAGE_MEAN) {
            ga.n_seg = 2;
            ga.seg[0] = GemmSeg{buf_prev, ld_prev, L->W_self, L->d_out, d_in};
            ga.seg[1] = GemmSeg{agg, agg_ld, L->W_nb, L->d_out, d_in};
        } else {
            ga.n_seg = 1;
            ga.seg[0] = GemmSeg{agg, agg_ld, L->W_nb, L->d_out, d_in};
        }
    }
    // launches of few blocks (the last layer: one row per query) split their K-tiles over more blocks
    if (n_rows <= 128 * 64 && split_buf != nullptr) {
        ga.split_buf = split_buf;
        ga.split_floats = (int64_t)split_floats;
    }
    return omg_launch_update(ga, ctx->stream);
}

static int run_layer(omg_ctx* ctx, const omg_graph* g, int is_last, const omg_table* table_prev, const float* buf_prev,
                     int64_t ld_prev, const omg_layer* L, float* buf_out, int64_t ld_out, const float* init_rows,
                     int64_t init_ld, const LocalOut* local = nullptr, bool static_scratch = false) {
    if (ctx == nullptr || g == nullptr || (buf_out == nullptr && local == nullptr)) return OMG_EINVAL;
    if (!g->built || g->ctx != ctx) return OMG_ESTATE;
    OMG_TRY(check_table(table_prev));
    OMG_TRY(check_layer(L));
    const int d_in = L->d_in;
    if (table_prev->dim != d_in || table_prev->n_rows < ctx->base.n_nodes) return OMG_EINVAL;
    if (buf_prev == nullptr || ld_prev < d_in || ld_prev % 4 != 0 || !aligned16(buf_prev)) return OMG_EINVAL;
    if (local == nullptr && ld_out < layer_out_width(L)) return OMG_EINVAL;
    if (local == nullptr && L->model == OMG_GCNII && (init_rows == nullptr || init_ld < d_in || init_ld % 4 != 0 || !aligned16(init_rows)))
        return OMG_EINVAL;

    hipStream_t s = ctx->stream;
    const int64_t n_rows = is_last ? g->n_query : g->rows_in;
    const int64_t n_parts = is_last ? g->c.n_parts_last : g->c.n_parts;
    const int64_t n_split = is_last ? g->c.n_split_last : g->c.n_split;
    const int64_t agg_ld = round_up(d_in, 8);
    const int li = ctx->layer_cursor;
    const bool timed = ctx->profiling && li < OMG_MAX_LAYERS && local == nullptr;
    const bool timed_main = timed && (ctx->profiling == 1 || li == 0);       // the main kernel apart from the combine
    if (timed) ctx->main_timed[li] = timed_main;
    if (n_rows == 0) return OMG_OK;
    // A table much larger than the memory-side cache, read several times over by one launch: walk the work
    // items by table region rather than by row (the order is built once per graph, before the timed part).
    const int32_t* order = nullptr;
    {
        const int64_t row_bytes = table_prev->ld * (table_prev->dtype == OMG_F32 ? 4 : 2);
        const int64_t table_bytes = table_prev->n_rows * row_bytes;
        // (building the order allocates: a caller that must not allocate gets it only if the graph already has it)
        if (!is_last && L->model != OMG_GAT && table_bytes > OMG_ORDER_MIN_TABLE_BYTES &&
            omg_order_pays(g->c.nnz_in * row_bytes, table_bytes) &&
            (static_scratch ? g->order_ready : omg_graph_order(ctx, const_cast<omg_graph*>(g)) == OMG_OK))
            order = g->order.as<int32_t>();
    }
    LayerScratch sc;
    {
        const LayerScratchSizes z = layer_scratch_sizes(g, is_last, L);
        if (static_scratch) {
            if (L->model == OMG_GAT && L->src_logits == nullptr) return OMG_EINVAL;      // the side table would be an allocation
            OMG_TRY(scratch_from_static(ctx, z, &sc));
        } else {
            OMG_TRY(scratch_from_context(ctx, z, &sc));
        }
    }
    if (timed) {
        const int prev_end = li == 0 ? (ctx->build_timed ? 1 : -1) : 5 + 4 * (li - 1);
        if (ctx->chain_events && prev_end >= 0) {
            ctx->start_idx[li] = prev_end;
        } else {
            ctx->start_idx[li] = 2 + 4 * li;
            OMG_HIP(hipEventRecord(ctx->ev[2 + 4 * li], s));
        }
    }

    if (L->model == OMG_SAGE_MEAN || L->model == OMG_GCN_SYM || L->model == OMG_GCNII) {
        GatherArgs a{};
        a.indptr = g->indptr.as<int64_t>();
        a.cols = g->cols.as<int32_t>();
        a.cdeg = g->cdeg.as<int32_t>();
        a.part_ptr = g->part_ptr.as<int32_t>();
        a.part_row = g->part_row.as<int32_t>();
        a.n_parts = n_parts;
        a.nnz = is_last ? g->n_qedges : g->c.nnz_in;
        a.multi_ok = ctx->gather_multi ? 1 : 0;
        a.multi_min_parts = ctx->gather_multi_min_parts;
        a.part_edges = g->part_edges;
        a.split_rows = is_last ? g->split_rows_q.as<int32_t>() : g->split_rows.as<int32_t>();
        a.split_big = is_last ? g->split_big_q.as<int32_t>() : g->split_big.as<int32_t>();
        a.n_split_big = is_last ? g->c.n_split_big_last : g->c.n_split_big;
        a.n_split = n_split;
        a.n_rows = n_rows;
        a.table = table_prev->data;
        a.table_dtype = table_prev->dtype;
        a.table_ld = table_prev->ld;
        a.buf = buf_prev;
        a.buf_ld = ld_prev;
        a.dim = d_in;
        a.agg_p = L->agg_p;
        a.agg_eps = L->agg_eps;
        a.agg = sc.agg;
        a.agg_ld = agg_ld;
        a.partial = sc.partial;
        a.order = order;
        static const int op_of[] = {OMG_OP_MEAN, OMG_OP_SUM, OMG_OP_MAX, OMG_OP_POW, OMG_OP_MOM};
        a.op = L->model == OMG_SAGE_MEAN ? op_of[L->aggregator] : OMG_OP_GCN;
        if (L->model == OMG_GCNII) {
            a.h0 = init_rows;
            a.h0_ld = init_ld;
            a.alpha = L->alpha;
        }
        if (local != nullptr) {
            // a partition's local aggregation: unfinished rows straight into the caller's records.  The mean is
            // a sum until the merge; the moments take the rows' overall means from the caller (their first step
            // is a plain sum, merged by omg_cgp_merge_mean)
            a.raw = 1;
            a.agg = local->wire;
            a.agg_stride = local->ld_wire;
            a.h0 = nullptr;
            if (a.op == OMG_OP_MEAN) a.op = OMG_OP_SUM;
            if (a.op == OMG_OP_MOM) {
                if (local->row_mean == nullptr) a.op = OMG_OP_SUM;
                a.mean = local->row_mean;
                a.mean_ld = local->ld_mean;
            }
            return omg_launch_gather(a, s, nullptr);
        }
        if (a.op == OMG_OP_MOM) {
            // two passes, as the moment is defined around the row's mean: the mean first (into agg), then the
            // powers of the differences from it (into agg2); the partial sums of the first pass are consumed
            // by its own combine before the second pass overwrites them (same stream)
            a.op = OMG_OP_MEAN;
            OMG_TRY(omg_launch_gather(a, s, timed_main ? ctx->ev[3 + 4 * li] : nullptr));
            a.op = OMG_OP_MOM;
            a.mean = sc.agg;
            a.agg = sc.agg2;
            OMG_TRY(omg_launch_gather(a, s, nullptr));
        } else {
            OMG_TRY(omg_launch_gather(a, s, timed_main ? ctx->ev[3 + 4 * li] : nullptr));
        }
        if (timed) OMG_HIP(hipEventRecord(ctx->ev[4 + 4 * li], s));
        OMG_TRY(launch_layer_update(ctx, L, n_rows, a.agg, agg_ld, buf_prev, ld_prev, buf_out, ld_out, sc.split, sc.split_floats));
    } else {
        const int H = L->heads;
        const size_t fold = (size_t)H * d_in;
        const float* src_logits = L->src_logits;
        if (src_logits == nullptr) OMG_TRY(ctx->srclog.ensure(sizeof(float) * (size_t)(table_prev->n_rows * H + 4)));
        const float* fs = L->fold;
        if (fs == nullptr) {                             // no folded vectors supplied: take them now
            OMG_TRY(omg_launch_gat_fold(L, sc.fold, sc.fold + fold, s));
            fs = sc.fold;
        }
        if (src_logits == nullptr) {
            // no side table supplied: take the stored rows' score halves now (a full pass over the table)
            OMG_TRY(omg_launch_table_logits(table_prev, fs, H, ctx->srclog.as<float>(), s));
            src_logits = ctx->srclog.as<float>();
        }
        GatArgs a{};
        a.indptr = g->indptr.as<int64_t>();
        a.cols = g->cols.as<int32_t>();
        a.part_ptr = g->part_ptr.as<int32_t>();
        a.part_row = g->part_row.as<int32_t>();
        a.n_parts = n_parts;
        a.part_edges = g->part_edges;
        a.split_rows = is_last ? g->split_rows_q.as<int32_t>() : g->split_rows.as<int32_t>();
        a.split_big = is_last ? g->split_big_q.as<int32_t>() : g->split_big.as<int32_t>();
        a.n_split_big = is_last ? g->c.n_split_big_last : g->c.n_split_big;
        a.n_split = n_split;
        a.n_rows = n_rows;
        a.table = table_prev->data;
        a.table_dtype = table_prev->dtype;
        a.table_ld = table_prev->ld;
        a.buf = buf_prev;
        a.buf_ld = ld_prev;
        a.dim = d_in;
        a.heads = H;
        a.leaky = L->leaky_slope;
        a.fold_src = fs;
        a.fold_dst = fs + fold;
        a.src_logits = src_logits;
        a.buf_logits = sc.logits;
        a.dst_logits = sc.logits + (size_t)(g->rows_in * H + 4);
        a.n_buf_rows = g->rows_in;
        a.agg = sc.agg;
        a.agg_ld = agg_ld;
        a.partial = sc.partial;
        if (local != nullptr) {
            a.raw = 1;
            a.agg = local->wire;
            a.agg_stride = local->ld_wire;
            return omg_launch_gat(a, s, nullptr);
        }
        OMG_TRY(omg_launch_gat(a, s, timed_main ? ctx->ev[3 + 4 * li] : nullptr));
        if (timed) OMG_HIP(hipEventRecord(ctx->ev[4 + 4 * li], s));
        OMG_TRY(launch_layer_update(ctx, L, n_rows, a.agg, agg_ld, buf_prev, ld_prev, buf_out, ld_out, sc.split, sc.split_floats));
    }
    if (timed) {
        OMG_HIP(hipEventRecord(ctx->ev[5 + 4 * li], s));
        ctx->layer_cursor = li + 1;
    }
    return OMG_OK;
}

int omg_run_layer(omg_ctx* ctx, const omg_graph* g, int is_last, const omg_table* table_prev, const float* buf_prev,
                  int64_t ld_prev, const omg_layer* L, float* buf_out, int64_t ld_out) {
    if (L == nullptr) return OMG_EINVAL;
    return run_layer(ctx, g, is_last, table_prev, buf_prev, ld_prev, L, buf_out, ld_out, L->init_rows, L->init_ld);
}

int omg_run_layer_static(omg_ctx* ctx, const omg_graph* g, int is_last, const omg_table* table_prev, const float* buf_prev,
                         int64_t ld_prev, const omg_layer* L, float* buf_out, int64_t ld_out) {
    if (L == nullptr) return OMG_EINVAL;
    return run_layer(ctx, g, is_last, table_prev, buf_prev, ld_prev, L, buf_out, ld_out, L->init_rows, L->init_ld, nullptr, true);
}

int64_t omg_static_scratch_bytes(void) { return (int64_t)OMG_STATIC_SCRATCH_BYTES; }

int omg_serve_batch(omg_ctx* ctx, int32_t k, const omg_table* tables, const omg_layer* layers,
                    const float* query_feats, int64_t ld_q, int32_t n_query, int64_t n_qedges,
                    const int32_t* qe_query, const omg_node_t* qe_node, int where, uint32_t gamma_ppm, float* out,
                    int64_t ld_o) {
    if (ctx == nullptr || tables == nullptr || layers == nullptr || (out == nullptr && n_query > 0)) return OMG_EINVAL;
    if (k < 1 || k > OMG_MAX_LAYERS) return OMG_EINVAL;
    // the request is checked before anything is sized from it (the buffers below grow with gamma_ppm)
    OMG_TRY(check_request(ctx, n_query, n_qedges, qe_query, qe_node, where, gamma_ppm, nullptr, 0));
    int64_t max_w = 0;
    for (int l = 0; l < k; ++l) {
        OMG_TRY(check_table(&tables[l]));
        OMG_TRY(check_layer(&layers[l]));
        if (tables[l].dim != layers[l].d_in) return OMG_EINVAL;
        if (l > 0 && layer_out_width(&layers[l - 1]) != layers[l].d_in) return OMG_EINVAL;
        if (layers[l].d_in > max_w) max_w = layers[l].d_in;
    }
    if (ld_o < layer_out_width(&layers[k - 1])) return OMG_EINVAL;
    if (n_query > 0 && (query_feats == nullptr || ld_q < tables[0].dim)) return OMG_EINVAL;

    // announce the largest table an inner layer gathers by rows, so that the build can order the work items
    ctx->hint_table_bytes = ctx->hint_row_bytes = 0;
    {
        for (int l = 0; l + 1 < k; ++l) {
            if (layers[l].model == OMG_GAT) continue;
            const int64_t row_bytes = tables[l].ld * (tables[l].dtype == OMG_F32 ? 4 : 2);
            if (tables[l].n_rows * row_bytes > ctx->hint_table_bytes) {
                ctx->hint_table_bytes = tables[l].n_rows * row_bytes;
                ctx->hint_row_bytes = row_bytes;
            }
        }
    }
    ctx->hint_min_part_edges = 0;
    for (int l = 0; l < k; ++l)
        if (layers[l].model == OMG_GAT) ctx->hint_min_part_edges = 64;
    // The buffers of freshly computed rows are sized before the graph is built, from what the budget allows at
    // most (|T| <= floor(gamma |R|), |R| <= number of request edges and of nodes): the layer-0 values can then be
    // written right behind the builder's read-back, while the host is still waiting for it.
    const int64_t ld = round_up(max_w, 8);
    const int64_t cand_max = n_qedges < ctx->base.n_nodes ? n_qedges : ctx->base.n_nodes;
    const int64_t rows_max = (int64_t)n_query + (int64_t)(((uint64_t)gamma_ppm * (uint64_t)cand_max) / 1000000ull);
    bool keep_init = false;
    for (int l = 0; l < k; ++l) keep_init = keep_init || layers[l].model == OMG_GCNII;
    if (n_query > 0) {
        // The layer-0 values go to buf[0], or to a buffer of their own when a layer reads them again later
        // (GCNII's initial residual): the two layer buffers are then free to alternate from layer 1 on.
        DevBuf* bufs[] = {&ctx->buf[0], &ctx->buf[1], keep_init ? &ctx->bufInit : nullptr};
        for (DevBuf* b : bufs) {
            const size_t need = sizeof(float) * (size_t)(rows_max * ld);
            if (b != nullptr && need > b->cap) {
                OMG_TRY(b->ensure(need));
                OMG_HIP(hipMemsetAsync(b->p, 0, b->cap, ctx->stream));
            }
        }
        ctx->early.armed = true;
        ctx->early.done = false;
        ctx->early.features = &tables[0];
        ctx->early.query_feats = query_feats;
        ctx->early.ld_q = ld_q;
        ctx->early.buf0 = keep_init ? ctx->bufInit.as<float>() : ctx->buf[0].as<float>();
        ctx->early.ld0 = ld;
        ctx->early.max_rows = rows_max;
    }
    const int rc_build = omg_build_computation_graph(ctx, n_query, n_qedges, qe_query, qe_node, where, gamma_ppm, nullptr, 0,
                                                     &ctx->serve_graph);
    const bool init_done = ctx->early.done;
    ctx->early.armed = ctx->early.done = false;
    ctx->hint_table_bytes = ctx->hint_row_bytes = 0;
    ctx->hint_min_part_edges = 0;
    OMG_TRY(rc_build);
    omg_graph* g = ctx->serve_graph;
    if (g->n_query == 0) return OMG_OK;
    if (g->rows_in > rows_max) return OMG_ESTATE;            // cannot happen: the bound is the budget's own
    float* init = keep_init ? ctx->bufInit.as<float>() : ctx->buf[0].as<float>();
    if (!init_done) OMG_TRY(omg_init_buffer(ctx, g, &tables[0], query_feats, ld_q, init, ld));
    ctx->chain_events = init_done;                           // nothing is launched between the phases from here on
    int rc = OMG_OK;
    for (int l = 1; l <= k && rc == OMG_OK; ++l) {
        const bool last = l == k;
        const float* prev = l == 1 ? init : ctx->buf[(l - 1) & 1].as<float>();
        float* next = last ? out : ctx->buf[l & 1].as<float>();
        rc = run_layer(ctx, g, last ? 1 : 0, &tables[l - 1], prev, ld, &layers[l - 1], next, last ? ld_o : ld, init, ld);
    }
    ctx->chain_events = false;
    return rc;
}

int omg_precompute_embeddings(omg_ctx* ctx, int32_t k, const omg_table* features, const omg_layer* layers,
                              const omg_table* out_tables) {
    if (ctx == nullptr || features == nullptr || layers == nullptr || k < 1 || k > OMG_MAX_LAYERS) return OMG_EINVAL;
    if (k > 1 && out_tables == nullptr) return OMG_EINVAL;
    OMG_TRY(check_table(features));
    for (int l = 1; l < k; ++l) {
        OMG_TRY(check_layer(&layers[l - 1]));
        OMG_TRY(check_table(&out_tables[l - 1]));
        const omg_table* prev = l == 1 ? features : &out_tables[l - 2];
        if (prev->dim != layers[l - 1].d_in || out_tables[l - 1].dim != layer_out_width(&layers[l - 1])) return OMG_EINVAL;
        if (prev->n_rows < ctx->base.n_nodes || out_tables[l - 1].n_rows < ctx->base.n_nodes) return OMG_EINVAL;
    }
    for (int l = 1; l < k; ++l)
        OMG_TRY(omg_precompute_layer(ctx, features, l == 1 ? features : &out_tables[l - 2], &layers[l - 1],
                                     &out_tables[l - 1]));
    return OMG_OK;
}

// ---- computation graph parallelism (Sec. 6): one partition's share, and the merge

static int64_t wire_width(const omg_layer* L) {
    const int64_t agg_ld = round_up(L->d_in, 8);
    return L->model == OMG_GAT ? (int64_t)L->heads * agg_ld + OMG_GAT_STAT_PAD : agg_ld + 4;
}

int64_t omg_cgp_wire_width(const omg_layer* layer) {
    if (check_layer(layer) != OMG_OK) return 0;
    return wire_width(layer);
}

int omg_cgp_partition_graph(omg_ctx* ctx, const omg_graph* graph, const int32_t* node_part, int32_t n_part, int32_t p,
                            omg_graph** part_graph) {
    if (ctx == nullptr || graph == nullptr || node_part == nullptr || part_graph == nullptr) return OMG_EINVAL;
    if (n_part < 1 || n_part > OMG_CGP_MAX_PARTS || p < 0 || p >= n_part) return OMG_EINVAL;
    if (!graph->built || graph->ctx != ctx) return OMG_ESTATE;
    omg_graph* g = *part_graph;
    bool fresh = false;
    if (g == nullptr) {
        g = new (std::nothrow) omg_graph();
        if (g == nullptr) return OMG_ENOMEM;
        g->ctx = ctx;
        fresh = true;
    } else if (g->ctx != ctx || g == graph) {
        return OMG_ESTATE;
    }
    const int rc = omg_cgp_partition_impl(ctx, graph, node_part, n_part, p, g);
    if (rc != OMG_OK) {
        if (fresh) omg_graph_destroy(g);
        return rc;
    }
    *part_graph = g;
    return OMG_OK;
}

int omg_cgp_local_aggregate(omg_ctx* ctx, const omg_graph* part_graph, int is_last, const omg_table* table_prev,
                            const float* buf_prev, int64_t ld_prev, const omg_layer* layer, const float* row_mean,
                            int64_t ld_mean, float* wire, int64_t ld_wire) {
    if (ctx == nullptr || part_graph == nullptr || layer == nullptr || wire == nullptr) return OMG_EINVAL;
    OMG_TRY(check_layer(layer));
    if (ld_wire < wire_width(layer) || ld_wire % 4 != 0 || !aligned16(wire)) return OMG_EINVAL;
    if (row_mean != nullptr) {
        if (layer->model != OMG_SAGE_MEAN || layer->aggregator != OMG_AGG_MOMENT) return OMG_EINVAL;
        if (ld_mean < round_up(layer->d_in, 8) || ld_mean % 4 != 0 || !aligned16(row_mean)) return OMG_EINVAL;
    }
    const LocalOut lo{wire, ld_wire, row_mean, ld_mean};
    return run_layer(ctx, part_graph, is_last, table_prev, buf_prev, ld_prev, layer, nullptr, 0, nullptr, 0, &lo);
}

static int check_wire(const omg_layer* L, int64_t n_rows, int32_t n_part, const float* wire, int64_t ld_wire) {
    OMG_TRY(check_layer(L));
    if (n_rows < 0 || n_part < 1 || n_part > OMG_CGP_MAX_PARTS) return OMG_EINVAL;
    if (n_rows > 0 && (wire == nullptr || ld_wire < wire_width(L) || ld_wire % 4 != 0 || !aligned16(wire))) return OMG_EINVAL;
    return OMG_OK;
}

int omg_cgp_merge_mean(omg_ctx* ctx, int64_t n_rows, int32_t n_part, const float* wire, int64_t ld_wire,
                       const omg_layer* layer, float* row_mean, int64_t ld_mean) {
    if (ctx == nullptr || layer == nullptr || (row_mean == nullptr && n_rows > 0)) return OMG_EINVAL;
    OMG_TRY(check_wire(layer, n_rows, n_part, wire, ld_wire));
    if (layer->model != OMG_SAGE_MEAN || layer->aggregator != OMG_AGG_MOMENT) return OMG_EINVAL;
    const int64_t agg_ld = round_up(layer->d_in, 8);
    if (ld_mean < agg_ld || ld_mean % 4 != 0 || !aligned16(row_mean)) return OMG_EINVAL;
    CgpMergeArgs m{};
    m.wire = wire; m.ld_wire = ld_wire; m.n_rows = n_rows; m.n_part = n_part;
    m.op = OMG_OP_MEAN; m.dim = layer->d_in; m.agg_ld = agg_ld; m.out = row_mean; m.out_ld = ld_mean;
    return omg_launch_cgp_merge(m, ctx->stream);
}

int omg_cgp_merge_update(omg_ctx* ctx, int64_t n_rows, int32_t n_part, const float* wire, int64_t ld_wire,
                         const omg_layer* layer, const float* buf_prev, int64_t ld_prev, float* buf_out, int64_t ld_out) {
    if (ctx == nullptr || layer == nullptr || (n_rows > 0 && (buf_prev == nullptr || buf_out == nullptr))) return OMG_EINVAL;
    OMG_TRY(check_wire(layer, n_rows, n_part, wire, ld_wire));
    const omg_layer* L = layer;
    const int d_in = L->d_in;
    if (n_rows == 0) return OMG_OK;
    if (ld_prev < d_in || ld_prev % 4 != 0 || !aligned16(buf_prev) || ld_out < layer_out_width(L)) return OMG_EINVAL;
    if (L->model == OMG_GCNII && (L->init_rows == nullptr || L->init_ld < d_in || L->init_ld % 4 != 0 || !aligned16(L->init_rows)))
        return OMG_EINVAL;
    const int64_t agg_ld = round_up(d_in, 8);
    const int H = L->model == OMG_GAT ? L->heads : 1;
    OMG_TRY(ctx->agg.ensure(sizeof(float) * (size_t)(n_rows * H * agg_ld)));
    CgpMergeArgs m{};
    m.wire = wire; m.ld_wire = ld_wire; m.n_rows = n_rows; m.n_part = n_part;
    m.dim = d_in; m.agg_ld = agg_ld; m.out = ctx->agg.as<float>(); m.out_ld = agg_ld; m.agg_p = L->agg_p;
    if (L->model == OMG_GAT) {
        m.heads = H;
    } else if (L->model == OMG_SAGE_MEAN) {
        static const int op_of[] = {OMG_OP_MEAN, OMG_OP_SUM, OMG_OP_MAX, OMG_OP_POW, OMG_OP_MOM};
        m.op = op_of[L->aggregator];
    } else {
        m.op = OMG_OP_GCN;
        m.self = buf_prev; m.self_ld = ld_prev;
        if (L->model == OMG_GCNII) { m.h0 = L->init_rows; m.h0_ld = L->init_ld; m.alpha = L->alpha; }
    }
    OMG_TRY(omg_launch_cgp_merge(m, ctx->stream));
    float* split = nullptr;
    if (n_rows <= 128 * 64) {
        OMG_TRY(ctx->gemmSplit.ensure(OMG_GEMM_SPLIT_BYTES));
        split = ctx->gemmSplit.as<float>();
    }
    return launch_layer_update(ctx, L, n_rows, ctx->agg.as<float>(), agg_ld, buf_prev, ld_prev, buf_out, ld_out, split,
                               OMG_GEMM_SPLIT_BYTES / sizeof(float));
}

int omg_last_graph_sizes(const omg_ctx* ctx, int64_t sizes[4]) {
    if (ctx == nullptr || ctx->serve_graph == nullptr) return OMG_ESTATE;
    return omg_graph_sizes(ctx->serve_graph, sizes);
}

}  // extern "C"
