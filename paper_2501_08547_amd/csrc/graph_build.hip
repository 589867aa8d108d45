// Computation-graph construction for one batch, on the device, in integers only.
//
// Steps (paper passages): candidates = distinct training endpoints of the request's edges
// and the number of query edges at each (Sec. 5.2.1); recompute targets = the best
// floor(gamma |R|) candidates by query-edge ratio (Sec. 5.2.2, budget of Eq. 2); rows of the
// inner layers = queries and targets, each target row holding every edge that ends at it,
// from the base graph and from the request (Sec. 6.1).  The output is the canonical tagged
// CSR described in omega_srpe.h plus a work list that cuts long rows into parts.
//
// Everything up to the sizes of the result runs without host involvement; one copy brings
// the counters back, then the column arrays are filled.
#include "internal.h"

#include <cstring>
#include <rocprim/rocprim.hpp>

namespace {

constexpr int TPB = 256;

inline unsigned grid_for(int64_t n) { return (unsigned)((n + TPB - 1) / TPB); }

__device__ inline int64_t gtid() { return (int64_t)blockIdx.x * blockDim.x + threadIdx.x; }

__device__ inline int64_t base_deg(const int64_t* __restrict__ indptr, int32_t u) {
    return indptr[(int64_t)u + 1] - indptr[u];
}

// ---- a0: sort keys -------------------------------------------------------------------------
// Keys are packed as narrowly as the batch allows: (node << bits(query)) | query and
// (query << bits(node)) | node, in 32 bits when both fit and 64 otherwise, so that the radix
// sorts only walk the bits that carry information.
template <typename K>
__global__ void k_make_keys(const int32_t* __restrict__ qe_query, const int32_t* __restrict__ qe_node,
                            int64_t n_e, int32_t n_query, int64_t n_nodes, int sq, int sn,
                            K* __restrict__ key_nq, K* __restrict__ key_qn, BuildCounts* c) {
    int64_t i = gtid();
    if (i >= n_e) return;
    int32_t q = qe_query[i], u = qe_node[i];
    if (q < 0 || q >= n_query || u < 0 || (int64_t)u >= n_nodes) {
        atomicOr(&c->err, 1);
        q = 0;      // keep every later access in bounds; the build is rejected after the read-back
        u = 0;
    }
    key_nq[i] = ((K)(uint32_t)u << sq) | (K)(uint32_t)q;   // by node, then query
    key_qn[i] = ((K)(uint32_t)q << sn) | (K)(uint32_t)u;   // by query, then node
}

template <typename K>
__global__ void k_heads(const K* __restrict__ key_nq, int64_t n_e, int sq, int32_t* __restrict__ head) {
    int64_t i = gtid();
    if (i >= n_e) return;
    head[i] = (i == 0 || (key_nq[i] >> sq) != (key_nq[i - 1] >> sq)) ? 1 : 0;
}

// candidates R (ascending node id), first edge of each in the node-sorted list, node -> slot
template <typename K>
__global__ void k_candidates(const K* __restrict__ key_nq, const int32_t* __restrict__ head,
                             const int32_t* __restrict__ ridx, int64_t n_e, int sq, int32_t* __restrict__ cand,
                             int32_t* __restrict__ cand_start, int32_t* __restrict__ node_slot, BuildCounts* c) {
    int64_t i = gtid();
    if (i >= n_e) return;
    if (head[i]) {
        int32_t r = ridx[i];
        int32_t u = (int32_t)(key_nq[i] >> sq);
        cand[r] = u;
        cand_start[r] = (int32_t)i;
        node_slot[u] = r;
    }
    if (i == n_e - 1) {
        int32_t n = ridx[i] + head[i];
        c->n_cand = n;
        cand_start[n] = (int32_t)n_e;
    }
}

// ---- a1: ranking key -----------------------------------------------------------------------
// floor(2^64 a / (a + b)) for 1 <= a, a + b < 2^32: two different ratios with denominators below
// 2^32 differ by more than 2^-64, so this 64-bit key orders them exactly; b == 0 (ratio 1) maps
// to the all-ones key, above every other value.
__device__ inline uint64_t ratio_key(uint64_t a, uint64_t b) {
    if (b == 0) return ~0ull;
    uint64_t d = a + b;
    uint64_t hi = (a << 32) / d;
    uint64_t rem = (a << 32) - hi * d;
    uint64_t lo = (rem << 32) / d;
    return (hi << 32) | lo;
}

__global__ void k_score(const int32_t* __restrict__ cand, const int32_t* __restrict__ cand_start,
                        const int64_t* __restrict__ base_indptr, int64_t n_e, const BuildCounts* c,
                        int32_t* __restrict__ qdeg, uint64_t* __restrict__ skey, int32_t* __restrict__ sval,
                        int32_t* __restrict__ in_t) {
    int64_t r = gtid();
    if (r >= n_e) return;
    uint64_t key = 0;                         // padding entries rank last (a real key is never 0)
    if (r < c->n_cand) {
        int32_t a = cand_start[r + 1] - cand_start[r];
        qdeg[r] = a;
        key = ratio_key((uint64_t)a, (uint64_t)base_deg(base_indptr, cand[r]));
    }
    skey[r] = key;
    sval[r] = (int32_t)r;
    in_t[r] = 0;
}

__global__ void k_mark_top(const int32_t* __restrict__ sval_sorted, int64_t n_e, uint32_t gamma_ppm,
                           const BuildCounts* c, int32_t* __restrict__ in_t) {
    int64_t i = gtid();
    if (i >= n_e) return;
    int64_t take = (int64_t)(((uint64_t)gamma_ppm * (uint64_t)c->n_cand) / 1000000ull);
    if (i < take) in_t[sval_sorted[i]] = 1;
}

__global__ void k_mark_given(const int32_t* __restrict__ rset, int64_t n_rset, int64_t n_nodes,
                             const int32_t* __restrict__ node_slot, int32_t* __restrict__ in_t, BuildCounts* c) {
    int64_t t = gtid();
    if (t >= n_rset) return;
    int32_t u = rset[t];
    bool ok = u >= 0 && (int64_t)u < n_nodes && (t == 0 || rset[t - 1] < u);
    int32_t r = ok ? node_slot[u] : -1;
    if (r < 0) atomicOr(&c->err, 2);
    else in_t[r] = 1;
}

__global__ void k_targets(const int32_t* __restrict__ cand, const int32_t* __restrict__ in_t,
                          const int32_t* __restrict__ trow, int32_t n_query, BuildCounts* c,
                          int32_t* __restrict__ targets, int32_t* __restrict__ target_slot,
                          int32_t* __restrict__ cand_row) {
    int64_t r = gtid();
    int64_t n = c->n_cand;
    if (r >= n) return;
    if (in_t[r]) {
        int32_t t = trow[r];
        targets[t] = cand[r];
        target_slot[t] = (int32_t)r;
        cand_row[r] = n_query + t;
    } else {
        cand_row[r] = -1;
    }
    if (r == n - 1) c->n_target = trow[r] + in_t[r];
}

// ---- a2: row pointers ----------------------------------------------------------------------
__global__ void k_target_len(const int32_t* __restrict__ targets, const int32_t* __restrict__ target_slot,
                             const int32_t* __restrict__ qdeg, const int64_t* __restrict__ base_indptr,
                             int64_t n_slots, const BuildCounts* c, int64_t* __restrict__ len) {
    int64_t t = gtid();
    if (t >= n_slots) return;
    len[t] = (t < c->n_target) ? base_deg(base_indptr, targets[t]) + qdeg[target_slot[t]] : 0;
}

template <typename K>
__global__ void k_indptr(const K* __restrict__ key_qn, int64_t n_e, int32_t n_query, int sn,
                         const int64_t* __restrict__ toff, BuildCounts* c, int64_t* __restrict__ indptr) {
    int64_t i = gtid();
    int64_t n_t = c->n_target;
    if (i <= n_query) {                       // query rows: first edge with query index >= i
        int64_t lo = 0, hi = n_e;              // compare query indices, not shifted keys: i << sn may not fit K
        while (lo < hi) {
            int64_t mid = (lo + hi) >> 1;
            if ((int64_t)(key_qn[mid] >> sn) < i) lo = mid + 1; else hi = mid;
        }
        indptr[i] = lo;
    }
    if (i >= 1 && i <= n_t) indptr[n_query + i] = n_e + toff[i];
    if (i == 0) c->nnz_in = n_e + toff[n_t];
}

__global__ void k_row_parts(const int64_t* __restrict__ indptr, int32_t n_query, int64_t n_slots,
                            const BuildCounts* c, int32_t* __restrict__ nparts, int32_t* __restrict__ is_split) {
    int64_t v = gtid();
    if (v >= n_slots) return;
    int64_t rows_in = n_query + c->n_target;
    int32_t np = 0;
    if (v < rows_in) {
        int64_t len = indptr[v + 1] - indptr[v];
        np = (int32_t)((len + OMG_PART_EDGES - 1) / OMG_PART_EDGES);
        if (np < 1) np = 1;
    }
    nparts[v] = np;
    is_split[v] = np > 1 ? 1 : 0;
}

__global__ void k_final_counts(const int32_t* __restrict__ part_ptr, const int32_t* __restrict__ split_idx,
                               int32_t n_query, BuildCounts* c) {
    int64_t rows_in = n_query + c->n_target;
    c->n_parts = part_ptr[rows_in];
    c->n_parts_last = part_ptr[n_query];
    c->n_split = split_idx[rows_in];
    c->n_split_last = split_idx[n_query];
}

// ---- a2: columns, tags, source degrees -----------------------------------------------------
template <typename K>
__global__ void k_fill_cols(const K* __restrict__ key_qn, const K* __restrict__ key_nq, int sq, int sn,
                            const int64_t* __restrict__ indptr, const int32_t* __restrict__ targets,
                            const int32_t* __restrict__ target_slot, const int32_t* __restrict__ cand_start,
                            const int32_t* __restrict__ qdeg, const int32_t* __restrict__ cand_row,
                            const int32_t* __restrict__ node_slot, const int64_t* __restrict__ base_indptr,
                            const int32_t* __restrict__ base_indices, int64_t n_e, int32_t n_query,
                            int64_t n_target, int64_t nnz_in, int32_t* __restrict__ cols,
                            int32_t* __restrict__ cdeg) {
    int64_t p = gtid();
    if (p >= nnz_in) return;
    int32_t src;                 // training node that is the source, or -1 for a query source
    int32_t q_src = 0;
    if (p < n_e) {
        src = (int32_t)(key_qn[p] & (((K)1 << sn) - 1));
    } else {
        int64_t lo = 0, hi = n_target;            // last target row whose start is <= p
        const int64_t* tp = indptr + n_query;
        while (hi - lo > 1) {
            int64_t mid = (lo + hi) >> 1;
            if (tp[mid] <= p) lo = mid; else hi = mid;
        }
        int64_t j = p - tp[lo];
        int32_t u = targets[lo];
        int64_t b0 = base_indptr[u], dg = base_indptr[(int64_t)u + 1] - b0;
        if (j < dg) {
            src = base_indices[b0 + j];
        } else {
            src = -1;
            q_src = (int32_t)(key_nq[cand_start[target_slot[lo]] + (j - dg)] & (((K)1 << sq) - 1));
        }
    }
    if (src >= 0) {
        int32_t r = node_slot[src];
        int32_t row = r >= 0 ? cand_row[r] : -1;
        cols[p] = row >= 0 ? ~row : src;
        cdeg[p] = (int32_t)base_deg(base_indptr, src) + (r >= 0 ? qdeg[r] : 0);
    } else {
        cols[p] = ~q_src;
        cdeg[p] = (int32_t)(indptr[q_src + 1] - indptr[q_src]);
    }
}

__global__ void k_fill_parts(const int32_t* __restrict__ part_ptr, int64_t rows_in, int64_t n_parts,
                             int32_t* __restrict__ part_row) {
    int64_t j = gtid();
    if (j >= n_parts) return;
    int64_t lo = 0, hi = rows_in;                 // last row whose first part is <= j
    while (hi - lo > 1) {
        int64_t mid = (lo + hi) >> 1;
        if (part_ptr[mid] <= j) lo = mid; else hi = mid;
    }
    part_row[j] = (int32_t)lo;
}

__global__ void k_fill_split(const int32_t* __restrict__ is_split, const int32_t* __restrict__ split_idx,
                             int64_t rows_in, int32_t* __restrict__ split_rows) {
    int64_t v = gtid();
    if (v >= rows_in) return;
    if (is_split[v]) split_rows[split_idx[v]] = (int32_t)v;
}

__global__ void k_clear_slots(const int32_t* __restrict__ cand, const BuildCounts* c, int64_t n_e,
                              int32_t* __restrict__ node_slot) {
    int64_t r = gtid();
    if (r >= n_e || r >= c->n_cand) return;
    node_slot[cand[r]] = -1;
}

__global__ void k_check_indptr(const int64_t* __restrict__ indptr, int64_t n, BuildCounts* c) {
    int64_t i = gtid();
    if (i >= n) return;
    const int64_t a = indptr[i], b = indptr[i + 1];
    if ((i == 0 && a != 0) || b < a || b - a >= ((int64_t)1 << 31)) atomicOr(&c->err, 1);
    else atomicMax((unsigned long long*)&c->n_parts, (unsigned long long)(b - a));   // largest degree
    if (i == n - 1) c->nnz_in = b;
}

__global__ void k_check_indices(const int32_t* __restrict__ indices, int64_t nnz, int64_t n, int64_t per_thread,
                                BuildCounts* c) {
    const int64_t t = gtid();
    bool bad = false;
    for (int64_t j = 0; j < per_thread; ++j) {          // strided so that a wavefront reads consecutive entries
        const int64_t e = (t / 64) * 64 * per_thread + j * 64 + (t % 64);
        if (e < nnz) {
            const int32_t u = indices[e];
            bad |= (u < 0 || (int64_t)u >= n);
        }
    }
    if (bad) atomicOr(&c->err, 1);
}

__global__ void k_fill_i32(int32_t* p, int64_t n, int32_t v) {
    int64_t i = gtid();
    if (i < n) p[i] = v;
}

template <typename In, typename Out>
size_t scan_bytes(int64_t n) {
    size_t bytes = 0;
    (void)rocprim::exclusive_scan(nullptr, bytes, (const In*)nullptr, (Out*)nullptr, Out(0), (size_t)n,
                                  rocprim::plus<Out>(), (hipStream_t) nullptr);
    return bytes;
}

// exclusive prefix sum; `tmp` must already hold scan_bytes<In, Out>(n) bytes
template <typename In, typename Out>
int scan_excl(const DevBuf& tmp, const In* in, Out* out, int64_t n, hipStream_t s) {
    size_t bytes = tmp.cap;
    OMG_HIP(rocprim::exclusive_scan(tmp.p, bytes, in, out, Out(0), (size_t)n, rocprim::plus<Out>(), s));
    return OMG_OK;
}

int bits_for(uint64_t max_value) {
    int b = 1;
    while (b < 64 && (max_value >> b) != 0) ++b;
    return b;
}

}  // namespace

int omg_fill_node_slot(omg_ctx* ctx) {
    hipLaunchKernelGGL(k_fill_i32, dim3(grid_for(ctx->base.n_nodes)), dim3(TPB), 0, ctx->stream,
                       ctx->node_slot, ctx->base.n_nodes, -1);
    OMG_HIP(hipGetLastError());
    return OMG_OK;
}

// One pass over the training graph when a context is created: row pointers start at zero and never
// decrease, every degree fits 31 bits, every neighbour id is a node.  The kernels rely on this.
int omg_validate_base(omg_ctx* ctx) {
    hipStream_t s = ctx->stream;
    const int64_t n = ctx->base.n_nodes;
    OMG_HIP(hipMemsetAsync(ctx->counts_dev, 0, sizeof(BuildCounts), s));
    hipLaunchKernelGGL(k_check_indptr, dim3(grid_for(n)), dim3(TPB), 0, s, ctx->base.indptr, n, ctx->counts_dev);
    OMG_HIP(hipMemcpyAsync(ctx->counts_host, ctx->counts_dev, sizeof(BuildCounts), hipMemcpyDeviceToHost, s));
    OMG_HIP(hipStreamSynchronize(s));
    if (ctx->counts_host->err != 0) return OMG_EINVAL;
    const int64_t nnz = ctx->counts_host->nnz_in;
    ctx->max_base_deg = ctx->counts_host->n_parts;
    if (nnz > 0) {
        if (ctx->base.indices == nullptr) return OMG_EINVAL;
        const int64_t per_thread = 16;
        hipLaunchKernelGGL(k_check_indices, dim3(grid_for((nnz + per_thread - 1) / per_thread)), dim3(TPB), 0, s,
                           ctx->base.indices, nnz, n, per_thread, ctx->counts_dev);
        OMG_HIP(hipMemcpyAsync(ctx->counts_host, ctx->counts_dev, sizeof(BuildCounts), hipMemcpyDeviceToHost, s));
        OMG_HIP(hipStreamSynchronize(s));
        if (ctx->counts_host->err != 0) return OMG_ERANGE;
    }
    return OMG_OK;
}

namespace {

// rocPRIM switches to a merge sort below a million items, which costs two launches per doubling
// of the run length; the batches here are launch-bound, so ask for the one-sweep radix sort.
using SortCfg = rocprim::radix_sort_config<rocprim::default_config, rocprim::default_config,
                                           rocprim::default_config, 0>;

template <typename K>
int build_impl(omg_ctx* ctx, omg_graph* g, int32_t n_query, int64_t n_e, const int32_t* qe_query,
               const omg_node_t* qe_node, uint32_t gamma_ppm, const omg_node_t* rset, int64_t n_rset) {
    hipStream_t s = ctx->stream;
    const int64_t n_nodes = ctx->base.n_nodes;
    const int64_t n_slots = (int64_t)n_query + n_e + 2;     // upper bound of rows_in + 1, plus one
    const int bn = bits_for((uint64_t)n_nodes - 1);
    const int bq = bits_for((uint64_t)(n_query > 0 ? n_query - 1 : 0));
    const int key_bits = bn + bq;
    // Selection keys are 64-bit fixed-point ratios.  Every ratio has a denominator below
    // 2^m (m from the largest base degree plus the number of request edges), so the top 2m
    // bits already order them exactly and the sort can skip the rest.
    const int m_bits = bits_for((uint64_t)ctx->max_base_deg + (uint64_t)n_e);
    const unsigned sel_begin = 2 * m_bits >= 64 ? 0u : (unsigned)(64 - 2 * m_bits);
    g->built = false;
    g->n_query = n_query;
    g->n_qedges = n_e;

    // ---- every allocation that does not depend on the batch's content, before any launch
    const size_t ne = (size_t)n_e, ns = (size_t)n_slots;
    OMG_TRY(g->indptr.ensure(sizeof(int64_t) * ns));
    OMG_TRY(g->part_ptr.ensure(sizeof(int32_t) * ns));
    OMG_TRY(g->cand.ensure(sizeof(int32_t) * (ne + 1)));
    OMG_TRY(g->qdeg.ensure(sizeof(int32_t) * (ne + 1)));
    OMG_TRY(g->cand_row.ensure(sizeof(int32_t) * (ne + 1)));
    OMG_TRY(g->targets.ensure(sizeof(int32_t) * (ne + 1)));
    OMG_TRY(g->target_slot.ensure(sizeof(int32_t) * (ne + 1)));
    OMG_TRY(ctx->keyRaw.ensure(sizeof(K) * (2 * ne + 1)));
    OMG_TRY(ctx->keyNQ.ensure(sizeof(K) * (ne + 1)));
    OMG_TRY(ctx->keyQN.ensure(sizeof(K) * (ne + 1)));
    OMG_TRY(ctx->head.ensure(sizeof(int32_t) * (ne + 1)));
    OMG_TRY(ctx->ridx.ensure(sizeof(int32_t) * (ne + 1)));
    OMG_TRY(ctx->candStart.ensure(sizeof(int32_t) * (ne + 2)));
    OMG_TRY(ctx->skey.ensure(sizeof(uint64_t) * (ne + 1)));
    OMG_TRY(ctx->skeySorted.ensure(sizeof(uint64_t) * (ne + 1)));
    OMG_TRY(ctx->sval.ensure(sizeof(int32_t) * (ne + 1)));
    OMG_TRY(ctx->svalSorted.ensure(sizeof(int32_t) * (ne + 1)));
    OMG_TRY(ctx->inT.ensure(sizeof(int32_t) * (ne + 1)));
    OMG_TRY(ctx->tRow.ensure(sizeof(int32_t) * (ne + 1)));
    OMG_TRY(ctx->tLen.ensure(sizeof(int64_t) * (ne + 2)));
    OMG_TRY(ctx->tOff.ensure(sizeof(int64_t) * (ne + 2)));
    OMG_TRY(ctx->nParts.ensure(sizeof(int32_t) * ns));
    OMG_TRY(ctx->isSplit.ensure(sizeof(int32_t) * ns));
    OMG_TRY(ctx->splitIdx.ensure(sizeof(int32_t) * ns));
    {
        size_t need = scan_bytes<int32_t, int32_t>(n_slots);
        size_t b = scan_bytes<int64_t, int64_t>(n_e + 2);
        need = b > need ? b : need;
        if (n_e > 0) {
            b = 0;
            (void)rocprim::radix_sort_keys<SortCfg>(nullptr, b, (const K*)nullptr, (K*)nullptr, ne, 0, key_bits,
                                                    (hipStream_t) nullptr);
            need = b > need ? b : need;
            b = 0;
            (void)rocprim::radix_sort_pairs_desc<SortCfg>(nullptr, b, (const uint64_t*)nullptr, (uint64_t*)nullptr,
                                                          (const int32_t*)nullptr, (int32_t*)nullptr, ne, sel_begin,
                                                          64, (hipStream_t) nullptr);
            need = b > need ? b : need;
        }
        OMG_TRY(ctx->primTmp.ensure(need + 256));
    }

    K* raw_nq = ctx->keyRaw.as<K>();
    K* raw_qn = raw_nq + n_e;
    K* key_nq = ctx->keyNQ.as<K>();
    K* key_qn = ctx->keyQN.as<K>();
    int32_t* head = ctx->head.as<int32_t>();
    int32_t* ridx = ctx->ridx.as<int32_t>();
    int32_t* cand_start = ctx->candStart.as<int32_t>();
    uint64_t* skey = ctx->skey.as<uint64_t>();
    uint64_t* skey_sorted = ctx->skeySorted.as<uint64_t>();
    int32_t* sval = ctx->sval.as<int32_t>();
    int32_t* sval_sorted = ctx->svalSorted.as<int32_t>();
    int32_t* in_t = ctx->inT.as<int32_t>();
    int32_t* trow = ctx->tRow.as<int32_t>();
    int64_t* tlen = ctx->tLen.as<int64_t>();
    int64_t* toff = ctx->tOff.as<int64_t>();
    int32_t* nparts = ctx->nParts.as<int32_t>();
    int32_t* is_split = ctx->isSplit.as<int32_t>();
    int32_t* split_idx = ctx->splitIdx.as<int32_t>();
    int32_t* cand = g->cand.as<int32_t>();
    int32_t* qdeg = g->qdeg.as<int32_t>();
    int32_t* cand_row = g->cand_row.as<int32_t>();
    int32_t* targets = g->targets.as<int32_t>();
    int32_t* target_slot = g->target_slot.as<int32_t>();
    int64_t* indptr = g->indptr.as<int64_t>();
    int32_t* part_ptr = g->part_ptr.as<int32_t>();
    BuildCounts* cd = ctx->counts_dev;
    const unsigned ge = grid_for(n_e > 0 ? n_e : 1);

    OMG_HIP(hipMemsetAsync(cd, 0, sizeof(BuildCounts), s));

    if (n_e > 0) {
        hipLaunchKernelGGL(k_make_keys<K>, dim3(ge), dim3(TPB), 0, s, qe_query, qe_node, n_e, n_query, n_nodes, bq, bn,
                           raw_nq, raw_qn, cd);
        size_t b = ctx->primTmp.cap;
        OMG_HIP(rocprim::radix_sort_keys<SortCfg>(ctx->primTmp.p, b, raw_nq, key_nq, ne, 0, key_bits, s));
        b = ctx->primTmp.cap;
        OMG_HIP(rocprim::radix_sort_keys<SortCfg>(ctx->primTmp.p, b, raw_qn, key_qn, ne, 0, key_bits, s));

        // candidates
        hipLaunchKernelGGL(k_heads<K>, dim3(ge), dim3(TPB), 0, s, key_nq, n_e, bq, head);
        OMG_TRY((scan_excl<int32_t, int32_t>(ctx->primTmp, head, ridx, n_e, s)));
        hipLaunchKernelGGL(k_candidates<K>, dim3(ge), dim3(TPB), 0, s, key_nq, head, ridx, n_e, bq, cand, cand_start,
                           ctx->node_slot, cd);

        // selection
        hipLaunchKernelGGL(k_score, dim3(ge), dim3(TPB), 0, s, cand, cand_start, ctx->base.indptr, n_e, cd, qdeg, skey,
                           sval, in_t);
        if (rset == nullptr) {
            if (gamma_ppm > 0) {
                b = ctx->primTmp.cap;
                OMG_HIP(rocprim::radix_sort_pairs_desc<SortCfg>(ctx->primTmp.p, b, skey, skey_sorted, sval, sval_sorted,
                                                                ne, sel_begin, 64, s));
                hipLaunchKernelGGL(k_mark_top, dim3(ge), dim3(TPB), 0, s, sval_sorted, n_e, gamma_ppm, cd, in_t);
            }
        } else if (n_rset > 0) {
            hipLaunchKernelGGL(k_mark_given, dim3(grid_for(n_rset)), dim3(TPB), 0, s, rset, n_rset, n_nodes,
                               ctx->node_slot, in_t, cd);
        }
        OMG_TRY((scan_excl<int32_t, int32_t>(ctx->primTmp, in_t, trow, n_e, s)));
        hipLaunchKernelGGL(k_targets, dim3(ge), dim3(TPB), 0, s, cand, in_t, trow, n_query, cd, targets, target_slot,
                           cand_row);

        // row pointers
        hipLaunchKernelGGL(k_target_len, dim3(grid_for(n_e + 1)), dim3(TPB), 0, s, targets, target_slot, qdeg,
                           ctx->base.indptr, n_e + 1, cd, tlen);
        OMG_TRY((scan_excl<int64_t, int64_t>(ctx->primTmp, tlen, toff, n_e + 1, s)));
        hipLaunchKernelGGL(k_indptr<K>, dim3(grid_for(n_slots)), dim3(TPB), 0, s, key_qn, n_e, n_query, bn, toff, cd,
                           indptr);
    } else {
        OMG_HIP(hipMemsetAsync(indptr, 0, sizeof(int64_t) * (size_t)(n_query + 1), s));
    }

    // work list: parts per row (an empty row still gets one part so that its output is written)
    hipLaunchKernelGGL(k_row_parts, dim3(grid_for(n_slots)), dim3(TPB), 0, s, indptr, n_query, n_slots, cd, nparts,
                       is_split);
    OMG_TRY((scan_excl<int32_t, int32_t>(ctx->primTmp, nparts, part_ptr, n_slots, s)));
    OMG_TRY((scan_excl<int32_t, int32_t>(ctx->primTmp, is_split, split_idx, n_slots, s)));
    hipLaunchKernelGGL(k_final_counts, dim3(1), dim3(1), 0, s, part_ptr, split_idx, n_query, cd);
    OMG_HIP(hipGetLastError());

    OMG_HIP(hipMemcpyAsync(ctx->counts_host, cd, sizeof(BuildCounts), hipMemcpyDeviceToHost, s));
    OMG_HIP(hipStreamSynchronize(s));
    g->c = *ctx->counts_host;
    g->rows_in = n_query + g->c.n_target;

    if (g->c.err != 0) {
        if (n_e > 0) hipLaunchKernelGGL(k_clear_slots, dim3(ge), dim3(TPB), 0, s, cand, cd, n_e, ctx->node_slot);
        OMG_HIP(hipStreamSynchronize(s));
        return OMG_ERANGE;
    }

    // ---- columns and work list, now that their sizes are known
    OMG_TRY(g->cols.ensure(sizeof(int32_t) * (size_t)(g->c.nnz_in + 1)));
    OMG_TRY(g->cdeg.ensure(sizeof(int32_t) * (size_t)(g->c.nnz_in + 1)));
    OMG_TRY(g->part_row.ensure(sizeof(int32_t) * (size_t)(g->c.n_parts + 1)));
    OMG_TRY(g->split_rows.ensure(sizeof(int32_t) * (size_t)(g->c.n_split + 1)));
    if (g->c.nnz_in > 0)
        hipLaunchKernelGGL(k_fill_cols<K>, dim3(grid_for(g->c.nnz_in)), dim3(TPB), 0, s, key_qn, key_nq, bq, bn, indptr, targets,
                           target_slot, cand_start, qdeg, cand_row, ctx->node_slot, ctx->base.indptr,
                           ctx->base.indices, n_e, n_query, g->c.n_target, g->c.nnz_in, g->cols.as<int32_t>(),
                           g->cdeg.as<int32_t>());
    if (g->c.n_parts > 0)
        hipLaunchKernelGGL(k_fill_parts, dim3(grid_for(g->c.n_parts)), dim3(TPB), 0, s, part_ptr, g->rows_in,
                           g->c.n_parts, g->part_row.as<int32_t>());
    if (g->c.n_split > 0)
        hipLaunchKernelGGL(k_fill_split, dim3(grid_for(g->rows_in)), dim3(TPB), 0, s, is_split, split_idx, g->rows_in,
                           g->split_rows.as<int32_t>());
    if (n_e > 0) hipLaunchKernelGGL(k_clear_slots, dim3(ge), dim3(TPB), 0, s, cand, cd, n_e, ctx->node_slot);
    OMG_HIP(hipGetLastError());
    g->built = true;
    return OMG_OK;
}

}  // namespace

int omg_build_impl(omg_ctx* ctx, omg_graph* g, int32_t n_query, int64_t n_e, const int32_t* qe_query,
                   const omg_node_t* qe_node, uint32_t gamma_ppm, const omg_node_t* rset, int64_t n_rset) {
    const int bn = bits_for((uint64_t)ctx->base.n_nodes - 1);
    const int bq = bits_for((uint64_t)(n_query > 0 ? n_query - 1 : 0));
    if (bn + bq <= 32) return build_impl<uint32_t>(ctx, g, n_query, n_e, qe_query, qe_node, gamma_ppm, rset, n_rset);
    return build_impl<uint64_t>(ctx, g, n_query, n_e, qe_query, qe_node, gamma_ppm, rset, n_rset);
}
