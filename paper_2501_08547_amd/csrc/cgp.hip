// Computation graph parallelism (Sec. 6) as far as one GPU shows it: the share of a batch's computation
// graph that one partition executes (its rows restricted to the edges whose source the partition holds,
// Sec. 6.1), and the merge functions that turn the partitions' local aggregations of a destination into
// the aggregation over its whole neighbourhood (Eq. 3, Sec. 6.2).  The local aggregation itself is the
// ordinary gather run on the partition's graph with unfinished ("raw") rows; between it and the merge
// sits, on several GPUs, one all-to-all, which is not part of this library.
#include "internal.h"

#include <math.h>

namespace {

constexpr int TPB = 256;

struct PartCounts {
    long long nnz, n_parts, n_parts_last, n_split, n_split_last, n_split_big, n_split_big_last, bad;
};

inline unsigned grid_for(int64_t n, int64_t per_block = TPB) {
    const int64_t g = (n + per_block - 1) / per_block;
    return (unsigned)(g > 0 ? g : 1);
}

// Partition of an edge = partition of its source (Sec. 6.1).  A stored row belongs to its node's partition; a
// freshly computed row to the partition that computed it: query q to q mod P (queries are dealt out
// evenly), a recompute target to its node's partition.
__device__ inline int edge_partition(int32_t c, const int32_t* __restrict__ node_part,
                                     const int32_t* __restrict__ targets, int n_query, int n_part) {
    if (c >= 0) return node_part[c];
    const int r = ~c;
    return r < n_query ? r % n_part : node_part[targets[r - n_query]];
}

__global__ void k_cgp_check(const int32_t* __restrict__ node_part, int64_t n, int n_part, PartCounts* c) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n && (node_part[i] < 0 || node_part[i] >= n_part)) c->bad = 1;      // same value from every writer
}

// Edges of work item j of the whole graph (a row's run of at most part_edges edges).
__device__ inline void part_range(const int64_t* __restrict__ indptr, const int32_t* __restrict__ part_ptr,
                                  const int32_t* __restrict__ part_row, int64_t j, int part_edges, int& v, int64_t& e0,
                                  int64_t& e1) {
    v = part_row[j];
    const int64_t end = indptr[v + 1];
    e0 = indptr[v] + (int64_t)(j - part_ptr[v]) * part_edges;
    e1 = e0 + part_edges < end ? e0 + part_edges : end;
}

// one wavefront per work item of the whole graph: how many of its edges partition p holds.  Work items are
// numbered row by row and edge run by edge run, so a prefix sum over these counts is at once the position of
// every kept edge in the partition's edge list and, read at the rows' first work items, its row pointers.
__global__ __launch_bounds__(TPB) void k_cgp_count(const int64_t* __restrict__ indptr, const int32_t* __restrict__ cols,
                                                   const int32_t* __restrict__ part_ptr,
                                                   const int32_t* __restrict__ part_row, int64_t n_parts, int part_edges,
                                                   const int32_t* __restrict__ node_part,
                                                   const int32_t* __restrict__ targets, int n_query, int n_part, int p,
                                                   int32_t* __restrict__ kept) {
    const int64_t j = ((int64_t)blockIdx.x * TPB + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (j >= n_parts) return;                                  // a whole wavefront at a time
    int v;
    int64_t e0, e1;
    part_range(indptr, part_ptr, part_row, j, part_edges, v, e0, e1);
    int cnt = 0;
    for (int64_t e = e0 + lane; e < e1; e += 64)
        cnt += edge_partition(cols[e], node_part, targets, n_query, n_part) == p ? 1 : 0;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off);
    if (lane == 0) kept[j] = cnt;
}

// exclusive prefix sum of n ints by one block (the total must stay below 2^31), out[n] = the total; *mark
// receives out[mark_at].  16 items per
// thread and round, sums inside a round in 32 bits (a round holds 16 k counts of at most part_edges each), the
// running total in 64.
__global__ __launch_bounds__(1024) void k_cgp_scan(const int32_t* __restrict__ in, int64_t n, int32_t* __restrict__ out,
                                                   int64_t mark_at, long long* mark, long long* total) {
    __shared__ int wave_tot[16];
    constexpr int ITEMS = 16;
    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
    long long carry = 0;                                       // every thread keeps its own copy
    for (int64_t base = 0; base < n; base += 1024 * ITEMS) {
        const int64_t i0 = base + (int64_t)threadIdx.x * ITEMS;
        int v[ITEMS];
        if (i0 + ITEMS <= n && (reinterpret_cast<uintptr_t>(in + i0) & 15u) == 0) {
#pragma unroll
            for (int k = 0; k < ITEMS; k += 4) {
                const int4 q = *reinterpret_cast<const int4*>(in + i0 + k);
                v[k] = q.x; v[k + 1] = q.y; v[k + 2] = q.z; v[k + 3] = q.w;
            }
        } else {
#pragma unroll
            for (int k = 0; k < ITEMS; ++k) v[k] = i0 + k < n ? in[i0 + k] : 0;
        }
        int sum = 0;
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) sum += v[k];
        int x = sum;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int y = __shfl_up(x, off);
            if (lane >= off) x += y;
        }
        if (lane == 63) wave_tot[wid] = x;
        __syncthreads();
        int before = 0, all = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int t = wave_tot[w];
            if (w < wid) before += t;
            all += t;
        }
        long long run = carry + before + x - sum;
        if (mark != nullptr && mark_at >= i0 && mark_at < i0 + ITEMS && mark_at < n) {
            long long r = run;
            for (int k = 0; k < (int)(mark_at - i0); ++k) r += v[k];
            *mark = r;
        }
        if (i0 + ITEMS <= n && (reinterpret_cast<uintptr_t>(out + i0) & 15u) == 0) {
            int o[ITEMS];
#pragma unroll
            for (int k = 0; k < ITEMS; ++k) {
                o[k] = (int)run;
                run += v[k];
            }
#pragma unroll
            for (int k = 0; k < ITEMS; k += 4)
                *reinterpret_cast<int4*>(out + i0 + k) = make_int4(o[k], o[k + 1], o[k + 2], o[k + 3]);
        } else {
#pragma unroll
            for (int k = 0; k < ITEMS; ++k) {
                if (i0 + k < n) out[i0 + k] = (int32_t)run;
                run += v[k];
            }
        }
        carry += all;
        __syncthreads();                                       // wave_tot is rewritten in the next round
    }
    if (threadIdx.x == 0) {
        out[n] = (int32_t)carry;
        *total = carry;
        if (mark != nullptr && mark_at >= n) *mark = carry;
    }
}

// per row: its pointer into the partition's edge list and the number of work items its kept edges make
__global__ void k_cgp_rows(const int32_t* __restrict__ part_ptr, const int32_t* __restrict__ kept_off, int64_t rows,
                           int part_edges, int64_t* __restrict__ indptr_p, int32_t* __restrict__ nparts) {
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v > rows) return;
    if (v == rows) {
        indptr_p[rows] = kept_off[part_ptr[rows]];
        return;
    }
    const int64_t b = kept_off[part_ptr[v]], e = kept_off[part_ptr[v + 1]];
    indptr_p[v] = b;
    const int64_t np = (e - b + part_edges - 1) / part_edges;
    nparts[v] = np > 0 ? (int32_t)np : 1;                      // an empty row is still one work item: it writes its identity
}

// one wavefront per work item of the whole graph: its kept edges, in order, to their places; the first work
// item of a row also writes the row index of each of the row's new work items
__global__ __launch_bounds__(TPB) void k_cgp_fill(const int64_t* __restrict__ indptr, const int32_t* __restrict__ cols,
                                                  const int32_t* __restrict__ cdeg, const int32_t* __restrict__ part_ptr,
                                                  const int32_t* __restrict__ part_row, int64_t n_parts, int part_edges,
                                                  const int32_t* __restrict__ node_part,
                                                  const int32_t* __restrict__ targets, int n_query, int n_part, int p,
                                                  const int32_t* __restrict__ kept_off,
                                                  const int32_t* __restrict__ part_ptr_p, int32_t* __restrict__ cols_p,
                                                  int32_t* __restrict__ cdeg_p, int32_t* __restrict__ part_row_p) {
    const int64_t j = ((int64_t)blockIdx.x * TPB + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (j >= n_parts) return;
    int v;
    int64_t e0, e1;
    part_range(indptr, part_ptr, part_row, j, part_edges, v, e0, e1);
    int64_t out = kept_off[j];
    for (int64_t base = e0; base < e1; base += 64) {
        const int64_t e = base + lane;
        int32_t c = 0;
        bool keep = false;
        if (e < e1) {
            c = cols[e];
            keep = edge_partition(c, node_part, targets, n_query, n_part) == p;
        }
        const unsigned long long mask = __ballot(keep);
        if (keep) {
            const int64_t pos = out + __popcll(mask & ((1ull << lane) - 1ull));
            cols_p[pos] = c;
            cdeg_p[pos] = cdeg[e];
        }
        out += __popcll(mask);
    }
    if (j == part_ptr[v]) {
        const int p0 = part_ptr_p[v], np = part_ptr_p[v + 1] - p0;
        for (int k = lane; k < np; k += 64) part_row_p[p0 + k] = v;
    }
}

__device__ inline int64_t wave_append(bool pred, long long* counter) {
    const unsigned long long mask = __ballot(pred);
    const int lane = threadIdx.x & 63;
    const int leader = mask ? __ffsll((long long)mask) - 1 : 0;
    unsigned long long base = 0;
    if (lane == leader && mask) base = atomicAdd((unsigned long long*)counter, (unsigned long long)__popcll(mask));
    base = __shfl(base, leader);
    return (int64_t)base + __popcll(mask & ((1ull << lane) - 1ull));
}

// rows cut into several work items, listed for the combine step (all rows / query rows only)
__global__ void k_cgp_lists(const int32_t* __restrict__ part_ptr, int64_t rows, int64_t n_query,
                            int32_t* __restrict__ split_rows, int32_t* __restrict__ split_rows_q,
                            int32_t* __restrict__ split_big, int32_t* __restrict__ split_big_q, PartCounts* c) {
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;      // whole wavefronts: no early return
    const int np = v < rows ? part_ptr[v + 1] - part_ptr[v] : 0;
    const bool few = np > 1 && np <= OMG_MANY_PARTS, many = np > OMG_MANY_PARTS, q = v < n_query;
    const int64_t a = wave_append(few, &c->n_split);
    if (few) split_rows[a] = (int32_t)v;
    const int64_t aq = wave_append(few && q, &c->n_split_last);
    if (few && q) split_rows_q[aq] = (int32_t)v;
    const int64_t b = wave_append(many, &c->n_split_big);
    if (many) split_big[b] = (int32_t)v;
    const int64_t bq = wave_append(many && q, &c->n_split_big_last);
    if (many && q) split_big_q[bq] = (int32_t)v;
}

// ---- merge functions (Sec. 6.2) ------------------------------------------------------------------------------
// A block per destination, a thread per 16-byte column group; partitions are taken in ascending order, so
// the result does not depend on scheduling.  The total number of messages (the sum of the records' counts)
// is the destination's degree.
__device__ inline int record_count(const float* rec, int64_t at) { return __float_as_int(rec[at]); }

__global__ __launch_bounds__(TPB) void k_cgp_merge(CgpMergeArgs a) {
    const int64_t v = blockIdx.x;
    const float* rec0 = a.wire + v * a.ld_wire;
    const int64_t pstride = a.n_rows * a.ld_wire;
    int total = 0;
    for (int p = 0; p < a.n_part; ++p) total += record_count(rec0 + p * pstride, a.agg_ld);
    const int dim4 = (a.dim + 3) & ~3;
    const float deg = (float)total;
    for (int c4 = threadIdx.x * 4; c4 < a.agg_ld; c4 += TPB * 4) {
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        if (c4 < dim4) {
            if (a.op == OMG_OP_MAX) s = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            for (int p = 0; p < a.n_part; ++p) {
                const float4 t = *reinterpret_cast<const float4*>(rec0 + p * pstride + c4);
                if (a.op == OMG_OP_MAX) { s.x = fmaxf(s.x, t.x); s.y = fmaxf(s.y, t.y); s.z = fmaxf(s.z, t.z); s.w = fmaxf(s.w, t.w); }
                else { s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w; }
            }
            float v4[4] = {s.x, s.y, s.z, s.w};
            if (a.op == OMG_OP_GCN) {
                const float rs = rsqrtf(deg + 1.f), inv = 1.f / (deg + 1.f);
                const float4 sv = *reinterpret_cast<const float4*>(a.self + v * a.self_ld + c4);
                const float self4[4] = {sv.x, sv.y, sv.z, sv.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) v4[i] = v4[i] * rs + self4[i] * inv;
                if (a.h0 != nullptr) {
                    const float4 h = *reinterpret_cast<const float4*>(a.h0 + v * a.h0_ld + c4);
                    const float h4[4] = {h.x, h.y, h.z, h.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) v4[i] = (1.f - a.alpha) * v4[i] + a.alpha * h4[i];
                }
            } else if (a.op != OMG_OP_SUM) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (total == 0) v4[i] = 0.f;
                    else if (a.op == OMG_OP_MEAN) v4[i] = v4[i] / deg;
                    else if (a.op == OMG_OP_POW || a.op == OMG_OP_MOM) v4[i] = __powf(v4[i] / deg, 1.f / a.agg_p);
                }
            }
            s = make_float4(v4[0], v4[1], v4[2], v4[3]);
        }
        *reinterpret_cast<float4*>(a.out + v * a.out_ld + c4) = s;
    }
}

// Softmax merge: every partition's sums are relative to its own maximum score m_p; with M = max_p m_p they are
// rescaled by exp(m_p - M), added, and divided by the rescaled sum of exponentials.
__global__ __launch_bounds__(TPB) void k_cgp_merge_softmax(CgpMergeArgs a) {
    const int64_t v = blockIdx.x;
    const int H = a.heads;
    const float* rec0 = a.wire + v * a.ld_wire;
    const int64_t pstride = a.n_rows * a.ld_wire;
    const int64_t stats = (int64_t)H * a.agg_ld;
    const int groups = (int)(a.agg_ld / 4);
    const int dim4 = (a.dim + 3) & ~3;
    for (int idx = threadIdx.x; idx < H * groups; idx += TPB) {
        const int h = idx / groups, c4 = (idx - h * groups) * 4;
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        if (c4 < dim4) {
            float M = -INFINITY;
            for (int p = 0; p < a.n_part; ++p) M = fmaxf(M, rec0[p * pstride + stats + h]);
            float S = 0.f;
            if (M > -INFINITY) {
                for (int p = 0; p < a.n_part; ++p) {
                    const float* rec = rec0 + p * pstride;
                    const float m = rec[stats + h];
                    if (!(m > -INFINITY)) continue;                   // a partition that holds none of the row's neighbours
                    const float f = __expf(m - M);
                    S += f * rec[stats + OMG_GAT_STAT_SUM + h];
                    const float4 t = *reinterpret_cast<const float4*>(rec + (int64_t)h * a.agg_ld + c4);
                    s.x = fmaf(f, t.x, s.x); s.y = fmaf(f, t.y, s.y); s.z = fmaf(f, t.z, s.z); s.w = fmaf(f, t.w, s.w);
                }
            }
            const float inv = S > 0.f ? 1.f / S : 0.f;
            s.x *= inv; s.y *= inv; s.z *= inv; s.w *= inv;
        }
        *reinterpret_cast<float4*>(a.out + (v * H + h) * a.agg_ld + c4) = s;
    }
}

}  // namespace

int omg_launch_cgp_merge(const CgpMergeArgs& a, hipStream_t s) {
    if (a.n_rows <= 0) return OMG_OK;
    if (a.n_part < 1 || a.n_part > OMG_CGP_MAX_PARTS || a.agg_ld % 4 != 0) return OMG_EINVAL;
    if (a.heads > 0) hipLaunchKernelGGL(k_cgp_merge_softmax, dim3((unsigned)a.n_rows), dim3(TPB), 0, s, a);
    else hipLaunchKernelGGL(k_cgp_merge, dim3((unsigned)a.n_rows), dim3(TPB), 0, s, a);
    OMG_HIP(hipGetLastError());
    return OMG_OK;
}

int omg_cgp_partition_impl(omg_ctx* ctx, const omg_graph* g, const int32_t* node_part, int n_part, int p, omg_graph* out) {
    hipStream_t s = ctx->stream;
    const int64_t rows = g->rows_in;
    const int n_query = g->n_query;
    out->built = false;
    out->order_ready = false;
    out->n_query = g->n_query;
    out->n_qedges = g->n_qedges;
    out->rows_in = rows;
    out->part_edges = g->part_edges;
    out->c = g->c;
    const size_t ns = (size_t)rows + 2, nz = (size_t)g->c.nnz_in + 1;
    if (g->c.n_parts >= ((int64_t)1 << 31) || g->c.nnz_in >= ((int64_t)1 << 31)) return OMG_EUNSUPPORTED;
    OMG_TRY(ctx->cgpLen.ensure(sizeof(int32_t) * (size_t)(g->c.n_parts + 2)));
    OMG_TRY(ctx->cgpOff.ensure(sizeof(int64_t) * (size_t)(g->c.n_parts + 2)));
    OMG_TRY(ctx->cgpNp.ensure(sizeof(int32_t) * ns));
    OMG_TRY(ctx->cgpCounts.ensure(sizeof(PartCounts)));
    OMG_TRY(out->indptr.ensure(sizeof(int64_t) * ns));
    OMG_TRY(out->part_ptr.ensure(sizeof(int32_t) * ns));
    OMG_TRY(out->cols.ensure(sizeof(int32_t) * nz));            // upper bound: the whole graph's edges
    OMG_TRY(out->cdeg.ensure(sizeof(int32_t) * nz));
    OMG_TRY(out->split_rows.ensure(sizeof(int32_t) * ns));
    OMG_TRY(out->split_big.ensure(sizeof(int32_t) * ns));
    OMG_TRY(out->split_rows_q.ensure(sizeof(int32_t) * (size_t)(n_query + 2)));
    OMG_TRY(out->split_big_q.ensure(sizeof(int32_t) * (size_t)(n_query + 2)));
    // the row lists of the whole graph, so that the share can be exported and inspected like any graph
    const size_t nc = (size_t)g->c.n_cand, nt = (size_t)g->c.n_target;
    OMG_TRY(out->cand.ensure(sizeof(int32_t) * (nc + 1)));
    OMG_TRY(out->qdeg.ensure(sizeof(int32_t) * (nc + 1)));
    OMG_TRY(out->targets.ensure(sizeof(int32_t) * (nt + 1)));
    if (nc) {
        OMG_HIP(hipMemcpyAsync(out->cand.p, g->cand.p, sizeof(int32_t) * nc, hipMemcpyDeviceToDevice, s));
        OMG_HIP(hipMemcpyAsync(out->qdeg.p, g->qdeg.p, sizeof(int32_t) * nc, hipMemcpyDeviceToDevice, s));
    }
    if (nt) OMG_HIP(hipMemcpyAsync(out->targets.p, g->targets.p, sizeof(int32_t) * nt, hipMemcpyDeviceToDevice, s));

    PartCounts* pc = ctx->cgpCounts.as<PartCounts>();
    OMG_HIP(hipMemsetAsync(pc, 0, sizeof(PartCounts), s));
    hipLaunchKernelGGL(k_cgp_check, dim3(grid_for(ctx->base.n_nodes)), dim3(TPB), 0, s, node_part, ctx->base.n_nodes,
                       n_part, pc);
    PartCounts host{};
    const int64_t n_parts = g->c.n_parts;                       // work items of the whole graph
    const unsigned item_grid = grid_for(n_parts * 64);
    int32_t* kept = ctx->cgpLen.as<int32_t>();
    int32_t* kept_off = ctx->cgpOff.as<int32_t>();
    if (rows > 0) {
        hipLaunchKernelGGL(k_cgp_count, dim3(item_grid), dim3(TPB), 0, s, g->indptr.as<int64_t>(), g->cols.as<int32_t>(),
                           g->part_ptr.as<int32_t>(), g->part_row.as<int32_t>(), n_parts, g->part_edges, node_part,
                           g->targets.as<int32_t>(), n_query, n_part, p, kept);
        hipLaunchKernelGGL(k_cgp_scan, dim3(1), dim3(1024), 0, s, kept, n_parts, kept_off, (int64_t)0,
                           (long long*)nullptr, &pc->nnz);
        hipLaunchKernelGGL(k_cgp_rows, dim3(grid_for(rows + 1)), dim3(TPB), 0, s, g->part_ptr.as<int32_t>(), kept_off, rows,
                           g->part_edges, out->indptr.as<int64_t>(), ctx->cgpNp.as<int32_t>());
        hipLaunchKernelGGL(k_cgp_scan, dim3(1), dim3(1024), 0, s, ctx->cgpNp.as<int32_t>(), rows,
                           out->part_ptr.as<int32_t>(), (int64_t)n_query, &pc->n_parts_last, &pc->n_parts);
        hipLaunchKernelGGL(k_cgp_lists, dim3(grid_for(rows)), dim3(TPB), 0, s, out->part_ptr.as<int32_t>(), rows,
                           (int64_t)n_query, out->split_rows.as<int32_t>(), out->split_rows_q.as<int32_t>(),
                           out->split_big.as<int32_t>(), out->split_big_q.as<int32_t>(), pc);
    }
    OMG_HIP(hipGetLastError());
    OMG_HIP(hipMemcpyAsync(&host, pc, sizeof(PartCounts), hipMemcpyDeviceToHost, s));
    OMG_HIP(hipStreamSynchronize(s));
    if (host.bad) return OMG_ERANGE;
    if (host.n_parts >= ((long long)1 << 31)) return OMG_EUNSUPPORTED;
    OMG_TRY(out->part_row.ensure(sizeof(int32_t) * (size_t)(host.n_parts + 1)));
    if (rows > 0) {
        hipLaunchKernelGGL(k_cgp_fill, dim3(item_grid), dim3(TPB), 0, s, g->indptr.as<int64_t>(), g->cols.as<int32_t>(),
                           g->cdeg.as<int32_t>(), g->part_ptr.as<int32_t>(), g->part_row.as<int32_t>(), n_parts,
                           g->part_edges, node_part, g->targets.as<int32_t>(), n_query, n_part, p, kept_off,
                           out->part_ptr.as<int32_t>(), out->cols.as<int32_t>(), out->cdeg.as<int32_t>(),
                           out->part_row.as<int32_t>());
        OMG_HIP(hipGetLastError());
    } else {
        OMG_HIP(hipMemsetAsync(out->indptr.p, 0, sizeof(int64_t), s));
    }
    out->c.nnz_in = host.nnz;
    out->c.n_parts = host.n_parts;
    out->c.n_parts_last = host.n_parts_last;
    out->c.n_split = host.n_split;
    out->c.n_split_last = host.n_split_last;
    out->c.n_split_big = host.n_split_big;
    out->c.n_split_big_last = host.n_split_big_last;
    out->built = true;
    return OMG_OK;
}
