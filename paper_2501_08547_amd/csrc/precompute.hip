// Precomputed embeddings (Sec. 5): layer l of the model applied to EVERY training node on the
// training graph alone, l = 1..k-1, each layer's output stored as the table the serving path
// reads.  Same kernels as serving: the training graph itself is handed to them as a computation
// graph whose columns all point into the stored table of the previous layer (no tagged columns),
// in chunks of rows so that the fp32 staging of a chunk's own rows stays small.
#include "internal.h"

#include <new>

namespace {

constexpr int TPB = 256;
constexpr int64_t CHUNK_ROWS = (int64_t)1 << 17;     // rows per pass: bounds the staging buffers (a chunk of `mid` still has 60 M edges)
constexpr int PART = OMG_PART_EDGES;

struct ChunkCounts {
    long long n_parts, n_split, n_split_big;
};

inline unsigned grid_for(int64_t n, int64_t per_block = TPB) {
    const int64_t g = (n + per_block - 1) / per_block;
    return (unsigned)(g > 0 ? g : 1);
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

// per row of the chunk: node id, number of work items, and the lists of rows cut into parts
__global__ void k_chunk_rows(const int64_t* __restrict__ indptr, int64_t r0, int64_t nr, int32_t* __restrict__ ids,
                             int32_t* __restrict__ nparts, int32_t* __restrict__ split_rows,
                             int32_t* __restrict__ split_big, ChunkCounts* c) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;     // whole wavefronts: no early return
    int32_t np = 0;
    if (i < nr) {
        const int64_t len = indptr[r0 + i + 1] - indptr[r0 + i];
        np = (int32_t)((len + PART - 1) / PART);
        if (np < 1) np = 1;
        ids[i] = (int32_t)(r0 + i);
        nparts[i] = np;
    } else if (i == nr) {
        nparts[i] = 0;
    }
    int64_t s = np;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if ((threadIdx.x & 63) == 0 && s) atomicAdd((unsigned long long*)&c->n_parts, (unsigned long long)s);
    const bool few = np > 1 && np <= OMG_MANY_PARTS, many = np > OMG_MANY_PARTS;
    const int64_t a = wave_append(few, &c->n_split);
    if (few) split_rows[a] = (int32_t)i;
    const int64_t b = wave_append(many, &c->n_split_big);
    if (many) split_big[b] = (int32_t)i;
}

// exclusive prefix sum of up to a few million ints by one block (offline path: simplicity over speed)
__global__ __launch_bounds__(1024) void k_scan_i32(const int32_t* __restrict__ in, int32_t* __restrict__ out, int64_t n) {
    __shared__ int64_t wave_tot[16];
    __shared__ int64_t carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    constexpr int ITEMS = 8;
    for (int64_t base = 0; base < n; base += 1024 * ITEMS) {
        const int64_t i0 = base + (int64_t)threadIdx.x * ITEMS;
        int32_t v[ITEMS];
        int64_t sum = 0;
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            v[j] = i0 + j < n ? in[i0 + j] : 0;
            sum += v[j];
        }
        int64_t x = sum;
        const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int64_t y = __shfl_up(x, off);
            if (lane >= off) x += y;
        }
        if (lane == 63) wave_tot[wid] = x;
        __syncthreads();
        int64_t before = 0, all = 0;
        for (int w = 0; w < 16; ++w) {
            const int64_t t = wave_tot[w];
            if (w < wid) before += t;
            all += t;
        }
        int64_t run = carry_s + before + x - sum;
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            if (i0 + j < n) out[i0 + j] = (int32_t)run;
            run += v[j];
        }
        __syncthreads();
        if (threadIdx.x == 0) carry_s += all;
        __syncthreads();
    }
}

__global__ void k_part_rows(const int32_t* __restrict__ part_ptr, int64_t nr, int64_t n_parts, int32_t* __restrict__ part_row) {
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= n_parts) return;
    int64_t lo = 0, hi = nr;                      // last row whose first part is <= j
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (part_ptr[mid] <= j) lo = mid; else hi = mid;
    }
    part_row[j] = (int32_t)lo;
}

// in-degree of every source of the chunk's edges (GCN's normalisation on the training graph)
__global__ void k_chunk_cdeg(const int64_t* __restrict__ indptr, const int32_t* __restrict__ indices, int64_t e0,
                             int64_t ne, int32_t* __restrict__ cdeg) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= ne) return;
    const int32_t u = indices[e0 + p];
    cdeg[p] = (int32_t)(indptr[(int64_t)u + 1] - indptr[u]);
}

// fp32 -> bf16, round to nearest even
__global__ void k_store_bf16(const float* __restrict__ src, int64_t lds, int64_t nr, int dim, uint16_t* __restrict__ dst,
                             int64_t ldd) {
    const int64_t row = blockIdx.x;
    if (row >= nr) return;
    for (int c = threadIdx.x; c < ldd; c += blockDim.x) {
        uint16_t o = 0;
        if (c < dim) {
            const uint32_t b = __float_as_uint(src[row * lds + c]);
            o = (uint16_t)((b + 0x7fffu + ((b >> 16) & 1u)) >> 16);
        }
        dst[row * ldd + c] = o;
    }
}

int layer_width(const omg_layer* L) { return (L->model == OMG_GAT && L->head_mean) ? L->d_out / L->heads : L->d_out; }

}  // namespace

int omg_precompute_layer(omg_ctx* ctx, const omg_table* first, const omg_table* prev, const omg_layer* L_in,
                         const omg_table* out) {
    omg_layer layer = *L_in;                      // a copy: GCNII's initial rows are pointed at the chunk's staging below
    const omg_layer* L = &layer;
    hipStream_t s = ctx->stream;
    const int64_t n = ctx->base.n_nodes;
    const int64_t* indptr = ctx->base.indptr;
    const int w_out = layer_width(L);
    if (prev->dim != L->d_in || out->dim != w_out || prev->n_rows < n || out->n_rows < n) return OMG_EINVAL;
    const int64_t ld_in = (prev->dim + 7) / 8 * 8;
    const int64_t ld_st = (w_out + 7) / 8 * 8;

    omg_graph view;                               // the training graph, a chunk of rows at a time; owns nothing but its lists
    view.ctx = ctx;
    view.part_edges = PART;
    view.built = true;
    int rc = OMG_OK;
    for (int64_t r0 = 0; r0 < n && rc == OMG_OK; r0 += CHUNK_ROWS) {
        const int64_t nr = n - r0 < CHUNK_ROWS ? n - r0 : CHUNK_ROWS;
        int64_t e_range[2];
        OMG_HIP(hipMemcpyAsync(&e_range[0], indptr + r0, sizeof(int64_t), hipMemcpyDeviceToHost, s));
        OMG_HIP(hipMemcpyAsync(&e_range[1], indptr + r0 + nr, sizeof(int64_t), hipMemcpyDeviceToHost, s));
        OMG_TRY(ctx->preIds.ensure(sizeof(int32_t) * (size_t)(nr + 1)));
        OMG_TRY(ctx->preNparts.ensure(sizeof(int32_t) * (size_t)(nr + 64)));
        OMG_TRY(view.part_ptr.ensure(sizeof(int32_t) * (size_t)(nr + 2)));
        OMG_TRY(view.split_rows.ensure(sizeof(int32_t) * (size_t)(nr + 1)));
        OMG_TRY(view.split_big.ensure(sizeof(int32_t) * (size_t)(nr + 1)));
        OMG_TRY(ctx->preCounts.ensure(sizeof(ChunkCounts)));
        ChunkCounts* cd = ctx->preCounts.as<ChunkCounts>();
        OMG_HIP(hipMemsetAsync(cd, 0, sizeof(ChunkCounts), s));
        hipLaunchKernelGGL(k_chunk_rows, dim3(grid_for(nr + 1)), dim3(TPB), 0, s, indptr, r0, nr, ctx->preIds.as<int32_t>(),
                           ctx->preNparts.as<int32_t>(), view.split_rows.as<int32_t>(), view.split_big.as<int32_t>(), cd);
        hipLaunchKernelGGL(k_scan_i32, dim3(1), dim3(1024), 0, s, ctx->preNparts.as<int32_t>(), view.part_ptr.as<int32_t>(),
                           nr + 1);
        ChunkCounts hc;
        OMG_HIP(hipMemcpyAsync(&hc, cd, sizeof(ChunkCounts), hipMemcpyDeviceToHost, s));
        OMG_HIP(hipStreamSynchronize(s));
        const int64_t e0 = e_range[0], ne = e_range[1] - e_range[0];
        OMG_TRY(view.part_row.ensure(sizeof(int32_t) * (size_t)(hc.n_parts + 1)));
        hipLaunchKernelGGL(k_part_rows, dim3(grid_for(hc.n_parts)), dim3(TPB), 0, s, view.part_ptr.as<int32_t>(), nr,
                           (int64_t)hc.n_parts, view.part_row.as<int32_t>());
        if (L->model == OMG_GCN_SYM || L->model == OMG_GCNII) {
            OMG_TRY(ctx->preCdeg.ensure(sizeof(int32_t) * (size_t)(ne + 1)));
            if (ne > 0)
                hipLaunchKernelGGL(k_chunk_cdeg, dim3(grid_for(ne)), dim3(TPB), 0, s, indptr, ctx->base.indices, e0, ne,
                                   ctx->preCdeg.as<int32_t>());
        }
        // the chunk's own rows of the previous layer, as fp32
        OMG_TRY(ctx->preSelf.ensure(sizeof(float) * (size_t)(nr * ld_in)));
        OMG_TRY(omg_launch_init_buffer(prev, nullptr, 0, ctx->preIds.as<omg_node_t>(), 0, nr, ctx->preSelf.as<float>(), ld_in, s));
        if (L->model == OMG_GCNII) {              // the chunk's layer-0 rows: the first table's
            if (first->dim != L->d_in) return OMG_EINVAL;
            if (first == prev) {
                layer.init_rows = ctx->preSelf.as<float>();
            } else {
                OMG_TRY(ctx->preInit.ensure(sizeof(float) * (size_t)(nr * ld_in)));
                OMG_TRY(omg_launch_init_buffer(first, nullptr, 0, ctx->preIds.as<omg_node_t>(), 0, nr, ctx->preInit.as<float>(),
                                               ld_in, s));
                layer.init_rows = ctx->preInit.as<float>();
            }
            layer.init_ld = ld_in;
        }

        // borrowed views: row pointers keep their absolute edge offsets, so columns and source degrees are
        // addressed from the start of the whole arrays
        view.n_query = 0;
        view.order_ready = false;
        view.rows_in = nr;
        view.c = BuildCounts{};
        view.c.n_target = nr;
        view.c.nnz_in = ne;
        view.c.n_parts = hc.n_parts;
        view.c.n_split = hc.n_split;
        view.c.n_split_big = hc.n_split_big;
        view.indptr.p = const_cast<int64_t*>(indptr + r0);
        view.cols.p = const_cast<int32_t*>(ctx->base.indices);
        view.cdeg.p = (L->model == OMG_GCN_SYM || L->model == OMG_GCNII) ? static_cast<void*>(ctx->preCdeg.as<int32_t>() - e0)
                                                                         : nullptr;

        float* dst = nullptr;
        int64_t ldo = 0;
        if (out->dtype == OMG_F32) {
            dst = const_cast<float*>(static_cast<const float*>(out->data)) + r0 * out->ld;
            ldo = out->ld;
        } else {
            OMG_TRY(ctx->preStage.ensure(sizeof(float) * (size_t)(nr * ld_st)));
            dst = ctx->preStage.as<float>();
            ldo = ld_st;
        }
        rc = omg_run_layer(ctx, &view, 0, prev, ctx->preSelf.as<float>(), ld_in, L, dst, ldo);
        if (rc == OMG_OK && out->dtype == OMG_BF16) {
            uint16_t* o = const_cast<uint16_t*>(static_cast<const uint16_t*>(out->data)) + r0 * out->ld;
            hipLaunchKernelGGL(k_store_bf16, dim3((unsigned)nr), dim3(128), 0, s, dst, ldo, nr, w_out, o, out->ld);
        }
        if (rc == OMG_OK && hipGetLastError() != hipSuccess) rc = OMG_EHIP;
        if (rc == OMG_OK && hipStreamSynchronize(s) != hipSuccess) rc = OMG_EHIP;      // the views and counts are reused by the next chunk
    }
    view.indptr.p = nullptr;                      // borrowed, not owned
    view.cols.p = nullptr;
    view.cdeg.p = nullptr;
    (void)hipStreamSynchronize(s);
    for (DevBuf* b : {&view.part_ptr, &view.part_row, &view.split_rows, &view.split_big, &view.order}) b->release();
    return rc;
}
