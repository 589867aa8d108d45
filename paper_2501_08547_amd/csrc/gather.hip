// Neighbour aggregation of one layer over the batch's computation graph (Eq. 1, the
// aggregate step; Sec. 6.1 "local aggregation" with a single partition).
//
// One wavefront owns one work item = (row, at most OMG_PART_EDGES consecutive edges).  A
// feature row is read as 16-byte pieces: G lanes (a power of two) cover one row, so a
// wavefront reads 64 / G rows per load instruction, and a lane keeps NP pieces when a row
// is longer than 64 pieces.  Column ids (and the GCN source degrees) are fetched 64 at a
// time, one per lane, and handed to the lanes that need them with cross-lane reads.
// Sources are rows of the stored table (fp32 or bf16) or, for tagged columns, rows of the
// fp32 buffer of freshly computed embeddings.  Accumulation is fp32.  Rows cut into several
// parts write partial sums that a second kernel adds in part order, so results do not
// depend on scheduling.
#include "internal.h"

namespace {

constexpr int WAVES_PER_BLOCK = 4;

struct F8 { float v[8]; };

__device__ inline void unpack_bf16x8(const uint4& r, float* o) {
    o[0] = __uint_as_float(r.x << 16); o[1] = __uint_as_float(r.x & 0xffff0000u);
    o[2] = __uint_as_float(r.y << 16); o[3] = __uint_as_float(r.y & 0xffff0000u);
    o[4] = __uint_as_float(r.z << 16); o[5] = __uint_as_float(r.z & 0xffff0000u);
    o[6] = __uint_as_float(r.w << 16); o[7] = __uint_as_float(r.w & 0xffff0000u);
}

// EPC = elements per 16-byte piece of the table: 4 (fp32) or 8 (bf16)
template <int EPC> struct Piece { float v[EPC]; };

template <int EPC>
__device__ inline void load_piece(const void* __restrict__ table, int64_t table_ld, const float* __restrict__ buf,
                                  int64_t buf_ld, int dim4, int32_t col, int piece, Piece<EPC>& out) {
    if (col >= 0) {
        if constexpr (EPC == 4) {
            const float4 r = *reinterpret_cast<const float4*>(static_cast<const float*>(table) + (int64_t)col * table_ld + piece * 4);
            out.v[0] = r.x; out.v[1] = r.y; out.v[2] = r.z; out.v[3] = r.w;
        } else {
            const uint4 r = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(table) + (int64_t)col * table_ld + piece * 8);
            unpack_bf16x8(r, out.v);
        }
    } else {
        const float* row = buf + (int64_t)(~col) * buf_ld + piece * EPC;
#pragma unroll
        for (int g = 0; g < EPC / 4; ++g) {
            float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
            if (piece * EPC + g * 4 < dim4) r = *reinterpret_cast<const float4*>(row + g * 4);
            out.v[g * 4 + 0] = r.x; out.v[g * 4 + 1] = r.y; out.v[g * 4 + 2] = r.z; out.v[g * 4 + 3] = r.w;
        }
    }
}

// G lanes per row, NP pieces per lane (NP > 1 only with G == 64), U edge slots in flight per group.
template <int EPC, int G, int NP, int U, bool GCN>
__global__ __launch_bounds__(WAVES_PER_BLOCK * 64) void k_gather(GatherArgs a) {
    const int lane = threadIdx.x & 63;
    const int64_t part = (int64_t)blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x >> 6);
    if (part >= a.n_parts) return;
    const int v = a.part_row[part];
    const int first_part = a.part_ptr[v];
    const int n_row_parts = a.part_ptr[v + 1] - first_part;
    const int64_t row_beg = a.indptr[v], row_end = a.indptr[v + 1];
    const int64_t e0 = row_beg + (int64_t)(part - first_part) * omg_row_part(row_end - row_beg, a.part_edges);
    const int64_t e1 = (e0 + omg_row_part(row_end - row_beg, a.part_edges) < row_end) ? e0 + omg_row_part(row_end - row_beg, a.part_edges) : row_end;
    const float row_d1 = (float)(row_end - row_beg + 1);

    constexpr int EPI = 64 / G;                 // edges per load instruction
    const int grp = lane / G;
    const int sub = lane % G;
    const int n_pieces = (a.dim + EPC - 1) / EPC;
    const int dim4 = (a.dim + 3) & ~3;

    float acc[NP][EPC];
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int i = 0; i < EPC; ++i) acc[p][i] = 0.f;

    for (int64_t base = e0; base < e1; base += 64) {
        const int n = (int)((e1 - base < 64) ? (e1 - base) : 64);
        int32_t my_col = 0;
        float my_w = 0.f;
        if (lane < n) {
            my_col = a.cols[base + lane];
            if constexpr (GCN) my_w = rsqrtf((float)(a.cdeg[base + lane] + 1) * row_d1);
            else my_w = 1.f;
        }
        for (int j = 0; j < n; j += EPI * U) {
            Piece<EPC> x[U][NP];
            float w[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int idx = j + u * EPI + grp;
                const int src_lane = idx < 64 ? idx : 63;
                const int32_t c = __shfl(my_col, src_lane);
                const float wu = __shfl(my_w, src_lane);
                w[u] = (idx < n) ? wu : 0.f;
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    const int piece = sub + p * 64;
                    if (idx < n && piece < n_pieces) {
                        load_piece<EPC>(a.table, a.table_ld, a.buf, a.buf_ld, dim4, c, piece, x[u][p]);
                    } else {
#pragma unroll
                        for (int i = 0; i < EPC; ++i) x[u][p].v[i] = 0.f;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int p = 0; p < NP; ++p)
#pragma unroll
                    for (int i = 0; i < EPC; ++i) {
                        if constexpr (GCN) acc[p][i] = fmaf(w[u], x[u][p].v[i], acc[p][i]);
                        else acc[p][i] += w[u] * x[u][p].v[i];
                    }
        }
    }

    // fold the 64 / G groups of the wavefront into group 0
#pragma unroll
    for (int off = G; off < 64; off <<= 1)
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int i = 0; i < EPC; ++i) acc[p][i] += __shfl_xor(acc[p][i], off);

    if (grp != 0) return;
    const bool whole = n_row_parts == 1;
    float scale = 1.f;
    if (whole && !GCN) {
        const int64_t deg = row_end - row_beg;
        scale = deg > 0 ? 1.f / (float)deg : 0.f;
    }
    float* dst = whole ? a.agg + (int64_t)v * a.agg_ld : a.partial + part * a.agg_ld;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int piece = sub + p * 64;
        if (piece >= n_pieces) continue;
#pragma unroll
        for (int g = 0; g < EPC / 4; ++g) {
            const int col0 = piece * EPC + g * 4;
            if (col0 >= a.agg_ld) continue;
            float4 o = make_float4(acc[p][g * 4] * scale, acc[p][g * 4 + 1] * scale, acc[p][g * 4 + 2] * scale,
                                   acc[p][g * 4 + 3] * scale);
            if (whole && GCN && col0 < dim4) {
                const float4 sv = *reinterpret_cast<const float4*>(a.buf + (int64_t)v * a.buf_ld + col0);
                const float inv = 1.f / row_d1;
                o.x += sv.x * inv; o.y += sv.y * inv; o.z += sv.z * inv; o.w += sv.w * inv;
            }
            *reinterpret_cast<float4*>(dst + col0) = o;
        }
    }
}

// Rows cut into several parts: add up the partial sums, then scale / add the self term.  The order
// of additions is fixed, so the result does not depend on scheduling.  Two shapes:
//   combine_few     rows of 2..OMG_MANY_PARTS parts: a block per row, a thread per 16-byte column
//                   group, the parts fetched together and added in part order;
//   combine_many    longer rows: a block per (row, 32 column groups), 8 thread groups that each add
//                   every 8th part, then the 8 sums added in group order through LDS.
template <bool GCN>
__device__ inline void finish_row(const GatherArgs& a, int v, int c4, float4 s) {
    const int64_t deg = a.indptr[v + 1] - a.indptr[v];
    if constexpr (GCN) {
        if (c4 < ((a.dim + 3) & ~3)) {
            const float4 sv = *reinterpret_cast<const float4*>(a.buf + (int64_t)v * a.buf_ld + c4);
            const float inv = 1.f / (float)(deg + 1);
            s.x += sv.x * inv; s.y += sv.y * inv; s.z += sv.z * inv; s.w += sv.w * inv;
        }
    } else {
        const float inv = deg > 0 ? 1.f / (float)deg : 0.f;
        s.x *= inv; s.y *= inv; s.z *= inv; s.w *= inv;
    }
    *reinterpret_cast<float4*>(a.agg + (int64_t)v * a.agg_ld + c4) = s;
}

template <bool GCN>
__device__ inline void combine_few(const GatherArgs& a, int v) {
    const int p0 = a.part_ptr[v], np = a.part_ptr[v + 1] - p0;
    for (int c4 = threadIdx.x * 4; c4 < a.agg_ld; c4 += 1024) {
        float4 t[OMG_MANY_PARTS];
#pragma unroll
        for (int i = 0; i < OMG_MANY_PARTS; ++i)
            t[i] = i < np ? *reinterpret_cast<const float4*>(a.partial + (int64_t)(p0 + i) * a.agg_ld + c4)
                          : make_float4(0.f, 0.f, 0.f, 0.f);
        float4 s = t[0];
#pragma unroll
        for (int i = 1; i < OMG_MANY_PARTS; ++i) { s.x += t[i].x; s.y += t[i].y; s.z += t[i].z; s.w += t[i].w; }
        finish_row<GCN>(a, v, c4, s);
    }
}

constexpr int COMB_COLS = 32, COMB_GROUPS = 8;

template <bool GCN>
__device__ inline void combine_many(const GatherArgs& a, int v, int chunk, float4 (*red)[COMB_COLS]) {
    const int col = threadIdx.x % COMB_COLS, grp = threadIdx.x / COMB_COLS;
    const int c4 = (chunk * COMB_COLS + col) * 4;
    const int p0 = a.part_ptr[v], p1 = a.part_ptr[v + 1];
    const bool live = c4 < a.agg_ld;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (live) {
        for (int p = p0 + grp; p < p1; p += COMB_GROUPS * 4) {
            float4 t[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                t[i] = (p + i * COMB_GROUPS < p1)
                           ? *reinterpret_cast<const float4*>(a.partial + (int64_t)(p + i * COMB_GROUPS) * a.agg_ld + c4)
                           : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int i = 0; i < 4; ++i) { s.x += t[i].x; s.y += t[i].y; s.z += t[i].z; s.w += t[i].w; }
        }
    }
    red[grp][col] = s;
    __syncthreads();
    if (grp != 0 || !live) return;
#pragma unroll
    for (int g2 = 1; g2 < COMB_GROUPS; ++g2) {
        const float4 t = red[g2][col];
        s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    finish_row<GCN>(a, v, c4, s);
}

// one launch for both shapes: the first n_split blocks take one short row each, the others one
// (long row, column chunk) each
template <bool GCN>
__global__ __launch_bounds__(COMB_COLS * COMB_GROUPS) void k_combine(GatherArgs a, int n_chunks) {
    __shared__ float4 red[COMB_GROUPS][COMB_COLS];
    const int64_t b = blockIdx.x;
    if (b < a.n_split) {
        combine_few<GCN>(a, a.split_rows[b]);
    } else {
        const int64_t r = (b - a.n_split) / n_chunks;
        combine_many<GCN>(a, a.split_big[r], (int)((b - a.n_split) - r * n_chunks), red);
    }
}

template <int EPC, int G, int NP, int U>
int launch_shape(const GatherArgs& a, hipStream_t s) {
    const unsigned grid = (unsigned)((a.n_parts + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
    if (a.mode == OMG_GCN_SYM)
        hipLaunchKernelGGL((k_gather<EPC, G, NP, U, true>), dim3(grid), dim3(WAVES_PER_BLOCK * 64), 0, s, a);
    else
        hipLaunchKernelGGL((k_gather<EPC, G, NP, U, false>), dim3(grid), dim3(WAVES_PER_BLOCK * 64), 0, s, a);
    return OMG_OK;
}

template <int EPC>
int launch_dtype(const GatherArgs& a, hipStream_t s) {
    const int n_pieces = (a.dim + EPC - 1) / EPC;
    if (n_pieces <= 8) return launch_shape<EPC, 8, 1, 4>(a, s);
    if (n_pieces <= 16) return launch_shape<EPC, 16, 1, 4>(a, s);
    if (n_pieces <= 32) return launch_shape<EPC, 32, 1, 4>(a, s);
    if (n_pieces <= 64) return launch_shape<EPC, 64, 1, 8>(a, s);
    if (n_pieces <= 128) return launch_shape<EPC, 64, 2, 4>(a, s);
    if (n_pieces <= 192) return launch_shape<EPC, 64, 3, 4>(a, s);
    if (n_pieces <= 256) return launch_shape<EPC, 64, 4, 2>(a, s);
    return OMG_EUNSUPPORTED;
}

__global__ void k_init_buffer(const void* __restrict__ table, int dtype, int64_t table_ld, int dim,
                              const float* __restrict__ qf, int64_t ld_q, const int32_t* __restrict__ targets,
                              int32_t n_query, int64_t n_rows, float* __restrict__ buf0, int64_t ld0) {
    const int64_t row = blockIdx.x;
    if (row >= n_rows) return;
    for (int c = threadIdx.x; c < ld0; c += blockDim.x) {
        float x = 0.f;
        if (c < dim) {
            if (row < n_query) {
                x = qf[row * ld_q + c];
            } else {
                const int64_t u = targets[row - n_query];
                if (dtype == OMG_F32) x = static_cast<const float*>(table)[u * table_ld + c];
                else x = __uint_as_float((uint32_t) static_cast<const uint16_t*>(table)[u * table_ld + c] << 16);
            }
        }
        buf0[row * ld0 + c] = x;
    }
}

}  // namespace

int omg_launch_gather(const GatherArgs& a, hipStream_t s, hipEvent_t after_main) {
    int rc = OMG_OK;
    if (a.n_parts > 0) rc = (a.table_dtype == OMG_F32) ? launch_dtype<4>(a, s) : launch_dtype<8>(a, s);
    if (rc != OMG_OK) return rc;
    if (after_main != nullptr) OMG_HIP(hipEventRecord(after_main, s));
    if (a.n_split + a.n_split_big > 0) {
        const int n_chunks = (int)((a.agg_ld / 4 + COMB_COLS - 1) / COMB_COLS);
        const unsigned grid = (unsigned)(a.n_split + a.n_split_big * n_chunks);
        if (a.mode == OMG_GCN_SYM)
            hipLaunchKernelGGL(k_combine<true>, dim3(grid), dim3(COMB_COLS * COMB_GROUPS), 0, s, a, n_chunks);
        else
            hipLaunchKernelGGL(k_combine<false>, dim3(grid), dim3(COMB_COLS * COMB_GROUPS), 0, s, a, n_chunks);
    }
    OMG_HIP(hipGetLastError());
    return OMG_OK;
}

int omg_launch_init_buffer(const omg_table* feat, const float* qf, int64_t ld_q, const omg_node_t* targets,
                           int32_t n_query, int64_t n_target, float* buf0, int64_t ld0, hipStream_t s) {
    const int64_t n_rows = (int64_t)n_query + n_target;
    if (n_rows <= 0) return OMG_OK;
    hipLaunchKernelGGL(k_init_buffer, dim3((unsigned)n_rows), dim3(128), 0, s, feat->data, feat->dtype, feat->ld,
                       feat->dim, qf, ld_q, targets, n_query, n_rows, buf0, ld0);
    OMG_HIP(hipGetLastError());
    return OMG_OK;
}
