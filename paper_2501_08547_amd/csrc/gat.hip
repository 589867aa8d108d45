// Attention aggregation of a GAT layer over the batch's computation graph: per-edge scores,
// row-wise softmax and the weighted neighbour sum (the softmax-based aggregation of Sec. 6.2).
//
// The score of edge u -> v is LeakyReLU(a_src . z_u + a_dst . z_v) with z = h W.  Because
// a . (h W_head) = (W_head a) . h, each half is a dot product of the *input* row with a folded
// vector, and sum_u alpha_uv z_u = (sum_u alpha_uv h_u) W_head, so the projection is applied
// once per destination by the update kernel.  Source halves of stored rows come from a
// per-node side table (omg_gat_src_logits); those of freshly computed rows are taken once per
// row here.  A work item stages its edges' scores in LDS, normalises them, then runs the same
// 16-byte-piece row gather as the plain aggregation with one accumulator set per head.
// A row cut into parts keeps (max score, sum of exponentials) per part and head; the combine
// kernel rescales and adds the parts - the two-step softmax the paper uses for its merge.
#include "internal.h"

#include <math.h>

namespace {

constexpr int WAVES_PER_BLOCK = 4;
constexpr int PART_PAD = OMG_GAT_STAT_PAD;   // floats appended to a partial row: max and exp-sum per head

__device__ inline float wave_max(float x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
    return x;
}
__device__ inline float wave_sum(float x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
}

// fold[h][k] = sum_j W[k][h * dh + j] * a[h][j]; one wavefront per (h, k), lanes along j (a contiguous piece
// of row k of W)
__global__ __launch_bounds__(256) void k_fold(const float* __restrict__ W, const float* __restrict__ a_src,
                                              const float* __restrict__ a_dst, int d_in, int d_out, int heads,
                                              float* __restrict__ fold_src, float* __restrict__ fold_dst) {
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x >> 6);
    if (i >= heads * d_in) return;
    const int h = i / d_in, k = i % d_in, dh = d_out / heads;
    float s = 0.f, d = 0.f;
    for (int j = lane; j < dh; j += 64) {
        const float w = W[(int64_t)k * d_out + h * dh + j];
        s = fmaf(w, a_src[h * dh + j], s);
        d = fmaf(w, a_dst[h * dh + j], d);
    }
    s = wave_sum(s);
    d = wave_sum(d);
    if (lane == 0) {
        fold_src[i] = s;
        fold_dst[i] = d;
    }
}

// Sums of N values per lane over the 64 lanes of a wavefront with N - 1 + log2(64 / N) exchanges instead of
// 6 N: at each halving step a lane keeps one half of its values and receives the other lanes' share of that
// half.  Afterwards v[0] of lane l holds the sum of value number l / (64 / N).  N a power of two, <= 16; all
// indices are compile-time, so the values stay in registers.
template <int N>
__device__ inline void wave_sum_many(float (&v)[N], int lane) {
    int off = 32;
#pragma unroll
    for (int n = N; n > 1; n >>= 1, off >>= 1) {
        const bool hi = (lane & off) != 0;
#pragma unroll
        for (int i = 0; i < n / 2; ++i) {
            const float send = hi ? v[i] : v[i + n / 2];
            const float keep = hi ? v[i + n / 2] : v[i];
            v[i] = keep + __shfl_xor(send, off);
        }
    }
#pragma unroll
    for (; off > 0; off >>= 1) v[0] += __shfl_xor(v[0], off);
}

// both score halves of every freshly computed row: one wavefront per row, one pass over the row for all heads,
// the 2 H dot products reduced together
template <int H>
__global__ __launch_bounds__(256) void k_buf_logits(const float* __restrict__ buf, int64_t buf_ld, int64_t n_rows, int dim,
                                                    const float* __restrict__ fold_src,
                                                    const float* __restrict__ fold_dst, float* __restrict__ src_out,
                                                    float* __restrict__ dst_out) {
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x >> 6);
    if (r >= n_rows) return;
    float v[2 * H];                     // [h] source halves, [H + h] destination halves
#pragma unroll
    for (int i = 0; i < 2 * H; ++i) v[i] = 0.f;
    for (int k = lane; k < dim; k += 64) {
        const float x = buf[r * buf_ld + k];
#pragma unroll
        for (int h = 0; h < H; ++h) {
            v[h] = fmaf(x, fold_src[h * dim + k], v[h]);
            v[H + h] = fmaf(x, fold_dst[h * dim + k], v[H + h]);
        }
    }
    wave_sum_many<2 * H>(v, lane);
    constexpr int LANES_PER_VALUE = 64 / (2 * H);
    if (lane % LANES_PER_VALUE == 0) {
        const int i = lane / LANES_PER_VALUE;
        if (i < H) src_out[r * H + i] = v[0];
        else dst_out[r * H + (i - H)] = v[0];
    }
}

// The same with the folded vectors in LDS and 16 lanes per row (four rows per wavefront, 16-byte loads): a quarter of
// the wavefronts and, per row, a quarter of the cross-lane steps.  Used when the 2 H vectors fit 48 KB of LDS.
template <int N>
__device__ inline void group16_sum_many(float (&v)[N], int lane) {
    int off = 8;
#pragma unroll
    for (int n = N; n > 1; n >>= 1, off >>= 1) {
        if (off == 0) break;
        const bool hi = (lane & off) != 0;
#pragma unroll
        for (int i = 0; i < n / 2; ++i) {
            const float send = hi ? v[i] : v[i + n / 2];
            const float keep = hi ? v[i + n / 2] : v[i];
            v[i] = keep + __shfl_xor(send, off);
        }
    }
#pragma unroll
    for (; off > 0; off >>= 1) v[0] += __shfl_xor(v[0], off);
}

template <int H>
__global__ __launch_bounds__(256) void k_buf_logits16(const float* __restrict__ buf, int64_t buf_ld, int64_t n_rows, int dim,
                                                      const float* __restrict__ fold_src,
                                                      const float* __restrict__ fold_dst, float* __restrict__ src_out,
                                                      float* __restrict__ dst_out) {
    extern __shared__ __attribute__((aligned(16))) float fl[];      // [2 H][fw]: source vectors, then destination vectors
    const int fw = (dim + 3) & ~3;
    for (int i = threadIdx.x; i < 2 * H * fw; i += 256) {
        const int h = i / fw, k = i - h * fw;
        fl[i] = k < dim ? (h < H ? fold_src[h * dim + k] : fold_dst[(h - H) * dim + k]) : 0.f;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, sub = lane & 15;
    const int64_t r = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 4 + (lane >> 4);
    const bool live = r < n_rows;
    float v[2 * H];
#pragma unroll
    for (int i = 0; i < 2 * H; ++i) v[i] = 0.f;
    for (int k4 = sub * 4; k4 < fw; k4 += 64) {
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
        if (live) x = *reinterpret_cast<const float4*>(buf + r * buf_ld + k4);
        if (k4 + 1 >= dim) x.y = 0.f;                   // what lies beyond dim in the row is not defined
        if (k4 + 2 >= dim) x.z = 0.f;
        if (k4 + 3 >= dim) x.w = 0.f;
#pragma unroll
        for (int i = 0; i < 2 * H; ++i) {
            const float4 f = *reinterpret_cast<const float4*>(&fl[i * fw + k4]);
            v[i] = fmaf(x.x, f.x, v[i]);
            v[i] = fmaf(x.y, f.y, v[i]);
            v[i] = fmaf(x.z, f.z, v[i]);
            v[i] = fmaf(x.w, f.w, v[i]);
        }
    }
    group16_sum_many<2 * H>(v, lane);
    constexpr int LANES_PER_VALUE = 16 / (2 * H) > 0 ? 16 / (2 * H) : 1;
    if (live && sub % LANES_PER_VALUE == 0) {
        const int i = sub / LANES_PER_VALUE;
        if (i < H) src_out[r * H + i] = v[0];
        else if (i < 2 * H) dst_out[r * H + (i - H)] = v[0];
    }
}

// Source score half of every stored row; run once per table and layer: a streaming pass over the table.
// G lanes (a power of two) share a row, each taking every G-th 16-byte piece, up to four of them (G is the smallest
// power of two with 4 G >= pieces of a row): the sums of a row are then folded over few lanes, and the cross-lane
// steps - the part of this kernel that is not streaming - are spread over four times as many bytes as with one
// piece per lane.  The folded vectors sit in LDS, zero-padded to 4 G pieces, and every 16 bytes of them are read once
// for all the rows a lane has in flight; loads are unconditional (a piece or a row beyond the end reads a valid
// place: the piece meets zeros of the folded vectors, the row is not stored), so the loop body has no branches.
// Two row steps are in flight per wavefront (8 KB of a 512-byte-row table).
template <int G, int H>
__device__ inline void group_sum(float (&s)[H]) {
#pragma unroll
    for (int off = G >> 1; off > 0; off >>= 1)
#pragma unroll
        for (int h = 0; h < H; ++h) s[h] += __shfl_xor(s[h], off);
}

template <int EPC, int H>
__global__ __launch_bounds__(256) void k_table_logits(const void* __restrict__ table, int64_t ld, int64_t n_rows, int dim,
                                                      int G, const float* __restrict__ fold_src,
                                                      float* __restrict__ out) {
    extern __shared__ __attribute__((aligned(16))) float fs[];   // [H][4 G * EPC]
    constexpr int U = 2, NPL = 4;
    const int n_pieces = (dim + EPC - 1) / EPC;
    const int fw = NPL * G * EPC;
    for (int i = threadIdx.x; i < H * fw; i += 256) {
        const int h = i / fw, k = i - h * fw;
        fs[i] = k < dim ? fold_src[h * dim + k] : 0.f;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int grp = lane / G, sub = lane - grp * G;
    const int rows_per_wave = 64 / G;
    const int64_t wave = (int64_t)blockIdx.x * (256 / 64) + (threadIdx.x >> 6);
    const int64_t n_waves = (int64_t)gridDim.x * (256 / 64);
    const int64_t step = n_waves * rows_per_wave;
    int poff[NPL];                                        // element offset of this lane's pieces inside a row
#pragma unroll
    for (int j = 0; j < NPL; ++j) {
        const int p = sub + G * j;
        poff[j] = (p < n_pieces ? p : 0) * EPC;
    }
#pragma unroll 1
    for (int64_t r0 = wave * rows_per_wave; r0 < n_rows; r0 += U * step) {
        float xv[U][NPL][EPC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int64_t r = r0 + u * step + grp;
            r = r < n_rows ? r : n_rows - 1;
#pragma unroll
            for (int j = 0; j < NPL; ++j) {
                if constexpr (EPC == 4) {
                    const float4 x = *reinterpret_cast<const float4*>(static_cast<const float*>(table) + r * ld + poff[j]);
                    xv[u][j][0] = x.x; xv[u][j][1] = x.y; xv[u][j][2] = x.z; xv[u][j][3] = x.w;
                } else {
                    unpack_bf16x8(*reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(table) + r * ld + poff[j]), xv[u][j]);
                }
            }
        }
        // Where the folded vectors stay between the steps, by measurement: for a bf16 table in registers (the reads
        // below are loop invariants and the compiler hoists them: 128 registers for four heads, two wavefronts per
        // SIMD, 1.23 GB in 271 us against 310 us); for an fp32 table, whose pieces hold half as many elements, in
        // LDS, read again in every step (the opaque offset below keeps the reads in the loop: 185 us against 194 us).
        int fbase = 0;
        if constexpr (EPC == 4) asm volatile("" : "+v"(fbase));
        float s[U][H];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int h = 0; h < H; ++h) s[u][h] = 0.f;
#pragma unroll
        for (int j = 0; j < NPL; ++j) {
#pragma unroll
            for (int h = 0; h < H; ++h)
#pragma unroll
                for (int q = 0; q < EPC / 4; ++q) {
                    const float4 f = *reinterpret_cast<const float4*>(&fs[fbase + h * fw + (sub + G * j) * EPC + 4 * q]);
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        s[u][h] = fmaf(xv[u][j][4 * q], f.x, s[u][h]);
                        s[u][h] = fmaf(xv[u][j][4 * q + 1], f.y, s[u][h]);
                        s[u][h] = fmaf(xv[u][j][4 * q + 2], f.z, s[u][h]);
                        s[u][h] = fmaf(xv[u][j][4 * q + 3], f.w, s[u][h]);
                    }
                }
            // keeps the next piece's reads of the folded vectors behind this piece's arithmetic: hoisted to the top,
            // all of them together hold a hundred registers and halve the wavefronts per SIMD
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            switch (G) {                                   // the same in every lane
                case 64: group_sum<64, H>(s[u]); break;
                case 32: group_sum<32, H>(s[u]); break;
                case 16: group_sum<16, H>(s[u]); break;
                case 8: group_sum<8, H>(s[u]); break;
                case 4: group_sum<4, H>(s[u]); break;
                case 2: group_sum<2, H>(s[u]); break;
                default: break;
            }
            const int64_t r = r0 + u * step + grp;
            if (sub == 0 && r < n_rows) {
#pragma unroll
                for (int h = 0; h < H; ++h) out[r * H + h] = s[u][h];
            }
        }
    }
}

template <int EPC> struct Piece { float v[EPC]; };

template <int EPC>
__device__ inline void load_piece(const GatArgs& a, int dim4, int32_t col, int piece, Piece<EPC>& out) {
    if (col >= 0) {
        if constexpr (EPC == 4) {
            const float4 r = *reinterpret_cast<const float4*>(static_cast<const float*>(a.table) + (int64_t)col * a.table_ld + piece * 4);
            out.v[0] = r.x; out.v[1] = r.y; out.v[2] = r.z; out.v[3] = r.w;
        } else {
            unpack_bf16x8(*reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(a.table) + (int64_t)col * a.table_ld + piece * 8), out.v);
        }
    } else {
        const float* row = a.buf + (int64_t)(~col) * a.buf_ld + piece * EPC;
#pragma unroll
        for (int g = 0; g < EPC / 4; ++g) {
            float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
            if (piece * EPC + g * 4 < dim4) r = *reinterpret_cast<const float4*>(row + g * 4);
            out.v[g * 4 + 0] = r.x; out.v[g * 4 + 1] = r.y; out.v[g * 4 + 2] = r.z; out.v[g * 4 + 3] = r.w;
        }
    }
}

template <int EPC, int G, int NP, int U, int H>
__global__ __launch_bounds__(WAVES_PER_BLOCK * 64) void k_gat(GatArgs a) {
    __shared__ float p_lds[WAVES_PER_BLOCK][H][OMG_PART_EDGES];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t part = (int64_t)blockIdx.x * WAVES_PER_BLOCK + wave;
    if (part >= a.n_parts) return;                 // no block-wide barrier below
    const int v = a.part_row[part];
    const int first_part = a.part_ptr[v];
    const bool whole = (a.part_ptr[v + 1] - first_part) == 1;
    const int64_t row_beg = a.indptr[v], row_end = a.indptr[v + 1];
    const int64_t e0 = row_beg + (int64_t)(part - first_part) * omg_row_part(row_end - row_beg, a.part_edges);
    const int64_t e1 = (e0 + omg_row_part(row_end - row_beg, a.part_edges) < row_end) ? e0 + omg_row_part(row_end - row_beg, a.part_edges) : row_end;
    const int ne = (int)(e1 - e0);

    // ---- the rows of the first edges are asked for before anything else: they need the column ids only, and their
    // trip to memory then overlaps the one of the scores below instead of following it
    constexpr int EPI = 64 / G;
    const int grp = lane / G, sub = lane % G;
    const int n_pieces = (a.dim + EPC - 1) / EPC;
    const int dim4 = (a.dim + 3) & ~3;
    const int n_first = ne < 64 ? ne : 64;
    const int32_t col_first = lane < n_first ? a.cols[e0 + lane] : 0;
    Piece<EPC> x[U][NP];
    auto fetch_rows = [&](int n, int j, int32_t my_col) {       // edges j + u EPI + grp of a block of n <= 64 edges
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int idx = j + u * EPI + grp;
            const int src_lane = idx < 64 ? idx : 63;
            const int32_t c = __shfl(my_col, src_lane);
            const bool ok = idx < n;
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                const int piece = sub + p * 64;
                if (ok && piece < n_pieces) {
                    load_piece<EPC>(a, dim4, c, piece, x[u][p]);
                } else {
#pragma unroll
                    for (int i = 0; i < EPC; ++i) x[u][p].v[i] = 0.f;
                }
            }
        }
    };
    fetch_rows(n_first, 0, col_first);

    // ---- scores of this part's edges -> LDS, then exp(score - max) and its sum
    float dl[H], mx[H], sm[H];
#pragma unroll
    for (int h = 0; h < H; ++h) {
        dl[h] = a.dst_logits[(int64_t)v * H + h];
        mx[h] = -INFINITY;
        sm[h] = 0.f;
    }
    for (int i = lane; i < ne; i += 64) {
        const int32_t c = i < 64 ? col_first : a.cols[e0 + i];
        const float* sl = c >= 0 ? a.src_logits + (int64_t)c * H : a.buf_logits + (int64_t)(~c) * H;
#pragma unroll
        for (int h = 0; h < H; ++h) {
            float e = sl[h] + dl[h];
            e = e > 0.f ? e : a.leaky * e;
            p_lds[wave][h][i] = e;
            mx[h] = fmaxf(mx[h], e);
        }
    }
#pragma unroll
    for (int h = 0; h < H; ++h) mx[h] = wave_max(mx[h]);
    for (int i = lane; i < ne; i += 64) {
#pragma unroll
        for (int h = 0; h < H; ++h) {
            const float p = __expf(p_lds[wave][h][i] - mx[h]);     // same lane wrote this slot
            p_lds[wave][h][i] = p;
            sm[h] += p;
        }
    }
#pragma unroll
    for (int h = 0; h < H; ++h) sm[h] = wave_sum(sm[h]);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- weighted gather
    float acc[H][NP][EPC];
#pragma unroll
    for (int h = 0; h < H; ++h)
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int i = 0; i < EPC; ++i) acc[h][p][i] = 0.f;

    for (int base = 0; base < ne; base += 64) {
        const int n = (ne - base < 64) ? (ne - base) : 64;
        int32_t my_col = col_first;
        if (base > 0) {
            my_col = 0;
            if (lane < n) my_col = a.cols[e0 + base + lane];
        }
        for (int j = 0; j < n; j += EPI * U) {
            if (base + j > 0) fetch_rows(n, j, my_col);
            float pw[U][H];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int idx = j + u * EPI + grp;
                const bool ok = idx < n;
#pragma unroll
                for (int h = 0; h < H; ++h) pw[u][h] = ok ? p_lds[wave][h][base + idx] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int h = 0; h < H; ++h)
#pragma unroll
                    for (int p = 0; p < NP; ++p)
#pragma unroll
                        for (int i = 0; i < EPC; ++i) acc[h][p][i] = fmaf(pw[u][h], x[u][p].v[i], acc[h][p][i]);
        }
    }
#pragma unroll
    for (int off = G; off < 64; off <<= 1)
#pragma unroll
        for (int h = 0; h < H; ++h)
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int i = 0; i < EPC; ++i) acc[h][p][i] += __shfl_xor(acc[h][p][i], off);
    if (grp != 0) return;

    const int64_t pstride = (int64_t)H * a.agg_ld + PART_PAD;
    float* dst = whole ? a.agg + (int64_t)v * a.agg_stride : a.partial + part * pstride;
#pragma unroll
    for (int h = 0; h < H; ++h) {
        const float scale = (whole && !a.raw) ? (sm[h] > 0.f ? 1.f / sm[h] : 0.f) : 1.f;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int piece = sub + p * 64;
            if (piece >= n_pieces) continue;
#pragma unroll
            for (int g = 0; g < EPC / 4; ++g) {
                const int col0 = piece * EPC + g * 4;
                if (col0 >= a.agg_ld) continue;
                *reinterpret_cast<float4*>(dst + (int64_t)h * a.agg_ld + col0) =
                    make_float4(acc[h][p][g * 4] * scale, acc[h][p][g * 4 + 1] * scale, acc[h][p][g * 4 + 2] * scale,
                                acc[h][p][g * 4 + 3] * scale);
            }
        }
    }
    if ((!whole || a.raw) && lane == 0) {
#pragma unroll
        for (int h = 0; h < H; ++h) {
            dst[(int64_t)H * a.agg_ld + h] = mx[h];
            dst[(int64_t)H * a.agg_ld + OMG_GAT_STAT_SUM + h] = sm[h];
        }
        if (whole) dst[(int64_t)H * a.agg_ld + OMG_GAT_STAT_COUNT] = __int_as_float(ne);
    }
}

// Rows cut into parts: softmax merge (the two-step softmax of Sec. 6.2: every part carries its maximum score and
// its sum of exponentials, the merge rescales to the row's maximum).  Fixed order of additions, so reruns are
// bit-identical.  One launch, two block shapes:
//   rows of 2..OMG_MANY_PARTS parts  a block per row, a thread per (head, 16-byte column group); the thread takes the
//                                    row's maximum and rescaled exp-sum from the parts' statistics (a few floats
//                                    per part) and adds the parts' rescaled sums in part order;
//   longer rows                      a block per (row, head, 32 column groups): 8 thread groups that each add every
//                                    8th part, the 8 sums added in group order through LDS.
constexpr int COMB_COLS = 32, COMB_GROUPS = 8;

__device__ inline void gat_combine_few(const GatArgs& a, int v) {
    const int H = a.heads;
    const int p0 = a.part_ptr[v], np = a.part_ptr[v + 1] - p0;
    const int64_t pstride = (int64_t)H * a.agg_ld + PART_PAD;
    const int groups = (int)(a.agg_ld / 4);
    float* dst = a.agg + (int64_t)v * a.agg_stride;
    for (int i = threadIdx.x; i < H * groups; i += COMB_COLS * COMB_GROUPS) {
        const int h = i / groups, c4 = (i - h * groups) * 4;
        const float* part = a.partial + (int64_t)p0 * pstride;
        float mx[OMG_MANY_PARTS], sm[OMG_MANY_PARTS];
        float M = -INFINITY;
#pragma unroll
        for (int p = 0; p < OMG_MANY_PARTS; ++p) {
            mx[p] = p < np ? part[p * pstride + (int64_t)H * a.agg_ld + h] : -INFINITY;
            sm[p] = p < np ? part[p * pstride + (int64_t)H * a.agg_ld + OMG_GAT_STAT_SUM + h] : 0.f;
            M = fmaxf(M, mx[p]);
        }
        float S = 0.f;
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int p = 0; p < OMG_MANY_PARTS; ++p) {
            if (p < np) {
                const float f = __expf(mx[p] - M);
                S = fmaf(sm[p], f, S);
                const float4 x = *reinterpret_cast<const float4*>(part + p * pstride + (int64_t)h * a.agg_ld + c4);
                s.x = fmaf(f, x.x, s.x); s.y = fmaf(f, x.y, s.y); s.z = fmaf(f, x.z, s.z); s.w = fmaf(f, x.w, s.w);
            }
        }
        if (a.raw) {
            // a partition's record: the sums stay relative to the row's local maximum M, which goes along with S
            if (c4 == 0) {
                dst[(int64_t)H * a.agg_ld + h] = M;
                dst[(int64_t)H * a.agg_ld + OMG_GAT_STAT_SUM + h] = S;
                if (h == 0) dst[(int64_t)H * a.agg_ld + OMG_GAT_STAT_COUNT] = __int_as_float((int)(a.indptr[v + 1] - a.indptr[v]));
            }
        } else {
            const float inv = S > 0.f ? 1.f / S : 0.f;
            s.x *= inv; s.y *= inv; s.z *= inv; s.w *= inv;
        }
        *reinterpret_cast<float4*>(dst + (int64_t)h * a.agg_ld + c4) = s;
    }
}

__device__ inline void gat_combine_many(const GatArgs& a, int v, int h, int chunk, float4 (*red)[COMB_COLS], float* wred) {
    const int H = a.heads;
    const int col = threadIdx.x % COMB_COLS, grp = threadIdx.x / COMB_COLS;
    const int c4 = (chunk * COMB_COLS + col) * 4;
    const int p0 = a.part_ptr[v], p1 = a.part_ptr[v + 1];
    const int64_t pstride = (int64_t)H * a.agg_ld + PART_PAD;
    const float* stats = a.partial + (int64_t)H * a.agg_ld;       // + p * pstride: [h] max, [OMG_GAT_STAT_SUM + h] exp-sum
    // row maximum and rescaled exp-sum over all parts: one part per thread, fixed reduction tree
    constexpr int NW = COMB_COLS * COMB_GROUPS / 64;
    float m_loc = -INFINITY;
    for (int p = p0 + (int)threadIdx.x; p < p1; p += COMB_COLS * COMB_GROUPS) m_loc = fmaxf(m_loc, stats[p * pstride + h]);
    m_loc = wave_max(m_loc);
    if ((threadIdx.x & 63) == 0) wred[threadIdx.x >> 6] = m_loc;
    __syncthreads();
    float M = wred[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) M = fmaxf(M, wred[w]);
    __syncthreads();
    float s_loc = 0.f;
    for (int p = p0 + (int)threadIdx.x; p < p1; p += COMB_COLS * COMB_GROUPS)
        s_loc += stats[p * pstride + OMG_GAT_STAT_SUM + h] * __expf(stats[p * pstride + h] - M);
    s_loc = wave_sum(s_loc);
    if ((threadIdx.x & 63) == 0) wred[threadIdx.x >> 6] = s_loc;
    __syncthreads();
    float S = wred[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) S += wred[w];
    const bool live = c4 < a.agg_ld;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (live) {
        for (int p = p0 + grp; p < p1; p += COMB_GROUPS) {
            const float* t = a.partial + p * pstride;
            const float f = __expf(t[(int64_t)H * a.agg_ld + h] - M);
            const float4 x = *reinterpret_cast<const float4*>(t + (int64_t)h * a.agg_ld + c4);
            s.x = fmaf(f, x.x, s.x); s.y = fmaf(f, x.y, s.y); s.z = fmaf(f, x.z, s.z); s.w = fmaf(f, x.w, s.w);
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
    float* dst = a.agg + (int64_t)v * a.agg_stride;
    if (a.raw) {
        if (chunk == 0 && col == 0) {
            dst[(int64_t)H * a.agg_ld + h] = M;
            dst[(int64_t)H * a.agg_ld + OMG_GAT_STAT_SUM + h] = S;
            if (h == 0) dst[(int64_t)H * a.agg_ld + OMG_GAT_STAT_COUNT] = __int_as_float((int)(a.indptr[v + 1] - a.indptr[v]));
        }
    } else {
        const float inv = S > 0.f ? 1.f / S : 0.f;
        s.x *= inv; s.y *= inv; s.z *= inv; s.w *= inv;
    }
    *reinterpret_cast<float4*>(dst + (int64_t)h * a.agg_ld + c4) = s;
}

// blocks [0, n_split): one short row each; then (long row, head, column chunk) in that nesting
__global__ __launch_bounds__(COMB_COLS * COMB_GROUPS) void k_gat_combine(GatArgs a, int n_chunks) {
    __shared__ float4 red[COMB_GROUPS][COMB_COLS];
    __shared__ float wred[COMB_COLS * COMB_GROUPS / 64];
    const int64_t b = blockIdx.x;
    if (b < a.n_split) {
        gat_combine_few(a, a.split_rows[b]);
    } else {
        const int64_t i = b - a.n_split;
        const int per_row = a.heads * n_chunks;
        const int64_t r = i / per_row;
        const int rest = (int)(i - r * per_row);
        gat_combine_many(a, a.split_big[r], rest / n_chunks, rest % n_chunks, red, wred);
    }
}

template <int EPC, int G, int NP, int U>
int launch_heads(const GatArgs& a, hipStream_t s) {
    const unsigned grid = (unsigned)((a.n_parts + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
    const dim3 blk(WAVES_PER_BLOCK * 64);
    switch (a.heads) {
        case 1: hipLaunchKernelGGL((k_gat<EPC, G, NP, U, 1>), dim3(grid), blk, 0, s, a); break;
        case 2: hipLaunchKernelGGL((k_gat<EPC, G, NP, U, 2>), dim3(grid), blk, 0, s, a); break;
        case 4: hipLaunchKernelGGL((k_gat<EPC, G, NP, (U > 2 ? U / 2 : U), 4>), dim3(grid), blk, 0, s, a); break;
        case 8:
            // eight accumulators per value: the widest rows (more than 1,024 values) do not fit the register file
            if constexpr (NP * EPC <= 16) hipLaunchKernelGGL((k_gat<EPC, G, NP, (U > 2 ? 2 : 1), 8>), dim3(grid), blk, 0, s, a);
            else return OMG_EUNSUPPORTED;
            break;
        default: return OMG_EUNSUPPORTED;
    }
    return OMG_OK;
}

template <int EPC>
int launch_dtype(const GatArgs& a, hipStream_t s) {
    const int n_pieces = (a.dim + EPC - 1) / EPC;
    if (n_pieces <= 8) return launch_heads<EPC, 8, 1, 4>(a, s);
    if (n_pieces <= 16) return launch_heads<EPC, 16, 1, 4>(a, s);
    if (n_pieces <= 32) return launch_heads<EPC, 32, 1, 4>(a, s);
    if (n_pieces <= 64) return launch_heads<EPC, 64, 1, 4>(a, s);
    if (n_pieces <= 128) return launch_heads<EPC, 64, 2, 2>(a, s);
    if (n_pieces <= 256) return launch_heads<EPC, 64, 4, 2>(a, s);      // rows of up to 1,024 fp32 / 2,048 bf16 values
    return OMG_EUNSUPPORTED;
}

}  // namespace

int omg_launch_gat_fold(const omg_layer* L, float* fold_src, float* fold_dst, hipStream_t s) {
    const int n = L->heads * L->d_in;
    hipLaunchKernelGGL(k_fold, dim3((n + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK), dim3(256), 0, s, L->W_nb, L->a_src, L->a_dst, L->d_in, L->d_out,
                       L->heads, fold_src, fold_dst);
    OMG_HIP(hipGetLastError());
    return OMG_OK;
}

template <int EPC>
static int launch_table_logits(const omg_table* t, const float* fold_src, int heads, float* logits, hipStream_t s) {
    const int n_pieces = (t->dim + EPC - 1) / EPC;
    int G = 1;
    while (G < 64 && 4 * G < n_pieces) G <<= 1;
    const int64_t rows_per_block = (int64_t)(256 / 64) * (64 / G);
    int64_t blocks = (t->n_rows + rows_per_block - 1) / rows_per_block;
    if (blocks > 8192) blocks = 8192;                    // the rest by the kernel's stride loop
    const size_t lds = sizeof(float) * (size_t)heads * (size_t)(4 * G) * EPC;          // zero-padded to 4 G pieces
    if (lds > 64 * 1024 || n_pieces > 256) return OMG_EUNSUPPORTED;      // a lane takes at most four pieces of a row
    const dim3 g((unsigned)blocks), b(256);
    switch (heads) {
        case 1: hipLaunchKernelGGL((k_table_logits<EPC, 1>), g, b, lds, s, t->data, t->ld, t->n_rows, t->dim, G, fold_src, logits); break;
        case 2: hipLaunchKernelGGL((k_table_logits<EPC, 2>), g, b, lds, s, t->data, t->ld, t->n_rows, t->dim, G, fold_src, logits); break;
        case 4: hipLaunchKernelGGL((k_table_logits<EPC, 4>), g, b, lds, s, t->data, t->ld, t->n_rows, t->dim, G, fold_src, logits); break;
        case 8: hipLaunchKernelGGL((k_table_logits<EPC, 8>), g, b, lds, s, t->data, t->ld, t->n_rows, t->dim, G, fold_src, logits); break;
        default: return OMG_EUNSUPPORTED;
    }
    return OMG_OK;
}

int omg_launch_table_logits(const omg_table* t, const float* fold_src, int heads, float* logits, hipStream_t s) {
    if (t->n_rows <= 0) return OMG_OK;
    OMG_TRY(t->dtype == OMG_F32 ? launch_table_logits<4>(t, fold_src, heads, logits, s)
                                : launch_table_logits<8>(t, fold_src, heads, logits, s));
    OMG_HIP(hipGetLastError());
    return OMG_OK;
}

int omg_launch_gat(const GatArgs& a_in, hipStream_t s, hipEvent_t after_main) {
    GatArgs a = a_in;
    if (a.agg_stride == 0) a.agg_stride = (int64_t)a.heads * a.agg_ld;
    if (a.raw && a.agg_stride < (int64_t)a.heads * a.agg_ld + OMG_GAT_STAT_PAD) return OMG_EINVAL;
    const size_t fold_lds = sizeof(float) * 2 * (size_t)a.heads * (size_t)((a.dim + 3) & ~3);
    if (a.n_buf_rows > 0 && fold_lds <= 48 * 1024) {
        const dim3 g((unsigned)((a.n_buf_rows + 15) / 16)), b(256);
        switch (a.heads) {
            case 1: hipLaunchKernelGGL(k_buf_logits16<1>, g, b, fold_lds, s, a.buf, a.buf_ld, a.n_buf_rows, a.dim, a.fold_src, a.fold_dst, a.buf_logits, a.dst_logits); break;
            case 2: hipLaunchKernelGGL(k_buf_logits16<2>, g, b, fold_lds, s, a.buf, a.buf_ld, a.n_buf_rows, a.dim, a.fold_src, a.fold_dst, a.buf_logits, a.dst_logits); break;
            case 4: hipLaunchKernelGGL(k_buf_logits16<4>, g, b, fold_lds, s, a.buf, a.buf_ld, a.n_buf_rows, a.dim, a.fold_src, a.fold_dst, a.buf_logits, a.dst_logits); break;
            case 8: hipLaunchKernelGGL(k_buf_logits16<8>, g, b, fold_lds, s, a.buf, a.buf_ld, a.n_buf_rows, a.dim, a.fold_src, a.fold_dst, a.buf_logits, a.dst_logits); break;
            default: return OMG_EUNSUPPORTED;
        }
    } else if (a.n_buf_rows > 0) {
        const unsigned grid = (unsigned)((a.n_buf_rows + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
        const dim3 g(grid), b(256);
        switch (a.heads) {
            case 1: hipLaunchKernelGGL(k_buf_logits<1>, g, b, 0, s, a.buf, a.buf_ld, a.n_buf_rows, a.dim, a.fold_src, a.fold_dst, a.buf_logits, a.dst_logits); break;
            case 2: hipLaunchKernelGGL(k_buf_logits<2>, g, b, 0, s, a.buf, a.buf_ld, a.n_buf_rows, a.dim, a.fold_src, a.fold_dst, a.buf_logits, a.dst_logits); break;
            case 4: hipLaunchKernelGGL(k_buf_logits<4>, g, b, 0, s, a.buf, a.buf_ld, a.n_buf_rows, a.dim, a.fold_src, a.fold_dst, a.buf_logits, a.dst_logits); break;
            case 8: hipLaunchKernelGGL(k_buf_logits<8>, g, b, 0, s, a.buf, a.buf_ld, a.n_buf_rows, a.dim, a.fold_src, a.fold_dst, a.buf_logits, a.dst_logits); break;
            default: return OMG_EUNSUPPORTED;
        }
    }
    int rc = OMG_OK;
    if (a.n_parts > 0) rc = (a.table_dtype == OMG_F32) ? launch_dtype<4>(a, s) : launch_dtype<8>(a, s);
    if (rc != OMG_OK) return rc;
    if (after_main != nullptr) OMG_HIP(hipEventRecord(after_main, s));
    if (a.n_split + a.n_split_big > 0) {
        const int n_chunks = (int)((a.agg_ld / 4 + COMB_COLS - 1) / COMB_COLS);
        const int64_t blocks = a.n_split + a.n_split_big * a.heads * n_chunks;
        hipLaunchKernelGGL(k_gat_combine, dim3((unsigned)blocks), dim3(COMB_COLS * COMB_GROUPS), 0, s, a, n_chunks);
    }
    OMG_HIP(hipGetLastError());
    return OMG_OK;
}
