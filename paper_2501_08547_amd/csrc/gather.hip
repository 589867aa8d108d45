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
//
// The reduction is one of (Sec. 6.2 names the forms beyond the plain sum / mean): mean, GCN's
// degree-weighted sum with self term, sum, max, sum of p-th powers of positive messages (power
// mean), sum of n-th powers of differences from the row's mean (normalised moment; the mean is a
// first pass of this same kernel).  Parts are the "local aggregations" of that section and the
// second kernel is its merge function: add (or maximise), then scale / take the root.
#include "internal.h"

namespace {

constexpr int WAVES_PER_BLOCK = 4;

enum { OP_MEAN = OMG_OP_MEAN, OP_GCN = OMG_OP_GCN, OP_SUM = OMG_OP_SUM, OP_MAX = OMG_OP_MAX, OP_POW = OMG_OP_POW,
       OP_MOM = OMG_OP_MOM };

// d^n for even n >= 2
__device__ inline float even_power(float d, int n) {
    const float t = d * d;
    float r = t;
    for (int k = 2; k < n; k += 2) r *= t;
    return r;
}

// what a finished row holds, from the merged sum s (or maximum) and the row's edge count
template <int OP>
__device__ inline float finish_value(float s, float deg, float agg_p) {
    if constexpr (OP == OP_MEAN) return deg > 0.f ? s / deg : 0.f;
    if constexpr (OP == OP_MAX) return deg > 0.f ? s : 0.f;
    if constexpr (OP == OP_POW || OP == OP_MOM) return deg > 0.f ? __powf(s / deg, 1.f / agg_p) : 0.f;
    return s;
}

struct F8 { float v[8]; };

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
template <int EPC, int G, int NP, int U, int OP>
__global__ __launch_bounds__(WAVES_PER_BLOCK * 64) void k_gather(GatherArgs a) {
    const int lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x >> 6);
    if (item >= a.n_parts) return;
    const int64_t part = a.order != nullptr ? a.order[item] : item;
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
        for (int i = 0; i < EPC; ++i) acc[p][i] = OP == OP_MAX ? -INFINITY : 0.f;
    // normalised moment: this lane's pieces of the row's mean (the first pass's result)
    float mu[OP == OP_MOM ? NP : 1][EPC];
    if constexpr (OP == OP_MOM) {
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int piece = sub + p * 64;
#pragma unroll
            for (int g = 0; g < EPC / 4; ++g) {
                float4 m4 = make_float4(0.f, 0.f, 0.f, 0.f);
                if (piece < n_pieces && piece * EPC + g * 4 < a.agg_ld)
                    m4 = *reinterpret_cast<const float4*>(a.mean + (int64_t)v * a.mean_ld + piece * EPC + g * 4);
                mu[p][g * 4] = m4.x; mu[p][g * 4 + 1] = m4.y; mu[p][g * 4 + 2] = m4.z; mu[p][g * 4 + 3] = m4.w;
            }
        }
    }
    const int mom_n = (int)a.agg_p;

    for (int64_t base = e0; base < e1; base += 64) {
        const int n = (int)((e1 - base < 64) ? (e1 - base) : 64);
        int32_t my_col = 0;
        float my_w = 0.f;
        if (lane < n) {
            my_col = a.cols[base + lane];
            if constexpr (OP == OP_GCN) my_w = rsqrtf((float)(a.cdeg[base + lane] + 1) * (a.raw ? 1.f : row_d1));
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
                        const float xv = x[u][p].v[i];
                        if constexpr (OP == OP_GCN) acc[p][i] = fmaf(w[u], xv, acc[p][i]);
                        else if constexpr (OP == OP_MAX) acc[p][i] = w[u] != 0.f ? fmaxf(acc[p][i], xv) : acc[p][i];
                        else if constexpr (OP == OP_POW) acc[p][i] += w[u] * __powf(fmaxf(xv, 0.f) + a.agg_eps, a.agg_p);
                        else if constexpr (OP == OP_MOM) acc[p][i] += w[u] * even_power(xv - mu[p][i], mom_n);
                        else acc[p][i] += w[u] * xv;
                    }
        }
    }

    // fold the 64 / G groups of the wavefront into group 0
#pragma unroll
    for (int off = G; off < 64; off <<= 1)
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int i = 0; i < EPC; ++i) {
                const float o = __shfl_xor(acc[p][i], off);
                acc[p][i] = OP == OP_MAX ? fmaxf(acc[p][i], o) : acc[p][i] + o;
            }

    if (grp != 0) return;
    const bool whole = n_row_parts == 1;
    const float deg_f = (float)(row_end - row_beg);
    float* dst = whole ? a.agg + (int64_t)v * a.agg_stride : a.partial + part * a.agg_ld;
    const bool finish = whole && !a.raw;       // raw: the row's local aggregation is stored as it is
    if (whole && a.raw && sub == 0) dst[a.agg_ld] = __int_as_float((int)(row_end - row_beg));
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int piece = sub + p * 64;
        if (piece >= n_pieces) continue;
#pragma unroll
        for (int g = 0; g < EPC / 4; ++g) {
            const int col0 = piece * EPC + g * 4;
            if (col0 >= a.agg_ld) continue;
            float4 o = make_float4(acc[p][g * 4], acc[p][g * 4 + 1], acc[p][g * 4 + 2], acc[p][g * 4 + 3]);
            if (finish && OP != OP_GCN && OP != OP_SUM) {
                o.x = finish_value<OP>(o.x, deg_f, a.agg_p); o.y = finish_value<OP>(o.y, deg_f, a.agg_p);
                o.z = finish_value<OP>(o.z, deg_f, a.agg_p); o.w = finish_value<OP>(o.w, deg_f, a.agg_p);
            }
            if (finish && OP == OP_GCN && col0 < dim4) {
                const float4 sv = *reinterpret_cast<const float4*>(a.buf + (int64_t)v * a.buf_ld + col0);
                const float inv = 1.f / row_d1;
                o.x += sv.x * inv; o.y += sv.y * inv; o.z += sv.z * inv; o.w += sv.w * inv;
                if (a.h0 != nullptr) {            // GCNII: mix with the row's layer-0 value
                    const float4 h = *reinterpret_cast<const float4*>(a.h0 + (int64_t)v * a.h0_ld + col0);
                    const float k1 = 1.f - a.alpha;
                    o.x = k1 * o.x + a.alpha * h.x; o.y = k1 * o.y + a.alpha * h.y;
                    o.z = k1 * o.z + a.alpha * h.z; o.w = k1 * o.w + a.alpha * h.w;
                }
            }
            *reinterpret_cast<float4*>(dst + col0) = o;
        }
    }
}

// Short work items (rows of a few edges, most rows of a power-law batch): a wavefront of k_gather above spends its
// life in the chain work item -> row -> row pointers -> column ids -> rows for a dozen edges, and the launch is that
// chain times the number of rounds of wavefronts.  Here a wavefront takes 64 / G work items at once, one per group of
// G lanes (G lanes cover a row; rows of up to 32 pieces), each group walking its own edges with U of them in flight:
// a half to an eighth of the wavefronts, the same loads in flight in each.  No sums cross the groups.
template <int EPC, int G, int U, int OP>
__global__ __launch_bounds__(WAVES_PER_BLOCK * 64) void k_gather_multi(GatherArgs a) {
    constexpr int PPW = 64 / G;                 // work items per wavefront
    const int lane = threadIdx.x & 63;
    const int grp = lane / G, sub = lane % G;
    const int64_t wave = (int64_t)blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x >> 6);
    if (wave * PPW >= a.n_parts) return;
    const int64_t item = wave * PPW + grp;
    const bool live = item < a.n_parts;
    const int64_t part = live ? (a.order != nullptr ? a.order[item] : item) : 0;
    const int v = a.part_row[part];
    const int first_part = a.part_ptr[v];
    const int n_row_parts = a.part_ptr[v + 1] - first_part;
    const int64_t row_beg = a.indptr[v], row_end = a.indptr[v + 1];
    const int ps = omg_row_part(row_end - row_beg, a.part_edges);
    const int64_t e0 = row_beg + (int64_t)(part - first_part) * ps;
    const int64_t e1 = !live ? e0 : (e0 + ps < row_end ? e0 + ps : row_end);
    const float row_d1 = (float)(row_end - row_beg + 1);
    const int n_pieces = (a.dim + EPC - 1) / EPC;
    const int dim4 = (a.dim + 3) & ~3;
    const bool has_piece = sub < n_pieces;

    float acc[EPC];
#pragma unroll
    for (int i = 0; i < EPC; ++i) acc[i] = OP == OP_MAX ? -INFINITY : 0.f;
    float mu[EPC];
#pragma unroll
    for (int i = 0; i < EPC; ++i) mu[i] = 0.f;
    if constexpr (OP == OP_MOM) {
#pragma unroll
        for (int g = 0; g < EPC / 4; ++g) {
            float4 m4 = make_float4(0.f, 0.f, 0.f, 0.f);
            if (has_piece && sub * EPC + g * 4 < a.agg_ld)
                m4 = *reinterpret_cast<const float4*>(a.mean + (int64_t)v * a.mean_ld + sub * EPC + g * 4);
            mu[g * 4] = m4.x; mu[g * 4 + 1] = m4.y; mu[g * 4 + 2] = m4.z; mu[g * 4 + 3] = m4.w;
        }
    }
    const int mom_n = (int)a.agg_p;

    // every group walks its own edges, G column ids at a time; the loop runs as long as any group has edges left
    int rounds = (int)((e1 - e0 + G - 1) / G);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) rounds = max(rounds, __shfl_xor(rounds, off));
    for (int it = 0; it < rounds; ++it) {
        const int64_t base = e0 + (int64_t)it * G;
        const int n = base < e1 ? (int)((e1 - base < G) ? (e1 - base) : G) : 0;
        int32_t my_col = 0;
        float my_w = 0.f;
        if (sub < n) {
            my_col = a.cols[base + sub];
            if constexpr (OP == OP_GCN) my_w = rsqrtf((float)(a.cdeg[base + sub] + 1) * (a.raw ? 1.f : row_d1));
            else my_w = 1.f;
        }
        int n_max = n;                                    // the wavefront's longest chunk bounds the inner loop
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) n_max = max(n_max, __shfl_xor(n_max, off));
        for (int j = 0; j < n_max; j += U) {
            Piece<EPC> x[U];
            float w[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int idx = j + u;
                const int src_lane = grp * G + (idx < G ? idx : G - 1);
                const int32_t c = __shfl(my_col, src_lane);
                const float wu = __shfl(my_w, src_lane);
                w[u] = (idx < n) ? wu : 0.f;
                if (idx < n && has_piece) {
                    load_piece<EPC>(a.table, a.table_ld, a.buf, a.buf_ld, dim4, c, sub, x[u]);
                } else {
#pragma unroll
                    for (int i = 0; i < EPC; ++i) x[u].v[i] = 0.f;
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < EPC; ++i) {
                    const float xv = x[u].v[i];
                    if constexpr (OP == OP_GCN) acc[i] = fmaf(w[u], xv, acc[i]);
                    else if constexpr (OP == OP_MAX) acc[i] = w[u] != 0.f ? fmaxf(acc[i], xv) : acc[i];
                    else if constexpr (OP == OP_POW) acc[i] += w[u] * __powf(fmaxf(xv, 0.f) + a.agg_eps, a.agg_p);
                    else if constexpr (OP == OP_MOM) acc[i] += w[u] * even_power(xv - mu[i], mom_n);
                    else acc[i] += w[u] * xv;
                }
        }
    }
    if (!live || !has_piece) return;
    const bool whole = n_row_parts == 1;
    const float deg_f = (float)(row_end - row_beg);
    float* dst = whole ? a.agg + (int64_t)v * a.agg_stride : a.partial + part * a.agg_ld;
    const bool finish = whole && !a.raw;       // raw: the row's local aggregation is stored as it is
    if (whole && a.raw && sub == 0) dst[a.agg_ld] = __int_as_float((int)(row_end - row_beg));
#pragma unroll
    for (int g = 0; g < EPC / 4; ++g) {
        const int col0 = sub * EPC + g * 4;
        if (col0 >= a.agg_ld) continue;
        float4 o = make_float4(acc[g * 4], acc[g * 4 + 1], acc[g * 4 + 2], acc[g * 4 + 3]);
        if (finish && OP != OP_GCN && OP != OP_SUM) {
            o.x = finish_value<OP>(o.x, deg_f, a.agg_p); o.y = finish_value<OP>(o.y, deg_f, a.agg_p);
            o.z = finish_value<OP>(o.z, deg_f, a.agg_p); o.w = finish_value<OP>(o.w, deg_f, a.agg_p);
        }
        if (finish && OP == OP_GCN && col0 < dim4) {
            const float4 sv = *reinterpret_cast<const float4*>(a.buf + (int64_t)v * a.buf_ld + col0);
            const float inv = 1.f / row_d1;
            o.x += sv.x * inv; o.y += sv.y * inv; o.z += sv.z * inv; o.w += sv.w * inv;
            if (a.h0 != nullptr) {            // GCNII: mix with the row's layer-0 value
                const float4 h = *reinterpret_cast<const float4*>(a.h0 + (int64_t)v * a.h0_ld + col0);
                const float k1 = 1.f - a.alpha;
                o.x = k1 * o.x + a.alpha * h.x; o.y = k1 * o.y + a.alpha * h.y;
                o.z = k1 * o.z + a.alpha * h.z; o.w = k1 * o.w + a.alpha * h.w;
            }
        }
        *reinterpret_cast<float4*>(dst + col0) = o;
    }
}

// Rows cut into several parts: add up the partial sums, then scale / add the self term.  The order
// of additions is fixed, so the result does not depend on scheduling.  Two shapes:
//   combine_few     rows of 2..OMG_MANY_PARTS parts: a thread per (row, 16-byte column group), rows packed
//                   into the blocks one after the other (a block per row leaves 3 of 4 lanes idle on
//                   rows of 256 values), the parts fetched together and added in part order;
//   combine_many    longer rows: a block per (row, 32 column groups), 8 thread groups that each add
//                   every 8th part, then the 8 sums added in group order through LDS.
template <int OP>
__device__ inline void finish_row(const GatherArgs& a, int v, int c4, float4 s) {
    const int64_t deg = a.indptr[v + 1] - a.indptr[v];
    if (a.raw) {
        float* dst = a.agg + (int64_t)v * a.agg_stride;
        *reinterpret_cast<float4*>(dst + c4) = s;
        if (c4 == 0) dst[a.agg_ld] = __int_as_float((int)deg);
        return;
    }
    if constexpr (OP == OP_GCN) {
        if (c4 < ((a.dim + 3) & ~3)) {
            const float4 sv = *reinterpret_cast<const float4*>(a.buf + (int64_t)v * a.buf_ld + c4);
            const float inv = 1.f / (float)(deg + 1);
            s.x += sv.x * inv; s.y += sv.y * inv; s.z += sv.z * inv; s.w += sv.w * inv;
            if (a.h0 != nullptr) {
                const float4 h = *reinterpret_cast<const float4*>(a.h0 + (int64_t)v * a.h0_ld + c4);
                const float k1 = 1.f - a.alpha;
                s.x = k1 * s.x + a.alpha * h.x; s.y = k1 * s.y + a.alpha * h.y;
                s.z = k1 * s.z + a.alpha * h.z; s.w = k1 * s.w + a.alpha * h.w;
            }
        }
    } else if constexpr (OP != OP_SUM) {
        const float d = (float)deg;
        s.x = finish_value<OP>(s.x, d, a.agg_p); s.y = finish_value<OP>(s.y, d, a.agg_p);
        s.z = finish_value<OP>(s.z, d, a.agg_p); s.w = finish_value<OP>(s.w, d, a.agg_p);
    }
    *reinterpret_cast<float4*>(a.agg + (int64_t)v * a.agg_stride + c4) = s;
}

// the merge of two local aggregations
template <int OP>
__device__ inline void merge4(float4& s, const float4& t) {
    if constexpr (OP == OP_MAX) { s.x = fmaxf(s.x, t.x); s.y = fmaxf(s.y, t.y); s.z = fmaxf(s.z, t.z); s.w = fmaxf(s.w, t.w); }
    else { s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w; }
}
template <int OP>
__device__ inline float4 merge_identity() {
    const float z = OP == OP_MAX ? -INFINITY : 0.f;
    return make_float4(z, z, z, z);
}

template <int OP>
__device__ inline void combine_few(const GatherArgs& a, int64_t idx, int groups) {
    const int64_t j = idx / groups;                       // which of the short rows, which of its column groups
    if (j >= a.n_split) return;
    const int c4 = (int)(idx - j * groups) * 4;
    const int v = a.split_rows[j];
    const int p0 = a.part_ptr[v], np = a.part_ptr[v + 1] - p0;
    float4 t[OMG_MANY_PARTS];
#pragma unroll
    for (int i = 0; i < OMG_MANY_PARTS; ++i)
        t[i] = i < np ? *reinterpret_cast<const float4*>(a.partial + (int64_t)(p0 + i) * a.agg_ld + c4)
                      : merge_identity<OP>();
    float4 s = t[0];
#pragma unroll
    for (int i = 1; i < OMG_MANY_PARTS; ++i) merge4<OP>(s, t[i]);
    finish_row<OP>(a, v, c4, s);
}

constexpr int COMB_COLS = 32, COMB_GROUPS = 8;

template <int OP>
__device__ inline void combine_many(const GatherArgs& a, int v, int chunk, float4 (*red)[COMB_COLS]) {
    const int col = threadIdx.x % COMB_COLS, grp = threadIdx.x / COMB_COLS;
    const int c4 = (chunk * COMB_COLS + col) * 4;
    const int p0 = a.part_ptr[v], p1 = a.part_ptr[v + 1];
    const bool live = c4 < a.agg_ld;
    float4 s = merge_identity<OP>();
    if (live) {
        for (int p = p0 + grp; p < p1; p += COMB_GROUPS * 4) {
            float4 t[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                t[i] = (p + i * COMB_GROUPS < p1)
                           ? *reinterpret_cast<const float4*>(a.partial + (int64_t)(p + i * COMB_GROUPS) * a.agg_ld + c4)
                           : merge_identity<OP>();
#pragma unroll
            for (int i = 0; i < 4; ++i) merge4<OP>(s, t[i]);
        }
    }
    red[grp][col] = s;
    __syncthreads();
    if (grp != 0 || !live) return;
#pragma unroll
    for (int g2 = 1; g2 < COMB_GROUPS; ++g2) merge4<OP>(s, red[g2][col]);
    finish_row<OP>(a, v, c4, s);
}

// one launch for both shapes: the first nb_few blocks take the short rows (a thread per row and column group),
// the others one (long row, column chunk) each
template <int OP>
__global__ __launch_bounds__(COMB_COLS * COMB_GROUPS) void k_combine(GatherArgs a, int n_chunks, int64_t nb_few) {
    __shared__ float4 red[COMB_GROUPS][COMB_COLS];
    const int64_t b = blockIdx.x;
    if (b < nb_few) {
        combine_few<OP>(a, b * (COMB_COLS * COMB_GROUPS) + threadIdx.x, (int)(a.agg_ld / 4));
    } else {
        const int64_t r = (b - nb_few) / n_chunks;
        combine_many<OP>(a, a.split_big[r], (int)((b - nb_few) - r * n_chunks), red);
    }
}

template <int EPC, int G, int NP, int U>
int launch_shape(const GatherArgs& a, hipStream_t s) {
    const unsigned grid = (unsigned)((a.n_parts + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
    const dim3 g(grid), b(WAVES_PER_BLOCK * 64);
    switch (a.op) {
        case OP_MEAN: hipLaunchKernelGGL((k_gather<EPC, G, NP, U, OP_MEAN>), g, b, 0, s, a); break;
        case OP_GCN: hipLaunchKernelGGL((k_gather<EPC, G, NP, U, OP_GCN>), g, b, 0, s, a); break;
        case OP_SUM: hipLaunchKernelGGL((k_gather<EPC, G, NP, U, OP_SUM>), g, b, 0, s, a); break;
        case OP_MAX: hipLaunchKernelGGL((k_gather<EPC, G, NP, U, OP_MAX>), g, b, 0, s, a); break;
        case OP_POW: hipLaunchKernelGGL((k_gather<EPC, G, NP, U, OP_POW>), g, b, 0, s, a); break;
        case OP_MOM: hipLaunchKernelGGL((k_gather<EPC, G, NP, U, OP_MOM>), g, b, 0, s, a); break;
        default: return OMG_EINVAL;
    }
    return OMG_OK;
}

template <int EPC, int G, int U>
int launch_multi(const GatherArgs& a, hipStream_t s) {
    constexpr int PPW = 64 / G;
    const int64_t waves = (a.n_parts + PPW - 1) / PPW;
    const dim3 g((unsigned)((waves + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK)), b(WAVES_PER_BLOCK * 64);
    switch (a.op) {
        case OP_MEAN: hipLaunchKernelGGL((k_gather_multi<EPC, G, U, OP_MEAN>), g, b, 0, s, a); break;
        case OP_GCN: hipLaunchKernelGGL((k_gather_multi<EPC, G, U, OP_GCN>), g, b, 0, s, a); break;
        case OP_SUM: hipLaunchKernelGGL((k_gather_multi<EPC, G, U, OP_SUM>), g, b, 0, s, a); break;
        case OP_MAX: hipLaunchKernelGGL((k_gather_multi<EPC, G, U, OP_MAX>), g, b, 0, s, a); break;
        case OP_POW: hipLaunchKernelGGL((k_gather_multi<EPC, G, U, OP_POW>), g, b, 0, s, a); break;
        case OP_MOM: hipLaunchKernelGGL((k_gather_multi<EPC, G, U, OP_MOM>), g, b, 0, s, a); break;
        default: return OMG_EINVAL;
    }
    return OMG_OK;
}

template <int EPC>
int launch_dtype(const GatherArgs& a, hipStream_t s) {
    const int n_pieces = (a.dim + EPC - 1) / EPC;
    // Work items of, on average, at most half a part's edges, rows of at most 32 pieces, and several times more work
    // items than wavefronts fit the chip at once (below that, fewer wavefronts only means less in flight: measured
    // +14 us on a launch of 2.5 k work items, -9 us on one of 40 k): several per wavefront
    if (a.multi_ok && n_pieces <= 32 && a.n_parts >= a.multi_min_parts && a.nnz * 2 <= a.n_parts * (int64_t)a.part_edges) {
        if (n_pieces <= 8) return launch_multi<EPC, 8, 4>(a, s);
        if (n_pieces <= 16) return launch_multi<EPC, 16, 2>(a, s);
        return launch_multi<EPC, 32, 4>(a, s);
    }
    if (n_pieces <= 8) return launch_shape<EPC, 8, 1, 4>(a, s);
    if (n_pieces <= 16) return launch_shape<EPC, 16, 1, 2>(a, s);      // (two slots: eight wavefronts per SIMD instead of five)
    if (n_pieces <= 32) return launch_shape<EPC, 32, 1, 2>(a, s);
    if (n_pieces <= 64) return launch_shape<EPC, 64, 1, 4>(a, s);
    // (two edge slots, not four: 2 KB bf16 rows scattered over a 61 GB table, 0.456 -> 0.385 ms per launch; the kernel
    // then holds six wavefronts per SIMD instead of four, and one slot gives 0.405 ms)
    if (n_pieces <= 128) return launch_shape<EPC, 64, 2, 2>(a, s);
    if (n_pieces <= 192) return launch_shape<EPC, 64, 3, 4>(a, s);
    if (n_pieces <= 256) return launch_shape<EPC, 64, 4, 2>(a, s);
    return OMG_EUNSUPPORTED;
}

__global__ void k_init_buffer(InitBufferArgs a) {
    omg_init_buffer_rows(a, (int64_t)blockIdx.x, (int64_t)gridDim.x, (int)threadIdx.x, (int)blockDim.x);
}

}  // namespace

int omg_launch_gather(const GatherArgs& a_in, hipStream_t s, hipEvent_t after_main) {
    GatherArgs a = a_in;
    if (a.agg_stride == 0) a.agg_stride = a.agg_ld;
    if (a.mean_ld == 0) a.mean_ld = a.agg_ld;
    if (a.raw && a.agg_stride < a.agg_ld + 4) return OMG_EINVAL;      // a raw row is followed by its edge count
    int rc = OMG_OK;
    if (a.n_parts > 0) rc = (a.table_dtype == OMG_F32) ? launch_dtype<4>(a, s) : launch_dtype<8>(a, s);
    if (rc != OMG_OK) return rc;
    if (after_main != nullptr) OMG_HIP(hipEventRecord(after_main, s));
    if (a.n_split + a.n_split_big > 0) {
        const int n_chunks = (int)((a.agg_ld / 4 + COMB_COLS - 1) / COMB_COLS);
        const int64_t nb_few = (a.n_split * (a.agg_ld / 4) + COMB_COLS * COMB_GROUPS - 1) / (COMB_COLS * COMB_GROUPS);
        const int64_t n_blocks = nb_few + a.n_split_big * n_chunks;
        if (n_blocks >= ((int64_t)1 << 31)) return OMG_EUNSUPPORTED;
        const dim3 g((unsigned)n_blocks), b(COMB_COLS * COMB_GROUPS);
        switch (a.op) {
            case OP_MEAN: hipLaunchKernelGGL(k_combine<OP_MEAN>, g, b, 0, s, a, n_chunks, nb_few); break;
            case OP_GCN: hipLaunchKernelGGL(k_combine<OP_GCN>, g, b, 0, s, a, n_chunks, nb_few); break;
            case OP_SUM: hipLaunchKernelGGL(k_combine<OP_SUM>, g, b, 0, s, a, n_chunks, nb_few); break;
            case OP_MAX: hipLaunchKernelGGL(k_combine<OP_MAX>, g, b, 0, s, a, n_chunks, nb_few); break;
            case OP_POW: hipLaunchKernelGGL(k_combine<OP_POW>, g, b, 0, s, a, n_chunks, nb_few); break;
            case OP_MOM: hipLaunchKernelGGL(k_combine<OP_MOM>, g, b, 0, s, a, n_chunks, nb_few); break;
            default: return OMG_EINVAL;
        }
    }
    OMG_HIP(hipGetLastError());
    return OMG_OK;
}

int omg_launch_init_buffer(const omg_table* feat, const float* qf, int64_t ld_q, const omg_node_t* targets,
                           int32_t n_query, int64_t n_target, float* buf0, int64_t ld0, hipStream_t s) {
    const int64_t n_rows = (int64_t)n_query + n_target;
    if (n_rows <= 0) return OMG_OK;
    const InitBufferArgs a{feat->data, feat->dtype, feat->ld, feat->dim, qf, ld_q, targets, n_query, n_rows, nullptr, buf0, ld0};
    hipLaunchKernelGGL(k_init_buffer, dim3((unsigned)n_rows), dim3(128), 0, s, a);
    OMG_HIP(hipGetLastError());
    return OMG_OK;
}

// the number of targets is read on the device (the host does not know it yet); the blocks stride over the rows
int omg_launch_init_buffer_dev(const omg_table* feat, const float* qf, int64_t ld_q, const omg_node_t* targets,
                               int32_t n_query, const BuildCounts* counts, int64_t max_rows, float* buf0, int64_t ld0,
                               hipStream_t s) {
    if (max_rows <= 0) return OMG_OK;
    const int64_t grid = max_rows < 16384 ? max_rows : 16384;
    const InitBufferArgs a{feat->data, feat->dtype, feat->ld, feat->dim, qf, ld_q, targets, n_query, max_rows, counts, buf0, ld0};
    hipLaunchKernelGGL(k_init_buffer, dim3((unsigned)grid), dim3(128), 0, s, a);
    OMG_HIP(hipGetLastError());
    return OMG_OK;
}
