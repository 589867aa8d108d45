// Dense update of one layer (Eq. 1, the update function U): out = act(scale * sum_s A_s W_s + bias)
// on the matrix cores, fp32 in and out (v_mfma_f32_32x32x2_f32).
//
// The product is a sum over "segments": SAGE has two (own embedding x W_self, aggregated
// neighbours x W_nb), GCN one, the GAT output layer one per head (mean of heads); GAT hidden
// layers run one grid z-slice per head on that head's columns.
//
// Block = 4 wavefronts computing a 64 x 64 output tile as 2 x 2 sub-tiles of 32 x 32.  K is walked
// 64 at a time over all segments.  A K-tile travels global memory -> registers -> LDS -> matrix
// cores; two register sets keep the loads of the next two K-tiles in flight while the current one
// is multiplied, because one dependent trip to memory (2-3 us) is far longer than the 0.85 us the
// 32 matrix instructions of a K-tile take.  Loads are unconditional (addresses clamped into the
// operand, values masked when they are written to LDS), so nothing between a load and its use
// forces a wait.  The loads of a later tile are issued between the matrix instructions of the tile
// being multiplied, not between the barriers, and the address of a W row is scalar arithmetic
// (the row is the same in every lane of a wavefront), so that the vector ALU work of a fetch no
// longer sits on the path between two barriers.  One LDS buffer so that several blocks fit a
// compute unit.
//
// LDS holds both operands K-contiguous: As[row][k], Bs[col][k], row stride 68 floats.  The matrix
// instruction takes, per lane, A[row = lane % 32][k'] and B[k'][col = lane % 32] with k' = lane / 32;
// which two k of the tile a step multiplies is free as long as both operands agree, so step j of a
// group of eight k uses k = 4 (lane / 32) + j and a lane reads its four steps with one 16-byte LDS
// read per operand.
#include "internal.h"

namespace {

constexpr int BM = 64, BN = 64, KT = 64;
constexpr int LS = KT + 4;          // LDS row stride in floats: 16-byte aligned, 8 rows cover all banks

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ inline float activate(float x, int act) {
    if (act == OMG_ACT_RELU) return x > 0.f ? x : 0.f;
    if (act == OMG_ACT_ELU) return x > 0.f ? x : expm1f(x);
    return x;
}

struct TileRegs {
    float4 a[4];        // four A rows x 4 consecutive k
    float4 b[4];        // one W column x 4 groups of 4 consecutive k
    int klim;           // number of valid k in this tile (may exceed KT)
};

// SPLIT: a launch of few blocks and many K-tiles (the last layer of every model has one row per query) leaves
// most compute units idle while each block walks its K-tiles.  g.k_split blocks then share an output tile:
// block j of them takes the K-tiles j, j + k_split, ... and stores its raw sums to g.split_buf;
// k_update_finish adds them in block order (fixed order: reruns are bit-identical) and applies the epilogue.
template <bool SPLIT>
__global__ __launch_bounds__(256) void k_update(GemmArgs g) {
    __shared__ __attribute__((aligned(16))) float As[BM * LS];
    __shared__ __attribute__((aligned(16))) float Bs[BN * LS];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int ks = SPLIT ? g.k_split : 1;
    const int kg = SPLIT ? (int)(blockIdx.x % (unsigned)ks) : 0;
    const int64_t m0 = (int64_t)(SPLIT ? blockIdx.x / (unsigned)ks : blockIdx.x) * BM;
    const int n0 = blockIdx.y * BN;
    const int z = blockIdx.z;

    floatx16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;

    // loader coordinates: A tile 64 x 64 -> rows tid / 16 + 16 h, k = 4 (tid % 16) .. + 3;
    // W tile 64 x 64 -> column tid % 64, k = 4 (tid / 64 + 4 i) .. + 3
    const int a_row = tid >> 4, a_k = (tid & 15) * 4;
    const int b_col = tid & 63, b_q = __builtin_amdgcn_readfirstlane(tid >> 6);
    // columns beyond n are computed from a real column and never stored
    const uint32_t w_byte = (uint32_t)min(n0 + b_col, g.n - 1) * 4u;
    int64_t a_off[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) a_off[h] = min(m0 + a_row + 16 * h, g.m - 1);   // same for rows beyond m

    int n_tiles = 0;
    for (int i = 0; i < g.n_seg; ++i)
        if (g.seg[i].k > 0) n_tiles += (g.seg[i].k + KT - 1) / KT;
    int f_sg = 0, f_k0 = 0;              // the K-tile the next fetch reads
    while (f_sg < g.n_seg && g.seg[f_sg].k <= 0) ++f_sg;
    const int first_sg = f_sg;

    // State of the fetch, the same in every lane of a wavefront except the row pointers.  Past the last
    // K-tile a fetch reads the first tile again and marks it empty: every fetch issues the same loads, so
    // the number of loads in flight is the same on every path, which lets the wait before a tile's use
    // leave the younger tile's loads outstanding.
    const float* f_W = nullptr;
    int64_t f_ldw = 0;
    int f_k = 1;
    bool f_live = false;
    const float* a_ptr[4] = {nullptr, nullptr, nullptr, nullptr};
    auto open_segment = [&]() {
        f_live = f_sg < g.n_seg;
        const GemmSeg sg = g.seg[f_live ? f_sg : first_sg];
        f_W = sg.W + (int64_t)z * g.w_z_stride;
        f_ldw = sg.ldw;
        f_k = sg.k;
        const float* A = sg.A + (int64_t)z * g.a_z_stride;
#pragma unroll
        for (int h = 0; h < 4; ++h) a_ptr[h] = A + a_off[h] * sg.lda;
    };
    auto advance_one = [&]() {
        if (!f_live) return;
        f_k0 += KT;
        if (f_k0 >= f_k) {
            f_k0 = 0;
            ++f_sg;
            while (f_sg < g.n_seg && g.seg[f_sg].k <= 0) ++f_sg;
            open_segment();
        }
    };
    auto advance = [&]() {                               // to this block's next K-tile
        if (SPLIT) {
            for (int j = 0; j < ks; ++j) advance_one();
        } else {
            advance_one();
        }
    };
    // The loads of a K-tile in five groups (the A rows, then four groups of W rows), so that they can be
    // issued between the matrix instructions of the tile being multiplied.  A W row's address is the same
    // in every lane up to the column: scalar arithmetic plus one 32-bit lane offset.
    auto load_a = [&](TileRegs& r) {
        const int ka = f_k0 + a_k < f_k ? f_k0 + a_k : 0;           // out-of-range pieces read a valid place, masked later
#pragma unroll
        for (int h = 0; h < 4; ++h) r.a[h] = *reinterpret_cast<const float4*>(a_ptr[h] + ka);
        r.klim = f_live ? f_k - f_k0 : 0;
    };
    auto load_w = [&](TileRegs& r, int i) {
        const int kb = f_k0 + 4 * (b_q + 4 * i);
        float w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float* wrow = f_W + (int64_t)min(kb + j, f_k - 1) * f_ldw;       // finite; meets zeros of A
            w[j] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(wrow) + w_byte);
        }
        r.b[i] = make_float4(w[0], w[1], w[2], w[3]);
    };
    auto stash = [&](const TileRegs& r) {
        const int lim = r.klim - a_k;                     // what lies beyond k is padding: never multiply it
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            float4 v = r.a[h];
            v.x = lim > 0 ? v.x : 0.f;
            v.y = lim > 1 ? v.y : 0.f;
            v.z = lim > 2 ? v.z : 0.f;
            v.w = lim > 3 ? v.w : 0.f;
            *reinterpret_cast<float4*>(&As[(a_row + 16 * h) * LS + a_k]) = v;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<float4*>(&Bs[b_col * LS + 4 * (b_q + 4 * i)]) = r.b[i];
    };
    const float* ap = As + (wm * 32 + (lane & 31)) * LS + 4 * (lane >> 5);
    const float* bp = Bs + (wn * 32 + (lane & 31)) * LS + 4 * (lane >> 5);
    // Multiplies the K-tile in LDS and, between its matrix instructions, issues the loads of a later tile
    // into `rf` (whose previous content went to LDS before the barrier).
    auto multiply = [&](TileRegs& rf) {
        float4 a[2], b[2], an[2], bn[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            a[q] = *reinterpret_cast<const float4*>(ap + 8 * q);
            b[q] = *reinterpret_cast<const float4*>(bp + 8 * q);
        }
#pragma unroll
        for (int c = 0; c < KT / 16; ++c) {               // 16 k per round: read the next round, multiply this one
            if (c + 1 < KT / 16) {
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    an[q] = *reinterpret_cast<const float4*>(ap + 16 * (c + 1) + 8 * q);
                    bn[q] = *reinterpret_cast<const float4*>(bp + 16 * (c + 1) + 8 * q);
                }
            }
            if (c == 0) load_a(rf);
            load_w(rf, c);
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q].x, b[q].x, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q].y, b[q].y, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q].z, b[q].z, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q].w, b[q].w, acc, 0, 0, 0);
            }
#pragma unroll
            for (int q = 0; q < 2; ++q) { a[q] = an[q]; b[q] = bn[q]; }
        }
    };
    static_assert(KT / 16 == 4, "one group of W loads per round of the multiply");

    if (n_tiles > 0) {
        TileRegs r0, r1;
        open_segment();
        for (int j = 0; j < kg; ++j) advance_one();
        load_a(r0);
#pragma unroll
        for (int i = 0; i < 4; ++i) load_w(r0, i);
        advance();
        load_a(r1);
#pragma unroll
        for (int i = 0; i < 4; ++i) load_w(r1, i);
        advance();
        const int n_iter = (n_tiles + ks - 1) / ks;
        for (int t = 0; t < n_iter; t += 2) {
            stash(r0);                              // K-tile t; the loads into r1 stay in flight
            __syncthreads();
            multiply(r0);                           // and fetch K-tile t + 2
            advance();
            __syncthreads();
            stash(r1);                              // K-tile t + 1 (empty past the end: adds zeros)
            __syncthreads();
            multiply(r1);                           // and fetch K-tile t + 3
            advance();
            __syncthreads();
        }
    }

    // accumulator layout of the 32 x 32 tile: register r of lane l holds
    // row 8 * (r / 4) + 4 * (l / 32) + r % 4, column l % 32
    const int col = n0 + wn * 32 + (lane & 31);
    if (SPLIT) {
        // raw sums: [k_split][m][gridDim.y * BN], columns beyond n included (they are never read)
        const int64_t pw = (int64_t)gridDim.y * BN;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = m0 + wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (row < g.m) g.split_buf[((int64_t)kg * g.m + row) * pw + col] = acc[r];
        }
        return;
    }
    if (col >= g.n) return;
    const int ocol = z * g.out_z_stride + col;
    float bias = 0.f;
    if (g.bias != nullptr) {
        if (g.bias_sum > 1) {
            for (int j = 0; j < g.bias_sum; ++j) bias += g.bias[col + j * g.n];
            bias /= (float)g.bias_sum;
        } else {
            bias = g.bias[ocol];
        }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int64_t row = m0 + wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < g.m) g.out[row * g.ldo + ocol] = activate(acc[r] * g.scale + bias, g.act);
    }
}

// Second step of a split launch: out = act(scale * (sum of the k_split raw sums, in block order) + bias).
__global__ __launch_bounds__(256) void k_update_finish(GemmArgs g, int64_t pw) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= g.m * g.n) return;
    const int64_t row = i / g.n;
    const int col = (int)(i - row * g.n);
    float sum = 0.f;
    for (int j = 0; j < g.k_split; ++j) sum += g.split_buf[((int64_t)j * g.m + row) * pw + col];
    float bias = 0.f;
    if (g.bias != nullptr) {
        if (g.bias_sum > 1) {
            for (int j = 0; j < g.bias_sum; ++j) bias += g.bias[col + j * g.n];
            bias /= (float)g.bias_sum;
        } else {
            bias = g.bias[col];
        }
    }
    g.out[row * g.ldo + col] = activate(sum * g.scale + bias, g.act);
}

// A few rows (a batch of one to a few dozen queries): the matrix-core tiles above would multiply 64 rows of
// padding and walk K in dependent steps, each a trip to memory.  Here a block takes RM rows x 8 columns; its 256
// threads are 32 slices of K x 8 columns, and a thread issues all the loads of eight of its k at once (for K up to
// 256 that is every load of the kernel in one round trip).  The 32 partial sums are added in a fixed tree (lanes,
// then wavefronts in order): reruns are bit-identical.
// Up to 256 rows by measurement: 157 rows x 256 x 128 per layer 13.2 -> 10.1 us (the matrix-core route shares its
// few tiles among blocks and needs a second launch to add them up), 220 rows x 512 x 256 equal, 800 rows and more
// twice as slow (every block of 8 rows streams the whole of W).
constexpr int ROWS_MAX = 256;

template <int RM>
__global__ __launch_bounds__(256) void k_update_rows(GemmArgs g) {
    __shared__ float red[4][RM][8];
    const int c = threadIdx.x & 7, ks = threadIdx.x >> 3;
    const int z = blockIdx.z;
    const int col = blockIdx.y * 8 + c;
    const int wcol = min(col, g.n - 1);
    const int64_t r0 = (int64_t)blockIdx.x * RM;
    int k_total = 0;
    for (int i = 0; i < g.n_seg; ++i) k_total += g.seg[i].k > 0 ? g.seg[i].k : 0;
    int64_t row[RM];
#pragma unroll
    for (int r = 0; r < RM; ++r) row[r] = min(r0 + r, g.m - 1);
    float acc[RM];
#pragma unroll
    for (int r = 0; r < RM; ++r) acc[r] = 0.f;
    for (int base = 0; base < k_total; base += 32 * 8) {
        float w[8], a[8][RM];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            int kk = base + ks + 32 * u;
            const bool valid = kk < k_total;
            kk = valid ? kk : 0;
            int sg = 0;                                   // the segment kk falls into
            while (sg + 1 < g.n_seg && kk >= (g.seg[sg].k > 0 ? g.seg[sg].k : 0)) {
                kk -= g.seg[sg].k > 0 ? g.seg[sg].k : 0;
                ++sg;
            }
            const float* A = g.seg[sg].A + (int64_t)z * g.a_z_stride + kk;
            const float wv = g.seg[sg].W[(int64_t)z * g.w_z_stride + (int64_t)kk * g.seg[sg].ldw + wcol];
            w[u] = valid ? wv : 0.f;
#pragma unroll
            for (int r = 0; r < RM; ++r) a[u][r] = A[row[r] * g.seg[sg].lda];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int r = 0; r < RM; ++r) acc[r] = fmaf(a[u][r], w[u], acc[r]);
    }
    // lanes of a wavefront: 8 slices x 8 columns
#pragma unroll
    for (int off = 8; off < 64; off <<= 1)
#pragma unroll
        for (int r = 0; r < RM; ++r) acc[r] += __shfl_xor(acc[r], off);
    if ((threadIdx.x & 63) < 8) {
#pragma unroll
        for (int r = 0; r < RM; ++r) red[threadIdx.x >> 6][r][c] = acc[r];
    }
    __syncthreads();
    if (threadIdx.x >= 8 || col >= g.n) return;
    const int ocol = z * g.out_z_stride + col;
    float bias = 0.f;
    if (g.bias != nullptr) {
        if (g.bias_sum > 1) {
            for (int j = 0; j < g.bias_sum; ++j) bias += g.bias[col + j * g.n];
            bias /= (float)g.bias_sum;
        } else {
            bias = g.bias[ocol];
        }
    }
#pragma unroll
    for (int r = 0; r < RM; ++r) {
        if (r0 + r >= g.m) break;
        const float sum = ((red[0][r][c] + red[1][r][c]) + red[2][r][c]) + red[3][r][c];
        g.out[(r0 + r) * g.ldo + ocol] = activate(sum * g.scale + bias, g.act);
    }
}

}  // namespace

int omg_launch_update(const GemmArgs& a_in, hipStream_t s) {
    if (a_in.m <= 0 || a_in.n <= 0) return OMG_OK;
    GemmArgs a = a_in;
    if (a.m <= ROWS_MAX) {
        const int rm = a.m <= 2 ? 2 : 8;
        const dim3 grid((unsigned)((a.m + rm - 1) / rm), (unsigned)((a.n + 7) / 8), (unsigned)(a.n_z > 0 ? a.n_z : 1));
        if (rm == 2) hipLaunchKernelGGL(k_update_rows<2>, grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL(k_update_rows<8>, grid, dim3(256), 0, s, a);
        OMG_HIP(hipGetLastError());
        return OMG_OK;
    }
    dim3 grid((unsigned)((a.m + BM - 1) / BM), (unsigned)((a.n + BN - 1) / BN), (unsigned)(a.n_z > 0 ? a.n_z : 1));
    int n_tiles = 0;
    for (int i = 0; i < a.n_seg; ++i)
        if (a.seg[i].k > 0) n_tiles += (a.seg[i].k + KT - 1) / KT;
    // Fewer blocks than half the compute units and several K-tiles each: share the K-tiles of an output tile
    // among two or four blocks, if the caller lent memory for their raw sums.
    const int64_t blocks = (int64_t)grid.x * grid.y;
    int ks = 1;
    if (grid.z == 1 && blocks <= 128 && a.split_buf != nullptr) ks = n_tiles >= 8 ? 4 : n_tiles >= 4 ? 2 : 1;
    const int64_t pw = (int64_t)grid.y * BN;
    if (ks > 1 && (int64_t)ks * a.m * pw > a.split_floats) ks = 1;
    a.k_split = ks;
    if (ks > 1) {
        grid.x *= (unsigned)ks;
        hipLaunchKernelGGL(k_update<true>, grid, dim3(256), 0, s, a);
        const int64_t n_out = a.m * a.n;
        hipLaunchKernelGGL(k_update_finish, dim3((unsigned)((n_out + 255) / 256)), dim3(256), 0, s, a, pw);
    } else {
        hipLaunchKernelGGL(k_update<false>, grid, dim3(256), 0, s, a);
    }
    OMG_HIP(hipGetLastError());
    return OMG_OK;
}
