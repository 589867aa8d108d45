// Dense update of one layer (Eq. 1, the update function U): out = act(scale * sum_s A_s W_s + bias)
// on the matrix cores, fp32 in and out (v_mfma_f32_32x32x2_f32).
//
// The product is a sum over "segments": SAGE has two (own embedding x W_self, aggregated
// neighbours x W_nb), GCN one, the GAT output layer one per head (mean of heads); GAT hidden
// layers run one grid z-slice per head on that head's columns.
//
// Block = 4 wavefronts computing a 64 x 64 output tile as 2 x 2 sub-tiles of 32 x 32.  K is walked
// 32 at a time over all segments; the next K-tile is fetched from global memory into registers
// while the current one is multiplied out of LDS (two LDS buffers, one barrier per K-tile).
// A-tile rows are padded to an odd stride so that the 32 lanes that fetch one K column hit 32
// different banks.
#include "internal.h"

namespace {

constexpr int BM = 64, BN = 64, KT = 32;
constexpr int A_STRIDE = KT + 1;

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ inline float activate(float x, int act) {
    if (act == OMG_ACT_RELU) return x > 0.f ? x : 0.f;
    if (act == OMG_ACT_ELU) return x > 0.f ? x : expm1f(x);
    return x;
}

struct TileRegs {
    float a[2][4];      // two A rows x 4 consecutive k
    float b[8];         // eight W rows, one column
};

__global__ __launch_bounds__(256) void k_update(GemmArgs g) {
    __shared__ float As[2][BM * A_STRIDE];
    __shared__ float Bs[2][KT * BN];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;
    const int z = blockIdx.z;

    floatx16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;

    // loader coordinates: A tile 64 x 32 -> rows tid / 8 and tid / 8 + 32, 4 consecutive k each;
    // W tile 32 x 64 -> column tid % 64, rows tid / 64 + 4 i
    const int a_row = tid >> 3, a_k = (tid & 7) * 4;
    const int b_col = tid & 63, b_row = tid >> 6;
    const bool col_ok = n0 + b_col < g.n;

    auto fetch = [&](int sgi, int k0, TileRegs& r) {
        const GemmSeg sg = g.seg[sgi];
        const float* A = sg.A + (int64_t)z * g.a_z_stride;
        const float* W = sg.W + (int64_t)z * g.w_z_stride;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int64_t row = m0 + a_row + 32 * h;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            const int k = k0 + a_k;
            if (row < g.m && k < sg.k) v = *reinterpret_cast<const float4*>(A + row * sg.lda + k);
            r.a[h][0] = v.x;                              // k < sg.k holds here
            r.a[h][1] = k + 1 < sg.k ? v.y : 0.f;         // what lies beyond k is padding: never multiply it
            r.a[h][2] = k + 2 < sg.k ? v.z : 0.f;
            r.a[h][3] = k + 3 < sg.k ? v.w : 0.f;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int k = k0 + b_row + 4 * i;
            r.b[i] = (col_ok && k < sg.k) ? W[(int64_t)k * sg.ldw + n0 + b_col] : 0.f;
        }
    };
    auto stash = [&](int buf, const TileRegs& r) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < 4; ++i) As[buf][(a_row + 32 * h) * A_STRIDE + a_k + i] = r.a[h][i];
#pragma unroll
        for (int i = 0; i < 8; ++i) Bs[buf][(b_row + 4 * i) * BN + b_col] = r.b[i];
    };

    int sgi = 0, k0 = 0;                 // the tile being fetched next
    while (sgi < g.n_seg && g.seg[sgi].k <= 0) ++sgi;
    TileRegs regs;
    int cur = 0;
    if (sgi < g.n_seg) {
        fetch(sgi, k0, regs);
        stash(0, regs);
    }
    __syncthreads();
    while (sgi < g.n_seg) {
        // advance to the following tile and start fetching it
        int nsg = sgi, nk = k0 + KT;
        if (nk >= g.seg[nsg].k) {
            nk = 0;
            ++nsg;
            while (nsg < g.n_seg && g.seg[nsg].k <= 0) ++nsg;
        }
        const bool more = nsg < g.n_seg;
        if (more) fetch(nsg, nk, regs);
        const float* as = As[cur];
        const float* bs = Bs[cur];
#pragma unroll
        for (int kk = 0; kk < KT; kk += 2) {
            const float a = as[(wm * 32 + (lane & 31)) * A_STRIDE + kk + (lane >> 5)];
            const float b = bs[(kk + (lane >> 5)) * BN + wn * 32 + (lane & 31)];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
        }
        if (more) stash(cur ^ 1, regs);
        __syncthreads();
        cur ^= 1;
        sgi = nsg;
        k0 = nk;
    }

    // accumulator layout of the 32 x 32 tile: register r of lane l holds
    // row 8 * (r / 4) + 4 * (l / 32) + r % 4, column l % 32
    const int col = n0 + wn * 32 + (lane & 31);
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

}  // namespace

int omg_launch_update(const GemmArgs& a, hipStream_t s) {
    if (a.m <= 0 || a.n <= 0) return OMG_OK;
    dim3 grid((unsigned)((a.m + BM - 1) / BM), (unsigned)((a.n + BN - 1) / BN), (unsigned)(a.n_z > 0 ? a.n_z : 1));
    hipLaunchKernelGGL(k_update, grid, dim3(256), 0, s, a);
    OMG_HIP(hipGetLastError());
    return OMG_OK;
}
