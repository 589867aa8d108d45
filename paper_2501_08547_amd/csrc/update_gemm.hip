// Dense update of one layer (Eq. 1, the update function U): out = act(scale * sum_s A_s W_s + bias)
// on the matrix cores, fp32 in and out (v_mfma_f32_32x32x2_f32).
//
// The product is a sum over "segments": SAGE has two (own embedding x W_self, aggregated
// neighbours x W_nb), GCN one, the GAT output layer one per head (mean of heads); GAT hidden
// layers run one grid z-slice per head on that head's columns.
//
// Block = 4 wavefronts computing a 64 x 64 output tile as 2 x 2 sub-tiles of 32 x 32; K is
// walked in steps of KT through LDS.  A-tile rows are padded to an odd stride so that the 32
// lanes that fetch one K column hit 32 different banks.
#include "internal.h"

namespace {

constexpr int BM = 64, BN = 64, KT = 16;
constexpr int A_STRIDE = KT + 1;

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ inline float activate(float x, int act) {
    if (act == OMG_ACT_RELU) return x > 0.f ? x : 0.f;
    if (act == OMG_ACT_ELU) return x > 0.f ? x : expm1f(x);
    return x;
}

__global__ __launch_bounds__(256) void k_update(GemmArgs g) {
    __shared__ float As[BM * A_STRIDE];
    __shared__ float Bs[KT * BN];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;
    const int z = blockIdx.z;

    floatx16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;

    // loader coordinates: A tile 64 x 16 -> thread (row = tid / 4, 4 consecutive k); B tile 16 x 64 -> 4 rows per thread
    const int a_row = tid >> 2, a_k = (tid & 3) * 4;
    const int b_col = tid & 63, b_row = tid >> 6;

    for (int sgi = 0; sgi < g.n_seg; ++sgi) {
        const GemmSeg sg = g.seg[sgi];
        const float* A = sg.A + (int64_t)z * g.a_z_stride;
        const float* W = sg.W + (int64_t)z * g.w_z_stride;
        for (int k0 = 0; k0 < sg.k; k0 += KT) {
            {
                const int64_t r = m0 + a_row;
                float v[4] = {0.f, 0.f, 0.f, 0.f};
                if (r < g.m) {
                    const float* src = A + r * sg.lda + k0 + a_k;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (k0 + a_k + i < sg.k) v[i] = src[i];
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) As[a_row * A_STRIDE + a_k + i] = v[i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int kr = b_row + i * 4;
                float v = 0.f;
                if (k0 + kr < sg.k && n0 + b_col < g.n) v = W[(int64_t)(k0 + kr) * sg.ldw + n0 + b_col];
                Bs[kr * BN + b_col] = v;
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < KT; kk += 2) {
                const float a = As[(wm * 32 + (lane & 31)) * A_STRIDE + kk + (lane >> 5)];
                const float b = Bs[(kk + (lane >> 5)) * BN + wn * 32 + (lane & 31)];
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
            }
            __syncthreads();
        }
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
