// Measurement aid: the rate at which this GPU's compute units can be fed with plain reads.  The gather's
// achieved rate is set against this figure as well as against the published HBM peak, because a buffer
// that fits the memory-side cache is not delivered any faster than one that streams from HBM.
#include "internal.h"

namespace {

// Grid-stride read of n16 16-byte pieces, four loads in flight per lane, `reps` times over.  Every
// repetition shifts the piece -> lane mapping, so that no block meets in its own caches what it read
// in an earlier repetition; the sum keeps the loads alive and is stored only for a value no input
// produces.
__global__ __launch_bounds__(256) void k_read_sweep(const float4* __restrict__ p, size_t n16, int reps,
                                                    float* __restrict__ sink) {
    float acc = 0.f;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int r = 0; r < reps; ++r) {
        const size_t shift = ((size_t)r * (n16 / 16 + 64 * 37)) % n16;
        for (size_t i = tid; i + 3 * stride < n16; i += 4 * stride) {
            size_t j0 = i + shift, j1 = j0 + stride, j2 = j1 + stride, j3 = j2 + stride;
            j0 -= j0 >= n16 ? n16 : 0; j1 -= j1 >= n16 ? n16 : 0;
            j2 -= j2 >= n16 ? n16 : 0; j3 -= j3 >= n16 ? n16 : 0;
            const float4 a = p[j0], b = p[j1], c = p[j2], d = p[j3];
            acc += a.x + b.y + c.z + d.w;
        }
    }
    if (acc == -123.4567f) sink[0] = acc;
}

}  // namespace

extern "C" int omg_measure_read_rate(omg_ctx* ctx, const void* buffer, int64_t bytes, int32_t reps, int32_t blocks,
                                     double* bytes_read, float* ms) {
    if (ctx == nullptr || buffer == nullptr || bytes_read == nullptr || ms == nullptr) return OMG_EINVAL;
    if (bytes < (int64_t)1 << 20 || reps < 1 || reps > 1024 || blocks < 1 || blocks > 65536) return OMG_EINVAL;
    if (reinterpret_cast<uintptr_t>(buffer) % 16 != 0) return OMG_EINVAL;
    // the sweep trusts `buffer` and `bytes`: refuse what the runtime does not know as device memory of that size
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, buffer) != hipSuccess) { (void)hipGetLastError(); return OMG_EINVAL; }
    if (attr.type != hipMemoryTypeDevice) return OMG_EINVAL;
    {
        void* range_base = nullptr;
        size_t range_size = 0;
        if (hipMemGetAddressRange(reinterpret_cast<hipDeviceptr_t*>(&range_base), &range_size,
                                  const_cast<void*>(buffer)) != hipSuccess) { (void)hipGetLastError(); return OMG_EINVAL; }
        const size_t off = reinterpret_cast<uintptr_t>(buffer) - reinterpret_cast<uintptr_t>(range_base);
        if (off + (size_t)bytes > range_size) return OMG_EINVAL;
    }
    const size_t n16 = (size_t)bytes / 16, stride = (size_t)blocks * 256;
    if (4 * stride > n16) return OMG_EINVAL;            // every lane must take at least one turn
    const size_t turns = (n16 - 3 * stride + 4 * stride - 1) / (4 * stride);   // per lane 0; others may take one fewer
    // pieces read in one repetition: lanes with index < n16 - 3 stride - (t - 1) 4 stride take turn t
    size_t pieces = 0;
    for (size_t t = 0; t < turns; ++t) {
        const size_t lim = n16 - 3 * stride - t * 4 * stride;
        pieces += 4 * (lim < stride ? lim : stride);
    }
    float* sink = nullptr;
    OMG_HIP(hipMalloc(&sink, 64));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = OMG_OK;
    do {
        if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) { rc = OMG_EHIP; break; }
        hipLaunchKernelGGL(k_read_sweep, dim3((unsigned)blocks), dim3(256), 0, ctx->stream,
                           static_cast<const float4*>(buffer), n16, 1, sink);          // warm-up, also fills the cache
        if (hipEventRecord(e0, ctx->stream) != hipSuccess) { rc = OMG_EHIP; break; }
        hipLaunchKernelGGL(k_read_sweep, dim3((unsigned)blocks), dim3(256), 0, ctx->stream,
                           static_cast<const float4*>(buffer), n16, reps, sink);
        if (hipEventRecord(e1, ctx->stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(ms, e0, e1) != hipSuccess || hipGetLastError() != hipSuccess) { rc = OMG_EHIP; break; }
        *bytes_read = (double)pieces * 16.0 * reps;
    } while (false);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(sink);
    return rc;
}
