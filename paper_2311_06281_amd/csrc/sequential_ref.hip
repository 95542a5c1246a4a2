// The sequential baseline of the paper's experiment (Sec. 4, Fig. 1: time to compute n elements one
// after the other, relative to the parallel computation, on the same GPU).  One lane walks the sequence
// x_t = a_t x_{t-1} + b_t in float32; the other 63 lanes only help to bring the inputs on chip and the
// results out in coalesced chunks, so the figure measures the dependent chain, not memory latency.
#include "../../include/heinsen.h"
#include <hip/hip_runtime.h>

namespace {

constexpr int kChunk = 64 * 16;

__global__ __launch_bounds__(64) void heinsen_sequential_kernel(const float *a, const float *b, const float *x0,
                                                                float *out, long long n)
{
    __shared__ float sa[kChunk], sb[kChunk], so[kChunk];
    const int lane = threadIdx.x;
    float x = x0[0];
    for (long long base = 0; base < n; base += kChunk) {
        const int m = (int)((n - base) < kChunk ? (n - base) : kChunk);
        for (int i = lane; i < m; i += 64) {
            sa[i] = a[base + i];
            sb[i] = b[base + i];
        }
        __syncthreads();
        if (lane == 0) {
            for (int i = 0; i < m; ++i) {
                x = sa[i] * x + sb[i]; // Sec. 3: x_t = a_t x_{t-1} + b_t
                so[i] = x;
            }
        }
        __syncthreads();
        for (int i = lane; i < m; i += 64) out[base + i] = so[i];
        __syncthreads();
    }
}

} // namespace

extern "C" int heinsen_sequential(const void *a, const void *b, const void *x0, void *out, int64_t n, void *stream)
{
    if (!a || !b || !x0 || !out || n < 1) return HEINSEN_ERR_INVALID_ARG;
    hipLaunchKernelGGL(heinsen_sequential_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream),
                       static_cast<const float *>(a), static_cast<const float *>(b), static_cast<const float *>(x0),
                       static_cast<float *>(out), (long long)n);
    return hipGetLastError() == hipSuccess ? HEINSEN_OK : HEINSEN_ERR_HIP;
}
