// Streaming yardsticks: out = a + b over a [B, n, D] float32 array with the memory access patterns of the
// scan kernels and nothing else -- no dependences between tiles, no arithmetic to speak of.  What these
// reach is the ceiling of an access pattern on this machine; the scan kernels are measured against it.
// All accesses are non-temporal (every byte is used once).
#include "../../include/heinsen.h"
#include <hip/hip_runtime.h>

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

// pattern 0: the array as one long vector, 16 bytes per lane, consecutive lanes consecutive vectors
__global__ __launch_bounds__(256) void heinsen_probe_linear(const f4 *a, const f4 *b, f4 *o, size_t n4)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) __builtin_nontemporal_store(__builtin_nontemporal_load(a + i) + __builtin_nontemporal_load(b + i), o + i);
}

// pattern 7: bf16 inputs widened to a float32 output (4 bytes read, 4 written per element: the mix of
// traffic of a scan with bf16 storage), one long vector; a lane takes 4 elements at a time (8 bytes from
// each input, 16 bytes out, so that every access of a wave is one contiguous piece), two such per lane
typedef unsigned int u2 __attribute__((ext_vector_type(2)));
__global__ __launch_bounds__(256) void heinsen_probe_linear_bf16(const u2 *a, const u2 *b, f4 *o, size_t n4)
{
    const size_t i0 = (size_t)blockIdx.x * 512 + threadIdx.x;
    u2 x[2], y[2];
#pragma unroll
    for (int k = 0; k < 2; ++k)
        if (i0 + k * 256 < n4) {
            x[k] = __builtin_nontemporal_load(a + i0 + k * 256);
            y[k] = __builtin_nontemporal_load(b + i0 + k * 256);
        }
#pragma unroll
    for (int k = 0; k < 2; ++k)
        if (i0 + k * 256 < n4) {
            f4 r;
            r[0] = __uint_as_float(x[k][0] << 16) + __uint_as_float(y[k][0] << 16);
            r[1] = __uint_as_float(x[k][0] & 0xffff0000u) + __uint_as_float(y[k][0] & 0xffff0000u);
            r[2] = __uint_as_float(x[k][1] << 16) + __uint_as_float(y[k][1] << 16);
            r[3] = __uint_as_float(x[k][1] & 0xffff0000u) + __uint_as_float(y[k][1] & 0xffff0000u);
            __builtin_nontemporal_store(r, o + i0 + k * 256);
        }
}

// patterns 1..3: a workgroup of CG x TS waves takes 64*CG adjacent channels for TS*32 steps; a lane owns one
// channel for 32 steps (the tiles of the [B, n, D] scan kernel: CG = 1 and CG = 2; CG = 4 for comparison).
// SEP: no output is stored before all of the lane's inputs have arrived, as in a scan.
template <int CG, int TS, bool SEP>
__global__ __launch_bounds__(CG * TS * 64) void heinsen_probe_tiles(const float *a, const float *b, float *o, int D, int ncols, int n)
{
    constexpr int T = 32;
    const unsigned tile = blockIdx.x;
    const int chunk = tile / ncols, col = tile % ncols;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int wc = w % CG, ts = w / CG;
    const size_t cols_per_b = D / (64 * CG);
    const size_t bidx = col / cols_per_b, cg = col % cols_per_b;
    const size_t t0 = (size_t)chunk * TS * T + (size_t)ts * T;
    const size_t base = (bidx * n + t0) * D + cg * 64 * CG + wc * 64 + lane;
    float x[T], y[T];
#pragma unroll
    for (int k = 0; k < T; ++k) {
        x[k] = __builtin_nontemporal_load(a + base + (size_t)k * D);
        y[k] = __builtin_nontemporal_load(b + base + (size_t)k * D);
    }
    float acc = 0.0f;
    if (SEP) {
#pragma unroll
        for (int k = 0; k < T; ++k) acc += x[k] * y[k];
        acc = acc == 12345.678f ? 1.0f : 0.0f;
    }
#pragma unroll
    for (int k = 0; k < T; ++k) __builtin_nontemporal_store(x[k] + y[k] + acc, o + base + (size_t)k * D);
}

} // namespace

extern "C" int heinsen_stream_probe(const void *a, const void *b, void *out, int64_t B, int64_t n, int64_t D, int pattern,
                                    void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (!a || !b || !out || B < 1 || n < 1 || D < 1 || B * n * D >= ((int64_t)1 << 40)) return HEINSEN_ERR_INVALID_ARG;
    const float *pa = static_cast<const float *>(a), *pb = static_cast<const float *>(b);
    float *po = static_cast<float *>(out);
    if (pattern == 0) {
        if ((B * n * D) % 4 != 0) return HEINSEN_ERR_UNSUPPORTED;
        const size_t n4 = (size_t)(B * n * D) / 4;
        hipLaunchKernelGGL(heinsen_probe_linear, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, stream,
                           reinterpret_cast<const f4 *>(pa), reinterpret_cast<const f4 *>(pb), reinterpret_cast<f4 *>(po), n4);
        return hipGetLastError() == hipSuccess ? HEINSEN_OK : HEINSEN_ERR_HIP;
    }
    if (pattern == 7) {
        if ((B * n * D) % 4 != 0) return HEINSEN_ERR_UNSUPPORTED;
        const size_t n4 = (size_t)(B * n * D) / 4;
        hipLaunchKernelGGL(heinsen_probe_linear_bf16, dim3((unsigned)((n4 + 511) / 512)), dim3(256), 0, stream,
                           static_cast<const u2 *>(a), static_cast<const u2 *>(b), reinterpret_cast<f4 *>(po), n4);
        return hipGetLastError() == hipSuccess ? HEINSEN_OK : HEINSEN_ERR_HIP;
    }
    const int cg = pattern == 1 || pattern == 4 ? 1 : (pattern == 2 || pattern == 5 ? 2 : 4);
    const int ts = 8 / cg;
    if (pattern < 0 || pattern > 6 || D % (64 * cg) != 0 || n % (ts * 32) != 0) return HEINSEN_ERR_UNSUPPORTED;
    const int ncols = (int)(B * D / (64 * cg));
    const dim3 grid((unsigned)((int64_t)ncols * (n / (ts * 32)))), block(512);
    switch (pattern) {
    case 1: hipLaunchKernelGGL((heinsen_probe_tiles<1, 8, false>), grid, block, 0, stream, pa, pb, po, (int)D, ncols, (int)n); break;
    case 2: hipLaunchKernelGGL((heinsen_probe_tiles<2, 4, false>), grid, block, 0, stream, pa, pb, po, (int)D, ncols, (int)n); break;
    case 3: hipLaunchKernelGGL((heinsen_probe_tiles<4, 2, false>), grid, block, 0, stream, pa, pb, po, (int)D, ncols, (int)n); break;
    case 4: hipLaunchKernelGGL((heinsen_probe_tiles<1, 8, true>), grid, block, 0, stream, pa, pb, po, (int)D, ncols, (int)n); break;
    case 5: hipLaunchKernelGGL((heinsen_probe_tiles<2, 4, true>), grid, block, 0, stream, pa, pb, po, (int)D, ncols, (int)n); break;
    default: hipLaunchKernelGGL((heinsen_probe_tiles<4, 2, true>), grid, block, 0, stream, pa, pb, po, (int)D, ncols, (int)n); break;
    }
    return hipGetLastError() == hipSuccess ? HEINSEN_OK : HEINSEN_ERR_HIP;
}
