// C ABI of libheinsen: argument validation, scratch cache, dispatch to the two layout paths.
#include "../../include/heinsen.h"
#include "heinsen_internal.hpp"

#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <utility>

namespace {

constexpr uint32_t kAllFlags =
    HEINSEN_LOG_INPUTS | HEINSEN_LOG_OUTPUT | HEINSEN_IN_BF16 | HEINSEN_POSITIVE | HEINSEN_X0_SCALAR;

thread_local int t_last_hip_error = 0;

struct Scratch {
    void *flags = nullptr;
    size_t flag_cap = 0;
    void *data = nullptr;
    size_t data_cap = 0;
};

std::mutex g_mutex;
std::map<std::pair<int, hipStream_t>, Scratch> g_scratch;

bool hip_ok(hipError_t e)
{
    if (e != hipSuccess) {
        t_last_hip_error = (int)e;
        return false;
    }
    return true;
}

// Validates sizes / layout / flags and fills the parts of ScanCall that do not depend on pointers.
int describe(int64_t B, int64_t D, int64_t n, int layout, uint32_t flags, hs::ScanCall &c, bool &bnd)
{
    if (B < 1 || D < 1 || n < 1) return HEINSEN_ERR_INVALID_ARG;
    if (layout != HEINSEN_LAYOUT_BND && layout != HEINSEN_LAYOUT_BDN) return HEINSEN_ERR_INVALID_ARG;
    if (flags & ~kAllFlags) return HEINSEN_ERR_INVALID_ARG;
    const int64_t lim = (int64_t)1 << 62;
    if (B > lim / D || B * D > lim / n || B * D * n >= lim) return HEINSEN_ERR_INVALID_ARG;
    const bool log_in = flags & HEINSEN_LOG_INPUTS;
    const bool positive = (flags & HEINSEN_POSITIVE) || log_in;
    if ((flags & HEINSEN_LOG_OUTPUT) && !positive) return HEINSEN_ERR_UNSUPPORTED;
    // tile counters are 32-bit: far beyond any array that fits the device, but checked all the same
    if (B * D * n >= ((int64_t)1 << 42)) return HEINSEN_ERR_UNSUPPORTED;
    c.B = B;
    c.D = D;
    c.n = n;
    c.is_signed = !positive;
    c.log_in = log_in;
    c.log_out = flags & HEINSEN_LOG_OUTPUT;
    c.bf16 = flags & HEINSEN_IN_BF16;
    c.x0_scalar = flags & HEINSEN_X0_SCALAR;
    c.vec_ok = false;
    // [B, n, 1] is the same memory as [B, 1, n]: a single channel per batch item is a plain row
    bnd = (layout == HEINSEN_LAYOUT_BND) && D > 1;
    return HEINSEN_OK;
}

int get_scratch(hipStream_t stream, const hs::ScratchNeed &need, Scratch &out)
{
    out = Scratch();
    if (need.flag_bytes == 0 && need.data_bytes == 0) return HEINSEN_OK;
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev))) return HEINSEN_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_mutex);
    Scratch &s = g_scratch[std::make_pair(dev, stream)];
    if (s.flag_cap < need.flag_bytes) {
        // work queued on the old buffer must drain before it is replaced
        if (s.flags) {
            if (!hip_ok(hipStreamSynchronize(stream))) return HEINSEN_ERR_HIP;
            (void)hipFree(s.flags);
            s.flags = nullptr;
            s.flag_cap = 0;
        }
        size_t cap = hs::align_up(need.flag_bytes + need.flag_bytes / 2, 4096);
        void *ptr = nullptr;
        if (!hip_ok(hipMalloc(&ptr, cap))) return HEINSEN_ERR_ALLOC;
        if (!hip_ok(hipMemset(ptr, 0, cap))) {
            (void)hipFree(ptr);
            return HEINSEN_ERR_HIP;
        }
        s.flags = ptr;
        s.flag_cap = cap;
    }
    if (s.data_cap < need.data_bytes) {
        if (s.data) {
            if (!hip_ok(hipStreamSynchronize(stream))) return HEINSEN_ERR_HIP;
            (void)hipFree(s.data);
            s.data = nullptr;
            s.data_cap = 0;
        }
        size_t cap = hs::align_up(need.data_bytes + need.data_bytes / 2, 4096);
        void *ptr = nullptr;
        if (!hip_ok(hipMalloc(&ptr, cap))) return HEINSEN_ERR_ALLOC;
        s.data = ptr;
        s.data_cap = cap;
    }
    out = s;
    return HEINSEN_OK;
}

} // namespace

extern "C" {

int heinsen_scan(const void *a, const void *b, const void *x0, void *out, int64_t B, int64_t D, int64_t n,
                 int layout, uint32_t flags, void *stream)
{
    if (!a || !b || !x0 || !out) return HEINSEN_ERR_INVALID_ARG;
    hs::ScanCall c = {};
    bool bnd = false;
    int st = describe(B, D, n, layout, flags, c, bnd);
    if (st != HEINSEN_OK) return st;
    const uintptr_t in_align = c.bf16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(a) % in_align || reinterpret_cast<uintptr_t>(b) % in_align ||
        reinterpret_cast<uintptr_t>(x0) % 4 || reinterpret_cast<uintptr_t>(out) % 4)
        return HEINSEN_ERR_INVALID_ARG;
    c.a = a;
    c.b = b;
    c.x0 = static_cast<const float *>(x0);
    c.out = static_cast<float *>(out);
    c.stream = static_cast<hipStream_t>(stream);

    const hs::ScratchNeed need = bnd ? hs::bnd_scratch(c) : hs::bdn_scratch(c);
    Scratch s;
    st = get_scratch(c.stream, need, s);
    if (st != HEINSEN_OK) return st;
    hipError_t e = bnd ? hs::bnd_launch(c, s.flags, s.data) : hs::bdn_launch(c, s.flags, s.data);
    if (!hip_ok(e)) return HEINSEN_ERR_HIP;
    return HEINSEN_OK;
}

const char *heinsen_status_string(int status)
{
    switch (status) {
    case HEINSEN_OK: return "ok";
    case HEINSEN_ERR_INVALID_ARG: return "invalid argument";
    case HEINSEN_ERR_UNSUPPORTED: return "unsupported combination of arguments";
    case HEINSEN_ERR_ALLOC: return "scratch allocation failed";
    case HEINSEN_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

int heinsen_last_hip_error(void) { return t_last_hip_error; }

int heinsen_version(void) { return 100; /* 0.1.0 */ }

int heinsen_release_scratch(void)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    int prev = 0;
    bool have_prev = hipGetDevice(&prev) == hipSuccess;
    int status = HEINSEN_OK;
    for (auto &kv : g_scratch) {
        if (hipSetDevice(kv.first.first) != hipSuccess) {
            status = HEINSEN_ERR_HIP;
            continue;
        }
        (void)hipDeviceSynchronize();
        if (kv.second.flags) (void)hipFree(kv.second.flags);
        if (kv.second.data) (void)hipFree(kv.second.data);
    }
    g_scratch.clear();
    if (have_prev) (void)hipSetDevice(prev);
    return status;
}

int heinsen_kernel_name(int64_t B, int64_t D, int64_t n, int layout, uint32_t flags, char *buf, int buflen)
{
    if (!buf || buflen < 1) return HEINSEN_ERR_INVALID_ARG;
    hs::ScanCall c = {};
    bool bnd = false;
    int st = describe(B, D, n, layout, flags, c, bnd);
    if (st != HEINSEN_OK) {
        buf[0] = '\0';
        return st;
    }
    const char *name = bnd ? hs::bnd_kernel_name(c) : hs::bdn_kernel_name(c);
    std::snprintf(buf, (size_t)buflen, "%s", name);
    return HEINSEN_OK;
}

} // extern "C"
