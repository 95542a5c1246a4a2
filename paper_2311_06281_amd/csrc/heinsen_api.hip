// C ABI of libheinsen: argument validation, scratch cache, dispatch to the two layout paths.
#include "../../include/heinsen.h"
#include "heinsen_internal.hpp"

#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <utility>
#include <vector>

namespace {

constexpr uint32_t kAllFlags =
    HEINSEN_LOG_INPUTS | HEINSEN_LOG_OUTPUT | HEINSEN_IN_BF16 | HEINSEN_POSITIVE | HEINSEN_X0_SCALAR |
    HEINSEN_OUT_COMPLEX | HEINSEN_LINEAR;

thread_local int t_last_hip_error = 0;

// One buffer of tagged 64-bit records per (device, stream); see heinsen_internal.hpp.  The host keeps no
// counters for it: tickets and the launch counter live in the buffer's header and are renewed by the
// kernels themselves.
struct Scratch {
    unsigned long long *records = nullptr;
    size_t capacity = 0;      // in 64-bit words, including the header
    bool in_graph = false;    // a captured launch holds this buffer's address: it is not freed on growth
    std::vector<unsigned long long *> retired; // such buffers, replaced by larger ones; freed on release
};

// Prepares a buffer for its first launch: all records cleared (no tag matches epoch 1), the ticket queues
// at {epoch 1 | ticket 0}, the size noted for the launch that has to clear the records again when the
// epochs come round.
__global__ void heinsen_scratch_init(unsigned long long *scratch, size_t capacity)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < capacity; i += stride) {
        unsigned long long v = 0ull;
        if (i < hs::kQueueStride * hs::kQueues && i % hs::kQueueStride == 0) v = 1ull << 32;
        if (i == hs::kHeaderCapacity) v = (unsigned long long)capacity;
        scratch[i] = v;
    }
}

// Testing aid: puts the launch counter of a buffer at `epoch` (1 .. 2^30 - 1), e.g. just before it comes round.
__global__ void heinsen_scratch_set_epoch(unsigned long long *scratch, uint32_t epoch)
{
    if (threadIdx.x < hs::kQueues) scratch[hs::kQueueStride * threadIdx.x] = (unsigned long long)epoch << 32;
}

std::mutex g_mutex;
std::map<std::pair<int, hipStream_t>, Scratch> g_scratch;

// Scratch of heinsen_scan_static: one fixed array per GPU, part of the loaded code, never allocated or
// freed.  In host code the array's name is not a device address; the address on each device is looked
// up once (hipGetSymbolAddress with that device current) and kept here.
constexpr size_t kStaticRecords = ((size_t)48 << 20) / sizeof(unsigned long long); // 48 MiB
static __device__ __align__(256) unsigned long long scratch[kStaticRecords];
constexpr int kMaxDevices = 64;
unsigned long long *g_static_scratch[kMaxDevices] = {};

// Settings of the carry waits and of the optional per-tile time stamps (process-wide, under g_mutex).
constexpr uint32_t kDefaultSpinLimit = 1u << 22; // polls of about a microsecond each: seconds
uint32_t g_spin_limit = kDefaultSpinLimit;
uint32_t g_drop_tile = 0xffffffffu;
unsigned long long *g_timeline = nullptr;
uint32_t g_timeline_tiles = 0;

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
    const bool linear = flags & HEINSEN_LINEAR;
    if (linear && (flags & (HEINSEN_LOG_INPUTS | HEINSEN_LOG_OUTPUT | HEINSEN_OUT_COMPLEX))) return HEINSEN_ERR_INVALID_ARG;
    const bool complex_out = flags & HEINSEN_OUT_COMPLEX;
    if (complex_out && !(flags & HEINSEN_LOG_OUTPUT)) return HEINSEN_ERR_INVALID_ARG;
    if (complex_out && log_in) return HEINSEN_ERR_UNSUPPORTED;
    // a complex output always tracks signs: a POSITIVE promise then changes nothing
    const bool positive = ((flags & HEINSEN_POSITIVE) && !complex_out) || log_in;
    if ((flags & HEINSEN_LOG_OUTPUT) && !positive && !complex_out) return HEINSEN_ERR_UNSUPPORTED;
    // tile counters are 32-bit: far beyond any array that fits the device, but checked all the same
    if (B * D * n >= ((int64_t)1 << 42)) return HEINSEN_ERR_UNSUPPORTED;
    c.B = B;
    c.D = D;
    c.n = n;
    c.is_signed = !positive && !linear;
    c.linear = linear;
    c.log_in = log_in;
    c.log_out = flags & HEINSEN_LOG_OUTPUT;
    c.bf16 = flags & HEINSEN_IN_BF16;
    c.x0_scalar = flags & HEINSEN_X0_SCALAR;
    // [B, n, 1] is the same memory as [B, 1, n]: a single channel per batch item is a plain row
    bnd = (layout == HEINSEN_LAYOUT_BND) && D > 1;
    return HEINSEN_OK;
}

// Makes sure the stream's buffer holds at least `want` words.  Called with g_mutex held; the caller keeps
// it until the kernel is enqueued.  While the stream is being captured nothing may be allocated: the call
// then needs the buffer an earlier ordinary call of at least this size has made.
int ensure_scratch(hipStream_t stream, size_t want, bool capturing, Scratch *&out)
{
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev))) return HEINSEN_ERR_HIP;
    if (capturing) {
        auto it = g_scratch.find(std::make_pair(dev, stream));
        if (it == g_scratch.end() || it->second.capacity < want) return HEINSEN_ERR_UNSUPPORTED;
        it->second.in_graph = true;
        out = &it->second;
        return HEINSEN_OK;
    }
    Scratch &s = g_scratch[std::make_pair(dev, stream)];
    if (s.capacity < want) {
        // work queued on the old buffer must drain before it is replaced
        if (s.records && !hip_ok(hipStreamSynchronize(stream))) return HEINSEN_ERR_HIP;
        if (s.records) {
            if (s.in_graph) s.retired.push_back(s.records); // a graph may still replay into it
            else (void)hipFree(s.records);
        }
        s.records = nullptr;
        s.capacity = 0;
        s.in_graph = false;
        const size_t cap = hs::align_up(want + want / 2, 512);
        void *ptr = nullptr;
        if (!hip_ok(hipMalloc(&ptr, cap * sizeof(unsigned long long)))) return HEINSEN_ERR_ALLOC;
        // cleared and armed on the call's own stream, ahead of the scan that is about to use it
        hipLaunchKernelGGL(heinsen_scratch_init, dim3(1024), dim3(256), 0, stream, static_cast<unsigned long long *>(ptr), cap);
        if (!hip_ok(hipGetLastError())) {
            (void)hipFree(ptr);
            return HEINSEN_ERR_HIP;
        }
        s.records = static_cast<unsigned long long *>(ptr);
        s.capacity = cap;
    }
    out = &s;
    return HEINSEN_OK;
}

// The fixed array of heinsen_scan_static on the current device (looked up and armed at the first call).
int static_scratch(hipStream_t stream, bool capturing, unsigned long long *&out)
{
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev))) return HEINSEN_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return HEINSEN_ERR_UNSUPPORTED;
    if (g_static_scratch[dev] == nullptr) {
        if (capturing) return HEINSEN_ERR_UNSUPPORTED; // the first call on a device has to be an ordinary one
        unsigned long long *ptr = nullptr;
        if (!hip_ok(hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch))) || ptr == nullptr)
            return HEINSEN_ERR_HIP;
        hipLaunchKernelGGL(heinsen_scratch_init, dim3(1024), dim3(256), 0, stream, ptr, kStaticRecords);
        if (!hip_ok(hipGetLastError())) return HEINSEN_ERR_HIP;
        // calls on other streams may follow: the array must be armed before any of them can run
        if (!hip_ok(hipStreamSynchronize(stream))) return HEINSEN_ERR_HIP;
        g_static_scratch[dev] = ptr;
    }
    out = g_static_scratch[dev];
    return HEINSEN_OK;
}

hs::LaunchCtx make_ctx(unsigned long long *records)
{
    return hs::LaunchCtx{records, g_spin_limit, g_drop_tile, g_timeline, g_timeline_tiles};
}

bool is_capturing(hipStream_t stream)
{
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    return stream != nullptr && hipStreamIsCapturing(stream, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone;
}

// Checks the arguments of a scan call and fills `c`; `bnd` tells which layout path serves it.
int make_call(const void *a, const void *b, const void *x0, void *out, int64_t B, int64_t D, int64_t n, int layout,
              uint32_t flags, void *stream, hs::ScanCall &c, bool &bnd)
{
    if (!a || !b || !x0 || !out) return HEINSEN_ERR_INVALID_ARG;
    int st = describe(B, D, n, layout, flags, c, bnd);
    if (st != HEINSEN_OK) return st;
    const uintptr_t in_align = c.bf16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(a) % in_align || reinterpret_cast<uintptr_t>(b) % in_align ||
        reinterpret_cast<uintptr_t>(x0) % 4 || reinterpret_cast<uintptr_t>(out) % ((flags & HEINSEN_OUT_COMPLEX) ? 8 : 4))
        return HEINSEN_ERR_INVALID_ARG;
    c.a = a;
    c.b = b;
    c.x0 = static_cast<const float *>(x0);
    c.out = static_cast<float *>(out);
    c.stream = static_cast<hipStream_t>(stream);
    return HEINSEN_OK;
}

} // namespace

extern "C" {

int heinsen_scan(const void *a, const void *b, const void *x0, void *out, int64_t B, int64_t D, int64_t n,
                 int layout, uint32_t flags, void *stream)
{
    hs::ScanCall c = {};
    bool bnd = false;
    int st = make_call(a, b, x0, out, B, D, n, layout, flags, stream, c, bnd);
    if (st != HEINSEN_OK) return st;

    const hs::ScratchNeed need = bnd ? hs::bnd_scratch(c) : hs::bdn_scratch(c);
    std::lock_guard<std::mutex> lock(g_mutex);
    unsigned long long *records = nullptr;
    if (need.records != 0) {
        // A call recorded into a HIP graph is replayed with the same arguments many times and may not
        // allocate: it uses the buffer the stream already has.  Nothing else is special about it -- the
        // kernels keep tickets and launch counter in the buffer themselves.
        Scratch *sc = nullptr;
        st = ensure_scratch(c.stream, hs::kRecordBase + need.records, is_capturing(c.stream), sc);
        if (st != HEINSEN_OK) return st;
        records = sc->records;
    }
    const hs::LaunchCtx ctx = make_ctx(records);
    const hipError_t e = bnd ? hs::bnd_launch(c, ctx) : hs::bdn_launch(c, ctx);
    return hip_ok(e) ? HEINSEN_OK : HEINSEN_ERR_HIP;
}

int heinsen_scan_static(const void *a, const void *b, const void *x0, void *out, int64_t B, int64_t D, int64_t n,
                        int layout, uint32_t flags, void *stream)
{
    hs::ScanCall c = {};
    bool bnd = false;
    int st = make_call(a, b, x0, out, B, D, n, layout, flags, stream, c, bnd);
    if (st != HEINSEN_OK) return st;
    c.scratch_budget = kStaticRecords; // the launchers choose tiles whose carries fit, if there are such
    const hs::ScratchNeed need = bnd ? hs::bnd_scratch(c) : hs::bdn_scratch(c);
    if (need.records != 0 && hs::kRecordBase + need.records > kStaticRecords) return HEINSEN_ERR_SCRATCH_LIMIT;
    std::lock_guard<std::mutex> lock(g_mutex);
    unsigned long long *records = nullptr;
    if (need.records != 0) {
        // The array keeps whatever the last call left in it.  Nothing has to be cleared: every launch finds
        // in the header a launch counter that no record in the array carries yet.
        st = static_scratch(c.stream, is_capturing(c.stream), records);
        if (st != HEINSEN_OK) return st;
    }
    const hs::LaunchCtx ctx = make_ctx(records);
    const hipError_t e = bnd ? hs::bnd_launch(c, ctx) : hs::bdn_launch(c, ctx);
    return hip_ok(e) ? HEINSEN_OK : HEINSEN_ERR_HIP;
}

int heinsen_check(void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    std::lock_guard<std::mutex> lock(g_mutex);
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev))) return HEINSEN_ERR_HIP;
    if (!hip_ok(hipStreamSynchronize(stream))) return HEINSEN_ERR_HIP;
    unsigned long long *bufs[2] = {nullptr, nullptr};
    size_t caps[2] = {0, 0};
    auto it = g_scratch.find(std::make_pair(dev, stream));
    if (it != g_scratch.end()) {
        bufs[0] = it->second.records;
        caps[0] = it->second.capacity;
    }
    if (dev >= 0 && dev < kMaxDevices) {
        bufs[1] = g_static_scratch[dev];
        caps[1] = kStaticRecords;
    }
    int status = HEINSEN_OK;
    for (int i = 0; i < 2; ++i) {
        if (bufs[i] == nullptr) continue;
        unsigned long long err = 0;
        if (!hip_ok(hipMemcpy(&err, bufs[i] + hs::kHeaderError, sizeof(err), hipMemcpyDeviceToHost))) return HEINSEN_ERR_HIP;
        if (err == 0) continue;
        status = HEINSEN_ERR_CARRY_LOST;
        // tickets and records may be in any state after two launches have shared the buffer: start it afresh
        hipLaunchKernelGGL(heinsen_scratch_init, dim3(1024), dim3(256), 0, stream, bufs[i], caps[i]);
        if (!hip_ok(hipGetLastError()) || !hip_ok(hipStreamSynchronize(stream))) return HEINSEN_ERR_HIP;
    }
    return status;
}

int heinsen_set_timeline(void *stamps, uint64_t tiles)
{
    if ((stamps == nullptr) != (tiles == 0) || tiles > 0xffffffffull || reinterpret_cast<uintptr_t>(stamps) % 8)
        return HEINSEN_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_mutex);
    g_timeline = static_cast<unsigned long long *>(stamps);
    g_timeline_tiles = (uint32_t)tiles;
    return HEINSEN_OK;
}

int heinsen_test_carry(uint32_t spin_limit, uint32_t drop_tile, uint32_t epoch, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (epoch > hs::kLastEpoch) return HEINSEN_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_mutex);
    g_spin_limit = spin_limit == 0 ? kDefaultSpinLimit : spin_limit;
    g_drop_tile = drop_tile;
    if (epoch != 0) {
        int dev = 0;
        if (!hip_ok(hipGetDevice(&dev))) return HEINSEN_ERR_HIP;
        auto it = g_scratch.find(std::make_pair(dev, stream));
        if (it != g_scratch.end() && it->second.records != nullptr)
            hipLaunchKernelGGL(heinsen_scratch_set_epoch, dim3(1), dim3(64), 0, stream, it->second.records, epoch);
        if (dev >= 0 && dev < kMaxDevices && g_static_scratch[dev] != nullptr)
            hipLaunchKernelGGL(heinsen_scratch_set_epoch, dim3(1), dim3(64), 0, stream, g_static_scratch[dev], epoch);
        if (!hip_ok(hipGetLastError())) return HEINSEN_ERR_HIP;
    }
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
    case HEINSEN_ERR_CARRY_LOST: return "a tile gave up waiting for a carry record (two launches shared one scratch buffer?)";
    case HEINSEN_ERR_SCRATCH_LIMIT: return "the call needs more scratch than the fixed buffer of heinsen_scan_static holds";
    default: return "unknown status";
    }
}

int heinsen_last_hip_error(void) { return t_last_hip_error; }

int heinsen_version(void) { return 301; /* 0.3.1: 0.3.0 (heinsen_scan_static, heinsen_check, heinsen_set_timeline) + heinsen_tile_shape */ }

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
        if (kv.second.records) (void)hipFree(kv.second.records);
        for (unsigned long long *old : kv.second.retired) (void)hipFree(old);
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

int heinsen_tile_shape(int64_t B, int64_t D, int64_t n, int layout, uint32_t flags, int *sequences, int64_t *steps)
{
    if (!sequences || !steps) return HEINSEN_ERR_INVALID_ARG;
    hs::ScanCall c = {};
    bool bnd = false;
    int st = describe(B, D, n, layout, flags, c, bnd);
    if (st != HEINSEN_OK) return st;
    if (bnd) hs::bnd_tile_shape(c, *sequences, *steps);
    else hs::bdn_tile_shape(c, *sequences, *steps);
    return HEINSEN_OK;
}

} // extern "C"
