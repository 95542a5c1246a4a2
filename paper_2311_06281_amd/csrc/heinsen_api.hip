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

// One buffer of tagged 64-bit records per (device, stream); see heinsen_internal.hpp.
struct Scratch {
    unsigned long long *records = nullptr;
    size_t capacity = 0;      // in records, including the header
    uint32_t epoch = 0;       // epoch of the last ordinary launch (even; 0: none yet)
    uint32_t ticket_base = 0; // value of the ticket counter when the next ordinary launch starts
    bool in_graph = false;    // a captured launch holds this buffer's address: it is not freed on growth
    std::vector<unsigned long long *> retired; // such buffers, replaced by larger ones; freed on release
};

// Recorded in front of every captured launch (one workgroup): gives the replay a fresh odd epoch and a
// ticket counter at zero.  When the 30-bit epoch comes round, the records are cleared so that no tag of
// an earlier cycle can match.
__global__ void heinsen_graph_prologue(unsigned long long *records, size_t capacity)
{
    __shared__ uint32_t s_next, s_wrap;
    if (threadIdx.x == 0) {
        const uint32_t e = (uint32_t)records[hs::kHeaderGraphEpoch];
        const uint32_t ne = e == 0 ? 1u : e + 2u;
        s_wrap = ne >= (1u << 30) ? 1u : 0u;
        s_next = s_wrap ? 1u : ne;
    }
    __syncthreads();
    if (s_wrap)
        for (size_t i = hs::kRecordBase + threadIdx.x; i < capacity; i += blockDim.x) records[i] = 0;
    __syncthreads();
    if (threadIdx.x == 0) {
        records[hs::kHeaderGraphTicket] = 0;
        records[hs::kHeaderGraphEpoch] = s_next;
    }
}

std::mutex g_mutex;
std::map<std::pair<int, hipStream_t>, Scratch> g_scratch;

// Scratch of heinsen_scan_static: one fixed array per GPU, part of the loaded code, never allocated or
// freed.  In host code the array's name is not a device address; the address on each device is looked
// up once (hipGetSymbolAddress with that device current) and kept here.
constexpr size_t kStaticRecords = ((size_t)40 << 20) / sizeof(unsigned long long); // 40 MiB
static __device__ __align__(256) unsigned long long scratch[kStaticRecords];
constexpr int kMaxDevices = 64;
unsigned long long *g_static_scratch[kMaxDevices] = {};

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

// Makes sure the stream's record buffer can hold `need`, and hands out the tag of the next launch.
// Called with g_mutex held; the caller keeps it until the kernel is enqueued so that launches enter
// the stream in epoch order.
int prepare_launch(hipStream_t stream, const hs::ScratchNeed &need, Scratch *&out, hs::LaunchTag &tag)
{
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev))) return HEINSEN_ERR_HIP;
    Scratch &s = g_scratch[std::make_pair(dev, stream)];
    const size_t want = hs::kRecordBase + need.records;
    const bool wrap = s.epoch >= 0x3ffffffcu; // 30-bit epochs: start over on a cleared buffer
    if (s.capacity < want || wrap) {
        // work queued on the old buffer must drain before it is replaced or cleared
        if (s.records && !hip_ok(hipStreamSynchronize(stream))) return HEINSEN_ERR_HIP;
        if (s.capacity < want) {
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
            s.records = static_cast<unsigned long long *>(ptr);
            s.capacity = cap;
        }
        if (!hip_ok(hipMemset(s.records, 0, s.capacity * sizeof(unsigned long long)))) return HEINSEN_ERR_HIP;
        s.epoch = 0;
        s.ticket_base = 0;
    }
    s.epoch += 2; // even: launches replayed from graphs use the odd ones
    tag.epoch = s.epoch;
    tag.ticket_base = s.ticket_base;
    tag.from_header = false;
    s.ticket_base += need.tickets; // wraps modulo 2^32 together with the device counter
    out = &s;
    return HEINSEN_OK;
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
    if (need.records == 0 && need.tickets == 0) {
        hipError_t e = bnd ? hs::bnd_launch(c, nullptr, hs::LaunchTag{0, 0, false}) : hs::bdn_launch(c, nullptr, hs::LaunchTag{0, 0, false});
        return hip_ok(e) ? HEINSEN_OK : HEINSEN_ERR_HIP;
    }
    // The carry records are told apart by a per-launch epoch.  An ordinary launch gets it from the host;
    // a launch that is recorded once and replayed many times (HIP graph capture) cannot, and nothing may
    // be allocated while a stream is capturing: such a call uses the scratch the stream already has (an
    // earlier ordinary call of at least this size made it) and takes epoch and tickets from its header,
    // which a small kernel recorded in front of it renews at every replay.
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (c.stream != nullptr && hipStreamIsCapturing(c.stream, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone) {
        std::lock_guard<std::mutex> lock(g_mutex);
        int dev = 0;
        if (!hip_ok(hipGetDevice(&dev))) return HEINSEN_ERR_HIP;
        auto it = g_scratch.find(std::make_pair(dev, c.stream));
        if (it == g_scratch.end() || it->second.capacity < hs::kRecordBase + need.records) return HEINSEN_ERR_UNSUPPORTED;
        Scratch &sc = it->second;
        sc.in_graph = true;
        hipLaunchKernelGGL(heinsen_graph_prologue, dim3(1), dim3(256), 0, c.stream, sc.records, sc.capacity);
        if (!hip_ok(hipGetLastError())) return HEINSEN_ERR_HIP;
        const hs::LaunchTag gtag{0, 0, true};
        hipError_t e = bnd ? hs::bnd_launch(c, sc.records, gtag) : hs::bdn_launch(c, sc.records, gtag);
        return hip_ok(e) ? HEINSEN_OK : HEINSEN_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(g_mutex);
    Scratch *s = nullptr;
    hs::LaunchTag tag{0, 0, false};
    st = prepare_launch(c.stream, need, s, tag);
    if (st != HEINSEN_OK) return st;
    hipError_t e = bnd ? hs::bnd_launch(c, s->records, tag) : hs::bdn_launch(c, s->records, tag);
    if (!hip_ok(e)) return HEINSEN_ERR_HIP;
    return HEINSEN_OK;
}

int heinsen_scan_static(const void *a, const void *b, const void *x0, void *out, int64_t B, int64_t D, int64_t n,
                        int layout, uint32_t flags, void *stream)
{
    hs::ScanCall c = {};
    bool bnd = false;
    int st = make_call(a, b, x0, out, B, D, n, layout, flags, stream, c, bnd);
    if (st != HEINSEN_OK) return st;
    const hs::ScratchNeed need = bnd ? hs::bnd_scratch(c) : hs::bdn_scratch(c);
    if (need.records == 0 && need.tickets == 0) {
        hipError_t e = bnd ? hs::bnd_launch(c, nullptr, hs::LaunchTag{0, 0, false}) : hs::bdn_launch(c, nullptr, hs::LaunchTag{0, 0, false});
        return hip_ok(e) ? HEINSEN_OK : HEINSEN_ERR_HIP;
    }
    if (hs::kRecordBase + need.records > kStaticRecords) return HEINSEN_ERR_SCRATCH_LIMIT;
    std::lock_guard<std::mutex> lock(g_mutex);
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev))) return HEINSEN_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return HEINSEN_ERR_UNSUPPORTED;
    if (g_static_scratch[dev] == nullptr) {
        unsigned long long *ptr = nullptr;
        if (!hip_ok(hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch))) || ptr == nullptr)
            return HEINSEN_ERR_HIP;
        g_static_scratch[dev] = ptr;
    }
    unsigned long long *records = g_static_scratch[dev];
    // The array keeps whatever the last call left in it.  Nothing has to be cleared: the one-workgroup
    // kernel in front of the scan gives this call a launch counter no record in the array carries yet and
    // a ticket counter at zero (and clears the records itself when the counter comes round).
    hipLaunchKernelGGL(heinsen_graph_prologue, dim3(1), dim3(256), 0, c.stream, records, kStaticRecords);
    if (!hip_ok(hipGetLastError())) return HEINSEN_ERR_HIP;
    const hs::LaunchTag tag{0, 0, true};
    hipError_t e = bnd ? hs::bnd_launch(c, records, tag) : hs::bdn_launch(c, records, tag);
    return hip_ok(e) ? HEINSEN_OK : HEINSEN_ERR_HIP;
}

const char *heinsen_status_string(int status)
{
    switch (status) {
    case HEINSEN_OK: return "ok";
    case HEINSEN_ERR_INVALID_ARG: return "invalid argument";
    case HEINSEN_ERR_UNSUPPORTED: return "unsupported combination of arguments";
    case HEINSEN_ERR_ALLOC: return "scratch allocation failed";
    case HEINSEN_ERR_HIP: return "HIP runtime error";
    case HEINSEN_ERR_SCRATCH_LIMIT: return "the call needs more scratch than the fixed buffer of heinsen_scan_static holds";
    default: return "unknown status";
    }
}

int heinsen_last_hip_error(void) { return t_last_hip_error; }

int heinsen_version(void) { return 200; /* 0.2.0: OUT_COMPLEX, LINEAR */ }

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

} // extern "C"
