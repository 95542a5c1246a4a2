// Host-side plumbing shared by the translation units of libheinsen (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace hs {

// Validated description of one heinsen_scan call, as seen by the kernel launchers.
struct ScanCall {
    const void *a;
    const void *b;
    const float *x0;
    float *out;           // float32 per element, or (re, im) pairs when is_signed && log_out
    int64_t B, D, n;      // for the sequence-contiguous path: rows = B*D, row length n
    bool is_signed;       // sign tracking needed (neither POSITIVE nor LOG_INPUTS)
    bool log_in, log_out; // natural-log inputs / output
    bool linear;          // linear-domain comparison path (no logarithms anywhere)
    bool bf16;            // a, b stored as bfloat16
    bool x0_scalar;       // one x0 for all sequences
    hipStream_t stream;
};

// Scratch is one buffer of 64-bit tagged records per (device, stream) (see heinsen_math.hpp).  Header
// words: 0 = ticket counter of ordinary launches, 1 = ticket counter and 16 = epoch of launches replayed
// from a HIP graph; carry records start at kRecordBase.  (The epoch, which every workgroup reads, has a
// 128-byte line of its own: on the line of a ticket counter its readers would queue with the atomics.)
// Every launch gets a fresh epoch, so the buffer never needs clearing.  An ordinary launch gets its
// epoch (even) and `ticket_base`, the value word 0 has when the launch starts, from the host, which
// adds the tickets drawn after every launch.  A launch recorded into a graph cannot: the same kernel
// arguments are replayed many times.  It reads its epoch (odd) from word 16 and draws tickets from
// word 1, both set by a one-workgroup kernel recorded in front of it (heinsen_api.hip), and leaves
// word 0 and the host's copy of it alone.
constexpr size_t kRecordBase = 32;
constexpr size_t kHeaderGraphTicket = 1, kHeaderGraphEpoch = 16;

struct LaunchTag {
    uint32_t epoch;       // 2, 4, .. 2^30 - 2 (ignored when from_header)
    uint32_t ticket_base; // ticket counter value at launch (ignored when from_header)
    bool from_header;     // launch recorded into a graph: epoch and tickets come from the header
};

// Each path reports how many records it needs beyond kRecordBase (may be 0) and how many tickets a
// launch draws, launches on call.stream, and names the kernel it would launch.
struct ScratchNeed {
    size_t records;
    uint32_t tickets;
};
ScratchNeed bnd_scratch(const ScanCall &c);
hipError_t bnd_launch(const ScanCall &c, unsigned long long *records, LaunchTag tag);
const char *bnd_kernel_name(const ScanCall &c);

ScratchNeed bdn_scratch(const ScanCall &c);
hipError_t bdn_launch(const ScanCall &c, unsigned long long *records, LaunchTag tag);
const char *bdn_kernel_name(const ScanCall &c);

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Expands to a switch over the fourteen legal (DOM, LOG_IN, LOG_OUT, InT) combinations and invokes
// F<DOM, LOG_IN, LOG_OUT, InT>(__VA_ARGS__); DOM is 0 (positive), 1 (signed) or 2 (linear), see heinsen_math.hpp.
#define HS_DISPATCH_MODE(call, F, ...)                                                         \
    do {                                                                                       \
        const ::hs::ScanCall &c_ = (call);                                                     \
        if (c_.bf16) {                                                                         \
            if (c_.linear) return F<2, false, false, uint16_t>(__VA_ARGS__);                   \
            if (c_.log_in) {                                                                   \
                if (c_.log_out) return F<false, true, true, uint16_t>(__VA_ARGS__);            \
                return F<false, true, false, uint16_t>(__VA_ARGS__);                           \
            }                                                                                  \
            if (c_.is_signed && c_.log_out) return F<true, false, true, uint16_t>(__VA_ARGS__); \
            if (c_.is_signed) return F<true, false, false, uint16_t>(__VA_ARGS__);             \
            if (c_.log_out) return F<false, false, true, uint16_t>(__VA_ARGS__);               \
            return F<false, false, false, uint16_t>(__VA_ARGS__);                              \
        } else {                                                                               \
            if (c_.linear) return F<2, false, false, float>(__VA_ARGS__);                      \
            if (c_.log_in) {                                                                   \
                if (c_.log_out) return F<false, true, true, float>(__VA_ARGS__);               \
                return F<false, true, false, float>(__VA_ARGS__);                              \
            }                                                                                  \
            if (c_.is_signed && c_.log_out) return F<true, false, true, float>(__VA_ARGS__);    \
            if (c_.is_signed) return F<true, false, false, float>(__VA_ARGS__);                \
            if (c_.log_out) return F<false, false, true, float>(__VA_ARGS__);                  \
            return F<false, false, false, float>(__VA_ARGS__);                                 \
        }                                                                                      \
    } while (0)

} // namespace hs
