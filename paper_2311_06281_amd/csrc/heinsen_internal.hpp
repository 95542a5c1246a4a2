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
    float *out;
    int64_t B, D, n;      // for the sequence-contiguous path: rows = B*D, row length n
    bool is_signed;       // sign tracking needed (neither POSITIVE nor LOG_INPUTS)
    bool log_in, log_out; // natural-log inputs / output
    bool bf16;            // a, b stored as bfloat16
    bool x0_scalar;       // one x0 for all sequences
    bool vec_ok;          // pointers and row pitch allow 16-byte vector access
    hipStream_t stream;
};

// Scratch comes in two buffers per (device, stream): `flags` holds counters and ready-flags and is
// all-zero whenever no kernel is running (allocated zeroed; every kernel restores the zeros it
// disturbed before it finishes), `data` holds the published summaries and may contain anything.
struct ScratchNeed {
    size_t flag_bytes;
    size_t data_bytes;
};

// Each path reports how much scratch it needs (either may be 0), launches on call.stream, and names
// the kernel it would launch.  The layouts inside the two buffers are private to each path.
ScratchNeed bnd_scratch(const ScanCall &c);
hipError_t bnd_launch(const ScanCall &c, void *flags, void *data);
const char *bnd_kernel_name(const ScanCall &c);

ScratchNeed bdn_scratch(const ScanCall &c);
hipError_t bdn_launch(const ScanCall &c, void *flags, void *data);
const char *bdn_kernel_name(const ScanCall &c);

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Expands to a switch over the ten legal (SIGNED, LOG_IN, LOG_OUT, InT) combinations and invokes
// F<SIGNED, LOG_IN, LOG_OUT, InT>(__VA_ARGS__).
#define HS_DISPATCH_MODE(call, F, ...)                                                         \
    do {                                                                                       \
        const ::hs::ScanCall &c_ = (call);                                                     \
        if (c_.bf16) {                                                                         \
            if (c_.log_in) {                                                                   \
                if (c_.log_out) return F<false, true, true, uint16_t>(__VA_ARGS__);            \
                return F<false, true, false, uint16_t>(__VA_ARGS__);                           \
            }                                                                                  \
            if (c_.is_signed) return F<true, false, false, uint16_t>(__VA_ARGS__);             \
            if (c_.log_out) return F<false, false, true, uint16_t>(__VA_ARGS__);               \
            return F<false, false, false, uint16_t>(__VA_ARGS__);                              \
        } else {                                                                               \
            if (c_.log_in) {                                                                   \
                if (c_.log_out) return F<false, true, true, float>(__VA_ARGS__);               \
                return F<false, true, false, float>(__VA_ARGS__);                              \
            }                                                                                  \
            if (c_.is_signed) return F<true, false, false, float>(__VA_ARGS__);                \
            if (c_.log_out) return F<false, false, true, float>(__VA_ARGS__);                  \
            return F<false, false, false, float>(__VA_ARGS__);                                 \
        }                                                                                      \
    } while (0)

} // namespace hs
