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
    size_t scratch_budget; // 64-bit words of scratch the call may use, header included (0: no limit)
    hipStream_t stream;
};

// Scratch is one buffer of 64-bit words: a header, then the tagged carry records (see heinsen_math.hpp).
//
// Header.  Words 16*q, q = 0..7, are the ticket queues, each on a 128-byte line of its own.  A queue word is
// {launch counter ("epoch"): high 32 bits | next ticket: low 32 bits}: one fetch-add hands a workgroup its
// tile and the epoch its carry records are tagged with.  A launch draws a fixed number of tickets from
// each queue it uses (its grid size over the number of queues); the workgroup that draws the last ticket
// of a queue knows that nobody will draw from it again in this launch, and the one that completes the last
// queue (kHeaderQueuesDone counts them) rewrites all eight queue words to {epoch + 1 | 0}.  So every launch,
// ordinary or replayed from a HIP graph, finds the queues at zero with an epoch no record carries yet,
// without any bookkeeping on the host and without anything to undo when a launch fails.  Epochs run
// 1 .. 2^30 - 1; the launch that has the last one clears the records when its last workgroup ends.
// Other header words: the buffer's size, an error word (a carry wait that gave up), and the two counters
// just named.  Records start at kRecordBase.
constexpr int kQueues = 8;                 // one per compute die
constexpr size_t kQueueStride = 16;        // words between queue counters (128 bytes)
constexpr size_t kHeaderCapacity = kQueueStride * kQueues;    // size of the buffer in words, header included
constexpr size_t kHeaderError = kHeaderCapacity + 1;          // non-zero: some tile gave up waiting for a carry record
constexpr size_t kHeaderQueuesDone = kHeaderCapacity + 16;    // queues of the current launch that have handed out all their tickets
constexpr size_t kHeaderExited = kHeaderCapacity + 32;        // workgroups that have ended (counted only by the launch that clears)
constexpr size_t kRecordBase = kHeaderCapacity + 128;
constexpr uint32_t kLastEpoch = (1u << 30) - 1u;

// What the host tells a launch that uses carry records.
struct LaunchCtx {
    unsigned long long *scratch;   // header + records; null when the launch needs no carries
    uint32_t spin_limit;           // polls after which a tile gives up waiting for a carry record
    uint32_t drop_tile;            // testing aid: this tile never publishes its summary (0xffffffff: none)
    unsigned long long *timeline;  // optional [timeline_tiles][8] wall-clock stamps per tile, or null
    uint32_t timeline_tiles;
};

// Each path reports how many records it needs beyond kRecordBase (may be 0), launches on call.stream, and
// names the kernel it would launch.
struct ScratchNeed {
    size_t records;
};
ScratchNeed bnd_scratch(const ScanCall &c);
hipError_t bnd_launch(const ScanCall &c, const LaunchCtx &ctx);
const char *bnd_kernel_name(const ScanCall &c);
void bnd_tile_shape(const ScanCall &c, int &channels, int64_t &steps); // of one workgroup

ScratchNeed bdn_scratch(const ScanCall &c);
hipError_t bdn_launch(const ScanCall &c, const LaunchCtx &ctx);
const char *bdn_kernel_name(const ScanCall &c);
void bdn_tile_shape(const ScanCall &c, int &rows, int64_t &steps); // of one workgroup

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
