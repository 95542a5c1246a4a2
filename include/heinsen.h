/*
 * heinsen.h -- C ABI of libheinsen: the first-order linear recurrence
 *
 *        x_t = a_t * x_{t-1} + b_t ,  t = 1..n ,  x_0 given            (paper: Abstract; Sec. 3)
 *
 * evaluated on one AMD MI355X (gfx950) for B*D independent sequences with the paper's log-space
 * closed form (Sec. 1 Eq. (1)-(2); stabilised form of Sec. 4):
 *
 *        a*_t     = cumsum_t  log a_t
 *        log x_t  = a*_t + LCSE( cat(log x_0, log b_t - a*_t) )_t ,    LCSE := log cumsum exp
 *
 * Both prefix sums are carried by one associative pair so every element crosses HBM once.  Negative
 * a_t, b_t, x_0 (complex logarithms in the paper, Sec. 1 last paragraph) are carried as a real
 * logarithm of the magnitude plus a sign bit.
 *
 * All data pointers are DEVICE pointers owned by the caller.  Nothing is retained after a call
 * returns except library-owned scratch memory (see heinsen_release_scratch).  No torch types, no
 * C++ types, no exceptions cross this boundary.
 */
#ifndef HEINSEN_H
#define HEINSEN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Memory layout of a, b and out (x0 is always [B, D]).  t below is 0-based; out[t] = x_{t+1}:
 * the initial value x_0 is an input only and is never written (tail() in Sec. 4). */
typedef enum {
    HEINSEN_LAYOUT_BND = 0, /* [B, n, D] channel-contiguous : element (b,t,d) at ((b*n + t)*D + d) */
    HEINSEN_LAYOUT_BDN = 1  /* [B, D, n] sequence-contiguous: element (b,t,d) at ((b*D + d)*n + t) */
} heinsen_layout_t;

/* Flag bits. */
enum {
    HEINSEN_LOG_INPUTS = 1u << 0, /* a, b, x0 hold natural logs log a_t, log b_t, log x_0 (all quantities
                                     positive; -inf encodes 0).  Eq. (2) then starts from these logs.  */
    HEINSEN_LOG_OUTPUT = 1u << 1, /* out receives log x_t (Eq. (1)) instead of x_t (Eq. (3)).  Needs a
                                     positive domain (LOG_INPUTS or POSITIVE also set) or OUT_COMPLEX.  */
    HEINSEN_IN_BF16    = 1u << 2, /* a and b are stored as bfloat16 (x0 and out stay float32).          */
    HEINSEN_POSITIVE   = 1u << 3, /* caller promises a_t > 0, b_t >= 0, x_0 >= 0: sign tracking skipped.
                                     With a negative input the result is unspecified but memory-safe.   */
    HEINSEN_X0_SCALAR  = 1u << 4, /* x0 points to ONE float32 that is broadcast to all B*D sequences.    */
    HEINSEN_OUT_COMPLEX = 1u << 5, /* with LOG_OUTPUT on signed data: out holds B*D*n complex64 values
                                     (re, im interleaved), the complex logarithm of x_t (Sec. 1, last
                                     paragraph): re = log|x_t|, im = pi where x_t < 0, else 0; x_t = 0
                                     gives re = -inf.  Signs are always tracked (POSITIVE is ignored).
                                     Not available with LOG_INPUTS.                                     */
    HEINSEN_LINEAR     = 1u << 6  /* comparison path: the same single-pass scan with the plain operator
                                     (a1, b1) o (a2, b2) = (a1 a2, a2 b1 + b2) of the general formulation
                                     the paper compares itself with (Sec. 2), in float32, without any
                                     logarithm.  Partial products of a_t over up to a tile group of steps
                                     are formed, so they overflow or flush where the log-space form does
                                     not.  Excludes LOG_INPUTS, LOG_OUTPUT, OUT_COMPLEX; POSITIVE is
                                     ignored.                                                            */
};

typedef enum {
    HEINSEN_OK = 0,
    HEINSEN_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, size overflow, misaligned pointer,
                                    unknown layout or flag bit, contradictory flags (OUT_COMPLEX without
                                    LOG_OUTPUT, LINEAR with a log-domain flag)                           */
    HEINSEN_ERR_UNSUPPORTED = 2, /* a legal but unimplemented combination: LOG_OUTPUT on a signed domain
                                    without OUT_COMPLEX, OUT_COMPLEX with LOG_INPUTS, a call that needs
                                    scratch recorded into a graph on a stream that has none yet         */
    HEINSEN_ERR_ALLOC = 3,       /* scratch memory could not be allocated; nothing was launched          */
    HEINSEN_ERR_HIP = 4,         /* a HIP runtime call failed; see heinsen_last_hip_error()              */
    HEINSEN_ERR_SCRATCH_LIMIT = 5, /* heinsen_scan_static only: the shape needs more scratch than its fixed
                                    buffer holds; nothing was launched                                   */
    HEINSEN_ERR_CARRY_LOST = 6   /* heinsen_check only: a tile gave up waiting for a carry record and wrote
                                    NaN from there on (two launches used one scratch buffer at once)     */
} heinsen_status_t;

/*
 * heinsen_scan -- compute x_1..x_n of every sequence (Sec. 3 definition, via Sec. 4's expression).
 *
 *   a_or_log_a, b_or_log_b : device, B*D*n elements in `layout`; float32, or bfloat16 with IN_BF16.
 *                            With LOG_INPUTS they hold natural logarithms.
 *   x0                     : device, B*D float32 indexed [b*D + d] (or 1 value with X0_SCALAR);
 *                            log x_0 with LOG_INPUTS.
 *   out                    : device, B*D*n float32 in `layout`; x_t, or log x_t with LOG_OUTPUT
 *                            (B*D*n complex64, 8-byte aligned, with OUT_COMPLEX; no aliasing then).
 *                            May be exactly a_or_log_a or b_or_log_b when those are float32 (every tile
 *                            reads its inputs before it writes; "in situ", Sec. 1); any other overlap
 *                            is undefined.
 *   B, D, n                : batch, channels, sequence length; all >= 1 and B*D*n < 2^62 (beyond 2^42
 *                            elements the call is refused as unsupported: tile counters are 32-bit).
 *   layout                 : a heinsen_layout_t value.
 *   flags                  : OR of the flag bits above.
 *   stream                 : a hipStream_t (NULL = the default stream).
 *
 * Asynchronous: work is enqueued on `stream` and the call returns without synchronising.  The
 * returned status covers argument validation, scratch allocation and launch errors only.
 *
 * Scratch: a grow-only buffer per (device, stream) holds the inter-tile carries and the ticket queues
 * that hand out the tiles.  It is allocated with hipMalloc on the first call that needs it or needs more
 * (that call synchronises the stream if it replaces a buffer) and cleared by a small kernel on `stream`;
 * later calls of the same or smaller shape allocate nothing.  Calls on different streams never share
 * scratch; calls on one stream may come from several host threads.  Carries of different launches are
 * told apart by a launch counter that lives in the buffer and is renewed by the kernels themselves, so the
 * host keeps no per-launch state, a failed launch leaves nothing to repair, and a call recorded into a
 * HIP graph (stream capture) replays like any other.  Such a call may not allocate, though: it uses the
 * scratch its stream already has -- make one ordinary call of at least the same shape on that stream
 * first, as a warm-up does -- and without it is refused with HEINSEN_ERR_UNSUPPORTED, nothing recorded.
 * A graph keeps using the scratch it was recorded with (a later, larger ordinary call gets a new buffer
 * and the old one lives on until heinsen_release_scratch): its replays must not overlap with one another
 * or with ordinary calls on the stream it was recorded on, and heinsen_release_scratch must not be called
 * while the graph may still be replayed.  Two launches that do use one buffer at the same time get wrong
 * results but always end: a tile whose carry never arrives gives up after a few seconds of polling, writes
 * NaN from there on and leaves a note that heinsen_check reports.  Shapes that need no carries (sequences
 * of at most 16384 steps in the [B, D, n] layout and of at most 64 steps in [B, n, D]) use no scratch.
 *
 * Data-dependent conditions are not errors and follow IEEE arithmetic: a NaN input gives NaN from
 * that step on in that sequence only; a_t = 0 restarts the sequence at b_t; b_t = 0 and x_0 = 0 are
 * ordinary values; magnitudes beyond float32 give +-inf.  float32 subnormal inputs are read as 0
 * and subnormal results are written as 0.  Results are bit-reproducible from run to run.
 *
 * Returns a heinsen_status_t.
 */
int heinsen_scan(const void *a_or_log_a, const void *b_or_log_b, const void *x0, void *out,
                 int64_t B, int64_t D, int64_t n, int layout, uint32_t flags, void *stream);

/*
 * heinsen_scan_static -- heinsen_scan for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels.  It
 * never calls hipMalloc, hipFree or any allocating routine: the inter-tile carries live in a fixed
 * 48 MiB device array that is part of the library (each GPU the library runs on holds its own copy
 * until the process ends).  Results are those of heinsen_scan bit for bit, except for large [B, n, D]
 * shapes whose preferred (wider) tiles would not fit the array: those run with the narrower tiles, whose
 * float32 rounding differs in the last bits.
 *
 *   limit   : shapes whose carries do not fit are refused with HEINSEN_ERR_SCRATCH_LIMIT and nothing is
 *             launched.  In records of 8 bytes, 256 + the following must stay within 6 * 2^20:
 *               [B, n, D], n > 64 : about 160 * ceil(D/64) * B * ceil(n/256)
 *               [B, D, n], n > 16384 : about 16 * B * D * ceil(n/16384) * 1.04
 *             (all five benchmark shapes fit; [16, 16384, 2048] float32 takes 40 of the 48 MiB.)  Shapes
 *             that need no carries have no limit.
 *   sharing : every call on a GPU uses that GPU's one array, whatever the stream.  Calls that may run at
 *             the same time on one GPU race on it and give wrong results: keep them on one stream or
 *             order them with events.  heinsen_scan's own scratch is separate and never conflicts.
 *   capture : may be recorded into a HIP graph; the first call on a device looks up the array's address
 *             (hipGetSymbolAddress), clears it with a small kernel and synchronises `stream` once, and
 *             must be made outside a capture (inside one it is refused with HEINSEN_ERR_UNSUPPORTED).
 * Returns a heinsen_status_t.
 */
int heinsen_scan_static(const void *a_or_log_a, const void *b_or_log_b, const void *x0, void *out,
                        int64_t B, int64_t D, int64_t n, int layout, uint32_t flags, void *stream);

/*
 * heinsen_check -- synchronises `stream` and reports whether any launch since the last check gave up
 * waiting for a carry record, in the scratch of (current device, stream) or in the fixed array of
 * heinsen_scan_static on the current device.  Returns HEINSEN_OK, or HEINSEN_ERR_CARRY_LOST after
 * putting the affected buffer back into its initial state (outputs written by the launches concerned
 * hold NaN from the failing tile on).  Never needed in correct use; meant for debugging concurrency.
 */
int heinsen_check(void *stream);

/* Static, NUL-terminated description of a heinsen_status_t value (never NULL). */
const char *heinsen_status_string(int status);

/* The hipError_t of the last failing HIP call made by this thread inside the library
 * (0 = hipSuccess).  Meaningful after HEINSEN_ERR_HIP or HEINSEN_ERR_ALLOC. */
int heinsen_last_hip_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int heinsen_version(void);

/* Frees every cached scratch buffer (synchronises the devices involved).  Optional: call when no
 * heinsen_scan is in flight, e.g. before unloading the library.  Returns a heinsen_status_t. */
int heinsen_release_scratch(void);

/* Name of the kernel heinsen_scan would launch for these arguments (for profilers), written as a
 * NUL-terminated string into buf (at most buflen bytes).  Launches nothing.  Returns a
 * heinsen_status_t from the same validation heinsen_scan performs (pointers are not checked). */
/* The piece of the problem one workgroup of that kernel takes ("tile"): `sequences` adjacent sequences
 * (channels of [B, n, D], rows of [B, D, n]) for `steps` consecutive steps (the last tile of a sequence may
 * be shorter).  For profilers and for reading the tile ids of heinsen_set_timeline.  Launches nothing.
 * Returns a heinsen_status_t from the same validation heinsen_scan performs (pointers are not checked). */
int heinsen_tile_shape(int64_t B, int64_t D, int64_t n, int layout, uint32_t flags, int *sequences,
                       int64_t *steps);

int heinsen_kernel_name(int64_t B, int64_t D, int64_t n, int layout, uint32_t flags, char *buf,
                        int buflen);

/*
 * heinsen_sequential -- the baseline of the paper's experiment (Sec. 4, Fig. 1): ONE sequence computed
 * one element after the other on the GPU, x_t = a_t x_{t-1} + b_t in float32 (Sec. 3), by a single lane.
 * a, b, out: device, n float32 each; x0: device, one float32; out[t-1] = x_t.  Asynchronous on `stream`.
 * It exists to be timed against heinsen_scan; it is not a fallback of anything.
 * Returns a heinsen_status_t.
 */
int heinsen_sequential(const void *a, const void *b, const void *x0, void *out, int64_t n, void *stream);

/*
 * heinsen_stream_probe -- measurement aid: out = a + b over a [B, n, D] float32 array (device pointers,
 * B*n*D elements each) with nothing but the memory access pattern of a scan kernel, all accesses
 * non-temporal.  What it reaches is the ceiling of that pattern on the machine at hand, the yardstick
 * beside the published peak.  pattern: 0 the array as one long vector, 16 bytes per lane; 1 the default
 * tile of the [B, n, D] kernel (workgroup = 64 channels x 256 steps, rows of 256 bytes); 2 its wide tile
 * (128 channels x 128 steps, rows of 512 bytes); 3 256 channels x 64 steps; 4, 5, 6 = 1, 2, 3 with no output
 * stored before all of a lane's inputs have arrived, as in a scan; 7 as 0 with a and b stored as bf16
 * (B*n*D elements of 2 bytes each, 8-byte aligned; out float32): the traffic mix of bf16 storage, one
 * byte read per byte written.  Patterns 1..6 need D a multiple of 64, 128, 256 and n a multiple of 256,
 * 128, 64, patterns 0 and 7 B*n*D a multiple of 4 (HEINSEN_ERR_UNSUPPORTED otherwise).  Asynchronous on
 * `stream`.  Returns a heinsen_status_t.
 */
int heinsen_stream_probe(const void *a, const void *b, void *out, int64_t B, int64_t n, int64_t D, int pattern,
                         void *stream);

/*
 * heinsen_set_timeline -- profiling aid (the per-tile view that a kernel-level profiler cannot give).
 * While set, every tile of every later launch of the two carry-chained kernels writes eight 64-bit
 * time stamps of the GPU's 100 MHz wall clock to stamps[tile * 8 + i], for tiles below `tiles`:
 *   0 workgroup started, 1 ticket drawn (tile known), 2 inputs loaded and scanned in the lanes,
 *   3 summary handed to the other waves, 4 carry records of the earlier tiles in, 5 start state known,
 *   6 outputs issued, 7 end (all taken by the tile's first wave).
 * Tile ids: [B, n, D]: chunk * columns + column; [B, D, n]: row-major.
 * stamps: device memory, 8-byte aligned, tiles * 64 bytes, owned by the caller; (NULL, 0) switches the
 * stamps off again (a launch without them pays one untaken branch per stamp).  Process-wide setting.
 * Returns a heinsen_status_t.
 */
int heinsen_set_timeline(void *stamps, uint64_t tiles);

/*
 * heinsen_test_carry -- testing aid for the error path of the carry chain; not for production use.
 *   spin_limit : polls after which a tile gives up waiting for a carry record (0 = the default, seconds);
 *   drop_tile  : this tile id never publishes its summary, as if another launch had overwritten it
 *                (0xffffffff = none);
 *   epoch      : if non-zero, a small kernel on `stream` sets the launch counter of the stream's scratch
 *                and of the fixed array to this value (1 .. 2^30 - 1), e.g. just before it comes round.
 * Process-wide settings.  Every kernel still ends normally.  Returns a heinsen_status_t.
 */
int heinsen_test_carry(uint32_t spin_limit, uint32_t drop_tile, uint32_t epoch, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HEINSEN_H */
