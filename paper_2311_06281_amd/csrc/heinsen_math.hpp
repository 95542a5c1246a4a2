// Device-side arithmetic of the fused log-space scan (gfx950, wave64).
//
// A real number v is carried as (log2|v|, sign) -- the complex logarithm of the paper (Sec. 1, last
// paragraph) has imaginary part 0 or pi, which is one bit.  Logs are base 2 inside the kernels because
// v_log_f32 / v_exp_f32 are base 2; natural logs appear only at the API (LOG_INPUTS / LOG_OUTPUT).
//
// A segment of consecutive steps s+1..e of x_t = a_t x_{t-1} + b_t is summarised by the pair
//     A = sum log|a_t|                 (first prefix sum of Eq. (2))
//     M = log| sum_t b_t prod_{u>t} a_u |   (what the segment contributes when it starts from 0)
// so that x_e = (+-2^A) x_s + (+-2^M).  M = A + L where L = log of the second prefix sum of Eq. (2);
// carrying M instead of L keeps every addend at the size of its actual contribution, so float32 never
// has to cancel two large numbers (Eq. (1) adds a*_t and a logarithm of opposite size).
// Composition (Sec. 1, footnote: prefix sums are associative, so they can be computed by parts):
//     (A1,M1) then (A2,M2)  =  (A1 + A2,  slae(M1 + A2, M2)).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hs {

typedef unsigned long long rec_t; // a tagged carry record, see the end of this file

// Sign words: bit 31 is the sign (1 = negative); the other 31 bits are undefined and every consumer
// either ignores them or masks them.  This lets the raw bits of an input float serve as its sign word.

// Domain of the scan, the first template argument of everything below.  A bool converts to the first two
// (false: positive, true: signed), which is how most callers name them.
//   kPositive, kSigned: the paper's log-space form (Sec. 1, Sec. 4); A = sum of log2|a|, M = log2 of the
//                       segment's zero-input response, signs tracked or not;
//   kLinear:            the same scan with the plain operator (a1, b1) o (a2, b2) = (a1 a2, a2 b1 + b2) of the
//                       general formulation the paper compares itself with (Sec. 2): A = product of a,
//                       M = zero-input response, no logarithms.  A comparison path.
constexpr int kPositive = 0, kSigned = 1, kLinear = 2;

constexpr float kLog2e = 1.44269504088896340736f;
constexpr float kLn2 = 0.69314718055994530942f;
constexpr uint32_t kSignBit = 0x80000000u;

__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float log2_hw(float x) { return __builtin_amdgcn_logf(x); }
__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }

// Signed log-add-exp (the scan operator of Sec. 4's LCSE, extended to signed terms):
//   (r, sr) = log2| sp 2^p + sq 2^q |, with its sign.  Shifted by the larger operand, so the argument
//   of exp2 is <= 0.  p == q covers equal infinities (their difference would be NaN).
template <bool SIGNED>
__device__ __forceinline__ void slae(float p, uint32_t sp, float q, uint32_t sq, float &r, uint32_t &sr)
{
    float m = fmaxf(p, q);
    float t = p - q;
    t = (p == q) ? 0.0f : t;
    float e = exp2_hw(-fabsf(t));
    if (SIGNED) {
        e = u2f(f2u(e) ^ ((sp ^ sq) & kSignBit));
        sr = (t >= 0.0f) ? sp : sq;
    } else {
        sr = 0;
    }
    r = m + log2_hw(1.0f + e);
}

// One segment summary.
struct Seg {
    float A, M;
    uint32_t sA, sM; // sign words
};

template <int DOM>
__device__ __forceinline__ Seg seg_identity()
{
    return DOM == kLinear ? Seg{1.0f, 0.0f, 0u, 0u} : Seg{0.0f, -INFINITY, 0u, 0u};
}

template <int DOM>
__device__ __forceinline__ Seg seg_combine(const Seg &g1, const Seg &g2)
{
    constexpr bool SIGNED = DOM == kSigned;
    Seg r;
    if (DOM == kLinear) {
        r.A = g1.A * g2.A;
        r.M = g1.M * g2.A + g2.M;
        r.sA = r.sM = 0u;
        return r;
    }
    r.A = g1.A + g2.A;
    r.sA = SIGNED ? (g1.sA ^ g2.sA) : 0u;
    slae<SIGNED>(g1.M + g2.A, SIGNED ? (g1.sM ^ g2.sA) : 0u, g2.M, g2.sM, r.M, r.sM);
    return r;
}

// State = (log2|x|, sign); in the linear domain lx holds x itself.  Applying a segment to the state at its start gives the state at its end:
//   log2|x_e| = slae(log2|x_s| + A, M)       (Eq. (1) with x_0 := x_s, i.e. Sec. 4's cat(log x_0, .))
struct State {
    float lx;
    uint32_t s;
};

template <int DOM>
__device__ __forceinline__ State seg_apply(const State &x, const Seg &g)
{
    constexpr bool SIGNED = DOM == kSigned;
    State r;
    if (DOM == kLinear) {
        r.lx = x.lx * g.A + g.M;
        r.s = 0u;
        return r;
    }
    slae<SIGNED>(x.lx + g.A, SIGNED ? (x.s ^ g.sA) : 0u, g.M, g.sM, r.lx, r.s);
    return r;
}

// The state handed from tile to tile along a long sequence is kept in float64, so that a chain of
// thousands of links does not accumulate float32 rounding of the state itself.
struct State64 {
    double lx;
    uint32_t s;
};

// seg_apply with the state kept in float64: only the (small) correction log2(1 +- 2^-|t|) is formed in
// float32.
template <int DOM>
__device__ __forceinline__ State64 seg_apply64(const State64 &x, const Seg &g)
{
    constexpr bool SIGNED = DOM == kSigned;
    if (DOM == kLinear) return State64{x.lx * (double)g.A + (double)g.M, 0u};
    const double p = x.lx + (double)g.A;
    const double q = (double)g.M;
    const uint32_t sp = SIGNED ? (x.s ^ g.sA) : 0u;
    const double m = fmax(p, q);
    float t = (float)(p - q);
    t = (p == q) ? 0.0f : t;
    float e = exp2_hw(-fabsf(t));
    State64 r;
    r.s = 0u;
    if (SIGNED) {
        e = u2f(f2u(e) ^ ((sp ^ g.sM) & kSignBit));
        r.s = (t >= 0.0f) ? sp : g.sM;
    }
    r.lx = m + (double)log2_hw(1.0f + e);
    return r;
}

// ---- element encode / decode ---------------------------------------------------------------------

__device__ __forceinline__ float widen(float v) { return v; }
__device__ __forceinline__ float widen(uint16_t bf16_bits) { return u2f((uint32_t)bf16_bits << 16); }

// log2|v| and sign of a stored input value.  LOG_IN: v is a natural log of a positive number.
template <int DOM, bool LOG_IN>
__device__ __forceinline__ void encode(float v, float &l, uint32_t &s)
{
    constexpr bool SIGNED = DOM == kSigned;
    if (DOM == kLinear) {
        l = v;
        s = 0;
    } else if (LOG_IN) {
        l = v * kLog2e;
        s = 0;
    } else if (SIGNED) {
        l = log2_hw(fabsf(v));
        s = f2u(v);
    } else {
        l = log2_hw(v);
        s = 0;
    }
}

// Extends the running summary of a lane's steps by one encoded step (la, sa), (lb, sb).
template <int DOM>
__device__ __forceinline__ void seg_step(Seg &run, float la, uint32_t sa, float lb, uint32_t sb)
{
    constexpr bool SIGNED = DOM == kSigned;
    if (DOM == kLinear) {
        run.M = run.M * la + lb;
        run.A *= la;
        return;
    }
    const uint32_t sp = SIGNED ? (run.sM ^ sa) : 0u;
    slae<SIGNED>(run.M + la, sp, lb, sb, run.M, run.sM);
    run.A += la;
    if (SIGNED) run.sA ^= sa;
}

// ---- per-element record between the scan and the emit ------------------------------------------------
//
// After the serial scan a lane holds, for each of its elements k, the summary (A_k, M_k) of the lane's
// steps up to k.  Once the state x_s = (+-)2^lx at the lane's first step is known, the element is
//     x_k = (+-)2^(lx + A_k) + (+-)2^(M_k)                    (Eq. (3) with x_0 := x_s)
// or, for a log output, log x_k = slae(lx + A_k, M_k) (Eq. (1)).  Two floats are kept per element:
//   linear output: r0 = A_k, r1 = (+-)2^(M_k) already exponentiated with its sign in the sign bit; the
//                  sign of the 2^A factor goes to bit k of the lane's sign word `sw`;
//   log output:    r0 = A_k, r1 = M_k; on a signed domain the signs of the two terms go to bit k of
//                  `sw` and of `sm`.
// The first term is formed in the log domain so that a large local product times a small state (or
// the reverse) does not overflow or flush on the way.
template <int DOM, bool LOG_OUT>
__device__ __forceinline__ void stash(const Seg &run, int k, float &r0, float &r1, uint32_t &sw, uint32_t &sm)
{
    constexpr bool SIGNED = DOM == kSigned;
    r0 = run.A;
    if (DOM == kLinear) {
        r1 = run.M; // x_k = x_s A_k + M_k
    } else if (LOG_OUT) {
        r1 = run.M;
        if (SIGNED) {
            sw |= (run.sA >> 31) << k;
            sm |= (run.sM >> 31) << k;
        }
    } else {
        const float e = exp2_hw(run.M);
        r1 = SIGNED ? u2f(f2u(e) ^ (run.sM & kSignBit)) : e;
        if (SIGNED) sw |= (run.sA >> 31) << k;
        // Materialise the record here: left alone the optimiser sinks this work to the emit phase and
        // keeps (A_k, M_k, sign) of every element alive in separate registers until then.
        asm volatile("" : "+v"(r1));
        if (SIGNED) asm volatile("" : "+v"(sw));
    }
}

// ---- a lane's serial scan --------------------------------------------------------------------------
//
// A lane owns T consecutive steps.  lane_step takes step k's stored inputs (in av, mv) and leaves the
// element's record there (see stash); lane_close turns the running state into the summary (A, M) of the
// lane's steps, which is what the log-space composition across lanes, waves and tiles works on.
//
// Two ways to run the steps inside the lane.  Log inputs and log outputs go through the log domain step by
// step (seg_step: one signed log-add-exp per element, Sec. 4's LCSE).  Plain inputs with a plain output
// need the zero-input response Z_k = sum_t b_t prod_{t<u<=k} a_u of the lane's steps in the linear domain
// anyway (the record is (A_k, Z_k), and x_k = (+-)2^(lx + A_k) + Z_k, Eq. (3) with x_0 := the lane's start
// state): there it is formed directly by the definition, Z_k = a_k Z_{k-1} + b_k (Sec. 3), one fused
// multiply-add, while the first prefix sum A_k = sum log2|a_t| of Eq. (2) runs beside it.  Z_k has the
// range of the outputs themselves (it is x_k for a lane that starts from 0), its signs are the floats'
// own, and the element costs two transcendentals (log2|a_k|, and the exponential of the emit) instead of
// six.  The lane's summary takes one more logarithm, M = log2|Z_T|.
template <int DOM, bool LOG_IN, bool LOG_OUT>
constexpr bool lane_is_direct()
{
    return DOM != kLinear && !LOG_IN && !LOG_OUT;
}

template <int DOM, bool LOG_IN, bool LOG_OUT>
__device__ __forceinline__ void lane_step(int k, Seg &run, float &av, float &mv, uint32_t &sw, uint32_t &sm)
{
    constexpr bool SIGNED = DOM == kSigned;
    if constexpr (lane_is_direct<DOM, LOG_IN, LOG_OUT>()) {
        const float a = av, b = mv;
        const float la = log2_hw(SIGNED ? fabsf(a) : a);
        if (k == 0) {
            run.A = la;
            run.M = b; // Z_0 = b_0
            run.sA = SIGNED ? f2u(a) : 0u;
            run.sM = 0u;
        } else {
            run.M = fmaf(a, run.M, b); // Z_k = a_k Z_{k-1} + b_k
            run.A += la;
            if (SIGNED) run.sA ^= f2u(a);
        }
        av = run.A;
        mv = run.M;
        if (SIGNED) sw |= (run.sA >> 31) << k;
        // Materialise the record here: left alone the optimiser keeps the inputs of many steps alive and
        // forms the records late, which costs registers.
        asm volatile("" : "+v"(av), "+v"(mv));
        if (SIGNED) asm volatile("" : "+v"(sw));
    } else {
        float la, lb;
        uint32_t sa, sb;
        encode<DOM, LOG_IN>(av, la, sa);
        encode<DOM, LOG_IN>(mv, lb, sb);
        if (k == 0) {
            run = Seg{la, lb, sa, sb};
        } else {
            seg_step<DOM>(run, la, sa, lb, sb);
        }
        stash<DOM, LOG_OUT>(run, k, av, mv, sw, sm);
    }
}

template <int DOM, bool LOG_IN, bool LOG_OUT>
__device__ __forceinline__ void lane_close(Seg &run)
{
    if constexpr (lane_is_direct<DOM, LOG_IN, LOG_OUT>()) {
        const float z = run.M;
        run.sM = DOM == kSigned ? f2u(z) : 0u;
        run.M = log2_hw(fabsf(z));
    }
}

// Folds the sign of the lane's start state into the sign word, once per lane.
template <int DOM>
__device__ __forceinline__ uint32_t fold_state_sign(uint32_t sw, const State &x)
{
    constexpr bool SIGNED = DOM == kSigned;
    return SIGNED ? (sw ^ (uint32_t)((int32_t)x.s >> 31)) : 0u;
}

// swx = fold_state_sign(sw, x).
template <int DOM, bool LOG_OUT>
__device__ __forceinline__ float emit(const State &x, float r0, float r1, uint32_t swx, int k)
{
    constexpr bool SIGNED = DOM == kSigned;
    if (DOM == kLinear) return x.lx * r0 + r1;
    if (LOG_OUT) {
        float r;
        uint32_t sr;
        slae<false>(x.lx + r0, 0u, r1, 0u, r, sr);
        return r * kLn2;
    }
    float e = exp2_hw(x.lx + r0);
    if (SIGNED) e = u2f(f2u(e) ^ ((swx << (31 - k)) & kSignBit));
    return e + r1;
}

// Log output on a signed domain: the complex logarithm of x_k (Sec. 1, last paragraph), real part
// log|x_k|, imaginary part pi where x_k < 0 and 0 elsewhere.
constexpr float kPi = 3.14159265358979323846f;
__device__ __forceinline__ void emit_clog(const State &x, float r0, float r1, uint32_t swx, uint32_t sm, int k, float &re,
                                          float &im)
{
    float r;
    uint32_t sr;
    slae<true>(x.lx + r0, swx << (31 - k), r1, sm << (31 - k), r, sr);
    re = r * kLn2;
    im = (sr & kSignBit) ? kPi : 0.0f;
}

// ---- wave64 cross-lane scan of segment summaries (DPP row shifts + row broadcasts) -----------------

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f(float oldv, float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(oldv), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_u(uint32_t oldv, uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)oldv, (int)v, CTRL, ROW_MASK, 0xf, false);
}

// Segment held by the lane CTRL positions earlier (identity where there is none or the row is masked).
template <int CTRL, int ROW_MASK, int DOM>
__device__ __forceinline__ Seg seg_dpp(const Seg &g)
{
    constexpr bool SIGNED = DOM == kSigned;
    const Seg id = seg_identity<DOM>();
    Seg r;
    r.A = dpp_f<CTRL, ROW_MASK>(id.A, g.A);
    r.M = dpp_f<CTRL, ROW_MASK>(id.M, g.M);
    r.sA = SIGNED ? dpp_u<CTRL, ROW_MASK>(0u, g.sA) : 0u;
    r.sM = SIGNED ? dpp_u<CTRL, ROW_MASK>(0u, g.sM) : 0u;
    return r;
}

// Inclusive scan over the 64 lanes, lane order = time order (6 steps).
template <int DOM>
__device__ __forceinline__ Seg wave_inclusive_scan(Seg g)
{
    g = seg_combine<DOM>(seg_dpp<0x111, 0xf, DOM>(g), g); // row_shr:1
    g = seg_combine<DOM>(seg_dpp<0x112, 0xf, DOM>(g), g); // row_shr:2
    g = seg_combine<DOM>(seg_dpp<0x114, 0xf, DOM>(g), g); // row_shr:4
    g = seg_combine<DOM>(seg_dpp<0x118, 0xf, DOM>(g), g); // row_shr:8
    g = seg_combine<DOM>(seg_dpp<0x142, 0xa, DOM>(g), g); // row_bcast:15 into rows 1,3
    g = seg_combine<DOM>(seg_dpp<0x143, 0xc, DOM>(g), g); // row_bcast:31 into rows 2,3
    return g;
}

// Inclusive scan inside each row of 16 lanes (4 steps): lanes 15, 31, 47, 63 end up with the fold of
// their row, in lane order.
template <int DOM>
__device__ __forceinline__ Seg row16_inclusive_scan(Seg g)
{
    g = seg_combine<DOM>(seg_dpp<0x111, 0xf, DOM>(g), g);
    g = seg_combine<DOM>(seg_dpp<0x112, 0xf, DOM>(g), g);
    g = seg_combine<DOM>(seg_dpp<0x114, 0xf, DOM>(g), g);
    g = seg_combine<DOM>(seg_dpp<0x118, 0xf, DOM>(g), g);
    return g;
}

// Inclusive scan inside each half of the wave (5 steps): lanes 31 and 63 end up with the fold of lanes
// 0..31 and 32..63, in lane order.
template <int DOM>
__device__ __forceinline__ Seg half_inclusive_scan(Seg g)
{
    g = row16_inclusive_scan<DOM>(g);
    g = seg_combine<DOM>(seg_dpp<0x142, 0xa, DOM>(g), g); // row_bcast:15 into rows 1,3
    return g;
}

// Inclusive scan inside aligned groups of `group` lanes (a power of two, 1..64): the same six steps, a
// step taking effect only in lanes that have that many predecessors inside their group.
template <int DOM>
__device__ __forceinline__ Seg group_inclusive_scan(Seg g, int lane, int group)
{
    const int pos = lane & (group - 1);
    auto step = [&](const Seg &shifted, bool ok) {
        const Seg c = seg_combine<DOM>(shifted, g);
        g.A = ok ? c.A : g.A;
        g.M = ok ? c.M : g.M;
        g.sA = ok ? c.sA : g.sA;
        g.sM = ok ? c.sM : g.sM;
    };
    step(seg_dpp<0x111, 0xf, DOM>(g), pos >= 1);
    step(seg_dpp<0x112, 0xf, DOM>(g), pos >= 2);
    step(seg_dpp<0x114, 0xf, DOM>(g), pos >= 4);
    step(seg_dpp<0x118, 0xf, DOM>(g), pos >= 8);
    step(seg_dpp<0x142, 0xa, DOM>(g), group >= 32); // row_bcast:15 reaches lanes whose pos is >= 16 then
    step(seg_dpp<0x143, 0xc, DOM>(g), group >= 64); // row_bcast:31
    return g;
}

template <int DOM>
__device__ __forceinline__ Seg seg_readlane(const Seg &g, int lane)
{
    constexpr bool SIGNED = DOM == kSigned;
    Seg r;
    r.A = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(g.A), lane));
    r.M = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(g.M), lane));
    r.sA = SIGNED ? (uint32_t)__builtin_amdgcn_readlane((int)g.sA, lane) : 0u;
    r.sM = SIGNED ? (uint32_t)__builtin_amdgcn_readlane((int)g.sM, lane) : 0u;
    return r;
}

// Exclusive version of an inclusive result: lane i receives lane i-1's value, lane 0 the identity.
template <int DOM>
__device__ __forceinline__ Seg wave_shift_up(const Seg &g)
{
    return seg_dpp<0x138, 0xf, DOM>(g); // wave_shr:1
}

__device__ __forceinline__ float readlane_f(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ uint32_t readlane_u(uint32_t v, int lane)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, lane);
}

// ---- publishing carries between workgroups ------------------------------------------------------------
//
// Carries travel through global memory as 64-bit records {payload: 32 bits, tag: 32 bits} written and
// read with relaxed agent-scope atomics.  Such accesses are served at the level of the memory
// hierarchy all compute dies share (no cache write-back or invalidate is needed) and an aligned 64-bit
// access is indivisible, so a record is its own ready-flag: it is valid for a launch iff its tag
// carries that launch's epoch.  tag = epoch << 2 | two user bits (signs).  Nothing has to be ordered on
// the publishing side, nothing has to be cleared between launches (older epochs never match), and a
// consumer gets flag and payload in one round trip.

__device__ __forceinline__ void rec_put(rec_t *p, uint32_t payload, uint32_t epoch, uint32_t bits)
{
    const rec_t v = ((rec_t)((epoch << 2) | (bits & 3u)) << 32) | payload;
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ rec_t rec_get(const rec_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bool rec_ok(rec_t r, uint32_t epoch) { return ((uint32_t)(r >> 34)) == (epoch & 0x3fffffffu); }
__device__ __forceinline__ uint32_t rec_payload(rec_t r) { return (uint32_t)r; }
__device__ __forceinline__ uint32_t rec_bits(rec_t r) { return (uint32_t)(r >> 32) & 3u; }

// A float64 state travels as two records: the high and low word of the double; the sign rides in the user
// bits of the first.
__device__ __forceinline__ void state64_put(rec_t *p_hi, rec_t *p_lo, const State64 &x, uint32_t epoch, bool with_sign)
{
    const unsigned long long bits = (unsigned long long)__double_as_longlong(x.lx);
    rec_put(p_hi, (uint32_t)(bits >> 32), epoch, with_sign ? (x.s >> 31) : 0u);
    rec_put(p_lo, (uint32_t)bits, epoch, 0u);
}
__device__ __forceinline__ State64 state64_from(rec_t r_hi, rec_t r_lo, bool with_sign)
{
    State64 x;
    x.lx = __longlong_as_double((long long)(((unsigned long long)rec_payload(r_hi) << 32) | rec_payload(r_lo)));
    x.s = with_sign ? (rec_bits(r_hi) << 31) : 0u;
    return x;
}

// A segment summary is two records: {A, tag | sA, sM} and {M, tag}.
template <int DOM>
__device__ __forceinline__ void seg_put(rec_t *pa, rec_t *pm, const Seg &g, uint32_t epoch)
{
    constexpr bool SIGNED = DOM == kSigned;
    rec_put(pa, f2u(g.A), epoch, SIGNED ? ((g.sA >> 31) | ((g.sM >> 31) << 1)) : 0u);
    rec_put(pm, f2u(g.M), epoch, 0u);
}
template <int DOM>
__device__ __forceinline__ Seg seg_from(rec_t ra, rec_t rm)
{
    constexpr bool SIGNED = DOM == kSigned;
    Seg g;
    g.A = u2f(rec_payload(ra));
    g.M = u2f(rec_payload(rm));
    g.sA = SIGNED ? (rec_bits(ra) << 31) : 0u;
    g.sM = SIGNED ? (rec_bits(ra) << 30) : 0u;
    return g;
}

} // namespace hs
