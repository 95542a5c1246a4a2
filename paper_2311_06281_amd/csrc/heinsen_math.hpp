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
        e = u2f(f2u(e) ^ (sp ^ sq));
        sr = (t >= 0.0f) ? sp : sq;
    } else {
        sr = 0;
    }
    r = m + log2_hw(1.0f + e);
}

// sp 2^p + sq 2^q as a float32 number (Eq. (3): the exponential of Eq. (1), with the logarithm of the
// last addition never formed).  2^m is applied as two factors 2^(m/2) so that a sum that fits
// float32 is not lost to an intermediate overflow of its larger term.
template <bool SIGNED>
__device__ __forceinline__ float lin_sum(float p, uint32_t sp, float q, uint32_t sq)
{
    float m = fmaxf(p, q);
    float t = p - q;
    t = (p == q) ? 0.0f : t;
    float e = exp2_hw(-fabsf(t));
    uint32_t sr = 0;
    if (SIGNED) {
        e = u2f(f2u(e) ^ (sp ^ sq));
        sr = (t >= 0.0f) ? sp : sq;
    }
    float u = 1.0f + e;
    float h = exp2_hw(0.5f * m);
    float x = (u * h) * h;
    return SIGNED ? u2f(f2u(x) ^ sr) : x;
}

// One segment summary.
struct Seg {
    float A, M;
    uint32_t sA, sM; // 0 or kSignBit
};

__device__ __forceinline__ Seg seg_identity() { return Seg{0.0f, -INFINITY, 0u, 0u}; }

template <bool SIGNED>
__device__ __forceinline__ Seg seg_combine(const Seg &g1, const Seg &g2)
{
    Seg r;
    r.A = g1.A + g2.A;
    r.sA = SIGNED ? (g1.sA ^ g2.sA) : 0u;
    slae<SIGNED>(g1.M + g2.A, SIGNED ? (g1.sM ^ g2.sA) : 0u, g2.M, g2.sM, r.M, r.sM);
    return r;
}

// State = (log2|x|, sign).  Applying a segment to the state at its start gives the state at its end:
//   log2|x_e| = slae(log2|x_s| + A, M)       (Eq. (1) with x_0 := x_s, i.e. Sec. 4's cat(log x_0, .))
struct State {
    float lx;
    uint32_t s;
};

template <bool SIGNED>
__device__ __forceinline__ State seg_apply(const State &x, const Seg &g)
{
    State r;
    slae<SIGNED>(x.lx + g.A, SIGNED ? (x.s ^ g.sA) : 0u, g.M, g.sM, r.lx, r.s);
    return r;
}

// ---- element encode / decode ---------------------------------------------------------------------

__device__ __forceinline__ float widen(float v) { return v; }
__device__ __forceinline__ float widen(uint16_t bf16_bits) { return u2f((uint32_t)bf16_bits << 16); }

// log2|v| and sign of a stored input value.  LOG_IN: v is a natural log of a positive number.
template <bool SIGNED, bool LOG_IN>
__device__ __forceinline__ void encode(float v, float &l, uint32_t &s)
{
    if (LOG_IN) {
        l = v * kLog2e;
        s = 0;
    } else if (SIGNED) {
        l = log2_hw(fabsf(v));
        s = f2u(v) & kSignBit;
    } else {
        l = log2_hw(v);
        s = 0;
    }
}

// Output value of an element whose segment-from-lane-start summary is g and whose lane started from x.
template <bool SIGNED, bool LOG_OUT>
__device__ __forceinline__ float emit(const State &x, float A, uint32_t sA, float M, uint32_t sM)
{
    if (LOG_OUT) {
        float r;
        uint32_t sr;
        slae<false>(x.lx + A, 0u, M, 0u, r, sr);
        return r * kLn2;
    }
    return lin_sum<SIGNED>(x.lx + A, SIGNED ? (x.s ^ sA) : 0u, M, sM);
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
template <int CTRL, int ROW_MASK, bool SIGNED>
__device__ __forceinline__ Seg seg_dpp(const Seg &g)
{
    Seg r;
    r.A = dpp_f<CTRL, ROW_MASK>(0.0f, g.A);
    r.M = dpp_f<CTRL, ROW_MASK>(-INFINITY, g.M);
    r.sA = SIGNED ? dpp_u<CTRL, ROW_MASK>(0u, g.sA) : 0u;
    r.sM = SIGNED ? dpp_u<CTRL, ROW_MASK>(0u, g.sM) : 0u;
    return r;
}

// Inclusive scan over the 64 lanes, lane order = time order (6 steps).
template <bool SIGNED>
__device__ __forceinline__ Seg wave_inclusive_scan(Seg g)
{
    g = seg_combine<SIGNED>(seg_dpp<0x111, 0xf, SIGNED>(g), g); // row_shr:1
    g = seg_combine<SIGNED>(seg_dpp<0x112, 0xf, SIGNED>(g), g); // row_shr:2
    g = seg_combine<SIGNED>(seg_dpp<0x114, 0xf, SIGNED>(g), g); // row_shr:4
    g = seg_combine<SIGNED>(seg_dpp<0x118, 0xf, SIGNED>(g), g); // row_shr:8
    g = seg_combine<SIGNED>(seg_dpp<0x142, 0xa, SIGNED>(g), g); // row_bcast:15 into rows 1,3
    g = seg_combine<SIGNED>(seg_dpp<0x143, 0xc, SIGNED>(g), g); // row_bcast:31 into rows 2,3
    return g;
}

// Exclusive version of an inclusive result: lane i receives lane i-1's value, lane 0 the identity.
template <bool SIGNED>
__device__ __forceinline__ Seg wave_shift_up(const Seg &g)
{
    return seg_dpp<0x138, 0xf, SIGNED>(g); // wave_shr:1
}

__device__ __forceinline__ float readlane_f(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ uint32_t readlane_u(uint32_t v, int lane)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, lane);
}

} // namespace hs
