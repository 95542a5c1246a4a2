// Sequence-contiguous path: a, b, out are [rows, n] with rows = B*D; time runs along the lanes.
//
// Three kernels.
//  * rows_wave: one wave per row for rows that fit 64*ITEMS elements.  Lane i owns ITEMS consecutive
//    steps, scans them serially, the 64 lane summaries are scanned with DPP, each lane derives the
//    state at its first step and emits its elements.  No barrier, no global scratch; LDS only as the
//    wave's private staging area for coalesced global accesses.
//  * rows_packed: rows of at most 256 steps, several per wave; the wave scan is confined to the lanes
//    of a row.
//  * tiles: rows longer than that are cut into tiles of NW*64*ITEMS elements, one workgroup per
//    tile: the same lane and wave scans, wave summaries chained through LDS, tile summaries chained
//    through global memory in a two-level tree (see below); folds happen in a fixed order, so results
//    are bit-reproducible.
//
// What is computed is Sec. 4's expression applied by parts (Sec. 1, footnote on associativity); the
// arithmetic is in heinsen_math.hpp.
#include "heinsen_internal.hpp"
#include "heinsen_math.hpp"
#include "heinsen_tickets.hpp"

namespace hs {
namespace {

// ---- lane-level pieces shared by the kernels ----------------------------------------------------------

// Encodes and scans the lane's elements serially.  On return Av[k], Mv[k] and bit k of sw (and of sm)
// hold the per-element records (see stash); the summary of all ITEMS steps is returned.
template <int DOM, bool LOG_IN, bool LOG_OUT, int ITEMS>
__device__ __forceinline__ Seg lane_scan(float (&Av)[ITEMS], float (&Mv)[ITEMS], uint32_t &sw, uint32_t &sm)
{
    static_assert(ITEMS <= 32, "sign bits are kept in one word");
    sw = sm = 0u;
    Seg run;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) lane_step<DOM, LOG_IN, LOG_OUT>(k, run, Av[k], Mv[k], sw, sm);
    lane_close<DOM, LOG_IN, LOG_OUT>(run);
    return run;
}

// ---- one wave per row -------------------------------------------------------------------------------

struct RowsParams {
    const void *a;
    const void *b;
    const float *x0;
    float *out;
    int64_t rows, n;
    int x0_stride;
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// A wave moves a row between global memory and its lanes through a private LDS region so that global
// accesses are coalesced (consecutive lanes touch consecutive 16-byte vectors) while each lane ends up
// with NV consecutive vectors of the row ("blocked").  Vector c of the row lives at slot c + c/NV: one
// empty slot after every lane's NV slots keeps both access patterns free of bank conflicts.  LDS
// operations of one wave execute in order, so only the compiler has to be kept from reordering them.
__device__ __forceinline__ void wave_lds_order() { asm volatile("" ::: "memory"); __builtin_amdgcn_wave_barrier(); }

// Global (striped, coalesced) -> lanes (blocked).  Vectors at or beyond n_vec are replaced by `fill`.
template <int NV>
__device__ __forceinline__ void wave_load_blocked(const u32x4 *row, int64_t n_vec, u32x4 fill, u32x4 *lds, int lane,
                                                  u32x4 (&v)[NV])
{
    if (NV == 1) {
        v[0] = (lane < n_vec) ? __builtin_nontemporal_load(row + lane) : fill;
        return;
    }
    u32x4 t[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int c = j * 64 + lane;
        t[j] = (c < n_vec) ? __builtin_nontemporal_load(row + c) : fill; // streamed once: keep it out of the caches' way
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int c = j * 64 + lane;
        lds[c + c / NV] = t[j];
    }
    wave_lds_order();
#pragma unroll
    for (int q = 0; q < NV; ++q) v[q] = lds[lane * (NV + 1) + q];
    wave_lds_order();
}

// Lanes (blocked) -> global (striped, coalesced).
template <int NV>
__device__ __forceinline__ void wave_store_blocked(u32x4 *row, int64_t n_vec, u32x4 *lds, int lane, const u32x4 (&v)[NV])
{
#pragma unroll
    for (int q = 0; q < NV; ++q) lds[lane * (NV + 1) + q] = v[q];
    wave_lds_order();
    u32x4 t[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int c = j * 64 + lane;
        t[j] = lds[c + c / NV];
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int c = j * 64 + lane;
        if (c < n_vec) __builtin_nontemporal_store(t[j], row + c);
    }
    wave_lds_order();
}

// Lanes (blocked) -> global when a lane owns NV * PARTS consecutive vectors of the row: they are staged
// NV at a time (round `part` moves vectors part*NV .. part*NV + NV - 1 of every lane), so the region is
// the same size as for NV vectors and every store instruction still writes whole runs of NV vectors.
template <int NV, int PARTS>
__device__ __forceinline__ void wave_store_blocked_part(u32x4 *row, int64_t n_vec, u32x4 *lds, int lane, int part,
                                                        const u32x4 (&v)[NV])
{
#pragma unroll
    for (int q = 0; q < NV; ++q) lds[lane * (NV + 1) + q] = v[q];
    wave_lds_order();
    u32x4 t[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int c = j * 64 + lane;
        t[j] = lds[c + c / NV];
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int c = j * 64 + lane;
        const int gi = (c / NV) * (NV * PARTS) + part * NV + c % NV;
        if (gi < n_vec) __builtin_nontemporal_store(t[j], row + gi);
    }
    wave_lds_order();
}

// The same two moves one element at a time, for rows whose pointers or length do not allow 16-byte
// vectors: global accesses are still coalesced (consecutive lanes, consecutive elements), the region
// holds 32-bit slots, element c of the wave's span at slot c + c/ITEMS.  `left` elements of the row exist
// from the wave's first one on.
template <typename InT, int ITEMS>
__device__ __forceinline__ void wave_load_blocked_elems(const InT *row, int64_t left, float fill, uint32_t *lds, int lane,
                                                        float (&x)[ITEMS])
{
    float t[ITEMS];
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const int c = j * 64 + lane;
        t[j] = (c < left) ? widen(__builtin_nontemporal_load(row + c)) : fill;
    }
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const int c = j * 64 + lane;
        lds[c + c / ITEMS] = f2u(t[j]);
    }
    wave_lds_order();
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) x[k] = u2f(lds[lane * (ITEMS + 1) + k]);
    wave_lds_order();
}

// Lanes (blocked) -> global, one float at a time; a lane owns ITEMS * PARTS consecutive floats of the
// span and round `part` moves floats part*ITEMS .. part*ITEMS + ITEMS - 1 of every lane.
template <int ITEMS, int PARTS>
__device__ __forceinline__ void wave_store_blocked_elems(float *row, int64_t left, uint32_t *lds, int lane, int part,
                                                         const float (&x)[ITEMS])
{
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) lds[lane * (ITEMS + 1) + k] = f2u(x[k]);
    wave_lds_order();
    float t[ITEMS];
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const int c = j * 64 + lane;
        t[j] = u2f(lds[c + c / ITEMS]);
    }
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const int c = j * 64 + lane;
        const int gi = (c / ITEMS) * (ITEMS * PARTS) + part * ITEMS + c % ITEMS;
        if (gi < left) __builtin_nontemporal_store(t[j], row + gi);
    }
    wave_lds_order();
}

template <typename InT, int NVI, int ITEMS>
__device__ __forceinline__ void unpack_inputs(const u32x4 (&v)[NVI], float (&x)[ITEMS])
{
    if (sizeof(InT) == 4) {
#pragma unroll
        for (int q = 0; q < NVI; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i) x[q * 4 + i] = u2f(v[q][i]);
    } else {
#pragma unroll
        for (int q = 0; q < NVI; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[q * 8 + 2 * i] = u2f(v[q][i] << 16);
                x[q * 8 + 2 * i + 1] = u2f(v[q][i] & 0xffff0000u);
            }
    }
}


// Complex output (log output on a signed domain), vector path: emits the lane's elements and writes them,
// coalesced, through the wave's LDS region.  `orow` points at the wave's first output element, n_elems
// elements of the row are left from there (a multiple of four).  The output has twice the bytes of a real
// one and goes through the region in two rounds.
template <int ITEMS>
__device__ __forceinline__ void wave_emit_clog_blocked(float *orow, int64_t n_elems, u32x4 *lds, int lane, const State &st,
                                                       const float (&Av)[ITEMS], const float (&Mv)[ITEMS], uint32_t sw,
                                                       uint32_t sm)
{
    constexpr int NVO = ITEMS / 4;
    const uint32_t swx = fold_state_sign<true>(sw, st);
    n_elems = n_elems < 0 ? 0 : n_elems;
#pragma unroll
    for (int part = 0; part < 2; ++part) {
        u32x4 vo[NVO];
#pragma unroll
        for (int q = 0; q < NVO; ++q)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int k = part * (ITEMS / 2) + q * 2 + i;
                float re, im;
                emit_clog(st, Av[k], Mv[k], swx, sm, k, re, im);
                vo[q][2 * i] = f2u(re);
                vo[q][2 * i + 1] = f2u(im);
            }
        wave_store_blocked_part<NVO, 2>(reinterpret_cast<u32x4 *>(orow), n_elems / 2, lds, lane, part, vo);
    }
}

// Element-wise counterpart of the vector emit: `orow` points at the wave's first output element, `left`
// elements of the row exist from there on.
template <int DOM, bool LOG_OUT, int ITEMS>
__device__ __forceinline__ void wave_emit_blocked_elems(float *orow, int64_t left, uint32_t *lds, int lane, const State &st,
                                                        const float (&Av)[ITEMS], const float (&Mv)[ITEMS], uint32_t sw,
                                                        uint32_t sm)
{
    constexpr bool SIGNED = DOM == kSigned;
    const uint32_t swx = fold_state_sign<DOM>(sw, st);
    left = left < 0 ? 0 : left;
    if constexpr (SIGNED && LOG_OUT) {
#pragma unroll
        for (int part = 0; part < 2; ++part) {
            float o[ITEMS];
#pragma unroll
            for (int i = 0; i < ITEMS / 2; ++i) {
                const int k = part * (ITEMS / 2) + i;
                emit_clog(st, Av[k], Mv[k], swx, sm, k, o[2 * i], o[2 * i + 1]);
            }
            wave_store_blocked_elems<ITEMS, 2>(orow, 2 * left, lds, lane, part, o);
        }
    } else {
        float o[ITEMS];
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) o[k] = emit<DOM, LOG_OUT>(st, Av[k], Mv[k], swx, k);
        wave_store_blocked_elems<ITEMS, 1>(orow, left, lds, lane, 0, o);
    }
}

template <int DOM, bool LOG_IN, bool LOG_OUT, typename InT, int ITEMS, bool VECIO>
__global__ __launch_bounds__(256, VECIO ? 4 : 1) void heinsen_scan_rows_wave(RowsParams p)
{
    constexpr bool SIGNED = DOM == kSigned;
    // 16-byte slots per wave: the output row (ITEMS/4 vectors per lane, the larger of the two) plus padding.
    // (Writing the output in two rounds through half the region, for twice the workgroups per CU, was
    // measured on bf16 rows of 2048: 908 us against 713 -- the rounds write 64-byte pieces.)
    __shared__ u32x4 stage[4][64 * (ITEMS / 4 + 1)];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row = (int64_t)blockIdx.x * 4 + w;
    if (row >= p.rows) return; // whole wave leaves together
    const InT *arow = reinterpret_cast<const InT *>(p.a) + row * p.n;
    const InT *brow = reinterpret_cast<const InT *>(p.b) + row * p.n;
    constexpr int OW = (SIGNED && LOG_OUT) ? 2 : 1; // floats per output element
    float *orow = p.out + OW * row * p.n;

    float Av[ITEMS], Mv[ITEMS];
    uint32_t sw, sm;
    if (VECIO) {
        constexpr int VL = 16 / (int)sizeof(InT);
        constexpr int NVI = ITEMS / VL;
        static_assert(ITEMS % VL == 0 && NVI >= 1 && NVI <= 8, "lane chunk must be 1..8 vectors");
        // a = 1, b = 0 (log domain: 0, -inf) for the steps past the end of the row
        const uint32_t one = sizeof(InT) == 4 ? 0x3f800000u : 0x3f803f80u;
        const uint32_t ninf = sizeof(InT) == 4 ? 0xff800000u : 0xff80ff80u;
        const uint32_t fa = LOG_IN ? 0u : one, fb = LOG_IN ? ninf : 0u;
        const int64_t n_vec = p.n / VL;
        u32x4 va[NVI], vb[NVI];
        wave_load_blocked<NVI>(reinterpret_cast<const u32x4 *>(arow), n_vec, u32x4{fa, fa, fa, fa}, stage[w], lane, va);
        wave_load_blocked<NVI>(reinterpret_cast<const u32x4 *>(brow), n_vec, u32x4{fb, fb, fb, fb}, stage[w], lane, vb);
        unpack_inputs<InT, NVI, ITEMS>(va, Av);
        unpack_inputs<InT, NVI, ITEMS>(vb, Mv);
    } else {
        uint32_t *slots = reinterpret_cast<uint32_t *>(stage[w]);
        wave_load_blocked_elems<InT, ITEMS>(arow, p.n, LOG_IN ? 0.0f : 1.0f, slots, lane, Av);
        wave_load_blocked_elems<InT, ITEMS>(brow, p.n, LOG_IN ? -INFINITY : 0.0f, slots, lane, Mv);
    }
    Seg mine = lane_scan<DOM, LOG_IN, LOG_OUT, ITEMS>(Av, Mv, sw, sm);
    Seg excl = wave_shift_up<DOM>(wave_inclusive_scan<DOM>(mine));

    State st;
    encode<DOM, LOG_IN>(p.x0[p.x0_stride ? row : 0], st.lx, st.s);
    st = seg_apply<DOM>(st, excl);
    if constexpr (VECIO && SIGNED && LOG_OUT) {
        wave_emit_clog_blocked<ITEMS>(orow, p.n, stage[w], lane, st, Av, Mv, sw, sm);
    } else if (VECIO) {
        constexpr int NVO = ITEMS / 4;
        const uint32_t swx = fold_state_sign<DOM>(sw, st);
        u32x4 vo[NVO];
#pragma unroll
        for (int q = 0; q < NVO; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                vo[q][i] = f2u(emit<DOM, LOG_OUT>(st, Av[q * 4 + i], Mv[q * 4 + i], swx, q * 4 + i));
        wave_store_blocked<NVO>(reinterpret_cast<u32x4 *>(orow), p.n / 4, stage[w], lane, vo);
    } else {
        wave_emit_blocked_elems<DOM, LOG_OUT, ITEMS>(orow, p.n, reinterpret_cast<uint32_t *>(stage[w]), lane, st, Av, Mv, sw, sm);
    }
}

// ---- several short rows per wave ---------------------------------------------------------------------
//
// Rows of at most 256 steps would leave most lanes of a wave idle.  Here a row takes `group` lanes
// (a power of two, 8 steps per lane) and a wave takes 64 / group consecutive rows; the wave scan is
// confined to the groups.  When the rows fill their lanes exactly (n = 8 * group) the wave's rows are
// one contiguous span of 512 elements and move through LDS like a single long row (VECIO); otherwise
// the span is still read and written coalesced, one element at a time, and sorted into the lanes' slots.
struct PackedParams {
    const void *a;
    const void *b;
    const float *x0;
    float *out;
    int64_t rows, n;
    int x0_stride;
    int group; // lanes per row
};

template <int DOM, bool LOG_IN, bool LOG_OUT, typename InT, bool VECIO>
__global__ __launch_bounds__(256, 4) void heinsen_scan_rows_packed(PackedParams p)
{
    constexpr bool SIGNED = DOM == kSigned;
    constexpr int ITEMS = 8;
    constexpr int OW = (SIGNED && LOG_OUT) ? 2 : 1; // floats per output element
    __shared__ u32x4 stage[4][64 * (ITEMS / 4 + 1)];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rows_per_wave = 64 / p.group;
    const int64_t row0 = ((int64_t)blockIdx.x * 4 + w) * rows_per_wave; // first row of this wave
    if (row0 >= p.rows) return; // whole wave leaves together
    const int64_t row = row0 + lane / p.group; // this lane's row (may be past the last one)
    const bool row_ok = row < p.rows;
    const int64_t start = (int64_t)(lane & (p.group - 1)) * ITEMS; // this lane's first step inside its row

    float Av[ITEMS], Mv[ITEMS];
    uint32_t sw, sm;
    // elements of the wave's span that exist (VECIO: the rows are contiguous and fill their lanes)
    const int64_t span = ((p.rows - row0 < rows_per_wave) ? (p.rows - row0) : rows_per_wave) * p.n;
    // slot of element c of the span when rows do not fill their lanes; c / n through a reciprocal: c + 1/2
    // over n is at least 1/(2n) >= 1/512 away from every integer, far more than the rounding of the product
    const float inv_n = 1.0f / (float)p.n;
    auto span_slot = [&](int c) -> int {
        const int r = (int)(((float)c + 0.5f) * inv_n);
        const int s_ = c - r * (int)p.n;
        return (r * p.group + (s_ >> 3)) * (ITEMS + 1) + (s_ & 7);
    };
    if (VECIO) {
        constexpr int VL = 16 / (int)sizeof(InT);
        constexpr int NVI = ITEMS / VL;
        const uint32_t one = sizeof(InT) == 4 ? 0x3f800000u : 0x3f803f80u;
        const uint32_t ninf = sizeof(InT) == 4 ? 0xff800000u : 0xff80ff80u;
        const uint32_t fa = LOG_IN ? 0u : one, fb = LOG_IN ? ninf : 0u;
        u32x4 va[NVI], vb[NVI];
        wave_load_blocked<NVI>(reinterpret_cast<const u32x4 *>(reinterpret_cast<const InT *>(p.a) + row0 * p.n), span / VL,
                               u32x4{fa, fa, fa, fa}, stage[w], lane, va);
        wave_load_blocked<NVI>(reinterpret_cast<const u32x4 *>(reinterpret_cast<const InT *>(p.b) + row0 * p.n), span / VL,
                               u32x4{fb, fb, fb, fb}, stage[w], lane, vb);
        unpack_inputs<InT, NVI, ITEMS>(va, Av);
        unpack_inputs<InT, NVI, ITEMS>(vb, Mv);
    } else {
        // The wave's rows are still one contiguous span of memory, but a row does not fill its lanes: read
        // the span coalesced, one element per lane and round, and drop element c = (row r, step s) into
        // the slot of the lane that owns it, (r * group + s / 8) * 9 + s % 8.
        uint32_t *slots = reinterpret_cast<uint32_t *>(stage[w]);
        auto gather = [&](const InT *src, float fill, float (&x)[ITEMS]) {
            float t[ITEMS];
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                const int c = j * 64 + lane;
                t[j] = (c < span) ? widen(__builtin_nontemporal_load(src + c)) : fill;
            }
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                const int c = j * 64 + lane;
                if (c < span) slots[span_slot(c)] = f2u(t[j]);
            }
            wave_lds_order();
#pragma unroll
            for (int k = 0; k < ITEMS; ++k) x[k] = (row_ok && start + k < p.n) ? u2f(slots[lane * (ITEMS + 1) + k]) : fill;
            wave_lds_order();
        };
        gather(reinterpret_cast<const InT *>(p.a) + row0 * p.n, LOG_IN ? 0.0f : 1.0f, Av);
        gather(reinterpret_cast<const InT *>(p.b) + row0 * p.n, LOG_IN ? -INFINITY : 0.0f, Mv);
    }
    Seg mine = lane_scan<DOM, LOG_IN, LOG_OUT, ITEMS>(Av, Mv, sw, sm);
    const Seg incl = group_inclusive_scan<DOM>(mine, lane, p.group);
    Seg excl = wave_shift_up<DOM>(incl);
    if ((lane & (p.group - 1)) == 0) excl = seg_identity<DOM>(); // first lane of a row

    State st;
    encode<DOM, LOG_IN>(p.x0[(p.x0_stride && row_ok) ? row : 0], st.lx, st.s);
    st = seg_apply<DOM>(st, excl);
    if constexpr (VECIO && SIGNED && LOG_OUT) {
        wave_emit_clog_blocked<ITEMS>(p.out + OW * row0 * p.n, span, stage[w], lane, st, Av, Mv, sw, sm);
    } else if (VECIO) {
        constexpr int NVO = ITEMS / 4;
        const uint32_t swx = fold_state_sign<DOM>(sw, st);
        u32x4 vo[NVO];
#pragma unroll
        for (int q = 0; q < NVO; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                vo[q][i] = f2u(emit<DOM, LOG_OUT>(st, Av[q * 4 + i], Mv[q * 4 + i], swx, q * 4 + i));
        wave_store_blocked<NVO>(reinterpret_cast<u32x4 *>(p.out + row0 * p.n), span / 4, stage[w], lane, vo);
    } else {
        // the reverse move: lanes drop their results into their slots, the span is written coalesced
        // (a complex output in two rounds, real parts then imaginary parts)
        uint32_t *slots = reinterpret_cast<uint32_t *>(stage[w]);
        const uint32_t swx = fold_state_sign<DOM>(sw, st);
        float *dst = p.out + OW * row0 * p.n;
#pragma unroll
        for (int part = 0; part < OW; ++part) {
#pragma unroll
            for (int k2 = 0; k2 < ITEMS; ++k2) {
                float o;
                if constexpr (SIGNED && LOG_OUT) {
                    float re, im;
                    emit_clog(st, Av[k2], Mv[k2], swx, sm, k2, re, im);
                    o = part == 0 ? re : im;
                } else {
                    o = emit<DOM, LOG_OUT>(st, Av[k2], Mv[k2], swx, k2);
                }
                slots[lane * (ITEMS + 1) + k2] = f2u(o);
            }
            wave_lds_order();
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                const int c = j * 64 + lane;
                if (c < span) __builtin_nontemporal_store(u2f(slots[span_slot(c)]), dst + OW * c + part);
            }
            wave_lds_order();
        }
    }
}

// ---- tiles with a chained carry ------------------------------------------------------------------------
//
// Tile index c inside a row is read in base 32: c = (s*32 + g)*32 + r.  Summaries are published at two
// levels -- a tile's own (level 1) and the 32 tiles of a group folded by its last tile (level 2) -- and
// the state at the start of every 1024-tile super-block s, in float64, by the last tile of the previous
// one.  A tile therefore reads at most 31 + 31 summaries and one state, all in one round of loads (one
// per lane of wave 0), and folds them in a fixed order: results do not depend on timing.  A level-2
// summary is published as soon as the level-1 summaries it is made of are in, so no tile waits for
// another tile's wait; only the super-block states form a chain, n / (1024 * tile) links long.

// records per summary slot: the two records of a summary (or state) get a 128-byte line of their own, so
// that the tiles polling for one summary do not queue with the accesses to its neighbours
constexpr uint32_t kRecStride = 16;
constexpr int kTileWaves = 8;   // waves per workgroup (4 and 16 measured 12 % and 28 % slower on one row of 2^26)
constexpr int kTileItems = 32;  // elements per lane (rows of one tile may use 8 or 16: a shorter serial chain)
constexpr int kTile = kTileWaves * 64 * kTileItems;
// A launch of few tiles is bound by the latency of a tile, not by memory: up to this many tiles it takes
// tiles of half the size (16 elements per lane).  Measured on one row: 6.0 against 7.4 us for 2^16 steps,
// 9.5 against 10.1 us for 2^20 (128 half tiles), even at 2^21, slower beyond.
constexpr int64_t kHalfTilesUpTo = 128;

struct TileParams {
    const void *a;
    const void *b;
    const float *x0;
    float *out;
    int64_t rows, n;
    int x0_stride;
    uint32_t tpr;          // tiles per row
    uint32_t ntiles;       // rows * tpr
    rec_t *header;         // scratch header (ticket queue 0 hands out the tiles in row-major order)
    rec_t *recs;           // per row: level-1 and level-2 summaries (2 records each), states (2 records each)
    uint32_t off2, off4, row_stride; // record offsets of level 2 and of the states inside a row's block
    uint32_t spin_limit;
    uint32_t drop_tile;
    Timeline tl;
};

template <int DOM, bool LOG_IN, bool LOG_OUT, typename InT, bool VECIO, bool MULTI, int ITEMS>
__device__ __forceinline__ void tiles_tile(const TileParams &p, const uint32_t tile, const uint32_t epoch)
{
    constexpr bool SIGNED = DOM == kSigned;
    constexpr int NW = kTileWaves;
    constexpr int kTile = NW * 64 * ITEMS; // elements per tile
    static_assert(!MULTI || ITEMS == kTileItems || ITEMS == kTileItems / 2, "rows of several tiles use the full or the half tile");
    __shared__ float lds_A[NW], lds_M[NW];
    __shared__ uint32_t lds_S[NW];
    __shared__ float lds_startL;
    __shared__ uint32_t lds_startS;

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    const int64_t row = tile / p.tpr;
    const uint32_t c = tile % p.tpr;
    const InT *arow = reinterpret_cast<const InT *>(p.a) + row * p.n;
    const InT *brow = reinterpret_cast<const InT *>(p.b) + row * p.n;

    // ---- wave 0 asks for the carry records it needs before the tile's own loads (see scan_bnd.hip) ---
    const uint32_t r = c & 31u, g = (c >> 5) & 31u, sb = c >> 10;
    const bool more = c + 1 < p.tpr;
    rec_t *const rrow = p.recs + (size_t)row * p.row_stride;
    rec_t ra = 0, rm = 0;
    const rec_t *fp = nullptr;
    bool need = false;
    if (MULTI && w == 0) {
        // lanes 0-30: level 2 (earlier groups of the super-block), lane 31: the super-block state,
        // lanes 32-62: level 1 (earlier tiles of the group)
        const uint32_t sub = (uint32_t)lane & 31u;
        if (lane < 31 && sub < g) { need = true; fp = rrow + p.off2 + kRecStride * (size_t)(((c >> 10) << 5) + sub); }
        if (lane == 31 && sb > 0) { need = true; fp = rrow + p.off4 + kRecStride * (size_t)sb; }
        if (lane >= 32 && lane < 63 && sub < r) { need = true; fp = rrow + kRecStride * (size_t)(((c >> 5) << 5) + sub); }
    }
    bool got = !need; // this lane's records are in
    auto fetch_records = [&]() -> uint64_t {
        if (!got) {
            ra = rec_get(fp);
            rm = rec_get(fp + 1);
            got = rec_ok(ra, epoch) && rec_ok(rm, epoch);
        }
        return __builtin_amdgcn_ballot_w64(got);
    };
    uint64_t have = 0;
    if (MULTI && w == 0) have = fetch_records();

    // global <-> lane traffic of each wave goes through its own LDS region (coalesced both ways); the pad
    // slot after the last lane is never used, and leaving it out lets four workgroups share a CU
    __shared__ u32x4 stage[NW][64 * (ITEMS / 4 + 1) - (VECIO ? 1 : 0)];
    const int64_t wstart = (int64_t)c * kTile + (int64_t)w * (64 * ITEMS); // first element of this wave
    float Av[ITEMS], Mv[ITEMS];
    uint32_t sw, sm;
    if (VECIO) {
        constexpr int VL = 16 / (int)sizeof(InT);
        constexpr int NVI = ITEMS / VL;
        const uint32_t one = sizeof(InT) == 4 ? 0x3f800000u : 0x3f803f80u;
        const uint32_t ninf = sizeof(InT) == 4 ? 0xff800000u : 0xff80ff80u;
        const uint32_t fa = LOG_IN ? 0u : one, fb = LOG_IN ? ninf : 0u;
        int64_t n_vec = (p.n - wstart) / VL; // vectors of the row left from this wave's first element
        n_vec = n_vec < 0 ? 0 : n_vec;
        u32x4 va[NVI], vb[NVI];
        wave_load_blocked<NVI>(reinterpret_cast<const u32x4 *>(arow + wstart), n_vec, u32x4{fa, fa, fa, fa}, stage[w], lane, va);
        wave_load_blocked<NVI>(reinterpret_cast<const u32x4 *>(brow + wstart), n_vec, u32x4{fb, fb, fb, fb}, stage[w], lane, vb);
        unpack_inputs<InT, NVI, ITEMS>(va, Av);
        unpack_inputs<InT, NVI, ITEMS>(vb, Mv);
    } else {
        uint32_t *slots = reinterpret_cast<uint32_t *>(stage[w]);
        wave_load_blocked_elems<InT, ITEMS>(arow + wstart, p.n - wstart, LOG_IN ? 0.0f : 1.0f, slots, lane, Av);
        wave_load_blocked_elems<InT, ITEMS>(brow + wstart, p.n - wstart, LOG_IN ? -INFINITY : 0.0f, slots, lane, Mv);
    }
    Seg mine = lane_scan<DOM, LOG_IN, LOG_OUT, ITEMS>(Av, Mv, sw, sm);
    Seg incl = wave_inclusive_scan<DOM>(mine);
    Seg lane_excl = wave_shift_up<DOM>(incl);
    p.tl.mark(tile, 2);
    if (lane == 63) {
        lds_A[w] = incl.A;
        lds_M[w] = incl.M;
        lds_S[w] = (incl.sA >> 31) | ((incl.sM >> 31) << 1);
    }
    __syncthreads();

    // summary of the waves before this one, and (wave 0) of the whole tile, in wave order
    Seg wave_excl = seg_identity<DOM>();
    Seg total = seg_identity<DOM>();
#pragma unroll
    for (int j = 0; j < NW; ++j) {
        Seg h;
        h.A = lds_A[j];
        h.M = lds_M[j];
        h.sA = SIGNED ? (lds_S[j] << 31) : 0u;
        h.sM = SIGNED ? (lds_S[j] << 30) : 0u;
        total = (j == 0) ? h : seg_combine<DOM>(total, h);
        if (j + 1 == w) wave_excl = total;
    }

    if (w == 0) {
        State64 st;
        {
            float lx;
            encode<DOM, LOG_IN>(p.x0[p.x0_stride ? row : 0], lx, st.s);
            st.lx = (double)lx;
        }
        p.tl.mark(tile, 3);
        if (MULTI) {
            if (more && r < 31u && lane == 0 && tile != p.drop_tile)
                seg_put<DOM>(rrow + kRecStride * (size_t)c, rrow + kRecStride * (size_t)c + 1, total, epoch);
            // The last tile of a group owes the later groups the summary of its group; it needs level 1
            // only and is published as soon as that is in, whatever else is still on its way.
            const bool lead = more && r == 31u;
            bool pub2 = !lead;
            Seg f1 = seg_identity<DOM>(), f2 = seg_identity<DOM>(), a2 = seg_identity<DOM>();
            const uint64_t m1 = 0x7fffffff00000000ull, all = ~0ull;
            bool lost = false; // some record never came
            uint32_t polls = 0;
            for (;;) {
                if (!lost && have != all && ++polls > p.spin_limit) {
                    // give up: go on as if everything were in, with NaN as the state, which is also handed on
                    lost = true;
                    have = all;
                    if (lane == 0) note_wait_gave_up(p.header);
                }
                if ((!pub2 && (have & m1) == m1) || have == all) {
                    Seg part = (need && got && lane != 31) ? seg_from<DOM>(ra, rm) : seg_identity<DOM>();
                    if (lost) part.M = __builtin_nanf("");
                    part = half_inclusive_scan<DOM>(part);
                    f2 = seg_readlane<DOM>(part, 31);
                    f1 = seg_readlane<DOM>(part, 63);
                    if (!pub2) {
                        a2 = seg_combine<DOM>(f1, total); // this group of 32 tiles
                        if (g < 31u && lane == 0)
                            seg_put<DOM>(rrow + p.off2 + kRecStride * (size_t)(c >> 5), rrow + p.off2 + kRecStride * (size_t)(c >> 5) + 1, a2, epoch);
                        pub2 = true;
                    }
                }
                if (have == all) break;
                __builtin_amdgcn_s_sleep(2);
                have = fetch_records();
            }
            p.tl.mark(tile, 4);
            if (sb > 0) {
                // lane 31 holds the super-block state: payloads are the high and low word of the double,
                // the sign rides in the user bits of the first record
                const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)rec_payload(ra), 31);
                const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)rec_payload(rm), 31);
                const uint32_t sg = (uint32_t)__builtin_amdgcn_readlane((int)rec_bits(ra), 31);
                st.lx = __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
                st.s = SIGNED ? (sg << 31) : 0u;
            }
            if (lost) st.lx = __builtin_nan("");
            const State64 st2 = seg_apply64<DOM>(st, f2); // state at the start of the group
            if (lead && g == 31u) {
                const State64 nx = seg_apply64<DOM>(st2, a2); // start of the next super-block
                const unsigned long long bits = (unsigned long long)__double_as_longlong(nx.lx);
                if (lane == 0) {
                    rec_put(rrow + p.off4 + kRecStride * (size_t)(sb + 1), (uint32_t)(bits >> 32), epoch, SIGNED ? (nx.s >> 31) : 0u);
                    rec_put(rrow + p.off4 + kRecStride * (size_t)(sb + 1) + 1, (uint32_t)bits, epoch, 0u);
                }
            }
            st = seg_apply64<DOM>(st2, f1);
        }
        if (lane == 0) {
            lds_startL = (float)st.lx;
            lds_startS = st.s;
        }
    }
    __syncthreads();

    p.tl.mark(tile, 5);
    State st;
    st.lx = lds_startL;
    st.s = lds_startS;
    st = seg_apply<DOM>(st, seg_combine<DOM>(wave_excl, lane_excl));
    constexpr int OW = (SIGNED && LOG_OUT) ? 2 : 1; // floats per output element
    float *orow = p.out + OW * row * p.n;
    if constexpr (VECIO && SIGNED && LOG_OUT) {
        wave_emit_clog_blocked<ITEMS>(orow + OW * wstart, p.n - wstart, stage[w], lane, st, Av, Mv, sw, sm);
    } else if (VECIO) {
        constexpr int NVO = ITEMS / 4;
        const uint32_t swx = fold_state_sign<DOM>(sw, st);
        u32x4 vo[NVO];
#pragma unroll
        for (int qv = 0; qv < NVO; ++qv)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                vo[qv][i] = f2u(emit<DOM, LOG_OUT>(st, Av[qv * 4 + i], Mv[qv * 4 + i], swx, qv * 4 + i));
        int64_t n_vec = (p.n - wstart) / 4;
        n_vec = n_vec < 0 ? 0 : n_vec;
        wave_store_blocked<NVO>(reinterpret_cast<u32x4 *>(orow + wstart), n_vec, stage[w], lane, vo);
    } else {
        wave_emit_blocked_elems<DOM, LOG_OUT, ITEMS>(orow + OW * wstart, p.n - wstart, reinterpret_cast<uint32_t *>(stage[w]), lane,
                                                     st, Av, Mv, sw, sm);
    }
    p.tl.mark(tile, 6);
}

template <int DOM, bool LOG_IN, bool LOG_OUT, typename InT, bool VECIO, bool MULTI, int ITEMS>
__global__ __launch_bounds__(kTileWaves * 64) void heinsen_scan_tiles(TileParams p)
{
    __shared__ uint32_t s_tile, s_epoch, s_flag;
    const unsigned long long t_begin = p.tl.stamps != nullptr ? wall_clock64() : 0ull;
    uint32_t tile = blockIdx.x, epoch = 0u;
    if (MULTI) {
        // tickets: a tile only ever waits for tiles with smaller tickets, which are already running
        if (threadIdx.x == 0) {
            const Draw d = draw_ticket(p.header, 0, p.ntiles, 1);
            s_tile = d.ticket;
            s_epoch = d.epoch;
        }
        __syncthreads();
        tile = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_tile);
        epoch = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_epoch);
    }
    if (tile < p.ntiles) {
        p.tl.mark_at(tile, 0, t_begin);
        p.tl.mark(tile, 1);
        tiles_tile<DOM, LOG_IN, LOG_OUT, InT, VECIO, MULTI, ITEMS>(p, tile, epoch);
        p.tl.mark(tile, 7);
    }
    if (MULTI) end_of_workgroup(p.header, epoch, &s_flag);
}

// ---- host side -------------------------------------------------------------------------------------------

constexpr int64_t kRowsWaveMax = 64 * 32; // longest row the one-wave kernel takes

struct BdnPlan {
    bool wave_kernel;
    int group;    // > 0: several rows per wave, this many lanes per row
    int items;    // wave kernel: elements per lane
    bool vecio;
    bool multi;
    int tile_items; // tiles kernel: elements per lane
    int64_t rows;
    uint32_t tpr, ntiles;
    uint32_t off2, off4, row_stride;
    size_t records;
};

BdnPlan make_plan(const ScanCall &c)
{
    BdnPlan pl = {};
    pl.rows = c.B * c.D;
    const int64_t vl = c.bf16 ? 8 : 4;
    auto aligned16 = [](const void *ptr) { return (reinterpret_cast<uintptr_t>(ptr) % 16) == 0; };
    pl.vecio = aligned16(c.a) && aligned16(c.b) && aligned16(c.out) && (c.n % vl == 0);
    pl.wave_kernel = c.n <= kRowsWaveMax && !(pl.rows < 64 && c.n > 512);
    if (pl.wave_kernel) {
        pl.items = c.n > 1024 ? 32 : (c.n > 512 ? 16 : 8);
        if (c.n <= 256 && pl.rows > 1) {
            // at least two rows fit the 64 lanes x 8 steps of a wave
            pl.group = 1;
            while (pl.group * 8 < c.n) pl.group *= 2;
            // the vector path needs the rows to fill their lanes: then a wave's rows are one contiguous span
            pl.vecio = pl.vecio && c.n == (int64_t)pl.group * 8;
        }
        return pl;
    }
    // a row of one tile is bound by latency: spread it over all waves of the workgroup
    pl.tile_items = c.n <= kTileWaves * 64 * 8 ? 8 : (c.n <= kTileWaves * 64 * 16 ? 16 : kTileItems);
    if (c.n > kTile && pl.rows * ceil_div(c.n, kTile / 2) <= kHalfTilesUpTo) pl.tile_items = kTileItems / 2;
    pl.tpr = (uint32_t)ceil_div(c.n, (int64_t)kTileWaves * 64 * pl.tile_items);
    pl.ntiles = (uint32_t)(pl.rows * pl.tpr);
    pl.multi = pl.tpr > 1;
    if (!pl.multi) return pl;
    const uint32_t n1 = pl.tpr, n2 = (pl.tpr + 31) / 32, n4 = (pl.tpr + 1023) / 1024 + 1;
    pl.off2 = kRecStride * n1;
    pl.off4 = pl.off2 + kRecStride * n2;
    pl.row_stride = pl.off4 + kRecStride * n4;
    pl.records = (size_t)pl.rows * pl.row_stride;
    return pl;
}

template <int DOM, bool LOG_IN, bool LOG_OUT, typename InT>
hipError_t launch_mode(const ScanCall &c, const BdnPlan &pl, const LaunchCtx &ctx)
{
    if (pl.wave_kernel && pl.group > 0) {
        PackedParams p;
        p.a = c.a;
        p.b = c.b;
        p.x0 = c.x0;
        p.out = c.out;
        p.rows = pl.rows;
        p.n = c.n;
        p.x0_stride = c.x0_scalar ? 0 : 1;
        p.group = pl.group;
        const int64_t waves = ceil_div(pl.rows, 64 / pl.group);
        dim3 grid((unsigned)ceil_div(waves, 4)), block(256);
        if (pl.vecio)
            hipLaunchKernelGGL((heinsen_scan_rows_packed<DOM, LOG_IN, LOG_OUT, InT, true>), grid, block, 0, c.stream, p);
        else
            hipLaunchKernelGGL((heinsen_scan_rows_packed<DOM, LOG_IN, LOG_OUT, InT, false>), grid, block, 0, c.stream, p);
        return hipGetLastError();
    }
    if (pl.wave_kernel) {
        RowsParams p;
        p.a = c.a;
        p.b = c.b;
        p.x0 = c.x0;
        p.out = c.out;
        p.rows = pl.rows;
        p.n = c.n;
        p.x0_stride = c.x0_scalar ? 0 : 1;
        dim3 grid((unsigned)ceil_div(pl.rows, 4)), block(256);
#define HS_ROWS(ITEMS_, VEC_)                                                                            \
    hipLaunchKernelGGL((heinsen_scan_rows_wave<DOM, LOG_IN, LOG_OUT, InT, ITEMS_, VEC_>), grid, block, 0, \
                       c.stream, p)
        if (pl.vecio) {
            if (pl.items == 32) HS_ROWS(32, true);
            else if (pl.items == 16) HS_ROWS(16, true);
            else HS_ROWS(8, true);
        } else {
            if (pl.items == 32) HS_ROWS(32, false);
            else if (pl.items == 16) HS_ROWS(16, false);
            else HS_ROWS(8, false);
        }
#undef HS_ROWS
        return hipGetLastError();
    }
    TileParams p;
    p.a = c.a;
    p.b = c.b;
    p.x0 = c.x0;
    p.out = c.out;
    p.rows = pl.rows;
    p.n = c.n;
    p.x0_stride = c.x0_scalar ? 0 : 1;
    p.tpr = pl.tpr;
    p.ntiles = pl.ntiles;
    rec_t *records = pl.multi ? ctx.scratch : nullptr;
    if (pl.multi && records == nullptr) return hipErrorInvalidValue;
    p.header = records;
    p.recs = records ? records + kRecordBase : nullptr;
    p.spin_limit = ctx.spin_limit;
    p.drop_tile = ctx.drop_tile;
    p.tl.stamps = ctx.timeline;
    p.tl.tiles = ctx.timeline_tiles;
    p.off2 = pl.off2;
    p.off4 = pl.off4;
    p.row_stride = pl.row_stride;
    dim3 grid(pl.ntiles), block(kTileWaves * 64);
#define HS_TILES(VEC_, MULTI_, ITEMS_) \
    hipLaunchKernelGGL((heinsen_scan_tiles<DOM, LOG_IN, LOG_OUT, InT, VEC_, MULTI_, ITEMS_>), grid, block, 0, c.stream, p)
    if (pl.multi && pl.tile_items == kTileItems / 2) {
        if (pl.vecio) HS_TILES(true, true, kTileItems / 2);
        else HS_TILES(false, true, kTileItems / 2);
    } else if (pl.multi) {
        if (pl.vecio) HS_TILES(true, true, kTileItems);
        else HS_TILES(false, true, kTileItems);
    } else if (pl.tile_items == 8) {
        if (pl.vecio) HS_TILES(true, false, 8);
        else HS_TILES(false, false, 8);
    } else if (pl.tile_items == 16) {
        if (pl.vecio) HS_TILES(true, false, 16);
        else HS_TILES(false, false, 16);
    } else {
        if (pl.vecio) HS_TILES(true, false, kTileItems);
        else HS_TILES(false, false, kTileItems);
    }
#undef HS_TILES
    return hipGetLastError();
}

hipError_t launch_dispatch(const ScanCall &c, const BdnPlan &pl, const LaunchCtx &ctx)
{
    HS_DISPATCH_MODE(c, launch_mode, c, pl, ctx);
}

} // namespace

ScratchNeed bdn_scratch(const ScanCall &c)
{
    BdnPlan pl = make_plan(c);
    return ScratchNeed{pl.records};
}

hipError_t bdn_launch(const ScanCall &c, const LaunchCtx &ctx)
{
    BdnPlan pl = make_plan(c);
    return launch_dispatch(c, pl, ctx);
}


const char *bdn_kernel_name(const ScanCall &c)
{
    const BdnPlan pl = make_plan(c);
    if (pl.wave_kernel) return pl.group > 0 ? "heinsen_scan_rows_packed" : "heinsen_scan_rows_wave";
    return "heinsen_scan_tiles";
}

void bdn_tile_shape(const ScanCall &c, int &rows, int64_t &steps)
{
    const BdnPlan pl = make_plan(c);
    if (pl.wave_kernel) {
        // one wave per row, or 64 / group rows per wave; workgroups of four waves
        rows = pl.group > 0 ? 4 * (64 / pl.group) : 4;
        steps = c.n;
    } else {
        rows = 1;
        steps = (int64_t)kTileWaves * 64 * pl.tile_items;
    }
}

} // namespace hs
