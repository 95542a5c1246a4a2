// Channel-contiguous path: a, b, out are [B, n, D]; lanes own channels, time runs down the rows.
//
// A workgroup of NW waves owns CH = 64*VEC adjacent channels for NW*T consecutive time steps ("tile").
// Wave w of the workgroup scans steps [w*T, (w+1)*T) of the tile serially in each lane (one lane = VEC
// adjacent channels, so a wave's loads and stores are contiguous runs of 256*VEC bytes), keeping the T
// per-element records in registers.  The wave summaries go to LDS, where the first CH threads of the
// workgroup -- one per channel -- turn them into exclusive prefixes; the same threads chain the tiles of
// their channel through global memory: tiles are grouped G at a time along the time axis, a tile folds
// the published summaries of the earlier tiles of its group (always in the same order, so results are
// bit-reproducible) onto the state at the start of the group, and the last tile of a group publishes the
// state at the start of the next.  Every element is read once and written once.
//
// Tiles are handed out by ticket queues, one per compute die: the channel columns are dealt to the
// queues in contiguous runs and a queue hands out its columns' tiles in time order, so a tile only ever
// waits for tiles that were started before it, the draws of the eight dies do not queue behind one
// another, and each die streams through a compact part of memory.
//
// Variations chosen on the host (make_plan): the tile shape; fewer waves per tile for short sequences, no
// tickets at all when a column is one short tile; with few columns, longer groups and a second carry
// level (SG); with fewer than 33 channels, several batch items side by side in the lanes of a column
// (PACKB).
//
// What is computed is Sec. 4's expression applied by parts (Sec. 1, footnote on associativity); the
// arithmetic is in heinsen_math.hpp.
#include "heinsen_internal.hpp"
#include "heinsen_math.hpp"
#include "heinsen_tickets.hpp"

namespace hs {
namespace {

struct BndParams {
    const void *a;
    const void *b;
    const float *x0;
    float *out;       // float32 per element; (re, im) float32 pairs for a log output on a signed domain
    int64_t D, n;
    int x0_stride;    // 0: one x0 for all, 1: x0[b*D + d]
    int cols_per_b;   // ceil(D / CH)
    int ncols;        // B * cols_per_b; narrow rows (PACKB): ceil(B / bpack)
    int64_t B;        // PACKB only below: batch items,
    int dp_shift;     //   log2 of the lanes one batch item takes (the power of two >= D),
    int bpack;        //   batch items per 64-lane column = 64 >> dp_shift
    int nchunks;      // ceil(n / (NW*T))
    uint32_t ntiles;  // ncols * nchunks; tile id = chunk * ncols + col
    int nq;           // ticket queues in use (1 or 8); workgroup i draws from queue i mod nq
    int cols_per_q;   // columns dealt to each queue (the last queues may get fewer, or none)
    uint32_t draws_per_q; // workgroups per queue = grid size / nq
    rec_t *header;    // scratch header (ticket queues); null when the launch needs no carries
    rec_t *agg;       // [ntiles][2][CH]  tile summaries: plane 0 = {A | signs}, plane 1 = {M}
    rec_t *state;     // [ngroups][ncols][2][CH] state at the start of a group: float64 log2|x| in two records
                      // (high word | sign, low word)
                      // (SG > 0: [nsuper][ncols][2][CH], at the start of a super-group of SG groups)
    rec_t *gagg;      // SG > 0: [ngroups][ncols][2][CH] group summaries, planes as in agg
    uint32_t spin_limit;
    uint32_t drop_tile;
    Timeline tl;
};

// every element is touched once: non-temporal accesses keep the stream out of the caches' way
template <typename InT>
__device__ __forceinline__ float load_elem(const InT *p)
{
    return widen(__builtin_nontemporal_load(p));
}

// NT: the output is larger than the last-level cache and is written past it; otherwise it is written
// normally and stays cached for whoever consumes it next.  (A compile-time choice: written as a run-time
// branch the optimiser merges the two stores into one plain store.)
template <bool NT>
__device__ __forceinline__ void store_elem(float *p, float v)
{
    if (NT)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}
template <bool NT>
__device__ __forceinline__ void store_pair(float *p, float re, float im)
{
    typedef float vec_t __attribute__((ext_vector_type(2)));
    const vec_t x = {re, im};
    if (NT)
        __builtin_nontemporal_store(x, reinterpret_cast<vec_t *>(p));
    else
        *reinterpret_cast<vec_t *>(p) = x;
}

__device__ __forceinline__ uint32_t pack_signs(const Seg &g) { return (g.sA >> 31) | ((g.sM >> 31) << 1); }
__device__ __forceinline__ void unpack_signs(uint32_t s, Seg &g)
{
    g.sA = s << 31;
    g.sM = s << 30;
}

// Hand-over between the waves of a workgroup through LDS without a barrier: the producer writes its data,
// then the flag; the consumer polls the flag, then reads the data.  LDS operations of one wave are carried
// out in order, so only the compiler has to be kept from moving them.
__device__ __forceinline__ void lds_signal(volatile uint32_t *flag)
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    *flag = 1u;
}
__device__ __forceinline__ void lds_await(volatile uint32_t *flag)
{
    while (*flag == 0u) __builtin_amdgcn_s_sleep(1);
    asm volatile("" ::: "memory");
}

// One tile.  The NW waves of the workgroup stand CG side by side along the channels and TS = NW / CG deep
// along time; a lane owns one channel for T steps.  G tiles per group along time.  SB: keep the scheduler
// from hoisting work across time steps (bounds register pressure).  PACKB: fewer than 64 channels -- the
// 64 lanes of a column are the channels of several batch items side by side (same tiles, carries and
// arithmetic; only the lane -> memory mapping differs, and a wave's accesses are then pieces of D
// elements, one per batch item).  SG > 0: a second carry level for launches of few columns, where the
// chain of group states would bound the launch: the last tile of a group also publishes the summary of
// its group, states are handed on only from one super-group of SG groups to the next, and a tile folds
// the summaries of the earlier groups of its super-group (a second round of record loads, into the
// registers of the first).
//
// No wave waits for more than it needs.  The first wave along time of each 64-channel column fetches the
// carry records, forms the state at the start of the tile and hands it to the waves behind it through
// LDS; a later wave waits only for the summaries of the waves before it in its own column; the last wave
// along time publishes the tile's summary (and, closing a group, the state for the next group).  `flags`
// are TS*CG + CG words of LDS, zero when the tile begins.
template <int DOM, bool LOG_IN, bool LOG_OUT, typename InT, int T, int NW, int G, bool SB, bool PACKB, int SG, int CG, bool NT>
__device__ __forceinline__ void bnd_tile(const BndParams &p, const uint32_t tile, const uint32_t epoch, volatile uint32_t *flags)
{
    constexpr bool SIGNED = DOM == kSigned;
    constexpr int CH = 64 * CG;  // channels of the tile
    constexpr int TS = NW / CG;  // waves one after the other along time
    constexpr int GP = G > 1 ? G - 1 : 1;
    static_assert(T <= 32, "one sign word per channel");
    static_assert(NW % CG == 0, "the waves form a CG x TS grid");
    static_assert(!PACKB || CG == 1, "narrow rows are mapped one channel per lane");
    static_assert(SG == 0 || (SG <= G && G > 1), "the second round of records reuses the registers of the first");
    __shared__ float lds_A[TS][CH];
    __shared__ float lds_M[TS][CH];
    __shared__ uint32_t lds_S[SIGNED ? TS : 1][CH];
    __shared__ double lds_startL[CH]; // float64: the wave that closes a group hands it on as it is
    __shared__ uint32_t lds_startS[CH];

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // wave-uniform, kept in an SGPR
    // The rows the workgroup reads and writes are runs of 256*CG contiguous bytes, requested by its CG
    // columns at about the same time, which is what the memory system wants to see.
    const int wc = w % CG, ts = w / CG;
    volatile uint32_t *flag_run = flags;              // [TS][CG]: the wave's summary is in LDS
    volatile uint32_t *flag_start = flags + TS * CG;  // [CG]: the column's start state is in LDS

    const int chunk = (int)(tile / (uint32_t)p.ncols);
    const int col = (int)(tile % (uint32_t)p.ncols);
    const int bidx = col / p.cols_per_b;
    const int cg = col % p.cols_per_b;
    const int g = chunk / G;
    const int r = chunk % G;
    const bool more = chunk + 1 < p.nchunks;

    const int c = wc * 64 + lane; // the lane's channel inside the tile
    const int64_t t0 = (int64_t)chunk * (TS * T) + (int64_t)ts * T;
    uint32_t moff;   // the only per-lane part of every global address (elements): the addresses are a
                     // wave-uniform 64-bit base, advanced by scalar arithmetic, plus this 32-bit offset
    bool chan_ok;    // the lane has a channel
    int64_t ubase;   // wave-uniform part of the addresses
    int64_t x0_at;   // the channel's place in x0
    if constexpr (PACKB) {
        const int bb = lane >> p.dp_shift;               // batch item inside the column
        const int d = lane & ((1 << p.dp_shift) - 1);    // channel
        const int64_t b = (int64_t)col * p.bpack + bb;
        chan_ok = d < p.D && b < p.B;
        moff = (uint32_t)(bb * (int)(p.n * p.D) + d);    // the host checks that this fits 31 bits
        ubase = ((int64_t)col * p.bpack * p.n + t0) * p.D;
        x0_at = b * p.D + d;
    } else {
        const int64_t d0 = (int64_t)cg * CH + c;
        chan_ok = d0 < p.D;
        moff = (uint32_t)c;
        ubase = ((int64_t)bidx * p.n + t0) * p.D + (int64_t)cg * CH;
        x0_at = (int64_t)bidx * p.D + d0;
    }
    const InT *ap = reinterpret_cast<const InT *>(p.a) + ubase;
    const InT *bp = reinterpret_cast<const InT *>(p.b) + ubase;

    // ---- the first wave of a column asks for the carry records it will need before anything else is in
    //      flight: once the kernel is past its first round the earlier tiles of the group have usually
    //      published, and the records then arrive ahead of the tile's own loads at no cost in latency ---
    const bool first = ts == 0; // wave-uniform
    rec_t rA[GP], rM[GP], rS = 0, rS2 = 0;
    const int q = SG > 0 ? g / (SG > 0 ? SG : 1) : 0;  // super-group, and the group's place in it
    const int gi = SG > 0 ? g % (SG > 0 ? SG : 1) : 0;
    auto issue_records = [&]() {
        if (SG == 0 && g > 0) {
            const rec_t *sp = p.state + ((size_t)g * p.ncols + col) * (2 * CH) + c;
            rS = rec_get(sp);
            rS2 = rec_get(sp + CH);
        }
#pragma unroll
        for (int j = 0; j < G - 1; ++j) {
            if (j < r) {
                const rec_t *tp = p.agg + ((size_t)(g * G + j) * p.ncols + col) * (2 * CH) + c;
                rA[j] = rec_get(tp);
                rM[j] = rec_get(tp + CH);
            }
        }
    };
    auto records_in = [&]() -> bool { // this lane's records carry the launch's tag
        bool ok = true;
        if (SG == 0 && g > 0) ok = rec_ok(rS, epoch) && rec_ok(rS2, epoch);
#pragma unroll
        for (int j = 0; j < G - 1; ++j) {
            if (j < r) ok = ok && rec_ok(rA[j], epoch) && rec_ok(rM[j], epoch);
        }
        return ok;
    };
    auto wave_all = [](bool ok) -> bool { return __builtin_amdgcn_ballot_w64(!ok) == 0ull; };
    bool have_records = false;
    if (first) issue_records();

    // ---- load: the lane's T inputs ---------------------------------------------------------------
    float Av[T], Mv[T];
    const float id_a = LOG_IN ? 0.0f : 1.0f; // a = 1, b = 0 leave the state unchanged
    const float id_b = LOG_IN ? -INFINITY : 0.0f;
    if (chan_ok && t0 + T <= p.n) {
        const InT *arow = ap, *brow = bp; // wave-uniform row pointers
#pragma unroll
        for (int k = 0; k < T; ++k) {
            Av[k] = load_elem<InT>(arow + moff);
            Mv[k] = load_elem<InT>(brow + moff);
            arow += p.D;
            brow += p.D;
        }
    } else {
#pragma unroll
        for (int k = 0; k < T; ++k) {
            if (chan_ok && t0 + k < p.n) {
                Av[k] = load_elem<InT>(ap + (int64_t)k * p.D + moff);
                Mv[k] = load_elem<InT>(bp + (int64_t)k * p.D + moff);
            } else {
                Av[k] = id_a;
                Mv[k] = id_b;
            }
        }
    }

    if (first) have_records = wave_all(records_in()); // first look: answered while the tile's loads were in flight

    // ---- encode + serial scan in each lane; Av/Mv become the per-element records (see stash) --------
    uint32_t sw = 0u, sm = 0u;
    Seg run;
#pragma unroll
    for (int k = 0; k < T; ++k) {
        lane_step<DOM, LOG_IN, LOG_OUT>(k, run, Av[k], Mv[k], sw, sm);
        if (SB) __builtin_amdgcn_sched_barrier(0);
    }
    lane_close<DOM, LOG_IN, LOG_OUT>(run);
    p.tl.mark(tile, 2);

    // ---- the waves behind this one in the column need its summary --------------------------------
    if (TS > 1 && ts < TS - 1) {
        lds_A[ts][c] = run.A;
        lds_M[ts][c] = run.M;
        if (SIGNED) lds_S[ts][c] = pack_signs(run);
        lds_signal(&flag_run[ts * CG + wc]);
    }
    p.tl.mark(tile, 3);

    State st;                // state at the wave's first step
    State64 st64{0.0, 0u};   // the same in float64, along the chain of tiles
    auto state_from_x0 = [&]() {
        float x0v = LOG_IN ? 0.0f : 1.0f, lx;
        if (chan_ok) x0v = p.x0[p.x0_stride ? x0_at : 0];
        encode<DOM, LOG_IN>(x0v, lx, st64.s);
        st64.lx = (double)lx;
    };
    if (first) {
        // ---- obtain the state at the start of the tile ------------------------------------------
        if (!have_records) issue_records();
        bool lost = false; // this lane's records never came
        if (!have_records) {
            uint32_t polls = 0;
            for (;;) {
                const bool ok = records_in();
                if (wave_all(ok)) break;
                if (++polls > p.spin_limit) {
                    lost = !ok;
                    break;
                }
                __builtin_amdgcn_s_sleep(2);
                issue_records();
            }
        }
        p.tl.mark(tile, 4);
        if constexpr (SG > 0) {
            // the earlier tiles of the group as one summary, kept for the group's summary below
            Seg grp = seg_identity<DOM>();
#pragma unroll
            for (int j = 0; j < G - 1; ++j) {
                if (j < r) grp = seg_combine<DOM>(grp, seg_from<DOM>(rA[j], rM[j]));
            }
            if (lost) grp.M = __builtin_nanf("");
            // second round: the state at the start of the super-group and the earlier groups of it
            auto issue2 = [&]() {
                if (q > 0) {
                    const rec_t *sp = p.state + ((size_t)q * p.ncols + col) * (2 * CH) + c;
                    rS = rec_get(sp);
                    rS2 = rec_get(sp + CH);
                }
#pragma unroll
                for (int j = 0; j < SG - 1; ++j) {
                    if (j < gi) {
                        const rec_t *gp = p.gagg + ((size_t)(q * SG + j) * p.ncols + col) * (2 * CH) + c;
                        rA[j] = rec_get(gp);
                        rM[j] = rec_get(gp + CH);
                    }
                }
            };
            auto in2 = [&]() -> bool {
                bool ok = true;
                if (q > 0) ok = rec_ok(rS, epoch) && rec_ok(rS2, epoch);
#pragma unroll
                for (int j = 0; j < SG - 1; ++j) {
                    if (j < gi) ok = ok && rec_ok(rA[j], epoch) && rec_ok(rM[j], epoch);
                }
                return ok;
            };
            issue2();
            {
                uint32_t polls = 0;
                for (;;) {
                    const bool ok = in2();
                    if (wave_all(ok)) break;
                    if (++polls > p.spin_limit) {
                        lost = lost || !ok;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(2);
                    issue2();
                }
            }
            if (q == 0) {
                state_from_x0();
            } else {
                st64 = state64_from(rS, rS2, SIGNED);
            }
#pragma unroll
            for (int j = 0; j < SG - 1; ++j) {
                if (j < gi) st64 = seg_apply64<DOM>(st64, seg_from<DOM>(rA[j], rM[j]));
            }
            st64 = seg_apply64<DOM>(st64, grp);
            if (lost) {
                st64.lx = __builtin_nan("");
                note_wait_gave_up(p.header);
            }
            st.lx = (float)st64.lx;
            st.s = st64.s;
            if (TS > 1) {
                lds_startL[c] = st64.lx;
                lds_startS[c] = st64.s;
                // the wave that closes the tile also needs the fold of the earlier tiles of the group (the
                // last slot of the summaries is free: the closing wave never writes its own there)
                lds_A[TS - 1][c] = grp.A;
                lds_M[TS - 1][c] = grp.M;
                if (SIGNED) lds_S[TS - 1][c] = pack_signs(grp);
                lds_signal(&flag_start[wc]);
            }
            if (TS == 1) { // a single wave along time closes the tile itself
                if (more && r < G - 1 && tile != p.drop_tile) {
                    rec_t *tp = p.agg + (size_t)tile * (2 * CH) + c;
                    seg_put<DOM>(tp, tp + CH, run, epoch);
                }
                if (more && r == G - 1 && gi < SG - 1) {
                    rec_t *gp = p.gagg + ((size_t)g * p.ncols + col) * (2 * CH) + c;
                    seg_put<DOM>(gp, gp + CH, seg_combine<DOM>(grp, run), epoch);
                }
                if (more && r == G - 1 && gi == SG - 1) {
                    rec_t *sp = p.state + ((size_t)(q + 1) * p.ncols + col) * (2 * CH) + c;
                    state64_put(sp, sp + CH, seg_apply64<DOM>(st64, run), epoch, SIGNED);
                }
            }
        } else {
            if (g == 0) {
                state_from_x0();
            } else {
                st64 = state64_from(rS, rS2, SIGNED);
            }
            // fold the earlier tiles of the group in tile order
#pragma unroll
            for (int j = 0; j < G - 1; ++j) {
                if (j < r) st64 = seg_apply64<DOM>(st64, seg_from<DOM>(rA[j], rM[j]));
            }
            if (lost) {
                st64.lx = __builtin_nan("");
                note_wait_gave_up(p.header);
            }
            st.lx = (float)st64.lx;
            st.s = st64.s;
            if (TS > 1) {
                lds_startL[c] = st64.lx;
                lds_startS[c] = st64.s;
                lds_signal(&flag_start[wc]);
            } else {
                // a single wave along time closes the tile itself
                if (more && r < G - 1 && tile != p.drop_tile) {
                    rec_t *tp = p.agg + (size_t)tile * (2 * CH) + c;
                    seg_put<DOM>(tp, tp + CH, run, epoch);
                }
                if (more && r == G - 1) {
                    rec_t *sp = p.state + ((size_t)(g + 1) * p.ncols + col) * (2 * CH) + c;
                    state64_put(sp, sp + CH, seg_apply64<DOM>(st64, run), epoch, SIGNED);
                }
            }
        }
    } else {
        // ---- a later wave: the fold of the waves before it in its column, in wave order ------------
        Seg pre;
#pragma unroll
        for (int j = 0; j < TS - 1; ++j) {
            if (j < ts) {
                lds_await(&flag_run[j * CG + wc]);
                Seg h;
                h.A = lds_A[j][c];
                h.M = lds_M[j][c];
                h.sA = h.sM = 0u;
                if (SIGNED) unpack_signs(lds_S[j][c], h);
                pre = (j == 0) ? h : seg_combine<DOM>(pre, h);
            }
        }
        // the last wave along time closes the tile: its fold with its own summary is the tile's
        const bool closing = ts == TS - 1; // wave-uniform
        Seg total = seg_identity<DOM>();
        if (closing && more) {
            total = seg_combine<DOM>(pre, run);
            if (r < G - 1 && tile != p.drop_tile) {
                rec_t *tp = p.agg + (size_t)tile * (2 * CH) + c;
                seg_put<DOM>(tp, tp + CH, total, epoch);
            }
        }
        lds_await(&flag_start[wc]);
        st64.lx = lds_startL[c];
        st64.s = lds_startS[c];
        st.lx = (float)st64.lx;
        st.s = st64.s;
        if (closing && more && r == G - 1) {
            if constexpr (SG > 0) {
                Seg grp;
                grp.A = lds_A[TS - 1][c];
                grp.M = lds_M[TS - 1][c];
                grp.sA = grp.sM = 0u;
                if (SIGNED) unpack_signs(lds_S[TS - 1][c], grp);
                if (gi < SG - 1) {
                    rec_t *gp = p.gagg + ((size_t)g * p.ncols + col) * (2 * CH) + c;
                    seg_put<DOM>(gp, gp + CH, seg_combine<DOM>(grp, total), epoch);
                } else {
                    rec_t *sp = p.state + ((size_t)(q + 1) * p.ncols + col) * (2 * CH) + c;
                    state64_put(sp, sp + CH, seg_apply64<DOM>(st64, total), epoch, SIGNED);
                }
            } else {
                // last tile of a group: the state after this tile starts the next group
                rec_t *sp = p.state + ((size_t)(g + 1) * p.ncols + col) * (2 * CH) + c;
                state64_put(sp, sp + CH, seg_apply64<DOM>(st64, total), epoch, SIGNED);
            }
        }
        st = seg_apply<DOM>(st, pre);
    }

    p.tl.mark(tile, 5);
    // ---- every element ----------------------------------------------------------------------------
    constexpr int OW = (SIGNED && LOG_OUT) ? 2 : 1; // floats per output element
    float *op = p.out + OW * ubase;
    const bool full = chan_ok && t0 + T <= p.n;
    const uint32_t swx = fold_state_sign<DOM>(sw, st);
    auto emit_store = [&](int k, bool wanted) {
        if constexpr (SIGNED && LOG_OUT) {
            // complex output: (re, im) pairs, two floats per element
            float re, im;
            emit_clog(st, Av[k], Mv[k], swx, sm, k, re, im);
            if (wanted) store_pair<NT>(op + 2 * ((int64_t)k * p.D + moff), re, im);
        } else {
            const float o = emit<DOM, LOG_OUT>(st, Av[k], Mv[k], swx, k);
            if (wanted) store_elem<NT>(op + (int64_t)k * p.D + moff, o);
        }
    };
    if (full) {
        float *orow = op; // wave-uniform row pointer
#pragma unroll
        for (int k = 0; k < T; ++k) {
            if constexpr (SIGNED && LOG_OUT) {
                float re, im;
                emit_clog(st, Av[k], Mv[k], swx, sm, k, re, im);
                store_pair<NT>(orow + 2 * (size_t)moff, re, im);
            } else {
                store_elem<NT>(orow + moff, emit<DOM, LOG_OUT>(st, Av[k], Mv[k], swx, k));
            }
            orow += OW * p.D;
            if (SB) __builtin_amdgcn_sched_barrier(0);
        }
    } else {
#pragma unroll
        for (int k = 0; k < T; ++k) {
            emit_store(k, chan_ok && t0 + k < p.n);
            if (SB) __builtin_amdgcn_sched_barrier(0);
        }
    }
    p.tl.mark(tile, 6);
}

template <int DOM, bool LOG_IN, bool LOG_OUT, typename InT, int T, int NW, int G, int MINW, bool SB, bool PACKB = false, int SG = 0, int CG = 1, bool NT = false>
__global__ __launch_bounds__(NW * 64, MINW) void heinsen_scan_bnd(BndParams p)
{
    __shared__ uint32_t s_tile, s_epoch, s_flag;
    __shared__ uint32_t s_flags[NW + CG];
    const unsigned long long t_begin = p.tl.stamps != nullptr ? wall_clock64() : 0ull;
    uint32_t tile, epoch = 0u;
    if (threadIdx.x < NW + CG) s_flags[threadIdx.x] = 0u;
    if (p.header == nullptr) {
        // A launch whose columns are one short tile long (at most 64 steps) has nothing to wait for and
        // comes without tickets: there the draw's round trip would be a large part of a tile's life.
        // Workgroups go to the eight compute dies in turn (workgroup i to die i mod 8): give every die a
        // contiguous eighth of the tiles, so that the tiles in flight form eight compact windows of memory
        // instead of a wide, ragged one.
        const uint32_t die = blockIdx.x & 7u, j = blockIdx.x >> 3;
        const uint32_t qn = p.ntiles >> 3, rem = p.ntiles & 7u;
        tile = die * qn + (die < rem ? die : rem) + j;
    } else {
        // Tiles are handed out in start order, so every tile a workgroup may wait for (same column,
        // earlier chunk => same queue, smaller ticket) belongs to a workgroup that is already running.
        if (threadIdx.x == 0) {
            const int qi = (int)(blockIdx.x % (uint32_t)p.nq);
            const Draw d = draw_ticket(p.header, qi, p.draws_per_q, p.nq);
            int cols = p.ncols - qi * p.cols_per_q; // columns of this queue
            cols = cols > p.cols_per_q ? p.cols_per_q : cols;
            uint32_t t = 0xffffffffu;
            if (cols > 0) {
                const uint32_t chunk = d.ticket / (uint32_t)cols, cq = d.ticket % (uint32_t)cols;
                if (chunk < (uint32_t)p.nchunks) t = chunk * (uint32_t)p.ncols + (uint32_t)(qi * p.cols_per_q) + cq;
            }
            s_tile = t;
            s_epoch = d.epoch;
        }
    }
    __syncthreads(); // the only barrier of a tile: ticket and cleared flags are in LDS
    if (p.header != nullptr) {
        tile = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_tile);
        epoch = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_epoch);
    }
    if (tile < p.ntiles) {
        p.tl.mark_at(tile, 0, t_begin);
        p.tl.mark(tile, 1);
        bnd_tile<DOM, LOG_IN, LOG_OUT, InT, T, NW, G, SB, PACKB, SG, CG, NT>(p, tile, epoch, s_flags);
        p.tl.mark(tile, 7);
    }
    if (p.header != nullptr) end_of_workgroup(p.header, epoch, &s_flag);
}

// ---- host side ------------------------------------------------------------------------------------

// MI355X: 256 MB of memory-side cache; an output up to three quarters of it is left to be cached
constexpr int64_t kLastLevelCacheBytes = 192ll << 20;

// Ticket queues: as many (up to one per compute die) as leave every queue this many columns.  The tiles
// of a column start that many tickets apart, so a tile usually finds the tiles before it done; the wide
// tiles, whose rows are requested by two waves at a time, want the queues longer still (measured).
constexpr int kMinColsPerQueue = 16, kMinColsPerQueueWide = 128;

struct BndPlan {
    int cg, T, NW, G, CH;
    bool ticketless;
    int dp_shift, bpack; // bpack > 1: narrow rows, the channels of bpack batch items share a 64-lane column
    int cols_per_b, ncols, nchunks, ngroups;
    uint32_t ntiles;
    int nq, cols_per_q;
    uint32_t grid;
    int SG;             // > 0: groups per super-group (second carry level)
    size_t off_agg, off_gagg, off_state, records; // in records, relative to kRecordBase
};

BndPlan make_plan(const ScanCall &c, bool allow_wide = true)
{
    BndPlan pl;
    // Default tile: 64 channels x 256 steps (8 waves one after the other along time, 32 steps each;
    // <= 128 VGPRs, two workgroups per CU).  With many wide rows the tile is 128 channels x 128 steps
    // instead (two waves side by side): the rows a workgroup touches are then 512 contiguous bytes, which
    // the memory system serves about 4 % faster, at the price of twice as many tiles along time.
    pl.cg = 1;
    pl.T = 32;
    pl.NW = 8;
    pl.G = 4;
    const bool complex_out = c.is_signed && c.log_out;
    if (complex_out) {
        // complex output: the signed log-domain emit needs more registers per element; 16 steps per wave
        // and 16 waves keep the tile the same and the kernel free of spills
        pl.T = 16;
        pl.NW = 16;
    } else if (c.n <= 128) {
        // short sequences: no more waves than have steps to work on
        pl.NW = c.n <= 32 ? 1 : (c.n <= 64 ? 2 : 4);

    } else if (allow_wide && c.D % 128 == 0 && c.B * (c.D / 128) >= 2 * kMinColsPerQueueWide && c.n >= 1024) {
        pl.cg = 2;
    }
    pl.CH = 64 * pl.cg;
    pl.cols_per_b = (int)ceil_div(c.D, pl.CH);
    pl.ncols = (int)(c.B * pl.cols_per_b);

    pl.dp_shift = 6;
    pl.bpack = 1;
    if (c.D <= 32 && c.B > 1) {
        int sh = 0;
        while ((1 << sh) < c.D) ++sh;
        // a lane's offset from its column's base must fit a 32-bit byte offset
        if ((int64_t)(64 >> sh) * c.n * c.D < ((int64_t)1 << 29)) {
            pl.dp_shift = sh;
            pl.bpack = 64 >> sh;
            pl.ncols = (int)ceil_div(c.B, pl.bpack);
        }
    }
    // Few columns: the states handed from group to group (0.9 us per link) bound the launch, not the
    // memory.  Below 64 columns the groups are eight tiles long (half the links); up to 8 columns a second
    // carry level hands states on only between super-groups (4 x 4 tiles: n / 4096 links, no spills; one
    // or two columns: 8 x 8 tiles, n / 16384 links, at the price of some spilled registers).  With many
    // columns the longer folds and the second round of record loads would cost a few percent.  Not for the
    // modes whose kernels are short of registers already.
    pl.SG = 0;
    if (pl.cg == 1 && pl.NW == 8 && pl.T == 32 && !(c.log_in && c.log_out)) {
        if (pl.ncols <= 2) {
            pl.G = 8;
            pl.SG = 8;
        } else if (pl.ncols <= 8) {
            pl.G = 4;
            pl.SG = 4;
        } else if (pl.ncols < 64) {
            pl.G = 8;
        }
    }
    pl.nchunks = (int)ceil_div(c.n, (int64_t)(pl.NW / pl.cg) * pl.T);
    pl.ngroups = (int)ceil_div(pl.nchunks, pl.G);
    pl.ntiles = (uint32_t)pl.ncols * (uint32_t)pl.nchunks;
    pl.off_agg = 0;
    pl.off_gagg = (size_t)pl.ntiles * 2 * pl.CH;
    pl.off_state = pl.off_gagg + (pl.SG ? (size_t)pl.ngroups * pl.ncols * 2 * pl.CH : 0);
    pl.records = pl.off_state + (size_t)(pl.SG ? ceil_div(pl.ngroups, pl.SG) + 1 : pl.ngroups) * pl.ncols * 2 * pl.CH;
    pl.ticketless = pl.nchunks == 1 && c.n <= 64; // short single-tile columns: no records, no tickets
    // A queue's workgroups that find no tile behind their ticket (uneven deal) end at once.
    pl.nq = kQueues;
    while (pl.nq > 1 && pl.ncols < pl.nq * (pl.cg > 1 ? kMinColsPerQueueWide : kMinColsPerQueue)) pl.nq /= 2;
    pl.cols_per_q = (int)ceil_div(pl.ncols, pl.nq);
    pl.grid = pl.ntiles;
    if (pl.ticketless) {
        pl.records = 0;
    } else {
        pl.grid = (uint32_t)pl.nq * (uint32_t)pl.cols_per_q * (uint32_t)pl.nchunks;
    }
    // the wide tiles take twice the records: a caller with a fixed scratch buffer may have to do without them
    if (pl.cg > 1 && c.scratch_budget != 0 && kRecordBase + pl.records > c.scratch_budget) return make_plan(c, false);
    return pl;
}

template <int DOM, bool LOG_IN, bool LOG_OUT, typename InT>
hipError_t launch_mode(const ScanCall &c, const BndPlan &pl, const LaunchCtx &ctx)
{
    constexpr bool SIGNED = DOM == kSigned;
    rec_t *records = pl.ticketless ? nullptr : ctx.scratch;
    BndParams p;
    p.a = c.a;
    p.b = c.b;
    p.x0 = c.x0;
    p.out = c.out;
    p.D = c.D;
    p.n = c.n;
    p.x0_stride = c.x0_scalar ? 0 : 1;
    // the output does not fit the last-level cache: write it non-temporally (shapes with a kernel for it)
    const bool nt_out = c.B * c.D * c.n * ((SIGNED && LOG_OUT) ? 8 : 4) > kLastLevelCacheBytes;
    p.cols_per_b = pl.cols_per_b;
    p.B = c.B;
    p.dp_shift = pl.dp_shift;
    p.bpack = pl.bpack;
    p.ncols = pl.ncols;
    p.nchunks = pl.nchunks;
    p.ntiles = pl.ntiles;
    p.nq = pl.nq;
    p.cols_per_q = pl.cols_per_q;
    p.draws_per_q = pl.grid / (uint32_t)pl.nq;
    p.header = records; // null when the launch needs no carries
    p.agg = records ? records + kRecordBase + pl.off_agg : nullptr;
    p.state = records ? records + kRecordBase + pl.off_state : nullptr;
    p.gagg = records ? records + kRecordBase + pl.off_gagg : nullptr;
    p.spin_limit = ctx.spin_limit;
    p.drop_tile = ctx.drop_tile;
    p.tl.stamps = ctx.timeline;
    p.tl.tiles = ctx.timeline_tiles;
    if (!pl.ticketless && records == nullptr) return hipErrorInvalidValue;
    dim3 grid(pl.grid), block(pl.NW * 64);
    if constexpr (SIGNED && LOG_OUT) {
        if (pl.bpack > 1)
            hipLaunchKernelGGL((heinsen_scan_bnd<DOM, LOG_IN, LOG_OUT, InT, 16, 16, 4, 4, true, true>), grid, block, 0, c.stream, p);
        else if (nt_out)
            hipLaunchKernelGGL((heinsen_scan_bnd<DOM, LOG_IN, LOG_OUT, InT, 16, 16, 4, 4, true, false, 0, 1, true>), grid, block, 0, c.stream, p);
        else
            hipLaunchKernelGGL((heinsen_scan_bnd<DOM, LOG_IN, LOG_OUT, InT, 16, 16, 4, 4, true>), grid, block, 0, c.stream, p);
    } else {
        if (pl.cg == 2) {
            if (nt_out)
                hipLaunchKernelGGL((heinsen_scan_bnd<DOM, LOG_IN, LOG_OUT, InT, 32, 8, 4, 4, true, false, 0, 2, true>), grid, block, 0, c.stream, p);
            else
                hipLaunchKernelGGL((heinsen_scan_bnd<DOM, LOG_IN, LOG_OUT, InT, 32, 8, 4, 4, true, false, 0, 2, false>), grid, block, 0, c.stream, p);
            return hipGetLastError();
        }
#define HS_BND(NW_, PACKB_) \
    hipLaunchKernelGGL((heinsen_scan_bnd<DOM, LOG_IN, LOG_OUT, InT, 32, NW_, 4, 4, true, PACKB_>), grid, block, 0, c.stream, p)
        if constexpr (!(LOG_IN && LOG_OUT)) {
            if (pl.G == 8 || pl.SG > 0) {
#define HS_BND_CARRY(G_, SG_, PACKB_) \
    hipLaunchKernelGGL((heinsen_scan_bnd<DOM, LOG_IN, LOG_OUT, InT, 32, 8, G_, 4, true, PACKB_, SG_>), grid, block, 0, c.stream, p)
                if (pl.bpack > 1) {
                    if (pl.SG == 8) HS_BND_CARRY(8, 8, true);
                    else if (pl.SG == 4) HS_BND_CARRY(4, 4, true);
                    else HS_BND_CARRY(8, 0, true);
                } else {
                    if (pl.SG == 8) HS_BND_CARRY(8, 8, false);
                    else if (pl.SG == 4) HS_BND_CARRY(4, 4, false);
                    else HS_BND_CARRY(8, 0, false);
                }
#undef HS_BND_CARRY
                return hipGetLastError();
            }
        }
        if (pl.bpack > 1) {
            if (pl.NW == 1) HS_BND(1, true);
            else if (pl.NW == 2) HS_BND(2, true);
            else if (pl.NW == 4) HS_BND(4, true);
            else HS_BND(8, true);
        } else {
            if (pl.NW == 1) HS_BND(1, false);
            else if (pl.NW == 2) HS_BND(2, false);
            else if (pl.NW == 4) HS_BND(4, false);
            else if (nt_out)
                hipLaunchKernelGGL((heinsen_scan_bnd<DOM, LOG_IN, LOG_OUT, InT, 32, 8, 4, 4, true, false, 0, 1, true>), grid, block, 0, c.stream, p);
            else HS_BND(8, false);
        }
#undef HS_BND
    }
    return hipGetLastError();
}

hipError_t launch_dispatch(const ScanCall &c, const BndPlan &pl, const LaunchCtx &ctx)
{
    HS_DISPATCH_MODE(c, launch_mode, c, pl, ctx);
}

} // namespace

ScratchNeed bnd_scratch(const ScanCall &c)
{
    BndPlan pl = make_plan(c);
    return ScratchNeed{pl.records};
}

hipError_t bnd_launch(const ScanCall &c, const LaunchCtx &ctx)
{
    BndPlan pl = make_plan(c);
    return launch_dispatch(c, pl, ctx);
}

const char *bnd_kernel_name(const ScanCall &) { return "heinsen_scan_bnd"; }

void bnd_tile_shape(const ScanCall &c, int &channels, int64_t &steps)
{
    const BndPlan pl = make_plan(c);
    channels = pl.bpack > 1 ? (int)c.D : pl.CH; // narrow rows: the channels of pl.bpack batch items side by side
    steps = (int64_t)(pl.NW / pl.cg) * pl.T;
}

} // namespace hs
