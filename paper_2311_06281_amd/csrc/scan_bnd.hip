// Channel-contiguous path: a, b, out are [B, n, D]; lanes own channels, time runs down the rows.
//
// A workgroup of NW waves owns CH = 64*VEC adjacent channels for NW*T consecutive time steps ("tile").
// Wave w of the workgroup scans steps [w*T, (w+1)*T) of the tile serially in each lane (one lane = VEC
// channels, loads and stores coalesced across lanes), keeping the T per-element records in registers.
// Summaries of the waves are chained through LDS, summaries of the tiles of one channel column through
// global memory: tiles are grouped G at a time along the time axis, a tile folds the published
// summaries of the earlier tiles of its group (always in the same order, so results are
// bit-reproducible) onto the state at the start of the group, and the last tile of a group publishes
// the state at the start of the next.  Every element is read once and written once.
//
// Variations chosen on the host (make_plan): fewer waves per tile for short sequences, no tickets at
// all when a column is one short tile; with few columns, longer groups and a second carry level (SG);
// with fewer than 33 channels, several batch items side by side in the lanes of a column (PACKB).
//
// What is computed is Sec. 4's expression applied by parts (Sec. 1, footnote on associativity); the
// arithmetic is in heinsen_math.hpp.
#include "heinsen_internal.hpp"
#include "heinsen_math.hpp"
#include <cstdlib>

namespace hs {
namespace {

struct BndParams {
    const void *a;
    const void *b;
    const float *x0;
    float *out;       // float32 per element; (re, im) float32 pairs for a log output on a signed domain
    int64_t D, n;
    int x0_stride;    // 0: one x0 for all, 1: x0[b*D + d]
    int stream_out;   // 1: the output does not fit the last-level cache, write it non-temporally
    int cols_per_b;   // ceil(D / CH)
    int ncols;        // B * cols_per_b; narrow rows (PACKB): ceil(B / bpack)
    int64_t B;        // PACKB only below: batch items,
    int dp_shift;     //   log2 of the lanes one batch item takes (the power of two >= D),
    int bpack;        //   batch items per 64-lane column = 64 >> dp_shift
    int nchunks;      // ceil(n / (NW*T))
    uint32_t ntiles;  // ncols * nchunks
    uint32_t epoch;
    uint32_t ticket_base;
    int from_header;  // replayed from a graph: epoch and tickets come from the scratch header
    rec_t *ticket;    // word 0 of the record buffer (the scratch header)
    rec_t *agg;       // [ntiles][2][CH]  tile summaries: plane 0 = {A | signs}, plane 1 = {M}
    rec_t *state;     // [ngroups][ncols][CH] state at the start of a group: {log2|x| | sign}
                      // (SG > 0: [nsuper][ncols][CH], at the start of a super-group of SG groups)
    rec_t *gagg;      // SG > 0: [ngroups][ncols][2][CH] group summaries, planes as in agg
#ifdef HS_TRACE
    unsigned long long *trace; // [ntiles][8] wall-clock stamps of wave 0 (100 MHz), development only
#endif
};

#ifdef HS_TRACE
#define HS_STAMP(i)                                                              \
    do {                                                                         \
        if (threadIdx.x == 0) p.trace[(size_t)tile * 8 + (i)] = wall_clock64(); \
    } while (0)
#else
#define HS_STAMP(i) \
    do {            \
    } while (0)
#endif

template <typename InT, int VEC>
__device__ __forceinline__ void load_vec(const InT *p, float (&v)[VEC])
{
    // every element is touched once: non-temporal accesses keep the stream out of the caches' way
    typedef InT vec_t __attribute__((ext_vector_type(VEC)));
    vec_t x = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(p));
#pragma unroll
    for (int i = 0; i < VEC; ++i) v[i] = widen(x[i]);
}
template <typename InT>
__device__ __forceinline__ void load_vec(const InT *p, float (&v)[1])
{
    v[0] = widen(__builtin_nontemporal_load(p));
}

// stream: the output is larger than the last-level cache and is written past it; otherwise it is
// written normally and stays cached for whoever consumes it next.
template <int VEC>
__device__ __forceinline__ void store_vec(float *p, const float (&v)[VEC], bool stream)
{
    typedef float vec_t __attribute__((ext_vector_type(VEC)));
    vec_t x;
#pragma unroll
    for (int i = 0; i < VEC; ++i) x[i] = v[i];
    if (stream)
        __builtin_nontemporal_store(x, reinterpret_cast<vec_t *>(p));
    else
        *reinterpret_cast<vec_t *>(p) = x;
}
__device__ __forceinline__ void store_vec(float *p, const float (&v)[1], bool stream)
{
    if (stream)
        __builtin_nontemporal_store(v[0], p);
    else
        *p = v[0];
}

__device__ __forceinline__ uint32_t pack_signs(const Seg &g) { return (g.sA >> 31) | ((g.sM >> 31) << 1); }
__device__ __forceinline__ void unpack_signs(uint32_t s, Seg &g)
{
    g.sA = s << 31;
    g.sM = s << 30;
}

// VEC channels per lane, T steps per wave, NW waves per workgroup, G tiles per group along time,
// MINW waves per SIMD the register allocation must allow, SB: keep the scheduler from hoisting work
// across time steps (bounds register pressure).  PACKB: fewer than 64 channels -- the 64 lanes of a column
// are the channels of several batch items side by side (same tiles, carries and arithmetic; only the
// lane -> memory mapping differs, and a wave's accesses are then pieces of D elements, one per batch item).
// SG > 0: a second carry level for launches of few columns, where the chain of group states would bound
// the launch: the last tile of a group also publishes the summary of its group, states are handed on only
// from one super-group of SG groups to the next, and a tile folds the summaries of the earlier groups of
// its super-group (a second round of record loads, into the registers of the first).
template <int DOM, bool LOG_IN, bool LOG_OUT, typename InT, int VEC, int T, int NW, int G, int MINW, bool SB, bool PACKB = false, int SG = 0>
__global__ __launch_bounds__(NW * 64, MINW) void heinsen_scan_bnd(BndParams p)
{
    constexpr bool SIGNED = DOM == kSigned;
    constexpr int CH = 64 * VEC;
    constexpr int GP = G > 1 ? G - 1 : 1;
    static_assert(T <= 32, "one sign word per channel");
    __shared__ uint32_t s_tile;
    __shared__ uint32_t s_epoch;
    __shared__ float lds_A[NW][CH];
    __shared__ float lds_M[NW][CH];
    __shared__ uint32_t lds_S[NW][CH];
    __shared__ float lds_startL[CH];
    __shared__ uint32_t lds_startS[CH];

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // wave-uniform, kept in an SGPR
#ifdef HS_TRACE
    const unsigned long long t_begin = wall_clock64();
#endif

    // Tiles are handed out in start order, so every tile a workgroup may wait for (same column,
    // earlier chunk => smaller ticket) belongs to a workgroup that is already running.  A launch whose
    // columns are one short tile long (at most 64 steps) has nothing to wait for and comes without a
    // ticket counter: there the draw's round trip would be a large part of a tile's life.  (Longer
    // single-tile columns keep the ticket although they have no carries: measured 8 % faster with it.)
    uint32_t tile;
    if (p.ticket == nullptr) {
        // Workgroups go to the eight compute dies in turn (workgroup i to die i mod 8): give every die a
        // contiguous eighth of the tiles, so that the tiles in flight form eight compact windows of memory
        // instead of a wide, ragged one (measured 2-3 % faster).
        const uint32_t die = blockIdx.x & 7u, j = blockIdx.x >> 3;
        const uint32_t q = p.ntiles >> 3, rem = p.ntiles & 7u;
        tile = die * q + (die < rem ? die : rem) + j;
    } else {
        if (threadIdx.x == 0) {
            uint32_t *counter = reinterpret_cast<uint32_t *>(p.ticket + (p.from_header ? kHeaderGraphTicket : 0));
            s_tile = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) -
                     (p.from_header ? 0u : p.ticket_base);
            // a replayed launch finds its epoch in the header (written by the kernel recorded before this one)
            s_epoch = p.from_header ? (uint32_t)p.ticket[kHeaderGraphEpoch] : p.epoch;
        }
        __syncthreads();
        tile = __builtin_amdgcn_readfirstlane(s_tile);
    }
    const uint32_t epoch = p.ticket != nullptr ? (uint32_t)__builtin_amdgcn_readfirstlane((int)s_epoch) : 0u;
    // A ticket outside the launch can only mean that the counter and the host's record of it have come
    // apart (an earlier launch on this stream died): touch nothing rather than index out of bounds.
    if (tile >= p.ntiles) return;
    HS_STAMP(0);
    const int chunk = (int)(tile / (uint32_t)p.ncols);
    const int col = (int)(tile % (uint32_t)p.ncols);
    const int bidx = col / p.cols_per_b;
    const int cg = col % p.cols_per_b;
    const int g = chunk / G;
    const int r = chunk % G;
    const bool more = chunk + 1 < p.nchunks;

    const int loff = lane * VEC; // the lane's place in LDS arrays and carry records
    const int64_t t0 = (int64_t)chunk * (NW * T) + (int64_t)w * T;
    int moff;        // the only per-lane part of every global address (elements)
    bool chan_ok;    // the lane has a channel
    int64_t ubase;   // wave-uniform part of the addresses
    int64_t x0_at;   // index of the lane's first channel in x0
    if constexpr (PACKB) {
        static_assert(VEC == 1, "narrow rows are mapped one channel per lane");
        const int bb = lane >> p.dp_shift;               // batch item inside the column
        const int d = lane & ((1 << p.dp_shift) - 1);    // channel
        const int64_t b = (int64_t)col * p.bpack + bb;
        chan_ok = d < p.D && b < p.B;
        moff = bb * (int)(p.n * p.D) + d;                // the host checks that this fits 31 bits
        ubase = ((int64_t)col * p.bpack * p.n + t0) * p.D;
        x0_at = b * p.D + d;
    } else {
        const int64_t d0 = (int64_t)cg * CH + loff;
        chan_ok = d0 < p.D; // D is a multiple of VEC, so the whole vector is in range
        moff = loff;
        ubase = ((int64_t)bidx * p.n + t0) * p.D + (int64_t)cg * CH;
        x0_at = (int64_t)bidx * p.D + d0;
    }
    const InT *ap = reinterpret_cast<const InT *>(p.a) + ubase;
    const InT *bp = reinterpret_cast<const InT *>(p.b) + ubase;

    // ---- wave 0 asks for the carry records it will need before anything else is in flight: once the
    //      kernel is past its first round the earlier tiles of the group have usually published, and the
    //      records then arrive ahead of the tile's own loads at no cost in latency --------------------
    rec_t rA[GP][VEC], rM[GP][VEC], rS[VEC];
    static_assert(SG == 0 || (SG <= G && G > 1), "the second round of records reuses the registers of the first");
    const int q = SG > 0 ? g / (SG > 0 ? SG : 1) : 0;  // super-group, and the group's place in it
    const int gi = SG > 0 ? g % (SG > 0 ? SG : 1) : 0;
    auto issue_records = [&]() {
        if (SG == 0 && g > 0) {
            const rec_t *sp = p.state + ((size_t)g * p.ncols + col) * CH + loff;
#pragma unroll
            for (int v = 0; v < VEC; ++v) rS[v] = rec_get(sp + v);
        }
#pragma unroll
        for (int j = 0; j < G - 1; ++j) {
            if (j < r) {
                const rec_t *tp = p.agg + ((size_t)(g * G + j) * p.ncols + col) * (2 * CH) + loff;
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    rA[j][v] = rec_get(tp + v);
                    rM[j][v] = rec_get(tp + CH + v);
                }
            }
        }
    };
    auto records_in = [&]() -> bool {
        bool ok = true;
        if (SG == 0 && g > 0) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) ok = ok && rec_ok(rS[v], epoch);
        }
#pragma unroll
        for (int j = 0; j < G - 1; ++j) {
            if (j < r) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) ok = ok && rec_ok(rA[j][v], epoch) && rec_ok(rM[j][v], epoch);
            }
        }
        return __builtin_amdgcn_ballot_w64(!ok) == 0ull;
    };
    bool have_records = false;
    if (w == 0) issue_records();

    // ---- load: the lane's T x VEC inputs -------------------------------------------------------
    float Av[T][VEC], Mv[T][VEC];
    const float id_a = LOG_IN ? 0.0f : 1.0f; // a = 1, b = 0 leave the state unchanged
    const float id_b = LOG_IN ? -INFINITY : 0.0f;
    if (chan_ok && t0 + T <= p.n) {
#pragma unroll
        for (int k = 0; k < T; ++k) {
            load_vec<InT>(ap + (int64_t)k * p.D + moff, Av[k]);
            load_vec<InT>(bp + (int64_t)k * p.D + moff, Mv[k]);
        }
    } else {
#pragma unroll
        for (int k = 0; k < T; ++k) {
            if (chan_ok && t0 + k < p.n) {
                load_vec<InT>(ap + (int64_t)k * p.D + moff, Av[k]);
                load_vec<InT>(bp + (int64_t)k * p.D + moff, Mv[k]);
            } else {
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    Av[k][v] = id_a;
                    Mv[k][v] = id_b;
                }
            }
        }
    }

    if (w == 0) have_records = records_in(); // first look: answered while the tile's loads were in flight

    // ---- encode + serial scan in each lane; Av/Mv become the per-element records (see stash) --------
    uint32_t sw[VEC], sm[VEC];
    Seg run[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) sw[v] = sm[v] = 0u;
#pragma unroll
    for (int k = 0; k < T; ++k) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            float la, lb;
            uint32_t sa, sb;
            encode<DOM, LOG_IN>(Av[k][v], la, sa);
            encode<DOM, LOG_IN>(Mv[k][v], lb, sb);
            if (k == 0) {
                run[v] = Seg{la, lb, sa, sb};
            } else {
                seg_step<DOM>(run[v], la, sa, lb, sb);
            }
            stash<DOM, LOG_OUT>(run[v], k, Av[k][v], Mv[k][v], sw[v], sm[v]);
        }
        if (SB) __builtin_amdgcn_sched_barrier(0);
    }

    HS_STAMP(1);
    // second look, asked now and read after the barrier and the fold below
    if (w == 0 && !have_records) issue_records();

    // ---- chain the waves of the workgroup through LDS ------------------------------------------
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        lds_A[w][loff + v] = run[v].A;
        lds_M[w][loff + v] = run[v].M;
        if (SIGNED) lds_S[w][loff + v] = pack_signs(run[v]);
    }
    __syncthreads();

    // wave w folds the summaries of waves 0..w-1 (its exclusive prefix inside the tile);
    // wave 0 instead folds all NW of them: the summary of the whole tile.
    Seg pre[VEC];
    {
        const int cnt = (w == 0) ? NW : w;
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            Seg acc;
            acc.A = lds_A[0][loff + v];
            acc.M = lds_M[0][loff + v];
            acc.sA = acc.sM = 0u;
            if (SIGNED) unpack_signs(lds_S[0][loff + v], acc);
            for (int j = 1; j < cnt; ++j) {
                Seg h;
                h.A = lds_A[j][loff + v];
                h.M = lds_M[j][loff + v];
                h.sA = h.sM = 0u;
                if (SIGNED) unpack_signs(lds_S[j][loff + v], h);
                acc = seg_combine<DOM>(acc, h);
            }
            pre[v] = acc;
        }
    }

    // ---- wave 0: publish the tile summary, obtain the state at the start of the tile -------------
    if (w == 0) {
        HS_STAMP(2);
        if (more && r < G - 1) {
            rec_t *tp = p.agg + (size_t)tile * (2 * CH) + loff;
#pragma unroll
            for (int v = 0; v < VEC; ++v) seg_put<DOM>(tp + v, tp + CH + v, pre[v], epoch);
        }
#ifdef HS_TRACE
        if (threadIdx.x == 0) p.trace[(size_t)tile * 8 + 3] = t_begin; // slot 3: workgroup start, before the ticket
#endif
        if (!have_records) {
            while (!records_in()) {
                __builtin_amdgcn_s_sleep(2);
                issue_records();
            }
        }
        HS_STAMP(4);
        State st[VEC];
        if constexpr (SG > 0) {
            // the earlier tiles of the group as one summary; the last tile of a group owes the later groups
            // of its super-group the summary of the whole group (no state needed for it)
            Seg grp[VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) grp[v] = seg_identity<DOM>();
#pragma unroll
            for (int j = 0; j < G - 1; ++j) {
                if (j < r) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) grp[v] = seg_combine<DOM>(grp[v], seg_from<DOM>(rA[j][v], rM[j][v]));
                }
            }
            if (more && r == G - 1 && gi < SG - 1) {
                rec_t *gp = p.gagg + ((size_t)g * p.ncols + col) * (2 * CH) + loff;
#pragma unroll
                for (int v = 0; v < VEC; ++v) seg_put<DOM>(gp + v, gp + CH + v, seg_combine<DOM>(grp[v], pre[v]), epoch);
            }
            // second round: the state at the start of the super-group and the earlier groups of it
            auto issue2 = [&]() {
                if (q > 0) {
                    const rec_t *sp = p.state + ((size_t)q * p.ncols + col) * CH + loff;
#pragma unroll
                    for (int v = 0; v < VEC; ++v) rS[v] = rec_get(sp + v);
                }
#pragma unroll
                for (int j = 0; j < SG - 1; ++j) {
                    if (j < gi) {
                        const rec_t *gp = p.gagg + ((size_t)(q * SG + j) * p.ncols + col) * (2 * CH) + loff;
#pragma unroll
                        for (int v = 0; v < VEC; ++v) {
                            rA[j][v] = rec_get(gp + v);
                            rM[j][v] = rec_get(gp + CH + v);
                        }
                    }
                }
            };
            auto in2 = [&]() -> bool {
                bool ok = true;
                if (q > 0) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) ok = ok && rec_ok(rS[v], epoch);
                }
#pragma unroll
                for (int j = 0; j < SG - 1; ++j) {
                    if (j < gi) {
#pragma unroll
                        for (int v = 0; v < VEC; ++v) ok = ok && rec_ok(rA[j][v], epoch) && rec_ok(rM[j][v], epoch);
                    }
                }
                return __builtin_amdgcn_ballot_w64(!ok) == 0ull;
            };
            issue2();
            while (!in2()) {
                __builtin_amdgcn_s_sleep(2);
                issue2();
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                if (q == 0) {
                    float x0v = LOG_IN ? 0.0f : 1.0f;
                    if (chan_ok) x0v = p.x0[p.x0_stride ? (x0_at + v) : 0];
                    encode<DOM, LOG_IN>(x0v, st[v].lx, st[v].s);
                } else {
                    st[v].lx = u2f(rec_payload(rS[v]));
                    st[v].s = SIGNED ? (rec_bits(rS[v]) << 31) : 0u;
                }
            }
#pragma unroll
            for (int j = 0; j < SG - 1; ++j) {
                if (j < gi) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) st[v] = seg_apply<DOM>(st[v], seg_from<DOM>(rA[j][v], rM[j][v]));
                }
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                st[v] = seg_apply<DOM>(st[v], grp[v]);
                lds_startL[loff + v] = st[v].lx;
                lds_startS[loff + v] = st[v].s;
            }
            HS_STAMP(5);
            // last tile of a super-group: the state after this tile starts the next one
            if (more && r == G - 1 && gi == SG - 1) {
                rec_t *sp = p.state + ((size_t)(q + 1) * p.ncols + col) * CH + loff;
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    State nx = seg_apply<DOM>(st[v], pre[v]);
                    rec_put(sp + v, f2u(nx.lx), epoch, SIGNED ? (nx.s >> 31) : 0u);
                }
            }
        } else {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            if (g == 0) {
                float x0v = LOG_IN ? 0.0f : 1.0f;
                if (chan_ok) x0v = p.x0[p.x0_stride ? (x0_at + v) : 0];
                encode<DOM, LOG_IN>(x0v, st[v].lx, st[v].s);
            } else {
                st[v].lx = u2f(rec_payload(rS[v]));
                st[v].s = SIGNED ? (rec_bits(rS[v]) << 31) : 0u;
            }
        }
        // fold the earlier tiles of the group in tile order
#pragma unroll
        for (int j = 0; j < G - 1; ++j) {
            if (j < r) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) st[v] = seg_apply<DOM>(st[v], seg_from<DOM>(rA[j][v], rM[j][v]));
            }
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            lds_startL[loff + v] = st[v].lx;
            lds_startS[loff + v] = st[v].s;
        }
        HS_STAMP(5);
        // last tile of a group: the state after this tile starts the next group
        if (more && r == G - 1) {
            rec_t *sp = p.state + ((size_t)(g + 1) * p.ncols + col) * CH + loff;
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                State nx = seg_apply<DOM>(st[v], pre[v]);
                rec_put(sp + v, f2u(nx.lx), epoch, SIGNED ? (nx.s >> 31) : 0u);
            }
        }
        }
    }
    __syncthreads();

    HS_STAMP(6);
    // ---- state at the start of this wave's steps, then every element -----------------------------
    State st[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        st[v].lx = lds_startL[loff + v];
        st[v].s = lds_startS[loff + v];
        if (w > 0) st[v] = seg_apply<DOM>(st[v], pre[v]);
    }
    constexpr int OW = (SIGNED && LOG_OUT) ? 2 : 1; // floats per output element
    float *op = p.out + OW * ubase;
    const bool full = chan_ok && t0 + T <= p.n;
    uint32_t swx[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) swx[v] = fold_state_sign<DOM>(sw[v], st[v]);
#pragma unroll
    for (int k = 0; k < T; ++k) {
        if constexpr (SIGNED && LOG_OUT) {
            // complex output: (re, im) pairs, two floats per element
            float o[2 * VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) emit_clog(st[v], Av[k][v], Mv[k][v], swx[v], sm[v], k, o[2 * v], o[2 * v + 1]);
            if (full || (chan_ok && t0 + k < p.n)) store_vec(op + 2 * ((int64_t)k * p.D + moff), o, p.stream_out != 0);
        } else {
            float o[VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) o[v] = emit<DOM, LOG_OUT>(st[v], Av[k][v], Mv[k][v], swx[v], k);
            if (full || (chan_ok && t0 + k < p.n)) store_vec(op + (int64_t)k * p.D + moff, o, p.stream_out != 0);
        }
        if (SB) __builtin_amdgcn_sched_barrier(0);
    }
    HS_STAMP(7);
}

// ---- host side ------------------------------------------------------------------------------------

#ifdef HS_TRACE
unsigned long long *g_trace = nullptr;
#endif

// MI355X: 256 MB of memory-side cache; an output up to three quarters of it is left to be cached
constexpr int64_t kLastLevelCacheBytes = 192ll << 20;

struct BndPlan {
    int vec, T, NW, G, CH, variant;
    bool ticketless;
    int dp_shift, bpack; // bpack > 1: narrow rows, the channels of bpack batch items share a 64-lane column
    int cols_per_b, ncols, nchunks, ngroups;
    uint32_t ntiles;
    int SG;             // > 0: groups per super-group (second carry level)
    size_t off_agg, off_gagg, off_state, records; // in records, relative to kRecordBase
};

#ifdef HS_TUNING
// tuning variants (development builds; signed float32, or bf16 logs in / logs out with -DHS_TUNING_BF16LOG):
// ID, VEC, T, NW, G, MINW, SB
#define HS_VARIANTS(X) \
    X(1, 4, 4, 16, 4, 4, true) X(2, 4, 8, 8, 4, 4, true) X(3, 4, 16, 4, 4, 2, true) X(4, 2, 8, 16, 4, 4, true) \
    X(5, 2, 16, 8, 4, 4, true) X(6, 2, 32, 4, 4, 2, true) X(7, 1, 16, 16, 4, 8, true) X(8, 1, 32, 8, 4, 4, true) \
    X(9, 4, 8, 16, 4, 2, true) X(10, 2, 16, 16, 4, 2, true) X(11, 4, 4, 8, 4, 4, true) X(12, 4, 2, 16, 4, 8, true) \
    X(13, 1, 8, 16, 4, 8, true) X(14, 2, 4, 16, 4, 8, true) X(15, 1, 16, 8, 4, 8, true) X(16, 2, 8, 8, 4, 8, true) \
    X(17, 1, 32, 4, 4, 4, true) X(18, 1, 16, 4, 4, 8, true) X(19, 1, 8, 8, 4, 8, true) X(20, 1, 32, 8, 8, 4, true) \
    X(21, 1, 32, 8, 2, 4, true) X(22, 1, 16, 8, 8, 8, true) X(23, 1, 32, 4, 8, 4, true) X(24, 1, 32, 2, 8, 4, true)
constexpr int kVariants[][4] = {{0, 0, 0, 0},
#define X(ID, V, T_, NW_, G_, MW, SB_) {V, T_, NW_, G_},
                                HS_VARIANTS(X)
#undef X
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);
#endif

BndPlan make_plan(const ScanCall &c)
{
    BndPlan pl;
    // One channel per lane, 32 steps per wave, 8 waves (tile = 64 channels x 256 steps, <= 128 VGPRs, two
    // workgroups per CU) measured best on MI355X among the shapes tried, for float32 and for bf16 storage
    // (two bf16 channels per lane, which keeps a wave's reads at 256 contiguous bytes, measured 8 % slower).
    pl.vec = 1;
    pl.T = 32;
    pl.NW = 8;
    pl.G = 4;
    if (c.is_signed && c.log_out) {
        // complex output: the signed log-domain emit needs more registers per element; 16 steps per wave
        // and 16 waves keep the tile the same and the kernel free of spills
        pl.T = 16;
        pl.NW = 16;
    } else if (c.n <= 128) {
        // short sequences: no more waves than have steps to work on
        pl.NW = c.n <= 32 ? 1 : (c.n <= 64 ? 2 : 4);
    }
    pl.variant = 0;
#ifdef HS_TUNING
    if (const char *ev = getenv("HEINSEN_BND_VARIANT")) {
        pl.variant = atoi(ev);
#ifdef HS_TUNING_BF16LOG
        const bool tuned_mode = !c.is_signed && c.bf16 && c.log_in && c.log_out;
#else
        const bool tuned_mode = c.is_signed && !c.log_out && !c.bf16;
#endif
        if (pl.variant >= 1 && pl.variant < kNumVariants && tuned_mode && c.D % 4 == 0) {
            pl.vec = kVariants[pl.variant][0];
            pl.T = kVariants[pl.variant][1];
            pl.NW = kVariants[pl.variant][2];
            pl.G = kVariants[pl.variant][3];
        } else {
            pl.variant = 0;
        }
    }
#endif
    pl.CH = 64 * pl.vec;
    pl.cols_per_b = (int)ceil_div(c.D, pl.CH);
    pl.ncols = (int)(c.B * pl.cols_per_b);

    pl.dp_shift = 6;
    pl.bpack = 1;
    if (c.D <= 32 && c.B > 1 && pl.variant == 0) {
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
    if (pl.variant == 0 && pl.NW == 8 && pl.T == 32 && !(c.log_in && c.log_out)) {
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
    pl.nchunks = (int)ceil_div(c.n, (int64_t)pl.NW * pl.T);
    pl.ngroups = (int)ceil_div(pl.nchunks, pl.G);
    pl.ntiles = (uint32_t)pl.ncols * (uint32_t)pl.nchunks;
    pl.off_agg = 0;
    pl.off_gagg = (size_t)pl.ntiles * 2 * pl.CH;
    pl.off_state = pl.off_gagg + (pl.SG ? (size_t)pl.ngroups * pl.ncols * 2 * pl.CH : 0);
    pl.records = pl.off_state + (size_t)(pl.SG ? ceil_div(pl.ngroups, pl.SG) + 1 : pl.ngroups) * pl.ncols * pl.CH;
    pl.ticketless = pl.nchunks == 1 && c.n <= 64; // short single-tile columns: no records, no tickets
    if (pl.ticketless) pl.records = 0;
    return pl;
}

template <int DOM, bool LOG_IN, bool LOG_OUT, typename InT>
hipError_t launch_mode(const ScanCall &c, const BndPlan &pl, rec_t *records, LaunchTag tag)
{
    constexpr bool SIGNED = DOM == kSigned;
    BndParams p;
    p.a = c.a;
    p.b = c.b;
    p.x0 = c.x0;
    p.out = c.out;
    p.D = c.D;
    p.n = c.n;
    p.x0_stride = c.x0_scalar ? 0 : 1;
    p.stream_out = (c.B * c.D * c.n * ((SIGNED && LOG_OUT) ? 8 : 4) > kLastLevelCacheBytes) ? 1 : 0;
    p.cols_per_b = pl.cols_per_b;
    p.B = c.B;
    p.dp_shift = pl.dp_shift;
    p.bpack = pl.bpack;
    p.ncols = pl.ncols;
    p.nchunks = pl.nchunks;
    p.ntiles = pl.ntiles;
    p.epoch = tag.epoch;
    p.ticket_base = tag.ticket_base;
    p.from_header = tag.from_header ? 1 : 0;
    p.ticket = records; // null when the launch needs no carries
    p.agg = records ? records + kRecordBase + pl.off_agg : nullptr;
    p.state = records ? records + kRecordBase + pl.off_state : nullptr;
    p.gagg = records ? records + kRecordBase + pl.off_gagg : nullptr;
#ifdef HS_TRACE
    if (!g_trace) (void)hipMalloc(&g_trace, (size_t)(1u << 20) * 8 * sizeof(unsigned long long));
    p.trace = g_trace;
#endif
    dim3 grid(pl.ntiles), block(pl.NW * 64);
#ifdef HS_TUNING
#ifdef HS_TUNING_BF16LOG
    constexpr bool kTunedMode = DOM == kPositive && LOG_IN && LOG_OUT && sizeof(InT) == 2;
#else
    constexpr bool kTunedMode = SIGNED && !LOG_OUT && sizeof(InT) == 4;
#endif
    if constexpr (kTunedMode) {
#define X(ID, V, T_, NW_, G_, MW, SB_)                                                                                 \
    if (pl.variant == ID) {                                                                                            \
        hipLaunchKernelGGL((heinsen_scan_bnd<DOM, LOG_IN, LOG_OUT, InT, V, T_, NW_, G_, MW, SB_>), grid, block, 0,  \
                           c.stream, p);                                                                               \
        return hipGetLastError();                                                                                      \
    }
        HS_VARIANTS(X)
#undef X
    }
#endif
    if constexpr (SIGNED && LOG_OUT) {
        if (pl.bpack > 1)
            hipLaunchKernelGGL((heinsen_scan_bnd<DOM, LOG_IN, LOG_OUT, InT, 1, 16, 16, 4, 4, true, true>), grid, block, 0, c.stream, p);
        else
            hipLaunchKernelGGL((heinsen_scan_bnd<DOM, LOG_IN, LOG_OUT, InT, 1, 16, 16, 4, 4, true>), grid, block, 0, c.stream, p);
    } else {
#define HS_BND(NW_, PACKB_) \
    hipLaunchKernelGGL((heinsen_scan_bnd<DOM, LOG_IN, LOG_OUT, InT, 1, 32, NW_, 4, 4, true, PACKB_>), grid, block, 0, c.stream, p)
        if constexpr (!(LOG_IN && LOG_OUT)) {
            if (pl.G == 8 || pl.SG > 0) {
#define HS_BND_CARRY(G_, SG_, PACKB_) \
    hipLaunchKernelGGL((heinsen_scan_bnd<DOM, LOG_IN, LOG_OUT, InT, 1, 32, 8, G_, 4, true, PACKB_, SG_>), grid, block, 0, c.stream, p)
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
            else HS_BND(8, false);
        }
#undef HS_BND
    }
    return hipGetLastError();
}

hipError_t launch_dispatch(const ScanCall &c, const BndPlan &pl, rec_t *records, LaunchTag tag)
{
    HS_DISPATCH_MODE(c, launch_mode, c, pl, records, tag);
}

} // namespace

ScratchNeed bnd_scratch(const ScanCall &c)
{
    BndPlan pl = make_plan(c);
    return ScratchNeed{pl.records, pl.ticketless ? 0u : pl.ntiles};
}

hipError_t bnd_launch(const ScanCall &c, unsigned long long *records, LaunchTag tag)
{
    BndPlan pl = make_plan(c);
    return launch_dispatch(c, pl, records, tag);
}

const char *bnd_kernel_name(const ScanCall &) { return "heinsen_scan_bnd"; }

#ifdef HS_TRACE
extern "C" int heinsen_debug_trace(unsigned long long *host, size_t ntiles)
{
    return (int)hipMemcpy(host, g_trace, ntiles * 8 * sizeof(unsigned long long), hipMemcpyDeviceToHost);
}
#endif

} // namespace hs
