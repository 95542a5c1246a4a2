// Channel-contiguous path: a, b, out are [B, n, D]; lanes own channels, time runs down the rows.
//
// A workgroup of NW waves owns CH = 64*VEC adjacent channels for NW*T consecutive time steps ("tile").
// Wave w of the workgroup scans steps [w*T, (w+1)*T) of the tile serially in each lane (one lane = VEC
// channels, loads and stores coalesced across lanes), keeping the T local segment summaries in
// registers.  Summaries of the waves are chained through LDS, summaries of the tiles of one channel
// column through global memory: tiles are grouped G at a time along the time axis, a tile folds the
// published summaries of the earlier tiles of its group (always in the same order, so results are
// bit-reproducible) onto the state at the start of the group, and the last tile of a group publishes
// the state at the start of the next.  Every element is read once and written once.
//
// What is computed is Sec. 4's expression applied by parts (Sec. 1, footnote on associativity); the
// arithmetic is in heinsen_math.hpp.
#include "heinsen_internal.hpp"
#include "heinsen_math.hpp"
#include <cstdlib>

namespace hs {
namespace {

constexpr int kGroup = 8; // tiles per group along time

struct BndParams {
    const void *a;
    const void *b;
    const float *x0;
    float *out;
    int64_t D, n;
    int x0_stride;     // 0: one x0 for all, 1: x0[b*D + d]
    int cols_per_b;    // ceil(D / CH)
    int ncols;         // B * cols_per_b
    int nchunks;       // ceil(n / (NW*T))
    uint32_t ntiles;   // ncols * nchunks
    uint32_t nflags;   // number of 32-bit words in the flag region (after the two counters)
    uint32_t *counters; // [0] ticket, [1] done
    uint32_t *agg_flag; // [ntiles]
    uint32_t *st_flag;  // [ngroups * ncols]
    float *agg_A;       // [ntiles * CH]
    float *agg_M;
    uint32_t *agg_S;    // bit0: sign of 2^A factor, bit1: sign of 2^M term
    float *st_L;        // [ngroups * ncols * CH] state at the start of a group
    uint32_t *st_S;
};

template <typename InT, int VEC>
__device__ __forceinline__ void load_vec(const InT *p, float (&v)[VEC])
{
    typedef InT vec_t __attribute__((ext_vector_type(VEC)));
    vec_t x = *reinterpret_cast<const vec_t *>(p);
#pragma unroll
    for (int i = 0; i < VEC; ++i) v[i] = widen(x[i]);
}
template <typename InT>
__device__ __forceinline__ void load_vec(const InT *p, float (&v)[1])
{
    v[0] = widen(*p);
}

template <int VEC>
__device__ __forceinline__ void store_vec(float *p, const float (&v)[VEC])
{
    typedef float vec_t __attribute__((ext_vector_type(VEC)));
    vec_t x;
#pragma unroll
    for (int i = 0; i < VEC; ++i) x[i] = v[i];
    *reinterpret_cast<vec_t *>(p) = x;
}
__device__ __forceinline__ void store_vec(float *p, const float (&v)[1]) { *p = v[0]; }

__device__ __forceinline__ uint32_t pack_signs(const Seg &g) { return (g.sA >> 31) | ((g.sM >> 31) << 1); }
__device__ __forceinline__ void unpack_signs(uint32_t s, Seg &g)
{
    g.sA = s << 31;
    g.sM = s << 30;
}

template <bool SIGNED, bool LOG_IN, bool LOG_OUT, typename InT, int VEC, int T, int NW, int MINW = 1>
__global__ __launch_bounds__(NW * 64, MINW) void heinsen_scan_bnd(BndParams p)
{
    constexpr int CH = 64 * VEC;
    static_assert(T <= 32, "one sign word per channel");
    __shared__ uint32_t s_tile;
    __shared__ uint32_t s_last;
    __shared__ float lds_A[NW][CH];
    __shared__ float lds_M[NW][CH];
    __shared__ uint32_t lds_S[NW][CH];
    __shared__ float lds_startL[CH];
    __shared__ uint32_t lds_startS[CH];

    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;

    // Tiles are handed out in start order, so every tile a workgroup may wait for (same column,
    // earlier chunk => smaller ticket) belongs to a workgroup that is already running.
    if (threadIdx.x == 0) s_tile = atomicAdd(&p.counters[0], 1u);
    __syncthreads();
    const uint32_t tile = s_tile;
    const int chunk = (int)(tile / (uint32_t)p.ncols);
    const int col = (int)(tile % (uint32_t)p.ncols);
    const int bidx = col / p.cols_per_b;
    const int cg = col % p.cols_per_b;

    const int64_t d0 = (int64_t)cg * CH + (int64_t)lane * VEC;
    const bool chan_ok = d0 < p.D; // D is a multiple of VEC, so the whole vector is in range
    const int64_t t0 = (int64_t)chunk * (NW * T) + (int64_t)w * T;
    const int64_t base = ((int64_t)bidx * p.n + t0) * p.D + d0;
    const InT *ap = reinterpret_cast<const InT *>(p.a) + base;
    const InT *bp = reinterpret_cast<const InT *>(p.b) + base;

    // ---- load: the lane's T x VEC inputs -------------------------------------------------------
    float Av[T][VEC], Mv[T][VEC];
    const float id_a = LOG_IN ? 0.0f : 1.0f;       // a = 1, b = 0 leave the state unchanged
    const float id_b = LOG_IN ? -INFINITY : 0.0f;
    if (chan_ok && t0 + T <= p.n) {
#pragma unroll
        for (int k = 0; k < T; ++k) {
            load_vec<InT>(ap + (int64_t)k * p.D, Av[k]);
            load_vec<InT>(bp + (int64_t)k * p.D, Mv[k]);
        }
    } else {
#pragma unroll
        for (int k = 0; k < T; ++k) {
            if (chan_ok && t0 + k < p.n) {
                load_vec<InT>(ap + (int64_t)k * p.D, Av[k]);
                load_vec<InT>(bp + (int64_t)k * p.D, Mv[k]);
            } else {
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    Av[k][v] = id_a;
                    Mv[k][v] = id_b;
                }
            }
        }
    }

    // ---- encode + serial scan in each lane; Av/Mv become the per-element records (see stash) --------
    uint32_t sw[VEC];
    Seg run[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) sw[v] = 0u;
#pragma unroll
    for (int k = 0; k < T; ++k) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            float la, lb;
            uint32_t sa, sb;
            encode<SIGNED, LOG_IN>(Av[k][v], la, sa);
            encode<SIGNED, LOG_IN>(Mv[k][v], lb, sb);
            if (k == 0) {
                run[v] = Seg{la, lb, sa, sb};
            } else {
                uint32_t sp = SIGNED ? (run[v].sM ^ sa) : 0u;
                slae<SIGNED>(run[v].M + la, sp, lb, sb, run[v].M, run[v].sM);
                run[v].A += la;
                if (SIGNED) run[v].sA ^= sa;
            }
            stash<SIGNED, LOG_OUT>(run[v], k, Av[k][v], Mv[k][v], sw[v]);
        }
    }

    // ---- chain the waves of the workgroup through LDS ------------------------------------------
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        lds_A[w][lane * VEC + v] = run[v].A;
        lds_M[w][lane * VEC + v] = run[v].M;
        if (SIGNED) lds_S[w][lane * VEC + v] = pack_signs(run[v]);
    }
    __syncthreads();

    // wave w folds the summaries of waves 0..w-1 (its exclusive prefix inside the tile);
    // wave 0 instead folds all NW of them: the summary of the whole tile.
    Seg pre[VEC];
    {
        const int cnt = (w == 0) ? NW : w;
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            Seg g;
            g.A = lds_A[0][lane * VEC + v];
            g.M = lds_M[0][lane * VEC + v];
            g.sA = g.sM = 0u;
            if (SIGNED) unpack_signs(lds_S[0][lane * VEC + v], g);
            for (int j = 1; j < cnt; ++j) {
                Seg h;
                h.A = lds_A[j][lane * VEC + v];
                h.M = lds_M[j][lane * VEC + v];
                h.sA = h.sM = 0u;
                if (SIGNED) unpack_signs(lds_S[j][lane * VEC + v], h);
                g = seg_combine<SIGNED>(g, h);
            }
            pre[v] = g;
        }
    }

    // ---- wave 0: publish the tile summary, obtain the state at the start of the tile -------------
    if (w == 0) {
        const int g = chunk / kGroup;
        const int r = chunk % kGroup;
        const bool more = chunk + 1 < p.nchunks;
        const size_t my = (size_t)tile * CH + (size_t)lane * VEC;
        if (more && r < kGroup - 1) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                pub_f(&p.agg_A[my + v], pre[v].A);
                pub_f(&p.agg_M[my + v], pre[v].M);
                if (SIGNED) pub_u(&p.agg_S[my + v], pack_signs(pre[v]));
            }
            order_release();
            if (lane == 0) __hip_atomic_store(&p.agg_flag[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }

        // wait for the r earlier tiles of the group (lanes 0..r-1) and for the group's start state
        // (lane 63), all polls in flight together
        {
            const bool need_agg = lane < r;
            const bool need_st = (lane == 63) && (g > 0);
            const uint32_t *fp = need_agg ? &p.agg_flag[(size_t)(g * kGroup + lane) * p.ncols + col]
                                          : &p.st_flag[(size_t)g * p.ncols + col];
            if (need_agg || need_st) {
                while (__hip_atomic_load(fp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u)
                    __builtin_amdgcn_s_sleep(2);
            }
            order_acquire();
        }

        State st[VEC];
        if (g == 0) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                float x0v = LOG_IN ? 0.0f : 1.0f;
                if (chan_ok) x0v = p.x0[p.x0_stride ? ((int64_t)bidx * p.D + d0 + v) : 0];
                encode<SIGNED, LOG_IN>(x0v, st[v].lx, st[v].s);
            }
        } else {
            const size_t si = ((size_t)g * p.ncols + col) * CH + (size_t)lane * VEC;
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                st[v].lx = get_f(&p.st_L[si + v]);
                st[v].s = SIGNED ? get_u(&p.st_S[si + v]) : 0u;
            }
        }
        if (r > 0) {
            // all payload loads first (independent), then the fold in tile order
            float fA[kGroup - 1][VEC], fM[kGroup - 1][VEC];
            uint32_t fS[kGroup - 1][VEC];
#pragma unroll
            for (int j = 0; j < kGroup - 1; ++j) {
                if (j < r) {
                    const size_t ti = ((size_t)(g * kGroup + j) * p.ncols + col) * CH + (size_t)lane * VEC;
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        fA[j][v] = get_f(&p.agg_A[ti + v]);
                        fM[j][v] = get_f(&p.agg_M[ti + v]);
                        fS[j][v] = SIGNED ? get_u(&p.agg_S[ti + v]) : 0u;
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < kGroup - 1; ++j) {
                if (j < r) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        Seg h;
                        h.A = fA[j][v];
                        h.M = fM[j][v];
                        h.sA = h.sM = 0u;
                        if (SIGNED) unpack_signs(fS[j][v], h);
                        st[v] = seg_apply<SIGNED>(st[v], h);
                    }
                }
            }
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            lds_startL[lane * VEC + v] = st[v].lx;
            lds_startS[lane * VEC + v] = st[v].s;
        }
        // last tile of a group: the state after this tile starts the next group
        if (more && r == kGroup - 1) {
            const size_t si = ((size_t)(g + 1) * p.ncols + col) * CH + (size_t)lane * VEC;
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                State nx = seg_apply<SIGNED>(st[v], pre[v]);
                pub_f(&p.st_L[si + v], nx.lx);
                if (SIGNED) pub_u(&p.st_S[si + v], nx.s);
            }
            order_release();
            if (lane == 0)
                __hip_atomic_store(&p.st_flag[(size_t)(g + 1) * p.ncols + col], 1u, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __syncthreads();

    // ---- state at the start of this wave's steps, then every element -----------------------------
    State st[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        st[v].lx = lds_startL[lane * VEC + v];
        st[v].s = lds_startS[lane * VEC + v];
        if (w > 0) st[v] = seg_apply<SIGNED>(st[v], pre[v]);
    }
    float *op = p.out + base;
    const bool full = chan_ok && t0 + T <= p.n;
    uint32_t swx[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) swx[v] = fold_state_sign<SIGNED>(sw[v], st[v]);
#pragma unroll
    for (int k = 0; k < T; ++k) {
        float o[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) o[v] = emit<SIGNED, LOG_OUT>(st[v], Av[k][v], Mv[k][v], swx[v], k);
        if (full || (chan_ok && t0 + k < p.n)) store_vec(op + (int64_t)k * p.D, o);
    }

    // ---- the last workgroup to finish restores the zeros in the flag region ------------------------
    __syncthreads(); // wave 0's polls are over before this workgroup reports completion
    if (threadIdx.x == 0) {
        order_release();
        uint32_t prev = __hip_atomic_fetch_add(&p.counters[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = (prev == p.ntiles - 1u) ? 1u : 0u;
    }
    __syncthreads();
    if (s_last) {
        for (uint32_t i = threadIdx.x; i < p.nflags; i += NW * 64) p.agg_flag[i] = 0u; // agg_flag and st_flag are contiguous
        if (threadIdx.x == 0) {
            p.counters[0] = 0u;
            p.counters[1] = 0u;
        }
    }
}

// ---- host side ------------------------------------------------------------------------------------

struct BndPlan {
    int vec, T, NW, CH, variant;
    int cols_per_b, ncols, nchunks, ngroups;
    uint32_t ntiles;
    size_t off_agg_flag, off_st_flag, flag_bytes;                      // inside the flag buffer
    size_t off_agg_A, off_agg_M, off_agg_S, off_st_L, off_st_S, data_bytes; // inside the data buffer
};

BndPlan make_plan(const ScanCall &c)
{
    BndPlan pl;
    const size_t in_sz = c.bf16 ? 2 : 4;
    auto aligned = [](const void *ptr, size_t a) { return (reinterpret_cast<uintptr_t>(ptr) % a) == 0; };
    pl.vec = 1;
    if (c.D % 2 == 0 && aligned(c.a, 2 * in_sz) && aligned(c.b, 2 * in_sz) && aligned(c.out, 8)) pl.vec = 2;
    pl.T = 16;
    pl.NW = 8;
    pl.variant = 0;
    if (const char *ev = getenv("HEINSEN_BND_VARIANT")) {
        pl.variant = atoi(ev);
        static const int tab[][3] = {{0, 0, 0}, {2, 16, 8}, {2, 16, 4}, {2, 8, 8}, {4, 8, 8}, {4, 8, 4}, {1, 32, 4}, {2, 32, 4}, {1, 16, 8}, {4, 4, 16}, {2, 8, 16}};
        if (pl.variant >= 1 && pl.variant <= 10 && c.is_signed && !c.bf16 && c.D % 4 == 0) {
            pl.vec = tab[pl.variant][0];
            pl.T = tab[pl.variant][1];
            pl.NW = tab[pl.variant][2];
        } else {
            pl.variant = 0;
        }
    }
    pl.CH = 64 * pl.vec;
    pl.cols_per_b = (int)ceil_div(c.D, pl.CH);
    pl.ncols = (int)(c.B * pl.cols_per_b);
    pl.nchunks = (int)ceil_div(c.n, (int64_t)pl.NW * pl.T);
    pl.ngroups = (int)ceil_div(pl.nchunks, kGroup);
    pl.ntiles = (uint32_t)pl.ncols * (uint32_t)pl.nchunks;
    size_t off = 64; // counters
    pl.off_agg_flag = off;
    off += (size_t)pl.ntiles * 4;
    pl.off_st_flag = off;
    off += (size_t)pl.ngroups * pl.ncols * 4;
    pl.flag_bytes = align_up(off, 256);
    off = 0;
    const size_t agg = (size_t)pl.ntiles * pl.CH * 4;
    const size_t stt = (size_t)pl.ngroups * pl.ncols * pl.CH * 4;
    pl.off_agg_A = off; off += align_up(agg, 256);
    pl.off_agg_M = off; off += align_up(agg, 256);
    pl.off_agg_S = off; off += align_up(agg, 256);
    pl.off_st_L = off; off += align_up(stt, 256);
    pl.off_st_S = off; off += align_up(stt, 256);
    pl.data_bytes = off;
    return pl;
}

template <bool SIGNED, bool LOG_IN, bool LOG_OUT, typename InT>
hipError_t launch_mode(const ScanCall &c, const BndPlan &pl, char *flags, char *data)
{
    BndParams p;
    p.a = c.a;
    p.b = c.b;
    p.x0 = c.x0;
    p.out = c.out;
    p.D = c.D;
    p.n = c.n;
    p.x0_stride = c.x0_scalar ? 0 : 1;
    p.cols_per_b = pl.cols_per_b;
    p.ncols = pl.ncols;
    p.nchunks = pl.nchunks;
    p.ntiles = pl.ntiles;
    p.nflags = (uint32_t)((pl.off_st_flag - pl.off_agg_flag) / 4 + (size_t)pl.ngroups * pl.ncols);
    p.counters = reinterpret_cast<uint32_t *>(flags);
    p.agg_flag = reinterpret_cast<uint32_t *>(flags + pl.off_agg_flag);
    p.st_flag = reinterpret_cast<uint32_t *>(flags + pl.off_st_flag);
    p.agg_A = reinterpret_cast<float *>(data + pl.off_agg_A);
    p.agg_M = reinterpret_cast<float *>(data + pl.off_agg_M);
    p.agg_S = reinterpret_cast<uint32_t *>(data + pl.off_agg_S);
    p.st_L = reinterpret_cast<float *>(data + pl.off_st_L);
    p.st_S = reinterpret_cast<uint32_t *>(data + pl.off_st_S);
    dim3 grid(pl.ntiles), block(pl.NW * 64);
    if constexpr (SIGNED && sizeof(InT) == 4) {
#define HS_VAR(ID, V, T_, NW_, MW)                                                                                 \
    if (pl.variant == ID) {                                                                                        \
        hipLaunchKernelGGL((heinsen_scan_bnd<SIGNED, LOG_IN, LOG_OUT, InT, V, T_, NW_, MW>), grid, block, 0, c.stream, p); \
        return hipGetLastError();                                                                                  \
    }
        HS_VAR(1, 2, 16, 8, 2)
        HS_VAR(2, 2, 16, 4, 2)
        HS_VAR(3, 2, 8, 8, 2)
        HS_VAR(4, 4, 8, 8, 2)
        HS_VAR(5, 4, 8, 4, 2)
        HS_VAR(6, 1, 32, 4, 2)
        HS_VAR(7, 2, 32, 4, 1)
        HS_VAR(8, 1, 16, 8, 2)
        HS_VAR(9, 4, 4, 16, 4)
        HS_VAR(10, 2, 8, 16, 4)
#undef HS_VAR
    }
    if (pl.vec == 2)
        hipLaunchKernelGGL((heinsen_scan_bnd<SIGNED, LOG_IN, LOG_OUT, InT, 2, 16, 8>), grid, block, 0, c.stream, p);
    else
        hipLaunchKernelGGL((heinsen_scan_bnd<SIGNED, LOG_IN, LOG_OUT, InT, 1, 16, 8>), grid, block, 0, c.stream, p);
    return hipGetLastError();
}

hipError_t launch_dispatch(const ScanCall &c, const BndPlan &pl, char *flags, char *data)
{
    HS_DISPATCH_MODE(c, launch_mode, c, pl, flags, data);
}

} // namespace

ScratchNeed bnd_scratch(const ScanCall &c)
{
    BndPlan pl = make_plan(c);
    return ScratchNeed{pl.flag_bytes, pl.data_bytes};
}

hipError_t bnd_launch(const ScanCall &c, void *flags, void *data)
{
    BndPlan pl = make_plan(c);
    return launch_dispatch(c, pl, static_cast<char *>(flags), static_cast<char *>(data));
}

const char *bnd_kernel_name(const ScanCall &) { return "heinsen_scan_bnd"; }

} // namespace hs
