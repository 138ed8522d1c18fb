// The ring kernels: vector sweeps (scaling sweep, band mat-vec) and bf16 matrix sweeps (output map / dV, final
// sweeps) on a skewed ring of tiles in LDS.
#pragma once
#include "ska_common.h"

namespace {

// ------------------------------------------------------------------ vector sweeps
// Scaling sweep (M_LSE, M_LSE_FIRST) and band mat-vec (M_MATVEC): the result is one scalar per
// owner index, so the only state a wavefront carries is FR owner fragments and FR
// partial sums.  Wavefront w owns rows [o_blk + 32 FR w, +32 FR) and needs other-side
// tiles kbase + FR w ... kend + FR w: the same count S for every wavefront, shifted by
// FR per wavefront.  The tiles therefore go through an LDS ring with that skew: at
// step s wavefront w works on tile kbase + s + FR w, so all wavefronts are busy in
// every step, and one new tile enters the ring per step (one barrier per step).
template <typename T, int D, int MODE, int FR> struct VRing {
    using TL = Tile<T, D>;
    static constexpr int LEAD = FR * (NWAVES - 1);          // tiles between first and last wavefront
    static constexpr int NSLOT = (LEAD + 2 <= 8) ? 8 : 16;  // power of two >= LEAD + 2
    // tile rows in LDS: bf16 rows carry 16 bytes of padding (the 32 rows an MFMA operand
    // read touches then fall on distinct banks, and the chunks of one row sit at fixed
    // distances: one address register per step); fp32 rows are padded by four floats
    static constexpr int ROWB = TL::IS_BF16 ? D * 2 + 16 : f32_row_floats<D>() * 4;
    static constexpr int OFF_VY = 32 * ROWB;
    static constexpr int OFF_VW = OFF_VY + TT * 4;
    static constexpr int SLOT = OFF_VW + TT * 4;
    static constexpr int BYTES = NSLOT * SLOT;
};

// One block of owner rows (logical block lb of the launch) of a vector sweep; the whole workgroup
// calls it.  smem: the ring (VRing::BYTES), red: NWAVES floats of LDS.
// COH: the potentials (the only data one block of a chain hands to another) are read and written
// with accesses that are coherent across the XCDs' L2 caches.
template <bool COH> __device__ __forceinline__ float ld_pot(const float *p)
{
    if constexpr (COH) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else return *p;
}
template <bool COH> __device__ __forceinline__ void st_pot(float *p, float v)
{
    if constexpr (COH) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *p = v;
}

template <typename T, int D, int MODE, int FR, bool COH = false>
__device__ __forceinline__ void vsweep_block(const SweepArgs &a, const int lb, unsigned char *smem, float *red)
{
    using TL = Tile<T, D>;
    using RG = VRing<T, D, MODE, FR>;
    constexpr bool PRE = (sizeof(T) == 2);   // bf16 storage: the score operand is prescaled, c2 == 1
    constexpr int BM = NWAVES * FR * 32;
    static_assert(MODE == M_LSE || MODE == M_MATVEC || MODE == M_LSE_FIRST, "vector sweeps only");
    // The very first half-step has no previous iterate to take a stabiliser from: it keeps a
    // running maximum per lane and fragment instead (exact for any scores), and the owner-side
    // vector xs, when given, only carries the marks of inactive tokens.
    constexpr bool FIRST = (MODE == M_LSE_FIRST);

    const int n = lb / a.nbp;
    const int o_blk = (lb % a.nbp) * BM;

    // the wavefront index is uniform: keep it (and all tile bookkeeping) in scalar registers
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 31, h = lane >> 5;
    const int L = a.L, W = a.W;
    const Lens ln = problem_lens(a, n);
    const int Lt = ln.Lt, Le = ln.Le;
    if (o_blk >= Le) {
        zero_block<T, D, BM>(a, n, o_blk, false, true);
        return;
    }
    const long moff = (long)n * L * D;
    const T *Xb = reinterpret_cast<const T *>(a.X) + moff;
    const T *Yb = reinterpret_cast<const T *>(a.Y) + moff;
    const float *ytp = a.yt.p + n * a.yt.stride;
    const float *xsp = (FIRST && !a.xs.p) ? nullptr : a.xs.p + n * a.xs.stride;
    const float *wp = (MODE == M_MATVEC) ? a.w.p + n * a.w.stride : nullptr;


    // stabiliser input first, so that waiting for it waits for nothing else
    static_assert(BM <= NTHREADS, "one owner-side potential per thread");
    float mraw = FIRST ? 0.f : ld_pot<COH>(xsp + min(o_blk + min(tid, BM - 1), Le - 1));   // clamped repeats are harmless
    float mblk = 0.f, m2 = 0.f;
    OwnerFrag<T, D> xf[FR];
    int o_frag[FR];
    float sum[FR], mx[FR];
#pragma unroll
    for (int f = 0; f < FR; ++f) {
        o_frag[f] = o_blk + (wave * FR + f) * 32;
        xf[f].load(Xb, min(o_frag[f] + c, Le - 1), Le, h);   // clamped: rows beyond Le are written as zeros
        sum[f] = 0.f;
        mx[f] = -INFINITY;
    }

    // floor((o_blk - W) / 32) and floor((o_blk + 32 FR - 1 + W) / 32); W <= L so no overflow
    const int kbase = (o_blk - W) >= 0 ? (o_blk - W) / TT : -((W - o_blk + TT - 1) / TT);
    const int kend = (o_blk + 32 * FR - 1 + W) / TT;
    const int S = kend - kbase + 1;
    const int klast = (Lt - 1) / TT;

    // One tile in flight between global memory and LDS.  A tile is a contiguous block of
    // memory, so a thread's 16-byte pieces sit at fixed byte offsets from the tile's start:
    // the start is a scalar, the offset one register, and a load needs no address arithmetic
    // beyond a clamp that keeps the pieces of a ragged last tile inside the matrix.  Loads
    // are unconditional (an index outside [0, klast] reads the nearest tile and is zeroed
    // before it is stored), so nothing stalls until the values are stored.
    constexpr int ROW_BYTES = D * (int)sizeof(T);
    constexpr int TILE_BYTES = TT * ROW_BYTES;
    unsigned goff[TL::CPT], soff[TL::CPT];   // piece offsets: in memory, in the LDS tile
#pragma unroll
    for (int q = 0; q < TL::CPT; ++q) {
        const int idx = min(tid + q * NTHREADS, TL::CHUNKS - 1);
        goff[q] = idx * 16;
        soff[q] = (idx / TL::CPR) * RG::ROWB + (idx % TL::CPR) * 16;
    }
    const unsigned vrow = tid & (TT - 1);
    struct Inflight {
        uint4 y[TL::CPT];
        float vy, vw;
        int rows;          // valid rows of the tile: 32 = whole, 0 = outside the matrix (uniform)
    };
    // A block whose every tile (the prefetched ones included) is a whole tile inside the matrix and
    // whose owner rows are all valid takes the loop with no clamps, no zeroing and no validity
    // tests (FAST): all but the blocks at the two ends of a sequence.
    const bool fast_blk = kbase >= 0 && (long)(kbase + S + RG::LEAD + 1) * TT <= Lt && o_blk + BM <= Le;
    const unsigned char *ybytes = reinterpret_cast<const unsigned char *>(Yb);
    const unsigned char *ytbytes = reinterpret_cast<const unsigned char *>(ytp) + vrow * 4;
    const unsigned char *wbytes = (MODE == M_MATVEC) ? reinterpret_cast<const unsigned char *>(wp) + vrow * 4 : nullptr;
    auto g_load_fast = [&](Inflight &g, int k) {   // 0 <= k, tile k whole
        g.rows = TT;
        const unsigned char *tb = ybytes + (long)k * TILE_BYTES;
#pragma unroll
        for (int q = 0; q < TL::CPT; ++q) g.y[q] = *reinterpret_cast<const uint4 *>(tb + goff[q]);
        g.vy = ld_pot<COH>(reinterpret_cast<const float *>(ytbytes + (long)k * (TT * 4)));
        g.vw = 0.f;
        if constexpr (MODE == M_MATVEC) g.vw = *reinterpret_cast<const float *>(wbytes + (long)k * (TT * 4));
    };
    auto s_store_fast = [&](Inflight &g, int j) {
        unsigned char *sl = smem + (j & (RG::NSLOT - 1)) * RG::SLOT;
#pragma unroll
        for (int q = 0; q < TL::CPT; ++q)
            if (TL::CHUNKS % NTHREADS == 0 || tid + q * NTHREADS < TL::CHUNKS)
                *reinterpret_cast<uint4 *>(sl + soff[q]) = g.y[q];
        if (tid < TT) {
            reinterpret_cast<float *>(sl + RG::OFF_VY)[tid] = fmaf(g.vy, LOG2E, m2);
            if constexpr (MODE == M_MATVEC) reinterpret_cast<float *>(sl + RG::OFF_VW)[tid] = g.vw;
        }
    };
    auto g_load = [&](Inflight &g, int k) {
        const int kc = min(max(k, 0), klast);
        const int rows = min(TT, Lt - kc * TT);   // >= 1
        g.rows = (k == kc) ? rows : 0;
        const unsigned char *tb = reinterpret_cast<const unsigned char *>(Yb) + (long)kc * TILE_BYTES;
        const unsigned lim = rows * ROW_BYTES - 16;
#pragma unroll
        for (int q = 0; q < TL::CPT; ++q) g.y[q] = *reinterpret_cast<const uint4 *>(tb + min(goff[q], lim));
        const unsigned vo = min(vrow, (unsigned)(rows - 1)) * 4;
        g.vy = ld_pot<COH>(reinterpret_cast<const float *>(reinterpret_cast<const unsigned char *>(ytp + kc * TT) + vo));
        g.vw = 0.f;
        if constexpr (MODE == M_MATVEC)
            g.vw = *reinterpret_cast<const float *>(reinterpret_cast<const unsigned char *>(wp + kc * TT) + vo);
    };
    auto s_store = [&](Inflight &g, int j) {  // j = tile index relative to kbase
        unsigned char *sl = smem + (j & (RG::NSLOT - 1)) * RG::SLOT;
        if (g.rows != TT) {   // uniform: ragged or absent tile
            const unsigned lim = g.rows * ROW_BYTES;
#pragma unroll
            for (int q = 0; q < TL::CPT; ++q)
                if (goff[q] >= lim) g.y[q] = make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int q = 0; q < TL::CPT; ++q)
            if (TL::CHUNKS % NTHREADS == 0 || tid + q * NTHREADS < TL::CHUNKS)
                *reinterpret_cast<uint4 *>(sl + soff[q]) = g.y[q];
        if (tid < TT) {
            const bool ok = (int)vrow < g.rows;
            reinterpret_cast<float *>(sl + RG::OFF_VY)[tid] = ok ? fmaf(g.vy, LOG2E, m2) : -INFINITY;
            if constexpr (MODE == M_MATVEC) reinterpret_cast<float *>(sl + RG::OFF_VW)[tid] = ok ? g.vw : 0.f;
        }
    };

    // fill the ring with the tiles of step 0.  Everything the prologue needs from memory is
    // requested before anything is waited for: owner rows (above), the first tiles, and the
    // owner-side potentials the stabiliser is taken from.
    Inflight fill[RG::LEAD + 1];
#pragma unroll
    for (int j = 0; j <= RG::LEAD; ++j) g_load(fill[j], kbase + j);
    if constexpr (!FIRST) {
        float m = mraw;
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) m = fmaxf(m, __shfl_xor(m, s));
        if (lane == 0) red[wave] = m;
        __syncthreads();
        mblk = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        if (mblk == -INFINITY) mblk = 0.f;   // a block of inactive tokens only
    }
    m2 = mblk * LOG2E;
#pragma unroll
    for (int j = 0; j <= RG::LEAD; ++j) s_store(fill[j], j);
    __syncthreads();
    Inflight nxt;
    // Which fragment uses the tile of step s, and whether that tile lies wholly inside its band,
    // depends on d = s - f alone: with r0 the offset of the band's first column inside tile kbase,
    // the tile of step s starts 32 d - W - r0 columns from the fragment's first row.  Used for
    // 0 <= d <= dhi, inside the band for ilo <= d <= ihi.
    const int r0 = o_blk - W - kbase * TT;   // 0 .. 31
    const int dhi = (31 + 2 * W + r0) / TT, ilo = (31 + r0 + TT - 1) / TT;
    const int ihi = (2 * W - 31 + r0) >= 0 ? (2 * W - 31 + r0) / TT : -1;
    bool fvalid[FR];
#pragma unroll
    for (int f = 0; f < FR; ++f) fvalid[f] = o_frag[f] < Le;

    auto run = [&](auto fast_c) {
        constexpr bool FAST = decltype(fast_c)::value;
        for (int s = 0; s < S; ++s) {
            // the next tile is requested in every step, also when no later step reads it (its
            // address is clamped, its ring slot is free): a load under a condition would make
            // the compiler wait for it at once instead of at the store below
            const int jnew = s + 1 + RG::LEAD;
            if constexpr (FAST) g_load_fast(nxt, kbase + jnew);
            else g_load(nxt, kbase + jnew);

            const int j = s + wave * FR;
            const int k = kbase + j;
            if (FAST || (k >= 0 && k <= klast)) {
                const unsigned char *sl = smem + (j & (RG::NSLOT - 1)) * RG::SLOT;
                const int t0 = k * TT;
                bool use[FR], interior[FR];
                f32x16 acc[FR];
                // the staged potentials are the MFMA's initial accumulator when the score operand
                // carries the scale already (bf16 storage: make_scores_operand)
                float yv[16];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float4 v4 = *reinterpret_cast<const float4 *>(sl + RG::OFF_VY + (8 * q + 4 * h) * 4);
                    yv[4 * q + 0] = v4.x; yv[4 * q + 1] = v4.y; yv[4 * q + 2] = v4.z; yv[4 * q + 3] = v4.w;
                }
#pragma unroll
                for (int f = 0; f < FR; ++f) {
                    // (t0 - o_frag[f] = 32 (s - f) - W - r0: the wavefront's skew cancels)
                    const int dd = s - f;
                    use[f] = fvalid[f] && dd >= 0 && dd <= dhi;
                    interior[f] = dd >= ilo && dd <= ihi;
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[f][r] = PRE ? yv[r] : 0.f;
                }
                ring_dot_multi<D, FR, RG::ROWB>(sl, xf, lane, acc);   // unconditional: an unused tile costs MFMA only

                float wv[MODE == M_MATVEC ? 16 : 1];
                if constexpr (MODE == M_MATVEC) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float4 w4 = *reinterpret_cast<const float4 *>(sl + RG::OFF_VW + (8 * q + 4 * h) * 4);
                        wv[4 * q + 0] = w4.x; wv[4 * q + 1] = w4.y; wv[4 * q + 2] = w4.z; wv[4 * q + 3] = w4.w;
                    }
                }
#pragma unroll
                for (int f = 0; f < FR; ++f) {
                    if (!use[f]) continue;
                    float e[16];
#pragma unroll
                    for (int r = 0; r < 16; ++r) e[r] = PRE ? acc[f][r] : fmaf(acc[f][r], a.c2, yv[r]);
                    if (!interior[f]) {
                        // keep (o, t) iff -W <= t - o <= W; with t = t0 + 4h + off_r (off_r a
                        // constant of register r) this is lo <= off_r <= lo + 2W for the lane's
                        // lo = o - W - t0 - 4h.  A tile crosses the lower edge, the upper edge
                        // or (narrow bands) both: one compare against a constant per edge.
                        const int lo = o_frag[f] + c - W - t0 - 4 * h;
                        const int hi = lo + 2 * W;
                        if (o_frag[f] + 31 - t0 > W) {
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                if (lo > 8 * (r >> 2) + (r & 3)) e[r] = -INFINITY;
                        }
                        if (t0 + TT - 1 - o_frag[f] > W) {
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                if (hi < 8 * (r >> 2) + (r & 3)) e[r] = -INFINITY;
                        }
                    }
                    if constexpr (FIRST) {
                        float tm = e[0];
#pragma unroll
                        for (int r = 1; r < 16; ++r) tm = fmaxf(tm, e[r]);
                        const float mn = fmaxf(mx[f], tm);
                        const float ms = (mn == -INFINITY) ? 0.f : mn;
                        float sacc = sum[f] * fast_exp2(mx[f] - ms);
#pragma unroll
                        for (int r = 0; r < 16; ++r) sacc += fast_exp2(e[r] - ms);
                        sum[f] = sacc;
                        mx[f] = mn;
                    } else {
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const float p = fast_exp2(e[r]);
                            if constexpr (MODE == M_MATVEC) sum[f] = fmaf(p, wv[r], sum[f]);
                            else sum[f] += p;
                        }
                    }
                }
            }
            if constexpr (FAST) s_store_fast(nxt, jnew);
            else s_store(nxt, jnew);
            __syncthreads();
        }
    };
    if (fast_blk) run(std::true_type{});
    else run(std::false_type{});

#pragma unroll
    for (int f = 0; f < FR; ++f) {
        const int o = o_frag[f] + c;
        if constexpr (FIRST) {
            // the two lanes of a row merge their (maximum, sum) pairs; then the spoke edge
            const float mo = __shfl_xor(mx[f], 32), so = __shfl_xor(sum[f], 32);
            float mn = fmaxf(mx[f], mo);
            float tot = sum[f] * fast_exp2(mx[f] - mn) + so * fast_exp2(mo - mn);
            if (a.dustbin) {   // spoke edge (o, dustbin): its score, other-side potential yt[L]
                const float sp2 = a.spoke_own.p ? a.spoke_own.p[n * a.spoke_own.stride + min(o, L - 1)] * LOG2E : a.sdb2;
                const float xd = sp2 + ytp[L] * LOG2E;
                const float m3 = fmaxf(mn, xd);
                tot = tot * fast_exp2(mn - m3) + fast_exp2(xd - m3);
                mn = m3;
            }
            if (h == 0 && o < L) {
                float r = 0.f;   // rows beyond the valid length
                if (o < Le) {
                    if ((xsp && xsp[o] == -INFINITY) || !(mn > -INFINITY)) {
                        r = -INFINITY;   // inactive token, or one without an active partner
                    } else {
                        r = -LN2 * (mn + fast_log2(tot));
                        if (a.olog.p) r += a.olog.p[n * a.olog.stride + o];
                    }
                }
                a.out_vec.p[n * a.out_vec.stride + o] = r;
            }
            continue;
        }
        float tot = sum[f] + __shfl_xor(sum[f], 32);
        if (a.dustbin) {   // spoke edge (o, dustbin element of the other side)
            const float sp2 = a.spoke_own.p ? a.spoke_own.p[n * a.spoke_own.stride + min(o, L - 1)] * LOG2E : a.sdb2;
            float ed = fast_exp2(sp2 + ytp[L] * LOG2E + m2);
            tot += (MODE == M_MATVEC) ? ed * wp[L] : ed;
        }
        if (h == 0 && o < L) {
            float r;
            if (o >= Le) {
                r = 0.f;   // rows beyond the valid length
            } else if (ld_pot<COH>(xsp + o) == -INFINITY) {
                r = (MODE == M_LSE) ? -INFINITY : 0.f;   // inactive token: stays so
            } else if (MODE == M_LSE && !(tot > 0.f && tot < INFINITY)) {
                // An active token has active partners (activity is settled by the two cold
                // half-steps), so an empty or infinite sum here is underflow or overflow: the
                // potentials inside this workgroup's 128 or 256 rows are spread further than the
                // fp32 exponent reaches under one stabiliser per workgroup.  Say so.
                r = __builtin_nanf("");
            } else if constexpr (MODE == M_LSE) {
                r = mblk - LN2 * fast_log2(tot);
                if (a.olog.p) r += a.olog.p[n * a.olog.stride + o];
            } else {
                float pre = a.pre.p ? a.pre.p[n * a.pre.stride + o] : 0.f;
                r = pre - fast_exp2((xsp[o] - mblk) * LOG2E) * tot;
                if (a.olog.p) r *= __expf(-a.olog.p[n * a.olog.stride + o]);
            }
            st_pot<COH>(a.out_vec.p + n * a.out_vec.stride + o, r);
        }
    }
}

// Workgroup -> block of a launch: each XCD (workgroups are dealt round-robin to the eight of them)
// takes a contiguous eighth of the block sequence, walked forwards or backwards.
__device__ __forceinline__ int xcd_block(int bx, int nb_total, int rev)
{
    const int chunk = (nb_total + 7) >> 3;
    return (bx & 7) * chunk + (rev ? chunk - 1 - (bx >> 3) : (bx >> 3));
}

template <typename T, int D, int MODE, int FR>
__global__ __launch_bounds__(NTHREADS) void vsweep_kernel(const SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ float red[NWAVES];
    // a.lead workgroups come first (a multiple of 8, so the XCD of a sweep block is unchanged): one
    // per problem for the dustbin element, started first so that it ends under the sweep
    if ((int)blockIdx.x < a.lead) {
        if ((int)blockIdx.x < a.nb_total / a.nbp) dustbin_element(a, blockIdx.x, MODE == M_MATVEC);
        return;
    }
    const int lb = xcd_block((int)blockIdx.x - a.lead, a.nb_total, a.rev);
    if (lb >= a.nb_total) return;
    vsweep_block<T, D, MODE, FR>(a, lb, smem, red);
}

// ------------------------------------------------------------------ several half-steps in one launch
// The half-steps of Eq. 1-2 depend on each other only through the band: block b of half-step h
// reads the potentials that blocks b - reach ... b + reach wrote in half-step h - 1.  One launch of
// co-resident workgroups can therefore run a whole chain of half-steps (the differentiable tail
// of Sec. 2.2, or the base solve and the tail together) with no kernel boundary and no grid-wide
// barrier in between: every block publishes the number of half-steps it has completed, and a
// block starts half-step h as soon as its neighbourhood has published h.  The same blocks run
// the same arithmetic as in separate launches (vsweep_block), so results are identical.
//   Workgroups are persistent (a cooperative launch sized to what the device holds at once; a
// workgroup takes every gridDim.x-th block of each half-step) and only ever wait for half-steps
// with a smaller index, so some workgroup can always proceed.  Waits are bounded all the same:
// a wait that runs out (another spinning kernel holding the device, a lost workgroup) stops
// waiting, writes NaN into its block of the result, which reaches every output it feeds, and
// goes on, so the kernel always ends.
//   Potentials cross XCDs, whose L2 caches are not coherent with each other: inside a chain they
// are read and written with agent-coherent accesses (vsweep_block<..., COH = true>), as are the
// counters; a block raises its counter after all its threads' stores have been acknowledged, and
// a waiting workgroup issues its reads after it has seen the counters.  (Fences at agent scope
// would do too, but they write back and invalidate the whole L2, operand tiles included.)
constexpr int MAXCHAIN = 96;
struct ChainArgs {
    SweepArgs base;            // sizes, scales, nbp / nb_total; X, Y, vectors are set per half-step
    const void *Q, *K;         // score operands: a row half-step owns Q and streams K, a column one the reverse
    float *UV;                 // potentials: slot s of problem n at UV + n us + s Lp
    long us;
    int Lp;
    const float *log_a, *log_b;
    const int *len_q, *len_k;
    int nsteps;
    int rev0;                  // direction of the first half-step's walk over the blocks (alternates)
    int *done;                 // [nb_total] half-steps completed per block, zero at launch
    unsigned spin_limit;       // polls of a wait before it gives up
    unsigned code[MAXCHAIN];   // per half-step: bit 0 row step; bits 8-15, 16-23, 24-31 slots of yt, xs, out
};

template <typename T, int D, int FR>
__global__ __launch_bounds__(NTHREADS) void vchain_kernel(const ChainArgs c)
{
    constexpr int BM = NWAVES * FR * 32;
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ float red[NWAVES];
    const int tid = threadIdx.x;
    const int nb = c.base.nb_total, nbp = c.base.nbp;
    const int reach = (c.base.W + BM - 1) / BM;   // blocks on either side whose potentials a block reads
    const int slots = ((nb + 7) >> 3) * 8;
    for (int hs = 0; hs < c.nsteps; ++hs) {
        const unsigned code = c.code[hs];
        const bool row = code & 1;
        SweepArgs a = c.base;
        a.X = row ? c.Q : c.K; a.Y = row ? c.K : c.Q;
        a.yt = Vec{c.UV + (long)((code >> 8) & 255) * c.Lp, c.us};
        a.xs = Vec{c.UV + (long)((code >> 16) & 255) * c.Lp, c.us};
        a.out_vec = VecOut{c.UV + (long)(code >> 24) * c.Lp, c.us};
        a.olog = Vec{row ? c.log_a : c.log_b, (long)c.Lp};
        a.len_own = row ? c.len_q : c.len_k; a.len_oth = row ? c.len_k : c.len_q;
        a.rev = (c.rev0 + hs) & 1;
        for (int bx = blockIdx.x; bx < slots; bx += gridDim.x) {
            const int lb = xcd_block(bx, nb, a.rev);
            if (lb >= nb) continue;   // (uniform)
            const int n = lb / nbp, bi = lb % nbp;
            const int lo = n * nbp + max(bi - reach, 0), hi = n * nbp + min(bi + reach, nbp - 1);
            // wait until the neighbourhood (this block included: it reads its own previous iterate)
            // has completed hs half-steps; then acquire what they released
            bool ok = true;
            if (hs > 0) {
                unsigned polls = 0;
                for (;;) {
                    bool mine = true;
                    for (int j = lo + tid; j <= hi; j += NTHREADS)
                        mine = mine && __hip_atomic_load(c.done + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= hs;
                    ok = __syncthreads_and(mine);   // (the counters' values have arrived: later loads are issued after them)
                    if (ok || ++polls > c.spin_limit) break;
                    __builtin_amdgcn_s_sleep(4);
                }
            }
            if (ok) {
                vsweep_block<T, D, M_LSE, FR, true>(a, lb, smem, red);
            } else {   // gave up: poison this block's result
                for (int i = tid; i < BM; i += NTHREADS)
                    if (bi * BM + i < a.L) st_pot<true>(a.out_vec.p + n * a.out_vec.stride + bi * BM + i, __builtin_nanf(""));
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's stores are acknowledged ...
            __syncthreads();                                   // ... and so are everybody's
            if (tid == 0) __hip_atomic_store(c.done + lb, hs + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// ------------------------------------------------------------------ matrix sweeps (bf16)
// Output map / dV (M_APPLY) and the one-reference final sweep (M_FINAL) on the same skewed
// ring: wavefront w owns 32 rows, four wavefronts per workgroup, the tile of step s for
// wavefront w is kbase + s + w.  A ring slot holds the other-side score rows, the second
// streamed matrix (payload for M_APPLY, the other-side factor of Z for M_FINAL), the staged
// potentials and, for M_FINAL, the other-side modifier pack.  Tiles are row-major in LDS
// with 16 bytes of padding per row.  The four rank-1 modifier terms of Prop. 2 are not VALU
// work: each side's pack is written as 16 bf16 columns (every fp32 value split into a high
// and a low bf16 part; per term the three products hi*hi, hi*lo, lo*hi, the owner side
// negated), which extend the Z product by one K = 16 MFMA step: its result is
// Z - sum_k po_k qt_k directly.  The other side's 32 bytes per row sit in the padding of the
// row in the two tiles.  The second product needs its streamed operand with the
// band index contiguous, which the transposing LDS read (ds_read_b64_tr_b16) delivers from
// the row-major tile: within 16 lanes, lane i receives element (i & 3) of the 8-byte pieces
// addressed by lanes (i >> 2) + 4 e, e = 0..3.
template <int D, int MODE, int FR> struct MRing {
    static constexpr int LEAD = FR * (NWAVES - 1);
    static constexpr int NSLOT = LEAD + 2;             // exactly what the skew needs (5 or 8): LDS decides
                                                       // how many workgroups share a CU
    static constexpr int ROWB = D * 2 + 16;
    static constexpr int TILE = 32 * ROWB;
    static constexpr int OFF_Y = 0;
    static constexpr int OFF_B = TILE;                 // payload (M_APPLY) or Z factor (M_FINAL)
    static constexpr int OFF_VY = 2 * TILE;
    static constexpr int OFF_PK = D * 2;               // M_FINAL: the 16 bytes of padding of a row of either
                                                       // tile hold half of the row's 16 pack columns
    static constexpr int SLOT = OFF_VY + TT * 4;
    static constexpr int BYTES = NSLOT * SLOT;
    static constexpr int CHUNKS = 32 * D * 2 / 16;     // 16-byte pieces of a tile in memory
    static constexpr int CPT = (CHUNKS + NTHREADS - 1) / NTHREADS;
    static constexpr int CPR = D * 2 / 16;
    static_assert(LEAD + 2 <= NSLOT, "ring too small for the skew");
};

template <int D, int MODE, int FR>
__global__ __launch_bounds__(NTHREADS) void msweep_kernel(const SweepArgs a)
{
    using T = __bf16;
    using RG = MRing<D, MODE, FR>;
    constexpr int BM = NWAVES * FR * 32, KS = D / 16;
    static_assert(MODE == M_APPLY || MODE == M_FINAL, "matrix sweeps only");

    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ float red[NWAVES];

    const int chunk = (a.nb_total + 7) >> 3;
    const int lb = (blockIdx.x & 7) * chunk + (a.rev ? chunk - 1 - (int)(blockIdx.x >> 3) : (int)(blockIdx.x >> 3));
    if (lb >= a.nb_total) return;
    const int n = lb / a.nbp;
    const int o_blk = (lb % a.nbp) * BM;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 31, h = lane >> 5;
    const int L = a.L, W = a.W;
    const Lens ln = problem_lens(a, n);
    const int Lt = ln.Lt, Le = ln.Le;
    if (o_blk >= Le) {
        zero_block<T, D, BM>(a, n, o_blk, true, false);
        return;
    }
    const long moff = (long)n * L * D;
    const T *Xb = reinterpret_cast<const T *>(a.X) + moff;
    const unsigned char *Yb = reinterpret_cast<const unsigned char *>(reinterpret_cast<const T *>(a.Y) + moff);
    const unsigned char *Bb = reinterpret_cast<const unsigned char *>(
        reinterpret_cast<const T *>(MODE == M_FINAL ? a.Bm : a.Pay) + moff);
    const float *ytp = a.yt.p + n * a.yt.stride;
    const float *xsp = a.xs.p + n * a.xs.stride;

    float mblk, m2;
    {
        float m = -INFINITY;
        for (int i = tid; i < BM; i += NTHREADS) m = fmaxf(m, xsp[min(o_blk + i, Le - 1)]);
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) m = fmaxf(m, __shfl_xor(m, s));
        if (lane == 0) red[wave] = m;
        __syncthreads();
        mblk = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        if (mblk == -INFINITY) mblk = 0.f;   // a block of inactive tokens only
    }
    m2 = mblk * LOG2E;

    // owner side: score rows, and for M_FINAL the owner factor of Z and the modifier pack.
    // Rows beyond Le are clamped: they compute garbage that is never stored.
    const int o_w = o_blk + wave * FR * 32;
    OwnerFrag<T, D> xf[FR], af[MODE == M_FINAL ? FR : 1];
    bf16x8 pob[FR];   // M_FINAL: this lane's half of the owner row's 16 pack columns
    f32x16 outm[FR][D / 32];
#pragma unroll
    for (int f = 0; f < FR; ++f) {
        const int oc = min(o_w + 32 * f + c, Le - 1);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            uint4 z = *reinterpret_cast<const uint4 *>(Xb + (long)oc * D + (2 * s + h) * 8);
            xf[f].v[s] = *reinterpret_cast<bf16x8 *>(&z);
            if constexpr (MODE == M_FINAL) {
                uint4 y = *reinterpret_cast<const uint4 *>(reinterpret_cast<const T *>(a.A) + moff + (long)oc * D +
                                                           (2 * s + h) * 8);
                af[f].v[s] = *reinterpret_cast<bf16x8 *>(&y);
            }
        }
        if constexpr (MODE == M_FINAL) {
            uint4 z = *reinterpret_cast<const uint4 *>(reinterpret_cast<const unsigned char *>(a.poB) +
                                                       ((long)n * a.ldp + oc) * 32 + h * 16);
            pob[f] = *reinterpret_cast<bf16x8 *>(&z);
        }
#pragma unroll
        for (int j = 0; j < D / 32; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) outm[f][j][r] = 0.f;
    }

    const int kbase = (o_blk - W) >= 0 ? (o_blk - W) / TT : -((W - o_blk + TT - 1) / TT);
    const int kend = (o_blk + 32 * FR - 1 + W) / TT;
    const int S = kend - kbase + 1;
    const int klast = (Lt - 1) / TT;

    // one tile pair in flight between global memory and LDS (plain arrays: a struct holding
    // them ends up in scratch memory)
    auto g_load = [&](uint4 (&gy)[RG::CPT], uint4 (&gb)[RG::CPT], float &gvy, uint4 &gpk, int k) {
#pragma unroll
        for (int q = 0; q < RG::CPT; ++q) {
            int idx = tid + q * NTHREADS;
            if (idx >= RG::CHUNKS) idx = RG::CHUNKS - 1;
            const unsigned row = (unsigned)min(max(k * TT + idx / RG::CPR, 0), Lt - 1);
            const unsigned off = row * (unsigned)(D * 2) + (unsigned)(idx % RG::CPR) * 16u;
            gy[q] = *reinterpret_cast<const uint4 *>(Yb + off);
            gb[q] = *reinterpret_cast<const uint4 *>(Bb + off);
        }
        const unsigned tv = (unsigned)min(max(k * TT + (tid & (TT - 1)), 0), Lt - 1);
        gvy = ytp[tv];
        if constexpr (MODE == M_FINAL) {
            // 64 pieces of 16 bytes per tile: every wavefront requests them (same addresses; a
            // request under a condition would cost a full wait), the first one stores them
            const unsigned tp = (unsigned)min(max(k * TT + ((tid & 63) >> 1), 0), Lt - 1);
            gpk = *reinterpret_cast<const uint4 *>(reinterpret_cast<const unsigned char *>(a.qtA) +
                                                   ((long)n * a.ldp + tp) * 32 + (tid & 1) * 16);
        }
    };
    // rows outside [0, Lt) keep whatever the clamped fetch brought: their potential is -inf,
    // so their plan entries are exactly zero and finite data times zero adds nothing
    auto s_store = [&](const uint4 (&gy)[RG::CPT], const uint4 (&gb)[RG::CPT], float gvy, uint4 gpk, int j, int k) {
        unsigned char *sl = smem + (j % RG::NSLOT) * RG::SLOT;
#pragma unroll
        for (int q = 0; q < RG::CPT; ++q) {
            const int idx = tid + q * NTHREADS;
            if (idx < RG::CHUNKS) {
                const int off = (idx / RG::CPR) * RG::ROWB + (idx % RG::CPR) * 16;
                *reinterpret_cast<uint4 *>(sl + RG::OFF_Y + off) = gy[q];
                *reinterpret_cast<uint4 *>(sl + RG::OFF_B + off) = gb[q];
            }
        }
        if (tid < TT) {
            const bool live = k >= 0 && k * TT + tid < Lt;
            reinterpret_cast<float *>(sl + RG::OFF_VY)[tid] = live ? fmaf(gvy, LOG2E, m2) : -INFINITY;
        }
        if constexpr (MODE == M_FINAL) {
            if (tid < 64)   // (rows outside the matrix: clamped data, multiplied by a zero plan entry)
                *reinterpret_cast<uint4 *>(sl + ((tid & 1) ? RG::OFF_B : RG::OFF_Y) + (tid >> 1) * RG::ROWB +
                                           RG::OFF_PK) = gpk;
        }
    };

    {
        uint4 fy[RG::LEAD + 1][RG::CPT], fb[RG::LEAD + 1][RG::CPT];
        float fvy[RG::LEAD + 1];
        uint4 fvq[RG::LEAD + 1];
#pragma unroll
        for (int j = 0; j <= RG::LEAD; ++j) g_load(fy[j], fb[j], fvy[j], fvq[j], kbase + j);
#pragma unroll
        for (int j = 0; j <= RG::LEAD; ++j) s_store(fy[j], fb[j], fvy[j], fvq[j], j, kbase + j);
    }
    __syncthreads();
    uint4 ny[RG::CPT], nb[RG::CPT];
    float nvy = 0.f;
    uint4 nvq = make_uint4(0, 0, 0, 0);

    // per-lane LDS offsets: fragment rows for the score / Z products, and the 8-byte pieces
    // this lane addresses in a transposing read (row 4h + (lane & 15) / 4 of a 16-row block,
    // columns 16 (lane / 16 & 1) + 4 (lane & 3), + 32 per output column tile)
    const int rd_a = c * RG::ROWB + h * 16;
    const int rd_t = (4 * h + ((lane & 15) >> 2)) * RG::ROWB + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
    typedef __bf16 bf16x4v __attribute__((ext_vector_type(4)));

    for (int s = 0; s < S; ++s) {
        const int jnew = s + 1 + RG::LEAD;
        const bool more = (s + 1 < S);
        if (more) g_load(ny, nb, nvy, nvq, kbase + jnew);

        const int j = s + wave * FR;
        const int k = kbase + j;
        if (k >= 0 && k <= klast) {
            const unsigned char *sl = smem + (j % RG::NSLOT) * RG::SLOT;
            const int t0 = k * TT;
            // this tile's fragments (score rows, Z rows) and staged potentials, read once for
            // all FR owner fragments
            bf16x8 yfr[KS], bfr[MODE == M_FINAL ? KS : 1];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                yfr[ks] = *reinterpret_cast<const bf16x8 *>(sl + RG::OFF_Y + rd_a + 32 * ks);
                if constexpr (MODE == M_FINAL)
                    bfr[ks] = *reinterpret_cast<const bf16x8 *>(sl + RG::OFF_B + rd_a + 32 * ks);
            }
            f32x16 yv;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float4 v4 = *reinterpret_cast<const float4 *>(sl + RG::OFF_VY + (8 * q + 4 * h) * 4);
                yv[4 * q + 0] = v4.x; yv[4 * q + 1] = v4.y; yv[4 * q + 2] = v4.z; yv[4 * q + 3] = v4.w;
            }
            bf16x8 qpk;   // M_FINAL: row c of the tile, pack columns 8h .. 8h + 7
            if constexpr (MODE == M_FINAL)
                qpk = *reinterpret_cast<const bf16x8 *>(sl + (h ? RG::OFF_B : RG::OFF_Y) + c * RG::ROWB + RG::OFF_PK);
            bf16x8 pf[FR][2];
#pragma unroll
            for (int f = 0; f < FR; ++f) {
                const int of = o_w + 32 * f;
                const bool interior = (of + 31 - t0 <= W) && (t0 + TT - 1 - of <= W);
                // scores start from the staged potentials when the scale is folded into the operand
                f32x16 acc = yv;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(yfr[ks], xf[f].v[ks], acc, 0, 0, 0);
                float e[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) e[r] = acc[r];
                if (!interior) {   // also covers a tile that misses this fragment's band entirely
                    const int lo = of + c - W - t0 - 4 * h;
                    const unsigned span = 2u * (unsigned)W;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int off = 8 * (r >> 2) + (r & 3);
                        if ((unsigned)(off - lo) > span) e[r] = -INFINITY;
                    }
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) e[r] = fast_exp2(e[r]);

                if constexpr (MODE == M_FINAL) {
                    f32x16 z;
#pragma unroll
                    for (int r = 0; r < 16; ++r) z[r] = 0.f;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks)
                        z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ks], af[f].v[ks], z, 0, 0, 0);
                    z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qpk, pob[f], z, 0, 0, 0);   // - sum_k po_k qt_k
#pragma unroll
                    for (int r = 0; r < 16; ++r) e[r] *= z[r];
                }
#pragma unroll
                for (int m = 0; m < 2; ++m)
#pragma unroll
                    for (int r = 0; r < 8; ++r) pf[f][m][r] = (__bf16)e[8 * m + r];
            }

            // second product: out[dv, o] += sum_t M[t][dv] * e[t, o], M = payload (M_APPLY) or the
            // other-side score rows themselves (M_FINAL); the transposed fragment of M serves
            // every owner fragment
            const unsigned char *pm = sl + (MODE == M_FINAL ? RG::OFF_Y : RG::OFF_B) + rd_t;
#pragma unroll
            for (int m = 0; m < 2; ++m)
#pragma unroll
                for (int dvt = 0; dvt < D / 32; ++dvt) {
                    bf16x4v lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                        (bf16x4v __attribute__((address_space(3))) *)(pm + (16 * m) * RG::ROWB + dvt * 64));
                    bf16x4v hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                        (bf16x4v __attribute__((address_space(3))) *)(pm + (16 * m + 8) * RG::ROWB + dvt * 64));
                    bf16x8 am = {lo4[0], lo4[1], lo4[2], lo4[3], hi4[0], hi4[1], hi4[2], hi4[3]};
#pragma unroll
                    for (int f = 0; f < FR; ++f)   // (a fragment the tile misses has e == 0 throughout)
                        outm[f][dvt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, pf[f][m], outm[f][dvt], 0, 0, 0);
                }
        }
        if (more) s_store(ny, nb, nvy, nvq, jnew, kbase + jnew);
        __syncthreads();
    }

    // epilogue: owner-side factor, store (and the <dot_mat_o, out_o> reduction for dV).  The rows
    // of dot_mat are requested first, for all fragments at once: behind the stores they would wait
    // for every store before them to be acknowledged.
    uint2 draw[MODE == M_APPLY ? FR : 1][D / 32][4];
    if constexpr (MODE == M_APPLY) {
        if (a.dot_mat) {
#pragma unroll
            for (int f = 0; f < FR; ++f) {
                const T *drow = reinterpret_cast<const T *>(a.dot_mat) + moff + (long)min(o_w + 32 * f + c, L - 1) * D;
#pragma unroll
                for (int j = 0; j < D / 32; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        draw[f][j][q] = *reinterpret_cast<const uint2 *>(drow + 32 * j + 8 * q + 4 * h);
            }
        }
    }
#pragma unroll
    for (int f = 0; f < FR; ++f) {
        const int o = o_w + 32 * f + c;
        const int oc = min(o, L - 1);
        const float xso = xsp[min(o, Le - 1)];
        const bool dead = o >= Le || xso == -INFINITY;   // beyond the valid length, or an inactive token: zeros
        float fac = fast_exp2((xso - mblk) * LOG2E);
        if constexpr (MODE == M_FINAL) fac *= a.cs;
        float pdb = 0.f;   // plan entry of the spoke (o, dustbin) when the dustbin carries a payload
        if constexpr (MODE == M_APPLY)
            if (a.pay_db) pdb = __expf(a.spoke_own.p[n * a.spoke_own.stride + oc] + xsp[oc] + ytp[L]);
        T *orow = reinterpret_cast<T *>(a.out_mat) + moff + (long)oc * D;
        float dot = 0.f;
#pragma unroll
        for (int j = 0; j < D / 32; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int dv = 32 * j + 8 * q + 4 * h;
                float v0 = outm[f][j][4 * q + 0] * fac, v1 = outm[f][j][4 * q + 1] * fac;
                float v2 = outm[f][j][4 * q + 2] * fac, v3 = outm[f][j][4 * q + 3] * fac;
                if constexpr (MODE == M_APPLY) {
                    if (a.pay_db) {
                        const float4 pv = *reinterpret_cast<const float4 *>(a.pay_db + (long)n * D + dv);
                        v0 = fmaf(pdb, pv.x, v0); v1 = fmaf(pdb, pv.y, v1);
                        v2 = fmaf(pdb, pv.z, v2); v3 = fmaf(pdb, pv.w, v3);
                    }
                }
                if (dead) v0 = v1 = v2 = v3 = 0.f;
                if (o < L) {
                    store4<T>(orow + dv, v0, v1, v2, v3);
                    if constexpr (MODE == M_APPLY) {
                        if (a.dot_mat && !dead) {
                            const uint2 u = draw[f][j][q];   // four bf16: the upper half of a float each
                            const float d0 = __uint_as_float(u.x << 16), d1 = __uint_as_float(u.x & 0xffff0000u);
                            const float d2 = __uint_as_float(u.y << 16), d3 = __uint_as_float(u.y & 0xffff0000u);
                            dot += d0 * v0 + d1 * v1 + d2 * v2 + d3 * v3;
                        }
                    }
                }
            }
        if constexpr (MODE == M_APPLY) {
            if (a.dot_mat) {
                dot += __shfl_xor(dot, 32);
                if (h == 0 && o < L) {
                    if (a.olog.p && !dead) dot *= __expf(-a.olog.p[n * a.olog.stride + o]);
                    a.dot_out.p[n * a.dot_out.stride + o] = dot;
                }
            }
        }
    }
}

}  // namespace
