// The generic sweep kernel (double-buffered LDS tiles): matrix sweeps in fp32 storage and at d = 128, deep
// tails, and the direct plan-by-plan comparator.
#pragma once
#include "ska_common.h"

namespace {

// ------------------------------------------------------------------ the generic sweep kernel
// Double-buffered LDS staging, one other-side tile per barrier.  It serves every fp32-storage
// matrix sweep and the bf16 matrix sweeps at d = 128; the ring kernels take the rest.
template <typename T, int D, int MODE> struct Stage {
    using TL = Tile<T, D>;
    static constexpr bool HAS_B = (MODE == M_FINAL);
    static constexpr bool HAS_PAY = (MODE == M_APPLY) || (MODE == M_FINAL && TL::IS_BF16);
    static constexpr int OFF_Y = 0;
    static constexpr int OFF_B = OFF_Y + TL::RM_BYTES;
    static constexpr int OFF_PAY = OFF_B + (HAS_B ? TL::RM_BYTES : 0);
    static constexpr int OFF_VY = OFF_PAY + (HAS_PAY ? TL::PT_BYTES : 0);
    static constexpr int OFF_VQ = OFF_VY + TT * 4;
    static constexpr int BYTES = ((OFF_VQ + TT * 16 * MAXNQ) + 15) / 16 * 16;
};

// DIRECT (M_FINAL only): the comparator that forms every staircase plan factor by an
// exponential of its own, exp(S + u_t + v_t'), instead of scaling the one reference tile
// (Prop. 2 versus the plain evaluation of Prop. 1).  A pack group then holds two terms as
// (log2 modifier, weight) pairs: the term is exp2(score + l_row + l_col) w_row w_col.
template <typename T, int D, int MODE, int FR, bool DIRECT = false>
__global__ __launch_bounds__(NTHREADS) void sweep_kernel(const SweepArgs a)
{
    using TL = Tile<T, D>;
    using ST = Stage<T, D, MODE>;
    constexpr int BM = NWAVES * FR * 32;
    static_assert(MODE == M_APPLY || MODE == M_FINAL, "matrix sweeps only");

    extern __shared__ __align__(16) unsigned char smem[];   // two stages of ST::BYTES
    __shared__ float red[NWAVES];

    // XCD-aware placement: hardware deals workgroups round-robin over the 8 XCDs, so
    // give each XCD one contiguous eighth of the (problem, block) sequence; neighbours
    // that share band rows then meet in the same L2.
    const int chunk = (a.nb_total + 7) >> 3;
    const int bx = (int)blockIdx.x;
    const int lb = (bx & 7) * chunk + (a.rev ? chunk - 1 - (bx >> 3) : (bx >> 3));
    if (lb >= a.nb_total) return;
    const int n = lb / a.nbp;
    const int o_blk = (lb % a.nbp) * BM;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
    const T *Yb = reinterpret_cast<const T *>(a.Y) + moff;
    const float *ytp = a.yt.p + n * a.yt.stride;
    // owner-side potential: stabiliser and factor of the plan; -inf marks an inactive token (a
    // masked one, or one without any active partner), which stays inactive in every later
    // iterate.
    const float *xsp = a.xs.p + n * a.xs.stride;

    // workgroup stabiliser: largest owner-side potential in this block
    float mblk = 0.f;
    {
        float m = -INFINITY;
        for (int i = tid; i < BM; i += NTHREADS)
            if (o_blk + i < Le) m = fmaxf(m, xsp[o_blk + i]);
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) m = fmaxf(m, __shfl_xor(m, s));
        if (lane == 0) red[wave] = m;
        __syncthreads();
        mblk = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        if (mblk == -INFINITY) mblk = 0.f;   // a block of inactive tokens only
    }
    const float m2 = mblk * LOG2E;

    // owner-side fragments
    OwnerFrag<T, D> xf[FR];
    OwnerFrag<T, D> af[MODE == M_FINAL ? FR : 1];
    float4 pof[FR][MAXNQ];
    int o_frag[FR];
#pragma unroll
    for (int f = 0; f < FR; ++f) {
        o_frag[f] = o_blk + (wave * FR + f) * 32;
        xf[f].load(Xb, o_frag[f] + c, Le, h);
        if constexpr (MODE == M_FINAL) {
            af[f].load(reinterpret_cast<const T *>(a.A) + moff, o_frag[f] + c, Le, h);
#pragma unroll
            for (int g = 0; g < MAXNQ; ++g)
                pof[f][g] = (o_frag[f] + c < Le && g < a.nq) ? a.po[(n * a.ldp + o_frag[f] + c) * a.pstride + g]
                                                            : make_float4(0, 0, 0, 0);
        }
    }

    // accumulators
    f32x16 outm[FR][D / 32];
#pragma unroll
    for (int f = 0; f < FR; ++f)
#pragma unroll
        for (int j = 0; j < D / 32; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) outm[f][j][r] = 0.f;

    // other-side tile range of the whole block (tiles aligned to multiples of 32)
    int lo = o_blk - W;            // the host clamps W to L, so none of this overflows
    if (lo < 0) lo = 0;
    int hi = o_blk + BM - 1 + W;
    if (hi > Lt - 1) hi = Lt - 1;   // (lo <= hi: the block has a row below Le <= Lt + W)
    const int k_lo = lo / TT, k_hi = hi / TT;

    // staging registers
    uint4 ry[TL::CPT], rb[ST::HAS_B ? TL::CPT : 1], rp[MODE == M_APPLY ? TL::CPT : 1];
    float rvy = 0.f;
    float4 rvq[MAXNQ] = {make_float4(0, 0, 0, 0), make_float4(0, 0, 0, 0)};

    auto g_load = [&](int k) {
        const int t0 = k * TT;
        tile_load<T, D>(ry, Yb, t0, Lt);
        if constexpr (ST::HAS_B) tile_load<T, D>(rb, reinterpret_cast<const T *>(a.Bm) + moff, t0, Lt);
        if constexpr (MODE == M_APPLY) tile_load<T, D>(rp, reinterpret_cast<const T *>(a.Pay) + moff, t0, Lt);
        if (tid < TT) {
            const int t = t0 + tid;
            rvy = (t < Lt) ? ytp[t] * LOG2E + m2 : -INFINITY;
            if constexpr (MODE == M_FINAL) {
#pragma unroll
                for (int g = 0; g < MAXNQ; ++g)
                    rvq[g] = (t < Lt && g < a.nq) ? a.qt[(n * a.ldp + t) * a.pstride + g] : make_float4(0, 0, 0, 0);
            }
        }
    };
    auto s_store = [&](int buf) {
        unsigned char *s = smem + buf * ST::BYTES;
        tile_store_rm<T, D>(ry, s + ST::OFF_Y);
        if constexpr (ST::HAS_B) tile_store_rm<T, D>(rb, s + ST::OFF_B);
        if constexpr (MODE == M_APPLY) tile_store_pay<T, D>(rp, s + ST::OFF_PAY);
        if constexpr (MODE == M_FINAL && TL::IS_BF16) tile_store_pay<T, D>(ry, s + ST::OFF_PAY);
        if (tid < TT) {
            reinterpret_cast<float *>(s + ST::OFF_VY)[tid] = rvy;
            if constexpr (MODE == M_FINAL) {
#pragma unroll
                for (int g = 0; g < MAXNQ; ++g) reinterpret_cast<float4 *>(s + ST::OFF_VQ)[tid * MAXNQ + g] = rvq[g];
            }
        }
    };

    g_load(k_lo);
    s_store(0);
    __syncthreads();

    for (int k = k_lo; k <= k_hi; ++k) {
        const int buf = (k - k_lo) & 1;
        if (k < k_hi) g_load(k + 1);
        const unsigned char *s = smem + buf * ST::BYTES;
        const int t0 = k * TT;

#pragma unroll
        for (int f = 0; f < FR; ++f) {
            const int of = o_frag[f];
            // does this tile meet the band of this fragment at all?
            if (of >= Le || (long)t0 + TT - 1 < (long)of - W || (long)t0 > (long)of + 31 + W) continue;
            const bool interior = ((long)of + 31 - t0 <= W) && ((long)t0 + TT - 1 - of <= W);

            f32x16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
            acc = tile_dot<D>(s + ST::OFF_Y, xf[f], lane, acc);

            float yv[16];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float4 v4 = *reinterpret_cast<const float4 *>(s + ST::OFF_VY + (8 * q + 4 * h) * 4);
                yv[4 * q + 0] = v4.x; yv[4 * q + 1] = v4.y; yv[4 * q + 2] = v4.z; yv[4 * q + 3] = v4.w;
            }
            float e[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) e[r] = fmaf(acc[r], a.c2, yv[r]);
            if (!interior) {
                const int o = of + c;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int t = t0 + 8 * (r >> 2) + 4 * h + (r & 3);
                    const int dlt = o > t ? o - t : t - o;
                    if (dlt > W) e[r] = -INFINITY;
                }
            }

            {
                float el[DIRECT ? 16 : 1];
                if constexpr (DIRECT)
#pragma unroll
                    for (int r = 0; r < 16; ++r) el[r] = e[r];
#pragma unroll
                for (int r = 0; r < 16; ++r) e[r] = fast_exp2(e[r]);
                if constexpr (MODE == M_APPLY) {
                    tile_accum<T, D>(outm[f], s + ST::OFF_PAY, e, lane);
                } else {  // M_FINAL
                    f32x16 z;
#pragma unroll
                    for (int r = 0; r < 16; ++r) z[r] = 0.f;
                    if (!a.skipz) z = tile_dot<D>(s + ST::OFF_B, af[f], lane, z);
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int tl = 8 * (r >> 2) + 4 * h + (r & 3);
                        float md = z[r];
                        if constexpr (DIRECT) {
                            float sb = e[r] * md;
#pragma unroll
                            for (int g = 0; g < MAXNQ; ++g) {   // (an absent group has zero weights)
                                float4 q4 = *reinterpret_cast<const float4 *>(s + ST::OFF_VQ + (tl * MAXNQ + g) * 16);
                                const float p0 = (g == 0 && a.refterm) ? e[r]
                                                                       : fast_exp2(el[r] + pof[f][g].x + q4.x);
                                const float p1 = fast_exp2(el[r] + pof[f][g].z + q4.z);
                                sb = fmaf(-p0 * pof[f][g].y, q4.y, sb);
                                sb = fmaf(-p1 * pof[f][g].w, q4.w, sb);
                            }
                            e[r] = sb;
                        } else {
#pragma unroll
                            for (int g = 0; g < MAXNQ; ++g) {   // (an absent group is all zeros)
                                float4 q4 = *reinterpret_cast<const float4 *>(s + ST::OFF_VQ + (tl * MAXNQ + g) * 16);
                                md = fmaf(-pof[f][g].x, q4.x, md);
                                md = fmaf(-pof[f][g].y, q4.y, md);
                                md = fmaf(-pof[f][g].z, q4.z, md);
                                md = fmaf(-pof[f][g].w, q4.w, md);
                            }
                            e[r] *= md;
                        }
                    }
                    tile_accum<T, D>(outm[f], TL::IS_BF16 ? s + ST::OFF_PAY : s + ST::OFF_Y, e, lane);
                }
            }
        }

        if (k < k_hi) s_store(buf ^ 1);
        __syncthreads();
    }

    // ---------------------------------------------------------------- epilogue
#pragma unroll
    for (int f = 0; f < FR; ++f) {
        const int o = o_frag[f] + c;
        {
            float fac = 0.f;
            bool dead = true;   // beyond the valid length, or an inactive token: zeros
            if (o < Le) {
                fac = fast_exp2((xsp[o] - mblk) * LOG2E);
                dead = xsp[o] == -INFINITY;
            }
            if constexpr (MODE == M_FINAL) fac *= a.cs;
            float pdb = 0.f;   // plan entry of the spoke (o, dustbin) when the dustbin carries a payload
            if constexpr (MODE == M_APPLY)
                if (a.pay_db && o < L) pdb = __expf(a.spoke_own.p[n * a.spoke_own.stride + o] + xsp[o] + ytp[L]);
            T *orow = reinterpret_cast<T *>(a.out_mat) + moff + (long)o * D;
            const T *drow = a.dot_mat ? reinterpret_cast<const T *>(a.dot_mat) + moff + (long)o * D : nullptr;
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
                        if constexpr (MODE == M_FINAL) {
                            if (a.accum) {
                                float old[4];
                                load4<T>(orow + dv, old);
                                v0 += old[0]; v1 += old[1]; v2 += old[2]; v3 += old[3];
                            }
                        }
                        store4<T>(orow + dv, v0, v1, v2, v3);
                        if constexpr (MODE == M_APPLY) {
                            if (drow && !dead) {
                                float dd[4];
                                load4<T>(drow + dv, dd);
                                dot += dd[0] * v0 + dd[1] * v1 + dd[2] * v2 + dd[3] * v3;
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
}

}  // namespace
