// O(L d) and O(L) kernels around the sweeps: prescale, row dots, modifier packs, dustbin element, seeds,
// norms, masks, and the spoke work of learned dustbin tokens.
#pragma once
#include "ska_common.h"

namespace {

// ------------------------------------------------------------------ small kernels
__global__ void fill_kernel(float *p, long per, long stride, int nprob, float val)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < per * nprob) p[(i / per) * stride + (i % per)] = val;
}

// g_o = <A_o, B_o> for o below the problem's valid length (len[n / nh], or L if len is null);
// g = 0 from there to Lp.  A row is read by D * sizeof(T) / 16 neighbouring
// lanes, 16 bytes each (whole 128-byte lines per group of lanes), and reduced across them.
template <typename T, int D>
__global__ void rowdot_kernel(const T *A, const T *Bm, float *g, long gstride, int L, int Lp, const int *len, int nh,
                              int n0)
{   // (n0: index of this launch's first problem within the call, for the length lookup)
    constexpr int LPR = D * (int)sizeof(T) / 16;   // lanes per row: 4 ... 32, a power of two
    constexpr int EPL = 16 / (int)sizeof(T);       // elements per lane
    const int n = blockIdx.y;
    const long p = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int o = (int)(p / LPR), sub = (int)(p % LPR);
    float acc = 0.f;
    const int Lv = len ? min(max(len[(n + n0) / nh], 0), L) : L;
    if (o < Lv) {
        const T *pa = A + ((long)n * L + o) * D + sub * EPL, *pb = Bm + ((long)n * L + o) * D + sub * EPL;
#pragma unroll
        for (int k = 0; k < EPL; k += 4) {
            float x[4], y[4];
            load4<T>(pa + k, x);
            load4<T>(pb + k, y);
            acc += x[0] * y[0] + x[1] * y[1] + x[2] * y[2] + x[3] * y[3];
        }
    }
#pragma unroll
    for (int m = LPR / 2; m >= 1; m >>= 1) acc += __shfl_xor(acc, m);
    if (sub == 0 && o < Lp) g[n * gstride + o] = acc;
}

// ---- issue-rate probe (benchmark hook): what one SIMD sustains of the scaling sweep's instruction
// mix, with no memory traffic.  Per loop iteration ("tile") a wavefront runs, depending on WHAT,
// four dependent 32x32x16 bf16 MFMAs (M), 16 exp2 (E) and 16 adds (A), the VALU work consuming the
// MFMA result as in the sweep (other wavefronts of the SIMD are free to fill the gaps):
//   0: E + A   1: M   2: M + E + A (the sweep's pattern)   3: M + A   4: M + E   5: A
//   6: M + P + A and 7: M + 8 E + 8 P + A, where P is exp2 on the plain ALUs instead of the
//      transcendental unit: 2^x = ldexp(p(fract x), floor x) with a cubic p (six instructions:
//      v_fract_f32, v_cvt_flr_i32_f32, three FMAs, v_ldexp_f32; relative error 1e-4)
// Without adds the 16 values are folded by eight max3 instead.  One float per thread is written.
__device__ __forceinline__ float poly_exp2(float x)
{
    const float f = __builtin_amdgcn_fractf(x);
    int i;
    asm("v_cvt_flr_i32_f32 %0, %1" : "=v"(i) : "v"(x));
    float p = fmaf(f, 0.0790210f, 0.2240918f);
    p = fmaf(p, f, 0.6964571f);
    p = fmaf(p, f, 0.9998931f);
    return ldexpf(p, i);
}
template <int WHAT>
__global__ __launch_bounds__(256) void issue_probe_kernel(float *out, int tiles)
{
    constexpr bool M = (WHAT >= 1 && WHAT <= 4) || WHAT >= 6, E = (WHAT == 0 || WHAT == 2 || WHAT == 4 || WHAT >= 6);
    constexpr bool A = (WHAT == 0 || WHAT == 2 || WHAT == 3 || WHAT >= 5);
    constexpr int NPOLY = WHAT == 6 ? 16 : WHAT == 7 ? 8 : 0;   // how many of the 16 exponentials go the polynomial way
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(threadIdx.x * 0.01f); b[i] = (__bf16)(i * 0.1f); }
    f32x16 c0, c;
#pragma unroll
    for (int i = 0; i < 16; ++i) { c0[i] = -30.f - 0.01f * i; c[i] = -1.f - 0.01f * i; }
    float sum = 0.f;
    const float step = 1e-3f * (float)(threadIdx.x & 7);
    for (int it = 0; it < tiles; ++it) {
        if constexpr (M) {   // the first MFMA starts from a loop-invariant accumulator, as the sweep's does
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
#pragma unroll
            for (int k = 1; k < 4; ++k) c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
        }
        if constexpr (!M) {   // no MFMA: iterate on the values themselves so that every tile depends on the last
            if constexpr (E) {
#pragma unroll
                for (int r = 0; r < 16; ++r) { c[r] = fast_exp2(c[r]); sum += c[r]; }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) c[r] += step;
            }
        } else {
            float e[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) e[r] = !E ? c[r] : (NPOLY == 16 || (NPOLY == 8 && (r & 1))) ? poly_exp2(c[r]) : fast_exp2(c[r]);
            if constexpr (A) {
#pragma unroll
                for (int r = 0; r < 16; ++r) sum += e[r];
            } else if constexpr (E) {
                float m = e[0];
#pragma unroll
                for (int r = 1; r < 16; ++r) m = fmaxf(m, e[r]);
                sum += m;
            } else {
                sum = e[0];
            }
            a[0] = (__bf16)sum;   // the next tile depends on this one
        }
    }
    float s = sum;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c[r];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// ---- learned dustbin token (Sec. "Single-Active-Dustbin Bridge"): the O(L d) work on the spokes
// out[n][o] = scale <M[n][o], x[n]> for o < L, out[n][L] = scale <x[n], xc[n]> (the corner).
// LPR lanes per row, 16 bytes each, like rowdot_kernel.
template <typename T, int D>
__global__ void spoke_scores_kernel(const T *M, const float *x, const float *xc, float *out, long ostride, int L,
                                    float scale)
{
    constexpr int LPR = D * (int)sizeof(T) / 16, EPL = 16 / (int)sizeof(T);
    const int n = blockIdx.y;
    const long p = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int o = (int)(p / LPR), sub = (int)(p % LPR);
    float acc = 0.f;
    if (o <= L) {
        const float *xv = x + (long)n * D + sub * EPL;
#pragma unroll
        for (int k = 0; k < EPL; k += 4) {
            float a4[4];
            if (o < L) load4<T>(M + ((long)n * L + o) * D + sub * EPL + k, a4);
            else { const float *c4 = xc + (long)n * D + sub * EPL + k; a4[0] = c4[0]; a4[1] = c4[1]; a4[2] = c4[2]; a4[3] = c4[3]; }
            acc += a4[0] * xv[k] + a4[1] * xv[k + 1] + a4[2] * xv[k + 2] + a4[3] * xv[k + 3];
        }
    }
#pragma unroll
    for (int m = LPR / 2; m >= 1; m >>= 1) acc += __shfl_xor(acc, m);
    if (sub == 0 && o <= L) out[n * ostride + o] = scale * acc;
}

// Weights of a weighted row sum, two kinds:
//   plan : w_o = exp(spoke[o] + x[o] + yL)   (plan entries of the spokes (o, dustbin); yL = y[L])
//   given: w_o = wv[o]
// partial[n][chunk][dv] = sum over the chunk's rows o of w_o M[n][o][dv]; rows in chunks of WS_ROWS.
constexpr int WS_ROWS = 1024;
template <typename T, int D>
__global__ __launch_bounds__(256) void wsum_kernel(const T *M, Vec wv, Vec spoke, Vec x, Vec y, float *partial, int L)
{
    constexpr int TPR = D / 4;            // threads per row, four columns each
    constexpr int RPI = 256 / TPR;        // rows per iteration
    __shared__ float red[256][4];
    const int n = blockIdx.y, chunk = blockIdx.x, tid = threadIdx.x;
    const int col = (tid % TPR) * 4, r0 = tid / TPR;
    const int o_end = min(L, (chunk + 1) * WS_ROWS);
    float yL = 0.f;
    if (!wv.p) yL = y.p[n * y.stride + L];
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int o = chunk * WS_ROWS + r0; o < o_end; o += RPI) {
        const float w = wv.p ? wv.p[n * wv.stride + o]
                             : __expf(spoke.p[n * spoke.stride + o] + x.p[n * x.stride + o] + yL);
        float m4[4];
        load4<T>(M + ((long)n * L + o) * D + col, m4);
        acc[0] = fmaf(w, m4[0], acc[0]); acc[1] = fmaf(w, m4[1], acc[1]);
        acc[2] = fmaf(w, m4[2], acc[2]); acc[3] = fmaf(w, m4[3], acc[3]);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) red[tid][k] = acc[k];
    __syncthreads();
    if (tid < TPR) {
        float t4[4] = {0.f, 0.f, 0.f, 0.f};
        for (int r = 0; r < RPI; ++r)
#pragma unroll
            for (int k = 0; k < 4; ++k) t4[k] += red[r * TPR + tid][k];
        float *dst = partial + ((long)n * gridDim.x + chunk) * D + col;
        dst[0] = t4[0]; dst[1] = t4[1]; dst[2] = t4[2]; dst[3] = t4[3];
    }
}
// out[n][dv] = scale (sum_chunk partial[n][chunk][dv] + wc[n] xc[n][dv]); if dotv is given also
// dot_out[n] = <dotv[n], out[n]>.  wc_at: index of the corner weight in wc (null: no corner).
template <int D>
__global__ void wsum_final_kernel(const float *partial, int nchunk, Vec wc, int wc_at, const float *xc, float scale,
                                  float *out, const float *dotv, VecOut dot_out, int dot_at)
{
    const int n = blockIdx.x, dv = threadIdx.x;   // D threads
    float acc = 0.f;
    for (int c = 0; c < nchunk; ++c) acc += partial[((long)n * nchunk + c) * D + dv];
    if (wc.p) acc = fmaf(wc.p[n * wc.stride + wc_at], xc[(long)n * D + dv], acc);
    acc *= scale;
    out[(long)n * D + dv] = acc;
    if (dotv) {
        __shared__ float red[D];
        red[dv] = acc * dotv[(long)n * D + dv];
        __syncthreads();
        if (dv == 0) {
            float t = 0.f;
            for (int k = 0; k < D; ++k) t += red[k];
            dot_out.p[n * dot_out.stride + dot_at] = t;
        }
    }
}

// Score cotangent on the spokes (Prop. 2 on the augmented support), one-reference form:
//   sbr[i] = P_RR(i, d_k) (<dO_i, v_db> - sum_k rowp_k[i] colp_k[L])        i < L
//   sbc[j] = P_RR(d_q, j) (            - sum_k rowp_k[L] colp_k[j])          j < L
//   sbr[L] = sbc[L] = P_RR(d_q, d_k) (- sum_k rowp_k[L] colp_k[L])
// with P_RR(i, d_k) = exp(SQ[i] + u_R[i] + v_R[L]), P_RR(d_q, j) = exp(SK[j] + u_R[L] + v_R[j]).
template <typename T, int D>
__global__ void spoke_sbar_kernel(const T *G, const float *vdb, Vec uR, Vec vR, Vec SQ, Vec SK, const float4 *rowp,
                                  const float4 *colp, int nq, long ldp, float *sbr, float *sbc, long ostride, int L)
{
    constexpr int LPR = D * (int)sizeof(T) / 16, EPL = 16 / (int)sizeof(T);
    const int n = blockIdx.y;
    const long p = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int o = (int)(p / LPR), sub = (int)(p % LPR);
    float z = 0.f;
    if (o < L) {
        const float *xv = vdb + (long)n * D + sub * EPL;
#pragma unroll
        for (int k = 0; k < EPL; k += 4) {
            float a4[4];
            load4<T>(G + ((long)n * L + o) * D + sub * EPL + k, a4);
            z += a4[0] * xv[k] + a4[1] * xv[k + 1] + a4[2] * xv[k + 2] + a4[3] * xv[k + 3];
        }
    }
#pragma unroll
    for (int m = LPR / 2; m >= 1; m >>= 1) z += __shfl_xor(z, m);
    if (sub != 0 || o > L) return;
    const float4 *ro = rowp + ((long)n * ldp + o) * nq, *co = colp + ((long)n * ldp + o) * nq;
    const float4 *rL = rowp + ((long)n * ldp + L) * nq, *cL = colp + ((long)n * ldp + L) * nq;
    float mr = 0.f, mc = 0.f;   // sum_k rowp_k[o] colp_k[L], sum_k rowp_k[L] colp_k[o]
    for (int g = 0; g < nq; ++g) {
        const float4 a = ro[g], b = cL[g], c = rL[g], d = co[g];
        mr += a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w;
        mc += c.x * d.x + c.y * d.y + c.z * d.z + c.w * d.w;
    }
    const float uRo = uR.p[n * uR.stride + o], vRo = vR.p[n * vR.stride + o];
    const float uRL = uR.p[n * uR.stride + L], vRL = vR.p[n * vR.stride + L];
    if (o < L) {
        sbr[n * ostride + o] = __expf(SQ.p[n * SQ.stride + o] + uRo + vRL) * (z - mr);
        sbc[n * ostride + o] = -__expf(SK.p[n * SK.stride + o] + uRL + vRo) * mc;
    } else {
        const float c = -__expf(SQ.p[n * SQ.stride + L] + uRL + vRL) * mr;
        sbr[n * ostride + L] = c;
        sbc[n * ostride + L] = c;
    }
}

// M[n][o][:] += scale w[n][o] x[n][:] for o < L (the spoke part of dQ / dK), storage type T
template <typename T, int D>
__global__ void spoke_axpy_kernel(T *M, Vec w, const float *x, float scale, int L)
{
    constexpr int TPR = D / 4;
    const int n = blockIdx.y;
    const long p = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int o = (int)(p / TPR), col = (int)(p % TPR) * 4;
    if (o >= L) return;
    const float f = scale * w.p[n * w.stride + o];
    const float *xv = x + (long)n * D + col;
    T *dst = M + ((long)n * L + o) * D + col;
    float m4[4];
    load4<T>(dst, m4);
    store4<T>(dst, fmaf(f, xv[0], m4[0]), fmaf(f, xv[1], m4[1]), fmaf(f, xv[2], m4[2]), fmaf(f, xv[3], m4[3]));
}

// Start of the base solve with inactive tokens: u0[i] = -inf where mask_q[b][i] == 0,
// v0[j] = -inf where mask_k[b][j] == 0 (elsewhere they keep their zeros).  UV slots 0 and 1.
__global__ void mask_fill_kernel(float *UV, long us, int Lp, int L, const unsigned char *mq, const unsigned char *mk,
                                 int nh)
{
    const int n = blockIdx.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= L) return;
    const long m = (long)(n / nh) * L + i;
    if (mq && !mq[m]) UV[n * us + i] = -INFINITY;
    if (mk && !mk[m]) UV[n * us + Lp + i] = -INFINITY;
}

// dst[n][dslot0 + s][:] = src[n][sslot0 + s][:] for s < nslots: potential vectors between two UV arrays
// of different depth (problem strides sstride, dstride floats; a slot is Lp floats)
__global__ void slots_copy_kernel(const float *src, long sstride, int sslot0, float *dst, long dstride, int dslot0,
                                  int nslots, int Lp)
{
    const int n = blockIdx.y;
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (long)nslots * Lp) dst[n * dstride + (long)dslot0 * Lp + i] = src[n * sstride + (long)sslot0 * Lp + i];
}

// p[n][j] *= f for j < per (the base potentials between two stages of a continuation schedule)
__global__ void scale_kernel(float *p, long per, long stride, int nprob, float f)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < per * nprob) p[(i / per) * stride + (i % per)] *= f;
}

// *out = max(*out, max_i |x_i|) over n elements (a NaN counts as +inf).  Non-negative floats
// order like their bit patterns, so the maximum is taken on unsigned integers.
template <typename T>
__global__ __launch_bounds__(256) void absmax_kernel(const T *x, long n, float *out)
{
    float m = 0.f;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) {
        const float v = fabsf((float)x[i]);
        m = (v == v) ? fmaxf(m, v) : INFINITY;
    }
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) m = fmaxf(m, __shfl_xor(m, s));
    __shared__ float red[4];
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        atomicMax(reinterpret_cast<unsigned int *>(out), __float_as_uint(m));
    }
}

// out[n][j] = seed[n][j] / b_j for j < Lp: a cotangent handed in from outside enters the reverse
// recurrences in the form the workspace keeps (divided by the marginal target).
__global__ void seed_kernel(const float *seed, const float *olog, float *out, long ostride, int Lp)
{
    const int n = blockIdx.y;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= Lp) return;
    float r = seed[(long)n * Lp + j];
    if (olog) r *= __expf(-olog[(long)n * Lp + j]);
    out[n * ostride + j] = r;
}

// Qs = bf16(scale * Q): the score scale log2(e)/(eps sqrt d) folded into one operand once,
// so that no sweep pays a multiply per edge for it.  8 elements per thread.
__global__ void prescale_kernel(const __bf16 *src, __bf16 *dst, long n8, float scale)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n8) return;
    uint4 raw = reinterpret_cast<const uint4 *>(src)[i];
    bf16x8 v = *reinterpret_cast<bf16x8 *>(&raw);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (__bf16)((float)v[e] * scale);
    reinterpret_cast<uint4 *>(dst)[i] = *reinterpret_cast<uint4 *>(&v);
}

// Modifier packs of Prop. 2 for a tail of depth R.  With a_t = exp(u_t - u_R), b_t = exp(v_t - v_R)
// the score cotangent is P_RR . [Z - sum_k row_k(i) col_k(j)] over 2R rank-1 terms, two per
// tail step t = R ... 1:
//     row = a_t,           col = b_t vbar_t        (the factor P_tt     . (1 vbar_t^T))
//     row = a_t ubar_t,    col = b_{t-1}           (the factor P_t,t-1  . (ubar_t 1^T))
// (R = 2: row = (1, ubar2, alpha, alpha ubar1), col = (vbar2, beta, beta vbar1, delta).)
// Written as groups of four floats (generic final sweep) or, for the ring kernel (R <= 2), as
// 16 bf16 columns per index in two forms: "A" for the side that is streamed ([hi, lo, hi] per
// value) and "B" for the side that owns the rows ([-hi, -hi, -lo]); an A row times a B row is
// then -sum_k (hi hi + lo hi + hi lo) = -sum_k row_k col_k to about 2^-16 relative.
// aug = rowA, rowB, colA, colB, each [N][ldp][16].  Workspace vectors: vec 1 + 2(R - t) is
// vbar_t, vec 2 + 2(R - t) is ubar_t.
__device__ __forceinline__ void pack_cols(const float (&x)[4], __bf16 *A, __bf16 *B)
{
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const __bf16 hi = (__bf16)x[k];
        const __bf16 lo = (__bf16)(x[k] - (float)hi);
        A[3 * k + 0] = hi; A[3 * k + 1] = lo; A[3 * k + 2] = hi;
        B[3 * k + 0] = (__bf16)(-(float)hi); B[3 * k + 1] = (__bf16)(-(float)hi); B[3 * k + 2] = (__bf16)(-(float)lo);
    }
#pragma unroll
    for (int k = 12; k < 16; ++k) { A[k] = (__bf16)0.f; B[k] = (__bf16)0.f; }
}
// direct != 0 (comparator): a group holds the two terms of one tail step as (log2 modifier, weight)
// pairs, row side (l_t, 1, l_t, ubar_t), column side (m_t, vbar_t, m_{t-1}, 1) with
// l_t = (u_t - u_R) log2 e, m_t = (v_t - v_R) log2 e; nq = R groups.
__global__ void packs_kernel(const float *UV, int Lp, int R, const float *vecs, long nldw, long wstride,
                             float *rowp, float *colp, int nq, __bf16 *aug, long ldp, long nldp, int direct,
                             int both)
{
    // both != 0: the float groups are written next to the bf16 columns (the spokes of a learned
    // dustbin token read them)
    const int n = blockIdx.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= Lp) return;
    const float *uv = UV + (long)n * 2 * (R + 1) * Lp;
    const long w = n * wstride + i;
    const float uR = uv[(2 * R) * Lp + i], vR = uv[(2 * R + 1) * Lp + i];
    float r4[4] = {0.f, 0.f, 0.f, 0.f}, c4[4] = {0.f, 0.f, 0.f, 0.f};   // the first four terms (ring kernel)
    float *rp = rowp + (n * ldp + i) * 4L * nq, *cp = colp + (n * ldp + i) * 4L * nq;
    for (int q = 0; q < R; ++q) {   // q = R - t
        const int t = R - q;
        // an inactive token (potential -inf on its side) has all-zero modifiers
        const bool rdead = uR == -INFINITY, cdead = vR == -INFINITY;
        const float at = rdead ? 0.f : __expf(uv[(2 * t) * Lp + i] - uR);
        const float bt = cdead ? 0.f : __expf(uv[(2 * t + 1) * Lp + i] - vR);
        const float bp = cdead ? 0.f : __expf(uv[(2 * t - 1) * Lp + i] - vR);
        const float vb = vecs[(1 + 2 * q) * nldw + w], ub = vecs[(2 + 2 * q) * nldw + w];
        if (direct) {
            const float lt = rdead ? 0.f : (uv[(2 * t) * Lp + i] - uR) * LOG2E;
            const float mt = cdead ? 0.f : (uv[(2 * t + 1) * Lp + i] - vR) * LOG2E;
            const float mp = cdead ? 0.f : (uv[(2 * t - 1) * Lp + i] - vR) * LOG2E;
            rp[4 * q] = lt; rp[4 * q + 1] = rdead ? 0.f : 1.f; rp[4 * q + 2] = lt; rp[4 * q + 3] = ub;
            cp[4 * q] = mt; cp[4 * q + 1] = vb;  cp[4 * q + 2] = mp; cp[4 * q + 3] = cdead ? 0.f : 1.f;
            continue;
        }
        if (!aug || both) {
            rp[2 * q] = at;          cp[2 * q] = bt * vb;
            rp[2 * q + 1] = at * ub; cp[2 * q + 1] = bp;
        }
        if (aug && q < 2) {
            if (q == 0) { r4[0] = at; c4[0] = bt * vb; r4[1] = at * ub; c4[1] = bp; }
            else { r4[2] = at; c4[2] = bt * vb; r4[3] = at * ub; c4[3] = bp; }
        }
    }
    if (direct) return;   // (R groups, all written)
    if (!aug || both)
        for (int k = 2 * R; k < 4 * nq; ++k) { rp[k] = 0.f; cp[k] = 0.f; }   // pad the last group
    if (aug) {
        __align__(16) __bf16 A[16], B[16];
        const long e = (n * ldp + i) * 16;
        pack_cols(r4, A, B);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            reinterpret_cast<uint4 *>(aug + 0 * nldp * 16 + e)[q] = reinterpret_cast<const uint4 *>(A)[q];
            reinterpret_cast<uint4 *>(aug + 1 * nldp * 16 + e)[q] = reinterpret_cast<const uint4 *>(B)[q];
        }
        pack_cols(c4, A, B);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            reinterpret_cast<uint4 *>(aug + 2 * nldp * 16 + e)[q] = reinterpret_cast<const uint4 *>(A)[q];
            reinterpret_cast<uint4 *>(aug + 3 * nldp * 16 + e)[q] = reinterpret_cast<const uint4 *>(B)[q];
        }
    }
}

}  // namespace
