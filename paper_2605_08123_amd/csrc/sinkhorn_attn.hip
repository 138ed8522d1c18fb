// Banded Sinkhorn attention for gfx950 (MI355X): band-sweep kernels and the C ABI.
//
// Every step of the operator is a "band sweep": for each owner index o (a row of
// the plan for row-oriented sweeps, a column for column-oriented ones) reduce over
// the other index t with |o - t| <= W.  Because the band is symmetric, a column
// sweep is the row sweep of the transposed problem, i.e. the same kernel with the
// roles of Q and K exchanged, so nothing is ever read transposed from memory.
//
//   score tile   T[t, o] = <Y_t, X_o>            MFMA, recomputed in every sweep and
//                                                 never stored (Section 2.1; Prop. 2)
//   E[t, o]      = exp2(c2 * T[t, o] + y'_t + m') c2 = log2(e)/(eps sqrt d),
//                                                 y' = other-side potential * log2(e),
//                                                 m' = one stabiliser per workgroup
//   LSE          x_o  = -log sum_t exp(S_ot + y_t)            (Eq. 1 / Eq. 2)
//   MATVEC       out_o = pre_o - exp(x_o) sum_t exp(S_ot + y_t) w_t   (Prop. 1 recurrences)
//   APPLY        out_o = exp(x_o) sum_t exp(S_ot + y_t) Pay_t  (output map; dV)
//   FINAL        out_o = c exp(x_o) sum_t exp(S_ot + y_t) [<A_o, B_t> - sum_k p_k,o q_k,t] Y_t
//                                                 (Prop. 2: one reference tile + modifiers)
//
// Three kernels serve the sweeps: vsweep_kernel (LSE, MATVEC: a skewed ring of tiles in LDS),
// msweep_kernel (APPLY, FINAL for bf16 storage and d <= 64: the same ring, two products) and
// sweep_kernel (the first half-step, fp32 storage and d = 128: double-buffered tiles).
//
// MFMA tile layout (32x32 accumulators): lane l holds owner o = l & 31; register r
// holds other index t = 8*(r>>2) + 4*(l>>5) + (r&3).  Sums over t are therefore
// in-lane register sums plus one exchange between the two lane halves.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#include <new>
#include <type_traits>

#include "sinkhorn_attn.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int NTHREADS = 256;
constexpr int NWAVES = 4;
constexpr int TT = 32;  // other-side rows per tile
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

constexpr int MAXR = 32;     // deepest differentiable tail (T = 0 with R = T' + R' is full
                             // backpropagation through a T'-step base solve)
constexpr int MAXNQ = 2;     // float4 groups of modifier terms one final sweep takes (8 terms);
                             // deeper tails take several sweeps that accumulate
enum Mode { M_LSE_FIRST = 0, M_LSE = 1, M_MATVEC = 2, M_APPLY = 3, M_FINAL = 4,
            M_FINAL_DIRECT = 5 /* dispatch only: M_FINAL of the generic kernel with DIRECT = true */ };

struct Vec {          // one fp32 vector per problem
    const float *p;
    long stride;      // elements between consecutive problems
};
struct VecOut {
    float *p;
    long stride;
};

struct SweepArgs {
    const void *X;    // owner-side matrix      [N][L][D]
    const void *Y;    // other-side matrix      [N][L][D]
    const void *A;    // FINAL: owner-side factor of Z (dO for rows, V for columns)
    const void *Bm;   // FINAL: other-side factor of Z
    const void *Pay;  // APPLY: other-side payload (V for the output, dO for dV)
    void *out_mat;    // APPLY / FINAL result   [N][L][D]
    Vec yt;           // other-side potential (natural log units), length Lp
    Vec xs;           // owner-side potential / previous iterate (stabiliser), length Lp
    Vec w;            // MATVEC weights on the other side
    Vec pre;          // MATVEC additive term on the owner side (may be null)
    VecOut out_vec;   // LSE / MATVEC result
    Vec olog;         // log of the owner side's marginal target (null: unit targets).  LSE adds it
                      // to the result; MATVEC and the dot of APPLY divide their result by the target
    const float4 *po; // FINAL: owner-side modifier pack   [N][ldp][pstride], first group of this sweep
    const float4 *qt; // FINAL: other-side modifier pack   [N][ldp][pstride]
    int nq;           // groups of four terms this sweep takes (1 or 2)
    int pstride;      // groups per index in memory (2R terms in all)
    int skipz;        // FINAL: leave Z out (second and later sweeps of a deep tail)
    int refterm;      // direct FINAL: the first term of this sweep multiplies the reference plan itself
    int accum;        // FINAL: add to the output instead of overwriting it
    const void *poB;  // FINAL on the ring kernel: owner-side pack as 16 bf16 columns  [N][ldp][16]
    const void *qtA;  // FINAL on the ring kernel: other-side pack as 16 bf16 columns  [N][ldp][16]
    long ldp;
    const void *dot_mat;  // APPLY: if set, dot_out_o = <dot_mat_o, out_o> (fp32 accumulators)
    VecOut dot_out;
    int L, W;
    const int *len_own;   // valid owner-side length of each batch item (null: L), device memory [N / nh]
    const int *len_oth;   // valid other-side length of each batch item (null: L)
    int nh;               // problems per batch item (heads)
    float c2;         // log2(e) / (eps sqrt d)
    float cs;         // 1 / (eps sqrt d)
    int dustbin;
    float sdb2;       // dustbin score * log2(e)
    Vec spoke_own;    // learned dustbin token: score of the spoke (o, dustbin of the other side) per
                      // owner index, natural units (null: the scalar score above)
    const float *pay_db;  // APPLY with a learned token: payload row of the other side's dustbin [N][D]
    int nbp;          // workgroups per problem
    int nb_total;
    int rev;          // walk each XCD's share of the blocks backwards (alternates between launches)
};

// ------------------------------------------------------------------ element traits
template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int BYTES = 4;
};
template <> struct Elem<__bf16> {
    static constexpr int BYTES = 2;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// Valid lengths of problem n (padded batches, sequences of different lengths): Lt other-side
// indices exist, and Le owner indices have at least one band edge (o < Lo and o - W < Lt).
// Owner rows in [Le, L) take no part and get zeros.  Uniform over the workgroup.
struct Lens { int Lt, Le; };
__device__ __forceinline__ Lens problem_lens(const SweepArgs &a, int n)
{
    int Lo = a.L, Lt = a.L;
    if (a.len_own) Lo = min(max(a.len_own[n / a.nh], 0), a.L);
    if (a.len_oth) Lt = min(max(a.len_oth[n / a.nh], 0), a.L);
    return Lens{Lt, Lt > 0 ? min(Lo, Lt + a.W) : 0};
}
// A workgroup whose owner rows all lie beyond the valid length writes its zeros and leaves.
template <typename T, int D, int BM>
__device__ __forceinline__ void zero_block(const SweepArgs &a, int n, int o_blk, bool mat, bool vec)
{
    const int rows = min(BM, a.L - o_blk);
    if (mat && !a.accum) {
        uint4 *dst = reinterpret_cast<uint4 *>(reinterpret_cast<T *>(a.out_mat) + ((long)n * a.L + o_blk) * D);
        const int n16 = rows * D * (int)sizeof(T) / 16;
        for (int i = threadIdx.x; i < n16; i += NTHREADS) dst[i] = make_uint4(0, 0, 0, 0);
    }
    for (int i = threadIdx.x; i < rows; i += NTHREADS) {
        if (vec) a.out_vec.p[n * a.out_vec.stride + o_blk + i] = 0.f;
        if (mat && a.dot_mat) a.dot_out.p[n * a.dot_out.stride + o_blk + i] = 0.f;
    }
}

__device__ __forceinline__ bf16x8 pack8(const float *e)
{
    bf16x8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = (__bf16)e[i];
    return r;
}

// LDS layouts -------------------------------------------------------------------
// bf16 row-major tile [32][D]: 16-byte chunks XOR-swizzled so that the 32 lanes of
// an A-fragment read (one chunk per lane, consecutive rows) spread over all banks.
template <int D> __device__ __forceinline__ int bf16_chunk_off(int row, int chunk)
{
    constexpr int CH = D / 8;                       // chunks per row
    constexpr int RPB = (CH >= 8) ? 1 : 8 / CH;     // rows per 128-byte line
    constexpr int MASK = (CH >= 8) ? 7 : CH - 1;
    return (row * CH + (chunk ^ ((row / RPB) & MASK))) * 16;
}
// bf16 transposed payload tile [D][32 + 4] (t contiguous, 72-byte rows)
constexpr int PT_STRIDE = 72;
// fp32 row-major tile [32][D + 4]
template <int D> constexpr int f32_row_floats() { return D + 4; }

template <typename T, int D> struct Tile {
    static constexpr bool IS_BF16 = (Elem<T>::BYTES == 2);
    static constexpr int RM_BYTES = IS_BF16 ? 32 * D * 2 : 32 * f32_row_floats<D>() * 4;
    static constexpr int PT_BYTES = IS_BF16 ? D * PT_STRIDE : RM_BYTES;
    static constexpr int CHUNKS = 32 * D * Elem<T>::BYTES / 16;       // 16-byte pieces per tile
    static constexpr int CPT = (CHUNKS + NTHREADS - 1) / NTHREADS;    // per thread
    static constexpr int CPR = D * Elem<T>::BYTES / 16;               // per row
};

template <typename T, int D> using TileRegs = uint4[Tile<T, D>::CPT];

// ------------------------------------------------------------------ staging
// Global -> registers for one 32-row tile of a [L][D] matrix (rows beyond L read as 0).
template <typename T, int D>
__device__ __forceinline__ void tile_load(TileRegs<T, D> &reg, const T *base, int t0, int L)
{
    using TL = Tile<T, D>;
#pragma unroll
    for (int c = 0; c < TL::CPT; ++c) {
        int idx = threadIdx.x + c * NTHREADS;
        int row = idx / TL::CPR, ch = idx % TL::CPR;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (idx < TL::CHUNKS && t0 + row < L)
            v = *reinterpret_cast<const uint4 *>(base + (long)(t0 + row) * D + ch * (16 / Elem<T>::BYTES));
        reg[c] = v;
    }
}

// registers -> LDS, row-major (A-operand of the score / Z products)
template <typename T, int D>
__device__ __forceinline__ void tile_store_rm(const TileRegs<T, D> &reg, unsigned char *lds)
{
    using TL = Tile<T, D>;
#pragma unroll
    for (int c = 0; c < TL::CPT; ++c) {
        int idx = threadIdx.x + c * NTHREADS;
        if (idx < TL::CHUNKS) {
            int row = idx / TL::CPR, ch = idx % TL::CPR;
            if constexpr (TL::IS_BF16)
                *reinterpret_cast<uint4 *>(lds + bf16_chunk_off<D>(row, ch)) = reg[c];
            else
                *reinterpret_cast<uint4 *>(lds + (row * f32_row_floats<D>() + ch * 4) * 4) = reg[c];
        }
    }
}

// registers -> LDS in the layout the second product wants: bf16 transposed [dv][t],
// fp32 row-major.
template <typename T, int D>
__device__ __forceinline__ void tile_store_pay(const TileRegs<T, D> &reg, unsigned char *lds)
{
    using TL = Tile<T, D>;
    if constexpr (!TL::IS_BF16) {
        tile_store_rm<T, D>(reg, lds);
    } else {
#pragma unroll
        for (int c = 0; c < TL::CPT; ++c) {
            int idx = threadIdx.x + c * NTHREADS;
            if (idx < TL::CHUNKS) {
                int row = idx / TL::CPR, ch = idx % TL::CPR;
                const unsigned int wds[4] = {reg[c].x, reg[c].y, reg[c].z, reg[c].w};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    unsigned short v = (unsigned short)(wds[e >> 1] >> ((e & 1) * 16));
                    *reinterpret_cast<unsigned short *>(lds + (ch * 8 + e) * PT_STRIDE + row * 2) = v;
                }
            }
        }
    }
}

// ------------------------------------------------------------------ fragments
// Owner-side fragment kept in registers for the whole sweep (B operand, columns o).
template <typename T, int D> struct OwnerFrag;
template <int D> struct OwnerFrag<__bf16, D> {
    bf16x8 v[D / 16];
    __device__ __forceinline__ void load(const __bf16 *base, int o, int L, int h)
    {
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            uint4 z = make_uint4(0, 0, 0, 0);
            if (o < L) z = *reinterpret_cast<const uint4 *>(base + (long)o * D + (2 * s + h) * 8);
            v[s] = *reinterpret_cast<bf16x8 *>(&z);
        }
    }
};
template <int D> struct OwnerFrag<float, D> {
    float v[D / 2];   // feature k = h*D/2 + s
    __device__ __forceinline__ void load(const float *base, int o, int L, int h)
    {
#pragma unroll
        for (int q = 0; q < D / 8; ++q) {
            float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
            if (o < L) z = *reinterpret_cast<const float4 *>(base + (long)o * D + h * (D / 2) + 4 * q);
            v[4 * q + 0] = z.x; v[4 * q + 1] = z.y; v[4 * q + 2] = z.z; v[4 * q + 3] = z.w;
        }
    }
};

// acc[t, o] += sum_k tile[t][k] * frag[o][k]
template <int D>
__device__ __forceinline__ f32x16 tile_dot(const unsigned char *tile, const OwnerFrag<__bf16, D> &x,
                                           int lane, f32x16 acc)
{
    const int t = lane & 31, h = lane >> 5;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
        bf16x8 a = *reinterpret_cast<const bf16x8 *>(tile + bf16_chunk_off<D>(t, 2 * s + h));
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, x.v[s], acc, 0, 0, 0);
    }
    return acc;
}
template <int D>
__device__ __forceinline__ f32x16 tile_dot(const unsigned char *tile, const OwnerFrag<float, D> &x,
                                           int lane, f32x16 acc)
{
    const int t = lane & 31, h = lane >> 5;
    const float *row = reinterpret_cast<const float *>(tile) + t * f32_row_floats<D>() + h * (D / 2);
#pragma unroll
    for (int q = 0; q < D / 8; ++q) {
        float4 a = *reinterpret_cast<const float4 *>(row + 4 * q);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, x.v[4 * q + 0], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, x.v[4 * q + 1], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, x.v[4 * q + 2], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, x.v[4 * q + 3], acc, 0, 0, 0);
    }
    return acc;
}

// FR score tiles at once from one other-side tile of a ring kernel (rows ROWB bytes apart,
// no swizzle): the tile's fragments are read from LDS once and every product chain is
// issued before any of them is consumed.
template <int D, int FR, int ROWB>
__device__ __forceinline__ void ring_dot_multi(const unsigned char *tile, const OwnerFrag<__bf16, D> (&x)[FR],
                                               int lane, f32x16 (&acc)[FR])
{
    const unsigned char *row = tile + (lane & 31) * ROWB + (lane >> 5) * 16;
    bf16x8 a[D / 16];
#pragma unroll
    for (int s = 0; s < D / 16; ++s) a[s] = *reinterpret_cast<const bf16x8 *>(row + 32 * s);
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
#pragma unroll
        for (int f = 0; f < FR; ++f)
            acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s], x[f].v[s], acc[f], 0, 0, 0);
}
template <int D, int FR, int ROWB>
__device__ __forceinline__ void ring_dot_multi(const unsigned char *tile, const OwnerFrag<float, D> (&x)[FR],
                                               int lane, f32x16 (&acc)[FR])
{
    static_assert(ROWB == f32_row_floats<D>() * 4, "fp32 ring tiles use the padded fp32 layout");
#pragma unroll
    for (int f = 0; f < FR; ++f) acc[f] = tile_dot<D>(tile, x[f], lane, acc[f]);
}

// out[dvt][dv, o] += sum_t pay[t][dv] * e[t, o]   (e in the accumulator layout)
template <typename T, int D>
__device__ __forceinline__ void tile_accum(f32x16 (&out)[D / 32], const unsigned char *pay,
                                           const float (&e)[16], int lane)
{
    const int c = lane & 31, h = lane >> 5;
    if constexpr (Elem<T>::BYTES == 2) {
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            bf16x8 pf = pack8(&e[8 * m]);
#pragma unroll
            for (int dvt = 0; dvt < D / 32; ++dvt) {
                const unsigned char *rowp = pay + (32 * dvt + c) * PT_STRIDE;
                uint2 lo = *reinterpret_cast<const uint2 *>(rowp + (16 * m + 4 * h) * 2);
                uint2 hi = *reinterpret_cast<const uint2 *>(rowp + (16 * m + 8 + 4 * h) * 2);
                uint4 both = make_uint4(lo.x, lo.y, hi.x, hi.y);
                bf16x8 af = *reinterpret_cast<bf16x8 *>(&both);
                out[dvt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, pf, out[dvt], 0, 0, 0);
            }
        }
    } else {
        const float *p = reinterpret_cast<const float *>(pay);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int t = 8 * (r >> 2) + 4 * h + (r & 3);
#pragma unroll
            for (int dvt = 0; dvt < D / 32; ++dvt) {
                float a = p[t * f32_row_floats<D>() + 32 * dvt + c];
                out[dvt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, e[r], out[dvt], 0, 0, 0);
            }
        }
    }
}

template <typename T> __device__ __forceinline__ void store4(T *dst, float a, float b, float c, float d);
template <> __device__ __forceinline__ void store4<float>(float *dst, float a, float b, float c, float d)
{
    *reinterpret_cast<float4 *>(dst) = make_float4(a, b, c, d);
}
template <> __device__ __forceinline__ void store4<__bf16>(__bf16 *dst, float a, float b, float c, float d)
{
    bf16x4 v = {(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};
    *reinterpret_cast<bf16x4 *>(dst) = v;
}
template <typename T> __device__ __forceinline__ void load4(const T *src, float (&f)[4]);
template <> __device__ __forceinline__ void load4<float>(const float *src, float (&f)[4])
{
    float4 v = *reinterpret_cast<const float4 *>(src);
    f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
}
template <> __device__ __forceinline__ void load4<__bf16>(const __bf16 *src, float (&f)[4])
{
    bf16x4 v = *reinterpret_cast<const bf16x4 *>(src);
#pragma unroll
    for (int i = 0; i < 4; ++i) f[i] = (float)v[i];
}

// ------------------------------------------------------------------ the generic sweep kernel
// Double-buffered LDS staging, one other-side tile per barrier.  It serves the first row
// half-step (running-maximum LSE, no potentials yet), every fp32-storage matrix sweep
// and the bf16 matrix sweeps at d = 128; the ring kernels below take the rest.
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
    constexpr bool MAT_OUT = (MODE == M_APPLY || MODE == M_FINAL);

    extern __shared__ __align__(16) unsigned char smem[];   // two stages of ST::BYTES
    __shared__ float red[NWAVES];

    // XCD-aware placement: hardware deals workgroups round-robin over the 8 XCDs, so
    // give each XCD one contiguous eighth of the (problem, block) sequence; neighbours
    // that share band rows then meet in the same L2.
    const int chunk = (a.nb_total + 7) >> 3;
    const int lb = (blockIdx.x & 7) * chunk + (a.rev ? chunk - 1 - (int)(blockIdx.x >> 3) : (int)(blockIdx.x >> 3));
    if (lb >= a.nb_total) return;
    const int n = lb / a.nbp;
    const int o_blk = (lb % a.nbp) * BM;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int L = a.L, W = a.W;
    const Lens ln = problem_lens(a, n);
    const int Lt = ln.Lt, Le = ln.Le;
    if (o_blk >= Le) {
        zero_block<T, D, BM>(a, n, o_blk, MAT_OUT, !MAT_OUT);
        return;
    }
    const long moff = (long)n * L * D;
    const T *Xb = reinterpret_cast<const T *>(a.X) + moff;
    const T *Yb = reinterpret_cast<const T *>(a.Y) + moff;
    const float *ytp = a.yt.p + n * a.yt.stride;
    // owner-side potential: stabiliser and factor of the plan; -inf marks an inactive token (a
    // masked one, or one without any active partner), which stays inactive in every later
    // iterate.  The first half-step has no previous iterate: there xs only carries the marks.
    const float *xsp = a.xs.p ? a.xs.p + n * a.xs.stride : nullptr;

    // workgroup stabiliser: largest owner-side potential in this block
    float mblk = 0.f;
    if constexpr (MODE != M_LSE_FIRST) {
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
    float sum[FR], mx[FR];
    f32x16 outm[MAT_OUT ? FR : 1][D / 32];
#pragma unroll
    for (int f = 0; f < FR; ++f) {
        sum[f] = 0.f;
        mx[f] = -INFINITY;
        if constexpr (MAT_OUT)
#pragma unroll
            for (int j = 0; j < D / 32; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) outm[f][j][r] = 0.f;
    }

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

            if constexpr (MODE == M_LSE_FIRST) {
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
        if constexpr (MODE == M_LSE_FIRST) {
            float mo = __shfl_xor(mx[f], 32), so = __shfl_xor(sum[f], 32);
            float mn = fmaxf(mx[f], mo);
            float tot = sum[f] * fast_exp2(mx[f] - mn) + so * fast_exp2(mo - mn);
            if (a.dustbin) {   // spoke edge (o, dustbin): score sdb, other-side potential yt[L]
                const float sp2 = a.spoke_own.p ? a.spoke_own.p[n * a.spoke_own.stride + min(o, L - 1)] * LOG2E : a.sdb2;
                float xd = sp2 + ytp[L] * LOG2E;
                float m3 = fmaxf(mn, xd);
                tot = tot * fast_exp2(mn - m3) + fast_exp2(xd - m3);
                mn = m3;
            }
            if (h == 0 && o < L) {
                float r = 0.f;   // rows beyond the valid length
                if (o < Le) {
                    if ((xsp && xsp[o] == -INFINITY) || !(mn > -INFINITY)) {
                        r = -INFINITY;   // inactive token
                    } else {
                        r = -LN2 * (mn + fast_log2(tot));
                        if (a.olog.p) r += a.olog.p[n * a.olog.stride + o];
                    }
                }
                a.out_vec.p[n * a.out_vec.stride + o] = r;
            }
        } else {
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

// ------------------------------------------------------------------ vector sweeps
// Scaling sweep (M_LSE) and band mat-vec (M_MATVEC): the result is one scalar per
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

template <typename T, int D, int MODE, int FR>
__global__ __launch_bounds__(NTHREADS) void vsweep_kernel(const SweepArgs a)
{
    using TL = Tile<T, D>;
    using RG = VRing<T, D, MODE, FR>;
    constexpr bool PRE = (sizeof(T) == 2);   // bf16 storage: the score operand is prescaled, c2 == 1
    constexpr int BM = NWAVES * FR * 32;
    static_assert(MODE == M_LSE || MODE == M_MATVEC, "vector sweeps only");

    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ float red[NWAVES];

    const int chunk = (a.nb_total + 7) >> 3;
    const int lb = (blockIdx.x & 7) * chunk + (a.rev ? chunk - 1 - (int)(blockIdx.x >> 3) : (int)(blockIdx.x >> 3));
    if (lb >= a.nb_total) return;
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
    const float *xsp = a.xs.p + n * a.xs.stride;
    const float *wp = (MODE == M_MATVEC) ? a.w.p + n * a.w.stride : nullptr;


    // stabiliser input first, so that waiting for it waits for nothing else
    static_assert(BM <= NTHREADS, "one owner-side potential per thread");
    float mraw = xsp[min(o_blk + min(tid, BM - 1), Le - 1)];   // clamped repeats are harmless
    float mblk, m2 = 0.f;
    OwnerFrag<T, D> xf[FR];
    int o_frag[FR];
    float sum[FR];
#pragma unroll
    for (int f = 0; f < FR; ++f) {
        o_frag[f] = o_blk + (wave * FR + f) * 32;
        xf[f].load(Xb, min(o_frag[f] + c, Le - 1), Le, h);   // clamped: rows beyond Le are written as zeros
        sum[f] = 0.f;
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
    auto g_load = [&](Inflight &g, int k) {
        const int kc = min(max(k, 0), klast);
        const int rows = min(TT, Lt - kc * TT);   // >= 1
        g.rows = (k == kc) ? rows : 0;
        const unsigned char *tb = reinterpret_cast<const unsigned char *>(Yb) + (long)kc * TILE_BYTES;
        const unsigned lim = rows * ROW_BYTES - 16;
#pragma unroll
        for (int q = 0; q < TL::CPT; ++q) g.y[q] = *reinterpret_cast<const uint4 *>(tb + min(goff[q], lim));
        const unsigned vo = min(vrow, (unsigned)(rows - 1)) * 4;
        g.vy = *reinterpret_cast<const float *>(reinterpret_cast<const unsigned char *>(ytp + kc * TT) + vo);
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
    {
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

    for (int s = 0; s < S; ++s) {
        // the next tile is requested in every step, also when no later step reads it (its
        // address is clamped, its ring slot is free): a load under a condition would make
        // the compiler wait for it at once instead of at the store below
        const int jnew = s + 1 + RG::LEAD;
        g_load(nxt, kbase + jnew);

        const int j = s + wave * FR;
        const int k = kbase + j;
        if (k >= 0 && k <= klast) {
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
                const int of = o_frag[f];
                use[f] = !(of >= Le || t0 + TT - 1 < of - W || t0 > of + 31 + W);
                interior[f] = (of + 31 - t0 <= W) && (t0 + TT - 1 - of <= W);
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
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = fast_exp2(e[r]);
                    if constexpr (MODE == M_MATVEC) sum[f] = fmaf(p, wv[r], sum[f]);
                    else sum[f] += p;
                }
            }
        }
        s_store(nxt, jnew);
        __syncthreads();
    }

#pragma unroll
    for (int f = 0; f < FR; ++f) {
        const int o = o_frag[f] + c;
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
            } else if (xsp[o] == -INFINITY || (MODE == M_LSE && !(tot > 0.f))) {
                r = (MODE == M_LSE) ? -INFINITY : 0.f;   // inactive token (stays so), or none of its partners is active
            } else if constexpr (MODE == M_LSE) {
                r = mblk - LN2 * fast_log2(tot);
                if (a.olog.p) r += a.olog.p[n * a.olog.stride + o];
            } else {
                float pre = a.pre.p ? a.pre.p[n * a.pre.stride + o] : 0.f;
                r = pre - fast_exp2((xsp[o] - mblk) * LOG2E) * tot;
                if (a.olog.p) r *= __expf(-a.olog.p[n * a.olog.stride + o]);
            }
            a.out_vec.p[n * a.out_vec.stride + o] = r;
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

    // epilogue: owner-side factor, store (and the <dot_mat_o, out_o> reduction for dV)
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
        const T *drow = a.dot_mat ? reinterpret_cast<const T *>(a.dot_mat) + moff + (long)oc * D : nullptr;
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
__global__ void rowdot_kernel(const T *A, const T *Bm, float *g, long gstride, int L, int Lp, const int *len, int nh)
{
    constexpr int LPR = D * (int)sizeof(T) / 16;   // lanes per row: 4 ... 32, a power of two
    constexpr int EPL = 16 / (int)sizeof(T);       // elements per lane
    const int n = blockIdx.y;
    const long p = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int o = (int)(p / LPR), sub = (int)(p % LPR);
    float acc = 0.f;
    const int Lv = len ? min(max(len[n / nh], 0), L) : L;
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

// Dustbin element of a sweep result: the extra row (column) is joined to every
// index 0..L of the other side by an edge of score s_t (the scalar sdb, or spoke[t] when
// the dustbin is a learned token).
//   w == null: out[L] = -log sum_{t<=L} exp(s_t + y_t)
//   else     : out[L] = pre - exp(x[L]) sum_{t<=L} exp(s_t + y_t) w_t   (pre = 0)
__global__ __launch_bounds__(1024) void dustbin_kernel(Vec y, Vec w, Vec x, VecOut out, int L, float sdb, Vec spoke)
{
    __shared__ float sm[32], ss[32];
    const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const float *yp = y.p + n * y.stride;
    const float *sp = spoke.p ? spoke.p + n * spoke.stride : nullptr;
    if (sp) sdb = 0.f;
    float m = -INFINITY;
    for (int t = tid; t <= L; t += blockDim.x) m = fmaxf(m, yp[t] + (sp ? sp[t] : 0.f));
    for (int s = 32; s >= 1; s >>= 1) m = fmaxf(m, __shfl_xor(m, s));
    if (lane == 0) sm[wv] = m;
    __syncthreads();
    m = sm[0];
    for (int i = 1; i < (int)(blockDim.x >> 6); ++i) m = fmaxf(m, sm[i]);
    float acc = 0.f;
    for (int t = tid; t <= L; t += blockDim.x) {
        float e = __expf(yp[t] + (sp ? sp[t] : 0.f) - m);
        acc += w.p ? e * w.p[n * w.stride + t] : e;
    }
    for (int s = 32; s >= 1; s >>= 1) acc += __shfl_xor(acc, s);
    if (lane == 0) ss[wv] = acc;
    __syncthreads();
    if (tid == 0) {
        float tot = 0.f;
        for (int i = 0; i < (int)(blockDim.x >> 6); ++i) tot += ss[i];
        float r;
        if (!w.p) r = -(sdb + m + __logf(tot));
        else r = -__expf(x.p[n * x.stride + L] + sdb + m) * tot;
        out.p[n * out.stride + L] = r;
    }
}

// ------------------------------------------------------------------ host side
struct Problem {
    int B, H, L, d, W, T, R, dustbin, dtype;
    float eps, sdb;
    const float *log_a = nullptr, *log_b = nullptr;   // [N][Lp] logs of the marginal targets, or null
    const int *len_q = nullptr, *len_k = nullptr;     // [B] valid lengths of the two sequences, or null
    int variant = 0;                                  // backward: SKA_BWD_* (comparators of the final sweeps)
    const unsigned char *mask_q = nullptr, *mask_k = nullptr;        // [B][L] token activity (forward), or null
    const float *q_db = nullptr, *k_db = nullptr, *v_db = nullptr;   // learned dustbin tokens [N][d] fp32, or null
    float *dq_db = nullptr, *dk_db = nullptr, *dv_db = nullptr;      //   and their gradients (backward)
    bool token() const { return q_db != nullptr; }
    int n_stages = 0;                                 // forward: continuation schedule of the base solve
    const float *eps_stage = nullptr;                 //   (host arrays; 0 stages: T steps at eps)
    const int *T_stage = nullptr;
    bool direct() const { return variant == SKA_BWD_DIRECT; }
    int N() const { return B * H; }
    int Lp() const { return L + (dustbin ? 1 : 0); }
    long ldw() const { return ((long)Lp() + 3) / 4 * 4; }  // stride of workspace vectors
};

// workspace vectors of the backward: g_u, then vbar_R, ubar_R, vbar_{R-1}, ubar_{R-1}, ..., vbar_1, ubar_1
inline int ws_vecs(int R) { return 1 + 2 * R; }
inline int pack_groups(int R) { return (2 * R + 3) / 4; }
// bf16 storage: both directions keep a prescaled copy of Q in the workspace
size_t ws_qs_bytes(const Problem &p)
{
    return p.dtype == SKA_BF16 ? (size_t)p.N() * p.L * p.d * 2 : 0;
}
size_t ws_vec_bytes(const Problem &p)
{
    // 1 + 2R vectors, two packs of R float4 groups (the one-reference sweeps use the first
    // (2R + 3) / 4 of them, the direct comparator all), four packs of 16 bf16 columns
    return (size_t)p.N() * p.ldw() * (ws_vecs(p.R) * sizeof(float) + 2 * p.R * sizeof(float4) + 4 * 32);
}
// dustbin: spoke score vectors SQ, SK and spoke cotangents sbr, sbc (stride ldw), and the partial
// sums of the weighted row sums (learned tokens only, but sized by the flag alone)
inline int ws_chunks(const Problem &p) { return (p.L + WS_ROWS - 1) / WS_ROWS; }
size_t ws_tok_bytes(const Problem &p)
{
    return p.dustbin ? ((size_t)4 * p.N() * p.ldw() + (size_t)p.N() * ws_chunks(p) * p.d) * sizeof(float) : 0;
}
size_t ws_bytes(const Problem &p) { return ws_vec_bytes(p) + ws_qs_bytes(p) + ws_tok_bytes(p); }
inline float *ws_tok(const Problem &p, void *ws)
{
    return reinterpret_cast<float *>(reinterpret_cast<unsigned char *>(ws) + ws_vec_bytes(p) + ws_qs_bytes(p));
}
// spoke scores of the learned tokens: SQ[i] = c q_i.k_db, SK[j] = c q_db.k_j, SQ[L] = SK[L] = c q_db.k_db
template <typename T, int D>
int spoke_scores(const Problem &p, const void *Qin, const void *K, float *SQ, float *SK, hipStream_t st)
{
    constexpr int LPR = D * (int)sizeof(T) / 16;
    const float cs = 1.f / (p.eps * sqrtf((float)p.d));
    const dim3 grid((unsigned)(((long)(p.L + 1) * LPR + 255) / 256), p.N());
    hipLaunchKernelGGL((spoke_scores_kernel<T, D>), grid, dim3(256), 0, st, reinterpret_cast<const T *>(Qin), p.k_db,
                       p.q_db, SQ, p.ldw(), p.L, cs);
    hipLaunchKernelGGL((spoke_scores_kernel<T, D>), grid, dim3(256), 0, st, reinterpret_cast<const T *>(K), p.q_db,
                       p.k_db, SK, p.ldw(), p.L, cs);
    return hipGetLastError() == hipSuccess ? SKA_OK : SKA_EHIP;
}

template <typename T>
int make_scores_operand(const Problem &p, float eps, const void *Q, void *ws_qs, const void **Qs, float *c2,
                        hipStream_t st)
{
    const float cs = 1.f / (eps * sqrtf((float)p.d));
    if constexpr (sizeof(T) == 2) {
        const long n8 = (long)p.N() * p.L * p.d / 8;
        hipLaunchKernelGGL(prescale_kernel, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, st,
                           reinterpret_cast<const __bf16 *>(Q), reinterpret_cast<__bf16 *>(ws_qs), n8, cs * LOG2E);
        if (hipGetLastError() != hipSuccess) return SKA_EHIP;
        *Qs = ws_qs;
        *c2 = 1.f;
    } else {
        *Qs = Q;
        *c2 = cs * LOG2E;
    }
    return SKA_OK;
}

int check_common(const Problem &p)
{
    if (p.B < 1 || p.H < 1 || p.L < 1 || p.W < 0 || p.T < 0) return SKA_EINVAL;
    if (!(p.eps > 0.f) || !isfinite(p.eps) || !isfinite(p.sdb)) return SKA_EINVAL;
    if ((long)p.B * p.H > 65535) return SKA_EINVAL;
    if (p.L > (1 << 24)) return SKA_EUNSUPPORTED;   // 32-bit byte offsets inside one [L][d] matrix
    if ((p.log_a || p.log_b) && p.dustbin) return SKA_EUNSUPPORTED;   // the dustbin's targets are all one
    if ((p.len_q || p.len_k) && p.dustbin) return SKA_EUNSUPPORTED;   // the dustbin sits at index L
    if ((p.mask_q || p.mask_k) && p.dustbin) return SKA_EUNSUPPORTED;
    if (p.token() && (!p.dustbin || p.n_stages || p.variant != SKA_BWD_ONE_REFERENCE)) return SKA_EUNSUPPORTED;
    if (p.R < 1 || p.R > MAXR) return SKA_EUNSUPPORTED;
    if (p.d != 32 && p.d != 64 && p.d != 128) return SKA_EUNSUPPORTED;
    if (p.dtype != SKA_F32 && p.dtype != SKA_BF16) return SKA_EUNSUPPORTED;
    return SKA_OK;
}

template <typename T, int D, int MODE, int FR, bool DIRECT = false>
int launch_sweep(SweepArgs a, int N, hipStream_t st)
{
    constexpr int BM = NWAVES * FR * 32;
    a.nbp = (a.L + BM - 1) / BM;
    a.nb_total = a.nbp * N;
    const int chunk = (a.nb_total + 7) / 8;
    constexpr int LDS = 2 * Stage<T, D, MODE>::BYTES;
    static bool raised = false;    // static LDS tops out at 64 KB; the CU has 160 KB
    if (LDS > 48 * 1024 && !raised) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&sweep_kernel<T, D, MODE, FR, DIRECT>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS) != hipSuccess)
            return SKA_EHIP;
        raised = true;
    }
    hipLaunchKernelGGL((sweep_kernel<T, D, MODE, FR, DIRECT>), dim3(chunk * 8), dim3(NTHREADS), LDS, st, a);
    return hipGetLastError() == hipSuccess ? SKA_OK : SKA_EHIP;
}

template <typename T, int D, int MODE, int FR>
int launch_vsweep(SweepArgs a, int N, hipStream_t st)
{
    constexpr int BM = NWAVES * FR * 32;
    a.nbp = (a.L + BM - 1) / BM;
    a.nb_total = a.nbp * N;
    const int chunk = (a.nb_total + 7) / 8;
    constexpr int LDS = VRing<T, D, MODE, FR>::BYTES;
    static bool raised = false;
    if (LDS > 48 * 1024 && !raised) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&vsweep_kernel<T, D, MODE, FR>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS) != hipSuccess)
            return SKA_EHIP;
        raised = true;
    }
    hipLaunchKernelGGL((vsweep_kernel<T, D, MODE, FR>), dim3(chunk * 8), dim3(NTHREADS), LDS, st, a);
    return hipGetLastError() == hipSuccess ? SKA_OK : SKA_EHIP;
}

template <int D, int MODE, int FR>
int launch_msweep(SweepArgs a, int N, hipStream_t st)
{
    constexpr int BM = NWAVES * FR * 32;
    a.nbp = (a.L + BM - 1) / BM;
    a.nb_total = a.nbp * N;
    const int chunk = (a.nb_total + 7) / 8;
    constexpr int LDS = MRing<D, MODE, FR>::BYTES;
    static bool raised = false;
    if (LDS > 48 * 1024 && !raised) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&msweep_kernel<D, MODE, FR>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS) != hipSuccess)
            return SKA_EHIP;
        raised = true;
    }
    hipLaunchKernelGGL((msweep_kernel<D, MODE, FR>), dim3(chunk * 8), dim3(NTHREADS), LDS, st, a);
    return hipGetLastError() == hipSuccess ? SKA_OK : SKA_EHIP;
}

// Which kernel runs which sweep:
//   scaling sweeps and band mat-vecs      vsweep_kernel (skewed LDS ring), both storage types
//   output map / dV, final sweeps         msweep_kernel for bf16 storage with d <= 64,
//                                         sweep_kernel otherwise
//   the very first half-step              sweep_kernel<M_LSE_FIRST> (running maximum)
template <typename T, int D> int sweep(int mode, const SweepArgs &a, int N, hipStream_t st)
{
    constexpr int FRV = (sizeof(T) == 2) ? 2 : 1;   // vector sweeps: owner rows per wavefront / 32
    switch (mode) {
    case M_LSE_FIRST: return launch_sweep<T, D, M_LSE_FIRST, FRV>(a, N, st);
    case M_LSE: return launch_vsweep<T, D, M_LSE, FRV>(a, N, st);
    case M_MATVEC: return launch_vsweep<T, D, M_MATVEC, FRV>(a, N, st);
    case M_APPLY:
        if constexpr (sizeof(T) == 2 && D <= 64) return launch_msweep<D, M_APPLY, 2>(a, N, st);
        else return launch_sweep<T, D, M_APPLY, 1>(a, N, st);
    case M_FINAL_DIRECT: return launch_sweep<T, D, M_FINAL, 1, true>(a, N, st);
    default:
        if constexpr (sizeof(T) == 2 && D <= 64) {
            if (a.poB) return launch_msweep<D, M_FINAL, 1>(a, N, st);   // packs as bf16 columns (R <= 2)
        }
        return launch_sweep<T, D, M_FINAL, 1>(a, N, st);
    }
}

// benchmark hooks: while enabled, every phase of a call is bracketed by two events on the
// call's stream, so that the phases can be timed in place inside a larger timed region
struct ProfSpan { hipEvent_t a, b; int phase; long launches; };
int g_prof_on = 0;   // 0 off, 1 the scaling-sweep run only, 2 every phase
constexpr int PROF_MAX = 4096;
ProfSpan g_prof[PROF_MAX];
int g_prof_n = 0;

struct PhaseTimer {
    ProfSpan *sp = nullptr;
    hipStream_t st;
    PhaseTimer(int phase, hipStream_t st_) : st(st_)
    {
        if (g_prof_on < (phase == SKA_PH_SCALING ? 1 : 2) || g_prof_n >= PROF_MAX) return;
        ProfSpan *c = &g_prof[g_prof_n];
        if (hipEventCreate(&c->a) != hipSuccess) return;
        if (hipEventCreate(&c->b) != hipSuccess) { (void)hipEventDestroy(c->a); return; }
        c->phase = phase;
        c->launches = 0;
        (void)hipEventRecord(c->a, st);
        sp = c;
        ++g_prof_n;
    }
    void launched(long n = 1) { if (sp) sp->launches += n; }
    void end() { if (sp) { (void)hipEventRecord(sp->b, st); sp = nullptr; } }
    ~PhaseTimer() { end(); }
};

#define SKA_TRY(x)                      \
    do {                                \
        int rc_ = (x);                  \
        if (rc_ != SKA_OK) return rc_;  \
    } while (0)

template <typename T, int D>
int fwd_impl(const Problem &p, const void *Qin, const void *K, const void *V, void *O, float *UV,
             void *ws, hipStream_t st)
{
    // Q below is the score operand: for bf16 storage the prescaled copy, with c2 = 1
    const void *Q = nullptr;
    float c2 = 0.f;
    {
        PhaseTimer pt(SKA_PH_PRESCALE, st);
        SKA_TRY((make_scores_operand<T>(p, p.n_stages ? p.eps_stage[0] : p.eps, Qin, ws, &Q, &c2, st)));
        pt.launched(sizeof(T) == 2 ? 1 : 0);
    }
    const int N = p.N(), L = p.L, Lp = p.Lp();
    const int R = p.R;
    const long us = 2L * (R + 1) * Lp;
    auto vec = [&](int k) { return Vec{UV + (long)k * Lp, us}; };   // slot 2t: u_t, slot 2t + 1: v_t
    auto vout = [&](int k) { return VecOut{UV + (long)k * Lp, us}; };
    SweepArgs base{};
    base.L = L; base.W = p.W < L ? p.W : L;   // |i-j| <= L-1 always: W >= L is the dense problem
    base.cs = 1.f / (p.eps * sqrtf((float)p.d));
    base.c2 = c2;
    base.dustbin = p.dustbin; base.sdb2 = p.sdb * LOG2E;
    base.nh = p.H;

    // u0 = v0 = 0: the base solve starts from v = 0
    {
        long tot = 2L * Lp * N;
        hipLaunchKernelGGL(fill_kernel, dim3((tot + 255) / 256), dim3(256), 0, st, UV, 2L * Lp, us, N, 0.f);
        if (hipGetLastError() != hipSuccess) return SKA_EHIP;
    }
    if (p.mask_q || p.mask_k) {   // inactive tokens start, and stay, at -inf
        hipLaunchKernelGGL(mask_fill_kernel, dim3((L + 255) / 256, N), dim3(256), 0, st, UV, us, Lp, L, p.mask_q,
                           p.mask_k, p.H);
        if (hipGetLastError() != hipSuccess) return SKA_EHIP;
    }
    bool first = true;
    int nlaunch = 0;
    PhaseTimer pt_first(SKA_PH_FIRST, st);   // the first launch is the other (max-tracking) kernel
    PhaseTimer *pt_run = nullptr;
    alignas(PhaseTimer) unsigned char pt_run_mem[sizeof(PhaseTimer)];
    // half-step: out slot <- -LSE over the band of (S + yt); prev slot only stabilises
    // learned dustbin tokens: spoke score vectors instead of the scalar score
    Vec SQ{nullptr, 0}, SK{nullptr, 0};
    if (p.token()) {
        float *tok = ws_tok(p, ws);
        SQ = Vec{tok, p.ldw()};
        SK = Vec{tok + (long)N * p.ldw(), p.ldw()};
        SKA_TRY((spoke_scores<T, D>(p, Qin, K, tok, tok + (long)N * p.ldw(), st)));
    }
    float stage_c2 = c2, stage_sdb2 = base.sdb2;   // (a continuation stage has its own score scale)
    auto half = [&](bool row, int yslot, int prevslot, int outslot) -> int {
        SweepArgs a = base;
        a.c2 = stage_c2; a.sdb2 = stage_sdb2;
        a.spoke_own = row ? SQ : SK;
        a.X = row ? Q : K; a.Y = row ? K : Q;
        a.yt = vec(yslot); a.xs = vec(prevslot); a.out_vec = vout(outslot);
        a.olog = Vec{row ? p.log_a : p.log_b, (long)Lp};
        a.len_own = row ? p.len_q : p.len_k; a.len_oth = row ? p.len_k : p.len_q;
        // successive sweeps walk the blocks in opposite directions: a sweep then starts on
        // the rows its predecessor touched last, which are still in L2
        a.rev = nlaunch++ & 1;
        SKA_TRY((sweep<T, D>(first ? M_LSE_FIRST : M_LSE, a, N, st)));
        if (first) pt_first.launched();
        else pt_run->launched();
        if (p.dustbin) {
            hipLaunchKernelGGL(dustbin_kernel, dim3(N), dim3(1024), 0, st, vec(yslot), Vec{nullptr, 0},
                               Vec{nullptr, 0}, vout(outslot), L, stage_sdb2 * LN2, row ? SK : SQ);
            if (hipGetLastError() != hipSuccess) return SKA_EHIP;
        }
        if (first) {   // the run of identical scaling sweeps starts after the first launch
            first = false;
            pt_first.end();
            pt_run = new (pt_run_mem) PhaseTimer(SKA_PH_SCALING, st);
        }
        return SKA_OK;
    };
    auto halves = [&]() -> int {
        // base solve: T steps at eps, or the stages of the continuation schedule (remark
        // "Fixed-Budget eps-Scaling"): stage s runs on the scores A / eps_s; between stages both
        // potentials are carried in cost units, x -> x eps_s / eps_{s+1} (u only stabilises)
        const int nst = p.n_stages ? p.n_stages : 1;
        for (int sidx = 0; sidx < nst; ++sidx) {
            const float es = p.n_stages ? p.eps_stage[sidx] : p.eps;
            const int Ts = p.n_stages ? p.T_stage[sidx] : p.T;
            if (sidx > 0) {
                const float ratio = p.eps_stage[sidx - 1] / es;
                long tot = 2L * Lp * N;
                hipLaunchKernelGGL(scale_kernel, dim3((tot + 255) / 256), dim3(256), 0, st, UV, 2L * Lp, us, N, ratio);
                if (hipGetLastError() != hipSuccess) return SKA_EHIP;
                SKA_TRY((make_scores_operand<T>(p, es, Qin, ws, &Q, &stage_c2, st)));
            }
            stage_sdb2 = p.sdb * (p.eps / es) * LOG2E;
            for (int t = 0; t < Ts; ++t) {
                SKA_TRY(half(true, 1, 0, 0));
                SKA_TRY(half(false, 0, 1, 1));
            }
        }
        stage_c2 = base.c2 = (sizeof(T) == 2) ? 1.f : base.cs * LOG2E;   // the tail runs at eps (= the last stage's)
        stage_sdb2 = base.sdb2;
        for (int t = 1; t <= R; ++t) {
            SKA_TRY(half(true, 2 * t - 1, 2 * t - 2, 2 * t));    // u_t from v_{t-1}
            SKA_TRY(half(false, 2 * t, 2 * t - 1, 2 * t + 1));   // v_t from u_t
        }
        return SKA_OK;
    };
    const int rc_halves = halves();
    if (pt_run) pt_run->~PhaseTimer();
    SKA_TRY(rc_halves);
    // output map with the terminal plan
    PhaseTimer pt_out(SKA_PH_OUTPUT, st);
    SweepArgs a = base;
    a.X = Q; a.Y = K; a.Pay = V; a.out_mat = O; a.xs = vec(2 * R); a.yt = vec(2 * R + 1);
    a.len_own = p.len_q; a.len_oth = p.len_k;
    if (p.token()) { a.spoke_own = SQ; a.pay_db = p.v_db; }   // O_i += P(i, d_k) v_db
    a.rev = nlaunch & 1;
    pt_out.launched();
    return sweep<T, D>(M_APPLY, a, N, st);
}

template <typename T, int D>
int bwd_impl(const Problem &p, const void *Qin, const void *K, const void *V, const void *O,
             const void *G, const float *UV, void *dQ, void *dK, void *dV, float *eta0, void *ws,
             hipStream_t st, const float *seed = nullptr)
{
    // seed != null: no output map at the end of the chain.  The reverse recurrences start from
    // vbar_R = seed (a cotangent of v^(R) given by the caller), Z = 0, and only dQ, dK are
    // produced: the vector-Jacobian product through R full steps started at v = 0.
    // Q below is the score operand (bf16 storage: prescaled copy at the end of the workspace,
    // c2 = 1); it also serves as the payload of the dK sweep, whose output scale absorbs it
    const void *Q = nullptr;
    float c2 = 0.f;
    {
        PhaseTimer pt(SKA_PH_PRESCALE, st);
        SKA_TRY((make_scores_operand<T>(p, p.eps, Qin, reinterpret_cast<unsigned char *>(ws) + ws_vec_bytes(p), &Q, &c2, st)));
        pt.launched(sizeof(T) == 2 ? 1 : 0);
    }
    const int N = p.N(), L = p.L, Lp = p.Lp();
    const int R = p.R, nq = p.direct() ? R : pack_groups(R);
    const long us = 2L * (R + 1) * Lp, ldw = p.ldw();
    const long nldp = (long)N * ldw;
    auto uv = [&](int k) { return Vec{UV + (long)k * Lp, us}; };   // slot 2t: u_t, slot 2t + 1: v_t
    float *wf = reinterpret_cast<float *>(ws);
    float *gu = wf;
    auto vbar = [&](int t) { return wf + (1 + 2 * (R - t)) * nldp; };   // t = 1 ... R
    auto ubar = [&](int t) { return wf + (2 + 2 * (R - t)) * nldp; };
    float4 *rowp = reinterpret_cast<float4 *>(wf + (long)ws_vecs(R) * nldp);
    float4 *colp = rowp + nldp * R;   // (room for R groups per side)
    // the ring kernel (R <= 2) takes the packs as bf16 columns (rowA, rowB, colA, colB)
    const bool AUG = (sizeof(T) == 2 && D <= 64 && R <= 2 && !seed && p.variant == SKA_BWD_ONE_REFERENCE);   // (that kernel always adds Z)
    __bf16 *aug = reinterpret_cast<__bf16 *>(colp + nldp * R);
    const int final_mode = p.direct() ? M_FINAL_DIRECT : M_FINAL;
    auto wv = [&](float *q) { return Vec{q, ldw}; };
    auto wo = [&](float *q) { return VecOut{q, ldw}; };

    SweepArgs base{};
    base.L = L; base.W = p.W < L ? p.W : L;   // |i-j| <= L-1 always: W >= L is the dense problem
    base.cs = 1.f / (p.eps * sqrtf((float)p.d));
    base.c2 = c2;
    base.dustbin = p.dustbin; base.sdb2 = p.sdb * LOG2E;
    base.nh = p.H;
    const dim3 vgrid((Lp + 255) / 256, N);
    int nlaunch = 0;   // successive sweeps walk the blocks in opposite directions (L2 reuse)
    // learned dustbin tokens: spoke scores, spoke cotangents, partial sums
    Vec SQ{nullptr, 0}, SK{nullptr, 0};
    float *tok = p.token() ? ws_tok(p, ws) : nullptr;
    float *sbr = tok ? tok + 2 * nldp : nullptr, *sbc = tok ? tok + 3 * nldp : nullptr;
    float *partial = tok ? tok + 4 * nldp : nullptr;
    const int nchunk = ws_chunks(p);
    if (p.token()) {
        SQ = Vec{tok, ldw};
        SK = Vec{tok + nldp, ldw};
        SKA_TRY((spoke_scores<T, D>(p, Qin, K, tok, tok + nldp, st)));
    }

    // g_u = <dO_i, O_i> (= (P22 . Z) 1); dustbin row has dO = 0
    PhaseTimer pt_gu(SKA_PH_ROWDOT, st);
    pt_gu.launched();
    constexpr int LPR = D * (int)sizeof(T) / 16;
    if (seed) {
        hipLaunchKernelGGL(seed_kernel, vgrid, dim3(256), 0, st, seed, p.log_b, vbar(R), ldw, Lp);
        if (hipGetLastError() != hipSuccess) return SKA_EHIP;
    } else {
        hipLaunchKernelGGL((rowdot_kernel<T, D>), dim3(((long)Lp * LPR + 255) / 256, N), dim3(256), 0, st,
                           reinterpret_cast<const T *>(G),
                           reinterpret_cast<const T *>(O), gu, ldw, L, Lp, p.len_q, p.H);
        if (hipGetLastError() != hipSuccess) return SKA_EHIP;
        if (p.token()) {
            // dv_db = sum_i P_RR(i, d_k) dO_i and vbar_R at the dustbin column = <v_db, dv_db>
            hipLaunchKernelGGL((wsum_kernel<T, D>), dim3(nchunk, N), dim3(256), 0, st, reinterpret_cast<const T *>(G),
                               Vec{nullptr, 0}, SQ, uv(2 * R), uv(2 * R + 1), partial, L);
            hipLaunchKernelGGL((wsum_final_kernel<D>), dim3(N), dim3(D), 0, st, partial, nchunk, Vec{nullptr, 0}, 0,
                               nullptr, 1.f, p.dv_db, p.v_db, wo(vbar(R)), L);
            if (hipGetLastError() != hipSuccess) return SKA_EHIP;
        } else if (p.dustbin) {   // vbar_R at the dustbin column is 0 because V there is 0
            hipLaunchKernelGGL(fill_kernel, dim3((N + 255) / 256), dim3(256), 0, st, vbar(R) + L, 1L, ldw, N, 0.f);
            if (hipGetLastError() != hipSuccess) return SKA_EHIP;
        }
    }
    pt_gu.end();
    // dV_j = sum_i P_RR,ij dO_i ; vbar_R,j = <V_j, dV_j>  (column-oriented)
    if (!seed) {
        PhaseTimer pt(SKA_PH_DV, st);
        pt.launched();
        SweepArgs a = base;
        a.X = K; a.Y = Q; a.Pay = G; a.out_mat = dV; a.xs = uv(2 * R + 1); a.yt = uv(2 * R);
        a.dot_mat = V; a.dot_out = wo(vbar(R));
        a.len_own = p.len_k; a.len_oth = p.len_q;
        a.olog = Vec{p.log_b, (long)Lp};   // the workspace holds vbar / b and ubar / a (general marginals)
        a.rev = nlaunch++ & 1;
        SKA_TRY((sweep<T, D>(M_APPLY, a, N, st)));
    }
    // reverse recurrences of Prop. 1, each one band mat-vec with a staircase factor
    // written as P22 times row/column modifiers folded into the exponent (Prop. 2)
    auto matvec = [&](bool row, Vec xs, Vec yt, float *w, float *pre, VecOut out, bool scaled = true) -> int {
        SweepArgs a = base;
        a.X = row ? Q : K; a.Y = row ? K : Q;
        a.xs = xs; a.yt = yt; a.w = wv(w); a.pre = Vec{pre, ldw}; a.out_vec = out;
        if (scaled) a.olog = Vec{row ? p.log_a : p.log_b, (long)Lp};
        a.len_own = row ? p.len_q : p.len_k; a.len_oth = row ? p.len_k : p.len_q;
        a.spoke_own = row ? SQ : SK;
        a.rev = nlaunch++ & 1;
        SKA_TRY((sweep<T, D>(M_MATVEC, a, N, st)));
        if (p.dustbin) {
            hipLaunchKernelGGL(dustbin_kernel, dim3(N), dim3(1024), 0, st, yt, wv(w), xs, out, L, p.sdb,
                               row ? SK : SQ);
            if (hipGetLastError() != hipSuccess) return SKA_EHIP;
        }
        return SKA_OK;
    };
    {
        PhaseTimer pt(SKA_PH_MATVEC, st);
        pt.launched(2 * R - 1 + (eta0 ? 1 : 0));
        // ubar_R = g_u - P_RR vbar_R
        SKA_TRY(matvec(true, uv(2 * R), uv(2 * R + 1), vbar(R), seed ? nullptr : gu, wo(ubar(R))));
        for (int t = R; t >= 1; --t) {
            // vbar_{t-1} = -(P_t,t-1)^T ubar_t   (t = 1: the base cotangent, only on request)
            if (t >= 2) SKA_TRY(matvec(false, uv(2 * t - 1), uv(2 * t), ubar(t), nullptr, wo(vbar(t - 1))));
            else if (eta0) SKA_TRY(matvec(false, uv(1), uv(2), ubar(1), nullptr, VecOut{eta0, (long)Lp}, false));
            // ubar_{t-1} = -P_{t-1,t-1} vbar_{t-1}
            if (t >= 2) SKA_TRY(matvec(true, uv(2 * t - 2), uv(2 * t - 1), vbar(t - 1), nullptr, wo(ubar(t - 1))));
        }
    }
    PhaseTimer pt_final(SKA_PH_FINAL, st);   // modifier packs and the two final sweeps
    pt_final.launched(2 * ((nq + MAXNQ - 1) / MAXNQ));
    hipLaunchKernelGGL(packs_kernel, vgrid, dim3(256), 0, st, UV, Lp, R, wf, nldp, ldw,
                       reinterpret_cast<float *>(rowp), reinterpret_cast<float *>(colp), nq, AUG ? aug : nullptr,
                       ldw, nldp, p.direct() ? 1 : 0, p.token() ? 1 : 0);
    if (hipGetLastError() != hipSuccess) return SKA_EHIP;
    // one-reference final sweeps; a sweep takes eight modifier terms, so a tail deeper than
    // R = 4 takes several that accumulate (Z only in the first)
    for (int g0 = 0; g0 < nq; g0 += MAXNQ) {
        const int ng = nq - g0 < MAXNQ ? nq - g0 : MAXNQ;
        {
            SweepArgs a = base;
            a.X = Q; a.Y = K; a.A = G; a.Bm = V; a.out_mat = dQ; a.xs = uv(2 * R); a.yt = uv(2 * R + 1);
            a.po = rowp + g0; a.qt = colp + g0; a.ldp = ldw; a.nq = ng; a.pstride = nq;
            a.len_own = p.len_q; a.len_oth = p.len_k;
            a.skipz = a.accum = g0 > 0;
            a.refterm = g0 == 0;   // (direct: the first term of all is P_RR vbar_R itself)
            if (seed) { a.A = Q; a.Bm = K; a.skipz = 1; }   // Z = 0; the factors are fetched but unused
            if (AUG) { a.poB = aug + 1 * nldp * 16; a.qtA = aug + 2 * nldp * 16; }   // rows own, columns stream
            a.rev = nlaunch++ & 1;
            SKA_TRY((sweep<T, D>(final_mode, a, N, st)));
        }
        {
            SweepArgs a = base;
            a.X = K; a.Y = Q; a.A = V; a.Bm = G; a.out_mat = dK; a.xs = uv(2 * R + 1); a.yt = uv(2 * R);
            a.po = colp + g0; a.qt = rowp + g0; a.ldp = ldw; a.nq = ng; a.pstride = nq;
            a.len_own = p.len_k; a.len_oth = p.len_q;
            a.skipz = a.accum = g0 > 0;
            a.refterm = g0 == 0;
            if (seed) { a.A = K; a.Bm = Q; a.skipz = 1; }
            if (AUG) { a.poB = aug + 3 * nldp * 16; a.qtA = aug + 0 * nldp * 16; }   // columns own, rows stream
            // payload rows are Qs = (cs log2 e) Q when prescaled: cs sum Sbar^T Q = ln 2 sum Sbar^T Qs
            if (sizeof(T) == 2) a.cs = LN2;
            a.rev = nlaunch++ & 1;
            SKA_TRY((sweep<T, D>(final_mode, a, N, st)));
        }
    }
    if (p.token()) {
        // the spokes' share (Prop. 2 on the augmented support): cotangents of the 2L + 1 spoke
        // scores, then their chain rule to Q, K (rank-1 updates) and to the tokens (weighted sums)
        constexpr int LPR2 = D * (int)sizeof(T) / 16;
        const float cs = base.cs;
        hipLaunchKernelGGL((spoke_sbar_kernel<T, D>), dim3((unsigned)(((long)Lp * LPR2 + 255) / 256), N), dim3(256), 0,
                           st, reinterpret_cast<const T *>(G), p.v_db, uv(2 * R), uv(2 * R + 1), SQ, SK, rowp, colp, nq,
                           ldw, sbr, sbc, ldw, L);
        const dim3 agrid((unsigned)(((long)L * (D / 4) + 255) / 256), N);
        hipLaunchKernelGGL((spoke_axpy_kernel<T, D>), agrid, dim3(256), 0, st, reinterpret_cast<T *>(dQ), wv(sbr),
                           p.k_db, cs, L);
        hipLaunchKernelGGL((spoke_axpy_kernel<T, D>), agrid, dim3(256), 0, st, reinterpret_cast<T *>(dK), wv(sbc),
                           p.q_db, cs, L);
        // dk_db = c (sum_i sbr_i q_i + sbr_L q_db), dq_db = c (sum_j sbc_j k_j + sbc_L k_db)
        hipLaunchKernelGGL((wsum_kernel<T, D>), dim3(nchunk, N), dim3(256), 0, st, reinterpret_cast<const T *>(Qin),
                           wv(sbr), Vec{nullptr, 0}, Vec{nullptr, 0}, Vec{nullptr, 0}, partial, L);
        hipLaunchKernelGGL((wsum_final_kernel<D>), dim3(N), dim3(D), 0, st, partial, nchunk, wv(sbr), L, p.q_db, cs,
                           p.dk_db, nullptr, VecOut{nullptr, 0}, 0);
        hipLaunchKernelGGL((wsum_kernel<T, D>), dim3(nchunk, N), dim3(256), 0, st, reinterpret_cast<const T *>(K),
                           wv(sbc), Vec{nullptr, 0}, Vec{nullptr, 0}, Vec{nullptr, 0}, partial, L);
        hipLaunchKernelGGL((wsum_final_kernel<D>), dim3(N), dim3(D), 0, st, partial, nchunk, wv(sbc), L, p.k_db, cs,
                           p.dq_db, nullptr, VecOut{nullptr, 0}, 0);
        if (hipGetLastError() != hipSuccess) return SKA_EHIP;
    }
    return SKA_OK;
}

// the tail-depth selector's scratch, carved out of one workspace
size_t up256(size_t x) { return (x + 255) / 256 * 256; }
struct SelectLayout {
    size_t core, eq, ek, uvb, eta, norm, total;
};
SelectLayout select_layout(const Problem &p, int T, int R_max)
{
    Problem q = p;
    q.R = R_max > T ? R_max : T;   // workspace of the deepest call (it grows with the depth)
    SelectLayout l{};
    const size_t mat = (size_t)p.N() * p.L * p.d * (p.dtype == SKA_BF16 ? 2 : 4);
    l.core = 0;
    l.eq = up256(ws_bytes(q));
    l.ek = l.eq + up256(mat);
    l.uvb = l.ek + up256(mat);
    l.eta = l.uvb + up256((size_t)p.N() * 2 * (T + 1) * p.Lp() * sizeof(float));
    l.norm = l.eta + up256((size_t)p.N() * p.Lp() * sizeof(float));
    l.total = l.norm + 256;
    return l;
}
template <typename T> int absmax_launch(const void *x, long n, float *out, hipStream_t st)
{
    long blocks = (n + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL((absmax_kernel<T>), dim3((unsigned)blocks), dim3(256), 0, st, reinterpret_cast<const T *>(x), n, out);
    return hipGetLastError() == hipSuccess ? SKA_OK : SKA_EHIP;
}

}  // namespace

// ====================================================================== C ABI
extern "C" {

size_t sinkhorn_attn_workspace_bytes(int B, int H, int L, int d, int W, int T, int R, int dustbin, int dtype)
{
    Problem p{B, H, L, d, W, T, R, dustbin ? 1 : 0, dtype, 1.f, 0.f};
    if (check_common(p) != SKA_OK) return 0;
    return ws_bytes(p);
}

static int fwd_call(const Problem &p, const void *Q, const void *K, const void *V, void *O, float *UV,
                    void *workspace, size_t workspace_bytes, void *stream)
{
    const int d = p.d, dtype = p.dtype;
    if (!Q || !K || !V || !O || !UV) return SKA_EINVAL;
    int rc = check_common(p);
    if (rc != SKA_OK) return rc;
    if (ws_qs_bytes(p) && (!workspace || workspace_bytes < ws_qs_bytes(p))) return SKA_EWORKSPACE;
    if (p.token() && (!workspace || workspace_bytes < ws_bytes(p))) return SKA_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 15) return SKA_EINVAL;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
#define SKA_FWD(TT_, DD_) return fwd_impl<TT_, DD_>(p, Q, K, V, O, UV, workspace, st)
    if (dtype == SKA_F32) {
        if (d == 32) SKA_FWD(float, 32);
        if (d == 64) SKA_FWD(float, 64);
        SKA_FWD(float, 128);
    } else {
        if (d == 32) SKA_FWD(__bf16, 32);
        if (d == 64) SKA_FWD(__bf16, 64);
        SKA_FWD(__bf16, 128);
    }
#undef SKA_FWD
}

int sinkhorn_attn_fwd_varlen(const void *Q, const void *K, const void *V, const float *log_a,
                             const float *log_b, const int *len_q, const int *len_k, void *O, float *UV, int B,
                             int H, int L, int d, int W, int T, int R, float eps, int dustbin,
                             float dustbin_score, int dtype, void *workspace, size_t workspace_bytes,
                             void *stream)
{
    Problem p{B, H, L, d, W, T, R, dustbin ? 1 : 0, dtype, eps, dustbin_score, log_a, log_b, len_q, len_k};
    return fwd_call(p, Q, K, V, O, UV, workspace, workspace_bytes, stream);
}

int sinkhorn_attn_fwd_masked(const void *Q, const void *K, const void *V, const float *log_a,
                             const float *log_b, const unsigned char *mask_q, const unsigned char *mask_k,
                             void *O, float *UV, int B, int H, int L, int d, int W, int T, int R, float eps,
                             int dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    Problem p{B, H, L, d, W, T, R, 0, dtype, eps, 0.f, log_a, log_b};
    p.mask_q = mask_q; p.mask_k = mask_k;
    return fwd_call(p, Q, K, V, O, UV, workspace, workspace_bytes, stream);
}

int sinkhorn_attn_fwd_eps_schedule(const void *Q, const void *K, const void *V, const float *log_a,
                                   const float *log_b, const int *len_q, const int *len_k, void *O, float *UV,
                                   int B, int H, int L, int d, int W, int n_stages, const float *eps_stage,
                                   const int *T_stage, int R, float eps, int dustbin, float dustbin_score,
                                   int dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    if (n_stages < 1 || n_stages > 64 || !eps_stage || !T_stage) return SKA_EINVAL;
    int T = 0;
    for (int s = 0; s < n_stages; ++s) {
        if (!(eps_stage[s] > 0.f) || !isfinite(eps_stage[s]) || T_stage[s] < 0) return SKA_EINVAL;
        if (s > 0 && eps_stage[s] > eps_stage[s - 1]) return SKA_EINVAL;   // eps_1 >= ... >= eps_N
        T += T_stage[s];
    }
    if (fabsf(eps_stage[n_stages - 1] - eps) > 1e-6f * eps) return SKA_EINVAL;   // eps_N = eps
    Problem p{B, H, L, d, W, T, R, dustbin ? 1 : 0, dtype, eps, dustbin_score, log_a, log_b, len_q, len_k};
    p.n_stages = n_stages; p.eps_stage = eps_stage; p.T_stage = T_stage;
    return fwd_call(p, Q, K, V, O, UV, workspace, workspace_bytes, stream);
}

int sinkhorn_attn_fwd_marginals(const void *Q, const void *K, const void *V, const float *log_a,
                                const float *log_b, void *O, float *UV, int B, int H, int L, int d, int W,
                                int T, int R, float eps, int dustbin, float dustbin_score, int dtype,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    return sinkhorn_attn_fwd_varlen(Q, K, V, log_a, log_b, nullptr, nullptr, O, UV, B, H, L, d, W, T, R, eps,
                                    dustbin, dustbin_score, dtype, workspace, workspace_bytes, stream);
}

int sinkhorn_attn_fwd(const void *Q, const void *K, const void *V, void *O, float *UV, int B, int H, int L,
                      int d, int W, int T, int R, float eps, int dustbin, float dustbin_score, int dtype,
                      void *workspace, size_t workspace_bytes, void *stream)
{
    return sinkhorn_attn_fwd_marginals(Q, K, V, nullptr, nullptr, O, UV, B, H, L, d, W, T, R, eps, dustbin,
                                       dustbin_score, dtype, workspace, workspace_bytes, stream);
}

static int bwd_problem(const Problem &p, const void *Q, const void *K, const void *V, const void *O, const void *dO,
                       const float *UV, void *dQ, void *dK, void *dV, float *eta0, void *workspace,
                       size_t workspace_bytes, void *stream);

static int bwd_call(int variant, const void *Q, const void *K, const void *V, const float *log_a,
                    const float *log_b, const int *len_q, const int *len_k, const void *O, const void *dO,
                    const float *UV, void *dQ, void *dK, void *dV, float *eta0, int B, int H, int L, int d, int W,
                    int T, int R, float eps, int dustbin, float dustbin_score, int dtype, void *workspace,
                    size_t workspace_bytes, void *stream)
{
    Problem p{B, H, L, d, W, T, R, dustbin ? 1 : 0, dtype, eps, dustbin_score, log_a, log_b, len_q, len_k, variant};
    return bwd_problem(p, Q, K, V, O, dO, UV, dQ, dK, dV, eta0, workspace, workspace_bytes, stream);
}

static bool aligned16(const void *x) { return (reinterpret_cast<uintptr_t>(x) & 15) == 0; }

int sinkhorn_attn_fwd_dustbin_token(const void *Q, const void *K, const void *V, const float *q_db,
                                    const float *k_db, const float *v_db, void *O, float *UV, int B, int H, int L,
                                    int d, int W, int T, int R, float eps, int dtype, void *workspace,
                                    size_t workspace_bytes, void *stream)
{
    if (!q_db || !k_db || !v_db || !aligned16(q_db) || !aligned16(k_db) || !aligned16(v_db)) return SKA_EINVAL;
    Problem p{B, H, L, d, W, T, R, 1, dtype, eps, 0.f};
    p.q_db = q_db; p.k_db = k_db; p.v_db = v_db;
    return fwd_call(p, Q, K, V, O, UV, workspace, workspace_bytes, stream);
}

int sinkhorn_attn_bwd_dustbin_token(const void *Q, const void *K, const void *V, const float *q_db,
                                    const float *k_db, const float *v_db, const void *O, const void *dO,
                                    const float *UV, void *dQ, void *dK, void *dV, float *dq_db, float *dk_db,
                                    float *dv_db, float *eta0, int B, int H, int L, int d, int W, int T, int R,
                                    float eps, int dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!q_db || !k_db || !v_db || !dq_db || !dk_db || !dv_db) return SKA_EINVAL;
    if (!aligned16(q_db) || !aligned16(k_db) || !aligned16(v_db)) return SKA_EINVAL;
    Problem p{B, H, L, d, W, T, R, 1, dtype, eps, 0.f};
    p.q_db = q_db; p.k_db = k_db; p.v_db = v_db;
    p.dq_db = dq_db; p.dk_db = dk_db; p.dv_db = dv_db;
    return bwd_problem(p, Q, K, V, O, dO, UV, dQ, dK, dV, eta0, workspace, workspace_bytes, stream);
}

static int bwd_problem(const Problem &p, const void *Q, const void *K, const void *V, const void *O, const void *dO,
                       const float *UV, void *dQ, void *dK, void *dV, float *eta0, void *workspace,
                       size_t workspace_bytes, void *stream)
{
    const int d = p.d, dtype = p.dtype;
    if (!Q || !K || !V || !O || !dO || !UV || !dQ || !dK || !dV) return SKA_EINVAL;
    int rc = check_common(p);
    if (rc != SKA_OK) return rc;
    if (!workspace || workspace_bytes < ws_bytes(p)) return SKA_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 15) return SKA_EINVAL;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
#define SKA_BWD(TT_, DD_) return bwd_impl<TT_, DD_>(p, Q, K, V, O, dO, UV, dQ, dK, dV, eta0, workspace, st)
    if (dtype == SKA_F32) {
        if (d == 32) SKA_BWD(float, 32);
        if (d == 64) SKA_BWD(float, 64);
        SKA_BWD(float, 128);
    } else {
        if (d == 32) SKA_BWD(__bf16, 32);
        if (d == 64) SKA_BWD(__bf16, 64);
        SKA_BWD(__bf16, 128);
    }
#undef SKA_BWD
}

int sinkhorn_attn_base_vjp(const void *Q, const void *K, const float *log_a, const float *log_b,
                           const int *len_q, const int *len_k, const float *UV, const float *eta, void *dQ,
                           void *dK, int B, int H, int L, int d, int W, int T, float eps, int dustbin,
                           float dustbin_score, int dtype, void *workspace, size_t workspace_bytes,
                           void *stream)
{
    // T full steps from v = 0 are a tail of depth T without a stopped base in front of it
    Problem p{B, H, L, d, W, 0, T, dustbin ? 1 : 0, dtype, eps, dustbin_score, log_a, log_b, len_q, len_k};
    if (!Q || !K || !UV || !eta || !dQ || !dK) return SKA_EINVAL;
    int rc = check_common(p);
    if (rc != SKA_OK) return rc;
    if (!workspace || workspace_bytes < ws_bytes(p)) return SKA_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 15) return SKA_EINVAL;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
#define SKA_VJP(TT_, DD_) \
    return bwd_impl<TT_, DD_>(p, Q, K, nullptr, nullptr, nullptr, UV, dQ, dK, nullptr, nullptr, workspace, st, eta)
    if (dtype == SKA_F32) {
        if (d == 32) SKA_VJP(float, 32);
        if (d == 64) SKA_VJP(float, 64);
        SKA_VJP(float, 128);
    } else {
        if (d == 32) SKA_VJP(__bf16, 32);
        if (d == 64) SKA_VJP(__bf16, 64);
        SKA_VJP(__bf16, 128);
    }
#undef SKA_VJP
}

int sinkhorn_attn_bwd_varlen(const void *Q, const void *K, const void *V, const float *log_a,
                             const float *log_b, const int *len_q, const int *len_k, const void *O,
                             const void *dO, const float *UV, void *dQ, void *dK, void *dV, float *eta0, int B,
                             int H, int L, int d, int W, int T, int R, float eps, int dustbin,
                             float dustbin_score, int dtype, void *workspace, size_t workspace_bytes,
                             void *stream)
{
    return bwd_call(0, Q, K, V, log_a, log_b, len_q, len_k, O, dO, UV, dQ, dK, dV, eta0, B, H, L, d, W, T, R, eps,
                    dustbin, dustbin_score, dtype, workspace, workspace_bytes, stream);
}

int sinkhorn_attn_bwd_variant(int variant, const void *Q, const void *K, const void *V, const float *log_a,
                              const float *log_b, const int *len_q, const int *len_k, const void *O,
                              const void *dO, const float *UV, void *dQ, void *dK, void *dV, float *eta0, int B,
                              int H, int L, int d, int W, int T, int R, float eps, int dustbin,
                              float dustbin_score, int dtype, void *workspace, size_t workspace_bytes,
                              void *stream)
{
    if (variant != SKA_BWD_ONE_REFERENCE && variant != SKA_BWD_DIRECT && variant != SKA_BWD_ONE_REFERENCE_GENERIC)
        return SKA_EINVAL;
    return bwd_call(variant, Q, K, V, log_a, log_b, len_q, len_k, O, dO, UV, dQ, dK, dV, eta0, B, H, L, d, W, T, R, eps,
                    dustbin, dustbin_score, dtype, workspace, workspace_bytes, stream);
}

int sinkhorn_attn_bwd_marginals(const void *Q, const void *K, const void *V, const float *log_a,
                                const float *log_b, const void *O, const void *dO, const float *UV, void *dQ,
                                void *dK, void *dV, float *eta0, int B, int H, int L, int d, int W, int T,
                                int R, float eps, int dustbin, float dustbin_score, int dtype,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    return sinkhorn_attn_bwd_varlen(Q, K, V, log_a, log_b, nullptr, nullptr, O, dO, UV, dQ, dK, dV, eta0, B, H,
                                    L, d, W, T, R, eps, dustbin, dustbin_score, dtype, workspace,
                                    workspace_bytes, stream);
}

int sinkhorn_attn_bwd(const void *Q, const void *K, const void *V, const void *O, const void *dO,
                      const float *UV, void *dQ, void *dK, void *dV, float *eta0, int B, int H, int L, int d,
                      int W, int T, int R, float eps, int dustbin, float dustbin_score, int dtype,
                      void *workspace, size_t workspace_bytes, void *stream)
{
    return sinkhorn_attn_bwd_marginals(Q, K, V, nullptr, nullptr, O, dO, UV, dQ, dK, dV, eta0, B, H, L, d, W,
                                       T, R, eps, dustbin, dustbin_score, dtype, workspace, workspace_bytes,
                                       stream);
}

size_t sinkhorn_attn_select_workspace_bytes(int B, int H, int L, int d, int W, int T, int R_max, int dustbin,
                                            int dtype)
{
    Problem p{B, H, L, d, W, T, R_max, dustbin ? 1 : 0, dtype, 1.f, 0.f};
    if (check_common(p) != SKA_OK || T < 1 || T > MAXR) return 0;
    return select_layout(p, T, R_max).total;
}

int sinkhorn_attn_select_tail_depth(const void *Q, const void *K, const void *V, const void *dO,
                                    const float *log_a, const float *log_b, const int *len_q, const int *len_k,
                                    void *O, float *UV, void *dQ, void *dK, void *dV, int B, int H, int L, int d,
                                    int W, int T, int R_max, float eps, int dustbin, float dustbin_score,
                                    int dtype, float tau, int *R_selected, float *e_absmax, float *eta_absmax,
                                    void *workspace, size_t workspace_bytes, void *stream)
{
    Problem p{B, H, L, d, W, T, R_max, dustbin ? 1 : 0, dtype, eps, dustbin_score, log_a, log_b, len_q, len_k};
    if (!Q || !K || !V || !dO || !O || !UV || !dQ || !dK || !dV || !R_selected || !e_absmax) return SKA_EINVAL;
    if (!(tau >= 0.f)) return SKA_EINVAL;
    int rc = check_common(p);
    if (rc != SKA_OK) return rc;
    if (T < 1 || T > MAXR) return SKA_EUNSUPPORTED;   // the base iterates are kept: 2(T + 1) vectors
    const SelectLayout l = select_layout(p, T, R_max);
    if (!workspace || workspace_bytes < l.total) return SKA_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return SKA_EINVAL;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    unsigned char *w = reinterpret_cast<unsigned char *>(workspace);
    void *eQ = w + l.eq, *eK = w + l.ek;
    float *UVb = reinterpret_cast<float *>(w + l.uvb), *eta = reinterpret_cast<float *>(w + l.eta);
    float *norm = reinterpret_cast<float *>(w + l.norm);   // [0] certificate, [1] eta
    const long nmat = (long)p.N() * L * d, nvec = (long)p.N() * p.Lp();
    for (int r = 0; r < R_max; ++r) {
        e_absmax[r] = -1.f;
        if (eta_absmax) eta_absmax[r] = -1.f;
    }
    *R_selected = 0;
    // all iterates of the base solve, once (O is scratch here)
    SKA_TRY(sinkhorn_attn_fwd_varlen(Q, K, V, log_a, log_b, len_q, len_k, O, UVb, B, H, L, d, W, 0, T, eps, dustbin,
                                     dustbin_score, dtype, w, l.eq, stream));
    for (int R = 1; R <= R_max; ++R) {
        SKA_TRY(sinkhorn_attn_fwd_varlen(Q, K, V, log_a, log_b, len_q, len_k, O, UV, B, H, L, d, W, T, R, eps,
                                         dustbin, dustbin_score, dtype, w, l.eq, stream));
        SKA_TRY(sinkhorn_attn_bwd_varlen(Q, K, V, log_a, log_b, len_q, len_k, O, dO, UV, dQ, dK, dV, eta, B, H, L,
                                         d, W, T, R, eps, dustbin, dustbin_score, dtype, w, l.eq, stream));
        SKA_TRY(sinkhorn_attn_base_vjp(Q, K, log_a, log_b, len_q, len_k, UVb, eta, eQ, eK, B, H, L, d, W, T, eps,
                                       dustbin, dustbin_score, dtype, w, l.eq, stream));
        hipLaunchKernelGGL(fill_kernel, dim3(1), dim3(64), 0, st, norm, 2L, 2L, 1, 0.f);
        if (hipGetLastError() != hipSuccess) return SKA_EHIP;
        if (dtype == SKA_F32) {
            SKA_TRY(absmax_launch<float>(eQ, nmat, norm, st));
            SKA_TRY(absmax_launch<float>(eK, nmat, norm, st));
        } else {
            SKA_TRY(absmax_launch<__bf16>(eQ, nmat, norm, st));
            SKA_TRY(absmax_launch<__bf16>(eK, nmat, norm, st));
        }
        SKA_TRY(absmax_launch<float>(eta, nvec, norm + 1, st));
        float host[2] = {0.f, 0.f};
        if (hipMemcpyAsync(host, norm, sizeof(host), hipMemcpyDeviceToHost, st) != hipSuccess) return SKA_EHIP;
        if (hipStreamSynchronize(st) != hipSuccess) return SKA_EHIP;
        e_absmax[R - 1] = host[0];
        if (eta_absmax) eta_absmax[R - 1] = host[1];
        if (host[0] <= tau) {
            *R_selected = R;
            return SKA_OK;
        }
    }
    return SKA_OK;
}

int sinkhorn_attn_profile_enable(int on)
{
    g_prof_on = on < 0 ? 0 : (on > 2 ? 2 : on);
    return SKA_OK;
}

int sinkhorn_attn_profile_read_phases(double *elapsed_ms, long *launches)
{
    if (!elapsed_ms || !launches) return SKA_EINVAL;
    for (int k = 0; k < SKA_PH_COUNT; ++k) { elapsed_ms[k] = 0.0; launches[k] = 0; }
    int rc = SKA_OK;
    for (int i = 0; i < g_prof_n; ++i) {
        float t = 0.f;
        if (hipEventSynchronize(g_prof[i].b) != hipSuccess ||
            hipEventElapsedTime(&t, g_prof[i].a, g_prof[i].b) != hipSuccess)
            rc = SKA_EHIP;
        elapsed_ms[g_prof[i].phase] += t;
        launches[g_prof[i].phase] += g_prof[i].launches;
        (void)hipEventDestroy(g_prof[i].a);
        (void)hipEventDestroy(g_prof[i].b);
    }
    g_prof_n = 0;
    return rc;
}

int sinkhorn_attn_profile_read(double *elapsed_ms, long *launches)
{
    if (!elapsed_ms || !launches) return SKA_EINVAL;
    double ms[SKA_PH_COUNT];
    long n[SKA_PH_COUNT];
    const int rc = sinkhorn_attn_profile_read_phases(ms, n);
    *elapsed_ms = ms[SKA_PH_SCALING];
    *launches = n[SKA_PH_SCALING];
    return rc;
}

const char *sinkhorn_attn_strerror(int status)
{
    switch (status) {
    case SKA_OK: return "ok";
    case SKA_EINVAL: return "invalid argument (null pointer, non-positive size, bad eps, misaligned workspace)";
    case SKA_EUNSUPPORTED: return "unsupported configuration (need R in 1..32, L <= 2^24, d in {32, 64, 128}, dtype f32 or bf16; no dustbin with marginal targets or lengths)";
    case SKA_EWORKSPACE: return "workspace missing or smaller than sinkhorn_attn_workspace_bytes()";
    case SKA_EHIP: return "a HIP launch failed";
    default: return "unknown status";
    }
}

}  // extern "C"
