// Banded Sinkhorn attention for gfx950: types, sweep arguments, LDS tile layouts, staging and MFMA fragment helpers
// shared by all sweep kernels (see sinkhorn_attn.hip for the overall scheme).
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <type_traits>

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
    int n0;               // index of this launch's first problem within the call (launches may take a part)
    float c2;         // log2(e) / (eps sqrt d)
    float cs;         // 1 / (eps sqrt d)
    int dustbin;
    float sdb2;       // dustbin score * log2(e)
    Vec spoke_own;    // learned dustbin token: score of the spoke (o, dustbin of the other side) per
                      // owner index, natural units (null: the scalar score above)
    Vec spoke_oth;    // ... and the scores of the spokes from this side's dustbin element to the other side's indices
    const float *pay_db;  // APPLY with a learned token: payload row of the other side's dustbin [N][D]
    int nbp;          // workgroups per problem
    int nb_total;
    int lead;         // workgroups in front of the sweep's own (dustbin elements; a multiple of 8)
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
    if (a.len_own) Lo = min(max(a.len_own[(n + a.n0) / a.nh], 0), a.L);
    if (a.len_oth) Lt = min(max(a.len_oth[(n + a.n0) / a.nh], 0), a.L);
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

// Dustbin element of a sweep result (one workgroup per problem, appended to the sweep's own
// launch: it reads only the sweep's inputs): the extra row (column) is joined to every index
// 0..L of the other side by an edge of score s_t (the scalar, or spoke_oth[t] when the dustbin
// is a learned token).
//   half-steps: out[L] = -log sum_{t<=L} exp(s_t + y_t)
//   mat-vec   : out[L] = -exp(x[L]) sum_{t<=L} exp(s_t + y_t) w_t    (its additive term is 0)
__device__ __forceinline__ void dustbin_element(const SweepArgs &a, int n, bool matvec)
{
    __shared__ float sm[NWAVES], ss[NWAVES];
    const int L = a.L, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const float *yp = a.yt.p + n * a.yt.stride;
    const float *sp = a.spoke_oth.p ? a.spoke_oth.p + n * a.spoke_oth.stride : nullptr;
    const float *wp = matvec ? a.w.p + n * a.w.stride : nullptr;
    const float sdb = sp ? 0.f : a.sdb2 * LN2;
    // one pass: running maximum m and sum of exp(. - m) (times the weight), merged pairwise
    float m = -INFINITY, acc = 0.f;
    for (int t = tid; t <= L; t += NTHREADS) {
        const float v = yp[t] + (sp ? sp[t] : 0.f);
        const float wt = wp ? wp[t] : 1.f;
        const float mn = fmaxf(m, v);
        if (mn > -INFINITY) acc = acc * __expf(m - mn) + wt * __expf(v - mn);
        m = mn;
    }
    auto merge = [](float &m0, float &s0, float m1, float s1) {
        const float mn = fmaxf(m0, m1);
        s0 = (mn > -INFINITY) ? s0 * __expf(m0 - mn) + s1 * __expf(m1 - mn) : 0.f;
        m0 = mn;
    };
    for (int s = 32; s >= 1; s >>= 1) merge(m, acc, __shfl_xor(m, s), __shfl_xor(acc, s));
    if (lane == 0) { sm[wv] = m; ss[wv] = acc; }
    __syncthreads();
    if (tid == 0) {
        m = sm[0]; acc = ss[0];
        for (int i = 1; i < NWAVES; ++i) merge(m, acc, sm[i], ss[i]);
        a.out_vec.p[n * a.out_vec.stride + L] =
            matvec ? -__expf(a.xs.p[n * a.xs.stride + L] + sdb + m) * acc : -(sdb + m + __logf(acc));
    }
}

}  // namespace
