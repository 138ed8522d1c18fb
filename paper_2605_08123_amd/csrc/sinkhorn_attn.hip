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
// Three kernels serve the sweeps: vsweep_kernel (every half-step, the first one in its
// running-maximum form, and the band mat-vecs: a skewed ring of tiles in LDS), msweep_kernel
// (APPLY, FINAL for bf16 storage and d <= 64: the same ring, two products) and sweep_kernel
// (APPLY, FINAL for fp32 storage and d = 128, deep tails: double-buffered tiles).
//
// MFMA tile layout (32x32 accumulators): lane l holds owner o = l & 31; register r
// holds other index t = 8*(r>>2) + 4*(l>>5) + (r&3).  Sums over t are therefore
// in-lane register sums plus one exchange between the two lane halves.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#include <mutex>
#include <new>
#include <type_traits>

#include "sinkhorn_attn.h"
#include "ska_common.h"
#include "ska_small_kernels.h"
#include "ska_sweep_generic.h"
#include "ska_sweep_ring.h"

namespace {

// ------------------------------------------------------------------ host side
constexpr int MAX_DEVICES = 16;   // per-device state of the library (helper stream, raised LDS limits, static scratch)

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
    long uv_us = 0;                                   // floats between the UV blocks of consecutive problems (0: dense, 2(R+1) Lp)
    int resume_t = 0;                                 // forward: UV holds the iterates up to tail step resume_t - 1; run that
                                                      //   tail step and the output map only (the depth selector's increments)
    size_t ws_given = 0;                              // bytes of the caller's workspace (forward: room for the chain's counters?)
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
// counters of a fused chain of half-steps (one int per block of 128 owner rows, the smallest block)
size_t ws_chain_bytes(const Problem &p) { return ((size_t)p.N() * ((p.L + 127) / 128) * sizeof(int) + 255) / 256 * 256; }
size_t ws_core_bytes(const Problem &p) { return (ws_vec_bytes(p) + ws_qs_bytes(p) + ws_tok_bytes(p) + 255) / 256 * 256; }
size_t ws_bytes(const Problem &p) { return ws_core_bytes(p) + ws_chain_bytes(p); }
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
int launch_sweep(SweepArgs a, int N, hipStream_t st, int dev)
{
    constexpr int BM = NWAVES * FR * 32;
    a.nbp = (a.L + BM - 1) / BM;
    a.nb_total = a.nbp * N;
    const int chunk = (a.nb_total + 7) / 8;
    constexpr int LDS = 2 * Stage<T, D, MODE>::BYTES;
    static bool raised[MAX_DEVICES];    // static LDS tops out at 64 KB; the CU has 160 KB (an attribute per device)
    if (LDS > 48 * 1024 && !raised[dev]) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&sweep_kernel<T, D, MODE, FR, DIRECT>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS) != hipSuccess)
            return SKA_EHIP;
        raised[dev] = true;
    }
    a.lead = 0;
    hipLaunchKernelGGL((sweep_kernel<T, D, MODE, FR, DIRECT>), dim3(chunk * 8), dim3(NTHREADS), LDS, st, a);
    return hipGetLastError() == hipSuccess ? SKA_OK : SKA_EHIP;
}

template <typename T, int D, int MODE, int FR>
int launch_vsweep(SweepArgs a, int N, hipStream_t st, int dev)
{
    constexpr int BM = NWAVES * FR * 32;
    a.nbp = (a.L + BM - 1) / BM;
    a.nb_total = a.nbp * N;
    const int chunk = (a.nb_total + 7) / 8;
    constexpr int LDS = VRing<T, D, MODE, FR>::BYTES;
    static bool raised[MAX_DEVICES];
    if (LDS > 48 * 1024 && !raised[dev]) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&vsweep_kernel<T, D, MODE, FR>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS) != hipSuccess)
            return SKA_EHIP;
        raised[dev] = true;
    }
    a.lead = a.dustbin ? (N + 7) / 8 * 8 : 0;   // one workgroup per problem in front: the dustbin element
    hipLaunchKernelGGL((vsweep_kernel<T, D, MODE, FR>), dim3(chunk * 8 + a.lead), dim3(NTHREADS), LDS, st, a);
    return hipGetLastError() == hipSuccess ? SKA_OK : SKA_EHIP;
}

template <int D, int MODE, int FR>
int launch_msweep(SweepArgs a, int N, hipStream_t st, int dev)
{
    constexpr int BM = NWAVES * FR * 32;
    a.nbp = (a.L + BM - 1) / BM;
    a.nb_total = a.nbp * N;
    const int chunk = (a.nb_total + 7) / 8;
    constexpr int LDS = MRing<D, MODE, FR>::BYTES;
    static bool raised[MAX_DEVICES];
    if (LDS > 48 * 1024 && !raised[dev]) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&msweep_kernel<D, MODE, FR>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS) != hipSuccess)
            return SKA_EHIP;
        raised[dev] = true;
    }
    hipLaunchKernelGGL((msweep_kernel<D, MODE, FR>), dim3(chunk * 8), dim3(NTHREADS), LDS, st, a);
    return hipGetLastError() == hipSuccess ? SKA_OK : SKA_EHIP;
}

// Which kernel runs which sweep:
//   scaling sweeps and band mat-vecs      vsweep_kernel (skewed LDS ring), both storage types; the very
//                                         first half-step is its running-maximum variant
//   output map / dV, final sweeps         msweep_kernel for bf16 storage with d <= 64,
//                                         sweep_kernel otherwise
template <typename T, int D> int sweep_one(int mode, const SweepArgs &a, int N, hipStream_t st, int dev)
{
    constexpr int FRV = (sizeof(T) == 2) ? 2 : 1;   // vector sweeps: owner rows per wavefront / 32
    switch (mode) {
    case M_LSE_FIRST:
    case M_LSE:
    case M_MATVEC: {
        // 64 rows per wavefront reuse every tile fragment twice, but a launch then has N L / 256
        // workgroups.  The 256 CUs hold four of them each; up to three per CU (measured: two per CU
        // gains 4-7 %, four per CU loses 3 %) halve the block instead: twice the workgroups
        constexpr long SMALL_ROWS = 3L * 256 * 256;
        if constexpr (sizeof(T) == 2) {
            if ((long)N * a.L <= SMALL_ROWS)
                return mode == M_LSE         ? launch_vsweep<T, D, M_LSE, 1>(a, N, st, dev)
                       : mode == M_MATVEC    ? launch_vsweep<T, D, M_MATVEC, 1>(a, N, st, dev)
                                             : launch_vsweep<T, D, M_LSE_FIRST, 1>(a, N, st, dev);
        }
        return mode == M_LSE      ? launch_vsweep<T, D, M_LSE, FRV>(a, N, st, dev)
               : mode == M_MATVEC ? launch_vsweep<T, D, M_MATVEC, FRV>(a, N, st, dev)
                                  : launch_vsweep<T, D, M_LSE_FIRST, FRV>(a, N, st, dev);
    }
    case M_APPLY:
        if constexpr (sizeof(T) == 2 && D <= 64) return launch_msweep<D, M_APPLY, 2>(a, N, st, dev);
        else return launch_sweep<T, D, M_APPLY, 1>(a, N, st, dev);
    case M_FINAL_DIRECT: return launch_sweep<T, D, M_FINAL, 1, true>(a, N, st, dev);
    default:
        if constexpr (sizeof(T) == 2 && D <= 64) {
            if (a.poB) return launch_msweep<D, M_FINAL, 1>(a, N, st, dev);   // packs as bf16 columns (R <= 2)
        }
        return launch_sweep<T, D, M_FINAL, 1>(a, N, st, dev);
    }
}

#define SKA_TRY(x)                      \
    do {                                \
        int rc_ = (x);                  \
        if (rc_ != SKA_OK) return rc_;  \
    } while (0)

// Two problem groups on two streams.  The (batch, head) problems are independent, and one sweep
// launch leaves the chip part idle while it ramps up and drains (all its workgroups start, load
// their first tiles and finish together).  So every band sweep of a call is launched twice, the
// first half of the problems on the caller's stream and the second half on a helper stream of
// the library: the two chains run concurrently and each fills the other's gaps (paper workload:
// 3.45 -> 3.05 ms per step).  The helper stream is forked from the caller's stream by an event
// before the first sweep and joined to it again before every kernel that needs all problems and
// at the end of the call, so for the caller all work stays ordered on the stream it passed.
struct Side {
    hipStream_t s = nullptr;
    hipEvent_t fork_ev = nullptr, join_ev = nullptr;
    bool tried = false;
};
// State shared by all calls of the process; g_mutex guards all of it.  A call holds the mutex
// while it enqueues (host work only, the GPU runs on), so calls from several host threads are
// serialised at the enqueue and each sees consistent helper streams, events and flags.
std::mutex g_mutex;
Side g_side[MAX_DEVICES];
int g_streams = 2;            // sinkhorn_attn_set_streams: 1 = everything on the caller's stream
int g_fuse = 0;               // sinkhorn_attn_set_fused_half_steps: 0 off, 1 the tail, 2 all but the first half-step
unsigned g_spin_limit = 1u << 18;   // polls of a chain's wait before it gives up (a poll is a few hundred cycles: about 0.1 s)
int g_chain_cap[MAX_DEVICES][8];    // workgroups of a chain kernel the device holds at once (0: not asked yet)
double g_split_min_edges = 50e6;   // sinkhorn_attn_set_split_min_edges

Side *side_for_device(int dev)   // (g_mutex held)
{
    Side &sd = g_side[dev];
    if (!sd.tried) {
        sd.tried = true;
        if (hipStreamCreateWithFlags(&sd.s, hipStreamNonBlocking) != hipSuccess) sd.s = nullptr;
        if (sd.s && (hipEventCreateWithFlags(&sd.fork_ev, hipEventDisableTiming) != hipSuccess ||
                     hipEventCreateWithFlags(&sd.join_ev, hipEventDisableTiming) != hipSuccess))
            sd.s = nullptr;
    }
    return sd.s ? &sd : nullptr;
}

// One library call: the stream it enqueues on, the device, and whether its sweeps are split
// over the helper stream.  Splitting doubles the dispatches of a call, which pays only while a
// dispatch is long against the host's cost of enqueueing it: at least 50 M band edges per
// dispatch (about 10 us).  Below that (measured: 17 M and 34 M edges per dispatch) two streams
// are no faster or slower.  The destructor joins the helper stream, so every way out of a call,
// a failed launch included, leaves all of its work ordered on the caller's stream (a capture
// in progress stays a valid graph).
struct Call {
    hipStream_t st;
    int dev = 0;
    int rc = SKA_OK;
    Side *side = nullptr;    // the helper stream while this call splits its sweeps
    bool busy = false;       // the helper stream holds work that st has not joined
    bool noalloc = false;    // a call that may create nothing: no helper stream, no profiling events
    std::unique_lock<std::mutex> lk;
    Call(void *stream, int nproblems, int L, int W, bool may_split = true)
        : st(reinterpret_cast<hipStream_t>(stream)), noalloc(!may_split), lk(g_mutex)
    {
        if (hipGetDevice(&dev) != hipSuccess) { rc = SKA_EHIP; dev = 0; return; }
        if (dev < 0 || dev >= MAX_DEVICES) { rc = SKA_EUNSUPPORTED; dev = 0; return; }
        const double edges = (double)(nproblems / 2) * L * (2.0 * (W < L ? W : L) + 1.0);
        if (may_split && g_streams >= 2 && nproblems >= 2 && edges >= g_split_min_edges) side = side_for_device(dev);
    }
    Call(const Call &) = delete;
    ~Call() { (void)join(); }
    // the helper stream waits for everything enqueued on st so far
    int fork()
    {
        if (!side) return SKA_OK;
        if (hipEventRecord(side->fork_ev, st) != hipSuccess || hipStreamWaitEvent(side->s, side->fork_ev, 0) != hipSuccess)
            return SKA_EHIP;
        return SKA_OK;
    }
    // st waits for everything enqueued on the helper stream so far
    int join()
    {
        if (!side || !busy) return SKA_OK;
        busy = false;
        if (hipEventRecord(side->join_ev, side->s) != hipSuccess || hipStreamWaitEvent(st, side->join_ev, 0) != hipSuccess)
            return SKA_EHIP;
        return SKA_OK;
    }
};

// A chain of half-steps in one cooperative launch (vchain_kernel); returns SKA_EUNSUPPORTED if the
// device cannot hold a useful grid, so that the caller launches the half-steps one by one instead.
template <typename T, int D, int FR> int launch_vchain(ChainArgs &c, int N, hipStream_t st, int dev, int slot)
{
    constexpr int BM = NWAVES * FR * 32;
    c.base.nbp = (c.base.L + BM - 1) / BM;
    c.base.nb_total = c.base.nbp * N;
    c.base.lead = 0;
    constexpr int LDS = VRing<T, D, M_LSE, FR>::BYTES;
    const void *fn = reinterpret_cast<const void *>(&vchain_kernel<T, D, FR>);
    static bool raised[MAX_DEVICES];
    if (LDS > 48 * 1024 && !raised[dev]) {
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, LDS) != hipSuccess) return SKA_EHIP;
        raised[dev] = true;
    }
    int &cap = g_chain_cap[dev][slot];
    if (cap == 0) {
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, NTHREADS, LDS) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return SKA_EHIP;
        cap = per_cu * cus > 0 ? per_cu * cus : -1;
    }
    const int want = (c.base.nb_total + 7) / 8 * 8;
    const int grid = want < cap ? want : cap / 8 * 8;   // a multiple of eight: a workgroup's blocks stay on its XCD
    if (grid < 8) return SKA_EUNSUPPORTED;
    void *args[] = {&c};
    if (hipLaunchCooperativeKernel(fn, dim3(grid), dim3(NTHREADS), args, LDS, st) != hipSuccess) {
        (void)hipGetLastError();
        return SKA_EUNSUPPORTED;
    }
    return SKA_OK;
}

template <typename T, int D> int sweep(Call &cx, int mode, const SweepArgs &a, int N)
{
    if (!cx.side || N < 2) return sweep_one<T, D>(mode, a, N, cx.st, cx.dev);
    const int n0 = N / 2;
    SweepArgs b = a;
    const long mb = (long)n0 * a.L * D * (long)sizeof(T);
    auto mat = [&](const void *p) -> const void * { return p ? reinterpret_cast<const unsigned char *>(p) + mb : nullptr; };
    auto vec = [&](Vec v) { return Vec{v.p ? v.p + n0 * v.stride : nullptr, v.stride}; };
    b.X = mat(a.X); b.Y = mat(a.Y); b.A = mat(a.A); b.Bm = mat(a.Bm); b.Pay = mat(a.Pay); b.dot_mat = mat(a.dot_mat);
    b.out_mat = const_cast<void *>(mat(a.out_mat));
    b.yt = vec(a.yt); b.xs = vec(a.xs); b.w = vec(a.w); b.pre = vec(a.pre); b.olog = vec(a.olog);
    b.spoke_own = vec(a.spoke_own); b.spoke_oth = vec(a.spoke_oth);
    b.out_vec = VecOut{a.out_vec.p ? a.out_vec.p + n0 * a.out_vec.stride : nullptr, a.out_vec.stride};
    b.dot_out = VecOut{a.dot_out.p ? a.dot_out.p + n0 * a.dot_out.stride : nullptr, a.dot_out.stride};
    if (a.po) b.po = a.po + (long)n0 * a.ldp * a.pstride;
    if (a.qt) b.qt = a.qt + (long)n0 * a.ldp * a.pstride;
    if (a.poB) b.poB = reinterpret_cast<const unsigned char *>(a.poB) + (long)n0 * a.ldp * 32;
    if (a.qtA) b.qtA = reinterpret_cast<const unsigned char *>(a.qtA) + (long)n0 * a.ldp * 32;
    if (a.pay_db) b.pay_db = a.pay_db + (long)n0 * D;
    b.n0 = a.n0 + n0;
    SKA_TRY((sweep_one<T, D>(mode, a, n0, cx.st, cx.dev)));
    cx.busy = true;
    return sweep_one<T, D>(mode, b, N - n0, cx.side->s, cx.dev);
}

// benchmark hooks: while enabled, every phase of a call is bracketed by events on the call's
// streams, so that the phases can be timed in place inside a larger timed region.  Level 1 (the
// run of scaling sweeps only) leaves the schedule as it is: the span ends with one event on each
// of the two streams and its time is the later of the two.  Level 2 (every phase) joins the
// helper stream at the end of each phase so that the phases do not overlap.
struct ProfSpan { hipEvent_t a, b, b2; int phase; long launches; };
int g_prof_on = 0;   // 0 off, 1 the scaling-sweep run only, 2 every phase
constexpr int PROF_MAX = 4096;
ProfSpan g_prof[PROF_MAX];
int g_prof_n = 0;

struct PhaseTimer {
    ProfSpan *sp = nullptr;
    Call &cx;
    PhaseTimer(int phase, Call &cx_) : cx(cx_)
    {
        if (cx.noalloc || g_prof_on < (phase == SKA_PH_SCALING ? 1 : 2) || g_prof_n >= PROF_MAX) return;
        ProfSpan *c = &g_prof[g_prof_n];
        c->b2 = nullptr;
        if (hipEventCreate(&c->a) != hipSuccess) return;
        if (hipEventCreate(&c->b) != hipSuccess) { (void)hipEventDestroy(c->a); return; }
        c->phase = phase;
        c->launches = 0;
        (void)hipEventRecord(c->a, cx.st);
        sp = c;
        ++g_prof_n;
    }
    void launched(long n = 1) { if (sp) sp->launches += n; }
    void end()
    {
        if (!sp) return;
        if (g_prof_on >= 2) (void)cx.join();   // the span covers the helper stream's share of the phase as well
        else if (cx.side && cx.busy && hipEventCreate(&sp->b2) == hipSuccess) (void)hipEventRecord(sp->b2, cx.side->s);
        (void)hipEventRecord(sp->b, cx.st);
        sp = nullptr;
    }
    ~PhaseTimer() { end(); }
};


// one-call step without a dustbin: the forward's output map writes g_u (the dustbin's extra row
// needs a zero there that only the row-dot kernel writes)
inline bool fused_gu(const Problem &p, bool fused, const void *G) { return fused && G && !p.dustbin; }

template <typename T, int D>
int fwd_impl(Call &cx, const Problem &p, const void *Qin, const void *K, const void *V, void *O, float *UV,
             void *ws, bool fused = false, const void *G = nullptr)
{
    const hipStream_t st = cx.st;
    // fused: the backward of the same call follows (sinkhorn_attn_step).  The prescaled operand
    // then goes where the backward expects it, and the helper stream is not joined at the end:
    // each half of the problems runs its forward and backward as one uninterrupted chain.
    // G (fused, no dustbin): the output cotangent; the output map then also leaves
    // g_u = <dO_i, O_i> (Sec. 2.2), taken from its fp32 accumulators, in the backward's first
    // workspace vector, so that the backward needs no pass over O and dO for it.
    // Q below is the score operand: for bf16 storage the prescaled copy, with c2 = 1
    const void *Q = nullptr;
    float c2 = 0.f;
    {
        PhaseTimer pt(SKA_PH_PRESCALE, cx);
        void *ws_q = fused ? reinterpret_cast<unsigned char *>(ws) + ws_vec_bytes(p) : ws;
        SKA_TRY((make_scores_operand<T>(p, p.n_stages ? p.eps_stage[0] : p.eps, Qin, ws_q, &Q, &c2, st)));
        pt.launched(sizeof(T) == 2 ? 1 : 0);
    }
    const int N = p.N(), L = p.L, Lp = p.Lp();
    const int R = p.R;
    const long us = p.uv_us ? p.uv_us : 2L * (R + 1) * Lp;
    auto vec = [&](int k) { return Vec{UV + (long)k * Lp, us}; };   // slot 2t: u_t, slot 2t + 1: v_t
    auto vout = [&](int k) { return VecOut{UV + (long)k * Lp, us}; };
    SweepArgs base{};
    base.L = L; base.W = p.W < L ? p.W : L;   // |i-j| <= L-1 always: W >= L is the dense problem
    base.cs = 1.f / (p.eps * sqrtf((float)p.d));
    base.c2 = c2;
    base.dustbin = p.dustbin; base.sdb2 = p.sdb * LOG2E;
    base.nh = p.H;

    // u0 = v0 = 0: the base solve starts from v = 0
    if (!p.resume_t) {
        long tot = 2L * Lp * N;
        hipLaunchKernelGGL(fill_kernel, dim3((tot + 255) / 256), dim3(256), 0, st, UV, 2L * Lp, us, N, 0.f);
        if (hipGetLastError() != hipSuccess) return SKA_EHIP;
    }
    if (p.mask_q || p.mask_k) {   // inactive tokens start, and stay, at -inf
        hipLaunchKernelGGL(mask_fill_kernel, dim3((L + 255) / 256, N), dim3(256), 0, st, UV, us, Lp, L, p.mask_q,
                           p.mask_k, p.H);
        if (hipGetLastError() != hipSuccess) return SKA_EHIP;
    }
    // The first row half-step has no previous iterate to stabilise with: it runs on the kernel
    // that tracks a running maximum, which is exact whatever the scores are and tells an empty sum
    // (no active partner) from a small one.  With token masks the first column half-step does so
    // too: after these two every token's activity is settled, and an empty sum later is an error.
    int cold = p.resume_t ? 0 : (p.mask_q || p.mask_k) ? 2 : 1;
    int nlaunch = 0;
    PhaseTimer pt_first(SKA_PH_FIRST, cx);   // the two cold launches are the other (max-tracking) kernel
    PhaseTimer *pt_run = nullptr;
    alignas(PhaseTimer) unsigned char pt_run_mem[sizeof(PhaseTimer)];
    if (cold == 0) {
        pt_first.end();
        pt_run = new (pt_run_mem) PhaseTimer(SKA_PH_SCALING, cx);
    }
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
    // Fused half-steps (sinkhorn_attn_set_fused_half_steps): the half-steps after the cold ones, or
    // only those of the tail, are queued and run as one launch (vchain_kernel) on the caller's
    // stream for all problems.  Not with the dustbin (its extra element depends on every block
    // of the half-step before), not with a continuation schedule (a prescale between stages), not
    // under stream capture, and only if the workspace has room for the block counters.
    ChainArgs chain{};
    int *chain_done = nullptr;
    bool tail_now = false;
    {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        const bool capturing = hipStreamIsCapturing(st, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone;
        const size_t off = fused ? ws_core_bytes(p) : (ws_qs_bytes(p) + 255) / 256 * 256;
        if (g_fuse && !cx.noalloc && !capturing && !p.dustbin && !p.n_stages && ws && p.ws_given >= off + ws_chain_bytes(p))
            chain_done = reinterpret_cast<int *>(reinterpret_cast<unsigned char *>(ws) + off);
    }
    // the block size of the separate launches (sweep_one: 128 rows while a dispatch has few rows, else
    // 256) is taken per dispatch; the chain is one launch, so it needs the two halves of a split call
    // to agree (they differ only for an odd number of problems around the threshold): results stay
    // those of the separate launches bit for bit
    constexpr long SMALL_ROWS = 3L * 256 * 256;
    const int n_half = (cx.side && N >= 2) ? N / 2 : N;
    const bool chain_fr1 = sizeof(T) == 4 || (long)n_half * L <= SMALL_ROWS;
    if (chain_fr1 != (sizeof(T) == 4 || (long)(N - n_half ? N - n_half : N) * L <= SMALL_ROWS)) chain_done = nullptr;
    auto flush_chain = [&]() -> int {
        if (chain.nsteps == 0) return SKA_OK;
        SKA_TRY(cx.join());   // the chain takes all problems on the caller's stream
        chain.base = base;
        chain.base.c2 = stage_c2; chain.base.sdb2 = stage_sdb2;
        chain.Q = Q; chain.K = K; chain.UV = UV; chain.us = us; chain.Lp = Lp;
        chain.log_a = p.log_a; chain.log_b = p.log_b; chain.len_q = p.len_q; chain.len_k = p.len_k;
        chain.done = chain_done; chain.spin_limit = g_spin_limit;
        chain.rev0 = nlaunch & 1;
        const bool fr1 = chain_fr1;
        const long nflag = (long)N * ((L + 127) / 128);
        hipLaunchKernelGGL(fill_kernel, dim3((unsigned)((nflag + 255) / 256)), dim3(256), 0, st,
                           reinterpret_cast<float *>(chain_done), nflag, nflag, 1, 0.f);
        if (hipGetLastError() != hipSuccess) return SKA_EHIP;
        int rc;
        if constexpr (sizeof(T) == 2) rc = fr1 ? launch_vchain<T, D, 1>(chain, N, st, cx.dev, 0) : launch_vchain<T, D, 2>(chain, N, st, cx.dev, 1);
        else rc = launch_vchain<T, D, 1>(chain, N, st, cx.dev, 0);
        if (rc == SKA_EUNSUPPORTED) {   // the device cannot hold the grid: one launch per half-step after all
            for (int i = 0; i < chain.nsteps; ++i) {
                const unsigned code = chain.code[i];
                const bool row = code & 1;
                SweepArgs a = base;
                a.c2 = stage_c2; a.sdb2 = stage_sdb2;
                a.X = row ? Q : K; a.Y = row ? K : Q;
                a.yt = vec((code >> 8) & 255); a.xs = vec((code >> 16) & 255); a.out_vec = vout(code >> 24);
                a.olog = Vec{row ? p.log_a : p.log_b, (long)Lp};
                a.len_own = row ? p.len_q : p.len_k; a.len_oth = row ? p.len_k : p.len_q;
                a.rev = (chain.rev0 + i) & 1;
                SKA_TRY((sweep_one<T, D>(M_LSE, a, N, st, cx.dev)));
            }
            rc = SKA_OK;
        }
        nlaunch += chain.nsteps;
        if (pt_run) pt_run->launched(chain.nsteps);
        chain.nsteps = 0;
        SKA_TRY(rc);
        return cx.fork();
    };
    auto half = [&](bool row, int yslot, int prevslot, int outslot) -> int {
        if (chain_done && cold == 0 && (g_fuse >= 2 || tail_now)) {
            if (chain.nsteps == MAXCHAIN) SKA_TRY(flush_chain());
            chain.code[chain.nsteps++] = (row ? 1u : 0u) | ((unsigned)yslot << 8) | ((unsigned)prevslot << 16) | ((unsigned)outslot << 24);
            return SKA_OK;
        }
        SweepArgs a = base;
        a.c2 = stage_c2; a.sdb2 = stage_sdb2;
        a.spoke_own = row ? SQ : SK; a.spoke_oth = row ? SK : SQ;
        a.X = row ? Q : K; a.Y = row ? K : Q;
        a.yt = vec(yslot); a.xs = vec(prevslot); a.out_vec = vout(outslot);
        a.olog = Vec{row ? p.log_a : p.log_b, (long)Lp};
        a.len_own = row ? p.len_q : p.len_k; a.len_oth = row ? p.len_k : p.len_q;
        // successive sweeps walk the blocks in opposite directions: a sweep then starts on
        // the rows its predecessor touched last, which are still in L2
        a.rev = nlaunch++ & 1;
        SKA_TRY((sweep<T, D>(cx, cold > 0 ? M_LSE_FIRST : M_LSE, a, N)));
        if (cold > 0) pt_first.launched();
        else pt_run->launched();
        if (cold > 0 && --cold == 0) {   // the run of identical scaling sweeps starts after the cold launches
            pt_first.end();
            pt_run = new (pt_run_mem) PhaseTimer(SKA_PH_SCALING, cx);
        }
        return SKA_OK;
    };
    auto halves = [&]() -> int {
        // base solve: T steps at eps, or the stages of the continuation schedule (remark
        // "Fixed-Budget eps-Scaling"): stage s runs on the scores A / eps_s; between stages both
        // potentials are carried in cost units, x -> x eps_s / eps_{s+1} (u only stabilises)
        const int nst = p.resume_t ? 0 : p.n_stages ? p.n_stages : 1;
        for (int sidx = 0; sidx < nst; ++sidx) {
            const float es = p.n_stages ? p.eps_stage[sidx] : p.eps;
            const int Ts = p.n_stages ? p.T_stage[sidx] : p.T;
            if (sidx > 0) {
                SKA_TRY(cx.join());
                const float ratio = p.eps_stage[sidx - 1] / es;
                long tot = 2L * Lp * N;
                hipLaunchKernelGGL(scale_kernel, dim3((tot + 255) / 256), dim3(256), 0, st, UV, 2L * Lp, us, N, ratio);
                if (hipGetLastError() != hipSuccess) return SKA_EHIP;
                SKA_TRY((make_scores_operand<T>(p, es, Qin, ws, &Q, &stage_c2, st)));
                SKA_TRY(cx.fork());
            }
            stage_sdb2 = p.sdb * (p.eps / es) * LOG2E;
            for (int t = 0; t < Ts; ++t) {
                SKA_TRY(half(true, 1, 0, 0));
                SKA_TRY(half(false, 0, 1, 1));
            }
        }
        stage_c2 = base.c2 = (sizeof(T) == 2) ? 1.f : base.cs * LOG2E;   // the tail runs at eps (= the last stage's)
        stage_sdb2 = base.sdb2;
        tail_now = true;
        for (int t = p.resume_t ? p.resume_t : 1; t <= R; ++t) {
            SKA_TRY(half(true, 2 * t - 1, 2 * t - 2, 2 * t));    // u_t from v_{t-1}
            SKA_TRY(half(false, 2 * t, 2 * t - 1, 2 * t + 1));   // v_t from u_t
        }
        return flush_chain();
    };
    SKA_TRY(cx.fork());   // everything above ran for all problems on st
    const int rc_halves = halves();
    if (pt_run) pt_run->~PhaseTimer();
    SKA_TRY(rc_halves);
    // output map with the terminal plan
    PhaseTimer pt_out(SKA_PH_OUTPUT, cx);
    SweepArgs a = base;
    a.X = Q; a.Y = K; a.Pay = V; a.out_mat = O; a.xs = vec(2 * R); a.yt = vec(2 * R + 1);
    a.len_own = p.len_q; a.len_oth = p.len_k;
    if (p.token()) { a.spoke_own = SQ; a.pay_db = p.v_db; }   // O_i += P(i, d_k) v_db
    if (fused_gu(p, fused, G)) { a.dot_mat = G; a.dot_out = VecOut{reinterpret_cast<float *>(ws), p.ldw()}; }
    a.rev = nlaunch & 1;
    pt_out.launched();
    SKA_TRY((sweep<T, D>(cx, M_APPLY, a, N)));
    pt_out.end();
    return fused ? SKA_OK : cx.join();
}

template <typename T, int D>
int bwd_impl(Call &cx, const Problem &p, const void *Qin, const void *K, const void *V, const void *O,
             const void *G, const float *UV, void *dQ, void *dK, void *dV, float *eta0, void *ws,
             const float *seed = nullptr, bool fused = false)
{
    const hipStream_t st = cx.st;
    // fused: the forward of the same call has just run (sinkhorn_attn_step): its prescaled operand
    // is in place, and the helper stream is still running its half of the problems.
    // seed != null: no output map at the end of the chain.  The reverse recurrences start from
    // vbar_R = seed (a cotangent of v^(R) given by the caller), Z = 0, and only dQ, dK are
    // produced: the vector-Jacobian product through R full steps started at v = 0.
    // Q below is the score operand (bf16 storage: prescaled copy at the end of the workspace,
    // c2 = 1); it also serves as the payload of the dK sweep, whose output scale absorbs it
    const void *Q = nullptr;
    float c2 = 0.f;
    if (fused) {
        Q = (sizeof(T) == 2) ? reinterpret_cast<unsigned char *>(ws) + ws_vec_bytes(p) : Qin;
        c2 = (sizeof(T) == 2) ? 1.f : LOG2E / (p.eps * sqrtf((float)p.d));
    } else {
        PhaseTimer pt(SKA_PH_PRESCALE, cx);
        SKA_TRY((make_scores_operand<T>(p, p.eps, Qin, reinterpret_cast<unsigned char *>(ws) + ws_vec_bytes(p), &Q, &c2, st)));
        pt.launched(sizeof(T) == 2 ? 1 : 0);
    }
    const int N = p.N(), L = p.L, Lp = p.Lp();
    const int R = p.R, nq = p.direct() ? R : pack_groups(R);
    const long us = p.uv_us ? p.uv_us : 2L * (R + 1) * Lp, ldw = p.ldw();
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
    // the kernels before the sweeps take all problems on st -- except the plain row dot of a fused
    // step, which each stream does for its own half so that the two chains stay apart
    const bool own_halves = fused && cx.side && !seed && !p.dustbin;
    if (fused && !own_halves) SKA_TRY(cx.join());
    if (p.token()) {
        SQ = Vec{tok, ldw};
        SK = Vec{tok + nldp, ldw};
        SKA_TRY((spoke_scores<T, D>(p, Qin, K, tok, tok + nldp, st)));
    }

    // g_u = <dO_i, O_i> (= (P22 . Z) 1); dustbin row has dO = 0
    PhaseTimer pt_gu(SKA_PH_ROWDOT, cx);
    if (seed || !fused_gu(p, fused, G)) pt_gu.launched();
    constexpr int LPR = D * (int)sizeof(T) / 16;
    if (seed) {
        hipLaunchKernelGGL(seed_kernel, vgrid, dim3(256), 0, st, seed, p.log_b, vbar(R), ldw, Lp);
        if (hipGetLastError() != hipSuccess) return SKA_EHIP;
    } else if (fused_gu(p, fused, G)) {
        // the forward's output map has left g_u in place (from its fp32 accumulators)
    } else {
        const int n1 = own_halves ? N / 2 : N;
        hipLaunchKernelGGL((rowdot_kernel<T, D>), dim3(((long)Lp * LPR + 255) / 256, n1), dim3(256), 0, st,
                           reinterpret_cast<const T *>(G),
                           reinterpret_cast<const T *>(O), gu, ldw, L, Lp, p.len_q, p.H, 0);
        if (N > n1)
            hipLaunchKernelGGL((rowdot_kernel<T, D>), dim3(((long)Lp * LPR + 255) / 256, N - n1), dim3(256), 0,
                               cx.side->s, reinterpret_cast<const T *>(G) + (long)n1 * L * D,
                               reinterpret_cast<const T *>(O) + (long)n1 * L * D, gu + n1 * ldw, ldw, L, Lp, p.len_q,
                               p.H, n1);
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
    if (!own_halves) SKA_TRY(cx.fork());   // everything above ran for all problems on st
    // dV_j = sum_i P_RR,ij dO_i ; vbar_R,j = <V_j, dV_j>  (column-oriented)
    if (!seed) {
        PhaseTimer pt(SKA_PH_DV, cx);
        pt.launched();
        SweepArgs a = base;
        a.X = K; a.Y = Q; a.Pay = G; a.out_mat = dV; a.xs = uv(2 * R + 1); a.yt = uv(2 * R);
        a.dot_mat = V; a.dot_out = wo(vbar(R));
        a.len_own = p.len_k; a.len_oth = p.len_q;
        a.olog = Vec{p.log_b, (long)Lp};   // the workspace holds vbar / b and ubar / a (general marginals)
        a.rev = nlaunch++ & 1;
        SKA_TRY((sweep<T, D>(cx, M_APPLY, a, N)));
    }
    // reverse recurrences of Prop. 1, each one band mat-vec with a staircase factor
    // written as P22 times row/column modifiers folded into the exponent (Prop. 2)
    auto matvec = [&](bool row, Vec xs, Vec yt, float *w, float *pre, VecOut out, bool scaled = true) -> int {
        SweepArgs a = base;
        a.X = row ? Q : K; a.Y = row ? K : Q;
        a.xs = xs; a.yt = yt; a.w = wv(w); a.pre = Vec{pre, ldw}; a.out_vec = out;
        if (scaled) a.olog = Vec{row ? p.log_a : p.log_b, (long)Lp};
        a.len_own = row ? p.len_q : p.len_k; a.len_oth = row ? p.len_k : p.len_q;
        a.spoke_own = row ? SQ : SK; a.spoke_oth = row ? SK : SQ;
        a.rev = nlaunch++ & 1;
        SKA_TRY((sweep<T, D>(cx, M_MATVEC, a, N)));
        return SKA_OK;
    };
    {
        PhaseTimer pt(SKA_PH_MATVEC, cx);
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
    PhaseTimer pt_final(SKA_PH_FINAL, cx);   // modifier packs and the two final sweeps
    pt_final.launched(2 * ((nq + MAXNQ - 1) / MAXNQ));
    {   // a problem's packs need only its own recurrences: each stream writes those of its half
        const int n1 = (cx.side && N >= 2) ? N / 2 : N;
        for (int part = 0; part < 2; ++part) {
            const int nb = part ? n1 : 0, cnt = part ? N - n1 : n1;
            if (cnt == 0) continue;
            hipLaunchKernelGGL(packs_kernel, dim3((Lp + 255) / 256, cnt), dim3(256), 0, part ? cx.side->s : st,
                               UV + (long)nb * us, Lp, R, wf + nb * ldw, nldp, ldw,
                               reinterpret_cast<float *>(rowp) + nb * ldw * 4L * nq,
                               reinterpret_cast<float *>(colp) + nb * ldw * 4L * nq, nq,
                               AUG ? aug + nb * ldw * 16 : nullptr, ldw, nldp, p.direct() ? 1 : 0, p.token() ? 1 : 0);
        }
        if (hipGetLastError() != hipSuccess) return SKA_EHIP;
    }
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
            SKA_TRY((sweep<T, D>(cx, final_mode, a, N)));
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
            SKA_TRY((sweep<T, D>(cx, final_mode, a, N)));
        }
    }
    pt_final.end();
    SKA_TRY(cx.join());
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
    size_t core, eq, ek, uvb, uvx, eta, norm, total;
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
    l.uvx = l.uvb + up256((size_t)p.N() * 2 * (T + 1) * p.Lp() * sizeof(float));
    l.eta = l.uvx + up256((size_t)p.N() * 2 * (R_max + 1) * p.Lp() * sizeof(float));
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

// Scratch of the entry point that allocates nothing (sinkhorn_attn_step_static): one array per
// GPU, held from the moment the library is loaded on it until the process ends.  In host code
// the array's name is only a handle for hipGetSymbolAddress; kernels get the device address
// that call returned (kept per device in g_scratch_ptr).
static __device__ __align__(256) unsigned char scratch[SKA_STATIC_SCRATCH_BYTES];

namespace {
void *g_scratch_ptr[MAX_DEVICES];   // (g_mutex held)
}

// ====================================================================== C ABI
extern "C" {

size_t sinkhorn_attn_workspace_bytes(int B, int H, int L, int d, int W, int T, int R, int dustbin, int dtype)
{
    Problem p{B, H, L, d, W, T, R, dustbin ? 1 : 0, dtype, 1.f, 0.f};
    if (check_common(p) != SKA_OK) return 0;
    return ws_bytes(p);
}

static int fwd_call(const Problem &p_in, const void *Q, const void *K, const void *V, void *O, float *UV,
                    void *workspace, size_t workspace_bytes, void *stream)
{
    Problem p = p_in;
    p.ws_given = workspace ? workspace_bytes : 0;
    const int d = p.d, dtype = p.dtype;
    if (!Q || !K || !V || !O || !UV) return SKA_EINVAL;
    int rc = check_common(p);
    if (rc != SKA_OK) return rc;
    if (ws_qs_bytes(p) && (!workspace || workspace_bytes < ws_qs_bytes(p))) return SKA_EWORKSPACE;
    if (p.token() && (!workspace || workspace_bytes < ws_bytes(p))) return SKA_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 15) return SKA_EINVAL;
    Call cx(stream, p.N(), p.L, p.W);
    if (cx.rc != SKA_OK) return cx.rc;
#define SKA_FWD(TT_, DD_) return fwd_impl<TT_, DD_>(cx, p, Q, K, V, O, UV, workspace)
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
    Call cx(stream, p.N(), p.L, p.W);
    if (cx.rc != SKA_OK) return cx.rc;
#define SKA_BWD(TT_, DD_) return bwd_impl<TT_, DD_>(cx, p, Q, K, V, O, dO, UV, dQ, dK, dV, eta0, workspace)
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
    Call cx(stream, p.N(), p.L, p.W);
    if (cx.rc != SKA_OK) return cx.rc;
#define SKA_VJP(TT_, DD_) \
    return bwd_impl<TT_, DD_>(cx, p, Q, K, nullptr, nullptr, nullptr, UV, dQ, dK, nullptr, nullptr, workspace, eta)
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

int sinkhorn_attn_step(const void *Q, const void *K, const void *V, const void *dO, const float *log_a,
                       const float *log_b, const int *len_q, const int *len_k, void *O, float *UV, void *dQ,
                       void *dK, void *dV, float *eta0, int B, int H, int L, int d, int W, int T, int R, float eps,
                       int dustbin, float dustbin_score, int dtype, void *workspace, size_t workspace_bytes,
                       void *stream)
{
    Problem p{B, H, L, d, W, T, R, dustbin ? 1 : 0, dtype, eps, dustbin_score, log_a, log_b, len_q, len_k};
    p.ws_given = workspace_bytes;
    if (!Q || !K || !V || !dO || !O || !UV || !dQ || !dK || !dV) return SKA_EINVAL;
    int rc = check_common(p);
    if (rc != SKA_OK) return rc;
    if (!workspace || workspace_bytes < ws_bytes(p)) return SKA_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 15) return SKA_EINVAL;
    Call cx(stream, p.N(), p.L, p.W);
    if (cx.rc != SKA_OK) return cx.rc;
#define SKA_STEP(TT_, DD_)                                                                              \
    do {                                                                                                \
        rc = fwd_impl<TT_, DD_>(cx, p, Q, K, V, O, UV, workspace, true, dO);                            \
        if (rc == SKA_OK)                                                                               \
            rc = bwd_impl<TT_, DD_>(cx, p, Q, K, V, O, dO, UV, dQ, dK, dV, eta0, workspace, nullptr, true); \
        return rc;                                                                                      \
    } while (0)
    if (dtype == SKA_F32) {
        if (d == 32) SKA_STEP(float, 32);
        if (d == 64) SKA_STEP(float, 64);
        SKA_STEP(float, 128);
    } else {
        if (d == 32) SKA_STEP(__bf16, 32);
        if (d == 64) SKA_STEP(__bf16, 64);
        SKA_STEP(__bf16, 128);
    }
#undef SKA_STEP
}

int sinkhorn_attn_step_static(const void *Q, const void *K, const void *V, const void *dO, const float *log_a,
                              const float *log_b, const int *len_q, const int *len_k, void *O, float *UV,
                              void *dQ, void *dK, void *dV, float *eta0, int B, int H, int L, int d, int W, int T,
                              int R, float eps, int dustbin, float dustbin_score, int dtype, void *stream)
{
    Problem p{B, H, L, d, W, T, R, dustbin ? 1 : 0, dtype, eps, dustbin_score, log_a, log_b, len_q, len_k};
    if (!Q || !K || !V || !dO || !O || !UV || !dQ || !dK || !dV) return SKA_EINVAL;
    int rc = check_common(p);
    if (rc != SKA_OK) return rc;
    if (ws_bytes(p) > (size_t)SKA_STATIC_SCRATCH_BYTES) return SKA_ESTATIC;
    // everything on the caller's stream: no helper stream, no events, nothing created
    Call cx(stream, p.N(), p.L, p.W, false);
    if (cx.rc != SKA_OK) return cx.rc;
    if (!g_scratch_ptr[cx.dev]) {   // once per device, with that device current
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SKA_EHIP;
        g_scratch_ptr[cx.dev] = ptr;
    }
    // Nothing in the scratch has to start at zero: every kernel of a step writes what a later
    // one reads (the same holds for a caller's workspace, which arrives uninitialised).
    void *ws = g_scratch_ptr[cx.dev];
#define SKA_STEP(TT_, DD_)                                                                              \
    do {                                                                                                \
        rc = fwd_impl<TT_, DD_>(cx, p, Q, K, V, O, UV, ws, true, dO);                                   \
        if (rc == SKA_OK)                                                                               \
            rc = bwd_impl<TT_, DD_>(cx, p, Q, K, V, O, dO, UV, dQ, dK, dV, eta0, ws, nullptr, true);    \
        return rc;                                                                                      \
    } while (0)
    if (dtype == SKA_F32) {
        if (d == 32) SKA_STEP(float, 32);
        if (d == 64) SKA_STEP(float, 64);
        SKA_STEP(float, 128);
    } else {
        if (d == 32) SKA_STEP(__bf16, 32);
        if (d == 64) SKA_STEP(__bf16, 64);
        SKA_STEP(__bf16, 128);
    }
#undef SKA_STEP
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
    // Depth R + 1 shares the base state and the tail steps 1 .. R with depth R, so nothing is solved
    // twice: UVx holds the iterates of the deepest tail so far at the stride of depth R_max, its
    // slots 0, 1 are the base state (u_T, v_T) the run above ended in, and depth R adds one tail
    // step (two half-steps) and an output map to it.
    float *UVx = reinterpret_cast<float *>(w + l.uvx);
    const int Lp = p.Lp(), N = p.N();
    const long usx = 2L * (R_max + 1) * Lp;
    hipLaunchKernelGGL(slots_copy_kernel, dim3((unsigned)((2L * Lp + 255) / 256), N), dim3(256), 0, st, UVb,
                       2L * (T + 1) * Lp, 2 * T, UVx, usx, 0, 2, Lp);
    if (hipGetLastError() != hipSuccess) return SKA_EHIP;
    int R_last = 0;
    for (int R = 1; R <= R_max; ++R) {
        R_last = R;
        Problem q = p;
        q.R = R; q.uv_us = usx;
        Problem qf = q;
        qf.resume_t = R;
        SKA_TRY(fwd_call(qf, Q, K, V, O, UVx, w, l.eq, stream));
        SKA_TRY(bwd_problem(q, Q, K, V, O, dO, UVx, dQ, dK, dV, eta, w, l.eq, stream));
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
            break;
        }
    }
    // the caller's UV: the iterates of the depth whose results are left in O, dQ, dK, dV, densely packed
    hipLaunchKernelGGL(slots_copy_kernel, dim3((unsigned)((2L * (R_last + 1) * Lp + 255) / 256), N), dim3(256), 0, st,
                       UVx, usx, 0, UV, 2L * (R_last + 1) * Lp, 0, 2 * (R_last + 1), Lp);
    return hipGetLastError() == hipSuccess ? SKA_OK : SKA_EHIP;
}

int sinkhorn_attn_probe_issue(float *scratch, size_t scratch_bytes, int tiles, int waves_per_simd, double *ms8,
                              void *stream)
{
    if (!scratch || !ms8 || tiles < 1 || tiles > (1 << 20) || waves_per_simd < 1 || waves_per_simd > 8) return SKA_EINVAL;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return SKA_EHIP;
    const int nblk = cus * waves_per_simd;   // a 256-thread workgroup puts one wavefront on each of a CU's four SIMDs
    if (scratch_bytes < (size_t)nblk * 256 * sizeof(float)) return SKA_EWORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return SKA_EHIP;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return SKA_EHIP; }
    int rc = SKA_OK;
    for (int what = 0; what < 8 && rc == SKA_OK; ++what) {
        for (int rep = 0; rep < 2; ++rep) {   // the second launch is the timed one
            if (rep == 1) (void)hipEventRecord(e0, st);
            if (what == 0) hipLaunchKernelGGL(issue_probe_kernel<0>, dim3(nblk), dim3(256), 0, st, scratch, tiles);
            if (what == 1) hipLaunchKernelGGL(issue_probe_kernel<1>, dim3(nblk), dim3(256), 0, st, scratch, tiles);
            if (what == 2) hipLaunchKernelGGL(issue_probe_kernel<2>, dim3(nblk), dim3(256), 0, st, scratch, tiles);
            if (what == 3) hipLaunchKernelGGL(issue_probe_kernel<3>, dim3(nblk), dim3(256), 0, st, scratch, tiles);
            if (what == 4) hipLaunchKernelGGL(issue_probe_kernel<4>, dim3(nblk), dim3(256), 0, st, scratch, tiles);
            if (what == 5) hipLaunchKernelGGL(issue_probe_kernel<5>, dim3(nblk), dim3(256), 0, st, scratch, tiles);
            if (what == 6) hipLaunchKernelGGL(issue_probe_kernel<6>, dim3(nblk), dim3(256), 0, st, scratch, tiles);
            if (what == 7) hipLaunchKernelGGL(issue_probe_kernel<7>, dim3(nblk), dim3(256), 0, st, scratch, tiles);
        }
        float ms = 0.f;
        if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess || hipGetLastError() != hipSuccess)
            rc = SKA_EHIP;
        ms8[what] = ms;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}

int sinkhorn_attn_set_streams(int n)
{
    if (n != 1 && n != 2) return SKA_EINVAL;
    std::lock_guard<std::mutex> lk(g_mutex);
    g_streams = n;
    return SKA_OK;
}

int sinkhorn_attn_set_fused_half_steps(int mode, unsigned spin_limit)
{
    if (mode < 0 || mode > 2) return SKA_EINVAL;
    std::lock_guard<std::mutex> lk(g_mutex);
    g_fuse = mode;
    g_spin_limit = spin_limit ? spin_limit : (1u << 18);
    return SKA_OK;
}

int sinkhorn_attn_set_split_min_edges(double edges)
{
    if (!(edges >= 0.0)) return SKA_EINVAL;
    std::lock_guard<std::mutex> lk(g_mutex);
    g_split_min_edges = edges;
    return SKA_OK;
}

int sinkhorn_attn_profile_enable(int on)
{
    std::lock_guard<std::mutex> lk(g_mutex);
    g_prof_on = on < 0 ? 0 : (on > 2 ? 2 : on);
    return SKA_OK;
}

int sinkhorn_attn_profile_read_phases(double *elapsed_ms, long *launches)
{
    if (!elapsed_ms || !launches) return SKA_EINVAL;
    for (int k = 0; k < SKA_PH_COUNT; ++k) { elapsed_ms[k] = 0.0; launches[k] = 0; }
    int rc = SKA_OK;
    std::lock_guard<std::mutex> lk(g_mutex);
    for (int i = 0; i < g_prof_n; ++i) {
        float t = 0.f, t2 = 0.f;
        if (hipEventSynchronize(g_prof[i].b) != hipSuccess ||
            hipEventElapsedTime(&t, g_prof[i].a, g_prof[i].b) != hipSuccess)
            rc = SKA_EHIP;
        if (g_prof[i].b2) {   // the helper stream's end of the span: the later of the two counts
            if (hipEventSynchronize(g_prof[i].b2) != hipSuccess ||
                hipEventElapsedTime(&t2, g_prof[i].a, g_prof[i].b2) != hipSuccess)
                rc = SKA_EHIP;
            (void)hipEventDestroy(g_prof[i].b2);
            if (t2 > t) t = t2;
        }
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
    case SKA_ESTATIC: return "problem too large for sinkhorn_attn_step_static: it needs more scratch than the library's static buffer (SKA_STATIC_SCRATCH_BYTES); use sinkhorn_attn_step with a workspace";
    default: return "unknown status";
    }
}

}  // extern "C"
