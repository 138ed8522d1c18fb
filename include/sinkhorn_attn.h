/*
 * sinkhorn_attn.h -- C ABI of the MI355X (gfx950) banded Sinkhorn attention library.
 *
 * The operator (paper: "Block-Wise Differentiable Sinkhorn Attention"):
 *   scores      S_ij = <Q_i, K_j> / (eps * sqrt(d))  on the band |i-j| <= W     (Section 2.1)
 *   half-steps  u_i = -log sum_j exp(S_ij + v_j),  v_j = -log sum_i exp(S_ij + u_i)
 *                                                                      (Eq. 1, Eq. 2)
 *   base        T steps (row half-step, then column half-step) from v = 0; the result
 *               (u0, v0) is a constant for differentiation              (Section 2.2)
 *   tail        R further steps giving (u1, v1), ..., (uR, vR); R = 2 is the paper's
 *               setting                                                 (Section 2.2)
 *   output      O_i = sum_j exp(S_ij + uR_i + vR_j) V_j, no renormalisation
 *                                                                      (Section 2.2)
 *   backward    exact adjoint of the tail + output (Prop. 1), evaluated from the
 *               single plan P_RR = exp(S + uR + vR) and vector modifiers (Prop. 2)
 *   dustbin     optional: one extra row d_q and column d_k joined to every token
 *               by an edge of constant score `dustbin_score`; all L+1 row and
 *               column targets are one; V at d_k is zero and the d_q output row is
 *               not returned (Section 2.3, sparse-spoke support)
 *
 * Conventions common to every entry point
 *   - Every pointer is a DEVICE pointer owned by the caller unless stated.  The
 *     library allocates no device memory, frees nothing and keeps no pointer after return.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     null stream) and is asynchronous with respect to the host.  A call on two or more
 *     problems (B*H >= 2) whose sweeps are long enough to be worth two dispatches (at least
 *     50 M band edges per half) runs the band sweeps of the second half of its problems on a helper
 *     stream that the library creates once per device (non-blocking, default priority, never
 *     destroyed): it is forked from `stream` by an event after the call's first kernels and
 *     joined to it again before the call returns, so everything the call does is ordered on
 *     `stream` as seen by the caller, also under stream capture, and also when a launch fails
 *     half-way through a call.  sinkhorn_attn_set_streams(1) keeps all work on `stream` itself.
 *   - Entry points may be called from several host threads at once (each on a stream of its
 *     own): a call holds a process-wide lock while it enqueues its kernels, so calls are
 *     serialised at the enqueue while their GPU work overlaps as the streams allow.
 *   - Tensors Q, K, V, O, dO, dQ, dK, dV are [B, H, L, d], contiguous, row-major,
 *     of the element type `dtype` (SKA_F32: float; SKA_BF16: bfloat16).  All
 *     scaling vectors and all accumulation are fp32.
 *   - UV is [B, H, 2(R+1), Lp] fp32 with Lp = L + (dustbin ? 1 : 0), the vectors
 *     ordered u0, v0, u1, v1, ..., uR, vR (natural-log potentials, ungauged;
 *     element L is the dustbin token when present).
 *   - Return value: SKA_OK or a negative ska_status.  Arguments are checked
 *     before anything is launched; nothing is written on an argument error.
 *   - Supported: d in {32, 64, 128}; R in 1 .. 32 (T = 0 with R = T' + R' stops nothing:
 *     the backward is then full backpropagation through a T'-step base solve, and its
 *     difference to the (T', R') backward is the bias of the a-posteriori certificate);
 *     1 <= L <= 2^24, B*H <= 65535, W >= 0 (W >= L-1 is the
 *     dense problem), T >= 0, eps > 0 and finite.
 */
#ifndef SINKHORN_ATTN_H
#define SINKHORN_ATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SKA_F32 = 0, SKA_BF16 = 1 } ska_dtype;

typedef enum {
    SKA_OK = 0,
    SKA_EINVAL = -1,       /* null required pointer, non-positive size, bad eps        */
    SKA_EUNSUPPORTED = -2, /* R outside 1..32, unsupported d, unknown dtype             */
    SKA_EWORKSPACE = -3,   /* workspace smaller than sinkhorn_attn_workspace_bytes()    */
    SKA_EHIP = -4,         /* a HIP launch failed (hipGetLastError)                     */
    SKA_ESTATIC = -5       /* sinkhorn_attn_step_static: the problem needs more scratch */
                           /* than SKA_STATIC_SCRATCH_BYTES                             */
} ska_status;

/*
 * Bytes of device scratch that sinkhorn_attn_bwd needs for these sizes; the
 * forward is content with the same buffer (it needs B*H*L*d*2 bytes for bf16
 * storage, none for fp32; with all of it, it can fuse half-steps, see
 * sinkhorn_attn_set_fused_half_steps).  Host-only, no GPU call.  Returns 0 on invalid sizes.
 */
size_t sinkhorn_attn_workspace_bytes(int B, int H, int L, int d, int W, int T, int R, int dustbin,
                                     int dtype);

/*
 * Forward: stopped T-step base solve, R-step tail, plan-weighted V
 * (Section 2.1-2.2, Eq. 1-2; Section 2.3 when dustbin != 0).
 *   in : Q, K, V [B,H,L,d]
 *   out: O [B,H,L,d]; UV [B,H,2(R+1),Lp] (all vectors are written)
 * workspace: 16-byte aligned scratch; bf16 storage needs at least B*H*L*d*2 bytes
 * (a copy of Q with the score scale folded in), fp32 storage needs none and accepts
 * NULL.  A buffer of sinkhorn_attn_workspace_bytes() always suffices.
 */
int sinkhorn_attn_fwd(const void *Q, const void *K, const void *V, void *O, float *UV, int B, int H,
                      int L, int d, int W, int T, int R, float eps, int dustbin,
                      float dustbin_score, int dtype, void *workspace, size_t workspace_bytes,
                      void *stream);

/*
 * Backward: exact VJP of the stopped-base surrogate for an arbitrary output
 * cotangent dO (Prop. 1), scheduled from the one reference plan P22 and the
 * modifiers a_t = exp(u_t - u_R), b_t = exp(v_t - v_R) (Prop. 2; for R = 2: alpha = a_1,
 * beta = b_1, delta = b_0).
 *   in : Q, K, V, O (as returned by the forward), dO [B,H,L,d]; UV from the forward
 *   out: dQ, dK, dV [B,H,L,d], overwritten
 *        eta0 [B,H,Lp] fp32 or NULL: the base cotangent vbar^(0) that the
 *        stop-gradient discards (Prop. 5 calls it eta_R)
 * workspace: at least sinkhorn_attn_workspace_bytes(...) bytes, 16-byte aligned;
 * its contents are scratch before and after the call.
 */
int sinkhorn_attn_bwd(const void *Q, const void *K, const void *V, const void *O, const void *dO,
                      const float *UV, void *dQ, void *dK, void *dV, float *eta0, int B, int H,
                      int L, int d, int W, int T, int R, float eps, int dustbin,
                      float dustbin_score, int dtype, void *workspace, size_t workspace_bytes,
                      void *stream);

/*
 * Forward and backward in one call, for a cotangent dO that is known beforehand (the paper's
 * "complete-step executable": output plus the Q/K/V VJP for a given output cotangent, which is
 * what its throughput is quoted on).  O, UV and dV are those of sinkhorn_attn_fwd_varlen followed
 * by sinkhorn_attn_bwd_varlen bit for bit; dQ, dK and eta0 agree with them to rounding: without a
 * dustbin the seed g_u = <dO_i, O_i> (Sec. 2.2) is taken from the output map's fp32 accumulators
 * instead of from the stored, dtype-rounded O (with a dustbin they too are bit for bit).  What the
 * single call saves is the second prescale of Q, the pass over O and dO for g_u, and the joining
 * of the two streams between the two directions: each half of the problems runs its forward and
 * its backward as one uninterrupted chain.
 *   in : Q, K, V, dO; log_a, log_b, len_q, len_k as in those calls (may be NULL)
 *   out: O, UV, dQ, dK, dV, eta0 (may be NULL)
 *   workspace: sinkhorn_attn_workspace_bytes(...) bytes, 16-byte aligned.
 */
int sinkhorn_attn_step(const void *Q, const void *K, const void *V, const void *dO,
                       const float *log_a, const float *log_b, const int *len_q, const int *len_k,
                       void *O, float *UV, void *dQ, void *dK, void *dV, float *eta0, int B, int H,
                       int L, int d, int W, int T, int R, float eps, int dustbin, float dustbin_score,
                       int dtype, void *workspace, size_t workspace_bytes, void *stream);

/*
 * sinkhorn_attn_step for callers that cannot allocate device memory or have it allocated for
 * them: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments and results as sinkhorn_attn_step, bit for bit, without the workspace: the
 * scratch is a static device array inside the library of SKA_STATIC_SCRATCH_BYTES bytes (32 MiB;
 * every GPU the library is loaded on holds it until the process ends).  The call allocates and
 * frees nothing, creates no stream and no event, and keeps all its kernels on `stream` (it never
 * uses the helper stream; the profiling hooks ignore it).
 *   A problem whose sinkhorn_attn_workspace_bytes(...) exceeds SKA_STATIC_SCRATCH_BYTES is
 *   refused with SKA_ESTATIC before anything is launched (about 98,000 token-heads B*H*L at
 *   d = 64, bf16, R = 2).
 *   All calls on one GPU share that GPU's array and it keeps the last call's contents (nothing
 *   in it needs clearing: each step writes what it reads).  Two calls that overlap on one GPU
 *   (different streams, or different host threads) race on it: the caller keeps them ordered.
 */
#define SKA_STATIC_SCRATCH_BYTES (32u << 20)
int sinkhorn_attn_step_static(const void *Q, const void *K, const void *V, const void *dO,
                              const float *log_a, const float *log_b, const int *len_q,
                              const int *len_k, void *O, float *UV, void *dQ, void *dK, void *dV,
                              float *eta0, int B, int H, int L, int d, int W, int T, int R, float eps,
                              int dustbin, float dustbin_score, int dtype, void *stream);

/*
 * The same two calls with compatible general marginals (appendix "Compatible General
 * Marginals": half-steps u_i = log a_i - log sum_j exp(S_ij + v_j), v_j = log b_j - log sum_i
 * exp(S_ij + u_i); in the backward every ubar is divided by a and every vbar by b where it
 * multiplies a plan, per the general-marginal half-step Jacobians and finite-tail VJP there).
 *   log_a, log_b: [B,H,L] fp32 device arrays, logarithms of the positive row / column
 *   targets; the caller makes them compatible (equal totals per problem).  NULL = unit
 *   targets (both NULL: exactly the calls above).  eta0, when requested, is the raw base
 *   cotangent vbar^(0) (not divided by b).  Not combined with the dustbin, whose targets are
 *   all one: SKA_EUNSUPPORTED.
 */
int sinkhorn_attn_fwd_marginals(const void *Q, const void *K, const void *V, const float *log_a,
                                const float *log_b, void *O, float *UV, int B, int H, int L, int d,
                                int W, int T, int R, float eps, int dustbin, float dustbin_score,
                                int dtype, void *workspace, size_t workspace_bytes, void *stream);
int sinkhorn_attn_bwd_marginals(const void *Q, const void *K, const void *V, const float *log_a,
                                const float *log_b, const void *O, const void *dO, const float *UV,
                                void *dQ, void *dK, void *dV, float *eta0, int B, int H, int L, int d,
                                int W, int T, int R, float eps, int dustbin, float dustbin_score,
                                int dtype, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same two calls on a padded batch of sequences of different lengths (the remark after
 * Eq. 1-2: rectangular masked examples run the same unit-target half-steps although their
 * active row and column counts differ).  Batch item b uses the support
 * {(i, j): |i - j| <= W, i < len_q[b], j < len_k[b]} in all of its H heads.
 *   len_q, len_k: int32 device arrays [B]; values are clamped to [0, L]; NULL = L.  Both
 *   NULL: exactly the calls above.  The arrays are read by the kernels, never by the host.
 *   Rows of Q, dO beyond len_q[b] and of K, V beyond len_k[b] are never used (they may hold
 *   anything).  Results there are zeros: rows of O, dQ beyond len_q[b], of dK, dV beyond
 *   len_k[b], and the potentials (and eta0) of indices beyond the lengths.  A query row whose
 *   band holds no valid key (i - W >= len_k[b]), and likewise a key column, takes no part
 *   either: potential 0, zero results.  Strides stay those of the padded [B,H,L,...] arrays.
 *   log_a, log_b as in the marginals calls (entries beyond the lengths are not read).
 *   Not combined with the dustbin (its element sits at index L): SKA_EUNSUPPORTED.
 */
int sinkhorn_attn_fwd_varlen(const void *Q, const void *K, const void *V, const float *log_a,
                             const float *log_b, const int *len_q, const int *len_k, void *O,
                             float *UV, int B, int H, int L, int d, int W, int T, int R, float eps,
                             int dustbin, float dustbin_score, int dtype, void *workspace,
                             size_t workspace_bytes, void *stream);
int sinkhorn_attn_bwd_varlen(const void *Q, const void *K, const void *V, const float *log_a,
                             const float *log_b, const int *len_q, const int *len_k, const void *O,
                             const void *dO, const float *UV, void *dQ, void *dK, void *dV,
                             float *eta0, int B, int H, int L, int d, int W, int T, int R, float eps,
                             int dustbin, float dustbin_score, int dtype, void *workspace,
                             size_t workspace_bytes, void *stream);

/*
 * Forward with inactive tokens (the masked half-steps of Eq. 1-2 with a boolean activity per
 * token on either side): the support is {(i, j): |i - j| <= W, mask_q[b][i], mask_k[b][j]}.
 *   mask_q, mask_k: uint8 device arrays [B,L] (shared by the heads), nonzero = active; NULL = all
 *   active.  An inactive token, and an active one whose band holds no active partner, takes no
 *   part: its potentials in UV are -inf in every iterate, its rows of O, dQ, dK, dV are zeros.
 *   The rows of Q, K, V, dO at inactive tokens must still hold finite numbers (they are
 *   multiplied by zero plan entries), unlike the padding of the _varlen calls.
 * There is no masked backward call: the -inf potentials in UV carry the masks, and every backward
 * entry point (sinkhorn_attn_bwd, _bwd_marginals, sinkhorn_attn_base_vjp, ...) applied to this UV
 * gives the masked operator's gradients.  Not combined with the dustbin: SKA_EUNSUPPORTED.
 */
int sinkhorn_attn_fwd_masked(const void *Q, const void *K, const void *V, const float *log_a,
                             const float *log_b, const unsigned char *mask_q,
                             const unsigned char *mask_k, void *O, float *UV, int B, int H, int L,
                             int d, int W, int T, int R, float eps, int dtype, void *workspace,
                             size_t workspace_bytes, void *stream);

/*
 * The dustbin as a learned token per side (Sec. "Single-Active-Dustbin Bridge": Q, K, V are
 * augmented by one active token, Q~ = [Q; q_db], K~ = [K; k_db], V~ = [V; v_db], and the same
 * unit-target operator runs on the augmented problem), on the sparse-spoke support
 * band + {(i, d_k)} + {(d_q, j)} + {(d_q, d_k)}: spoke scores q_i.k_db, q_db.k_j, q_db.k_db (all
 * divided by eps sqrt d) instead of one scalar, the dustbin key carries the value v_db, and the
 * backward also returns the gradients of the three tokens.  The dustbin query's output row is
 * dropped (no cotangent).  O(L d) extra work; the band sweeps are the same kernels.
 *   q_db, k_db, v_db : [B,H,d] fp32 device arrays, 16-byte aligned (in)
 *   dq_db, dk_db, dv_db : [B,H,d] fp32 (out)
 *   UV : [B,H,2(R+1),L+1] as with dustbin = 1; eta0 [B,H,L+1] or NULL.
 *   workspace: sinkhorn_attn_workspace_bytes(..., dustbin = 1, ...) bytes for BOTH calls.
 * Other arguments as in sinkhorn_attn_fwd / sinkhorn_attn_bwd.
 */
int sinkhorn_attn_fwd_dustbin_token(const void *Q, const void *K, const void *V, const float *q_db,
                                    const float *k_db, const float *v_db, void *O, float *UV, int B,
                                    int H, int L, int d, int W, int T, int R, float eps, int dtype,
                                    void *workspace, size_t workspace_bytes, void *stream);
int sinkhorn_attn_bwd_dustbin_token(const void *Q, const void *K, const void *V, const float *q_db,
                                    const float *k_db, const float *v_db, const void *O,
                                    const void *dO, const float *UV, void *dQ, void *dK, void *dV,
                                    float *dq_db, float *dk_db, float *dv_db, float *eta0, int B,
                                    int H, int L, int d, int W, int T, int R, float eps, int dtype,
                                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * Forward with a continuation schedule in the stopped base solve (remark "Fixed-Budget
 * eps-Scaling"): stage s = 1..n_stages runs T_stage[s] full steps on the scores A / eps_stage[s],
 * eps_stage[1] >= ... >= eps_stage[n_stages] = eps; T = sum of T_stage.  Between stages the
 * log-scalings are carried as potentials in cost units (multiplied by eps_s / eps_{s+1}; the paper
 * leaves this open).  The tail, the output and UV are those of the plain call at eps, and the
 * backward calls apply unchanged (the base is stopped; pass T = sum of T_stage, which they only
 * check).  eps_stage, T_stage: HOST arrays of n_stages entries (1 <= n_stages <= 64), read
 * before the call returns.  A schedule that increases, a last entry different from eps, a
 * negative count: SKA_EINVAL.  dustbin_score is the spoke score at eps and is rescaled like all
 * scores.  Other arguments as in sinkhorn_attn_fwd_varlen.
 */
int sinkhorn_attn_fwd_eps_schedule(const void *Q, const void *K, const void *V, const float *log_a,
                                   const float *log_b, const int *len_q, const int *len_k, void *O,
                                   float *UV, int B, int H, int L, int d, int W, int n_stages,
                                   const float *eps_stage, const int *T_stage, int R, float eps,
                                   int dustbin, float dustbin_score, int dtype, void *workspace,
                                   size_t workspace_bytes, void *stream);

/*
 * Vector-Jacobian product through the base solve: dQ, dK = (D_x z_T)^T eta for the base state
 * z_T = v^(T) reached by T full steps from v = 0 (the a-posteriori bias certificate,
 * Prop. "A Posteriori Bias Certificate": with eta = eta_R, the base cotangent that the
 * backward call returns as eta0, this is exactly the part of the full gradient that stopping
 * the base leaves out; V does not enter the base solve, so there is no dV).  Evaluated with
 * the same reverse recurrences and one-reference final sweeps as the backward call (Prop. 1,
 * Prop. 2 for a chain of depth T with no output map behind it).
 *   UV : [B,H,2(T+1),Lp] all iterates of the base solve, as sinkhorn_attn_fwd(T = 0, R = T)
 *        returns them (same kernels, so v^(T) there equals the base state of the (T, R) call).
 *   eta: [B,H,Lp] fp32, cotangent of v^(T) (raw, as eta0 is returned).
 *   dQ, dK: [B,H,L,d] out.  1 <= T <= 32.  log_a, log_b, len_q, len_k: as above, may be NULL.
 *   workspace: at least sinkhorn_attn_workspace_bytes(B, H, L, d, W, 0, T, dustbin, dtype).
 */
int sinkhorn_attn_base_vjp(const void *Q, const void *K, const float *log_a, const float *log_b,
                           const int *len_q, const int *len_k, const float *UV, const float *eta,
                           void *dQ, void *dK, int B, int H, int L, int d, int W, int T, float eps,
                           int dustbin, float dustbin_score, int dtype, void *workspace,
                           size_t workspace_bytes, void *stream);

/*
 * Certified tail-depth selection (Cor. "Certified Tail-Depth Selection"): for R = 1, 2, ...,
 * R_max run the forward and the stopped-base backward of depth R, take eta_R from it, evaluate
 * the certificate e_R = (D_x z_T)^T eta_R with sinkhorn_attn_base_vjp, and stop at the first R
 * whose largest absolute entry over (dQ, dK) parts of e_R is <= tau.  The T-step base solve runs
 * once (all its iterates are kept for the certificate) and depth R + 1 adds one tail step and an
 * output map to the iterates of depth R; per depth that leaves the depth-R backward and the
 * certificate's own T-deep vector-Jacobian product, which is most of the time (trying four depths
 * at T = 15 costs about six (T, 4) steps).  Then the gradient left in
 * dQ, dK, dV differs from full backpropagation through the same T-step base solve by at most
 * tau in every entry (the dV part of the gap is zero: V does not enter the base solve).
 *   Q, K, V, dO in; O, dQ, dK, dV out: results of the selected depth (of R_max if none passes).
 *   UV out: room for [B,H,2(R_max+1),Lp] floats; on return it holds the selected depth's
 *        [B,H,2(R+1),Lp] array, densely packed at the start.
 *   R_selected (host int): the depth chosen, 0 if no depth up to R_max passes.
 *   e_absmax (host, R_max floats): max |e_R| for every depth tried, -1 for depths not tried;
 *   eta_absmax (host, R_max floats, may be NULL): max |eta_R| likewise.
 *   1 <= T <= 32 (the 2(T+1) base iterates are kept), 1 <= R_max <= 32, tau >= 0.
 *   workspace: sinkhorn_attn_select_workspace_bytes(...) bytes, 256-byte aligned.
 * The call synchronises the stream once per depth tried (the decision is taken on the host);
 * it cannot be captured in a graph.  Depth 0 (no differentiable tail) is not a candidate:
 * the operator needs R >= 1.
 */
size_t sinkhorn_attn_select_workspace_bytes(int B, int H, int L, int d, int W, int T, int R_max,
                                            int dustbin, int dtype);
int sinkhorn_attn_select_tail_depth(const void *Q, const void *K, const void *V, const void *dO,
                                    const float *log_a, const float *log_b, const int *len_q,
                                    const int *len_k, void *O, float *UV, void *dQ, void *dK,
                                    void *dV, int B, int H, int L, int d, int W, int T, int R_max,
                                    float eps, int dustbin, float dustbin_score, int dtype,
                                    float tau, int *R_selected, float *e_absmax, float *eta_absmax,
                                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * Comparators for the final sweeps of the backward (same arguments and results as
 * sinkhorn_attn_bwd_varlen; they exist to be measured against it):
 *   SKA_BWD_ONE_REFERENCE          the production path (Prop. 2: one reference plan tile per
 *                                  edge, the other staircase factors by row/column modifiers);
 *   SKA_BWD_DIRECT                 the plain evaluation of Prop. 1: every staircase factor
 *                                  P^(t,t) and P^(t,t-1), t = R..1, is formed by an exponential
 *                                  of its own from the scores and its pair of potentials (four
 *                                  plans for R = 2; the paper's "direct four-plan" form);
 *   SKA_BWD_ONE_REFERENCE_GENERIC  Prop. 2 on the same generic kernel the direct form runs on
 *                                  (for bf16 storage with d <= 64 the production path uses a
 *                                  different, faster kernel), so that the two differ in nothing
 *                                  but how the plan factors are obtained.
 * Any other variant: SKA_EINVAL.
 */
#define SKA_BWD_ONE_REFERENCE 0
#define SKA_BWD_DIRECT 1
#define SKA_BWD_ONE_REFERENCE_GENERIC 2
int sinkhorn_attn_bwd_variant(int variant, const void *Q, const void *K, const void *V,
                              const float *log_a, const float *log_b, const int *len_q,
                              const int *len_k, const void *O, const void *dO, const float *UV,
                              void *dQ, void *dK, void *dV, float *eta0, int B, int H, int L, int d,
                              int W, int T, int R, float eps, int dustbin, float dustbin_score,
                              int dtype, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Benchmark hooks (no part of the operator).  While enabled, every forward and backward
 * call records two HIP events on its stream around each of its phases, so that a phase can
 * be timed in place, inside a larger timed region, without a profiler.  At most 4096 phase
 * spans are remembered between reads (further ones are dropped).  Level 1 leaves the schedule of
 * a call as it is (a span on two streams ends with an event on each, the later one counts);
 * level 2 joins the helper stream at the end of every phase so that phases do not overlap.
 *   sinkhorn_attn_profile_enable(level): 0 off, 1 only the SKA_PH_SCALING span of every
 *     forward call (two events per call), 2 every phase; returns SKA_OK.
 *   sinkhorn_attn_profile_read_phases(ms, launches): host arrays of SKA_PH_COUNT entries;
 *     waits for the recorded events, returns per phase the summed elapsed milliseconds and
 *     the number of sweep launches they bracket, then forgets them.
 *   sinkhorn_attn_profile_read(&ms, &launches): the same, SKA_PH_SCALING only (the run of
 *     2(T + R) - 1 identical launches of the scaling sweep of Eq. 1-2 in every forward call;
 *     one fewer in sinkhorn_attn_fwd_masked, whose first column half-step counts as SKA_PH_FIRST).
 */
/*
 * Number of streams a call spreads its band sweeps over: 2 (default; see the conventions at the
 * top) or 1.  Process-wide.  Returns SKA_OK, or SKA_EINVAL for any other number.
 */
int sinkhorn_attn_set_streams(int n);
/*
 * Fused half-steps (Sec. 2.2: the differentiable tail; App. "Algorithm Sketch": the tail line).
 * mode 0 (default): every half-step of Eq. 1-2 is a launch of its own.  mode 1: the 2R half-steps
 * of the tail run as ONE launch.  mode 2: all half-steps after the first one (base solve and
 * tail) run as one launch.  Inside such a launch the blocks of consecutive half-steps are chained
 * by per-block counters instead of kernel boundaries (a block starts half-step h when the blocks
 * within the band's reach have finished h - 1), the workgroups being co-resident (cooperative
 * launch); the arithmetic per block is that of the separate launches, so results are identical
 * bit for bit.  It trades the launch-to-launch latency and the ramp of every launch for a
 * counter hand-over between neighbouring blocks through memory that all XCDs see; on MI355X the
 * two cost about the same (measured: a half-step takes 16 us fused against 13 us in launches of
 * its own at B*H*L = 131072, 60 us against 59 us at 524288 on one stream), so the default is 0.
 *   It applies to forward calls (and the forward half of sinkhorn_attn_step) without a dustbin and
 * without a continuation schedule, outside stream capture, whose workspace has
 * sinkhorn_attn_workspace_bytes() bytes (the counters live at its end); other calls run unfused.
 * The fused launch takes all problems on the caller's stream.  At most one call with fused
 * half-steps may be in flight on a device at a time (two such launches can hold each other's
 * workgroups out).  Every wait inside the launch is bounded by spin_limit polls (0: the default,
 * 2^18, about a tenth of a second): a wait that runs out stops waiting and writes NaN into its block of the
 * potentials, which reaches every output depending on it, and the launch ends normally.
 * Process-wide.  Returns SKA_OK, or SKA_EINVAL for another mode.
 */
int sinkhorn_attn_set_fused_half_steps(int mode, unsigned spin_limit);
/*
 * The least number of band edges per dispatch (half of a call's problems times L times 2W + 1)
 * from which a call uses the helper stream; default 5e7.  0 makes every call on two or more
 * problems split (used by the tests to run small cases through both streams).  Process-wide.
 */
int sinkhorn_attn_set_split_min_edges(double edges);

/*
 * Issue-rate probe (benchmark hook, no part of the operator): runs eight register-only kernels
 * with parts of the instruction mix of one scaling-sweep tile per loop iteration -- M: four
 * dependent 32x32x16 bf16 MFMAs, E: 16 exp2, A: 16 adds, the VALU work consuming the MFMA result;
 * 0: E + A, 1: M, 2: M + E + A (the sweep's mix), 3: M + A, 4: M + E, 5: A, and the sweep's mix
 * with the exponentials computed on the plain ALUs (fract, floor, a cubic, ldexp) instead of the
 * transcendental unit: 6: all sixteen, 7: every second one --
 * with waves_per_simd (1..8) wavefronts resident on every SIMD of the current device, `tiles`
 * iterations each, and returns their elapsed milliseconds in ms8[0..7] (host array).  It shows
 * how far MFMA, transcendental and plain VALU work of different wavefronts overlap on one SIMD,
 * and whether moving exponentials off the transcendental unit would pay.  scratch: device
 * buffer of at least CUs * waves_per_simd * 256 floats.  Synchronises the stream.
 */
int sinkhorn_attn_probe_issue(float *scratch, size_t scratch_bytes, int tiles, int waves_per_simd,
                              double *ms8, void *stream);

typedef enum {
    SKA_PH_PRESCALE = 0, /* bf16 storage: copy of Q with the score scale folded in (fwd and bwd) */
    SKA_PH_FIRST = 1,    /* first row half-step of the base solve (no previous iterate:   */
                         /* running-maximum kernel); with masks also the first column one */
    SKA_PH_SCALING = 2,  /* the other 2(T + R) - 1 half-steps (Eq. 1-2)                   */
    SKA_PH_OUTPUT = 3,   /* O = P22 V (Section 2.2)                                      */
    SKA_PH_ROWDOT = 4,   /* g_u = <dO, O>                                                */
    SKA_PH_DV = 5,       /* dV = P22^T dO and vbar2 = <V, dV>                            */
    SKA_PH_MATVEC = 6,   /* reverse recurrences of Prop. 1 (2R - 1 band mat-vecs, +1 for eta0) */
    SKA_PH_FINAL = 7,    /* modifier packs and the two one-reference final sweeps (Prop. 2)  */
    SKA_PH_COUNT = 8
} ska_phase;
int sinkhorn_attn_profile_enable(int on);
int sinkhorn_attn_profile_read_phases(double *elapsed_ms, long *launches);
int sinkhorn_attn_profile_read(double *elapsed_ms, long *launches);

/* Static, human-readable text for a ska_status value. Never NULL. */
const char *sinkhorn_attn_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* SINKHORN_ATTN_H */
