/*
 * fp64 CPU oracle for banded Sinkhorn attention with a stopped base solve and
 * a depth-R differentiable tail.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke
 * check and the benchmark's cpu_baseline leg may load this library.  It shares
 * no code, header, table or helper with the HIP path.
 *
 * Everything is the definition written out: one generic fixed support
 * (a sparse set of active (row, col) pairs with one score per pair), plain
 * loops, fp64, stable logsumexp.  The banded operator, the dense operator and
 * the dustbin-augmented operator are all instances of the same support-generic
 * core, so a pin on a tiny dense or masked case exercises the code that is
 * later run on the band.
 *
 * What follows which passage of the paper:
 *   scores S = Q K^T / (eps sqrt d)                      Section 2.1
 *   row / column half-steps                              Eq. (1), Eq. (2)
 *   stopped T-step base, R-step tail                     Section 2.2
 *   transport application without renormalisation        Section 2.2 (map A)
 *   staircase plans P^(p,q)                              Section 2.2
 *   reverse pass through the tail                        Prop. 1 and its proof
 *                                                        (App. A), walked as an
 *                                                        explicit reverse sweep
 *                                                        over the 2R half-steps,
 *                                                        every factor built by
 *                                                        its own exponential
 *                                                        ("direct-four")
 *   sparse-spoke dustbin support                         Section 2.3
 *   compatible general marginals a, b (optional)         App. "Compatible General
 *                                                        Marginals": half-steps with
 *                                                        log a_i / log b_j added, and
 *                                                        the half-step Jacobians
 *                                                        -P/a_i, -P/b_j of its lemma in
 *                                                        the reverse sweep
 *
 * Readings fixed here (the paper is silent): the base solve starts from v = 0
 * and begins with a row half-step; one step = row half-step then column
 * half-step; the band is |i-j| <= W inclusive; potentials are kept ungauged.
 *
 * Parity pins: every exported function is pinned by tests that do not call it
 * to produce their own expectation (finite differences, dense brute force,
 * textbook matrix scaling, closed forms, marginal/zero-sum invariants).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int64_t m, n, nnz;
    const int64_t *rptr; /* m+1: edges of row i are rptr[i] .. rptr[i+1]-1   */
    const int32_t *col;  /* nnz: column of each edge (row-major edge order)   */
    int64_t *cptr;       /* n+1: column j owns cedge[cptr[j] .. cptr[j+1]-1]  */
    int64_t *cedge;      /* nnz: edge ids grouped by column                   */
    int32_t *erow;       /* nnz: row of each edge                             */
} support_t;

int ska_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Column-grouped view of a row-grouped edge list (counting sort). */
static int build_columns(support_t *sp)
{
    sp->cptr = (int64_t *)calloc((size_t)sp->n + 1, sizeof(int64_t));
    sp->cedge = (int64_t *)malloc((size_t)(sp->nnz ? sp->nnz : 1) * sizeof(int64_t));
    sp->erow = (int32_t *)malloc((size_t)(sp->nnz ? sp->nnz : 1) * sizeof(int32_t));
    if (!sp->cptr || !sp->cedge || !sp->erow) return -1;
    for (int64_t i = 0; i < sp->m; ++i)
        for (int64_t e = sp->rptr[i]; e < sp->rptr[i + 1]; ++e) {
            sp->erow[e] = (int32_t)i;
            sp->cptr[sp->col[e] + 1]++;
        }
    for (int64_t j = 0; j < sp->n; ++j) sp->cptr[j + 1] += sp->cptr[j];
    int64_t *fill = (int64_t *)malloc((size_t)(sp->n ? sp->n : 1) * sizeof(int64_t));
    if (!fill) return -1;
    memcpy(fill, sp->cptr, (size_t)sp->n * sizeof(int64_t));
    for (int64_t e = 0; e < sp->nnz; ++e) sp->cedge[fill[sp->col[e]]++] = e;
    free(fill);
    return 0;
}

static void free_columns(support_t *sp)
{
    free(sp->cptr);
    free(sp->cedge);
    free(sp->erow);
}

/* Eq. (1): u_i = log a_i - log sum_{j in row i} exp(S_ij + v_j)  (loga NULL: a = 1). */
static void row_half_step(const support_t *sp, const double *S, const double *v, const double *loga,
                          double *u)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < sp->m; ++i) {
        double mx = -INFINITY;
        for (int64_t e = sp->rptr[i]; e < sp->rptr[i + 1]; ++e) {
            double x = S[e] + v[sp->col[e]];
            if (x > mx) mx = x;
        }
        double s = 0.0;
        for (int64_t e = sp->rptr[i]; e < sp->rptr[i + 1]; ++e)
            s += exp(S[e] + v[sp->col[e]] - mx);
        /* a row without active edges (possible on rectangular supports) takes no part: its
           potential is reported as 0 and multiplies nothing */
        u[i] = sp->rptr[i] == sp->rptr[i + 1] ? 0.0 : (loga ? loga[i] : 0.0) - (mx + log(s));
    }
}

/* Eq. (2): v_j = log b_j - log sum_{i in column j} exp(S_ij + u_i)  (logb NULL: b = 1). */
static void col_half_step(const support_t *sp, const double *S, const double *u, const double *logb,
                          double *v)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < sp->n; ++j) {
        double mx = -INFINITY;
        for (int64_t c = sp->cptr[j]; c < sp->cptr[j + 1]; ++c) {
            int64_t e = sp->cedge[c];
            double x = S[e] + u[sp->erow[e]];
            if (x > mx) mx = x;
        }
        double s = 0.0;
        for (int64_t c = sp->cptr[j]; c < sp->cptr[j + 1]; ++c) {
            int64_t e = sp->cedge[c];
            s += exp(S[e] + u[sp->erow[e]] - mx);
        }
        v[j] = sp->cptr[j] == sp->cptr[j + 1] ? 0.0 : (logb ? logb[j] : 0.0) - (mx + log(s));
    }
}

/* Staircase factor P^(p,q)_e = exp(S_e + u^(p)_i + v^(q)_j), built by its own exp. */
static void form_plan(const support_t *sp, const double *S, const double *up, const double *vq,
                      double *P)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < sp->m; ++i)
        for (int64_t e = sp->rptr[i]; e < sp->rptr[i + 1]; ++e)
            P[e] = exp(S[e] + up[i] + vq[sp->col[e]]);
}

/*
 * Support-generic core.
 *
 *   S[nnz]           effective scores on the active edges
 *   Vv[n][dv]        values; G[m][dv] output cotangent (G may be NULL: forward only)
 *   v0_fixed         NULL: run the T-step base solve from v = 0.
 *                    else: use this vector as the stopped v^(0) and skip the
 *                    base solve (T is ignored, U[0] is filled with zeros).
 *   loga[m], logb[n] logarithms of the row / column targets, NULL for unit targets
 * Outputs (any may be NULL except U, Vp):
 *   O[m][dv]         transport output with the terminal plan P^(R,R)
 *   U[(R+1)][m], Vp[(R+1)][n]   u^(0..R), v^(0..R)
 *   Sbar[nnz]        score cotangent, Eq. (6)
 *   dV[n][dv]
 *   ubar[(R+1)][m], vbar[(R+1)][n]  dual cotangents; ubar[0] = 0, vbar[0] is the
 *                    discarded base cotangent
 */
int ska_oracle_core_marg(int64_t m, int64_t n, int64_t nnz, const int64_t *rptr, const int32_t *col,
                         const double *S, const double *Vv, const double *G, int dv, int T, int R,
                         const double *v0_fixed, const double *loga, const double *logb, double *O,
                         double *U, double *Vp, double *Sbar, double *dV, double *ubar, double *vbar)
{
    if (m < 1 || n < 1 || R < 1 || T < 0 || dv < 1 || !rptr || !col || !S || !U || !Vp) return -1;
    support_t sp = {m, n, nnz, rptr, col, NULL, NULL, NULL};
    if (build_columns(&sp)) { free_columns(&sp); return -2; }

    double *u0 = U, *v0 = Vp;
    if (v0_fixed) {
        memcpy(v0, v0_fixed, (size_t)n * sizeof(double));
        memset(u0, 0, (size_t)m * sizeof(double));
    } else {
        memset(v0, 0, (size_t)n * sizeof(double));
        memset(u0, 0, (size_t)m * sizeof(double));
        for (int t = 0; t < T; ++t) {
            row_half_step(&sp, S, v0, loga, u0);
            col_half_step(&sp, S, u0, logb, v0);
        }
    }
    /* tail: u^(t) from v^(t-1), then v^(t) from u^(t) */
    for (int t = 1; t <= R; ++t) {
        row_half_step(&sp, S, Vp + (size_t)(t - 1) * n, loga, U + (size_t)t * m);
        col_half_step(&sp, S, U + (size_t)t * m, logb, Vp + (size_t)t * n);
    }
    const double *uR = U + (size_t)R * m, *vR = Vp + (size_t)R * n;

    double *P = (double *)malloc((size_t)(nnz ? nnz : 1) * sizeof(double));
    if (!P) { free_columns(&sp); return -2; }
    form_plan(&sp, S, uR, vR, P);

    if (O) {
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < m; ++i) {
            double *o = O + (size_t)i * dv;
            for (int k = 0; k < dv; ++k) o[k] = 0.0;
            for (int64_t e = rptr[i]; e < rptr[i + 1]; ++e) {
                const double *vj = Vv + (size_t)col[e] * dv;
                for (int k = 0; k < dv; ++k) o[k] += P[e] * vj[k];
            }
        }
    }
    if (!G) { free(P); free_columns(&sp); return 0; }
    if (!Sbar || !ubar || !vbar) { free(P); free_columns(&sp); return -1; }

    /* ---- reverse sweep, newest operation first ---- */
    memset(ubar, 0, (size_t)(R + 1) * m * sizeof(double));
    memset(vbar, 0, (size_t)(R + 1) * n * sizeof(double));
    double *ubR = ubar + (size_t)R * m, *vbR = vbar + (size_t)R * n;

    /* transport application O_i = sum_j P_ij V_j with P = exp(S + u^R + v^R):
       Pbar_e = <G_i, V_j> =: Z_e, which flows to S_e, u^R_i and v^R_j alike. */
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        const double *gi = G + (size_t)i * dv;
        double acc = 0.0;
        for (int64_t e = rptr[i]; e < rptr[i + 1]; ++e) {
            const double *vj = Vv + (size_t)col[e] * dv;
            double z = 0.0;
            for (int k = 0; k < dv; ++k) z += gi[k] * vj[k];
            Sbar[e] = P[e] * z;
            acc += Sbar[e];
        }
        ubR[i] = acc;
    }
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; ++j) {
        double acc = 0.0;
        for (int64_t c = sp.cptr[j]; c < sp.cptr[j + 1]; ++c) acc += Sbar[sp.cedge[c]];
        vbR[j] = acc;
        if (dV) {
            double *d = dV + (size_t)j * dv;
            for (int k = 0; k < dv; ++k) d[k] = 0.0;
            for (int64_t c = sp.cptr[j]; c < sp.cptr[j + 1]; ++c) {
                int64_t e = sp.cedge[c];
                const double *gi = G + (size_t)sp.erow[e] * dv;
                for (int k = 0; k < dv; ++k) d[k] += P[e] * gi[k];
            }
        }
    }

    for (int t = R; t >= 1; --t) {
        const double *ut = U + (size_t)t * m;
        double *ubt = ubar + (size_t)t * m;
        double *vbt = vbar + (size_t)t * n;
        double *vbp = vbar + (size_t)(t - 1) * n;

        /* v^(t)_j = log b_j - log sum_i exp(S_ij + u^(t)_i): the weight of edge e in it
           is P^(t,t)_e / b_j (the column sums of P^(t,t) are b), with a minus sign. */
        form_plan(&sp, S, ut, Vp + (size_t)t * n, P);
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < m; ++i) {
            double acc = 0.0;
            for (int64_t e = rptr[i]; e < rptr[i + 1]; ++e) {
                double w = P[e] * vbt[col[e]] * (logb ? exp(-logb[col[e]]) : 1.0);
                Sbar[e] -= w;
                acc += w;
            }
            ubt[i] -= acc;
        }

        /* u^(t)_i = log a_i - log sum_j exp(S_ij + v^(t-1)_j): weight P^(t,t-1)_e / a_i
           (the row sums of P^(t,t-1) are a), minus sign. */
        form_plan(&sp, S, ut, Vp + (size_t)(t - 1) * n, P);
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < m; ++i) {
            const double ia = loga ? exp(-loga[i]) : 1.0;
            for (int64_t e = rptr[i]; e < rptr[i + 1]; ++e) Sbar[e] -= P[e] * ubt[i] * ia;
        }
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            double acc = 0.0;
            for (int64_t c = sp.cptr[j]; c < sp.cptr[j + 1]; ++c) {
                int64_t e = sp.cedge[c];
                acc += P[e] * ubt[sp.erow[e]] * (loga ? exp(-loga[sp.erow[e]]) : 1.0);
            }
            vbp[j] -= acc;
        }
    }
    free(P);
    free_columns(&sp);
    return 0;
}

/* Unit targets (the main text's balanced problem). */
int ska_oracle_core(int64_t m, int64_t n, int64_t nnz, const int64_t *rptr, const int32_t *col,
                    const double *S, const double *Vv, const double *G, int dv, int T, int R,
                    const double *v0_fixed, double *O, double *U, double *Vp, double *Sbar,
                    double *dV, double *ubar, double *vbar)
{
    return ska_oracle_core_marg(m, n, nnz, rptr, col, S, Vv, G, dv, T, R, v0_fixed, NULL, NULL, O, U,
                                Vp, Sbar, dV, ubar, vbar);
}

/*
 * Banded operator on Q, K, V in R^{L x d} (one problem), optional sparse-spoke
 * dustbin.  Builds the support and the scores, calls the core, and pushes the
 * score cotangent to Q and K.
 *
 * Support without dustbin: {(i,j): |i-j| <= W}.  With dustbin: one extra row
 * d_q = L and one extra column d_k = L; extra edges (i, d_k) for every i,
 * (d_q, j) for every j, and (d_q, d_k); all of them carry the scalar score
 * s_db.  V_{d_k} = 0; G_{d_q} = 0; all L+1 row and column targets are one.
 *
 *   Lp = L + (dustbin ? 1 : 0)
 *   O[L][d], dQ[L][d], dK[L][d], dV[L][d]
 *   UV[2(R+1)][Lp] ordered u^(0), v^(0), u^(1), v^(1), ..., u^(R), v^(R)
 *   bars[2(R+1)][Lp] same order for the dual cotangents (may be NULL)
 *   Sbar_band[L][2W+1] (may be NULL): Sbar_band[i][j-i+W] on band edges, 0 elsewhere
 *   v0_fixed[Lp] or NULL, as in the core
 *   loga[Lp], logb[Lp] or NULL: logarithms of the row / column targets
 * G may be NULL (forward only; the cotangent outputs are then untouched).
 */
int ska_oracle_band_marg(const double *Q, const double *K, const double *V, const double *G, int64_t L,
                         int d, int64_t W, int T, int R, double eps, int dustbin, double s_db,
                         const double *v0_fixed, const double *loga, const double *logb, double *O,
                         double *UV, double *dQ, double *dK, double *dV, double *bars,
                         double *Sbar_band)
{
    if (L < 1 || d < 1 || W < 0 || R < 1 || T < 0 || !(eps > 0.0) || !Q || !K || !V || !UV)
        return -1;
    const int64_t Lp = L + (dustbin ? 1 : 0);
    const double cs = 1.0 / (eps * sqrt((double)d));

    int64_t *rptr = (int64_t *)malloc((size_t)(Lp + 1) * sizeof(int64_t));
    if (!rptr) return -2;
    rptr[0] = 0;
    for (int64_t i = 0; i < L; ++i) {
        int64_t lo = i - W < 0 ? 0 : i - W, hi = i + W > L - 1 ? L - 1 : i + W;
        rptr[i + 1] = rptr[i] + (hi - lo + 1) + (dustbin ? 1 : 0);
    }
    if (dustbin) rptr[L + 1] = rptr[L] + L + 1;
    const int64_t nnz = rptr[Lp];
    int32_t *col = (int32_t *)malloc((size_t)nnz * sizeof(int32_t));
    double *S = (double *)malloc((size_t)nnz * sizeof(double));
    double *Sbar = G ? (double *)malloc((size_t)nnz * sizeof(double)) : NULL;
    double *Vaug = (double *)calloc((size_t)Lp * d, sizeof(double));
    double *Gaug = G ? (double *)calloc((size_t)Lp * d, sizeof(double)) : NULL;
    double *Oaug = (double *)malloc((size_t)Lp * d * sizeof(double));
    double *dVaug = G ? (double *)malloc((size_t)Lp * d * sizeof(double)) : NULL;
    double *U = (double *)malloc((size_t)(R + 1) * Lp * sizeof(double));
    double *Vp = (double *)malloc((size_t)(R + 1) * Lp * sizeof(double));
    double *ub = G ? (double *)malloc((size_t)(R + 1) * Lp * sizeof(double)) : NULL;
    double *vb = G ? (double *)malloc((size_t)(R + 1) * Lp * sizeof(double)) : NULL;
    int rc = -2;
    if (!col || !S || !Vaug || !Oaug || !U || !Vp || (G && (!Sbar || !Gaug || !dVaug || !ub || !vb)))
        goto done;

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < L; ++i) {
        int64_t lo = i - W < 0 ? 0 : i - W, hi = i + W > L - 1 ? L - 1 : i + W;
        int64_t e = rptr[i];
        for (int64_t j = lo; j <= hi; ++j, ++e) {
            double dot = 0.0;
            for (int k = 0; k < d; ++k) dot += Q[(size_t)i * d + k] * K[(size_t)j * d + k];
            col[e] = (int32_t)j;
            S[e] = dot * cs;
        }
        if (dustbin) { col[e] = (int32_t)L; S[e] = s_db; }
    }
    if (dustbin)
        for (int64_t j = 0; j <= L; ++j) { col[rptr[L] + j] = (int32_t)j; S[rptr[L] + j] = s_db; }
    memcpy(Vaug, V, (size_t)L * d * sizeof(double));
    if (G) memcpy(Gaug, G, (size_t)L * d * sizeof(double));

    rc = ska_oracle_core_marg(Lp, Lp, nnz, rptr, col, S, Vaug, G ? Gaug : NULL, d, T, R, v0_fixed, loga,
                              logb, Oaug, U, Vp, Sbar, dVaug, ub, vb);
    if (rc) goto done;

    if (O) memcpy(O, Oaug, (size_t)L * d * sizeof(double));
    for (int t = 0; t <= R; ++t) {
        memcpy(UV + (size_t)(2 * t) * Lp, U + (size_t)t * Lp, (size_t)Lp * sizeof(double));
        memcpy(UV + (size_t)(2 * t + 1) * Lp, Vp + (size_t)t * Lp, (size_t)Lp * sizeof(double));
    }
    if (G) {
        if (dV) memcpy(dV, dVaug, (size_t)L * d * sizeof(double));
        if (bars)
            for (int t = 0; t <= R; ++t) {
                memcpy(bars + (size_t)(2 * t) * Lp, ub + (size_t)t * Lp, (size_t)Lp * sizeof(double));
                memcpy(bars + (size_t)(2 * t + 1) * Lp, vb + (size_t)t * Lp,
                       (size_t)Lp * sizeof(double));
            }
        /* S_ij = cs * <Q_i, K_j>  =>  dQ_i = cs sum_j Sbar_ij K_j, dK_j = cs sum_i Sbar_ij Q_i.
           Spoke scores are the constant s_db and carry nothing back to Q or K. */
        if (dQ) memset(dQ, 0, (size_t)L * d * sizeof(double));
        if (dK) memset(dK, 0, (size_t)L * d * sizeof(double));
        if (Sbar_band) memset(Sbar_band, 0, (size_t)L * (2 * W + 1) * sizeof(double));
        if (dQ) {
#pragma omp parallel for schedule(static)
            for (int64_t i = 0; i < L; ++i)
                for (int64_t e = rptr[i]; e < rptr[i + 1]; ++e) {
                    int64_t j = col[e];
                    if (j >= L) continue;
                    for (int k = 0; k < d; ++k)
                        dQ[(size_t)i * d + k] += cs * Sbar[e] * K[(size_t)j * d + k];
                }
        }
        if (dK || Sbar_band) {
            support_t sp = {Lp, Lp, nnz, rptr, col, NULL, NULL, NULL};
            if (build_columns(&sp)) { free_columns(&sp); rc = -2; goto done; }
#pragma omp parallel for schedule(static)
            for (int64_t j = 0; j < L; ++j)
                for (int64_t c = sp.cptr[j]; c < sp.cptr[j + 1]; ++c) {
                    int64_t e = sp.cedge[c], i = sp.erow[e];
                    if (i >= L) continue;
                    if (dK)
                        for (int k = 0; k < d; ++k)
                            dK[(size_t)j * d + k] += cs * Sbar[e] * Q[(size_t)i * d + k];
                    if (Sbar_band) Sbar_band[(size_t)i * (2 * W + 1) + (j - i + W)] = Sbar[e];
                }
            free_columns(&sp);
        }
    }
done:
    free(rptr); free(col); free(S); free(Sbar); free(Vaug); free(Gaug); free(Oaug); free(dVaug);
    free(U); free(Vp); free(ub); free(vb);
    return rc;
}

/* Unit targets. */
int ska_oracle_band(const double *Q, const double *K, const double *V, const double *G, int64_t L,
                    int d, int64_t W, int T, int R, double eps, int dustbin, double s_db,
                    const double *v0_fixed, double *O, double *UV, double *dQ, double *dK,
                    double *dV, double *bars, double *Sbar_band)
{
    return ska_oracle_band_marg(Q, K, V, G, L, d, W, T, R, eps, dustbin, s_db, v0_fixed, NULL, NULL, O,
                                UV, dQ, dK, dV, bars, Sbar_band);
}
