"""Pins for the fp64 CPU oracle: each test fixes the oracle against something
that is not the oracle (finite differences, dense brute force with a library
logsumexp, textbook matrix scaling, closed forms, conservation identities, the
paper's printed ledger numbers).  CPU only.
"""
import json
import os

import numpy as np
import pytest

import oracle
from paper_2605_08123_amd.workloads import CONFIGS, Workload
from tests import dense_ref as dr

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rel(a, b):
    return np.linalg.norm(np.asarray(a) - np.asarray(b)) / max(np.linalg.norm(b), 1e-300)


def problem(L=24, d=4, seed=0, scale=1.0):
    rng = np.random.default_rng(seed)
    return tuple(scale * rng.standard_normal((L, d)) for _ in range(4))


CASE = dict(W=5, T=6, R=2, eps=0.7)


# ---------------------------------------------------------------- I1: finite differences
def _loss(Q, K, V, G, v0, **kw):
    return float((G * oracle.band(Q, K, V, None, v0_fixed=v0, **kw)["O"]).sum())


@pytest.mark.parametrize("R", [1, 2, 3])
@pytest.mark.parametrize("dustbin", [False, True])
def test_fd_gradients_with_frozen_base(R, dustbin):
    """Central differences of <G, O> with v^(0) held fixed (the stop-gradient of
    Section 2.2) reproduce dQ, dK, dV."""
    Q, K, V, G = problem()
    kw = dict(W=5, T=6, R=R, eps=0.7, dustbin=dustbin, dustbin_score=0.3)
    ref = oracle.band(Q, K, V, G, **kw)
    v0 = ref["UV"][1].copy()
    h = 1e-6
    for name, idx in (("dQ", 0), ("dK", 1), ("dV", 2)):
        fd = np.zeros_like(Q)
        for a in range(Q.shape[0]):
            for b in range(Q.shape[1]):
                args = [Q.copy(), K.copy(), V.copy()]
                args[idx][a, b] += h
                fp = _loss(*args, G, v0, **kw)
                args[idx][a, b] -= 2 * h
                fm = _loss(*args, G, v0, **kw)
                fd[a, b] = (fp - fm) / (2 * h)
        assert rel(ref[name], fd) < 2e-7, (name, rel(ref[name], fd))


def test_fd_through_unfrozen_base_differs():
    """Differentiating through the base solve as well gives a different gradient:
    the gap is the surrogate bias of Thm. 1, so the stop is really implemented."""
    Q, K, V, G = problem()
    kw = dict(**CASE)
    ref = oracle.band(Q, K, V, G, **kw)
    h = 1e-6
    fd = np.zeros_like(Q)
    for a in range(Q.shape[0]):
        for b in range(Q.shape[1]):
            Qp, Qm = Q.copy(), Q.copy()
            Qp[a, b] += h
            Qm[a, b] -= h
            fd[a, b] = (_loss(Qp, K, V, G, None, **kw) - _loss(Qm, K, V, G, None, **kw)) / (2 * h)
    assert rel(ref["dQ"], fd) > 1e-3


def test_full_backprop_is_the_tail_without_a_base():
    """With T = 0 nothing is stopped: the surrogate with tail depth T' + R' is the whole
    (T' + R')-step solve, so its gradient is the full gradient that central differences
    through the unfrozen solve measure.  The gap to the stopped-base gradient is the bias
    D_x z_T^T eta_R of the a-posteriori certificate; it shrinks as the tail deepens."""
    Q, K, V, G = problem()
    T, W, eps = 6, 5, 0.7
    h = 1e-6
    gaps = []
    for R in (1, 2, 3):
        kw = dict(W=W, T=T, R=R, eps=eps)
        full = oracle.band(Q, K, V, G, W=W, T=0, R=T + R, eps=eps)
        assert np.allclose(full["O"], oracle.band(Q, K, V, None, **kw)["O"], rtol=0, atol=1e-13)
        if R == 2:
            fd = np.zeros_like(K)
            for a in range(K.shape[0]):
                for b in range(K.shape[1]):
                    Kp, Km = K.copy(), K.copy()
                    Kp[a, b] += h
                    Km[a, b] -= h
                    fd[a, b] = (_loss(Q, Kp, V, G, None, **kw) - _loss(Q, Km, V, G, None, **kw)) / (2 * h)
            assert rel(full["dK"], fd) < 2e-7, rel(full["dK"], fd)
        stopped = oracle.band(Q, K, V, G, **kw)
        gaps.append(np.abs(full["dQ"] - stopped["dQ"]).max())
    assert gaps[0] > gaps[1] > gaps[2] > 0.0


# ---------------------------------------------------------------- P12: dense brute force
@pytest.mark.parametrize("L,W", [(24, 5), (17, 0), (9, 8), (9, 20), (33, 1)])
def test_band_matches_dense_brute_force(L, W):
    Q, K, V, G = problem(L=L, seed=L + W)
    T, R, eps = 4, 2, 0.9
    out = oracle.band(Q, K, V, G, W=W, T=T, R=R, eps=eps, want_sbar=True)
    mask = dr.band_mask(L, W)
    S = dr.scores(Q, K, eps)
    U, Vp = dr.half_steps(S, mask, T, R)
    for t in range(R + 1):
        if t == 0 and T == 0:
            continue
        # gauge-free comparison: u^(p)_i + v^(q)_j
        np.testing.assert_allclose(out["UV"][2 * t][:, None] + out["UV"][2 * t + 1][None, :],
                                   U[t][:, None] + Vp[t][None, :], atol=1e-12)
    cf = dr.closed_form_adjoint(S, mask, U, Vp, V, G)
    cs = 1.0 / (eps * np.sqrt(Q.shape[1]))
    assert rel(out["O"], cf["O"]) < 1e-13
    assert rel(out["dV"], cf["dV"]) < 1e-13
    assert rel(out["dQ"], cs * cf["Sbar"] @ K) < 1e-12
    assert rel(out["dK"], cs * cf["Sbar"].T @ Q) < 1e-12
    # score cotangent entry by entry, and nothing outside the band
    for i in range(L):
        for o in range(2 * W + 1):
            j = i + o - W
            want = cf["Sbar"][i, j] if 0 <= j < L else 0.0
            assert abs(out["Sbar"][i, o] - want) < 1e-13
    for t in range(1, R + 1):
        np.testing.assert_allclose(out["bars"][2 * t], cf["ubar"][t], atol=1e-13)
        np.testing.assert_allclose(out["bars"][2 * t + 1], cf["vbar"][t], atol=1e-13)
    np.testing.assert_allclose(out["bars"][1], cf["vbar"][0], atol=1e-13)


def test_negative_controls_are_detected():
    """Dropping the pull-back of the terminal v^(R) (App. A, proof of Prop. 1) or
    using beta where delta belongs must move the result far outside tolerance."""
    L = 24
    Q, K, V, G = problem(L=L)
    out = oracle.band(Q, K, V, G, want_sbar=True, **CASE)
    mask, S = dr.band_mask(L, CASE["W"]), dr.scores(Q, K, CASE["eps"])
    U, Vp = dr.half_steps(S, mask, CASE["T"], CASE["R"])
    good = dr.closed_form_adjoint(S, mask, U, Vp, V, G)
    bad = dr.closed_form_adjoint(S, mask, U, Vp, V, G, drop_terminal_pullback=True)
    cs = 1.0 / (CASE["eps"] * 2.0)
    assert rel(out["dQ"], cs * good["Sbar"] @ K) < 1e-12
    assert rel(out["dQ"], cs * bad["Sbar"] @ K) > 1e-2
    wrong = dr.one_reference_sbar(S, mask, U, Vp, V, G, good["ubar"], good["vbar"], delta_from=1)
    assert rel(wrong, good["Sbar"]) > 1e-3


# ---------------------------------------------------------------- I2: orbit identity / Prop. 2
def test_one_reference_formula_equals_direct_four():
    L = 24
    Q, K, V, G = problem(L=L, seed=3)
    out = oracle.band(Q, K, V, G, want_sbar=True, **CASE)
    mask, S = dr.band_mask(L, CASE["W"]), dr.scores(Q, K, CASE["eps"])
    UV, bars = out["UV"], out["bars"]
    U, Vp = UV[0::2], UV[1::2]
    one_ref = dr.one_reference_sbar(S, mask, U, Vp, V, G, bars[0::2], bars[1::2])
    dense = np.zeros((L, L))
    for i in range(L):
        for o in range(2 * CASE["W"] + 1):
            j = i + o - CASE["W"]
            if 0 <= j < L:
                dense[i, j] = out["Sbar"][i, o]
    assert np.abs(one_ref - dense).max() < 1e-13
    # every staircase factor is the reference plan rescaled by diagonal vectors
    P22 = dr.plan(S, mask, U[2], Vp[2])
    for p, q in ((2, 1), (1, 1), (1, 0)):
        direct = dr.plan(S, mask, U[p], Vp[q])
        orbit = P22 * np.exp(U[p] - U[2])[:, None] * np.exp(Vp[q] - Vp[2])[None, :]
        assert np.abs(direct - orbit).max() < 1e-13


# ---------------------------------------------------------------- I3/I4/I5: conservation
@pytest.mark.parametrize("dustbin", [False, True])
def test_marginals_and_zero_sum_identities(dustbin):
    L, W = 40, 6
    Q, K, V, G = problem(L=L, seed=5)
    kw = dict(W=W, T=7, R=2, eps=0.8, dustbin=dustbin, dustbin_score=-0.2)
    out = oracle.band(Q, K, V, G, want_sbar=True, **kw)
    Lp = L + int(dustbin)
    mask = np.zeros((Lp, Lp), bool)
    mask[:L, :L] = dr.band_mask(L, W)
    S = np.zeros((Lp, Lp))
    S[:L, :L] = dr.scores(Q, K, kw["eps"])
    if dustbin:
        mask[L, :] = mask[:, L] = True
        S[L, :] = S[:, L] = kw["dustbin_score"]
    U, Vp = out["UV"][0::2], out["UV"][1::2]
    ub, vb = out["bars"][0::2], out["bars"][1::2]
    for t in (1, 2):
        assert np.abs(dr.plan(S, mask, U[t], Vp[t]).sum(0) - 1).max() < 1e-13      # columns
        assert np.abs(dr.plan(S, mask, U[t], Vp[t - 1]).sum(1) - 1).max() < 1e-13  # rows
    # row marginal of the terminal plan is only approximately one at finite T
    assert 1e-8 < np.abs(dr.plan(S, mask, U[2], Vp[2]).sum(1) - 1).max() < 0.5
    for vec in (ub[2], vb[1], ub[1], vb[0]):
        assert abs(vec.sum()) < 1e-13
    Va = np.vstack([V, np.zeros((Lp - L, V.shape[1]))])
    Ga = np.vstack([G, np.zeros((Lp - L, G.shape[1]))])
    P22 = dr.plan(S, mask, U[2], Vp[2])
    gu = ub[2] + P22 @ vb[2]
    np.testing.assert_allclose(gu[:L], (G * out["O"]).sum(1), atol=1e-13)
    np.testing.assert_allclose(vb[2][:L], (V * out["dV"]).sum(1), atol=1e-13)
    assert abs(gu.sum() - vb[2].sum()) < 1e-12
    if not dustbin:
        assert np.abs(out["Sbar"].sum(1)).max() < 1e-13
        assert np.abs(out["dK"].sum(0)).max() < 1e-12
        # column sums of Sbar equal the discarded base cotangent
        colsum = np.zeros(L)
        for i in range(L):
            for o in range(2 * W + 1):
                j = i + o - W
                if 0 <= j < L:
                    colsum[j] += out["Sbar"][i, o]
        np.testing.assert_allclose(colsum, vb[0], atol=1e-13)
    assert Va.shape == Ga.shape


# ---------------------------------------------------------------- I6: K-shift, gauge
def test_shift_of_all_keys_leaves_output_unchanged():
    Q, K, V, G = problem(seed=7)
    a = oracle.band(Q, K, V, G, **CASE)
    shift = np.random.default_rng(1).standard_normal(K.shape[1])
    b = oracle.band(Q, K + shift[None, :], V, G, **CASE)
    assert rel(b["O"], a["O"]) < 1e-13
    assert rel(b["dV"], a["dV"]) < 1e-13
    assert rel(b["dK"], a["dK"]) < 1e-11


def test_gauge_equivariance_of_the_tail():
    """Lemma (gauge equivariance): v^(0) + c gives u^(t) - c, v^(t) + c; O and all
    gradients are unchanged."""
    Q, K, V, G = problem(seed=8)
    a = oracle.band(Q, K, V, G, **CASE)
    c = 1.7
    b = oracle.band(Q, K, V, G, v0_fixed=a["UV"][1] + c, **CASE)
    for t in (1, 2):
        np.testing.assert_allclose(b["UV"][2 * t], a["UV"][2 * t] - c, atol=1e-12)
        np.testing.assert_allclose(b["UV"][2 * t + 1], a["UV"][2 * t + 1] + c, atol=1e-12)
    for k in ("O", "dQ", "dK", "dV"):
        assert rel(b[k], a[k]) < 1e-12


# ---------------------------------------------------------------- P7/P8/P9: special cases
@pytest.mark.parametrize("T,R", [(0, 1), (3, 2), (5, 4)])
def test_zero_bandwidth_is_identity(T, R):
    Q, K, V, G = problem(L=13, seed=9)
    out = oracle.band(Q, K, V, G, W=0, T=T, R=R, eps=0.5)
    np.testing.assert_allclose(out["O"], V, atol=1e-13)
    np.testing.assert_allclose(out["dV"], G, atol=1e-13)
    assert np.abs(out["dQ"]).max() < 1e-13 and np.abs(out["dK"]).max() < 1e-13


# ---------------------------------------------------------------- compatible general marginals
def _marginals(L, seed):
    rng = np.random.default_rng(seed)
    a, b = rng.uniform(0.4, 1.8, L), rng.uniform(0.4, 1.8, L)
    return a, b * a.sum() / b.sum()


@pytest.mark.parametrize("R", [1, 2])
def test_marginals_fd_gradients_with_frozen_base(R):
    """Row targets a and column targets b (App. "Compatible General Marginals"): central
    differences of <G, O> with v^(0) frozen reproduce dQ, dK, dV."""
    Q, K, V, G = problem(L=20, seed=21)
    a, b = _marginals(20, 22)
    kw = dict(W=4, T=5, R=R, eps=0.8, log_a=np.log(a), log_b=np.log(b))
    ref = oracle.band(Q, K, V, G, **kw)
    v0 = ref["UV"][1].copy()
    h = 1e-6
    for name, idx in (("dQ", 0), ("dK", 1), ("dV", 2)):
        fd = np.zeros_like(Q)
        for i in range(Q.shape[0]):
            for k in range(Q.shape[1]):
                args = [Q.copy(), K.copy(), V.copy()]
                args[idx][i, k] += h
                fp = _loss(*args, G, v0, **kw)
                args[idx][i, k] -= 2 * h
                fm = _loss(*args, G, v0, **kw)
                fd[i, k] = (fp - fm) / (2 * h)
        assert rel(ref[name], fd) < 2e-7, (name, rel(ref[name], fd))


def test_marginals_match_dense_brute_force_and_targets():
    """Dense library logsumexp with log a / log b added, the closed-form general-marginal
    adjoint, and the target sums: rows of P^(t,t-1) sum to a, columns of P^(t,t) to b."""
    L, W, T, R, eps = 22, 6, 5, 2, 0.9
    Q, K, V, G = problem(L=L, seed=23)
    a, b = _marginals(L, 24)
    out = oracle.band(Q, K, V, G, W=W, T=T, R=R, eps=eps, want_sbar=True, log_a=np.log(a), log_b=np.log(b))
    mask = dr.band_mask(L, W)
    S = dr.scores(Q, K, eps)
    U, Vp = dr.half_steps(S, mask, T, R, a=a, b=b)
    for t in range(R + 1):
        np.testing.assert_allclose(out["UV"][2 * t][:, None] + out["UV"][2 * t + 1][None, :],
                                   U[t][:, None] + Vp[t][None, :], atol=1e-12)
    for t in range(1, R + 1):
        np.testing.assert_allclose(dr.plan(S, mask, out["UV"][2 * t], out["UV"][2 * t + 1]).sum(0), b, rtol=1e-13)
        np.testing.assert_allclose(dr.plan(S, mask, out["UV"][2 * t], out["UV"][2 * t - 1]).sum(1), a, rtol=1e-13)
    cf = dr.closed_form_adjoint(S, mask, U, Vp, V, G, a=a, b=b)
    cs = 1.0 / (eps * np.sqrt(Q.shape[1]))
    assert rel(out["O"], cf["O"]) < 1e-13 and rel(out["dV"], cf["dV"]) < 1e-13
    assert rel(out["dQ"], cs * cf["Sbar"] @ K) < 1e-12 and rel(out["dK"], cs * cf["Sbar"].T @ Q) < 1e-12
    for t in range(1, R + 1):
        np.testing.assert_allclose(out["bars"][2 * t], cf["ubar"][t], atol=1e-13)
        np.testing.assert_allclose(out["bars"][2 * t + 1], cf["vbar"][t], atol=1e-13)
    # unit targets passed explicitly are the balanced problem
    one = oracle.band(Q, K, V, G, W=W, T=T, R=R, eps=eps, log_a=np.zeros(L), log_b=np.zeros(L))
    bal = oracle.band(Q, K, V, G, W=W, T=T, R=R, eps=eps)
    assert all(np.array_equal(one[k], bal[k]) for k in ("O", "dQ", "dK", "dV"))


def test_marginals_dense_support_is_textbook_matrix_scaling():
    L, T, R, eps = 10, 7, 2, 1.1
    Q, K, V, _ = problem(L=L, seed=25)
    a, b = _marginals(L, 26)
    out = oracle.band(Q, K, V, None, W=L - 1, T=T, R=R, eps=eps, log_a=np.log(a), log_b=np.log(b))
    M = np.exp(Q @ K.T / (eps * np.sqrt(Q.shape[1])))
    y = np.ones(L)
    for _ in range(T + R):
        x = a / (M @ y)
        y = b / (M.T @ x)
    np.testing.assert_allclose(np.exp(out["UV"][2 * R]), x, rtol=1e-12)
    np.testing.assert_allclose(np.exp(out["UV"][2 * R + 1]), y, rtol=1e-12)
    np.testing.assert_allclose(out["O"], (x[:, None] * M * y[None, :]) @ V, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- rectangular band
@pytest.mark.parametrize("Lq,Lk,W", [(19, 26, 7), (30, 21, 9), (12, 12, 3), (25, 14, 5)])
def test_rectangular_band_matches_dense_brute_force(Lq, Lk, W):
    """Sequences of different lengths: |i - j| <= W on an Lq x Lk rectangle.  Dense library
    logsumexp with a boolean mask and the closed-form adjoint, entry by entry on dQ, dK, dV;
    the square case is the banded operator.  (25, 14, 5) leaves rows 19..24 without any edge.)"""
    rng = np.random.default_rng(Lq * 100 + Lk)
    Q, G = rng.standard_normal((Lq, 4)), rng.standard_normal((Lq, 4))
    K, V = rng.standard_normal((Lk, 4)), rng.standard_normal((Lk, 4))
    T, R, eps = 4, 2, 0.9
    out = oracle.band_rect(Q, K, V, G, W, T, R, eps)
    mask = np.abs(np.arange(Lq)[:, None] - np.arange(Lk)[None, :]) <= W
    S = dr.scores(Q, K, eps)
    live = mask.any(1)
    with np.errstate(invalid="ignore", divide="ignore"):
        U, Vp = dr.half_steps(S[live], mask[live], T, R)      # rows without edges take no part
        cf = dr.closed_form_adjoint(S[live], mask[live], U, Vp, V, G[live])
    cs = 1.0 / (eps * np.sqrt(4))
    assert rel(out["O"][live], cf["O"]) < 1e-13 and np.all(out["O"][~live] == 0.0)
    assert rel(out["dV"], cf["dV"]) < 1e-13
    assert rel(out["dQ"][live], cs * cf["Sbar"] @ K) < 1e-12 and np.all(out["dQ"][~live] == 0.0)
    assert rel(out["dK"], cs * cf["Sbar"].T @ Q[live]) < 1e-12
    if Lq == Lk:
        sq = oracle.band(Q, K, V, G, W, T, R, eps)
        assert all(rel(out[k], sq[k]) < 1e-14 for k in ("O", "dQ", "dK", "dV"))


# ---------------------------------------------------------------- inactive tokens
def test_masked_tokens_match_dense_brute_force():
    """Inactive tokens on either side: dense masked library logsumexp on the active rows and
    columns + closed-form adjoint; a prefix mask is the rectangular operator; an all-true mask is
    the plain one.  Row 7 is active but every key in its band is masked: it drops out too."""
    rng = np.random.default_rng(55)
    L, d, W, T, R, eps = 48, 4, 5, 4, 2, 0.8
    Q, K, V, G = (rng.standard_normal((L, d)) for _ in range(4))
    mq, mk = rng.random(L) > 0.25, rng.random(L) > 0.25
    mk[2:13] = False
    mq[7] = True
    out = oracle.band_masked(Q, K, V, G, mq, mk, W, T, R, eps)
    mask = dr.band_mask(L, W) & mq[:, None] & mk[None, :]
    ra, ca = mask.any(1), mask.any(0)
    assert not ra[7] and np.all(out["O"][7] == 0.0) and np.all(np.isneginf(out["U"][:, 7]))
    S = dr.scores(Q, K, eps)
    sub = np.ix_(ra, ca)
    U, Vp = dr.half_steps(S[sub], mask[sub], T, R)
    cf = dr.closed_form_adjoint(S[sub], mask[sub], U, Vp, V[ca], G[ra])
    cs = 1.0 / (eps * np.sqrt(d))
    assert rel(out["O"][ra], cf["O"]) < 1e-12 and np.all(out["O"][~ra] == 0.0)
    assert rel(out["dV"][ca], cf["dV"]) < 1e-12 and np.all(out["dV"][~ca] == 0.0)
    assert rel(out["dQ"][ra], cs * cf["Sbar"] @ K[ca]) < 1e-11 and np.all(out["dQ"][~ra] == 0.0)
    assert rel(out["dK"][ca], cs * cf["Sbar"].T @ Q[ra]) < 1e-11 and np.all(out["dK"][~ca] == 0.0)
    assert np.abs(out["U"][:, ra] - U).max() < 1e-12 and np.all(np.isneginf(out["Vp"][:, ~ca]))
    # prefix masks = rectangle; no mask = the plain operator
    pq, pk = np.arange(L) < 37, np.arange(L) < 29
    pm = oracle.band_masked(Q, K, V, G, pq, pk, W, T, R, eps)
    rc = oracle.band_rect(Q[:37], K[:29], V[:29], G[:37], W, T, R, eps)
    assert rel(pm["O"][:37], rc["O"]) < 1e-13 and rel(pm["dK"][:29], rc["dK"]) < 1e-13
    full = oracle.band_masked(Q, K, V, G, np.ones(L, bool), np.ones(L, bool), W, T, R, eps)
    plain = oracle.band(Q, K, V, G, W, T, R, eps)
    assert all(rel(full[k], plain[k]) < 1e-13 for k in ("O", "dQ", "dK", "dV"))


# ---------------------------------------------------------------- learned dustbin tokens
def test_dustbin_token_matches_dense_augmented_problem():
    """Learned dustbin tokens: the augmented (L+1) x (L+1) problem, dense, with a boolean mask
    for band + spokes, library logsumexp half-steps and the closed-form adjoint, against the
    oracle's sparse construction -- on the gradients of the tokens as well."""
    rng = np.random.default_rng(91)
    L, d, W, T, R, eps = 33, 4, 5, 5, 2, 0.7
    Q, K, V, G = (rng.standard_normal((L, d)) for _ in range(4))
    qd, kd, vd = (rng.standard_normal(d) for _ in range(3))
    out = oracle.band_dustbin_token(Q, K, V, G, qd, kd, vd, W, T, R, eps)
    Qa, Ka, Va = np.vstack([Q, qd]), np.vstack([K, kd]), np.vstack([V, vd])
    Ga = np.vstack([G, np.zeros(d)])
    mask = np.zeros((L + 1, L + 1), dtype=bool)
    mask[:L, :L] = dr.band_mask(L, W)
    mask[L, :] = True
    mask[:, L] = True
    S = dr.scores(Qa, Ka, eps)
    U, Vp = dr.half_steps(S, mask, T, R)
    cf = dr.closed_form_adjoint(S, mask, U, Vp, Va, Ga)
    cs = 1.0 / (eps * np.sqrt(d))
    dQa, dKa = cs * cf["Sbar"] @ Ka, cs * cf["Sbar"].T @ Qa
    assert rel(out["O"], cf["O"][:L]) < 1e-12
    for name, ref in (("dQ", dQa[:L]), ("dK", dKa[:L]), ("dV", cf["dV"][:L]), ("dq_db", dQa[L]),
                      ("dk_db", dKa[L]), ("dv_db", cf["dV"][L])):
        assert rel(out[name], ref) < 1e-11, name
    assert np.abs(out["UV"][2 * R] + 0 - U[R]).max() < 1e-12


def test_dustbin_token_with_zero_tokens_is_the_scalar_dustbin():
    """q_db = k_db = 0 makes every spoke score 0 and v_db = 0 removes the dustbin's value: the
    scalar-score dustbin operator with score 0."""
    rng = np.random.default_rng(92)
    L, d, W, T, R, eps = 40, 4, 6, 4, 2, 0.9
    Q, K, V, G = (rng.standard_normal((L, d)) for _ in range(4))
    z = np.zeros(d)
    tok = oracle.band_dustbin_token(Q, K, V, G, z, z, z, W, T, R, eps)
    sc = oracle.band(Q, K, V, G, W, T, R, eps, True, 0.0)
    assert all(rel(tok[k], sc[k]) < 1e-13 for k in ("O", "dQ", "dK", "dV"))
    assert np.abs(tok["UV"] - sc["UV"]).max() < 1e-12


# ---------------------------------------------------------------- eps-scaling of the stopped base
def test_eps_schedule_matches_dense_stage_loop():
    """Continuation schedule in the base solve: an explicit dense stage loop with the library
    logsumexp (scores A / eps_s, v carried as eps v) gives the same base state, output and --
    through the closed-form adjoint with that base state frozen -- the same gradients."""
    rng = np.random.default_rng(77)
    L, d, W, R, eps = 40, 4, 6, 2, 0.25
    Q, K, V, G = (rng.standard_normal((L, d)) for _ in range(4))
    stages, steps = [1.0, 0.5, 0.25], [3, 2, 4]
    out = oracle.band_eps_schedule(Q, K, V, G, W, stages, steps, R, eps)
    mask = dr.band_mask(L, W)
    A = (Q @ K.T) / np.sqrt(d)
    v = np.zeros(L)
    for s, (es, Ts) in enumerate(zip(stages, steps)):
        Sm = np.where(mask, A / es, -np.inf)
        for _ in range(Ts):
            u = -dr.logsumexp(Sm + v[None, :], axis=1)
            v = -dr.logsumexp(Sm + u[:, None], axis=0)
        if s + 1 < len(stages):
            v = v * es / stages[s + 1]
    assert np.abs(out["v_base"] - v).max() < 1e-12
    S = A / eps
    U, Vp = dr.half_steps(S, mask, 0, R, v0_fixed=v)
    cf = dr.closed_form_adjoint(S, mask, U, Vp, V, G)
    cs = 1.0 / (eps * np.sqrt(d))
    assert rel(out["O"], cf["O"]) < 1e-12 and rel(out["dV"], cf["dV"]) < 1e-12
    assert rel(out["dQ"], cs * cf["Sbar"] @ K) < 1e-11 and rel(out["dK"], cs * cf["Sbar"].T @ Q) < 1e-11
    # one stage at eps is the plain operator
    plain = oracle.band(Q, K, V, G, W, 9, R, eps)
    one = oracle.band_eps_schedule(Q, K, V, G, W, [eps], [9], R, eps)
    assert all(rel(one[k], plain[k]) < 1e-14 for k in ("O", "dQ", "dK", "dV"))
    # equal temperatures in every stage: the split into stages changes nothing
    split = oracle.band_eps_schedule(Q, K, V, G, W, [eps, eps, eps], [3, 2, 4], R, eps)
    assert all(rel(split[k], plain[k]) < 1e-13 for k in ("O", "dQ", "dK", "dV"))


def test_eps_schedule_helps_at_sharp_temperature():
    """What the continuation is for: at a sharp eps and a fixed budget of T steps, the terminal
    plan of the scheduled solve is closer to unit row sums than the plain one."""
    rng = np.random.default_rng(78)
    L, d, W, R, eps, T = 96, 8, 12, 1, 0.05, 8
    Q, K, V = (rng.standard_normal((L, d)) for _ in range(3))
    mask = dr.band_mask(L, W)
    S = dr.scores(Q, K, eps)

    def row_error(o):
        P = dr.plan(S, mask, o["UV"][2 * R], o["UV"][2 * R + 1])
        return np.abs(P.sum(1) - 1.0).max()
    plain = oracle.band(Q, K, V, None, W, T, R, eps)
    sched = oracle.band_eps_schedule(Q, K, V, None, W, [0.4, 0.2, 0.1, 0.05], [2, 2, 2, 2], R, eps)
    assert row_error(sched) < row_error(plain)


def test_dense_zero_scores_is_uniform_plan():
    L = 11
    _, K, V, G = problem(L=L, seed=10)
    out = oracle.band(np.zeros_like(K), K, V, G, W=L + 3, T=3, R=2, eps=1.0)
    np.testing.assert_allclose(out["O"], np.tile(V.mean(0), (L, 1)), atol=1e-13)
    np.testing.assert_allclose(out["dV"], np.tile(G.mean(0), (L, 1)), atol=1e-13)


def test_dense_support_is_textbook_matrix_scaling():
    L, T, R = 12, 9, 2
    Q, K, V, _ = problem(L=L, seed=11)
    eps = 1.3
    out = oracle.band(Q, K, V, None, W=L - 1, T=T, R=R, eps=eps)
    M = np.exp(Q @ K.T / (eps * np.sqrt(Q.shape[1])))
    b = np.ones(L)
    for _ in range(T + R):
        a = 1.0 / (M @ b)
        b = 1.0 / (M.T @ a)
    np.testing.assert_allclose(np.exp(out["UV"][2 * R]), a, rtol=1e-12)
    np.testing.assert_allclose(np.exp(out["UV"][2 * R + 1]), b, rtol=1e-12)
    P = a[:, None] * M * b[None, :]
    np.testing.assert_allclose(out["O"], P @ V, rtol=1e-12, atol=1e-14)
    assert np.abs(P.sum(0) - 1).max() < 1e-13
    # many iterations: doubly stochastic
    far = oracle.band(Q, K, V, None, W=L - 1, T=400, R=1, eps=eps)
    Pf = np.exp(far["UV"][2])[:, None] * M * np.exp(far["UV"][3])[None, :]
    assert np.abs(Pf.sum(1) - 1).max() < 1e-10


# ---------------------------------------------------------------- P11: dustbin bridge
def test_dustbin_is_unit_target_solve_on_augmented_space():
    """Prop. 3: the dustbin path equals the same balanced surrogate on the support
    band U spokes U corner, here built explicitly as a dense (L+1)x(L+1) problem
    and handed both to the support-generic core and to the dense brute force."""
    L, W, T, R, eps, sdb = 19, 3, 5, 2, 0.6, 0.4
    Q, K, V, G = problem(L=L, seed=12)
    out = oracle.band(Q, K, V, G, W=W, T=T, R=R, eps=eps, dustbin=True, dustbin_score=sdb)
    Lp = L + 1
    mask = np.zeros((Lp, Lp), bool)
    mask[:L, :L] = dr.band_mask(L, W)
    mask[L, :] = mask[:, L] = True
    S = np.full((Lp, Lp), sdb)
    S[:L, :L] = dr.scores(Q, K, eps)
    Va, Ga = np.vstack([V, np.zeros((1, 4))]), np.vstack([G, np.zeros((1, 4))])
    # (a) dense brute force with library logsumexp + closed-form adjoint
    U, Vp = dr.half_steps(S, mask, T, R)
    cf = dr.closed_form_adjoint(S, mask, U, Vp, Va, Ga)
    cs = 1.0 / (eps * 2.0)
    assert rel(out["O"], cf["O"][:L]) < 1e-13
    assert rel(out["dV"], cf["dV"][:L]) < 1e-13
    assert rel(out["dQ"], cs * cf["Sbar"][:L, :L] @ K) < 1e-12
    assert rel(out["dK"], cs * cf["Sbar"][:L, :L].T @ Q) < 1e-12
    assert np.abs(cf["O"][L]).max() > 1e-3          # the dustbin row does carry mass
    # (b) the same explicit problem through the generic core
    rows, cols = np.nonzero(mask)
    rptr = np.concatenate([[0], np.cumsum(mask.sum(1))])
    g = oracle.core(rptr, cols, S[rows, cols], Va, Ga, T, R)
    assert rel(out["O"], g["O"][:L]) < 1e-14
    np.testing.assert_allclose(out["UV"][0::2], g["U"], atol=1e-13)
    np.testing.assert_allclose(out["UV"][1::2], g["Vp"], atol=1e-13)
    # without a dustbin the numbers are different: the flag is not a no-op
    plain = oracle.band(Q, K, V, G, W=W, T=T, R=R, eps=eps)
    assert rel(plain["O"], out["O"]) > 1e-3


def test_generic_core_handles_rectangular_masked_support():
    rng = np.random.default_rng(13)
    m, n, dv = 7, 10, 3
    mask = rng.random((m, n)) < 0.6
    mask[np.arange(m), np.arange(m)] = True
    mask[0, :] = True
    mask[:, n - 1] = True
    S = rng.standard_normal((m, n))
    V, G = rng.standard_normal((n, dv)), rng.standard_normal((m, dv))
    rows, cols = np.nonzero(mask)
    rptr = np.concatenate([[0], np.cumsum(mask.sum(1))])
    g = oracle.core(rptr, cols, S[rows, cols], V, G, 5, 2)
    U, Vp = dr.half_steps(S, mask, 5, 2)
    cf = dr.closed_form_adjoint(S, mask, U, Vp, V, G)
    assert rel(g["O"], cf["O"]) < 1e-13 and rel(g["dV"], cf["dV"]) < 1e-13
    assert np.abs(g["Sbar"] - cf["Sbar"][rows, cols]).max() < 1e-13


# ---------------------------------------------------------------- printed numbers
def test_paper_ledger_numbers():
    """Band definition |i-j| <= W reproduces the printed support sizes
    (App. C, analytic memory ledger and the four-plan table caption)."""
    with open(os.path.join(GOLDEN, "paper_ledger.json")) as f:
        led = json.load(f)
    w = Workload("ledger", 0, 1, 1, led["L"], 64, led["W"], 15, 2, 1.0, "f32")
    assert round(w.edges / 1e6, 2) == led["active_entries_millions"]
    assert round(w.edges * 4 / 2**20, 2) == led["one_reference_plan_MiB"]
    assert round(4 * w.edges * 4 / 2**20, 2) == led["direct_four_plan_MiB"]
    assert round(6 * led["L"] * 4 / 2**20, 3) == led["tail_uv_vectors_MiB"]
    for L, mb in led["one_reference_MB_at_W256"].items():
        e = Workload("x", 0, 1, 1, int(L), 64, 256, 15, 2, 1.0, "f32").edges
        assert round(e * 4 / 1e6, 2) == mb
    # and the count agrees with the mask, and with what the oracle treats as active
    for L, W in ((24, 5), (9, 20), (33, 1)):
        e = Workload("x", 0, 1, 1, L, 4, W, 1, 1, 1.0, "f32").edges
        assert e == int(dr.band_mask(L, W).sum())
        Q, K, V, G = problem(L=L)
        sb = oracle.band(Q, K, V, G, W=W, T=1, R=1, eps=1.0, want_sbar=True)["Sbar"]
        assert int((sb != 0).sum()) == e
    assert CONFIGS["paper"].edges == 134414080


def test_centered_gauge_worked_example():
    """App. F.2 worked 2x2 example: a same-time plan is unchanged by centering,
    a mixed-time plan picks up exp(c_q - c_p) = exp(-3/2).  Our path keeps raw
    potentials, so this fixes the convention (no scalar factors on alpha, beta,
    delta) rather than an oracle function."""
    with open(os.path.join(GOLDEN, "gauge_example.json")) as f:
        ex = json.load(f)
    S, up, vp, vq = (np.array(ex[k]) for k in ("S", "u_p", "v_p", "v_q"))
    cp, cq = ex["c_p"], ex["c_q"]
    same = np.exp(S + up[:, None] + vp[None, :])
    same_c = np.exp(S + (up - cp)[:, None] + (vp + cp)[None, :])
    mixed = np.exp(S + up[:, None] + vq[None, :])
    mixed_c = np.exp(S + (up - cp)[:, None] + (vq + cq)[None, :])
    np.testing.assert_allclose(same_c, same, rtol=1e-15)
    np.testing.assert_allclose(mixed_c / mixed, np.exp(-1.5), rtol=1e-15)
    assert abs(ex["mixed_factor_log"] - (cq - cp)) < 1e-15
