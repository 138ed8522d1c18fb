"""Brute-force dense fp64 helpers used only to pin the oracle.

Everything here works on full m x n matrices with a boolean mask, uses
scipy's logsumexp as the library routine for the half-steps, and evaluates the
tail adjoint from the closed-form recurrences of Prop. 1 (Eqs. 3-6) rather than
by a reverse sweep, so that it is a second, differently-derived statement of
the same mathematics.
"""
import numpy as np
from scipy.special import logsumexp


def band_mask(L, W):
    i = np.arange(L)
    return np.abs(i[:, None] - i[None, :]) <= W


def scores(Q, K, eps):
    return (Q @ K.T) / (eps * np.sqrt(Q.shape[1]))


def half_steps(S, mask, T, R, v0_fixed=None, a=None, b=None):
    """u^(0..R), v^(0..R) by Eq. (1)-(2); base from v=0 unless v0_fixed is given.
    a, b: compatible positive row / column targets (None = ones)."""
    Sm = np.where(mask, S, -np.inf)
    m, n = S.shape
    la = np.zeros(m) if a is None else np.log(a)
    lb = np.zeros(n) if b is None else np.log(b)
    if v0_fixed is None:
        u, v = np.zeros(m), np.zeros(n)
        for _ in range(T):
            u = la - logsumexp(Sm + v[None, :], axis=1)
            v = lb - logsumexp(Sm + u[:, None], axis=0)
    else:
        u, v = np.zeros(m), np.array(v0_fixed, dtype=np.float64)
    U, Vp = [u], [v]
    for _ in range(R):
        u = la - logsumexp(Sm + Vp[-1][None, :], axis=1)
        v = lb - logsumexp(Sm + u[:, None], axis=0)
        U.append(u)
        Vp.append(v)
    return np.array(U), np.array(Vp)


def plan(S, mask, u, v):
    return np.where(mask, np.exp(np.where(mask, S, 0.0) + u[:, None] + v[None, :]), 0.0)


def closed_form_adjoint(S, mask, U, Vp, V, G, drop_terminal_pullback=False, a=None, b=None):
    """Prop. 1: dual cotangents and the score cotangent, any R >= 1.  With targets a, b:
    the general-marginal finite-tail VJP (every ubar is divided by a, every vbar by b where
    it multiplies a plan)."""
    R = U.shape[0] - 1
    a = np.ones(S.shape[0]) if a is None else np.asarray(a, dtype=np.float64)
    b = np.ones(S.shape[1]) if b is None else np.asarray(b, dtype=np.float64)
    P = lambda p, q: plan(S, mask, U[p], Vp[q])
    Z = G @ V.T
    PRR = P(R, R)
    gu, gv = (PRR * Z).sum(1), (PRR * Z).sum(0)
    ub = np.zeros_like(U)
    vb = np.zeros_like(Vp)
    vb[R] = gv
    ub[R] = gu if drop_terminal_pullback else gu - PRR @ (vb[R] / b)
    for t in range(R, 0, -1):
        vb[t - 1] = -P(t, t - 1).T @ (ub[t] / a)
        if t >= 2:
            ub[t - 1] = -P(t - 1, t - 1) @ (vb[t - 1] / b)
    Sbar = PRR * Z
    for t in range(1, R + 1):
        if not (drop_terminal_pullback and t == R):
            Sbar = Sbar - P(t, t) * (vb[t] / b)[None, :]
        Sbar = Sbar - P(t, t - 1) * (ub[t] / a)[:, None]
    return dict(Sbar=Sbar, ubar=ub, vbar=vb, dV=PRR.T @ G, O=PRR @ V, gu=gu, gv=gv)


def one_reference_sbar(S, mask, U, Vp, V, G, ubar, vbar, delta_from=0):
    """Prop. 2 (R = 2): score cotangent from P^(2,2) and vector modifiers only."""
    P22 = plan(S, mask, U[2], Vp[2])
    Z = G @ V.T
    alpha = np.exp(U[1] - U[2])
    beta = np.exp(Vp[1] - Vp[2])
    delta = np.exp(Vp[delta_from] - Vp[2])
    br = (Z - vbar[2][None, :] - beta[None, :] * ubar[2][:, None]
          - alpha[:, None] * (beta * vbar[1])[None, :]
          - (alpha * ubar[1])[:, None] * delta[None, :])
    return P22 * br
