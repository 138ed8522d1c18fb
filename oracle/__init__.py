"""ctypes front end of the fp64 CPU oracle (oracle/sinkhorn_oracle.c).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
cpu_baseline leg may import this; the product package never does.

The C file is compiled with gcc on first use if the shared object is missing
or older than its source.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sinkhorn_oracle.c")
_LIB = os.path.join(_HERE, "libska_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", _LIB,
                               _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        c_d = ctypes.POINTER(ctypes.c_double)
        i64, i32 = ctypes.c_int64, ctypes.c_int
        lib.ska_oracle_threads.restype = i32
        lib.ska_oracle_core.restype = i32
        lib.ska_oracle_core.argtypes = [i64, i64, i64, ctypes.c_void_p, ctypes.c_void_p, c_d, c_d,
                                        c_d, i32, i32, i32, c_d, c_d, c_d, c_d, c_d, c_d, c_d, c_d]
        lib.ska_oracle_band.restype = i32
        lib.ska_oracle_band.argtypes = [c_d, c_d, c_d, c_d, i64, i32, i64, i32, i32,
                                        ctypes.c_double, i32, ctypes.c_double, c_d, c_d, c_d, c_d,
                                        c_d, c_d, c_d, c_d]
        lib.ska_oracle_core_marg.restype = i32
        lib.ska_oracle_core_marg.argtypes = [i64, i64, i64, ctypes.c_void_p, ctypes.c_void_p, c_d, c_d,
                                             c_d, i32, i32, i32, c_d, c_d, c_d, c_d, c_d, c_d, c_d, c_d,
                                             c_d, c_d]
        lib.ska_oracle_band_marg.restype = i32
        lib.ska_oracle_band_marg.argtypes = [c_d, c_d, c_d, c_d, i64, i32, i64, i32, i32,
                                             ctypes.c_double, i32, ctypes.c_double, c_d, c_d, c_d, c_d,
                                             c_d, c_d, c_d, c_d, c_d, c_d]
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().ska_oracle_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def core(rptr, col, S, V, G, T, R, v0_fixed=None, log_a=None, log_b=None):
    """Support-generic solve on explicit edge scores.

    rptr[m+1], col[nnz] describe the active support row by row; S[nnz] are the
    effective scores.  Returns a dict with O, U[(R+1),m], Vp[(R+1),n] and, when
    G is given, Sbar[nnz], dV, ubar, vbar.  log_a[m], log_b[n]: logarithms of the row and
    column targets (compatible general marginals); None for unit targets.
    """
    lib = _load()
    rptr = np.ascontiguousarray(rptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    S, V, G, v0_fixed, log_a, log_b = _f64(S), _f64(V), _f64(G), _f64(v0_fixed), _f64(log_a), _f64(log_b)
    m, nnz = len(rptr) - 1, len(col)
    n, dv = V.shape
    assert rptr[-1] == nnz and S.shape == (nnz,)
    assert col.size == 0 or (col.min() >= 0 and col.max() < n)
    out = {"O": np.empty((m, dv)), "U": np.empty((R + 1, m)), "Vp": np.empty((R + 1, n))}
    if G is not None:
        assert G.shape == (m, dv)
        out.update(Sbar=np.empty(nnz), dV=np.empty((n, dv)), ubar=np.empty((R + 1, m)),
                   vbar=np.empty((R + 1, n)))
    assert (log_a is None or log_a.shape == (m,)) and (log_b is None or log_b.shape == (n,))
    rc = lib.ska_oracle_core_marg(m, n, nnz, rptr.ctypes.data, col.ctypes.data, _p(S), _p(V), _p(G), dv,
                                  T, R, _p(v0_fixed), _p(log_a), _p(log_b), _p(out["O"]), _p(out["U"]),
                                  _p(out["Vp"]), _p(out.get("Sbar")), _p(out.get("dV")),
                                  _p(out.get("ubar")), _p(out.get("vbar")))
    if rc:
        raise RuntimeError(f"ska_oracle_core failed ({rc})")
    return out


def band(Q, K, V, G, W, T, R, eps, dustbin=False, dustbin_score=0.0, v0_fixed=None,
         want_sbar=False, log_a=None, log_b=None):
    """Banded operator for one problem; Q, K, V, G are [L, d] arrays (G may be None).

    Returns a dict: O[L,d], UV[2(R+1), Lp] ordered u0,v0,u1,v1,...; with G also
    dQ, dK, dV [L,d], bars[2(R+1), Lp] (same order) and, if want_sbar,
    Sbar[L, 2W+1] indexed [i, j-i+W].  log_a, log_b [Lp]: logarithms of the row and
    column targets, None for unit targets.
    """
    lib = _load()
    Q, K, V, G, v0_fixed = _f64(Q), _f64(K), _f64(V), _f64(G), _f64(v0_fixed)
    log_a, log_b = _f64(log_a), _f64(log_b)
    L, d = Q.shape
    assert K.shape == (L, d) and V.shape == (L, d) and (G is None or G.shape == (L, d))
    Lp = L + (1 if dustbin else 0)
    assert v0_fixed is None or v0_fixed.shape == (Lp,)
    out = {"O": np.empty((L, d)), "UV": np.empty((2 * (R + 1), Lp))}
    if G is not None:
        out.update(dQ=np.empty((L, d)), dK=np.empty((L, d)), dV=np.empty((L, d)),
                   bars=np.empty((2 * (R + 1), Lp)))
        if want_sbar:
            out["Sbar"] = np.empty((L, 2 * W + 1))
    assert (log_a is None or log_a.shape == (Lp,)) and (log_b is None or log_b.shape == (Lp,))
    rc = lib.ska_oracle_band_marg(_p(Q), _p(K), _p(V), _p(G), L, d, W, T, R, float(eps),
                                  1 if dustbin else 0, float(dustbin_score), _p(v0_fixed), _p(log_a),
                                  _p(log_b), _p(out["O"]), _p(out["UV"]), _p(out.get("dQ")),
                                  _p(out.get("dK")), _p(out.get("dV")), _p(out.get("bars")),
                                  _p(out.get("Sbar")))
    if rc:
        raise RuntimeError(f"ska_oracle_band failed ({rc})")
    return out


def band_masked(Q, K, V, G, mask_q, mask_k, W, T, R, eps, log_a=None, log_b=None):
    """Banded operator with inactive tokens (the masked half-steps of Eq. 1-2: the support is
    {(i, j): |i - j| <= W, mask_q[i], mask_k[j]}).  Inactive tokens, and active ones left without
    any partner, take no part: potential -inf (reported as such), zero output and gradients.
    Q, K, V, G are [L, d]; returns O, dQ, dK, dV [L, d], U [(R+1), L], Vp [(R+1), L].  Support and
    scores are built here for the support-generic core, which runs on the active tokens only."""
    Q, K, V, G = _f64(Q), _f64(K), _f64(V), _f64(G)
    L, d = Q.shape
    mq, mk = np.asarray(mask_q, dtype=bool), np.asarray(mask_k, dtype=bool)
    ii, jj = np.nonzero((np.abs(np.arange(L)[:, None] - np.arange(L)[None, :]) <= W) & mq[:, None] & mk[None, :])
    rows_act, cols_act = np.unique(ii), np.unique(jj)         # tokens with at least one edge
    rmap, cmap = np.full(L, -1), np.full(L, -1)
    rmap[rows_act], cmap[cols_act] = np.arange(len(rows_act)), np.arange(len(cols_act))
    r_, c_ = rmap[ii], cmap[jj].astype(np.int32)              # nonzero() is row-major: rows sorted
    rptr = np.concatenate(([0], np.cumsum(np.bincount(r_, minlength=len(rows_act))))).astype(np.int64)
    cs = 1.0 / (eps * np.sqrt(d))
    S = cs * np.einsum("ek,ek->e", Q[ii], K[jj])
    r = core(rptr, c_, S, V[cols_act], None if G is None else G[rows_act], T, R,
             log_a=None if log_a is None else _f64(log_a)[rows_act],
             log_b=None if log_b is None else _f64(log_b)[cols_act])
    out = {"O": np.zeros((L, d)), "U": np.full((R + 1, L), -np.inf), "Vp": np.full((R + 1, L), -np.inf)}
    out["O"][rows_act] = r["O"]
    out["U"][:, rows_act], out["Vp"][:, cols_act] = r["U"], r["Vp"]
    if G is not None:
        dQ, dK, dV = np.zeros((L, d)), np.zeros((L, d)), np.zeros((L, d))
        np.add.at(dQ, ii, cs * r["Sbar"][:, None] * K[jj])
        np.add.at(dK, jj, cs * r["Sbar"][:, None] * Q[ii])
        dV[cols_act] = r["dV"]
        out.update(dQ=dQ, dK=dK, dV=dV)
    return out


def band_dustbin_token(Q, K, V, G, q_db, k_db, v_db, W, T, R, eps):
    """Single-active-dustbin bridge with a learned dustbin token per side (Sec. 'Single-Active-
    Dustbin Bridge'): the tensors are augmented by one row, Q~ = [Q; q_db], K~ = [K; k_db],
    V~ = [V; v_db], and the unit-target operator runs on the sparse-spoke support
    band + {(i, d_k)} + {(d_q, j)} + {(d_q, d_k)} with every score q~_i . k~_j / (eps sqrt d).
    The dustbin query row has no output cotangent (its output is dropped).  Returns O [L,d],
    dQ, dK, dV [L,d], dq_db, dk_db, dv_db [d], UV [2(R+1), L+1].  Support and scores are built
    here; the solve is the support-generic core."""
    Q, K, V, G = _f64(Q), _f64(K), _f64(V), _f64(G)
    L, d = Q.shape
    Qa, Ka, Va = (np.vstack([x, _f64(t)[None, :]]) for x, t in ((Q, q_db), (K, k_db), (V, v_db)))
    i = np.arange(L)
    lo, hi = np.maximum(i - W, 0), np.minimum(i + W, L - 1)
    cnt = hi - lo + 1
    rows_b = np.repeat(i, cnt)
    start = np.concatenate(([0], np.cumsum(cnt)))[:-1]
    cols_b = np.arange(cnt.sum()) - np.repeat(start, cnt) + np.repeat(lo, cnt)
    # row i: its band columns then the dustbin column; dustbin row: every column
    order_rows = np.concatenate([rows_b, i, np.full(L + 1, L)])
    order_cols = np.concatenate([cols_b, np.full(L, L), np.arange(L + 1)])
    key = np.lexsort((order_cols, order_rows))
    rows, cols = order_rows[key], order_cols[key].astype(np.int32)
    rptr = np.concatenate(([0], np.cumsum(np.bincount(rows, minlength=L + 1)))).astype(np.int64)
    cs = 1.0 / (eps * np.sqrt(d))
    S = cs * np.einsum("ek,ek->e", Qa[rows], Ka[cols])
    Ga = None if G is None else np.vstack([G, np.zeros((1, d))])
    r = core(rptr, cols, S, Va, Ga, T, R)
    UV = np.empty((2 * (R + 1), L + 1))
    UV[0::2], UV[1::2] = r["U"], r["Vp"]
    out = {"O": r["O"][:L], "UV": UV}
    if G is not None:
        dQa, dKa = np.zeros_like(Qa), np.zeros_like(Ka)
        np.add.at(dQa, rows, cs * r["Sbar"][:, None] * Ka[cols])
        np.add.at(dKa, cols, cs * r["Sbar"][:, None] * Qa[rows])
        out.update(dQ=dQa[:L], dK=dKa[:L], dV=r["dV"][:L], dq_db=dQa[L], dk_db=dKa[L], dv_db=r["dV"][L])
    return out


def band_eps_schedule(Q, K, V, G, W, eps_stages, T_stages, R, eps, dustbin=False, dustbin_score=0.0,
                      log_a=None, log_b=None):
    """Stopped base solve with a continuation schedule eps_1 >= ... >= eps_N = eps (remark
    "Fixed-Budget eps-Scaling"): stage s runs T_s full steps on the scores A / eps_s.  Between
    stages the column log-scaling is carried as a potential in cost units, eps_s v -> v' =
    v eps_s / eps_{s+1} (the paper does not say how; this is the usual continuation rule).  The
    tail and its backward are the ordinary ones at eps, started from the final base state, which
    is a constant for differentiation.  dustbin_score is the spoke score at eps and scales like
    every other score.  Built from `band` calls: a stage is T_s tail steps from a fixed v."""
    Q = _f64(Q)
    L = Q.shape[0]
    assert len(eps_stages) == len(T_stages) >= 1 and abs(eps_stages[-1] - eps) <= 1e-12 * eps
    v = np.zeros(L + (1 if dustbin else 0))
    for s, (es, Ts) in enumerate(zip(eps_stages, T_stages)):
        if Ts > 0:
            r = band(Q, K, V, None, W, 0, Ts, es, dustbin, dustbin_score * eps / es, v0_fixed=v,
                     log_a=log_a, log_b=log_b)
            v = r["UV"][2 * Ts + 1].copy()
        if s + 1 < len(eps_stages):
            v = v * (es / eps_stages[s + 1])
    out = band(Q, K, V, G, W, 0, R, eps, dustbin, dustbin_score, v0_fixed=v, log_a=log_a, log_b=log_b)
    out["v_base"] = v
    return out


def band_rect(Q, K, V, G, W, T, R, eps, log_a=None, log_b=None):
    """Banded operator on a rectangle: Q, G are [Lq, d], K, V are [Lk, d] (token sequences of
    different lengths, or a padded batch item cut to its valid lengths); the support is
    {(i, j): |i - j| <= W, i < Lq, j < Lk}.  The support and the edge scores are built here and
    handed to the support-generic core; the score cotangent is pushed to Q and K by the chain
    rule of S = Q K^T / (eps sqrt d).  Returns O, dQ [Lq, d], dK, dV [Lk, d], U [(R+1), Lq],
    Vp [(R+1), Lk] (rows or columns without any active edge have potential 0 and zero results).
    """
    Q, K, V, G = _f64(Q), _f64(K), _f64(V), _f64(G)
    (Lq, d), Lk = Q.shape, K.shape[0]
    assert K.shape == (Lk, d) and V.shape == (Lk, d) and (G is None or G.shape == (Lq, d))
    lo = np.maximum(np.arange(Lq) - W, 0)
    hi = np.minimum(np.arange(Lq) + W, Lk - 1)
    cnt = np.maximum(hi - lo + 1, 0)
    rptr = np.concatenate(([0], np.cumsum(cnt))).astype(np.int64)
    rows = np.repeat(np.arange(Lq), cnt)
    cols = (np.arange(rptr[-1]) - np.repeat(rptr[:-1], cnt) + np.repeat(lo, cnt)).astype(np.int32)
    cs = 1.0 / (eps * np.sqrt(d))
    S = cs * np.einsum("ek,ek->e", Q[rows], K[cols])
    r = core(rptr, cols, S, V, G, T, R, log_a=log_a, log_b=log_b)
    out = {"O": r["O"], "U": r["U"], "Vp": r["Vp"]}
    if G is not None:
        dQ, dK = np.zeros_like(Q), np.zeros_like(K)
        np.add.at(dQ, rows, cs * r["Sbar"][:, None] * K[cols])
        np.add.at(dK, cols, cs * r["Sbar"][:, None] * Q[rows])
        out.update(dQ=dQ, dK=dK, dV=r["dV"], ubar=r["ubar"], vbar=r["vbar"])
    return out


def band_batched(Q, K, V, G, W, T, R, eps, dustbin=False, dustbin_score=0.0, log_a=None, log_b=None):
    """[B,H,L,d] inputs, one independent problem per (b,h) (log_a, log_b: [B,H,Lp] or None).
    Returns stacked arrays."""
    B, H, L, d = Q.shape
    keys = ("O", "UV") + (("dQ", "dK", "dV") if G is not None else ())
    acc = {k: [] for k in keys}
    for b in range(B):
        for h in range(H):
            r = band(Q[b, h], K[b, h], V[b, h], None if G is None else G[b, h], W, T, R, eps,
                     dustbin, dustbin_score, log_a=None if log_a is None else log_a[b, h],
                     log_b=None if log_b is None else log_b[b, h])
            for k in keys:
                acc[k].append(r[k])
    return {k: np.stack(v).reshape((B, H) + v[0].shape) for k, v in acc.items()}
