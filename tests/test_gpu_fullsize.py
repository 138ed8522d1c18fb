"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The operator is local: one half-step moves information by at most W positions, so
after 2(T+R) half-steps, the output map and the five backward sweeps a value at
position p depends only on inputs within (2(T+R) + 6) W of p.  The oracle is
therefore run on windows of the sequence (a window's own ends behave like
sequence ends, which is exact when the window touches a real end) and compared
on the window's centre, element by element, with the GPU result of the whole
problem.  The dustbin couples all positions through its extra row and column, so
that configuration is compared on whole problems instead.
"""
import sys

import numpy as np
import pytest

import oracle
from paper_2605_08123_amd.workloads import CONFIGS, make_inputs
from tests.test_gpu_parity import TOL, run_gpu

pytestmark = pytest.mark.gpu


def window_check(w, got, arrays, b, h, c0, c1):
    """Compare rows [c0, c1) of problem (b, h) against the oracle run on a window with
    a margin of (2(T+R) + 7) W on each side (clipped at the true sequence ends)."""
    margin = (2 * (w.T + w.R) + 7) * w.W
    a0, a1 = max(0, c0 - margin), min(w.L, c1 + margin)
    q, k, v, g = (x[b, h, a0:a1] for x in arrays)
    ref = oracle.band(q, k, v, g, w.W, w.T, w.R, w.eps)
    errs = {}
    for name in ("O", "dQ", "dK", "dV"):
        r = ref[name][c0 - a0:c1 - a0]
        x = got[name][b, h, c0:c1]
        errs[name] = float(np.linalg.norm(x - r) / np.linalg.norm(r))
    print(f"   ({b},{h}) rows [{c0},{c1}) window [{a0},{a1}):", {k: f"{e:.2e}" for k, e in errs.items()},
          flush=True)
    for name, e in errs.items():
        assert e <= TOL[w.dtype], (name, e)


@pytest.mark.parametrize("name", ["paper", "long", "paper_w1024"])
def test_full_size_windows(name):
    w = CONFIGS[name]
    print(f"\n[case] {w}", flush=True)
    sys.stdout.flush()
    arrays = make_inputs(w)
    got = run_gpu(w, arrays)
    for key in ("O", "dQ", "dK", "dV"):
        assert np.isfinite(got[key]).all(), key
    L = w.L
    window_check(w, got, arrays, 0, 0, 0, 2048)                    # true left end
    window_check(w, got, arrays, 0, w.H - 1, L // 2 - 1000, L // 2 + 1048)   # interior, unaligned
    if w.W <= 256:   # (a window at W = 1024 is 86 k rows of 2049 edges: two of them are enough)
        window_check(w, got, arrays, 0, w.H - 1, L - 2048, L)      # true right end
    # properties that hold at any size: unit column sums of P22 show up as sum_j dK_j = 0
    # (every row of the score cotangent sums to zero) and <dO, O> totals equal <V, dV> totals
    for h in range(w.H):
        dk = got["dK"][0, h]
        assert np.abs(dk.sum(0)).max() <= 2e-2 * np.abs(dk).sum(0).max()
        lhs = float((arrays[3][0, h].astype(np.float64) * got["O"][0, h]).sum())
        rhs = float((arrays[2][0, h].astype(np.float64) * got["dV"][0, h]).sum())
        assert abs(lhs - rhs) <= 2e-2 * max(abs(lhs), abs(rhs), 1.0) + 2e-2 * np.sqrt(L)


def test_dustbin_config_full_size():
    """Dustbin configuration at its full size; the oracle checks two of the eight problems."""
    w = CONFIGS["dustbin"]
    print(f"\n[case] {w}", flush=True)
    arrays = make_inputs(w)
    got = run_gpu(w, arrays)
    for (b, h) in ((0, 0), (1, 3)):
        q, k, v, g = (x[b, h] for x in arrays)
        ref = oracle.band(q, k, v, g, w.W, w.T, w.R, w.eps, True, w.dustbin_score)
        errs = {n: float(np.linalg.norm(got[n][b, h] - ref[n]) / np.linalg.norm(ref[n]))
                for n in ("O", "dQ", "dK", "dV")}
        print(f"   ({b},{h}):", {k: f"{e:.2e}" for k, e in errs.items()}, flush=True)
        for n, e in errs.items():
            assert e <= TOL[w.dtype], (n, e)


def test_mid_config_full_size():
    """Mid configuration, all 32 problems on the GPU; the oracle checks four of them."""
    w = CONFIGS["mid"]
    print(f"\n[case] {w}", flush=True)
    arrays = make_inputs(w)
    got = run_gpu(w, arrays)
    for (b, h) in ((0, 0), (1, 5), (2, 2), (3, 7)):
        q, k, v, g = (x[b, h] for x in arrays)
        ref = oracle.band(q, k, v, g, w.W, w.T, w.R, w.eps)
        for n in ("O", "dQ", "dK", "dV"):
            e = float(np.linalg.norm(got[n][b, h] - ref[n]) / np.linalg.norm(ref[n]))
            assert e <= TOL[w.dtype], (b, h, n, e)
