"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The operator is local: one half-step moves information by at most W positions, so
after 2(T+R) half-steps, the output map and the five backward sweeps a value at
position p depends only on inputs within (2(T+R) + 6) W of p.  The oracle is
therefore run on windows of the sequence (a window's own ends behave like
sequence ends, which is exact when the window touches a real end) and compared
on the window's centre, element by element, with the GPU result of the whole
problem.  The dustbin couples all positions through its extra row and column, so
that configuration is compared on whole problems instead.  Where the oracle is cheap the
comparison is not sampled at all: every problem of the Mid, Dustbin and Long configurations and
both heads of the benchmark workload are compared whole, each of O, dQ, dK, dV by itself.
"""
import sys

import numpy as np
import pytest

import oracle
from paper_2605_08123_amd.workloads import CONFIGS, make_inputs
from tests.measures import assert_per_tensor, floors
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


def whole_problems(w, dustbin=False):
    """Every (batch, head) problem of the configuration, whole, against the oracle."""
    arrays = make_inputs(w)
    got = run_gpu(w, arrays, one_call=True)   # the one-call step is what bench.py times
    worst = {}
    for b in range(w.B):
        for h in range(w.H):
            q, k, v, g = (x[b, h] for x in arrays)
            ref = oracle.band(q, k, v, g, w.W, w.T, w.R, w.eps, dustbin, w.dustbin_score)
            res = assert_per_tensor({n: got[n][b, h] for n in ("O", "dQ", "dK", "dV")}, ref, w.dtype,
                                    floors(w.dtype, q, k, v, g, ref["O"], w.eps), where=f"{w.name} ({b},{h})")
            for n, r in res.items():
                assert r[2] <= TOL[w.dtype], (b, h, n, r[2])   # nothing cancels here: the relative bar itself
                worst[n] = max(worst.get(n, 0.0), r[2])
            for t in range(w.R + 1):
                s_got = got["UV"][b, h, 2 * t] + got["UV"][b, h, 2 * t + 1]
                s_ref = ref["UV"][2 * t] + ref["UV"][2 * t + 1]
                assert np.abs(s_got - s_ref).max() < 2e-2, (b, h, t)
    print(f"   worst rel-L2 over {w.B * w.H} whole problems:", {n: f"{e:.2e}" for n, e in worst.items()}, flush=True)


@pytest.mark.parametrize("name", ["paper", "paper_w1024"])
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
    """Dustbin configuration at its full size, all eight problems whole."""
    w = CONFIGS["dustbin"]
    print(f"\n[case] {w}", flush=True)
    whole_problems(w, dustbin=True)


def test_mid_config_full_size():
    """Mid configuration at its full size, all 32 problems whole."""
    w = CONFIGS["mid"]
    print(f"\n[case] {w}", flush=True)
    whole_problems(w)


def test_long_config_full_size():
    """Long configuration at its full size, all four heads whole."""
    w = CONFIGS["long"]
    print(f"\n[case] {w}", flush=True)
    whole_problems(w)


def test_full_size_padded_lengths():
    """The benchmark shape as a padded item: 200003 valid queries, 187654 valid keys of 262144.
    The oracle's rectangular operator runs on a window that ends at the true (ragged) end of
    the valid region; queries between len_k + W and len_q have no key in their band and are
    zeros like the padding, whose inputs are NaN here."""
    import torch

    import paper_2605_08123_amd as ska
    w = CONFIGS["paper"]
    lq, lk = 200003, 187654
    print(f"\n[case] {w} len_q={lq} len_k={lk}", flush=True)
    q, k, v, g = make_inputs(w)
    q[:, :, lq:] = np.nan
    g[:, :, lq:] = np.nan
    k[:, :, lk:] = np.nan
    v[:, :, lk:] = np.nan
    dev = torch.device("cuda:0")
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(torch.bfloat16) for x in (q, k, v, g))
    tq = torch.tensor([lq], dtype=torch.int32, device=dev)
    tk = torch.tensor([lk], dtype=torch.int32, device=dev)
    O, UV = ska.sinkhorn_attn_fwd_varlen(Q, K, V, None, None, tq, tk, w.W, w.T, w.R, w.eps)
    dQ, dK, dV = ska.sinkhorn_attn_bwd_varlen(Q, K, V, None, None, tq, tk, O, G, UV, w.W, w.T, w.R, w.eps)
    torch.cuda.synchronize()
    got = {n: x.float().cpu().numpy().astype(np.float64) for n, x in dict(O=O, dQ=dQ, dK=dK, dV=dV).items()}
    for n in got:
        assert np.isfinite(got[n]).all(), n
    le = lk + w.W                                   # first query row without any valid key
    for h in range(w.H):
        assert np.all(got["O"][0, h, le:] == 0.0) and np.all(got["dQ"][0, h, le:] == 0.0)
        assert np.all(got["dK"][0, h, lk:] == 0.0) and np.all(got["dV"][0, h, lk:] == 0.0)
        assert np.all(UV[0, h, 0::2, le:].cpu().numpy() == 0.0) and np.all(UV[0, h, 1::2, lk:].cpu().numpy() == 0.0)
    margin = (2 * (w.T + w.R) + 7) * w.W
    a0 = lk - 1500 - margin
    qr, kr, vr, gr = (x.float().cpu().numpy().astype(np.float64) for x in (Q, K, V, G))
    for h in (0, w.H - 1):
        ref = oracle.band_rect(qr[0, h, a0:lq], kr[0, h, a0:lk], vr[0, h, a0:lk], gr[0, h, a0:lq],
                               w.W, w.T, w.R, w.eps)
        errs = {}
        for n, end in (("O", le), ("dQ", le), ("dK", lk), ("dV", lk)):
            r = ref[n][lk - 1500 - a0:end - a0]
            errs[n] = float(np.linalg.norm(got[n][0, h, lk - 1500:end] - r) / np.linalg.norm(r))
        print(f"   (0,{h}) rows [{lk - 1500}, end):", {n: f"{e:.2e}" for n, e in errs.items()}, flush=True)
        for n, e in errs.items():
            assert e <= TOL[w.dtype], (n, e)
    # the left part is far from the ragged end: identical to an ordinary window of the full problem
    window_check(w, {n: got[n] for n in got}, (qr, kr, vr, gr), 0, 0, 0, 2048)


def test_dustbin_config_with_learned_tokens():
    """The dustbin configuration at its full size with a learned token per side instead of the
    scalar score; the oracle checks one of the eight problems (tokens' gradients included)."""
    import torch

    import paper_2605_08123_amd as ska
    w = CONFIGS["dustbin"]
    print(f"\n[case] {w} with learned dustbin tokens", flush=True)
    arrays = make_inputs(w)
    rng = np.random.default_rng(5)
    toks = [rng.standard_normal((w.B, w.H, w.d)).astype(np.float32) for _ in range(3)]
    dev = torch.device("cuda:0")
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(torch.bfloat16) for x in arrays)
    tq, tk, tv = (torch.from_numpy(x).to(dev) for x in toks)
    O, UV = ska.sinkhorn_attn_fwd_dustbin_token(Q, K, V, tq, tk, tv, w.W, w.T, w.R, w.eps)
    res = ska.sinkhorn_attn_bwd_dustbin_token(Q, K, V, tq, tk, tv, O, G, UV, w.W, w.T, w.R, w.eps)
    torch.cuda.synchronize()
    names = ("dQ", "dK", "dV", "dq_db", "dk_db", "dv_db")
    got = dict(zip(names, (x.float().cpu().numpy().astype(np.float64) for x in res)))
    got["O"] = O.float().cpu().numpy().astype(np.float64)
    b, h = 1, 2
    q, k, v, g = (x[b, h] for x in arrays)
    ref = oracle.band_dustbin_token(q, k, v, g, toks[0][b, h], toks[1][b, h], toks[2][b, h], w.W, w.T, w.R, w.eps)
    # every tensor by itself.  A token's gradient is one d-vector summed over all L spokes with
    # heavy cancellation (here |dq_db| is 0.8 against 3.5 and 3.2 for the other two): the rounding
    # floor of tests/measures.py is what bounds it, and the print says when it is used
    res = assert_per_tensor({n: got[n][b, h] for n in got}, ref, w.dtype,
                            floors(w.dtype, q, k, v, g, ref["O"], w.eps), tuple(got), where=f"dustbin tokens ({b},{h})")
    print(f"   ({b},{h}):", {n: f"{r[2]:.2e}" for n, r in res.items()}, flush=True)
    for n in ("O", "dQ", "dK", "dV", "dk_db", "dv_db"):
        assert res[n][2] <= TOL[w.dtype], (n, res[n][2])


def test_paper_scale_full_heads():
    """Both heads of the benchmark workload (262144 tokens each) against the oracle run on the
    whole head: rel-L2 over the full tensors, no windows (about a minute of CPU)."""
    w = CONFIGS["paper"]
    print(f"\n[case] {w}: both heads whole against the oracle", flush=True)
    whole_problems(w)


def test_four_million_tokens():
    """A sequence sixteen times the benchmark's (L = 2^22, a quarter of the largest L the 32-bit
    offsets inside one matrix allow), fewer base steps to keep the oracle windows small: both
    true ends and the middle against the oracle."""
    from paper_2605_08123_amd.workloads import Workload
    w = Workload("huge", 9, 1, 1, 1 << 22, 64, 256, 6, 2, 0.5, "bf16")
    print(f"\n[case] {w}", flush=True)
    arrays = make_inputs(w)
    got = run_gpu(w, arrays)
    for key in ("O", "dQ", "dK", "dV"):
        assert np.isfinite(got[key]).all(), key
    L = w.L
    window_check(w, got, arrays, 0, 0, 0, 1024)
    window_check(w, got, arrays, 0, 0, L // 2 - 500, L // 2 + 524)
    window_check(w, got, arrays, 0, 0, L - 1024, L)
