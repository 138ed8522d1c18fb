"""GPU parity on seeded random configurations: length, head dimension, window, base and tail
depth, batch, heads, storage type, eps and the dustbin drawn at random (fixed seeds, so the
cases are the same on every run), each against the fp64 CPU oracle.  The hand-picked cases of
test_gpu_parity.py sit on the tile boundaries; these fill the space between them.  The same
tolerances: rel-L2 <= 1e-4 (fp32 storage), <= 2e-2 (bf16 storage).

Measures: O and dV by their own norms; dQ and dK jointly (one norm over both), because a
configuration can leave one of them tiny next to the other.  Configurations whose score
gradient vanishes identically (window 0, a single query or key) are not drawn: they have
dedicated cases in test_gpu_parity.py.
"""
import numpy as np
import pytest

import oracle
from paper_2605_08123_amd.workloads import Workload, make_inputs

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
WINDOWS = [1, 5, 31, 32, 33, 64, 100, 255, 256, 300, 2000]


def joint(got, ref, keys):
    num = sum(np.linalg.norm(got[k] - ref[k]) ** 2 for k in keys) ** 0.5
    den = sum(np.linalg.norm(ref[k]) ** 2 for k in keys) ** 0.5
    return float(num / max(den, 1e-300))


def draw(rng, lo=8, hi=1400):
    return dict(dtype=["f32", "bf16"][int(rng.integers(2))], d=int(rng.choice([32, 64, 128])),
                L=int(rng.integers(lo, hi)), W=int(rng.choice(WINDOWS)), T=int(rng.integers(0, 7)),
                R=int(rng.integers(1, 5)), B=int(rng.integers(1, 4)), H=int(rng.integers(1, 4)),
                eps=float(rng.choice([0.5, 0.8, 1.0, 1.5])))


def on_device(c, arrays):
    import torch
    td = torch.float32 if c["dtype"] == "f32" else torch.bfloat16
    dev = torch.device("cuda:0")
    t = [torch.from_numpy(x).to(dev).to(td) for x in arrays]
    # the oracle gets the values the device holds (rounded to the storage type)
    return t, [x.float().cpu().numpy().astype(np.float64) for x in t]


def to_np(**kw):
    return {n: x.float().cpu().numpy().astype(np.float64) for n, x in kw.items()}


def worst_of(got, ref):
    return max(joint(got, ref, ["O"]), joint(got, ref, ["dV"]), joint(got, ref, ["dQ", "dK"]))


@pytest.mark.parametrize("split", [False, True])
@pytest.mark.parametrize("case", range(16))
def test_random_step(case, split):
    """One-call step (forward + backward), plain and with the scalar-score dustbin."""
    import torch

    import paper_2605_08123_amd as ska
    rng = np.random.default_rng(9100 + case)
    c = draw(rng)
    db = bool(rng.integers(4) == 0)
    score = float(rng.normal()) * 0.3
    w = Workload("random", 7, c["B"], c["H"], c["L"], c["d"], c["W"], c["T"], c["R"], c["eps"], c["dtype"],
                 dustbin=db, dustbin_score=score)
    print(f"\n[case] {w} split={split}", flush=True)
    (Q, K, V, G), rounded = on_device(c, make_inputs(w, 9200 + case))
    ska.sinkhorn_attn_set_split_min_edges(0.0 if split else 5e7)
    try:
        O, UV, dQ, dK, dV = ska.sinkhorn_attn_step(Q, K, V, G, w.W, w.T, w.R, w.eps, db, score)
        torch.cuda.synchronize()
    finally:
        ska.sinkhorn_attn_set_split_min_edges(5e7)
    got = to_np(O=O, dQ=dQ, dK=dK, dV=dV)
    ref = oracle.band_batched(*rounded, w.W, w.T, w.R, w.eps, db, score)
    e = worst_of(got, ref)
    print(f"   worst rel-L2 {e:.2e}", flush=True)
    assert all(np.isfinite(x).all() for x in got.values()) and e <= TOL[c["dtype"]], e


@pytest.mark.parametrize("case", range(10))
def test_random_lengths(case):
    """Per-item query and key lengths drawn independently in [8, L]; every fifth case also has
    an item with no queries or no keys, whose results are zero."""
    import torch

    import paper_2605_08123_amd as ska
    rng = np.random.default_rng(9300 + case)
    c = draw(rng, lo=8, hi=1100)
    B, H, L = c["B"], c["H"], c["L"]
    w = Workload("random", 7, B, H, L, c["d"], c["W"], c["T"], c["R"], c["eps"], c["dtype"])
    lq = rng.integers(8, L + 1, size=B).astype(np.int32)
    lk = rng.integers(8, L + 1, size=B).astype(np.int32)
    if case % 5 == 0:
        (lq if case % 2 else lk)[0] = 0
    print(f"\n[case] {w} lengths q={lq.tolist()} k={lk.tolist()}", flush=True)
    (Q, K, V, G), (q, k, v, g) = on_device(c, make_inputs(w, 9400 + case))
    tq, tk = (torch.from_numpy(x).to(Q.device) for x in (lq, lk))
    O, UV = ska.sinkhorn_attn_fwd_varlen(Q, K, V, None, None, tq, tk, w.W, w.T, w.R, w.eps)
    dQ, dK, dV = ska.sinkhorn_attn_bwd_varlen(Q, K, V, None, None, tq, tk, O, G, UV, w.W, w.T, w.R, w.eps)[:3]
    torch.cuda.synchronize()
    got = to_np(O=O, dQ=dQ, dK=dK, dV=dV)
    assert all(np.isfinite(x).all() for x in got.values())
    worst = 0.0
    for b in range(B):
        for h in range(H):
            a, n = int(lq[b]), int(lk[b])
            if a == 0 or n == 0:
                assert all(np.all(got[m][b, h] == 0.0) for m in got), (b, h)
                continue
            ref = oracle.band_rect(q[b, h, :a], k[b, h, :n], v[b, h, :n], g[b, h, :a], w.W, w.T, w.R, w.eps)
            mine = dict(O=got["O"][b, h, :a], dQ=got["dQ"][b, h, :a], dK=got["dK"][b, h, :n], dV=got["dV"][b, h, :n])
            worst = max(worst, worst_of(mine, ref))
            assert np.all(got["O"][b, h, a:] == 0.0) and np.all(got["dK"][b, h, n:] == 0.0)
    print(f"   worst rel-L2 {worst:.2e}", flush=True)
    assert worst <= TOL[c["dtype"]], worst


@pytest.mark.parametrize("case", range(10))
def test_random_masks(case):
    """Independent random activity masks at 5 %, 30 % or 70 % inactive tokens.  At 70 % the
    window is at least 31: in a narrower one most active rows keep a single partner, whose plan
    entry the marginal fixes, so the score gradient nearly cancels and its relative error
    measures the cancellation, not the kernels."""
    import torch

    import paper_2605_08123_amd as ska
    rng = np.random.default_rng(9500 + case)
    c = draw(rng, lo=8, hi=1100)
    B, H, L = c["B"], c["H"], c["L"]
    w = Workload("random", 7, B, H, L, c["d"], c["W"], c["T"], c["R"], c["eps"], c["dtype"])
    p = float(rng.choice([0.05, 0.3, 0.7]))
    W = max(c["W"], 31) if p == 0.7 else c["W"]
    w = Workload("random", 7, B, H, L, c["d"], W, c["T"], c["R"], c["eps"], c["dtype"])
    mq, mk = rng.random((B, L)) > p, rng.random((B, L)) > p
    print(f"\n[case] {w} inactive fraction {p}", flush=True)
    (Q, K, V, G), (q, k, v, g) = on_device(c, make_inputs(w, 9600 + case))
    tmq, tmk = (torch.from_numpy(x.astype(np.uint8)).to(Q.device) for x in (mq, mk))
    O, UV = ska.sinkhorn_attn_fwd_masked(Q, K, V, tmq, tmk, w.W, w.T, w.R, w.eps)
    dQ, dK, dV = ska.sinkhorn_attn_bwd_variant(0, Q, K, V, None, None, None, None, O, G, UV, w.W, w.T, w.R,
                                               w.eps)[:3]
    torch.cuda.synchronize()
    got = to_np(O=O, dQ=dQ, dK=dK, dV=dV)
    assert all(np.isfinite(x).all() for x in got.values())
    worst = 0.0
    for b in range(B):
        for h in range(H):
            ref = oracle.band_masked(q[b, h], k[b, h], v[b, h], g[b, h], mq[b], mk[b], w.W, w.T, w.R, w.eps)
            worst = max(worst, worst_of({m: got[m][b, h] for m in got}, ref))
    print(f"   worst rel-L2 {worst:.2e}", flush=True)
    assert worst <= TOL[c["dtype"]], worst


@pytest.mark.parametrize("case", range(8))
def test_random_learned_tokens(case):
    """Learned dustbin token per side: the six gradients, those of the tokens measured jointly
    with the ordinary ones of the same kind."""
    import torch

    import paper_2605_08123_amd as ska
    rng = np.random.default_rng(9700 + case)
    c = draw(rng, lo=40, hi=1300)
    B, H, d = c["B"], c["H"], c["d"]
    w = Workload("random", 7, B, H, c["L"], d, c["W"], c["T"], c["R"], c["eps"], c["dtype"], dustbin=True)
    toks = [rng.standard_normal((B, H, d)).astype(np.float32) * 0.7 for _ in range(3)]
    print(f"\n[case] {w} learned tokens", flush=True)
    (Q, K, V, G), (q, k, v, g) = on_device(c, make_inputs(w, 9800 + case))
    tq, tk, tv = (torch.from_numpy(x).to(Q.device) for x in toks)
    O, UV = ska.sinkhorn_attn_fwd_dustbin_token(Q, K, V, tq, tk, tv, w.W, w.T, w.R, w.eps)
    res = ska.sinkhorn_attn_bwd_dustbin_token(Q, K, V, tq, tk, tv, O, G, UV, w.W, w.T, w.R, w.eps)
    torch.cuda.synchronize()
    got = to_np(O=O, **dict(zip(("dQ", "dK", "dV", "dq_db", "dk_db", "dv_db"), res)))
    assert all(np.isfinite(x).all() for x in got.values())
    worst = 0.0
    for b in range(B):
        for h in range(H):
            ref = oracle.band_dustbin_token(q[b, h], k[b, h], v[b, h], g[b, h], toks[0][b, h], toks[1][b, h],
                                            toks[2][b, h], w.W, w.T, w.R, w.eps)
            mine = {m: got[m][b, h] for m in got}
            worst = max(worst, joint(mine, ref, ["O"]), joint(mine, ref, ["dV", "dv_db"]),
                        joint(mine, ref, ["dQ", "dK", "dq_db", "dk_db"]))
    print(f"   worst rel-L2 {worst:.2e}", flush=True)
    assert worst <= TOL[c["dtype"]], worst
