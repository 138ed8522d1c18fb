"""GPU parity on seeded random configurations: length, head dimension, window, base and tail
depth, batch, heads, storage type, eps and the dustbin drawn at random (fixed seeds, so the
cases are the same on every run), each against the fp64 CPU oracle.  The hand-picked cases of
test_gpu_parity.py sit on the tile boundaries; these fill the space between them.  The same
tolerances: rel-L2 <= 1e-4 (fp32 storage), <= 2e-2 (bf16 storage), asserted for each of O, dQ,
dK, dV (and each token gradient) by itself.  The draw includes the supports on which the score
gradient cancels structurally (window 0, 1-wide windows under heavy masks, items with a single
query or key); there, and only there, the rounding floor of tests/measures.py takes over from
the relative bar.
"""
import numpy as np
import pytest

import oracle
from paper_2605_08123_amd.workloads import Workload, make_inputs
from tests.measures import assert_per_tensor, floors, worst_ratio

pytestmark = pytest.mark.gpu

WINDOWS = [0, 1, 5, 31, 32, 33, 64, 100, 255, 256, 300, 2000]


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


def measure(got, ref, c, eps, q, k, v, g, where, names=("O", "dQ", "dK", "dV")):
    """Every tensor by itself against max(tol |ref|, rounding floor); returns the worst error / bound."""
    fl = floors(c["dtype"], q, k, v, g, ref["O"], eps)
    res = assert_per_tensor(got, ref, c["dtype"], fl, names, where)
    return worst_ratio(res), res


@pytest.mark.parametrize("split", [False, True])
@pytest.mark.parametrize("case", range(16))
def test_random_step(case, split):
    """One-call step (forward + backward), plain and with the scalar-score dustbin."""
    import torch

    import paper_2605_08123_amd as ska
    rng = np.random.default_rng(9100 + case)
    c = draw(rng)
    if case % 8 == 7:
        c["L"] = int(rng.integers(1, 5))   # every eighth case is a handful of tokens
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
    e, res = measure(got, ref, c, w.eps, *rounded, where=str(w))
    print("   rel-L2 " + " ".join(f"{n} {r[2]:.2e}" for n, r in res.items()) + f"; worst error/bound {e:.2f}", flush=True)


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
    if case % 5 == 1:
        (lq if case % 2 else lk)[B - 1] = 1   # an item with a single query or a single key
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
            worst = max(worst, measure(mine, ref, c, w.eps, q[b, h, :a], k[b, h, :n], v[b, h, :n], g[b, h, :a],
                                       where=f"{w} item {b} head {h}")[0])
            assert np.all(got["O"][b, h, a:] == 0.0) and np.all(got["dK"][b, h, n:] == 0.0)
    print(f"   worst error/bound {worst:.2f}", flush=True)


@pytest.mark.parametrize("case", range(10))
def test_random_masks(case):
    """Independent random activity masks at 5 %, 30 % or 70 % inactive tokens, any window (in a
    1-wide window under a 70 % mask most active rows keep a single partner, whose plan entry the
    marginal fixes: the score gradient nearly cancels there and the rounding floor applies)."""
    import torch

    import paper_2605_08123_amd as ska
    rng = np.random.default_rng(9500 + case)
    c = draw(rng, lo=8, hi=1100)
    B, H, L = c["B"], c["H"], c["L"]
    w = Workload("random", 7, B, H, L, c["d"], c["W"], c["T"], c["R"], c["eps"], c["dtype"])
    p = float(rng.choice([0.05, 0.3, 0.7]))
    if case >= 8:   # the two last cases: a 1-wide window under the heaviest mask
        p, w = 0.7, Workload("random", 7, B, H, L, c["d"], 1, c["T"], c["R"], c["eps"], c["dtype"])
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
            worst = max(worst, measure({m: got[m][b, h] for m in got}, ref, c, w.eps, q[b, h], k[b, h], v[b, h],
                                       g[b, h], where=f"{w} item {b} head {h}")[0])
    print(f"   worst error/bound {worst:.2f}", flush=True)


@pytest.mark.parametrize("case", range(8))
def test_random_learned_tokens(case):
    """Learned dustbin token per side: the six gradients, each by itself."""
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
            worst = max(worst, measure(mine, ref, c, w.eps, q[b, h], k[b, h], v[b, h], g[b, h],
                                       where=f"{w} item {b} head {h}",
                                       names=("O", "dQ", "dK", "dV", "dq_db", "dk_db", "dv_db"))[0])
    print(f"   worst error/bound {worst:.2f}", flush=True)
