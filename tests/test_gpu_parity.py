"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle
on the same seeded inputs.  Tolerances: rel-L2 <= 1e-4 for fp32 storage and
<= 2e-2 for bf16 storage with fp32 accumulation, on O, dQ, dK and dV.
"""
import sys

import numpy as np
import pytest

import oracle
from paper_2605_08123_amd.workloads import CONFIGS, Workload, make_inputs
from tests.measures import assert_per_tensor, floors

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, scope="module", params=["default", "two_streams"])
def stream_split(request):
    """Every case of this module runs twice: with the library's own choice (cases this small stay
    on one stream) and with the split onto the helper stream forced for every call on two or more
    problems."""
    import paper_2605_08123_amd as ska
    ska.sinkhorn_attn_set_split_min_edges(0.0 if request.param == "two_streams" else 5e7)
    yield request.param
    ska.sinkhorn_attn_set_split_min_edges(5e7)

TOL = {"f32": 1e-4, "bf16": 2e-2}


def rel(a, b):
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def run_gpu(w: Workload, arrays, want_eta0=False, one_call=False):
    """Forward then backward (two calls), or the one-call step the benchmark times."""
    import torch

    import paper_2605_08123_amd as ska
    dev = torch.device("cuda:0")
    td = torch.float32 if w.dtype == "f32" else torch.bfloat16
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(td) for x in arrays)
    if one_call:
        O, UV, *res = ska.sinkhorn_attn_step(Q, K, V, G, w.W, w.T, w.R, w.eps, w.dustbin, w.dustbin_score,
                                             want_eta0=want_eta0)
    else:
        O, UV = ska.sinkhorn_attn_fwd(Q, K, V, w.W, w.T, w.R, w.eps, w.dustbin, w.dustbin_score)
        res = ska.sinkhorn_attn_bwd(Q, K, V, O, G, UV, w.W, w.T, w.R, w.eps, w.dustbin, w.dustbin_score,
                                    want_eta0=want_eta0)
    torch.cuda.synchronize()
    out = dict(O=O, UV=UV, dQ=res[0], dK=res[1], dV=res[2])
    if want_eta0:
        out["eta0"] = res[3]
    return {k: v.float().cpu().numpy().astype(np.float64) for k, v in out.items()}


def check(w: Workload, seed=None, want_eta0=False, uv_atol=None):
    print(f"\n[case] {w}", flush=True)
    sys.stdout.flush()
    arrays = make_inputs(w, seed)
    got = run_gpu(w, arrays, want_eta0)
    ref = oracle.band_batched(*arrays, w.W, w.T, w.R, w.eps, w.dustbin, w.dustbin_score)
    # every tensor by itself; where the reference vanishes by cancellation (W = 0 gives
    # dQ = dK = 0) the rounding floor of tests/measures.py takes over from the relative bar
    res = assert_per_tensor(got, ref, w.dtype, floors(w.dtype, *arrays, ref["O"], w.eps), where=w.name)
    print("   rel-L2:", {k: f"{r[2]:.2e}" for k, r in res.items()}, flush=True)
    # potentials: both sides iterate the same ungauged map from v = 0, so the raw
    # vectors agree; compared through the gauge-free sums u^(t) + v^(t)
    # (bf16 storage: the score scale is folded into a bf16 copy of Q, which perturbs every
    # score by a relative 2^-9; the potentials absorb that as an absolute error ~1e-2)
    uv_atol = uv_atol or (2e-4 if w.dtype == "f32" else 2e-2)
    for t in range(1 if w.T == 0 else 0, w.R + 1):
        s_got = got["UV"][:, :, 2 * t] + got["UV"][:, :, 2 * t + 1]
        s_ref = ref["UV"][:, :, 2 * t] + ref["UV"][:, :, 2 * t + 1]
        assert np.abs(s_got - s_ref).max() < uv_atol, (t, np.abs(s_got - s_ref).max())
    return got, ref


def small(name, L, d, W, T, dtype, eps=1.0, B=1, H=1, R=2, **kw):
    return Workload(name, 7, B, H, L, d, W, T, R, eps, dtype, **kw)


def test_tiny_config_fp32():
    check(CONFIGS["tiny"])


@pytest.mark.parametrize("L,d,W,T", [
    (300, 32, 16, 8),      # ragged tail, several tiles
    (77, 64, 5, 3),        # shorter than one workgroup tile
    (257, 32, 0, 4),       # W = 0: identity plan
    (130, 64, 1000, 6),    # W >= L-1: dense
    (1, 32, 3, 2),         # single token
    (200, 128, 33, 5),     # d = 128, W not a multiple of the tile
    (96, 32, 40, 0),       # T = 0: tail starts from v = 0
    (513, 64, 256, 4),     # W on a tile boundary
])
def test_fp32_edge_shapes(L, d, W, T):
    check(small("edge", L, d, W, T, "f32", B=1, H=2), seed=L + W)


def test_fp32_w0_is_identity():
    w = small("w0", 257, 32, 0, 4, "f32")
    got, _ = check(w, seed=3)
    _, _, v, g = make_inputs(w, 3)
    assert np.abs(got["O"] - v).max() < 1e-5 and np.abs(got["dV"] - g).max() < 1e-5
    # dQ = dK = 0 exactly; what the kernels return is bounded by the rounding floor inside check()
    # (8 * 2^-24 * c * |(|dO_i| |O_i|)_i| * max|K_j|, Frobenius norm over the whole tensor)


@pytest.mark.parametrize("L,d,W,T,eps", [
    (1000, 64, 100, 10, 0.5),
    (700, 32, 64, 6, 1.0),
    (300, 128, 50, 5, 1.0),
    (2048, 64, 256, 20, 0.5),
])
def test_bf16_shapes(L, d, W, T, eps):
    check(small("bf16", L, d, W, T, "bf16", eps=eps, B=2, H=1), seed=L)


def test_mid_config_slice():
    """Mid configuration, two of its 32 (batch, head) problems."""
    check(CONFIGS["mid"].scaled(B=1, H=2))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_dustbin_small(dtype):
    w = small("db", 600, 64, 48, 8, dtype, eps=0.7, B=1, H=2, dustbin=True, dustbin_score=0.3)
    check(w, seed=11)


def test_dustbin_config_slice():
    """Dustbin configuration (alphabet embeddings), one problem at L = 4096."""
    check(CONFIGS["dustbin"].scaled(B=1, H=1, L=4096))


@pytest.mark.parametrize("R", [1, 3, 4])
@pytest.mark.parametrize("dtype,d", [("f32", 32), ("bf16", 64), ("bf16", 128)])
def test_tail_depth(R, dtype, d):
    """Tail depths other than the paper's R = 2 (Prop. 1 holds for any R): 2R rank-1 modifier
    terms in the final sweeps, 2R - 1 mat-vecs in the reverse chain."""
    check(small("tail", 520, d, 37, 5, dtype, eps=0.8, B=1, H=2, R=R), seed=40 + R)


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 64)])
def test_deep_tail_is_full_backprop(dtype, d):
    """T = 0 with a deep tail: nothing is stopped, the backward is full backpropagation through
    the whole solve (the final sweeps take the 2R modifier terms eight at a time)."""
    check(small("deep", 400, d, 30, 0, dtype, eps=0.8, B=1, H=2, R=7), seed=77)


def test_bias_certificate_by_difference():
    """The stopped-base bias D_x z_T^T eta_R (a-posteriori certificate) is the difference of two
    backward calls: (T = 0, R = T' + R') minus (T', R')."""
    T, R = 4, 2
    w_full = small("full", 300, 32, 20, 0, "f32", eps=0.8, R=T + R)
    w_stop = small("stop", 300, 32, 20, T, "f32", eps=0.8, R=R)
    arrays = make_inputs(w_full, 5)
    g_full, g_stop = run_gpu(w_full, arrays), run_gpu(w_stop, arrays)
    o_full = oracle.band_batched(*arrays, w_full.W, 0, T + R, w_full.eps)
    o_stop = oracle.band_batched(*arrays, w_stop.W, T, R, w_stop.eps)
    assert np.abs(g_full["O"] - g_stop["O"]).max() < 1e-5        # the same forward
    for k in ("dQ", "dK"):
        gap, ref = g_full[k] - g_stop[k], o_full[k] - o_stop[k]
        assert np.linalg.norm(ref) > 1e-4 * np.linalg.norm(o_stop[k])      # there is a bias to certify
        assert rel(gap, ref) < 5e-3, (k, rel(gap, ref))
    assert np.abs(g_full["dV"] - g_stop["dV"]).max() < 1e-4      # V does not enter the base solve


@pytest.mark.parametrize("dtype,d,kind", [("f32", 32, "plain"), ("bf16", 64, "plain"), ("f32", 64, "marginals"),
                                          ("f32", 32, "dustbin"), ("bf16", 128, "plain")])
def test_base_vjp_is_the_stopped_bias(dtype, d, kind):
    """One call gives the certificate's D_x z_T^T eta_R: eta_R is the backward's eta0, the base
    iterates come from a (T = 0, R = T) forward.  Reference: the oracle's full backpropagation
    (T = 0, R = T + R) minus its stopped-base backward, in fp64."""
    import torch

    import paper_2605_08123_amd as ska
    T, R = 5, 2
    db = kind == "dustbin"
    w = small("cert", 400, d, 24, T, dtype, eps=0.8, B=1, H=2, R=R, dustbin=db, dustbin_score=-0.3)
    print(f"\n[case] {w} base VJP ({kind})", flush=True)
    arrays = make_inputs(w, 9)
    la = lb = None
    if kind == "marginals":
        la, lb = _targets(w, 10)
    dev = torch.device("cuda:0")
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(td) for x in arrays)
    tla = torch.from_numpy(la).to(dev) if la is not None else None
    tlb = torch.from_numpy(lb).to(dev) if lb is not None else None
    O, UV = ska.sinkhorn_attn_fwd_marginals(Q, K, V, tla, tlb, w.W, T, R, w.eps, db, w.dustbin_score)
    _, _, _, eta = ska.sinkhorn_attn_bwd_marginals(Q, K, V, tla, tlb, O, G, UV, w.W, T, R, w.eps, db,
                                                   w.dustbin_score, want_eta0=True)
    _, UVb = ska.sinkhorn_attn_fwd_marginals(Q, K, V, tla, tlb, w.W, 0, T, w.eps, db, w.dustbin_score)
    assert torch.equal(UVb[:, :, 2 * T + 1], UV[:, :, 1])          # the same base state, bit for bit
    eQ, eK = ska.sinkhorn_attn_base_vjp(Q, K, UVb, eta, w.W, T, w.eps, db, w.dustbin_score, tla, tlb)
    torch.cuda.synchronize()
    kw = dict(log_a=None if la is None else la.astype(np.float64), log_b=None if lb is None else lb.astype(np.float64))
    o_full = oracle.band_batched(*arrays, w.W, 0, T + R, w.eps, db, w.dustbin_score, **kw)
    o_stop = oracle.band_batched(*arrays, w.W, T, R, w.eps, db, w.dustbin_score, **kw)
    tol = TOL[dtype]
    for name, got in (("dQ", eQ), ("dK", eK)):
        ref = o_full[name] - o_stop[name]
        e = rel(got.float().cpu().numpy().astype(np.float64), ref)
        print(f"   bias {name}: |ref| {np.linalg.norm(ref):.3e} of |grad| {np.linalg.norm(o_stop[name]):.3e}, "
              f"rel-L2 {e:.2e}", flush=True)
        assert np.linalg.norm(ref) > 1e-5 * np.linalg.norm(o_stop[name])
        assert e < tol, (name, e)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_certified_tail_depth_selection(seed):
    """Cor. 'Certified Tail-Depth Selection' on a setting shaped like the paper's certificate table
    (L = 128, T = 15, band covering the whole problem, eps = 1): the certificate max|e_R| of every
    depth against the oracle's full-minus-stopped gap, its decay with R, the depth chosen for a
    tolerance placed between two depths, and the guarantee itself -- the returned gradient is
    within tau (plus fp32 noise) of the oracle's full backpropagation."""
    import torch

    import paper_2605_08123_amd as ska
    T, Rmax = 15, 4
    w = small("table2", 128, 32, 128, T, "f32", eps=1.0, B=1, H=1, R=Rmax)
    print(f"\n[case] {w} seed {seed}: certified selector", flush=True)
    arrays = make_inputs(w, seed)
    dev = torch.device("cuda:0")
    Q, K, V, G = (torch.from_numpy(x).to(dev) for x in arrays)
    full = {R: oracle.band_batched(*arrays, w.W, 0, T + R, w.eps) for R in range(1, Rmax + 1)}
    stop = {R: oracle.band_batched(*arrays, w.W, T, R, w.eps) for R in range(1, Rmax + 1)}
    gap = [max(np.abs(full[R][k] - stop[R][k]).max() for k in ("dQ", "dK")) for R in range(1, Rmax + 1)]
    allr = ska.sinkhorn_attn_select_tail_depth(Q, K, V, G, w.W, T, Rmax, 0.0, w.eps)     # tau = 0: try every depth
    print("   max|e_R|  gpu:", [f"{x:.3e}" for x in allr["e_absmax"]], flush=True)
    print("   max|e_R|  ref:", [f"{x:.3e}" for x in gap], flush=True)
    print("   max|eta_R| gpu:", [f"{x:.3e}" for x in allr["eta_absmax"]], flush=True)
    assert allr["R"] == 0 and len(allr["e_absmax"]) == Rmax
    scale = max(np.abs(stop[1][k]).max() for k in ("dQ", "dK"))
    for R in range(1, Rmax + 1):
        assert abs(allr["e_absmax"][R - 1] - gap[R - 1]) <= 0.02 * gap[R - 1] + 2e-6 * scale, R
    assert all(gap[k + 1] < 0.5 * gap[k] for k in range(2))          # the bias falls with the depth
    assert all(allr["eta_absmax"][k + 1] < 0.5 * allr["eta_absmax"][k] for k in range(2))
    tau = float(np.sqrt(gap[0] * gap[1]))                            # between depth 1 and depth 2
    sel = ska.sinkhorn_attn_select_tail_depth(Q, K, V, G, w.W, T, Rmax, tau, w.eps)
    assert sel["R"] == 2 and len(sel["e_absmax"]) == 2 and sel["e_absmax"][1] <= tau < sel["e_absmax"][0]
    for k in ("dQ", "dK", "dV"):
        got = sel[k].cpu().numpy().astype(np.float64)
        assert rel(got, stop[2][k]) < TOL["f32"], k                  # the stopped gradient of depth 2
        assert np.abs(got - full[2][k]).max() <= tau + 1e-5 * scale, k   # ... certified against full BPTT
    O2, UV2 = ska.sinkhorn_attn_fwd(Q, K, V, w.W, T, 2, w.eps)
    assert torch.equal(sel["O"], O2) and torch.equal(sel["UV"], UV2)


@pytest.mark.parametrize("dtype,d,R,kind", [("f32", 32, 2, "plain"), ("bf16", 64, 2, "plain"), ("bf16", 128, 3, "plain"),
                                            ("f32", 64, 1, "marginals"), ("bf16", 32, 5, "plain"),
                                            ("f32", 32, 2, "dustbin")])
def test_backward_variants(dtype, d, R, kind):
    """The comparators of the final sweeps -- every staircase factor by its own exponential
    (direct; Prop. 1 as it stands) and Prop. 2 on the generic kernel -- against the oracle to
    the same tolerance as the production path; their dV and eta0 are the production path's."""
    import torch

    import paper_2605_08123_amd as ska
    from paper_2605_08123_amd.binding import SKA_BWD_DIRECT, SKA_BWD_ONE_REFERENCE_GENERIC
    db = kind == "dustbin"
    w = small("variants", 450, d, 29, 4, dtype, eps=0.8, B=1, H=2, R=R, dustbin=db, dustbin_score=0.2)
    print(f"\n[case] {w} backward variants ({kind})", flush=True)
    arrays = make_inputs(w, 13)
    la = lb = None
    if kind == "marginals":
        la, lb = _targets(w, 14)
    dev = torch.device("cuda:0")
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(td) for x in arrays)
    tla = torch.from_numpy(la).to(dev) if la is not None else None
    tlb = torch.from_numpy(lb).to(dev) if lb is not None else None
    O, UV = ska.sinkhorn_attn_fwd_marginals(Q, K, V, tla, tlb, w.W, w.T, R, w.eps, db, w.dustbin_score)
    prod = ska.sinkhorn_attn_bwd_marginals(Q, K, V, tla, tlb, O, G, UV, w.W, w.T, R, w.eps, db, w.dustbin_score,
                                           want_eta0=True)
    kw = dict(log_a=None if la is None else la.astype(np.float64), log_b=None if lb is None else lb.astype(np.float64))
    ref = oracle.band_batched(*arrays, w.W, w.T, R, w.eps, db, w.dustbin_score, **kw)
    for variant in (SKA_BWD_DIRECT, SKA_BWD_ONE_REFERENCE_GENERIC):
        got = ska.sinkhorn_attn_bwd_variant(variant, Q, K, V, tla, tlb, None, None, O, G, UV, w.W, w.T, R, w.eps,
                                            db, w.dustbin_score, want_eta0=True)
        torch.cuda.synchronize()
        errs = {n: rel(x.float().cpu().numpy().astype(np.float64), ref[n]) for n, x in zip(("dQ", "dK", "dV"), got)}
        print(f"   variant {variant} rel-L2:", {n: f"{e:.2e}" for n, e in errs.items()}, flush=True)
        for n, e in errs.items():
            assert e <= TOL[dtype], (variant, n, e)
        assert torch.equal(got[2], prod[2]) and torch.equal(got[3], prod[3])
    with pytest.raises(ska.SinkhornAttnError) as e:
        ska.sinkhorn_attn_bwd_variant(7, Q, K, V, tla, tlb, None, None, O, G, UV, w.W, w.T, R, w.eps, db,
                                      w.dustbin_score)
    assert e.value.status == -1


@pytest.mark.parametrize("dtype,d,kind", [("f32", 32, "plain"), ("bf16", 64, "plain"), ("f32", 64, "dustbin"),
                                          ("bf16", 128, "marginals")])
def test_eps_schedule_in_the_base_solve(dtype, d, kind):
    """Continuation schedule (remark 'Fixed-Budget eps-Scaling'): forward with three stages, the
    ordinary backward on its UV, against the oracle's scheduled solve; a single stage at eps is
    the plain forward bit for bit."""
    import torch

    import paper_2605_08123_amd as ska
    stages, steps, eps, R = [1.6, 0.8, 0.4], [3, 2, 4], 0.4, 2
    db = kind == "dustbin"
    w = small("sched", 500, d, 27, sum(steps), dtype, eps=eps, B=1, H=2, R=R, dustbin=db, dustbin_score=0.3)
    print(f"\n[case] {w} eps schedule {stages} x {steps} ({kind})", flush=True)
    arrays = make_inputs(w, 17)
    la = lb = None
    if kind == "marginals":
        la, lb = _targets(w, 18)
    dev = torch.device("cuda:0")
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(td) for x in arrays)
    tla = torch.from_numpy(la).to(dev) if la is not None else None
    tlb = torch.from_numpy(lb).to(dev) if lb is not None else None
    O, UV = ska.sinkhorn_attn_fwd_eps_schedule(Q, K, V, w.W, stages, steps, R, eps, db, w.dustbin_score, tla, tlb)
    dQ, dK, dV = ska.sinkhorn_attn_bwd_marginals(Q, K, V, tla, tlb, O, G, UV, w.W, w.T, R, eps, db, w.dustbin_score)
    torch.cuda.synchronize()
    got = {n: x.float().cpu().numpy().astype(np.float64) for n, x in dict(O=O, dQ=dQ, dK=dK, dV=dV).items()}
    worst = dict.fromkeys(got, 0.0)
    for h in range(w.H):
        q, k, v, g = (x[0, h] for x in arrays)
        ref = oracle.band_eps_schedule(q, k, v, g, w.W, stages, steps, R, eps, db, w.dustbin_score,
                                       log_a=None if la is None else la[0, h].astype(np.float64),
                                       log_b=None if lb is None else lb[0, h].astype(np.float64))
        plain = oracle.band(q, k, v, g, w.W, w.T, R, eps, db, w.dustbin_score,
                            log_a=None if la is None else la[0, h].astype(np.float64),
                            log_b=None if lb is None else lb[0, h].astype(np.float64))
        if dtype == "f32":      # the schedule matters on this input: far outside the tolerance of the plain solve
            assert rel(plain["O"], ref["O"]) > 10 * TOL[dtype]
        for n in got:
            worst[n] = max(worst[n], rel(got[n][0, h], ref[n]))
        vb = UV[0, h, 1].cpu().numpy().astype(np.float64)
        assert np.abs(vb - ref["v_base"]).max() < (5e-4 if dtype == "f32" else 5e-2)
    print("   rel-L2:", {n: f"{e:.2e}" for n, e in worst.items()}, flush=True)
    for n, e in worst.items():
        assert e <= TOL[dtype], (n, e)
    O1, UV1 = ska.sinkhorn_attn_fwd_eps_schedule(Q, K, V, w.W, [eps], [w.T], R, eps, db, w.dustbin_score, tla, tlb)
    O0, UV0 = ska.sinkhorn_attn_fwd_marginals(Q, K, V, tla, tlb, w.W, w.T, R, eps, db, w.dustbin_score)
    assert torch.equal(O1, O0) and torch.equal(UV1, UV0)


@pytest.mark.parametrize("dtype,d,R,L", [("f32", 32, 2, 300), ("bf16", 64, 2, 1500), ("bf16", 128, 2, 700),
                                         ("f32", 64, 3, 2100), ("bf16", 32, 1, 333)])
def test_learned_dustbin_tokens(dtype, d, R, L):
    """Learned dustbin token per side (Sec. 'Single-Active-Dustbin Bridge') on the sparse-spoke
    support: O, dQ, dK, dV and the gradients of the three tokens against the oracle's augmented
    problem; zero tokens reproduce the scalar-score dustbin with score 0."""
    import torch

    import paper_2605_08123_amd as ska
    w = small("token", L, d, 31, 5, dtype, eps=0.8, B=1, H=2, R=R, dustbin=True)
    print(f"\n[case] {w} learned dustbin tokens", flush=True)
    arrays = make_inputs(w, 23)
    rng = np.random.default_rng(24)
    toks = [rng.standard_normal((1, w.H, d)).astype(np.float32) for _ in range(3)]
    dev = torch.device("cuda:0")
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(td) for x in arrays)
    tq, tk, tv = (torch.from_numpy(x).to(dev) for x in toks)
    O, UV = ska.sinkhorn_attn_fwd_dustbin_token(Q, K, V, tq, tk, tv, w.W, w.T, R, w.eps)
    res = ska.sinkhorn_attn_bwd_dustbin_token(Q, K, V, tq, tk, tv, O, G, UV, w.W, w.T, R, w.eps)
    torch.cuda.synchronize()
    names = ("dQ", "dK", "dV", "dq_db", "dk_db", "dv_db")
    got = dict(zip(names, (x.float().cpu().numpy().astype(np.float64) for x in res)))
    got["O"] = O.float().cpu().numpy().astype(np.float64)
    worst = dict.fromkeys(got, 0.0)
    for h in range(w.H):
        q, k, v, g = (x[0, h] for x in arrays)
        ref = oracle.band_dustbin_token(q, k, v, g, toks[0][0, h], toks[1][0, h], toks[2][0, h], w.W, w.T, R, w.eps)
        for n in got:
            worst[n] = max(worst[n], rel(got[n][0, h], ref[n]))
        s_got = (UV[0, h, 2 * R] + UV[0, h, 2 * R + 1]).cpu().numpy().astype(np.float64)
        assert np.abs(s_got - (ref["UV"][2 * R] + ref["UV"][2 * R + 1])).max() < (2e-4 if dtype == "f32" else 3e-2)
    print("   rel-L2:", {n: f"{e:.2e}" for n, e in worst.items()}, flush=True)
    for n, e in worst.items():
        assert np.isfinite(got[n]).all() and e <= TOL[dtype], (n, e)
    z = torch.zeros_like(tq)
    Oz, UVz = ska.sinkhorn_attn_fwd_dustbin_token(Q, K, V, z, z, z, w.W, w.T, R, w.eps)
    Os, UVs = ska.sinkhorn_attn_fwd(Q, K, V, w.W, w.T, R, w.eps, True, 0.0)
    assert torch.equal(Oz, Os) and (UVz - UVs).abs().max().item() < 1e-5
    gz = ska.sinkhorn_attn_bwd_dustbin_token(Q, K, V, z, z, z, Oz, G, UVz, w.W, w.T, R, w.eps)
    gs = ska.sinkhorn_attn_bwd(Q, K, V, Os, G, UVs, w.W, w.T, R, w.eps, True, 0.0)
    for a, b in zip(gz[:3], gs):
        assert rel(a.float().cpu().numpy().astype(np.float64), b.float().cpu().numpy().astype(np.float64)) < 1e-5


@pytest.mark.parametrize("dtype,d,R,variant", [("f32", 32, 2, 0), ("bf16", 64, 2, 0), ("bf16", 128, 2, 0),
                                               ("f32", 64, 3, 0), ("bf16", 64, 2, 1), ("bf16", 32, 1, 0)])
def test_inactive_tokens(dtype, d, R, variant):
    """Boolean activity per token on both sides (the masked half-steps of Eq. 1-2): random masks,
    a run of masked keys wider than the band (so some active queries lose every partner), a
    whole masked block, per batch item.  The ordinary backward runs on the forward's UV."""
    import torch

    import paper_2605_08123_amd as ska
    w = small("masks", 900, d, 21, 5, dtype, eps=0.8, B=2, H=2, R=R)
    print(f"\n[case] {w} inactive tokens (backward variant {variant})", flush=True)
    arrays = make_inputs(w, 51)
    rng = np.random.default_rng(52)
    mq = (rng.random((w.B, w.L)) > 0.2)
    mk = (rng.random((w.B, w.L)) > 0.2)
    mk[0, 100:160] = False           # wider than 2W + 1: queries 121..138 lose every key
    mq[0, 125] = True
    mq[1, 256:540] = False           # more than a whole workgroup of inactive queries
    mk[1, 300:500] = False
    dev = torch.device("cuda:0")
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(td) for x in arrays)
    tmq, tmk = (torch.from_numpy(x.astype(np.uint8)).to(dev) for x in (mq, mk))
    O, UV = ska.sinkhorn_attn_fwd_masked(Q, K, V, tmq, tmk, w.W, w.T, R, w.eps)
    dQ, dK, dV, eta0 = ska.sinkhorn_attn_bwd_variant(variant, Q, K, V, None, None, None, None, O, G, UV, w.W, w.T, R,
                                                     w.eps, want_eta0=True)
    torch.cuda.synchronize()
    got = {n: x.float().cpu().numpy().astype(np.float64) for n, x in dict(O=O, dQ=dQ, dK=dK, dV=dV).items()}
    uv = UV.cpu().numpy().astype(np.float64)
    assert np.isfinite(eta0.cpu().numpy()).all()
    worst = dict.fromkeys(got, 0.0)
    for b in range(w.B):
        for h in range(w.H):
            q, k, v, g = (x[b, h] for x in arrays)
            ref = oracle.band_masked(q, k, v, g, mq[b], mk[b], w.W, w.T, R, w.eps)
            dead_q, dead_k = np.isneginf(ref["U"][R]), np.isneginf(ref["Vp"][R])
            assert dead_q[125] if b == 0 else dead_q[300]
            for n in got:
                assert np.isfinite(got[n][b, h]).all(), n
                worst[n] = max(worst[n], rel(got[n][b, h], ref[n]))
            assert np.all(got["O"][b, h][dead_q] == 0.0) and np.all(got["dQ"][b, h][dead_q] == 0.0)
            assert np.all(got["dK"][b, h][dead_k] == 0.0) and np.all(got["dV"][b, h][dead_k] == 0.0)
            for t in range(R + 1):
                assert np.array_equal(np.isneginf(uv[b, h, 2 * t]), dead_q)
                assert np.array_equal(np.isneginf(uv[b, h, 2 * t + 1]), dead_k)
            tol_uv = 2e-4 if dtype == "f32" else 3e-2
            assert np.abs(uv[b, h, 2 * R][~dead_q] - ref["U"][R][~dead_q]).max() < tol_uv
            assert np.abs(uv[b, h, 2 * R + 1][~dead_k] - ref["Vp"][R][~dead_k]).max() < tol_uv
    print("   worst rel-L2:", {n: f"{e:.2e}" for n, e in worst.items()}, flush=True)
    for n, e in worst.items():
        assert e <= TOL[dtype], (n, e)
    if variant == 0 and dtype == "f32":   # all-active masks are the plain call (one half-step runs on
        one = torch.ones_like(tmq)        # another kernel, so to rounding, not bit for bit)
        O1, UV1 = ska.sinkhorn_attn_fwd_masked(Q, K, V, one, one, w.W, w.T, R, w.eps)
        O0, UV0 = ska.sinkhorn_attn_fwd(Q, K, V, w.W, w.T, R, w.eps)
        assert torch.allclose(O1, O0, rtol=1e-4, atol=1e-5) and torch.allclose(UV1, UV0, rtol=1e-5, atol=1e-4)


def test_forward_backward_replay_from_a_hip_graph():
    """The calls only launch kernels on the caller's stream (no allocation, no memset, no host
    synchronisation), so a forward + backward pair can be captured into a HIP graph.  Three
    replays, with eager work and synchronisations between them, each against the eager result."""
    import torch

    import paper_2605_08123_amd as ska
    w = small("graph", 3000, 64, 40, 6, "bf16", eps=0.7, B=2, H=2)
    print(f"\n[case] {w} graph replay", flush=True)
    dev = torch.device("cuda:0")
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(torch.bfloat16) for x in make_inputs(w, 61))
    O, dQ, dK, dV = (torch.empty_like(Q) for _ in range(4))
    UV = torch.empty((w.B, w.H, 6, w.L), device=dev, dtype=torch.float32)
    ws = torch.empty(ska.sinkhorn_attn_workspace_bytes(w.B, w.H, w.L, w.d, w.W, w.T, w.R, False, 1), device=dev,
                     dtype=torch.uint8)

    def run():
        ska.sinkhorn_attn_fwd(Q, K, V, w.W, w.T, w.R, w.eps, O=O, UV=UV, workspace=ws)
        ska.sinkhorn_attn_bwd(Q, K, V, O, G, UV, w.W, w.T, w.R, w.eps, workspace=ws, dQ=dQ, dK=dK, dV=dV)

    run()
    torch.cuda.synchronize()
    want = [x.clone() for x in (O, UV, dQ, dK, dV)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run()
    for rep in range(3):
        for x in (O, UV, dQ, dK, dV):
            x.zero_()                           # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((O, UV, dQ, dK, dV), want):
            assert torch.equal(got, ref), rep


@pytest.mark.parametrize("dtype,d", [("f32", 32), ("bf16", 64)])
def test_degenerate_lengths_and_masks(dtype, d):
    """Items with no query, no key, lengths beyond L (clamped), a fully masked item and a
    single active pair: everything outside the problem is zero, nothing is NaN, and the
    ordinary item next to them is unaffected."""
    import torch

    import paper_2605_08123_amd as ska
    w = small("degenerate", 300, d, 17, 4, dtype, eps=0.9, B=4, H=1)
    print(f"\n[case] {w} degenerate lengths and masks", flush=True)
    arrays = make_inputs(w, 71)
    dev = torch.device("cuda:0")
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(td) for x in arrays)
    lq = torch.tensor([0, 300, 5000, 123], dtype=torch.int32, device=dev)      # item 2: clamped to L
    lk = torch.tensor([300, 0, 300, -7], dtype=torch.int32, device=dev)        # item 3: negative -> 0
    O, UV = ska.sinkhorn_attn_fwd_varlen(Q, K, V, None, None, lq, lk, w.W, w.T, w.R, w.eps)
    dQ, dK, dV = ska.sinkhorn_attn_bwd_varlen(Q, K, V, None, None, lq, lk, O, G, UV, w.W, w.T, w.R, w.eps)
    O0, UV0 = ska.sinkhorn_attn_fwd(Q[2:3], K[2:3], V[2:3], w.W, w.T, w.R, w.eps)
    g0 = ska.sinkhorn_attn_bwd(Q[2:3], K[2:3], V[2:3], O0, G[2:3], UV0, w.W, w.T, w.R, w.eps)
    torch.cuda.synchronize()
    for x in (O, UV, dQ, dK, dV):
        assert torch.isfinite(x).all()
    for b in (0, 1, 3):
        assert all(float(x[b].abs().max()) == 0.0 for x in (O, UV, dQ, dK, dV)), b
    assert torch.equal(O[2:3], O0) and all(torch.equal(x[2:3], y) for x, y in zip((dQ, dK, dV), g0))
    # masks: item 0 fully inactive, item 1 one active pair inside the band, item 2 one pair outside it
    mq = torch.zeros((4, 300), dtype=torch.uint8, device=dev)
    mk = torch.zeros((4, 300), dtype=torch.uint8, device=dev)
    mq[1, 40] = mk[1, 50] = 1
    mq[2, 40] = mk[2, 90] = 1
    mq[3], mk[3] = 1, 1
    O, UV = ska.sinkhorn_attn_fwd_masked(Q, K, V, mq, mk, w.W, w.T, w.R, w.eps)
    dQ, dK, dV = ska.sinkhorn_attn_bwd(Q, K, V, O, G, UV, w.W, w.T, w.R, w.eps)
    torch.cuda.synchronize()
    for x in (O, dQ, dK, dV):
        assert torch.isfinite(x).all()
    for b in (0, 2):
        assert all(float(x[b].abs().max()) == 0.0 for x in (O, dQ, dK, dV)) and bool(torch.isneginf(UV[b]).all())
    # a single edge: the plan is the 1 x 1 matrix [1], so O_40 = V_50, dV_50 = dO_40, dQ = dK = 0
    assert torch.allclose(O[1, 0, 40].float(), V[1, 0, 50].float(), rtol=1e-2, atol=1e-5)
    assert torch.allclose(dV[1, 0, 50].float(), G[1, 0, 40].float(), rtol=1e-2, atol=1e-5)
    assert float(dQ[1].abs().max()) < 1e-4 * float(G.float().abs().max()) + 1e-6
    assert float(O[1, 0, :40].abs().max()) == 0.0 and float(O[1, 0, 41:].abs().max()) == 0.0
    O3, UV3 = ska.sinkhorn_attn_fwd(Q[3:4], K[3:4], V[3:4], w.W, w.T, w.R, w.eps)
    assert torch.allclose(O[3:4].float(), O3.float(), rtol=2e-2 if dtype == "bf16" else 1e-4, atol=1e-2 if dtype == "bf16" else 1e-5)


@pytest.mark.parametrize("dtype,d,kind", [("f32", 32, "plain"), ("bf16", 64, "plain"), ("bf16", 64, "dustbin"),
                                          ("f32", 64, "marginals"), ("bf16", 128, "varlen")])
def test_step_is_forward_then_backward(dtype, d, kind):
    """The one-call step (forward + backward for a given cotangent) gives the results of the two
    separate calls: O, UV, dV bit for bit; dQ, dK, eta0 bit for bit with the dustbin and to rounding
    without it (the step takes g_u = <dO, O> from the output map's fp32 accumulators, the backward
    call from the stored O)."""
    import torch

    import paper_2605_08123_amd as ska
    db = kind == "dustbin"
    w = small("step", 700, d, 33, 5, dtype, eps=0.8, B=2, H=2, dustbin=db, dustbin_score=0.1)
    print(f"\n[case] {w} one-call step ({kind})", flush=True)
    arrays = make_inputs(w, 81)
    dev = torch.device("cuda:0")
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(td) for x in arrays)
    la = lb = lq = lk = None
    if kind == "marginals":
        la, lb = (torch.from_numpy(x).to(dev) for x in _targets(w, 82))
    if kind == "varlen":
        lq = torch.tensor([700, 333], dtype=torch.int32, device=dev)
        lk = torch.tensor([512, 700], dtype=torch.int32, device=dev)
    O, UV, dQ, dK, dV, eta = ska.sinkhorn_attn_step(Q, K, V, G, w.W, w.T, w.R, w.eps, db, w.dustbin_score, la, lb, lq,
                                                    lk, want_eta0=True)
    O0, UV0 = ska.sinkhorn_attn_fwd_varlen(Q, K, V, la, lb, lq, lk, w.W, w.T, w.R, w.eps, db, w.dustbin_score)
    g0 = ska.sinkhorn_attn_bwd_varlen(Q, K, V, la, lb, lq, lk, O0, G, UV0, w.W, w.T, w.R, w.eps, db, w.dustbin_score,
                                      want_eta0=True)
    torch.cuda.synchronize()
    assert torch.equal(O, O0) and torch.equal(UV, UV0)
    for name, x, y in zip(("dQ", "dK", "dV", "eta0"), (dQ, dK, dV, eta), g0):
        if db or name == "dV":
            assert torch.equal(x, y), name
        else:
            num, den = (x.float() - y.float()).norm().item(), y.float().norm().item()
            assert num <= (1e-5 if dtype == "f32" else 1e-2) * den, (name, num / den)


def test_caller_streams_and_ordering():
    """Work is ordered on the caller's stream whichever it is: results on a side stream of the
    caller equal those on the default stream, and a consumer enqueued on that stream right after
    the call (no host synchronisation) sees the finished output -- also when the library spreads
    the sweeps over its helper stream."""
    import torch

    import paper_2605_08123_amd as ska
    w = small("streams", 2000, 64, 30, 5, "bf16", eps=0.7, B=2, H=2)
    print(f"\n[case] {w} caller streams", flush=True)
    dev = torch.device("cuda:0")
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(torch.bfloat16) for x in make_inputs(w, 91))
    O0, UV0, dQ0, dK0, dV0 = ska.sinkhorn_attn_step(Q, K, V, G, w.W, w.T, w.R, w.eps)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    for rep in range(3):
        with torch.cuda.stream(s):
            O1, UV1, dQ1, dK1, dV1 = ska.sinkhorn_attn_step(Q, K, V, G, w.W, w.T, w.R, w.eps)
            checks = [(a.float() - b.float()).abs().max() for a, b in ((O1, O0), (dQ1, dQ0), (dK1, dK0), (dV1, dV0))]
        s.synchronize()
        assert all(float(c) == 0.0 for c in checks), rep
    ska.sinkhorn_attn_set_streams(1)
    try:
        O2, UV2, dQ2, dK2, dV2 = ska.sinkhorn_attn_step(Q, K, V, G, w.W, w.T, w.R, w.eps)
        torch.cuda.synchronize()
    finally:
        ska.sinkhorn_attn_set_streams(2)
    assert torch.equal(O2, O0) and torch.equal(dQ2, dQ0) and torch.equal(dK2, dK0) and torch.equal(dV2, dV0)


def test_dense_widened_band_dustbin():
    """The paper's own dustbin path: one learned token appended per side and a band wide enough
    to cover everything (W~ = max(W, L)).  That is the plain operator on the augmented tensors;
    the oracle is its support-generic core on the dense (L+1) x (L+1) support."""
    import torch

    import paper_2605_08123_amd as ska
    L, d, T, R, eps = 200, 32, 6, 2, 0.9
    w = small("widened", L + 1, d, L + 1, T, "f32", eps=eps, R=R)
    print(f"\n[case] {w}: dense widened-band dustbin", flush=True)
    arrays = make_inputs(w, 27)              # the last row of Q, K, V plays the learned token
    arrays[3][:, :, L] = 0.0                 # the dustbin query's output is dropped
    got, ref = None, None
    dev = torch.device("cuda:0")
    Q, K, V, G = (torch.from_numpy(x).to(dev) for x in arrays)
    O, UV = ska.sinkhorn_attn_fwd(Q, K, V, w.W, T, R, eps)
    dQ, dK, dV = ska.sinkhorn_attn_bwd(Q, K, V, O, G, UV, w.W, T, R, eps)
    torch.cuda.synchronize()
    q, k, v, g = (x[0, 0].astype(np.float64) for x in arrays)
    n = L + 1
    rptr = np.arange(n + 1, dtype=np.int64) * n
    cols = np.tile(np.arange(n, dtype=np.int32), n)
    S = ((q @ k.T) / (eps * np.sqrt(d))).reshape(-1)
    r = oracle.core(rptr, cols, S, v, g, T, R)
    cs = 1.0 / (eps * np.sqrt(d))
    Sb = r["Sbar"].reshape(n, n)
    for name, x, y in (("O", O, r["O"]), ("dQ", dQ, cs * Sb @ k), ("dK", dK, cs * Sb.T @ q), ("dV", dV, r["dV"])):
        e = rel(x[0, 0].cpu().numpy().astype(np.float64), y)
        print(f"   {name}: rel-L2 {e:.2e}", flush=True)
        assert e <= TOL["f32"], (name, e)


def _targets(w, seed):
    rng = np.random.default_rng(seed)
    a = rng.uniform(0.4, 1.8, (w.B, w.H, w.L))
    b = rng.uniform(0.4, 1.8, (w.B, w.H, w.L))
    b *= a.sum(-1, keepdims=True) / b.sum(-1, keepdims=True)      # compatible totals
    return np.log(a).astype(np.float32), np.log(b).astype(np.float32)


@pytest.mark.parametrize("dtype,d,R", [("f32", 32, 2), ("bf16", 64, 2), ("bf16", 64, 3), ("f32", 64, 1)])
def test_general_marginals(dtype, d, R):
    """Row targets a and column targets b (appendix on compatible general marginals) against
    the oracle; unit targets passed explicitly reproduce the balanced call bit for bit."""
    import torch

    import paper_2605_08123_amd as ska
    w = small("marg", 500, d, 33, 6, dtype, eps=0.8, B=1, H=2, R=R)
    print(f"\n[case] {w} with marginals", flush=True)
    arrays = make_inputs(w, 31)
    la, lb = _targets(w, 32)
    dev = torch.device("cuda:0")
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(td) for x in arrays)
    tla, tlb = torch.from_numpy(la).to(dev), torch.from_numpy(lb).to(dev)
    O, UV = ska.sinkhorn_attn_fwd_marginals(Q, K, V, tla, tlb, w.W, w.T, w.R, w.eps)
    dQ, dK, dV, eta0 = ska.sinkhorn_attn_bwd_marginals(Q, K, V, tla, tlb, O, G, UV, w.W, w.T, w.R, w.eps,
                                                       want_eta0=True)
    torch.cuda.synchronize()
    ref = oracle.band_batched(*arrays, w.W, w.T, w.R, w.eps, log_a=la.astype(np.float64),
                              log_b=lb.astype(np.float64))
    got = {k: v.float().cpu().numpy().astype(np.float64) for k, v in dict(O=O, dQ=dQ, dK=dK, dV=dV).items()}
    errs = {k: rel(got[k], ref[k]) for k in got}
    print("   rel-L2:", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    for k, e in errs.items():
        assert e <= TOL[dtype], (k, e)
    # the targets are met: column sums of P_RR are b, so <1, O-weights> ... checked through the
    # potentials: u_R + v_R agrees with the oracle's
    s_got = (UV[:, :, 2 * R] + UV[:, :, 2 * R + 1]).cpu().numpy()
    s_ref = ref["UV"][:, :, 2 * R] + ref["UV"][:, :, 2 * R + 1]
    assert np.abs(s_got - s_ref).max() < (2e-4 if dtype == "f32" else 2e-2)
    if dtype == "f32":
        q, k, v, g = (x[0, 0] for x in arrays)
        one = oracle.band(q, k, v, g, w.W, w.T, w.R, w.eps, log_a=la[0, 0].astype(np.float64),
                          log_b=lb[0, 0].astype(np.float64))
        assert rel(eta0[0, 0].cpu().numpy().astype(np.float64), one["bars"][1]) < 1e-3
    # unit targets given explicitly == the balanced entry point
    z = torch.zeros_like(tla)
    O1, UV1 = ska.sinkhorn_attn_fwd_marginals(Q, K, V, z, z, w.W, w.T, w.R, w.eps)
    O0, UV0 = ska.sinkhorn_attn_fwd(Q, K, V, w.W, w.T, w.R, w.eps)
    g1 = ska.sinkhorn_attn_bwd_marginals(Q, K, V, z, z, O1, G, UV1, w.W, w.T, w.R, w.eps)
    g0 = ska.sinkhorn_attn_bwd(Q, K, V, O0, G, UV0, w.W, w.T, w.R, w.eps)
    assert torch.equal(O1, O0) and all(torch.equal(x, y) for x, y in zip(g1, g0))
    with pytest.raises(ska.SinkhornAttnError) as e:      # no marginals on the dustbin's unit-target space
        ska.sinkhorn_attn_fwd_marginals(Q, K, V, tla, tlb, w.W, w.T, w.R, w.eps, dustbin=True)
    assert e.value.status == -2


@pytest.mark.parametrize("dtype,d,R,marg", [("f32", 32, 2, False), ("bf16", 64, 2, False), ("bf16", 128, 2, False),
                                            ("bf16", 64, 3, False), ("f32", 64, 1, True)])
def test_padded_batch_of_different_lengths(dtype, d, R, marg):
    """Per-item query and key lengths (rectangular supports, the remark after Eq. 1-2): every
    (item, head) against the oracle's rectangular operator on the unpadded slices.  The padding
    of every input holds NaN, so any use of it shows; results in the padding are exact zeros.
    Item 1 has query rows whose band holds no key (len_q > len_k + W), item 3 is shorter than
    one tile, item 4 is full length."""
    import torch

    import paper_2605_08123_amd as ska
    lq = np.array([700, 610, 333, 20, 700, 97], dtype=np.int32)
    lk = np.array([655, 140, 400, 9, 700, 260], dtype=np.int32)
    w = small("varlen", 700, d, 33, 5, dtype, eps=0.8, B=len(lq), H=2, R=R)
    print(f"\n[case] {w} lengths q={lq.tolist()} k={lk.tolist()} marginals={marg}", flush=True)
    q, k, v, g = make_inputs(w, 41)
    la = lb = None
    if marg:
        la, lb = _targets(w, 42)
    for b in range(w.B):
        q[b, :, lq[b]:] = np.nan
        g[b, :, lq[b]:] = np.nan
        k[b, :, lk[b]:] = np.nan
        v[b, :, lk[b]:] = np.nan
        if marg:
            la[b, :, lq[b]:] = np.nan
            lb[b, :, lk[b]:] = np.nan
    dev = torch.device("cuda:0")
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(td) for x in (q, k, v, g))
    tla = torch.from_numpy(la).to(dev) if marg else None
    tlb = torch.from_numpy(lb).to(dev) if marg else None
    tq, tk = torch.from_numpy(lq).to(dev), torch.from_numpy(lk).to(dev)
    O, UV = ska.sinkhorn_attn_fwd_varlen(Q, K, V, tla, tlb, tq, tk, w.W, w.T, w.R, w.eps)
    dQ, dK, dV, eta0 = ska.sinkhorn_attn_bwd_varlen(Q, K, V, tla, tlb, tq, tk, O, G, UV, w.W, w.T, w.R, w.eps,
                                                    want_eta0=True)
    torch.cuda.synchronize()
    got = {n: x.float().cpu().numpy().astype(np.float64)
           for n, x in dict(O=O, dQ=dQ, dK=dK, dV=dV, UV=UV, eta0=eta0).items()}
    for n in got:
        assert np.isfinite(got[n]).all(), n
    # the GPU rounds its inputs to the storage type; the oracle gets the same rounded values
    qr, kr, vr, gr = (x.float().cpu().numpy().astype(np.float64) for x in (Q, K, V, G))
    worst = dict(O=0.0, dQ=0.0, dK=0.0, dV=0.0)
    for b in range(w.B):
        for h in range(w.H):
            a, c = int(lq[b]), int(lk[b])
            ref = oracle.band_rect(qr[b, h, :a], kr[b, h, :c], vr[b, h, :c], gr[b, h, :a], w.W, w.T, w.R, w.eps,
                                   log_a=la[b, h, :a].astype(np.float64) if marg else None,
                                   log_b=lb[b, h, :c].astype(np.float64) if marg else None)
            for n, cut in (("O", a), ("dQ", a), ("dK", c), ("dV", c)):
                worst[n] = max(worst[n], rel(got[n][b, h, :cut], ref[n]))
                assert np.all(got[n][b, h, cut:] == 0.0), (n, b, h)
            for t in range(R + 1):
                assert np.all(got["UV"][b, h, 2 * t, a:] == 0.0) and np.all(got["UV"][b, h, 2 * t + 1, c:] == 0.0)
            # potentials of the rows that have edges, through the terminal plan's row sums being
            # unit (or a): u_R + logsumexp_j(S + v_R) = log a -- covered by the O comparison; here
            # the raw terminal potentials themselves
            tol_uv = 2e-4 if dtype == "f32" else 3e-2
            assert np.abs(got["UV"][b, h, 2 * R, :a] - ref["U"][R]).max() < tol_uv
            assert np.abs(got["UV"][b, h, 2 * R + 1, :c] - ref["Vp"][R]).max() < tol_uv
            assert np.all(got["eta0"][b, h, c:] == 0.0)
    print("   worst rel-L2 over items:", {n: f"{e:.2e}" for n, e in worst.items()}, flush=True)
    for n, e in worst.items():
        assert e <= TOL[dtype], (n, e)
    # lengths equal to L reproduce the plain call bit for bit (finite inputs for this one)
    Qf, Kf, Vf, Gf = (torch.nan_to_num(x) for x in (Q, K, V, G))
    full = torch.full((w.B,), w.L, dtype=torch.int32, device=dev)
    O1, UV1 = ska.sinkhorn_attn_fwd_varlen(Qf, Kf, Vf, None, None, full, full, w.W, w.T, w.R, w.eps)
    O0, UV0 = ska.sinkhorn_attn_fwd(Qf, Kf, Vf, w.W, w.T, w.R, w.eps)
    g1 = ska.sinkhorn_attn_bwd_varlen(Qf, Kf, Vf, None, None, full, full, O1, Gf, UV1, w.W, w.T, w.R, w.eps)
    g0 = ska.sinkhorn_attn_bwd(Qf, Kf, Vf, O0, Gf, UV0, w.W, w.T, w.R, w.eps)
    assert torch.equal(O1, O0) and torch.equal(UV1, UV0) and all(torch.equal(x, y) for x, y in zip(g1, g0))
    with pytest.raises(ska.SinkhornAttnError) as e:      # the dustbin sits at index L
        ska.sinkhorn_attn_fwd_varlen(Qf, Kf, Vf, None, None, tq, tk, w.W, w.T, w.R, w.eps, dustbin=True)
    assert e.value.status == -2


def test_tail_depth_dustbin():
    check(small("taildb", 300, 64, 24, 4, "bf16", eps=0.9, R=3, dustbin=True, dustbin_score=-0.2), seed=17)
    check(small("taildb", 300, 32, 24, 4, "f32", eps=0.9, R=1, dustbin=True, dustbin_score=0.4), seed=18)


@pytest.mark.parametrize("d,W,L", [(32, 300, 900), (64, 250, 800)])
def test_first_half_step_wide_dynamic_range(d, W, L):
    """Scores that rise by about 0.2 nats per column: inside one row's band they span about
    100 nats, more than one fixed stabiliser covers in fp32, so the very first half-step (no
    previous iterate to take one from) has to follow the running maximum while it sweeps the
    band.  fp32 storage (bf16 scores of this size carry an absolute error of a third of a nat
    from the rounding of the scaled operand alone).  Potentials and all four results against
    the oracle at the usual fp32 tolerance."""
    import torch

    import paper_2605_08123_amd as ska
    w = small("ramp", L, d, W, 3, "f32", eps=1.0, B=1, H=2, R=2)
    print(f"\n[case] {w} score ramp", flush=True)
    q, k, v, g = make_inputs(w, 77)
    c = 1.0 / (w.eps * np.sqrt(d))
    q[..., 0] = 1.0
    k[..., 0] = (0.2 / c) * np.arange(L, dtype=np.float32)
    q[..., 1:] *= 0.5
    dev = torch.device("cuda:0")
    Q, K, V, G = (torch.from_numpy(x).to(dev) for x in (q, k, v, g))
    O, UV = ska.sinkhorn_attn_fwd(Q, K, V, w.W, w.T, w.R, w.eps)
    dQ, dK, dV = ska.sinkhorn_attn_bwd(Q, K, V, O, G, UV, w.W, w.T, w.R, w.eps)[:3]
    torch.cuda.synchronize()
    got = {n: x.cpu().numpy().astype(np.float64) for n, x in dict(O=O, dQ=dQ, dK=dK, dV=dV, UV=UV).items()}
    ref = oracle.band_batched(q, k, v, g, w.W, w.T, w.R, w.eps)
    band_rise = 0.2 * (2 * W)
    assert band_rise > 88.0                           # exp() of the spread overflows fp32
    assert np.abs(ref["UV"][:, :, 0]).max() > 100.0   # potentials of that size
    for n in got:
        assert np.isfinite(got[n]).all(), n
    errs = {n: rel(got[n], ref[n]) for n in ("O", "dQ", "dK", "dV")}
    print("   rel-L2:", {n: f"{e:.2e}" for n, e in errs.items()}, flush=True)
    for t in range(w.R + 1):
        s_got = got["UV"][:, :, 2 * t] + got["UV"][:, :, 2 * t + 1]
        s_ref = ref["UV"][:, :, 2 * t] + ref["UV"][:, :, 2 * t + 1]
        assert np.abs(s_got - s_ref).max() < 1e-3, (t, np.abs(s_got - s_ref).max())
    for n, e in errs.items():
        assert e <= TOL["f32"], (n, e)


def test_eta0_general_tail():
    w = small("eta", 300, 32, 20, 4, "f32", R=3)
    got = run_gpu(w, make_inputs(w, 6), want_eta0=True)
    q, k, v, g = make_inputs(w, 6)
    ref = oracle.band(q[0, 0], k[0, 0], v[0, 0], g[0, 0], w.W, w.T, w.R, w.eps)
    assert rel(got["eta0"][0, 0], ref["bars"][1]) < 1e-3


def test_eta0_is_base_cotangent():
    w = small("eta", 400, 32, 20, 6, "f32")
    got = run_gpu(w, make_inputs(w, 5), want_eta0=True)
    q, k, v, g = make_inputs(w, 5)
    ref = oracle.band(q[0, 0], k[0, 0], v[0, 0], g[0, 0], w.W, w.T, w.R, w.eps)
    assert rel(got["eta0"][0, 0], ref["bars"][1]) < 1e-3
    assert abs(got["eta0"].sum()) < 1e-3 * np.abs(got["eta0"]).sum()


def test_error_codes_on_device():
    import torch

    import paper_2605_08123_amd as ska
    x = torch.zeros((1, 1, 64, 32), device="cuda")
    with pytest.raises(ska.SinkhornAttnError) as e:
        ska.sinkhorn_attn_fwd(x, x, x, 4, 2, R=33)
    assert e.value.status == -2
    with pytest.raises(ska.SinkhornAttnError) as e:
        ska.sinkhorn_attn_fwd(x, x, x, 4, 2, eps=0.0)
    assert e.value.status == -1


def test_issue_probe_hook():
    """The register-only probe returns eight positive times; MFMA and VALU work together cost at
    least as much as either alone and at most their sum (with some slack for clocks and launch
    overhead), and leaving the exponentials or the adds out does not cost more than the full mix."""
    import paper_2605_08123_amd as ska
    ms, simds = ska.sinkhorn_attn_probe_issue(tiles=2000, waves_per_simd=4)
    print(f"\n[case] issue probe: {ms} ms on {simds} SIMDs", flush=True)
    assert simds >= 4 and all(t > 0.0 for t in ms)
    assert len(ms) == 8
    assert max(ms[0], ms[1]) * 0.9 <= ms[2] <= (ms[0] + ms[1]) * 1.25
    assert ms[3] <= ms[2] * 1.1 and ms[4] <= ms[2] * 1.1 and ms[5] <= ms[0] * 1.1
    with pytest.raises(ska.SinkhornAttnError):
        ska.sinkhorn_attn_probe_issue(tiles=0)


def test_profile_hooks_count_launches():
    """Benchmark hooks: phase spans bracket the documented numbers of sweep launches."""
    import torch

    import paper_2605_08123_amd as ska
    w = small("prof", 500, 64, 40, 5, "bf16")
    arrays = make_inputs(w, 9)
    ska.sinkhorn_attn_profile_read_phases()          # forget anything recorded earlier
    ska.sinkhorn_attn_profile_enable(2)
    try:
        run_gpu(w, arrays)
    finally:
        ska.sinkhorn_attn_profile_enable(0)
    ph = ska.sinkhorn_attn_profile_read_phases()
    want = {"prescale": 2, "first_half_step": 1, "scaling_sweeps": 2 * w.T + 3, "output_map": 1,
            "rowdot": 1, "dV": 1, "matvec_chain": 3, "final_sweeps": 2}
    assert {k: v[1] for k, v in ph.items()} == want
    assert all(v[0] >= 0.0 for v in ph.values()) and ph["scaling_sweeps"][0] > 0.0
    # level 1 keeps the scaling-sweep span only; a read empties the record
    ska.sinkhorn_attn_profile_enable(1)
    try:
        run_gpu(w, arrays)
    finally:
        ska.sinkhorn_attn_profile_enable(0)
    ms, n = ska.sinkhorn_attn_profile_read()
    assert n == 2 * w.T + 3 and ms > 0.0
    assert all(v == (0.0, 0) for v in ska.sinkhorn_attn_profile_read_phases().values())
    torch.cuda.synchronize()
