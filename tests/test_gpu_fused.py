"""Fused half-steps (the tail of Sec. 2.2, or base solve and tail, as one launch chained by
per-block counters): the same blocks run the same arithmetic as in separate launches, so every
result must equal the unfused one bit for bit, in every mode, with lengths, marginals, masks,
dense windows, ragged sizes, both block sizes and several problems; and the oracle agrees.
A wait that runs out (forced here by a poll limit of one) must end the launch normally and either
leave the result untouched or poison it with NaN, never hang."""
import numpy as np
import pytest

import oracle
from paper_2605_08123_amd.workloads import Workload, make_inputs
from tests.measures import assert_per_tensor, floors

pytestmark = pytest.mark.gpu

CASES = [
    # name, B, H, L, d, W, T, R, eps, dtype, kind
    ("f32_tiny", 1, 1, 256, 32, 16, 8, 2, 1.0, "f32", "plain"),
    ("bf16_many", 2, 3, 3000, 64, 70, 6, 2, 0.5, "bf16", "plain"),
    ("bf16_big_blocks", 1, 2, 120000, 64, 256, 3, 2, 0.5, "bf16", "plain"),   # 256-row blocks, two per workgroup
    ("bf16_dense", 1, 2, 700, 64, 5000, 4, 2, 0.8, "bf16", "plain"),
    ("f32_ragged_R3", 1, 2, 1001, 64, 33, 0, 3, 1.0, "f32", "plain"),
    ("bf16_lengths", 2, 2, 2000, 64, 100, 4, 2, 0.7, "bf16", "varlen"),
    ("f32_marginals", 1, 2, 900, 32, 40, 5, 2, 1.0, "f32", "marginals"),
    ("bf16_masks", 2, 1, 1500, 64, 31, 4, 2, 0.6, "bf16", "masked"),
    ("bf16_d128", 1, 1, 1300, 128, 64, 3, 1, 0.5, "bf16", "plain"),
]


def _forward(ska, torch, w, kind, Q, K, V, extra):
    if kind == "varlen":
        return ska.sinkhorn_attn_fwd_varlen(Q, K, V, None, None, extra[0], extra[1], w.W, w.T, w.R, w.eps)
    if kind == "marginals":
        return ska.sinkhorn_attn_fwd_marginals(Q, K, V, extra[0], extra[1], w.W, w.T, w.R, w.eps)
    if kind == "masked":
        return ska.sinkhorn_attn_fwd_masked(Q, K, V, extra[0], extra[1], w.W, w.T, w.R, w.eps)
    return ska.sinkhorn_attn_fwd(Q, K, V, w.W, w.T, w.R, w.eps)


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_fused_half_steps_equal_separate_launches(case):
    import torch

    import paper_2605_08123_amd as ska
    name, B, H, L, d, W, T, R, eps, dtype, kind = case
    w = Workload(name, 31, B, H, L, d, W, T, R, eps, dtype)
    print(f"\n[case] {w} ({kind})", flush=True)
    dev = torch.device("cuda:0")
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    arrays = make_inputs(w, 310 + len(name))
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(td) for x in arrays)
    rng = np.random.default_rng(77)
    extra = None
    if kind == "varlen":
        extra = [torch.tensor(rng.integers(L // 3, L + 1, size=B), dtype=torch.int32, device=dev) for _ in range(2)]
    if kind == "marginals":
        a = rng.uniform(0.5, 1.5, size=(B, H, L)); b = rng.uniform(0.5, 1.5, size=(B, H, L))
        b *= a.sum(-1, keepdims=True) / b.sum(-1, keepdims=True)
        extra = [torch.from_numpy(np.log(x).astype(np.float32)).to(dev) for x in (a, b)]
    if kind == "masked":
        extra = [torch.from_numpy((rng.random((B, L)) > 0.3).astype(np.uint8)).to(dev) for _ in range(2)]
    results = {}
    try:
        for mode in (0, 1, 2):
            ska.sinkhorn_attn_set_fused_half_steps(mode)
            O, UV = _forward(ska, torch, w, kind, Q, K, V, extra)
            step = None
            if kind == "plain":
                step = ska.sinkhorn_attn_step(Q, K, V, G, w.W, w.T, w.R, w.eps)
            torch.cuda.synchronize()
            results[mode] = (O, UV, step)
    finally:
        ska.sinkhorn_attn_set_fused_half_steps(0)
    O0, UV0, step0 = results[0]
    assert torch.isfinite(O0.float()).all()
    for mode in (1, 2):
        O, UV, step = results[mode]
        assert torch.equal(O, O0), mode
        assert torch.equal(torch.nan_to_num(UV, neginf=-1e30), torch.nan_to_num(UV0, neginf=-1e30)), mode
        if step is not None:
            for x, y in zip(step, step0):
                assert torch.equal(x, y), mode
    if kind == "plain" and L <= 4000:   # and the fused result is the operator's: against the oracle
        O, UV, dQ, dK, dV = results[2][2]
        got = {n: x.float().cpu().numpy().astype(np.float64) for n, x in dict(O=O, dQ=dQ, dK=dK, dV=dV).items()}
        ref = oracle.band_batched(*arrays, w.W, w.T, w.R, w.eps)
        assert_per_tensor(got, ref, dtype, floors(dtype, *arrays, ref["O"], w.eps), where=name)


def test_a_wait_that_runs_out_ends_the_launch():
    """Poll limit one: waits give up at once.  The launch must end normally (no hang), and each
    result is either the right one (no wait ran out in time to matter) or carries the NaN a
    timed-out block wrote."""
    import torch

    import paper_2605_08123_amd as ska
    w = Workload("giveup", 32, 1, 2, 20000, 64, 256, 6, 2, 0.5, "bf16")
    print(f"\n[case] {w} poll limit 1", flush=True)
    dev = torch.device("cuda:0")
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(torch.bfloat16) for x in make_inputs(w, 3))
    O0, UV0 = ska.sinkhorn_attn_fwd(Q, K, V, w.W, w.T, w.R, w.eps)
    torch.cuda.synchronize()
    try:
        ska.sinkhorn_attn_set_fused_half_steps(2, 1)
        for rep in range(3):
            O, UV = ska.sinkhorn_attn_fwd(Q, K, V, w.W, w.T, w.R, w.eps)
            torch.cuda.synchronize()   # returns: the launch has ended
            bad = ~torch.isfinite(UV)
            same = torch.equal(O, O0)
            print(f"   rep {rep}: {int(bad.sum())} non-finite potentials, output identical: {same}", flush=True)
            assert same or bool(bad.any())   # right, or visibly poisoned; and it returned
    finally:
        ska.sinkhorn_attn_set_fused_half_steps(0)
    # and the library is intact afterwards
    O1, UV1 = ska.sinkhorn_attn_fwd(Q, K, V, w.W, w.T, w.R, w.eps)
    torch.cuda.synchronize()
    assert torch.equal(O1, O0) and torch.equal(UV1, UV0)
