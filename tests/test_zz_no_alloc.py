"""The entry point that allocates nothing (sinkhorn_attn_step_static: the step on the library's
static scratch) against sinkhorn_attn_step with a caller's workspace, through the raw C ABI: the
same kernels on the same inputs, so results are compared bit for bit; two calls in a row, the
second on a smaller problem (the scratch keeps the first call's contents), and a problem beyond
the static buffer is refused before anything is launched."""
import ctypes

import numpy as np
import pytest

from paper_2605_08123_amd import binding
from paper_2605_08123_amd.workloads import Workload, make_inputs

pytestmark = pytest.mark.gpu


def _tensors(w):
    import torch
    dev = torch.device("cuda:0")
    td = torch.float32 if w.dtype == "f32" else torch.bfloat16
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(td) for x in make_inputs(w))
    Lp = w.L + int(w.dustbin)
    outs = lambda: dict(O=torch.full_like(Q, float("nan")), dQ=torch.full_like(Q, float("nan")),
                        dK=torch.full_like(Q, float("nan")), dV=torch.full_like(Q, float("nan")),
                        UV=torch.full((w.B, w.H, 2 * (w.R + 1), Lp), float("nan"), device=dev, dtype=torch.float32),
                        eta0=torch.full((w.B, w.H, Lp), float("nan"), device=dev, dtype=torch.float32))
    return Q, K, V, G, outs


def _call(lib, static, w, Q, K, V, G, o, ws=None):
    import torch
    vp = ctypes.c_void_p
    head = [vp(x.data_ptr()) for x in (Q, K, V, G)] + [None, None, None, None] + \
           [vp(o[k].data_ptr()) for k in ("O", "UV", "dQ", "dK", "dV", "eta0")]
    sizes = [w.B, w.H, w.L, w.d, w.W, w.T, w.R, ctypes.c_float(w.eps), int(w.dustbin),
             ctypes.c_float(w.dustbin_score), 0 if w.dtype == "f32" else 1]
    st = vp(torch.cuda.current_stream().cuda_stream)
    if static:
        return lib.sinkhorn_attn_step_static(*head, *sizes, st)
    return lib.sinkhorn_attn_step(*head, *sizes, vp(ws.data_ptr()), ctypes.c_size_t(ws.numel()), st)


def _compare(lib, w):
    import torch
    print(f"\n[case] {w}", flush=True)
    Q, K, V, G, outs = _tensors(w)
    need = binding.sinkhorn_attn_workspace_bytes(w.B, w.H, w.L, w.d, w.W, w.T, w.R, w.dustbin,
                                                 0 if w.dtype == "f32" else 1)
    assert 0 < need <= binding.SKA_STATIC_SCRATCH_BYTES
    ws = torch.empty(need, device="cuda", dtype=torch.uint8)
    ref, got = outs(), outs()
    assert _call(lib, False, w, Q, K, V, G, ref, ws) == 0
    assert _call(lib, True, w, Q, K, V, G, got) == 0
    torch.cuda.synchronize()
    for k in ref:
        a, b = ref[k].float().cpu().numpy(), got[k].float().cpu().numpy()
        assert np.isfinite(a[np.isfinite(b)]).all() and np.array_equal(a, b, equal_nan=True), k
        assert np.isfinite(b).all() or w.L == 1 or k in ("UV", "eta0"), k
    return got


def test_static_scratch_step_matches_workspace_step():
    lib = binding.load()
    # first a problem that fills a good part of the 32 MiB, then a smaller one of another shape and type
    big = Workload("static_big", 21, 2, 2, 9000, 64, 70, 4, 2, 0.5, "bf16")
    small = Workload("static_small", 22, 1, 3, 777, 32, 19, 3, 2, 1.0, "f32")
    _compare(lib, big)
    _compare(lib, small)
    _compare(lib, Workload("static_db", 23, 1, 2, 1500, 64, 33, 3, 2, 0.5, "bf16", dustbin=True, dustbin_score=0.3))


def test_static_scratch_step_refuses_what_does_not_fit():
    import torch
    lib = binding.load()
    w = Workload("static_too_big", 24, 1, 2, 262144, 64, 256, 2, 2, 0.5, "bf16")
    assert binding.sinkhorn_attn_workspace_bytes(w.B, w.H, w.L, w.d, w.W, w.T, w.R, False, 1) > binding.SKA_STATIC_SCRATCH_BYTES
    x = torch.zeros(16, device="cuda")   # never touched: the refusal comes before any launch
    vp = ctypes.c_void_p
    rc = lib.sinkhorn_attn_step_static(*[vp(x.data_ptr())] * 4, None, None, None, None, *[vp(x.data_ptr())] * 5, None,
                                       w.B, w.H, w.L, w.d, w.W, w.T, w.R, ctypes.c_float(w.eps), 0,
                                       ctypes.c_float(0.0), 1, None)
    assert rc == binding.SKA_ESTATIC
    assert "static" in binding.sinkhorn_attn_strerror(rc)
