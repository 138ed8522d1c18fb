"""Host-side checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects bad arguments before anything is launched (so all
of this runs without a GPU)."""
import ctypes
import os
import re

import pytest

from paper_2605_08123_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "sinkhorn_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sinkhorn_attn_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    names = declared_symbols()
    assert names == ["sinkhorn_attn_base_vjp", "sinkhorn_attn_bwd", "sinkhorn_attn_bwd_dustbin_token",
                     "sinkhorn_attn_bwd_marginals", "sinkhorn_attn_bwd_variant", "sinkhorn_attn_bwd_varlen",
                     "sinkhorn_attn_fwd", "sinkhorn_attn_fwd_dustbin_token", "sinkhorn_attn_fwd_eps_schedule", "sinkhorn_attn_fwd_marginals",
                     "sinkhorn_attn_fwd_masked", "sinkhorn_attn_fwd_varlen",
                     "sinkhorn_attn_probe_issue", "sinkhorn_attn_profile_enable",
                     "sinkhorn_attn_profile_read", "sinkhorn_attn_profile_read_phases",
                     "sinkhorn_attn_select_tail_depth", "sinkhorn_attn_select_workspace_bytes",
                     "sinkhorn_attn_set_fused_half_steps", "sinkhorn_attn_set_split_min_edges", "sinkhorn_attn_set_streams", "sinkhorn_attn_step",
                     "sinkhorn_attn_step_static", "sinkhorn_attn_strerror",
                     "sinkhorn_attn_workspace_bytes"]
    for n in names:
        assert hasattr(lib, n), n


def test_workspace_bytes_and_strerror():
    assert binding.sinkhorn_attn_workspace_bytes(1, 2, 262144, 64, 256, 20) >= 2 * 262144 * 13 * 4
    assert binding.sinkhorn_attn_workspace_bytes(1, 1, 0, 64, 256, 20) == 0          # L < 1
    assert binding.sinkhorn_attn_workspace_bytes(1, 1, 16, 48, 256, 20) == 0         # d unsupported
    assert binding.sinkhorn_attn_workspace_bytes(1, 1, 16, 64, 4, 2, R=33) == 0
    assert binding.sinkhorn_attn_workspace_bytes(1, 1, 16, 64, 4, 2, R=0) == 0
    assert binding.sinkhorn_attn_workspace_bytes(1, 1, (1 << 24) + 1, 64, 4, 2) == 0   # L too long
    assert binding.sinkhorn_attn_workspace_bytes(1, 1, 1 << 24, 64, 4, 2) > 0
    assert (binding.sinkhorn_attn_workspace_bytes(1, 1, 16, 64, 4, 2, R=4)
            > binding.sinkhorn_attn_workspace_bytes(1, 1, 16, 64, 4, 2, R=1) > 0)
    a = binding.sinkhorn_attn_workspace_bytes(2, 2, 1000, 64, 10, 5, dustbin=False)
    b = binding.sinkhorn_attn_workspace_bytes(2, 2, 1000, 64, 10, 5, dustbin=True)
    assert b > a > 0
    for s in (0, -1, -2, -3, -4, -5, 17):
        assert isinstance(binding.sinkhorn_attn_strerror(s), str) and binding.sinkhorn_attn_strerror(s)


def _fwd(lib, ptr=1 << 20, **kw):
    a = dict(B=1, H=1, L=64, d=32, W=4, T=2, R=2, eps=1.0, dustbin=0, sdb=0.0, dtype=0)
    a.update(kw)
    p = ctypes.c_void_p(ptr)
    return lib.sinkhorn_attn_fwd(p, p, p, p, p, a["B"], a["H"], a["L"], a["d"], a["W"], a["T"], a["R"],
                                 a["eps"], a["dustbin"], a["sdb"], a["dtype"], None, 0, None)


def _bwd(lib, ws=None, ws_bytes=0, ptr=1 << 20, **kw):
    a = dict(B=1, H=1, L=64, d=32, W=4, T=2, R=2, eps=1.0, dustbin=0, sdb=0.0, dtype=0)
    a.update(kw)
    p = ctypes.c_void_p(ptr)
    return lib.sinkhorn_attn_bwd(p, p, p, p, p, p, p, p, p, None, a["B"], a["H"], a["L"], a["d"], a["W"],
                                 a["T"], a["R"], a["eps"], a["dustbin"], a["sdb"], a["dtype"], ws, ws_bytes,
                                 None)


def test_argument_errors_are_reported_before_any_launch():
    """The pointers below are never dereferenced: every call fails validation."""
    lib = binding.load()
    assert _fwd(lib, ptr=0) == binding.SKA_EINVAL
    for bad in (dict(B=0), dict(H=0), dict(L=0), dict(W=-1), dict(T=-1), dict(eps=0.0), dict(eps=-1.0),
                dict(eps=float("inf")), dict(eps=float("nan"))):
        assert _fwd(lib, **bad) == binding.SKA_EINVAL, bad
        assert _bwd(lib, **bad) == binding.SKA_EINVAL, bad
    for bad in (dict(R=0), dict(R=33), dict(d=48), dict(d=256), dict(dtype=7)):
        assert _fwd(lib, **bad) == binding.SKA_EUNSUPPORTED, bad
        assert _bwd(lib, **bad) == binding.SKA_EUNSUPPORTED, bad
    # lengths and marginal targets do not combine with the dustbin
    pp, nul = ctypes.c_void_p(1 << 20), None
    for la, lq in ((pp, nul), (nul, pp)):
        assert lib.sinkhorn_attn_fwd_varlen(pp, pp, pp, la, nul, lq, nul, pp, pp, 1, 1, 64, 32, 4, 2, 2, 1.0, 1,
                                            0.0, 0, None, 0, None) == binding.SKA_EUNSUPPORTED
    for T, want in ((0, binding.SKA_EUNSUPPORTED), (33, binding.SKA_EUNSUPPORTED), (4, binding.SKA_EWORKSPACE)):
        assert lib.sinkhorn_attn_base_vjp(pp, pp, nul, nul, nul, nul, pp, pp, pp, pp, 1, 1, 64, 32, 4, T, 1.0, 0,
                                          0.0, 0, None, 0, None) == want
    assert binding.sinkhorn_attn_select_workspace_bytes(1, 1, 64, 32, 4, 0, 4) == 0       # T >= 1
    assert (binding.sinkhorn_attn_select_workspace_bytes(1, 1, 64, 32, 4, 5, 4, dtype=0)
            > binding.sinkhorn_attn_workspace_bytes(1, 1, 64, 32, 4, 0, 5, dtype=0) + 2 * 64 * 32 * 4)
    def sched(eps_s, T_s, eps=0.5):
        n = len(eps_s)
        return lib.sinkhorn_attn_fwd_eps_schedule(pp, pp, pp, nul, nul, nul, nul, pp, pp, 1, 1, 64, 32, 4, n,
                                                  (ctypes.c_float * max(n, 1))(*eps_s), (ctypes.c_int * max(n, 1))(*T_s),
                                                  2, eps, 0, 0.0, 1, None, 0, None)
    assert sched([2.0, 1.0, 0.5], [1, 1, 1]) == binding.SKA_EWORKSPACE     # valid schedule: gets as far as the workspace
    assert sched([1.0, 2.0, 0.5], [1, 1, 1]) == binding.SKA_EINVAL         # increasing
    assert sched([2.0, 1.0], [1, 1]) == binding.SKA_EINVAL                 # does not end at eps
    assert sched([2.0, 0.5], [1, -1]) == binding.SKA_EINVAL
    assert sched([], []) == binding.SKA_EINVAL
    # learned dustbin tokens: missing or misaligned tokens, and the forward needs the full workspace
    tok = lambda q: lib.sinkhorn_attn_fwd_dustbin_token(pp, pp, pp, q, pp, pp, pp, pp, 1, 1, 64, 32, 4, 2, 2, 1.0, 0,
                                                        None, 0, None)
    assert tok(nul) == binding.SKA_EINVAL and tok(ctypes.c_void_p((1 << 20) + 4)) == binding.SKA_EINVAL
    assert tok(pp) == binding.SKA_EWORKSPACE
    assert lib.sinkhorn_attn_set_streams(3) == binding.SKA_EINVAL and lib.sinkhorn_attn_set_streams(2) == binding.SKA_OK
    assert _bwd(lib, ws=None, ws_bytes=0) == binding.SKA_EWORKSPACE
    assert _fwd(lib, dtype=1) == binding.SKA_EWORKSPACE          # bf16 forward needs its scratch
    need = binding.sinkhorn_attn_workspace_bytes(1, 1, 64, 32, 4, 2, dtype=0)
    assert _bwd(lib, ws=ctypes.c_void_p(1 << 20), ws_bytes=need - 1) == binding.SKA_EWORKSPACE
    assert _bwd(lib, ws=ctypes.c_void_p((1 << 20) + 4), ws_bytes=need) == binding.SKA_EINVAL


def test_binding_rejects_cpu_tensors():
    import torch
    x = torch.zeros((1, 1, 8, 32))
    with pytest.raises(ValueError):
        binding.sinkhorn_attn_fwd(x, x, x, 2, 1)


def test_step_static_rejects_before_any_launch():
    """The no-allocation entry point checks its arguments, and the size against the static scratch,
    on the host."""
    lib = binding.load()
    p = ctypes.c_void_p(1 << 20)

    def call(L=64, d=32, ptr=p, R=2, eps=1.0):
        return lib.sinkhorn_attn_step_static(ptr, p, p, p, None, None, None, None, p, p, p, p, p, None, 1, 2, L, d, 4, 2,
                                             R, ctypes.c_float(eps), 0, ctypes.c_float(0.0), 1, None)
    assert call(ptr=None) == binding.SKA_EINVAL
    assert call(eps=0.0) == binding.SKA_EINVAL
    assert call(d=48) == binding.SKA_EUNSUPPORTED
    assert call(R=0) == binding.SKA_EUNSUPPORTED
    big = 262144
    assert binding.sinkhorn_attn_workspace_bytes(1, 2, big, 64, 4, 2) > binding.SKA_STATIC_SCRATCH_BYTES
    assert call(L=big, d=64) == binding.SKA_ESTATIC
    assert "static" in binding.sinkhorn_attn_strerror(binding.SKA_ESTATIC)
