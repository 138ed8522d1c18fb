"""Thin Python binding of the C ABI in include/sinkhorn_attn.h.

Argument marshalling only: torch supplies device memory and the current HIP
stream; every step of the operator runs in the library's kernels.  There is no
CPU or eager fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsinkhorn_attn.so")

SKA_F32, SKA_BF16 = 0, 1
SKA_BWD_ONE_REFERENCE, SKA_BWD_DIRECT, SKA_BWD_ONE_REFERENCE_GENERIC = 0, 1, 2
SKA_OK, SKA_EINVAL, SKA_EUNSUPPORTED, SKA_EWORKSPACE, SKA_EHIP, SKA_ESTATIC = 0, -1, -2, -3, -4, -5
SKA_STATIC_SCRATCH_BYTES = 32 << 20

_lib = None


def load():
    """dlopen the in-tree library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with "
                "`python -c 'import __graft_entry__ as g; g.build()'` (needs hipcc)")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i, f, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
        lib.sinkhorn_attn_workspace_bytes.restype = sz
        lib.sinkhorn_attn_workspace_bytes.argtypes = [i] * 9
        lib.sinkhorn_attn_fwd.restype = i
        lib.sinkhorn_attn_fwd.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, f, i, f, i, vp, sz, vp]
        lib.sinkhorn_attn_bwd.restype = i
        lib.sinkhorn_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, f,
                                          i, f, i, vp, sz, vp]
        lib.sinkhorn_attn_fwd_marginals.restype = i
        lib.sinkhorn_attn_fwd_marginals.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, f, i, f, i,
                                                    vp, sz, vp]
        lib.sinkhorn_attn_bwd_marginals.restype = i
        lib.sinkhorn_attn_bwd_marginals.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i, i, i, i,
                                                    i, i, i, f, i, f, i, vp, sz, vp]
        lib.sinkhorn_attn_fwd_varlen.restype = i
        lib.sinkhorn_attn_fwd_varlen.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, f, i, f,
                                                 i, vp, sz, vp]
        lib.sinkhorn_attn_bwd_varlen.restype = i
        lib.sinkhorn_attn_bwd_varlen.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i, i, i,
                                                 i, i, i, i, f, i, f, i, vp, sz, vp]
        lib.sinkhorn_attn_base_vjp.restype = i
        lib.sinkhorn_attn_base_vjp.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, f, i, f, i,
                                               vp, sz, vp]
        lib.sinkhorn_attn_select_workspace_bytes.restype = sz
        lib.sinkhorn_attn_select_workspace_bytes.argtypes = [i] * 9
        lib.sinkhorn_attn_select_tail_depth.restype = i
        lib.sinkhorn_attn_select_tail_depth.argtypes = [vp] * 13 + [i] * 7 + [f, i, f, i, f, vp, vp, vp, vp, sz, vp]
        lib.sinkhorn_attn_bwd_variant.restype = i
        lib.sinkhorn_attn_bwd_variant.argtypes = [i] + lib.sinkhorn_attn_bwd_varlen.argtypes
        lib.sinkhorn_attn_fwd_eps_schedule.restype = i
        lib.sinkhorn_attn_fwd_eps_schedule.argtypes = [vp] * 9 + [i] * 6 + [vp, vp, i, f, i, f, i, vp, sz, vp]
        lib.sinkhorn_attn_fwd_dustbin_token.restype = i
        lib.sinkhorn_attn_fwd_dustbin_token.argtypes = [vp] * 8 + [i] * 7 + [f, i, vp, sz, vp]
        lib.sinkhorn_attn_bwd_dustbin_token.restype = i
        lib.sinkhorn_attn_bwd_dustbin_token.argtypes = [vp] * 16 + [i] * 7 + [f, i, vp, sz, vp]
        lib.sinkhorn_attn_fwd_masked.restype = i
        lib.sinkhorn_attn_fwd_masked.argtypes = [vp] * 9 + [i] * 7 + [f, i, vp, sz, vp]
        lib.sinkhorn_attn_probe_issue.restype = i
        lib.sinkhorn_attn_probe_issue.argtypes = [vp, sz, i, i, ctypes.POINTER(ctypes.c_double), vp]
        lib.sinkhorn_attn_set_streams.restype = i
        lib.sinkhorn_attn_set_streams.argtypes = [i]
        lib.sinkhorn_attn_set_fused_half_steps.restype = i
        lib.sinkhorn_attn_set_fused_half_steps.argtypes = [i, ctypes.c_uint]
        lib.sinkhorn_attn_set_split_min_edges.restype = i
        lib.sinkhorn_attn_set_split_min_edges.argtypes = [ctypes.c_double]
        lib.sinkhorn_attn_step.restype = i
        lib.sinkhorn_attn_step.argtypes = [vp] * 14 + [i] * 7 + [f, i, f, i, vp, sz, vp]
        lib.sinkhorn_attn_step_static.restype = i
        lib.sinkhorn_attn_step_static.argtypes = [vp] * 14 + [i] * 7 + [f, i, f, i, vp]
        lib.sinkhorn_attn_profile_enable.restype = i
        lib.sinkhorn_attn_profile_enable.argtypes = [i]
        lib.sinkhorn_attn_profile_read.restype = i
        lib.sinkhorn_attn_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double),
                                                   ctypes.POINTER(ctypes.c_long)]
        lib.sinkhorn_attn_profile_read_phases.restype = i
        lib.sinkhorn_attn_profile_read_phases.argtypes = [ctypes.POINTER(ctypes.c_double),
                                                          ctypes.POINTER(ctypes.c_long)]
        lib.sinkhorn_attn_strerror.restype = ctypes.c_char_p
        lib.sinkhorn_attn_strerror.argtypes = [i]
        _lib = lib
    return _lib


class SinkhornAttnError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"sinkhorn_attn status {status}: {sinkhorn_attn_strerror(status)}")


def sinkhorn_attn_strerror(status: int) -> str:
    return load().sinkhorn_attn_strerror(int(status)).decode()


def sinkhorn_attn_probe_issue(tiles=4000, waves_per_simd=4):
    """Milliseconds of the eight issue-rate probe kernels (exp2 + add, MFMA, all three, MFMA + add,
    MFMA + exp2, add, and all three with all or half of the exponentials as a cubic on the plain
    ALUs) and the number of SIMDs they ran on."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    scratch = torch.empty(cus * waves_per_simd * 256, device="cuda", dtype=torch.float32)
    ms = (ctypes.c_double * 8)()
    rc = load().sinkhorn_attn_probe_issue(scratch.data_ptr(), scratch.numel() * 4, int(tiles), int(waves_per_simd), ms,
                                          _stream_ptr())
    if rc != SKA_OK:
        raise SinkhornAttnError(rc)
    return [ms[k] for k in range(8)], 4 * cus


def sinkhorn_attn_set_streams(n: int) -> None:
    """2 (default): a call on several problems runs half of its sweeps on the library's helper
    stream; 1: everything on the caller's stream."""
    rc = load().sinkhorn_attn_set_streams(int(n))
    if rc != SKA_OK:
        raise SinkhornAttnError(rc)


def sinkhorn_attn_set_fused_half_steps(mode: int, spin_limit: int = 0) -> None:
    """0 (default): one launch per half-step; 1: the tail's 2R half-steps in one launch; 2: all
    half-steps after the first in one launch.  spin_limit bounds the waits inside it (0: default)."""
    rc = load().sinkhorn_attn_set_fused_half_steps(int(mode), int(spin_limit))
    if rc != SKA_OK:
        raise SinkhornAttnError(rc)


def sinkhorn_attn_set_split_min_edges(edges: float) -> None:
    """Band edges per dispatch from which a call uses the helper stream (default 5e7; 0: always)."""
    rc = load().sinkhorn_attn_set_split_min_edges(float(edges))
    if rc != SKA_OK:
        raise SinkhornAttnError(rc)


def sinkhorn_attn_profile_enable(level) -> None:
    """0/False off, 1/True the scaling-sweep run of every forward, 2 every phase."""
    load().sinkhorn_attn_profile_enable(int(level))


def sinkhorn_attn_profile_read():
    """(elapsed milliseconds, half-step launches bracketed) since the last read."""
    ms, n = ctypes.c_double(0.0), ctypes.c_long(0)
    rc = load().sinkhorn_attn_profile_read(ctypes.byref(ms), ctypes.byref(n))
    if rc != SKA_OK:
        raise SinkhornAttnError(rc)
    return ms.value, n.value


SKA_PHASES = ("prescale", "first_half_step", "scaling_sweeps", "output_map", "rowdot", "dV",
              "matvec_chain", "final_sweeps")   # order of ska_phase in the header


def sinkhorn_attn_profile_read_phases():
    """{phase name: (elapsed milliseconds, sweep launches bracketed)} since the last read."""
    k = len(SKA_PHASES)
    ms, n = (ctypes.c_double * k)(), (ctypes.c_long * k)()
    rc = load().sinkhorn_attn_profile_read_phases(ms, n)
    if rc != SKA_OK:
        raise SinkhornAttnError(rc)
    return {name: (ms[j], n[j]) for j, name in enumerate(SKA_PHASES)}


def sinkhorn_attn_workspace_bytes(B, H, L, d, W, T, R=2, dustbin=False, dtype=SKA_BF16) -> int:
    return int(load().sinkhorn_attn_workspace_bytes(B, H, L, d, W, T, R, int(bool(dustbin)), dtype))


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SKA_F32
    if t.dtype == torch.bfloat16:
        return SKA_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _check(x: torch.Tensor, shape, dtype, name):
    if not x.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if tuple(x.shape) != tuple(shape) or x.dtype != dtype or not x.is_contiguous():
        raise ValueError(f"{name}: expected contiguous {tuple(shape)} {dtype}, got {tuple(x.shape)} {x.dtype}")


def _stream_ptr() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _marg_ptr(x, shape, name):
    if x is None:
        return None
    _check(x, shape, torch.float32, name)
    return x.data_ptr()


def _len_ptr(x, B, name):
    if x is None:
        return None
    _check(x, (B,), torch.int32, name)
    return x.data_ptr()


def sinkhorn_attn_fwd(Q, K, V, W, T, R=2, eps=1.0, dustbin=False, dustbin_score=0.0, O=None, UV=None,
                      workspace=None):
    """Forward. Q, K, V: [B,H,L,d] CUDA tensors (float32 or bfloat16).
    Returns (O [B,H,L,d], UV [B,H,2(R+1),L+dustbin] float32)."""
    return sinkhorn_attn_fwd_marginals(Q, K, V, None, None, W, T, R, eps, dustbin, dustbin_score, O, UV,
                                       workspace)


def sinkhorn_attn_fwd_marginals(Q, K, V, log_a, log_b, W, T, R=2, eps=1.0, dustbin=False, dustbin_score=0.0,
                                O=None, UV=None, workspace=None):
    """Forward with marginal targets: log_a, log_b [B,H,L] float32 CUDA tensors or None (unit)."""
    return sinkhorn_attn_fwd_varlen(Q, K, V, log_a, log_b, None, None, W, T, R, eps, dustbin, dustbin_score, O,
                                    UV, workspace)


def sinkhorn_attn_fwd_masked(Q, K, V, mask_q, mask_k, W, T, R=2, eps=1.0, log_a=None, log_b=None, O=None, UV=None,
                             workspace=None):
    """Forward with inactive tokens: mask_q, mask_k uint8 CUDA tensors [B,L] (nonzero = active) or
    None.  The backward calls take the returned UV as it is (inactive potentials are -inf)."""
    B, H, L, d = Q.shape
    for n, x in (("Q", Q), ("K", K), ("V", V)):
        _check(x, (B, H, L, d), Q.dtype, n)
    for n, x in (("mask_q", mask_q), ("mask_k", mask_k)):
        if x is not None:
            _check(x, (B, L), torch.uint8, n)
    O = torch.empty_like(Q) if O is None else O
    if UV is None:
        UV = torch.empty((B, H, 2 * (R + 1), L), device=Q.device, dtype=torch.float32)
    _check(O, (B, H, L, d), Q.dtype, "O")
    _check(UV, (B, H, 2 * (R + 1), L), torch.float32, "UV")
    code = _dtype_code(Q)
    if workspace is None:
        workspace = torch.empty(max(sinkhorn_attn_workspace_bytes(B, H, L, d, W, T, R, False, code), 16),
                                device=Q.device, dtype=torch.uint8)
    rc = load().sinkhorn_attn_fwd_masked(
        Q.data_ptr(), K.data_ptr(), V.data_ptr(), _marg_ptr(log_a, (B, H, L), "log_a"),
        _marg_ptr(log_b, (B, H, L), "log_b"), None if mask_q is None else mask_q.data_ptr(),
        None if mask_k is None else mask_k.data_ptr(), O.data_ptr(), UV.data_ptr(), B, H, L, d, W, T, R, float(eps),
        code, workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr())
    if rc != SKA_OK:
        raise SinkhornAttnError(rc)
    return O, UV


def sinkhorn_attn_fwd_eps_schedule(Q, K, V, W, eps_stage, T_stage, R=2, eps=1.0, dustbin=False,
                                   dustbin_score=0.0, log_a=None, log_b=None, len_q=None, len_k=None, O=None,
                                   UV=None, workspace=None):
    """Forward whose stopped base solve follows a continuation schedule: T_stage[s] steps at
    eps_stage[s] (non-increasing, ending at eps).  Returns (O, UV) as sinkhorn_attn_fwd."""
    n = len(eps_stage)
    sched = ((ctypes.c_float * max(n, 1))(*[float(x) for x in eps_stage]),
             (ctypes.c_int * max(n, 1))(*[int(x) for x in T_stage]))
    return sinkhorn_attn_fwd_varlen(Q, K, V, log_a, log_b, len_q, len_k, W, sum(int(x) for x in T_stage), R, eps,
                                    dustbin, dustbin_score, O, UV, workspace, _sched=(n,) + sched)


def sinkhorn_attn_fwd_varlen(Q, K, V, log_a, log_b, len_q, len_k, W, T, R=2, eps=1.0, dustbin=False,
                             dustbin_score=0.0, O=None, UV=None, workspace=None, _sched=None):
    """Forward of a padded batch: len_q, len_k are int32 CUDA tensors [B] (or None: L) with the valid
    lengths of the query and key sequences of each batch item; results beyond them are zeros."""
    B, H, L, d = Q.shape
    for n, x in (("Q", Q), ("K", K), ("V", V)):
        _check(x, (B, H, L, d), Q.dtype, n)
    Lp = L + int(bool(dustbin))
    if O is None:
        O = torch.empty_like(Q)
    if UV is None:
        UV = torch.empty((B, H, 2 * (R + 1), Lp), device=Q.device, dtype=torch.float32)
    _check(O, (B, H, L, d), Q.dtype, "O")
    _check(UV, (B, H, 2 * (R + 1), Lp), torch.float32, "UV")
    if workspace is None:
        need = sinkhorn_attn_workspace_bytes(B, H, L, d, W, T, R, dustbin, _dtype_code(Q))
        workspace = torch.empty(max(need, 16), device=Q.device, dtype=torch.uint8)
    head = (Q.data_ptr(), K.data_ptr(), V.data_ptr(), _marg_ptr(log_a, (B, H, L), "log_a"),
            _marg_ptr(log_b, (B, H, L), "log_b"), _len_ptr(len_q, B, "len_q"), _len_ptr(len_k, B, "len_k"),
            O.data_ptr(), UV.data_ptr(), B, H, L, d, W)
    tail = (R, float(eps), int(bool(dustbin)), float(dustbin_score), _dtype_code(Q), workspace.data_ptr(),
            workspace.numel() * workspace.element_size(), _stream_ptr())
    if _sched is not None:
        rc = load().sinkhorn_attn_fwd_eps_schedule(*head, _sched[0], ctypes.addressof(_sched[1]),
                                                   ctypes.addressof(_sched[2]), *tail)
        if rc != SKA_OK:
            raise SinkhornAttnError(rc)
        return O, UV
    rc = load().sinkhorn_attn_fwd_varlen(
        Q.data_ptr(), K.data_ptr(), V.data_ptr(), _marg_ptr(log_a, (B, H, L), "log_a"),
        _marg_ptr(log_b, (B, H, L), "log_b"), _len_ptr(len_q, B, "len_q"), _len_ptr(len_k, B, "len_k"),
        O.data_ptr(), UV.data_ptr(), B, H, L, d, W, T, R, float(eps),
        int(bool(dustbin)), float(dustbin_score), _dtype_code(Q), workspace.data_ptr(),
        workspace.numel() * workspace.element_size(), _stream_ptr())
    if rc != SKA_OK:
        raise SinkhornAttnError(rc)
    return O, UV


def sinkhorn_attn_base_vjp(Q, K, UV, eta, W, T, eps=1.0, dustbin=False, dustbin_score=0.0, log_a=None,
                           log_b=None, len_q=None, len_k=None, workspace=None, dQ=None, dK=None):
    """(D_x z_T)^T eta through the T-step base solve: UV [B,H,2(T+1),Lp] from
    sinkhorn_attn_fwd(T=0, R=T), eta [B,H,Lp] (the eta0 of a backward call).  Returns (dQ, dK)."""
    B, H, L, d = Q.shape
    _check(K, (B, H, L, d), Q.dtype, "K")
    Lp = L + int(bool(dustbin))
    _check(UV, (B, H, 2 * (T + 1), Lp), torch.float32, "UV")
    _check(eta, (B, H, Lp), torch.float32, "eta")
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(Q) if dK is None else dK
    for n, x in (("dQ", dQ), ("dK", dK)):
        _check(x, (B, H, L, d), Q.dtype, n)
    code = _dtype_code(Q)
    if workspace is None:
        need = sinkhorn_attn_workspace_bytes(B, H, L, d, W, 0, T, dustbin, code)
        workspace = torch.empty(max(need, 16), device=Q.device, dtype=torch.uint8)
    rc = load().sinkhorn_attn_base_vjp(
        Q.data_ptr(), K.data_ptr(), _marg_ptr(log_a, (B, H, L), "log_a"), _marg_ptr(log_b, (B, H, L), "log_b"),
        _len_ptr(len_q, B, "len_q"), _len_ptr(len_k, B, "len_k"), UV.data_ptr(), eta.data_ptr(), dQ.data_ptr(),
        dK.data_ptr(), B, H, L, d, W, T, float(eps), int(bool(dustbin)), float(dustbin_score), code,
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr())
    if rc != SKA_OK:
        raise SinkhornAttnError(rc)
    return dQ, dK


def sinkhorn_attn_fwd_dustbin_token(Q, K, V, q_db, k_db, v_db, W, T, R=2, eps=1.0, O=None, UV=None,
                                    workspace=None):
    """Forward with a learned dustbin token per side: q_db, k_db, v_db [B,H,d] float32.
    Returns (O [B,H,L,d], UV [B,H,2(R+1),L+1])."""
    B, H, L, d = Q.shape
    for n, x in (("Q", Q), ("K", K), ("V", V)):
        _check(x, (B, H, L, d), Q.dtype, n)
    for n, x in (("q_db", q_db), ("k_db", k_db), ("v_db", v_db)):
        _check(x, (B, H, d), torch.float32, n)
    O = torch.empty_like(Q) if O is None else O
    if UV is None:
        UV = torch.empty((B, H, 2 * (R + 1), L + 1), device=Q.device, dtype=torch.float32)
    _check(O, (B, H, L, d), Q.dtype, "O")
    _check(UV, (B, H, 2 * (R + 1), L + 1), torch.float32, "UV")
    code = _dtype_code(Q)
    if workspace is None:
        workspace = torch.empty(sinkhorn_attn_workspace_bytes(B, H, L, d, W, T, R, True, code), device=Q.device,
                                dtype=torch.uint8)
    rc = load().sinkhorn_attn_fwd_dustbin_token(
        Q.data_ptr(), K.data_ptr(), V.data_ptr(), q_db.data_ptr(), k_db.data_ptr(), v_db.data_ptr(), O.data_ptr(),
        UV.data_ptr(), B, H, L, d, W, T, R, float(eps), code, workspace.data_ptr(),
        workspace.numel() * workspace.element_size(), _stream_ptr())
    if rc != SKA_OK:
        raise SinkhornAttnError(rc)
    return O, UV


def sinkhorn_attn_bwd_dustbin_token(Q, K, V, q_db, k_db, v_db, O, dO, UV, W, T, R=2, eps=1.0, want_eta0=False,
                                    workspace=None):
    """Backward with learned dustbin tokens. Returns (dQ, dK, dV, dq_db, dk_db, dv_db[, eta0])."""
    B, H, L, d = Q.shape
    for n, x in (("Q", Q), ("K", K), ("V", V), ("O", O), ("dO", dO)):
        _check(x, (B, H, L, d), Q.dtype, n)
    for n, x in (("q_db", q_db), ("k_db", k_db), ("v_db", v_db)):
        _check(x, (B, H, d), torch.float32, n)
    _check(UV, (B, H, 2 * (R + 1), L + 1), torch.float32, "UV")
    dQ, dK, dV = (torch.empty_like(Q) for _ in range(3))
    dq, dk, dv = (torch.empty_like(q_db) for _ in range(3))
    code = _dtype_code(Q)
    if workspace is None:
        workspace = torch.empty(sinkhorn_attn_workspace_bytes(B, H, L, d, W, T, R, True, code), device=Q.device,
                                dtype=torch.uint8)
    eta0 = torch.empty((B, H, L + 1), device=Q.device, dtype=torch.float32) if want_eta0 else None
    rc = load().sinkhorn_attn_bwd_dustbin_token(
        Q.data_ptr(), K.data_ptr(), V.data_ptr(), q_db.data_ptr(), k_db.data_ptr(), v_db.data_ptr(), O.data_ptr(),
        dO.data_ptr(), UV.data_ptr(), dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), dq.data_ptr(), dk.data_ptr(),
        dv.data_ptr(), eta0.data_ptr() if want_eta0 else None, B, H, L, d, W, T, R, float(eps), code,
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr())
    if rc != SKA_OK:
        raise SinkhornAttnError(rc)
    return (dQ, dK, dV, dq, dk, dv, eta0) if want_eta0 else (dQ, dK, dV, dq, dk, dv)


def sinkhorn_attn_step(Q, K, V, dO, W, T, R=2, eps=1.0, dustbin=False, dustbin_score=0.0, log_a=None, log_b=None,
                       len_q=None, len_k=None, want_eta0=False, workspace=None, O=None, UV=None, dQ=None, dK=None,
                       dV=None):
    """Forward and backward in one call for a cotangent known beforehand.
    Returns (O, UV, dQ, dK, dV[, eta0])."""
    B, H, L, d = Q.shape
    for n, x in (("Q", Q), ("K", K), ("V", V), ("dO", dO)):
        _check(x, (B, H, L, d), Q.dtype, n)
    Lp = L + int(bool(dustbin))
    O = torch.empty_like(Q) if O is None else O
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(Q) if dK is None else dK
    dV = torch.empty_like(Q) if dV is None else dV
    if UV is None:
        UV = torch.empty((B, H, 2 * (R + 1), Lp), device=Q.device, dtype=torch.float32)
    for n, x in (("O", O), ("dQ", dQ), ("dK", dK), ("dV", dV)):
        _check(x, (B, H, L, d), Q.dtype, n)
    _check(UV, (B, H, 2 * (R + 1), Lp), torch.float32, "UV")
    code = _dtype_code(Q)
    if workspace is None:
        workspace = torch.empty(max(sinkhorn_attn_workspace_bytes(B, H, L, d, W, T, R, dustbin, code), 16),
                                device=Q.device, dtype=torch.uint8)
    eta0 = torch.empty((B, H, Lp), device=Q.device, dtype=torch.float32) if want_eta0 else None
    rc = load().sinkhorn_attn_step(
        Q.data_ptr(), K.data_ptr(), V.data_ptr(), dO.data_ptr(), _marg_ptr(log_a, (B, H, L), "log_a"),
        _marg_ptr(log_b, (B, H, L), "log_b"), _len_ptr(len_q, B, "len_q"), _len_ptr(len_k, B, "len_k"), O.data_ptr(),
        UV.data_ptr(), dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), eta0.data_ptr() if want_eta0 else None, B, H, L, d,
        W, T, R, float(eps), int(bool(dustbin)), float(dustbin_score), code, workspace.data_ptr(),
        workspace.numel() * workspace.element_size(), _stream_ptr())
    if rc != SKA_OK:
        raise SinkhornAttnError(rc)
    return (O, UV, dQ, dK, dV, eta0) if want_eta0 else (O, UV, dQ, dK, dV)


def sinkhorn_attn_step_static(Q, K, V, dO, O, UV, dQ, dK, dV, W, T, R=2, eps=1.0, dustbin=False, dustbin_score=0.0,
                              log_a=None, log_b=None, len_q=None, len_k=None, eta0=None):
    """sinkhorn_attn_step on the library's static scratch: the caller passes every output, nothing
    is allocated here or in the library.  Problems beyond SKA_STATIC_SCRATCH_BYTES raise
    SinkhornAttnError(SKA_ESTATIC)."""
    B, H, L, d = Q.shape
    for n, x in (("Q", Q), ("K", K), ("V", V), ("dO", dO), ("O", O), ("dQ", dQ), ("dK", dK), ("dV", dV)):
        _check(x, (B, H, L, d), Q.dtype, n)
    Lp = L + int(bool(dustbin))
    _check(UV, (B, H, 2 * (R + 1), Lp), torch.float32, "UV")
    if eta0 is not None:
        _check(eta0, (B, H, Lp), torch.float32, "eta0")
    rc = load().sinkhorn_attn_step_static(
        Q.data_ptr(), K.data_ptr(), V.data_ptr(), dO.data_ptr(), _marg_ptr(log_a, (B, H, L), "log_a"),
        _marg_ptr(log_b, (B, H, L), "log_b"), _len_ptr(len_q, B, "len_q"), _len_ptr(len_k, B, "len_k"), O.data_ptr(),
        UV.data_ptr(), dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), None if eta0 is None else eta0.data_ptr(), B, H,
        L, d, W, T, R, float(eps), int(bool(dustbin)), float(dustbin_score), _dtype_code(Q), _stream_ptr())
    if rc != SKA_OK:
        raise SinkhornAttnError(rc)
    return O, UV, dQ, dK, dV


def sinkhorn_attn_select_workspace_bytes(B, H, L, d, W, T, R_max, dustbin=False, dtype=SKA_BF16) -> int:
    return int(load().sinkhorn_attn_select_workspace_bytes(B, H, L, d, W, T, R_max, int(bool(dustbin)), dtype))


def sinkhorn_attn_select_tail_depth(Q, K, V, dO, W, T, R_max, tau, eps=1.0, dustbin=False, dustbin_score=0.0,
                                    log_a=None, log_b=None, len_q=None, len_k=None):
    """First tail depth R <= R_max whose certificate max|(D_x z_T)^T eta_R| is <= tau.
    Returns a dict: R (0 if none passes), e_absmax and eta_absmax (lists over the depths tried),
    and O, UV, dQ, dK, dV of the selected depth (of R_max if none passes)."""
    B, H, L, d = Q.shape
    for n, x in (("Q", Q), ("K", K), ("V", V), ("dO", dO)):
        _check(x, (B, H, L, d), Q.dtype, n)
    Lp = L + int(bool(dustbin))
    code = _dtype_code(Q)
    O, dQ, dK, dV = (torch.empty_like(Q) for _ in range(4))
    UV = torch.empty(B * H * 2 * (R_max + 1) * Lp, device=Q.device, dtype=torch.float32)
    need = sinkhorn_attn_select_workspace_bytes(B, H, L, d, W, T, R_max, dustbin, code)
    if need == 0:
        raise SinkhornAttnError(SKA_EUNSUPPORTED)
    ws = torch.empty(need, device=Q.device, dtype=torch.uint8)
    sel = ctypes.c_int(0)
    e, eta = (ctypes.c_float * R_max)(), (ctypes.c_float * R_max)()
    rc = load().sinkhorn_attn_select_tail_depth(
        Q.data_ptr(), K.data_ptr(), V.data_ptr(), dO.data_ptr(), _marg_ptr(log_a, (B, H, L), "log_a"),
        _marg_ptr(log_b, (B, H, L), "log_b"), _len_ptr(len_q, B, "len_q"), _len_ptr(len_k, B, "len_k"),
        O.data_ptr(), UV.data_ptr(), dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), B, H, L, d, W, T, R_max,
        float(eps), int(bool(dustbin)), float(dustbin_score), code, float(tau), ctypes.addressof(sel),
        ctypes.addressof(e), ctypes.addressof(eta), ws.data_ptr(), need, _stream_ptr())
    if rc != SKA_OK:
        raise SinkhornAttnError(rc)
    R = sel.value or R_max
    tried = [k for k in range(R_max) if e[k] >= 0.0]
    return dict(R=sel.value, e_absmax=[e[k] for k in tried], eta_absmax=[eta[k] for k in tried], O=O,
                UV=UV[:B * H * 2 * (R + 1) * Lp].view(B, H, 2 * (R + 1), Lp), dQ=dQ, dK=dK, dV=dV)


def sinkhorn_attn_bwd(Q, K, V, O, dO, UV, W, T, R=2, eps=1.0, dustbin=False, dustbin_score=0.0,
                      want_eta0=False, workspace=None, dQ=None, dK=None, dV=None):
    """Backward. Returns (dQ, dK, dV[, eta0])."""
    return sinkhorn_attn_bwd_marginals(Q, K, V, None, None, O, dO, UV, W, T, R, eps, dustbin, dustbin_score,
                                       want_eta0, workspace, dQ, dK, dV)


def sinkhorn_attn_bwd_marginals(Q, K, V, log_a, log_b, O, dO, UV, W, T, R=2, eps=1.0, dustbin=False,
                                dustbin_score=0.0, want_eta0=False, workspace=None, dQ=None, dK=None,
                                dV=None):
    """Backward with marginal targets (see sinkhorn_attn_fwd_marginals)."""
    return sinkhorn_attn_bwd_varlen(Q, K, V, log_a, log_b, None, None, O, dO, UV, W, T, R, eps, dustbin,
                                    dustbin_score, want_eta0, workspace, dQ, dK, dV)


def sinkhorn_attn_bwd_varlen(Q, K, V, log_a, log_b, len_q, len_k, O, dO, UV, W, T, R=2, eps=1.0,
                             dustbin=False, dustbin_score=0.0, want_eta0=False, workspace=None, dQ=None,
                             dK=None, dV=None):
    """Backward of a padded batch (see sinkhorn_attn_fwd_varlen)."""
    return sinkhorn_attn_bwd_variant(SKA_BWD_ONE_REFERENCE, Q, K, V, log_a, log_b, len_q, len_k, O, dO, UV, W,
                                     T, R, eps, dustbin, dustbin_score, want_eta0, workspace, dQ, dK, dV)


def sinkhorn_attn_bwd_variant(variant, Q, K, V, log_a, log_b, len_q, len_k, O, dO, UV, W, T, R=2, eps=1.0,
                              dustbin=False, dustbin_score=0.0, want_eta0=False, workspace=None, dQ=None,
                              dK=None, dV=None):
    """The backward with its final sweeps evaluated as SKA_BWD_ONE_REFERENCE (production),
    SKA_BWD_DIRECT (every plan factor by its own exponential) or SKA_BWD_ONE_REFERENCE_GENERIC."""
    B, H, L, d = Q.shape
    for n, x in (("Q", Q), ("K", K), ("V", V), ("O", O), ("dO", dO)):
        _check(x, (B, H, L, d), Q.dtype, n)
    Lp = L + int(bool(dustbin))
    _check(UV, (B, H, 2 * (R + 1), Lp), torch.float32, "UV")
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(Q) if dK is None else dK
    dV = torch.empty_like(Q) if dV is None else dV
    for n, x in (("dQ", dQ), ("dK", dK), ("dV", dV)):
        _check(x, (B, H, L, d), Q.dtype, n)
    code = _dtype_code(Q)
    need = sinkhorn_attn_workspace_bytes(B, H, L, d, W, T, R, dustbin, code)
    if workspace is None:
        workspace = torch.empty(max(need, 16), device=Q.device, dtype=torch.uint8)
    eta0 = torch.empty((B, H, Lp), device=Q.device, dtype=torch.float32) if want_eta0 else None
    rc = load().sinkhorn_attn_bwd_variant(
        int(variant), Q.data_ptr(), K.data_ptr(), V.data_ptr(), _marg_ptr(log_a, (B, H, L), "log_a"),
        _marg_ptr(log_b, (B, H, L), "log_b"), _len_ptr(len_q, B, "len_q"), _len_ptr(len_k, B, "len_k"),
        O.data_ptr(), dO.data_ptr(), UV.data_ptr(), dQ.data_ptr(),
        dK.data_ptr(), dV.data_ptr(), eta0.data_ptr() if want_eta0 else None, B, H, L, d, W, T, R,
        float(eps), int(bool(dustbin)), float(dustbin_score), code, workspace.data_ptr(),
        workspace.numel() * workspace.element_size(), _stream_ptr())
    if rc != SKA_OK:
        raise SinkhornAttnError(rc)
    return (dQ, dK, dV, eta0) if want_eta0 else (dQ, dK, dV)
