"""MI355X-native banded Sinkhorn attention (forward + exact surrogate backward).

`binding` is the thin ctypes layer over the C ABI of include/sinkhorn_attn.h;
`workloads` holds the seeded synthetic inputs; `build` compiles the library.
"""
from .binding import (SinkhornAttnError, sinkhorn_attn_base_vjp, sinkhorn_attn_bwd,
                      sinkhorn_attn_bwd_dustbin_token, sinkhorn_attn_fwd_dustbin_token, sinkhorn_attn_bwd_marginals,  # noqa: F401
                      sinkhorn_attn_bwd_variant, sinkhorn_attn_bwd_varlen, sinkhorn_attn_fwd, sinkhorn_attn_fwd_marginals,
                      sinkhorn_attn_fwd_eps_schedule, sinkhorn_attn_fwd_masked, sinkhorn_attn_fwd_varlen,
                      sinkhorn_attn_probe_issue, sinkhorn_attn_profile_enable, sinkhorn_attn_profile_read,
                      sinkhorn_attn_profile_read_phases,
                      sinkhorn_attn_select_tail_depth, sinkhorn_attn_select_workspace_bytes, sinkhorn_attn_set_fused_half_steps, sinkhorn_attn_set_split_min_edges, sinkhorn_attn_set_streams, sinkhorn_attn_step,
                      sinkhorn_attn_step_static,
                      sinkhorn_attn_strerror, sinkhorn_attn_workspace_bytes)
