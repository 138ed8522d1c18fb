#!/usr/bin/env python3
"""Benchmark: fwd + bwd of banded Sinkhorn attention at the paper-scale single-device
configuration (B=1, H=2, L=262144, d=64, W=256, T=20, R=2, eps=0.5, bf16 storage,
fp32 accumulation) on one MI355X.  A step is one forward plus one backward over
one batch of seeded synthetic inputs that already sit in HBM.

Prints ONE JSON line: whole-job tokens/s, plus
  roofline     - the scaling-sweep kernel (Eq. 1-2; 2T+3 of the 51 launches of a
                 step are this one kernel) timed in place with HIP events on the
                 stream it runs on, against the plain-ALU ceiling that binds it, with
                 the HBM and MFMA fractions of the same launches beside it;
  phases       - every phase's launch time with its HBM and MFMA fractions;
  cpu_baseline - the fp64 CPU oracle timed on a bounded slice of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}   # dense matrix peak of the storage type's MFMA
# Plain-ALU ceiling of the scaling sweep: per band edge one exp2 and one add, nothing packed,
# nothing fused.  256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz = 78.6 T lane-issue-slots/s (the
# published 157.3 TFLOP/s fp32 vector peak is this times two for an FMA); an add takes one slot,
# v_exp_f32 four (quarter rate: 8 cycles per 64-wide wavefront against 2 for an add, both
# measured with two or more wavefronts on a SIMD), so the pair runs at 2 flop per 5 slots =
# 31.5 TFLOP/s at best.
ALU_SLOTS_PER_S = 256 * 4 * 32 * 2.4e9
ALU_PEAK_TFLOPS = ALU_SLOTS_PER_S * 2.0 / 5.0 / 1e12


def edges(w) -> float:
    """Band edges of the whole batch: |i-j| <= W, per (batch, head) problem L(2W+1) - W(W+1)."""
    Wc = min(w.W, w.L - 1)
    return float(w.N) * (w.L * (2 * Wc + 1) - Wc * (Wc + 1))


def phase_model(w):
    """Algorithmic HBM bytes per token-head and MFMA flops per band edge of one launch of each
    phase's kernel (every operand streamed once, scores recomputed, nothing of size L x W
    stored).  be = bytes per matrix element."""
    be, d = (4 if w.dtype == "f32" else 2), w.d
    return {
        "prescale": (2 * d * be, 0),
        "first_half_step": (2 * d * be + 8, 2 * d),
        "scaling_sweeps": (2 * d * be + 8, 2 * d),
        "output_map": (4 * d * be + 8, 4 * d),
        "rowdot": (2 * d * be + 4, 0),
        "dV": (5 * d * be + 12, 4 * d),
        "matvec_chain": (2 * d * be + 16, 2 * d),
        "final_sweeps": (5 * d * be + 40, 6 * d),
    }


def algorithmic_bytes_per_sweep(w) -> float:
    """One scaling sweep streams the two operand matrices once and reads one fp32 vector
    and writes one: (4d + 8) bytes per token and head for bf16 storage."""
    return phase_model(w)["scaling_sweeps"][0] * w.L * w.N


def cpu_baseline(w, budget_tokens: int):
    """Oracle as it stands on a slice of head 0 (first `budget_tokens` tokens)."""
    import oracle
    from paper_2605_08123_amd.workloads import make_inputs
    ws = w.scaled(B=1, H=1, L=budget_tokens)
    q, k, v, g = make_inputs(ws)
    t0 = time.perf_counter()
    oracle.band(q[0, 0], k[0, 0], v[0, 0], g[0, 0], ws.W, ws.T, ws.R, ws.eps, ws.dustbin, ws.dustbin_score)
    dt = time.perf_counter() - t0
    # one token of the metric carries H heads of work
    return {"value": budget_tokens / (dt * w.H), "unit": "tokens/s", "cores": oracle.threads(),
            "kind": "oracle",
            "sample": f"fp64 oracle fwd+bwd on one head, first {budget_tokens} tokens of the workload "
                      f"({dt:.2f} s); scaled by 1/H to the {w.H}-head token rate"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="paper")
    ap.add_argument("--backward", default="one_reference",
                    choices=["one_reference", "direct", "one_reference_generic"],
                    help="how the final sweeps of the backward obtain the plan factors (the last two are "
                         "comparators: every factor by its own exponential / Prop. 2 on the generic kernel)")
    ap.add_argument("--probe-issue", action="store_true",
                    help="also run the library's register-only issue-rate probe (exp2+add only, MFMA only, "
                         "both) and report cycles per tile and SIMD at the nominal clock")
    ap.add_argument("--streams", type=int, default=2, choices=[1, 2],
                    help="2 (the library's default): half of the problems' sweeps run on its helper stream")
    ap.add_argument("--separate-calls", action="store_true",
                    help="a step as two library calls (sinkhorn_attn_fwd, then the backward) instead of the "
                         "one-call step")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time its replays (the small workloads, whose "
                         "~50 launches of 10-20 us each are bound by the host's enqueue rate otherwise); the "
                         "scaling sweep is then timed in a short eager pass of its own")
    ap.add_argument("--fused", type=int, default=0, choices=[0, 1, 2],
                    help="fused half-steps (sinkhorn_attn_set_fused_half_steps): 1 the tail's 2R half-steps in one "
                         "launch, 2 all half-steps after the first in one launch")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-tokens", type=int, default=262144)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three 256 MiB device copies (a known-size kernel to scale "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings by)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (independent (batch, head) problems shard "
              "with no communication; nothing here launches a second rank). Use --gpus 1.", file=sys.stderr)
        return 2

    import torch

    import paper_2605_08123_amd as ska
    from paper_2605_08123_amd.workloads import CONFIGS, make_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    w = CONFIGS[args.workload]
    dev = torch.device("cuda:0")
    td = torch.float32 if w.dtype == "f32" else torch.bfloat16
    Q, K, V, G = (torch.from_numpy(x).to(dev).to(td) for x in make_inputs(w))
    O = torch.empty_like(Q)
    UV = torch.empty((w.B, w.H, 6, w.L + int(w.dustbin)), device=dev, dtype=torch.float32)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(Q), torch.empty_like(Q)
    code = 0 if w.dtype == "f32" else 1
    wsb = ska.sinkhorn_attn_workspace_bytes(w.B, w.H, w.L, w.d, w.W, w.T, w.R, w.dustbin, code)
    wsp = torch.empty(wsb, device=dev, dtype=torch.uint8)

    ska.sinkhorn_attn_set_streams(args.streams)
    ska.sinkhorn_attn_set_fused_half_steps(args.fused)
    variant = {"one_reference": 0, "direct": 1, "one_reference_generic": 2}[args.backward]

    def step():
        if not args.separate_calls and variant == 0:
            ska.sinkhorn_attn_step(Q, K, V, G, w.W, w.T, w.R, w.eps, w.dustbin, w.dustbin_score, workspace=wsp, O=O,
                                   UV=UV, dQ=dQ, dK=dK, dV=dV)
            return
        ska.sinkhorn_attn_fwd(Q, K, V, w.W, w.T, w.R, w.eps, w.dustbin, w.dustbin_score, O=O, UV=UV,
                              workspace=wsp)
        ska.sinkhorn_attn_bwd_variant(variant, Q, K, V, None, None, None, None, O, G, UV, w.W, w.T, w.R, w.eps,
                                      w.dustbin, w.dustbin_score, workspace=wsp, dQ=dQ, dK=dK, dV=dV)

    if args.calibrate_copy:
        src = torch.empty(256 << 20, device=dev, dtype=torch.uint8).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()                              # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        # the sweep's launch time: HIP events cannot sit inside a replayed graph, so a few eager steps
        ska.sinkhorn_attn_profile_enable(1)
        for _ in range(min(args.steps, 3)):
            step()
        torch.cuda.synchronize()
    else:
        # level 1: two events per forward call around its run of identical scaling sweeps, on the
        # streams the sweeps run on; the schedule of the call is unchanged
        ska.sinkhorn_attn_profile_enable(1)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    ska.sinkhorn_attn_profile_enable(0)
    sweep_ms, launches = ska.sinkhorn_attn_profile_read()
    # per-phase times from a short pass of their own (two events per phase are too many to
    # leave in the timed region)
    psteps = min(args.steps, 3)
    ska.sinkhorn_attn_profile_enable(2)
    tp0 = time.perf_counter()
    for _ in range(psteps):
        step()
    torch.cuda.synchronize()
    pdt = time.perf_counter() - tp0
    ska.sinkhorn_attn_profile_enable(0)
    ph = ska.sinkhorn_attn_profile_read_phases()

    # forward and backward apart (a few untimed-region steps each)
    def timed(fn, n=3):
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t) / n
    fwd_ms = timed(lambda: ska.sinkhorn_attn_fwd(Q, K, V, w.W, w.T, w.R, w.eps, w.dustbin, w.dustbin_score, O=O, UV=UV,
                                                 workspace=wsp))
    bwd_ms = timed(lambda: ska.sinkhorn_attn_bwd_variant(variant, Q, K, V, None, None, None, None, O, G, UV, w.W, w.T,
                                                         w.R, w.eps, w.dustbin, w.dustbin_score, workspace=wsp, dQ=dQ,
                                                         dK=dK, dV=dV))

    ms_per_step = 1e3 * dt / args.steps
    tokens_per_s = w.B * w.L * args.steps / dt
    avg_s = 1e-3 * sweep_ms / max(launches, 1)
    achieved = algorithmic_bytes_per_sweep(w) / avg_s / 1e9
    # HBM bytes per sweep beyond L2: not measurable from inside this process (rocprofv3 --pmc reads
    # FETCH_SIZE / WRITE_SIZE in runs of their own); the stored reading of those runs, with its source
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", f"lse_sweep_{w.name}_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            tj = json.load(f)
        traffic = tj.get("hbm_bytes_per_launch")
        traffic_source = (f"stored reading, profiles/lse_sweep_{w.name}_traffic.json (rocprofv3 --pmc FETCH_SIZE, "
                          f"WRITE_SIZE on build {tj.get('build', 'unrecorded')}); not re-measured in this run")
    dt_name = "bf16" if w.dtype == "bf16" else "f32"
    E = edges(w)
    model = phase_model(w)
    phases = {}
    for name, (ms, n) in ph.items():
        if n == 0:
            continue
        t = 1e-3 * ms / n                      # seconds per launch
        b, fl = model[name]
        phases[name] = {"launches": n, "avg_launch_us": 1e6 * t, "share_of_step": 1e-3 * ms / pdt,
                        "hbm_frac": b * w.L * w.N / t / 1e9 / HBM_PEAK_GBS,
                        "mfma_frac": fl * E / t / 1e12 / MFMA_PEAK_TFLOPS[dt_name]}
    alu_tflops = 2.0 * E / avg_s / 1e12
    out = {
        "metric": f"fwd+bwd tokens/sec at L={w.L} d={w.d} W={w.W} T={w.T} R={w.R}; % MFMA / HBM peak",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dt_name, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "L": w.L, "d": w.d, "W": w.W, "T": w.T,
                   "R": w.R, "eps": w.eps, "dustbin": w.dustbin, "backward": args.backward,
                   "streams": args.streams, "calls_per_step": 2 if (args.separate_calls or variant) else 1,
                   "graph_replay": bool(args.graph), "fused_half_steps": args.fused},
        # the scaling sweep against its three ceilings; the one that binds (the largest lower bound on
        # a launch's time: 17.1 us ALU, 17.3 us HBM, 13.8 us MFMA at the paper workload) is the plain-ALU
        # issue rate of one exp2 and one add per band edge
        "roofline": {"kernel": "scaling sweep (row/column half-step, Eq. 1-2)", "bound": "alu",
                     "achieved": alu_tflops, "peak": ALU_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": alu_tflops / ALU_PEAK_TFLOPS, "traffic": traffic, "traffic_source": traffic_source,
                     "flops": "one exp2 + one add per band edge; v_exp_f32 issues at quarter rate",
                     "launches_timed": launches, "avg_launch_us": 1e6 * avg_s,
                     "hbm": {"achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": achieved / HBM_PEAK_GBS,
                             "algorithmic_bytes_per_launch": algorithmic_bytes_per_sweep(w)},
                     "mfma": {"achieved": 2 * w.d * E / avg_s / 1e12, "peak": MFMA_PEAK_TFLOPS[dt_name],
                              "unit": "TFLOP/s", "frac": 2 * w.d * E / avg_s / 1e12 / MFMA_PEAK_TFLOPS[dt_name]}},
        "phases": phases,
        # the same run in other units: per (token, head), per band edge and sweep (2(T+R) half-steps,
        # the output map and six backward sweeps), and the two directions apart
        "extra": {"head_tokens_per_s": tokens_per_s * w.H, "edge_sweeps_per_s": E * (2 * (w.T + w.R) + 7) / (dt / args.steps),
                  "fwd_ms": fwd_ms, "bwd_ms": bwd_ms},
    }
    # What a SIMD sustains of the sweep's own instruction mix (register-only probe kernels in the
    # library: 16 exp2 + 16 adds and four 32x32x16 bf16 MFMAs per 32 x 32 tile, four wavefronts per
    # SIMD as in the sweep): MFMA and VALU work of different wavefronts overlap only in part, so this
    # measured rate, not either unit's peak, is what the sweep's inner loop can reach.
    tiles = 4000
    ms3, simds = ska.sinkhorn_attn_probe_issue(tiles, 4)
    tile_s = {k: 1e-3 * t / (tiles * 4) for k, t in zip(("valu_only", "mfma_only", "both"), ms3)}
    issue_peak = simds * 1024.0 * 1.0 / tile_s["both"] if w.d == 64 and dt_name == "bf16" else None
    out["roofline"]["issue"] = {
        "probe_ns_per_tile_and_simd": {k: 1e9 * v for k, v in tile_s.items()},
        "achieved": E / avg_s / 1e12, "peak": None if issue_peak is None else issue_peak / 1e12,
        "unit": "T band edges/s", "frac": None if issue_peak is None else E / avg_s / issue_peak,
        "note": "peak = SIMDs x 1024 edges per tile / measured time of one probe tile (d = 64 bf16 mix)"}
    if args.probe_issue:
        probe = {}
        for wps in (1, 2, 4, 8):
            ms, _ = ska.sinkhorn_attn_probe_issue(tiles, wps)
            # cycles one SIMD spends per tile of one wavefront, at the nominal 2.4 GHz
            probe[f"waves_per_simd_{wps}"] = {k: round(1e-3 * t * 2.4e9 / (tiles * wps), 1) for k, t in
                                              zip(("exp_add", "mfma", "mfma_exp_add", "mfma_add", "mfma_exp", "add", "mfma_polyexp_add",
                                                   "mfma_halfpolyexp_add"), ms)}
        out["issue_probe_cycles_per_tile"] = probe
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, min(args.cpu_tokens, w.L))
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
