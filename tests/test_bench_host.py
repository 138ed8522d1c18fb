"""Host logic of bench.py (CPU): the counts its roofline figures are built from, against brute
force, the ceilings it prices the scaling sweep against, and the refusal of more than one GPU."""
import os
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from paper_2605_08123_amd.workloads import CONFIGS, Workload  # noqa: E402


@pytest.mark.parametrize("B,H,L,W", [(1, 1, 7, 0), (2, 3, 50, 4), (1, 2, 33, 40), (1, 1, 1, 5), (2, 1, 64, 63)])
def test_band_edges_against_brute_force(B, H, L, W):
    w = Workload("x", 0, B, H, L, 32, W, 1, 2, 1.0, "f32")
    i, j = np.meshgrid(np.arange(L), np.arange(L), indexing="ij")
    assert bench.edges(w) == float(B * H * np.count_nonzero(np.abs(i - j) <= W))


def test_paper_workload_counts():
    """The figures quoted for the benchmark workload: 268.8 M band edges and 138,412,032
    algorithmic bytes per scaling sweep ((4d + 8) bytes per token and head, bf16, d = 64)."""
    w = CONFIGS["paper"]
    assert (w.B, w.H, w.L, w.d, w.W, w.T, w.R, w.dtype) == (1, 2, 262144, 64, 256, 20, 2, "bf16")
    assert bench.edges(w) == 2 * (262144 * 513 - 256 * 257)
    assert bench.algorithmic_bytes_per_sweep(w) == 138412032
    # fp32 storage doubles the matrix bytes, not the two fp32 vectors
    w32 = Workload("x", 0, 1, 2, 1024, 64, 16, 1, 2, 1.0, "f32")
    assert bench.algorithmic_bytes_per_sweep(w32) == (2 * 64 * 4 + 8) * 1024 * 2


def test_phase_model_is_consistent():
    """Per phase: bytes per token-head and MFMA flops per band edge.  Every sweep reads its two
    operands at least once (2 d elements per token-head); the matrix sweeps read or write two more
    matrices and run a second product."""
    for dtype, be in (("bf16", 2), ("f32", 4)):
        for d in (32, 64, 128):
            m = bench.phase_model(Workload("x", 0, 1, 1, 256, d, 8, 1, 2, 1.0, dtype))
            assert m["scaling_sweeps"] == (2 * d * be + 8, 2 * d) == m["first_half_step"]
            assert m["matvec_chain"] == (2 * d * be + 16, 2 * d)
            assert m["output_map"] == (4 * d * be + 8, 4 * d)
            assert m["dV"][1] == 4 * d and m["final_sweeps"][1] == 6 * d
            assert m["prescale"] == (2 * d * be, 0) and m["rowdot"][1] == 0


def test_alu_ceiling():
    """Plain-ALU ceiling of the scaling sweep: one exp2 (four issue slots) and one add (one slot)
    per band edge on 256 CUs x 4 SIMDs x 32 lanes at 2.4 GHz."""
    assert bench.ALU_SLOTS_PER_S == 256 * 4 * 32 * 2.4e9
    assert abs(bench.ALU_PEAK_TFLOPS - 31.45728) < 1e-9
    # the published fp32 vector peak is the same slot rate with an FMA counted as two flops
    assert abs(2 * bench.ALU_SLOTS_PER_S / 1e12 - 157.3) < 0.05
    assert bench.HBM_PEAK_GBS == 8000.0 and bench.MFMA_PEAK_TFLOPS == {"bf16": 2500.0, "f32": 157.3}


def test_more_than_one_gpu_is_refused_before_anything_runs():
    env = dict(os.environ)
    env.pop("WORLD_SIZE", None)
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       env=env, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
    env["WORLD_SIZE"] = "2"
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, env=env,
                       timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr
