"""bench.py's one JSON line (GPU): the keys the driver reads, on the small workload so that the
run takes seconds.  The numbers themselves are not asserted beyond being positive and consistent."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*flags):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *flags], capture_output=True, text=True,
                       timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines   # exactly one line on stdout
    return json.loads(lines[0])


def test_bench_line_small_workload():
    out = run_bench("--workload", "tiny", "--steps", "3", "--warmup", "1", "--cpu-tokens", "256")
    print(f"\n[case] bench.py --workload tiny: {out['ms_per_step']:.3f} ms/step", flush=True)
    assert out["unit"] == "tokens/s" and out["n_gpus"] == 1 and out["steps"] == 3 and out["warmup"] == 1
    assert out["higher_is_better"] is True and out["scaling"] == "weak" and out["vs_baseline"] is None
    assert out["dtype"] == "f32" and out["data"] == "synthetic" and out["config"]["workload"] == "tiny"
    assert "model" not in out["config"]
    assert out["value"] > 0 and out["ms_per_step"] > 0
    # value is tokens (B L) per second of the timed region
    assert abs(out["value"] * out["ms_per_step"] * 1e-3 / (out["config"]["B"] * out["config"]["L"]) - 1.0) < 1e-6
    rf = out["roofline"]
    assert rf["bound"] in ("alu", "hbm", "mfma") and rf["unit"] in ("TFLOP/s", "GB/s")
    assert rf["peak"] > 0 and rf["achieved"] > 0 and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9
    assert "traffic" in rf and "traffic_source" in rf and rf["launches_timed"] > 0 and rf["avg_launch_us"] > 0
    cb = out["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["unit"] == "tokens/s" and cb["value"] > 0 and cb["cores"] >= 1 and cb["sample"]


def test_bench_flags_are_reported():
    out = run_bench("--workload", "tiny", "--steps", "2", "--warmup", "1", "--no-cpu-baseline", "--streams", "1",
                    "--separate-calls")
    assert out["config"]["streams"] == 1 and out["config"]["calls_per_step"] == 2 and "cpu_baseline" not in out
