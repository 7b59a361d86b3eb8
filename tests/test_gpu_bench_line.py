"""bench.py end to end on the GPU at a small workload: exactly one JSON line with the fields of the
measurement contract (metric, value, roofline with a measured kernel time, CPU baseline from the
oracle, the sustained MFMA rates measured in the same run)."""
import json
import pathlib
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = pathlib.Path(__file__).resolve().parents[1]


def test_one_json_line_with_roofline_and_cpu_baseline():
    r = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--config", "2", "--steps", "2", "--warmup", "1",
                        "--cpu-sample-tokens", "2048"], capture_output=True, text=True, cwd=ROOT, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["unit"] == "TFLOP/s" and d["dtype"] == "bf16"
    assert d["vs_baseline"] is None and d["higher_is_better"] is True and "workload" in d["config"]
    roof = d["roofline"]
    assert roof["bound"] == "mfma" and roof["unit"] == "TFLOP/s" and roof["kernel"] == "dkdv"
    assert roof["peak"] == pytest.approx(d["peak_tflops_denominator"]) and 2000 < roof["peak"] < 3000
    assert roof["frac"] == pytest.approx(roof["achieved"] / roof["peak"]) and 0.05 < roof["frac"] < 1.0
    assert roof["achieved"] == pytest.approx(roof["flops_per_launch"] / (roof["avg_launch_ms"] * 1e-3) / 1e12, rel=1e-6)
    assert roof["traffic"] is None            # HBM counters exist for the metric's workload only
    # the value follows from the step time and the counted FLOPs of the workload (14 * D per unmasked pair)
    c = d["config"]
    flops = 14 * c["D"] * (c["S"] * (c["S"] + 1) // 2) * c["B"] * c["H"]
    assert d["value"] == pytest.approx(flops / (d["ms_per_step"] * 1e-3) / 1e12, rel=1e-6)
    assert sum(d["kernel_ms"].values()) <= d["ms_per_step"] * 1.02
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["unit"] == "TFLOP/s" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
    sus = d["sustained_mfma_tflops_measured"]
    assert sus["random_operands_forward_mix"] < sus["random_operands_backward_mix"] * 1.02
    assert sus["random_operands_backward_mix"] < sus["random_operands"] * 1.02 <= sus["constant_operands"] * 1.05
    assert set(d["executed_frac_of_mix_probe"]) == {"fwd", "dkdv", "dq"}
