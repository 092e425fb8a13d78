"""bench.py contract: what can be checked without a GPU, and the output of a short run on one."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""


@pytest.mark.gpu
def test_bench_prints_one_json_line_with_the_contract_keys():
    """A short run of the default workload: one JSON line on stdout, the keys of the contract,
    roofline and cpu_baseline filled in, the step consistent with its parts."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "6", "--warmup", "2",
                        "--layers", "2", "--pipeline-layers", "2"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    rec = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in rec, key
    assert rec["n_gpus"] == 1 and rec["steps"] == 6 and rec["warmup"] == 2 and rec["vs_baseline"] is None
    assert rec["dtype"] == "bf16" and rec["higher_is_better"] is True and "workload" in rec["config"]
    roof = rec["roofline"]
    assert roof["bound"] == "mfma" and roof["unit"] == "TFLOP/s" and roof["peak"] == 2500.0
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-4 and 0.05 < roof["frac"] < 1.0
    cpu = rec["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
    # a step is the attention launch plus linking: never shorter than the attention alone
    assert rec["ms_per_step"] >= 0.98 * roof["avg_launch_ms"]
    assert abs(rec["value"] - rec["attention"]["flops"] / (rec["ms_per_step"] * 1e-3) / 1e12) < 0.5
    for tier in ("disk", "host", "hbm"):
        assert rec["layer_pipeline"][tier]["ms_per_layer"] > 0
    # the clock sample is there when the box has the tool, and then below the peak's 2.4 GHz
    state = rec["device_state"]
    assert state is None or 100 < state["sclk_mhz_under_attention"] <= 2400
