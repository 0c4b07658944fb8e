"""The benchmark's command-line contract: one JSON line with the agreed fields (GPU), and a clear
refusal of more than one GPU (no GPU needed for that)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
def test_default_run_prints_one_json_line_with_roofline_and_cpu_baseline():
    """The default workload list end to end (every variant, the oracle baseline, the AdamW rest), two
    timed steps: the fields the harness reads must all be there."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "2", "--warmup", "1"],
                       capture_output=True, text=True, timeout=900, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["unit"] == "params/s"
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and d["higher_is_better"] is True
    assert d["value"] > 1e10 and d["ms_per_step"] > 0 and d["finite"] is True
    assert "llama7b_mini" in d["config"]["workload"]
    roof = d["roofline"]
    assert roof["bound"] in ("hbm", "mfma", "alu") and roof["peak"] > 0 and roof["unit"] in ("GB/s", "TFLOP/s")
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9 and 0.3 < roof["frac"] < 1.0
    assert roof["traffic"] is None or roof["traffic"] > 0
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["value"] > 0 and cpu["cores"] >= 1 and cpu["sample"]
    # four variants on the LLaMA-7B shapes, then the LLaMA-60M and LLaMA-1B sets and the two LLaMA-13B runs (five
    # timed steps whatever --steps says, the first of them re-sampling P)
    assert len(d["also"]) == 8 and all(a["finite"] and a["value"] > 1e10 for a in d["also"])
    assert [a["benchmark_config"] for a in d["also"]] == [4, 4, 4, 4, 2, 3, 5, 5]
    for a in d["also"][6:]:
        assert a["first_timed_step"] == 201 and a["phase_ms"]["update"] > 0
    assert d["also"][7]["phase_ms"]["projection_fill"] > 0          # the re-sampling step is inside the timed region
    assert d["adamw_rest"]["value"] > 1e9
