"""bench.py's command line and its one JSON line: the parts that need no GPU here, the line itself
on a GPU (the smallest bf16 workload, two timed steps)."""
import json
import subprocess
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent


def _bench(*args, timeout=600):
    return subprocess.run([sys.executable, str(ROOT / "bench.py"), *args], cwd=ROOT, capture_output=True, text=True,
                          timeout=timeout)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _bench("--gpus", "2")
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_unknown_workload_is_an_argument_error():
    r = _bench("--workload", "no_such_workload")
    assert r.returncode != 0 and r.stdout.strip() == ""


@pytest.mark.gpu
def test_one_json_line_with_the_agreed_fields():
    r = _bench("--workload", "wan1p3b_480p", "--steps", "2", "--warmup", "1")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 2 and out["warmup"] == 1
    assert out["higher_is_better"] is True and out["vs_baseline"] is None
    assert out["dtype"] == "bf16" and out["data"] == "synthetic" and out["unit"] == "TFLOP/s"
    assert out["config"]["workload"] == "wan1p3b_480p" and "model" not in out["config"]
    assert out["value"] > 0 and out["ms_per_step"] > 0
    roof = out["roofline"]
    assert roof["bound"] in ("hbm", "mfma", "alu") and roof["unit"] in ("GB/s", "TFLOP/s")
    assert roof["peak"] > 0 and abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9
    assert "traffic" in roof and roof["traffic_source"]   # a tracked counter record, or the reason there is none
    assert set(out["config"]["route"]) >= {"stage1", "stages23", "q", "k"}
    assert "sclk_mhz" in out["diagnostics"]
    cpu = out["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"] and cpu["unit"]
