"""bench.py's one JSON line: the keys the driver reads, on a small workload (a child process;
the GPU is used by one process at a time)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args, timeout=300):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=timeout, cwd=ROOT)


@pytest.mark.timeout(400)
def test_one_json_line_with_the_contract_keys():
    run = _bench("--workload", "cfg1", "--only", "--steps", "20", "--warmup", "5")
    assert run.returncode == 0, run.stderr[-2000:]
    lines = [ln for ln in run.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, lines
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 20 and d["warmup"] == 5 and d["unit"] == "tokens/s"
    assert d["higher_is_better"] is True and d["vs_baseline"] is None and d["data"] == "synthetic" and d["dtype"] == "bf16"
    assert d["config"]["workload"].startswith("cfg1:") and "model" not in d["config"]
    assert abs(d["value"] - 4 * 2048 / (d["ms_per_step"] * 1e-3)) <= 1e-6 * d["value"]       # tokens = B * L
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12 and 0 < r["frac"] < 1
    assert r["traffic"] is None or r["traffic"] > 0
    assert r["kernel_name"] in d["config"]["launches"]
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and c["unit"] == "tokens/s" and c["sample"]
    assert d["parity_on_sample"]["rel_l2_O"] <= 2e-2 and d["parity_on_sample"]["rel_l2_S_L"] <= 2e-2
    assert d["ms_per_step_first_pass"] > 0 and d["settle_steps"] >= 0


def test_more_than_one_gpu_is_refused():
    run = _bench("--gpus", "2", timeout=60)
    assert run.returncode != 0 and "ONE GPU" in run.stderr and not run.stdout.strip()
