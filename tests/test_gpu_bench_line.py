"""bench.py under the command line the harness uses: one JSON line with the agreed keys."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_driver_command_line_prints_one_complete_json_line():
    import torch
    torch.cuda.empty_cache()                      # the child needs 60 GB of its own
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "1", "--steps", "20", "--warmup", "5",
           "--cpu-seconds", "2", "--extras", "off"]
    r = subprocess.run(cmd, cwd=ROOT, capture_output=True, text=True, timeout=500)
    assert r.returncode == 0, r.stderr[-3000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, r.stdout[-2000:]
    d = json.loads(lines[0])
    assert d["metric"].startswith("sampled transitions/s") and d["unit"] == "transitions/s"
    assert (d["n_gpus"], d["steps"], d["warmup"], d["steps_requested"], d["warmup_requested"]) == (1, 100, 100, 20, 5)
    assert d["higher_is_better"] is True and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert d["dtype"] == "u64" and "model" not in d["config"] and d["config"]["workload"].startswith("atari")
    assert 1e6 < d["value"] < 1e9 and abs(d["value"] * d["ms_per_step"] * 1e-3 / 512 - 1.0) < 1e-6
    roof = d["roofline"]
    assert roof["bound"] == "hbm" and roof["unit"] == "GB/s" and roof["peak"] == 8000.0
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9 and 0.2 < roof["frac"] < 1.0
    assert roof["bytes_per_launch"] == 512 * 57030 and roof["traffic"] > roof["bytes_per_launch"]
    assert abs(roof["achieved"] - roof["bytes_per_launch"] / (roof["us_per_launch"] * 1e-6) / 1e9) < 1e-6
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] == 1 and cpu["value"] > 0 and cpu["cpu_model"] and cpu["sample"]
    assert d["hbm_frac_of_step"]["bytes_per_step"] == roof["bytes_per_launch"]
