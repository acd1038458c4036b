"""The benchmark script end to end on the GPU, with few steps: one JSON line with the keys its readers rely on."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
pytestmark = pytest.mark.gpu


def _run(*extra):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "5", "--warmup", "2",
                        "--event-calls", "6", "--cpu-seconds", "0.5", "--cpu-seqs", "8", "--naive-steps", "2", *extra],
                       capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    return json.loads(lines[0])


def test_default_line_carries_roofline_cpu_baseline_and_all_workloads():
    d = _run()
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "parity", "other_workloads"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["vs_baseline"] is None and d["parity"]["ok"]
    assert d["config"]["workload"].startswith("vlm7b")
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9 and 0.3 < r["frac"] < 1.0
    assert r["event_timed_calls"] == 6 and r["streaming_read_ceiling_GBps"] > 4000
    assert r["traffic"] is None or r["traffic"] > r["kernel_algorithmic_bytes"]
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["value"] > 0 and c["cores"] >= 1
    assert set(d["other_workloads"]) == {"tiny", "vlm3b", "agentic", "highbatch"}
    for name, o in d["other_workloads"].items():
        assert o["parity"]["ok"], name
        assert o["ms_per_step"] > 0 and o["algorithmic_bytes"]["total"] > 0


@pytest.mark.parametrize("extra", [("--op", "tree"), ("--op", "token_logprob", "--rows", "64"),
                                   ("--workload", "agentic", "--page-size", "64", "--finished", "0.25"),
                                   ("--workload", "vlm3b", "--kv", "e4m3")])
def test_other_modes_run(extra):
    d = _run(*extra)
    assert d["ms_per_step"] > 0 and d["n_gpus"] == 1
    assert d["parity"]["ok"] if isinstance(d.get("parity"), dict) and "ok" in d["parity"] else True
