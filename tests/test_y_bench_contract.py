"""bench.py as the driver runs it: one JSON line with the agreed fields, timed over at least 1000
launches, the roofline object consistent with itself, the counter-derived traffic reported only
from a committed summary taken on the present kernel source, the CPU baseline on the whole call."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def line():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "1", "--steps", "20",
                        "--warmup", "5"], capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, "bench.py prints ONE line on stdout, got %d" % len(lines)
    return json.loads(lines[0])


def test_fields_of_the_contract(line):
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in line, key
    assert line["n_gpus"] == 1 and line["steps"] == 20 and line["warmup"] == 5
    assert line["higher_is_better"] is True and line["vs_baseline"] is None and line["data"] == "synthetic"
    assert line["config"]["workload"].startswith("configs[2]")
    assert "model" not in line["config"]
    assert line["unit"] == "KV tokens/s"
    # value = B (n_vis + n_text) / t
    c = line["config"]
    tokens = c["batch"] * (c["n_vis"] + c["n_text"])
    assert line["value"] == pytest.approx(tokens / (line["ms_per_step"] * 1e-3), rel=1e-9)


def test_timed_region_is_long_enough(line):
    assert line["timed_region"]["launches_between_events"] >= 1000
    # the host's wall clock per launch cannot be shorter than the device time by more than noise
    assert line["timed_region"]["host_wall_ms_per_launch"] >= 0.9 * line["ms_per_step"]


def test_roofline_object(line):
    r = line["roofline"]
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert r["frac"] == pytest.approx(r["achieved"] / r["peak"], rel=1e-12)
    # algorithmic bytes: 44 B per visual token and 512 B per text token per KV head, plus q and out
    c = line["config"]
    want = (c["batch"] * c["n_kv_heads"] * (c["n_vis"] * 44 + c["n_text"] * 512)
            + 2 * c["batch"] * c["n_q_heads"] * c["head_dim"] * 2)
    assert r["algorithmic_bytes_per_call"] == want == 319815680
    assert r["achieved"] == pytest.approx(want / (line["ms_per_step"] * 1e-3) / 1e9, rel=1e-9)
    assert 0.5 < r["frac"] < 1.0
    # the traffic figure comes from the committed counter summary and only while the kernel source
    # is the one the counters were read on; here it must be (a changed kernel needs new counters)
    assert r["traffic_source"].startswith("profiles/"), r["traffic_source"]
    assert r["traffic"] is not None and 1.0 <= r["traffic"] / want < 1.05


def test_cpu_baseline_is_the_whole_call_on_the_oracle(line):
    b = line["cpu_baseline"]
    assert b["kind"] == "oracle" and b["unit"] == "KV tokens/s"
    assert b["cores"] >= 1 and "whole call" in b["sample"]
    assert b["value"] > 0 and line["value"] / b["value"] > 100        # a GPU, not a fallback
    assert b["parity_rel_l2_whole_call"] <= 4e-4
