"""The benchmark's command line contract: one GPU only, and one JSON line with the agreed fields."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_with_a_message():
    done = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True, timeout=300)
    assert done.returncode != 0
    assert "ONE GPU" in (done.stderr + done.stdout)
    assert not any(line.startswith("{") for line in done.stdout.splitlines())      # and no result line


@pytest.mark.gpu
def test_small_run_prints_one_json_line_with_roofline_and_cpu_baseline():
    done = subprocess.run([sys.executable, BENCH, "--small", "--steps", "3", "--warmup", "1", "--cpu-sample-elems", "200000"],
                          capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert done.returncode == 0, done.stderr[-2000:]
    lines = [line for line in done.stdout.splitlines() if line.startswith("{")]
    assert len(lines) == 1
    rec = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in rec, key
    assert rec["n_gpus"] == 1 and rec["steps"] == 3 and rec["warmup"] == 1 and rec["data"] == "synthetic"
    assert rec["value"] > 0 and rec["ms_per_step"] > 0 and "workload" in rec["config"] and "model" not in rec["config"]
    roof = rec["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert roof["frac"] == pytest.approx(roof["achieved"] / roof["peak"], abs=1e-3)
    cpu = rec["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in cpu, key
    assert cpu["kind"] == "oracle" and cpu["value"] > 0 and cpu["cores"] >= 1


def test_counter_traffic_is_quoted_only_for_the_sources_it_was_measured_on(tmp_path, monkeypatch):
    # `roofline.traffic` comes from the counter summary under profiles/: a line counts when its fingerprint is that of
    # the kernel sources in the tree, and any other line (or a missing file) gives None -- never a stale figure
    sys.path.insert(0, ROOT)
    import bench
    now = bench.kernel_source_hash()
    assert len(now) == 16 and now == bench.kernel_source_hash()
    summary = tmp_path / "hbm_traffic.md"
    summary.write_text("some text\n"
                       "traffic k_a fetch_bytes=1000 write_bytes=24 sources=%s\n"
                       "traffic k_b fetch_bytes=5 write_bytes=6 sources=0123456789abcdef\n" % now)
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(summary))
    assert bench.measured_traffic("k_a") == 1024
    assert bench.measured_traffic("k_b") is None          # measured on other sources
    assert bench.measured_traffic("k_c") is None          # no such line
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(tmp_path / "absent.md"))
    assert bench.measured_traffic("k_a") is None
    # the tracked summary parses: every line has the four fields
    import re
    text = open(os.path.join(ROOT, "profiles", "hbm_traffic.md")).read()
    lines = [ln for ln in text.splitlines() if ln.startswith("traffic ")]
    assert len(lines) >= 8
    for ln in lines:
        assert re.match(r"^traffic\s+\S+\s+fetch_bytes=\d+\s+write_bytes=\d+\s+sources=\w{16}$", ln), ln
