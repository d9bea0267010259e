"""The contract of bench.py: what it refuses, and the shape of the one JSON line it prints."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def _run(*args, timeout=600):
    return subprocess.run([sys.executable, BENCH, *args], cwd=ROOT, capture_output=True, text=True, timeout=timeout)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_follow_the_stated_formulas():
    sys.path.insert(0, ROOT)
    import bench
    Bs, B, S, K, out = 1000, 990, 62, 40, 2560
    assert bench.algorithmic_bytes("unstuff_count", Bs, B, S, K, out) == Bs
    assert bench.algorithmic_bytes("unstuff_scatter", Bs, B, S, K, out) == Bs + B
    assert bench.algorithmic_bytes("sync_intra", Bs, B, S, K, out) == B + 8 * S
    assert bench.algorithmic_bytes("write", Bs, B, S, K, out) == B + 8 * S + 128 * K
    assert bench.algorithmic_bytes("pixels", Bs, B, S, K, out) == 128 * K + out
    assert bench.HBM_PEAK_GBS == 8000.0


def test_traffic_figures_come_from_the_committed_profile_summaries():
    """bench.py takes the measured HBM traffic per kernel from the rocprofv3 summaries in profiles/ (no figures of
    its own), and marks them stale when the kernel sources have changed since the summary was made."""
    sys.path.insert(0, ROOT)
    import bench
    for c, name in bench.PROFILE_FILES.items():
        path = os.path.join(ROOT, "profiles", name)
        traffic, stale = bench.profile_traffic(c)
        if not os.path.isfile(path):
            assert traffic == {} and stale is None
            continue
        assert stale in (True, False)
        for k in ("sync_intra", "write", "pixels"):
            assert traffic[k] > 0
        issue = bench.profile_issue(c)      # share of the vector issue slots, lanes switched on: from the same summary
        for k in ("sync_intra", "write", "pixels"):
            assert 0.0 < issue[k][0] < 1.0 and 1.0 <= issue[k][1] <= 64.0
    assert len(bench.kernel_sources_sha16()) == 16


@pytest.mark.gpu
def test_the_json_line_has_the_agreed_fields():
    r = _run("--config", "1", "--steps", "8", "--warmup", "2", "--cpu-seconds", "0.3")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 8 and d["warmup"] == 2 and d["vs_baseline"] is None
    assert d["unit"] == "MB/s" and d["higher_is_better"] is True and d["data"] == "synthetic"
    assert "workload" in d["config"] and "model" not in d["config"]
    roof = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-4
    cpu = d["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in cpu, key
    assert cpu["kind"] == "oracle" and cpu["cores"] == 1 and cpu["value"] > 0
    assert d["value"] > 0 and d["ms_per_step"] > 0
    # every kernel of the path with its share of the HBM roofline, the sync and the write kernel among them
    for k in ("sync_intra", "write", "pixels"):
        e = d["kernels"][k]
        assert e["ms"] > 0 and abs(e["frac"] - e["achieved_gbs"] / 8000.0) < 1e-4 and "traffic" in e
    h = d["with_h2d"]
    assert h["serial_ms_per_step"] > 0 and h["overlapped_ms_per_step"] > 0 and h["from_files_ms_per_step"] > 0
