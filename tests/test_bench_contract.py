"""bench.py's command line, checked without a GPU, and (on a GPU) the shape of
the line it prints."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_with_a_message():
    for n in ("2", "8"):
        r = subprocess.run([sys.executable, BENCH, "--gpus", n], capture_output=True, text=True, timeout=120)
        assert r.returncode != 0
        assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_help_lists_the_contract_flags():
    r = subprocess.run([sys.executable, BENCH, "--help"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0
    for flag in ("--gpus", "--steps", "--warmup"):
        assert flag in r.stdout


def test_traffic_figure_matches_the_profile_it_cites_and_the_kernel_it_was_taken_for():
    """roofline.traffic comes from a counter profile, not from the run: the profile must name the
    benchmark's kernel and hold the same figures, and it must have been taken for the kernel source
    as it stands (a kernel edit changes the hash and forces the profile to be taken again)."""
    sys.path.insert(0, ROOT)
    import bench
    current = bench.kernel_source_hash()
    for (workload, budget), tp in bench.TRAFFIC_FROM_PROFILE.items():
        text = open(os.path.join(ROOT, tp["profile"])).read()
        assert tp["kernel"] in text, "the profile does not mention %s" % tp["kernel"]
        assert workload in text and ("cu_budget=%d" % budget) in text
        assert ("fetched %d KiB" % tp["fetched_KiB"]) in text and ("written %d KiB" % tp["written_KiB"]) in text
        assert ("kernel source sha256[:12] = %s" % tp["kernel_source_sha256_12"]) in text
        assert tp["kernel_source_sha256_12"] == current, (
            "tw_fused.hip / tw_device.h changed since %s was taken: take the counter profile again and "
            "update TRAFFIC_FROM_PROFILE" % tp["profile"])


@pytest.mark.gpu
def test_benchmark_line_has_the_contract_fields():
    r = subprocess.run([sys.executable, BENCH, "--steps", "20", "--warmup", "5", "--no-extras", "--no-cpu-baseline"],
                       capture_output=True, text=True, timeout=300, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 20 and d["warmup"] == 5 and d["unit"] == "GB/s"
    assert d["higher_is_better"] is True and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert "workload" in d["config"] and "model" not in d["config"]
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3
    assert rf["traffic"] is None or "counters in profiles/" in rf["traffic_source"]
    # whole-job throughput includes the gaps between launches, the kernel's own rate does not
    assert 0.5 * rf["achieved"] < d["value"] <= rf["achieved"] * 1.01
    assert abs(d["ms_per_step"] * 1e3 - rf["avg_launch_us"]) < 0.25 * rf["avg_launch_us"]
