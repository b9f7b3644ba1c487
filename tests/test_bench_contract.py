"""The contract of bench.py's one JSON line: host-side checks here (argument handling, the byte
accounting, the committed traffic file), and a GPU run of a small workload whose line must carry
every field the driver reads."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_follow_the_per_unit_figures():
    import bench
    N, D, V, K = 1000, 10, 50, 100
    # z step: per token the word id (4), the phi row (4K) and z (4); per document the theta row
    # (4K) and two offsets (8); up to 256 topics also the document table row (4K) and a byte a token
    assert bench.sample_z_algorithmic_bytes(N, D, K) == N * (4 + 4 * K + 4) + D * (4 * K + 8) + D * 4 * K + N
    assert bench.sample_z_algorithmic_bytes(N, D, 300) == N * (4 + 1200 + 4) + D * (1200 + 8)
    # word table: a permutation index and a topic per token, the table written once
    assert bench.count_algorithmic_bytes(N, D, V, K) == N * 5 + 4 * V * K
    assert bench.count_algorithmic_bytes(N, D, V, 300) == N * 8 + 4 * V * 300 + N * 4 + 4 * D * 300


def test_committed_traffic_file_names_its_commit_and_kernel_source():
    import bench
    with open(bench.TRAFFIC_FILE) as f:
        data = json.load(f)
    assert len(data["measured_at_commit"]) >= 7 and len(data["lda_sources_sha256_16"]) == 16
    for wl in ("large", "medium", "widek"):
        e = data["workloads"][wl]
        assert e["sample_z_hbm_bytes"] > 0 and 0 < e["texture_addresser_busy"] <= 1
        c = bench.measured_counters(wl)
        assert c["measured_at_commit"] == data["measured_at_commit"]
        assert isinstance(c["kernel_source_changed_since"], bool)
    assert bench.measured_counters("no such workload") is None


@pytest.mark.gpu
def test_bench_line_of_a_small_workload_has_every_field():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "medium", "--steps", "5",
                        "--warmup", "1", "--repeats", "3"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, "exactly one JSON line on stdout"
    d = json.loads(lines[0])
    for key, typ in [("metric", str), ("value", float), ("unit", str), ("n_gpus", int), ("steps", int),
                     ("warmup", int), ("ms_per_step", float), ("higher_is_better", bool), ("scaling", str),
                     ("dtype", str), ("data", str), ("config", dict), ("roofline", dict), ("cpu_baseline", dict)]:
        assert isinstance(d[key], typ), key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 1 and d["vs_baseline"] is None
    assert d["unit"] == "tokens/s" and d["higher_is_better"] is True and d["data"] == "synthetic"
    assert "workload" in d["config"] and "model" not in d["config"]
    # value is the whole job: tokens of the corpus times sweeps over the timed seconds
    assert abs(d["value"] * d["ms_per_step"] * 1e-3 / 2_999_304 - 1.0) < 1e-6
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9
    assert abs(rf["achieved"] - rf["algorithmic_bytes_per_launch"] / (rf["avg_launch_ms"] * 1e-3) / 1e9) < 1e-3 * rf["achieved"]
    assert rf["traffic"] is None or rf["traffic"] > 0
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] == 1 and cb["value"] > 0 and cb["unit"] == "tokens/s" and cb["sample"]
    for block in ("z_plus_count", "ceilings", "state_f64", "environment", "kernel_ms_per_sweep"):
        assert block in d, block
    assert d["ceilings"]["hbm_copy_GBs"] > 1000 and d["ceilings"]["gather_only_ms"] > 0
    assert d["state_f64"]["ms_per_step"] > d["ms_per_step"] * 0.9
