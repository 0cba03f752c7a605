"""The default bench line, as the driver runs it (fewer steps): one JSON line that carries the headline, the
other configurations and the admission sweep, each with its roofline entry, counter traffic that belongs to
the kernel and plan sources in the tree, and the oracle checks."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def roofline_ok(r, what):
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0, what
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3, what
    assert abs(r["achieved"] - r["bytes_per_launch"] / r["avg_launch_us"] / 1e3) <= 0.02 * r["achieved"], what
    assert 0.3 < r["frac"] < 1.0, what
    assert r["traffic"] is not None and r["traffic"] >= r["bytes_per_launch"], what
    d = r["traffic_detail"]
    assert d["profiled_at_this_kernel_source"], f"{what}: the stored counter profile is of other kernel or plan sources"
    assert d["fetch_bytes"] + d["write_bytes"] == r["traffic"] and r["traffic"] < 1.1 * r["bytes_per_launch"], what


def test_default_bench_line():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "4", "--warmup", "1"],
                         capture_output=True, text=True, timeout=600)
    assert run.returncode == 0, run.stderr[-2000:]
    lines = [ln for ln in run.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, "exactly one line on stdout"
    j = json.loads(lines[0])
    assert j["metric"] == "decode_step_attention_effective_kv_bandwidth" and j["unit"] == "GB/s"
    assert j["n_gpus"] == 1 and j["steps"] == 4 and j["warmup"] == 1 and j["higher_is_better"] is True
    assert j["vs_baseline"] is None and j["dtype"] == "bf16" and j["data"] == "synthetic"
    assert "config3_mixed" in j["config"]["workload"] and j["config"]["n_layers"] == 64
    # value = the whole step's algorithmic bytes over its duration
    alg = (j["config"]["kv_bytes_unique_per_layer"] + 2 * j["config"]["n_seqs"] * 64 * 128 * 2) * 64
    assert abs(j["value"] - alg / j["ms_per_step"] / 1e6) <= 0.01 * j["value"]
    roofline_ok(j["roofline"], "headline")
    assert 64 * j["roofline"]["avg_launch_us"] <= j["ms_per_step"] * 1e3 * 1.10  # (two measurements of the same launches)
    assert j["roofline"]["plain_read"]["kernel_over_plain_read"] < 1.05
    assert set(j["partial_rows"]["avg_launch_us"]) == {"f16_scaled", "f32"}
    cpu = j["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and "layers [0," in cpu["sample"]
    assert cpu["max_abs_err_gpu_vs_oracle"] <= 2e-2 and cpu["mean_abs_err_gpu_vs_oracle"] <= 2e-3
    for name in ("irp_off", "long"):
        row = j["other_workloads"][name]
        roofline_ok(row["roofline"], name)
        assert row["cpu_baseline"]["max_abs_err_gpu_vs_oracle"] <= 2e-2
    sweep = j["step_latency_vs_admitted_branches"]
    assert [r["k"] for r in sweep["rows"]] == [0, 2, 4, 8, 16]
    for r in sweep["rows"]:
        roofline_ok(r["roofline"], f"sweep k={r['k']}")
        assert r["admitted_branches"] == 32 * r["k"] and r["n_seqs"] == 128 + 32 * r["k"]
    ms = [r["ms_per_step"] for r in sweep["rows"]]
    assert ms == sorted(ms) and sweep["rows"][-1]["externality_ms"] > 0  # more admitted branches, longer steps
    assert sweep["cpu_baseline"]["max_abs_err_gpu_vs_oracle"] <= 2e-2 and "layers [0, 31, 63]" in sweep["cpu_baseline"]["sample"]
