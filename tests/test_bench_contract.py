"""bench.py's command line: what can be checked without a GPU (CPU), and the shape of its one JSON line (GPU)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_help_lists_the_contract_flags():
    r = subprocess.run([sys.executable, BENCH, "--help"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0
    for flag in ("--gpus", "--steps", "--warmup"):
        assert flag in r.stdout


@pytest.mark.gpu
def test_one_json_line_with_roofline_and_cpu_baseline():
    print("bench contract", flush=True)
    r = subprocess.run([sys.executable, BENCH, "--steps", "12", "--warmup", "2", "--layers", "2", "--iso-steps", "4",
                        "--graph-steps", "4"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-3000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 12 and out["warmup"] == 2 and out["unit"] == "GB/s" and out["dtype"] == "u8"
    assert out["vs_baseline"] is None and out["data"] == "synthetic" and "workload" in out["config"]
    rf = out["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3
    assert rf["launches"] == 12 and 0 < rf["frac"] < 1
    cb = out["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["sample"]
    assert out["bit_exact"] is True
    assert rf["traffic"] is None or "profiles/" in rf["traffic_source"]
    assert rf["frac_alone"] is not None and 0 < rf["frac_alone"] < 1 and 0 < rf["frac_of_plain_copy"] < 1.1
    assert out["config"]["blocks_per_step_mean_of_config"] == 20480
    legs = out["other_legs"]                       # the next seed's draw and the four other configurations, each checked
    assert len(legs) == 5 and all(leg["bit_exact"] is True and leg["value"] > 0 for leg in legs.values())
    assert {"configs[0]", "configs[2]", "configs[3]", "configs[4]"} <= set(legs)
    assert legs["configs[4]"]["together"]["over_sum_of_alone"] < 1.1
    assert legs["configs[2]"]["cpu_baseline"]["kind"] == "oracle" and legs["configs[3]"]["placed_per_step"] > 0
    assert out["value"] > 0 and abs(out["ms_per_step"] - 2 * out["config"]["payload_bytes_per_step"] / out["value"] / 1e6) \
        < 0.02 * out["ms_per_step"]


@pytest.mark.gpu
def test_latency_by_size_workload_delivers_the_same_bytes_from_either_tier():
    print("bench latency_by_size", flush=True)
    r = subprocess.run([sys.executable, BENCH, "--workload", "latency_by_size", "--steps", "50"], capture_output=True, text=True,
                       timeout=600)
    assert r.returncode == 0, r.stderr[-3000:]
    out = json.loads([l for l in r.stdout.splitlines() if l.strip()][-1])
    assert len(out["experts"]) == 6 and len(out["kv"]) == 6
    for row in out["experts"] + out["kv"]:
        assert row["same_bytes"] is True and row["host_tier_us"] > row["cache_tier_us"] > 0
    assert out["kv"][-1]["speed_up"] > 10 and out["experts"][-1]["speed_up"] > 10      # bandwidth-bound sizes: HBM against PCIe


@pytest.mark.gpu
def test_link_contention_workload():
    """Beside a placement on another stream a PCIe-bound fetch still delivers the same bytes, pays less the narrower the
    placement's copy runs, and with the default width keeps most of the link."""
    print("bench link_contention", flush=True)
    r = subprocess.run([sys.executable, BENCH, "--workload", "link_contention"], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads(r.stdout.strip().splitlines()[-1])
    rows = {str(x["pcie_wgs"]): x for x in d["rows"]}
    assert all(x["same_bytes"] for x in d["rows"])
    assert rows["64"]["fetch_beside_placement_ms_median"] > 2 * rows["8"]["fetch_beside_placement_ms_median"]
    default = rows["default (12)"]
    assert default["fetch_beside_placement_ms_median"] < 2.5 * default["fetch_alone_ms"]
    assert default["placement_alone_ms"] < 1.1 * rows["64"]["placement_alone_ms"]


@pytest.mark.gpu
def test_kv_and_experts_workload():
    """configs[4] as a benchmark line: both classes every step on two streams, revocations with fetches in flight; the
    end state agrees with the oracle's, and side by side the two cost no more than one after the other."""
    print("bench kv_and_experts", flush=True)
    r = subprocess.run([sys.executable, BENCH, "--workload", "kv_and_experts", "--steps", "30"], capture_output=True, text=True,
                       timeout=400)
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads(r.stdout.strip().splitlines()[-1])
    assert d["bit_exact"] is True and d["steps"] == 30
    assert d["together"]["churn"]["revoked"][0] > 1000 and d["together"]["churn"]["revoked"][1] > 0
    assert d["together"]["over_sum_of_alone"] < 1.1
