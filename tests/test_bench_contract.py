"""bench.py's command-line contract: one JSON line with the agreed keys, and a clear refusal
of more than one GPU."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in (p.stderr + p.stdout)
    assert not p.stdout.strip().startswith("{")


@pytest.mark.gpu
@pytest.mark.parametrize("config", [0, 1])
def test_bench_prints_one_json_line_with_the_contract_keys(config):
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--config", str(config),
                        "--steps", "3", "--warmup", "1", "--min-warmup-seconds", "0"],
                       capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [ln for ln in p.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step",
              "higher_is_better", "scaling", "vs_baseline", "dtype", "data", "config",
              "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1
    assert d["higher_is_better"] is True and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert d["dtype"] == "f32" and d["unit"] == "Grelax/s" and "workload" in d["config"]
    assert "model" not in d["config"]
    r = d["roofline"]
    for k in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert k in r, k
    assert r["bound"] in ("hbm", "alu") and abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] == 1 and c["value"] > 0 and c["sample"]
    if config == 1:      # 64 instances: the oracle is also timed on several cores side by side
        m = d["cpu_baseline_all_cores"]
        assert m["kind"] == "oracle" and 2 <= m["cores"] <= 16 and m["value"] > 0 and m["sample"]
    assert d["value"] > 0 and d["ms_per_step"] > 0
    # value = nominal relaxations of the step / wall time of the step
    assert abs(d["value"] - d["config"]["relaxations_per_step"] / d["ms_per_step"] / 1e6) \
        <= 1e-6 * d["value"]
    # every other configuration is timed beside the main workload, each with its own
    # latency and roofline block (vector ALU, HBM and, where profiled, LDS)
    others = d["other_configs"]
    assert sorted(int(o["workload"][len("configs["):].split("]")[0]) for o in others) == \
        sorted({0, 1, 2, 4} - {config})
    for o in others + [d]:
        assert o["ms_per_step"] > 0 and o["forward_ms"] > 0 and o["budget_curve_ms"] > 0
        r = o["roofline"]
        assert 0 < r["frac"] <= 1.0 and r["alu_frac"] > 0 and "hbm_frac" in r and "lds" in r
        assert "frac_is" in r and r["kernel"].startswith("k_dp_")
        if r["concurrent_launches"] > 1:
            assert 0 < r["frac_single_chain"] <= 1.0
        if r["lds"] is not None:
            assert r["lds"]["peak"] > 70 and 0 <= r["lds"]["frac"] <= 1.5
    assert 0 < d["executed_fraction"] <= 1.0 and d["executed_grelax_per_s"] > 0
    assert "general_r_grelax_per_s" in d and "traffic_commit" in d
    assert d["target_50pct_of_roofline_met"] in (True, False)
    assert d["pipeline_reduce_ms"] > 0            # configs[4]: the pipeline-aware outer reduction
