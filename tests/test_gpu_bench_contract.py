"""bench.py prints ONE JSON line with the agreed fields (a short run on two layers)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_prints_one_json_line_with_roofline_and_cpu_baseline():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--layers", "2", "--steps", "3", "--warmup", "1"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    j = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in j, k
    assert j["n_gpus"] == 1 and j["steps"] == 3 and j["warmup"] == 1 and j["unit"] == "tokens/s"
    assert j["vs_baseline"] is None and j["data"] == "synthetic" and j["dtype"] == "bf16"
    assert "workload" in j["config"] and "model" not in j["config"]
    roof = j["roofline"]
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert roof["frac"] == pytest.approx(roof["achieved"] / roof["peak"], abs=1e-3) and 0.0 < roof["frac"] < 1.0
    cpu = j["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["unit"] == "tokens/s"
    assert j["value"] == pytest.approx(1e3 / j["ms_per_step"], rel=1e-3)
    # regimes of the measurement plan, replay statistics, validity of the timed outputs
    for k in ("regime_indicators_off", "regime_indicators_on", "regime_negative_coefficients"):
        assert j[k]["ms_per_step"] > 0 and 0.0 <= j[k]["sparsity_union"] <= 1.0 and j[k]["ms_min"] <= j[k]["ms_median"]
    assert j["regime_indicators_on"]["sparsity_union"] >= j["sparsity_union"] >= j["regime_negative_coefficients"]["sparsity_union"]
    assert j["replays"]["n"] >= 50 and j["replays"]["ms_min"] <= j["replays"]["ms_median"]
    assert j["value_at_target_sparsity"] == pytest.approx(1e3 / j["regime_indicators_off"]["ms_per_step"], rel=1e-3)
    assert j["device_fault"] is False
    assert "traffic" in roof
    # the step goes through the whole-stack call; the per-layer calls and the other modes are reported beside it
    assert "clada_sparse_ffn_stack_decode" in j["step_path"]
    for k in ("natural", "indicators_off"):
        assert j["per_layer_calls"][k]["ms_per_step"] > 0
        for mode in ("lanes", "chained_launches", "persistent_kernel"):
            assert j["stack_modes"][mode][k]["bit_identical_to_per_layer_calls"] is True
    assert roof["in_step"]["frac"] == pytest.approx(roof["in_step"]["achieved"] / roof["peak"], abs=1e-3)
