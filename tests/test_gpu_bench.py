"""The bench line keeps its contract: one JSON object on stdout with the fields the driver reads,
the roofline of the dominant kernel measured with HIP events, and the oracle's CPU baseline."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_line_has_the_contract_fields():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "5", "--warmup", "2",
                        "--modes", "off_same_plan"], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, r.stdout
    j = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in j, k
    assert j["n_gpus"] == 1 and j["steps"] == 5 and j["warmup"] == 2 and j["unit"] == "tokens/s"
    assert j["higher_is_better"] is True and j["vs_baseline"] is None and j["dtype"] == "bf16"
    assert j["data"] == "synthetic" and "workload" in j["config"] and "model" not in j["config"]
    # value is tokens of one batch over the measured step time
    assert abs(j["value"] - j["config"]["T"] / (j["ms_per_step"] * 1e-3)) <= 1e-3 * j["value"]
    rf = j["roofline"]
    for k in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert k in rf, k
    assert rf["bound"] == "hbm" and rf["unit"] == "GB/s" and rf["peak"] == 8000.0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3 and 0.0 < rf["frac"] < 1.0
    # achieved = algorithmic bytes of the dominant kernel over its event-measured duration
    assert abs(rf["achieved"] - rf["algorithmic_bytes"] / (rf["avg_ms"] * 1e-3) / 1e9) <= 1e-3 * rf["achieved"]
    cb = j["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["unit"] == "tokens/s" and cb["value"] > 0 and cb["cores"] >= 1 and cb["sample"]
    m = j["replication_modes_ms"]
    assert m["on"] > 0 and m["off_same_plan"] > 0        # both modes timed (which is faster is the bench's finding)
    rt = j["config"]["routing"]
    assert rt["assignments"] == j["config"]["T"] and 0 < rt["max_expert_share"] <= 1
    assert rt["replicas_granted"] <= min(rt["replicas_wanted"], j["config"]["replica_budget"])
    mp = rf["measured_peak"]
    assert 2000 < mp["hbm_read_GBs"] < 8000 and 2000 < mp["hbm_read_nontemporal_GBs"] < 8000
    assert 300 < mp["mfma_bf16_operands_from_lds_TFLOPs"] < 2600 and 300 < mp["mfma_bf16_registers_TFLOPs"] < 2600
    assert 5 < mp["one_workgroup_read_GBs"] < 500
    assert abs(rf["frac_of_measured_peak"] - rf["achieved"] / mp["hbm_read_nontemporal_GBs"]) < 1e-3
    assert set(j["kept_tokens_per_s"]) == set(m)
    pc = j["per_call_ms_median"]
    assert set(pc) == {"moe_route", "moe_plan_dispatch", "moe_expert_ffn", "moe_combine"} and all(v > 0 for v in pc.values())
