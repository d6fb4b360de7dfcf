"""bench.py end to end on the GPU with small arguments: the default step on the 4K configuration
(with the CPU-oracle leg) must print one JSON line with the contract's fields, and the fused-tail
option, the chunked-prefill mode and the head-mapping mode must run and report."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                       timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.strip().splitlines() if l.startswith("{")]
    assert len(lines) == 1, r.stdout[-2000:]
    return json.loads(lines[0])


def test_default_step_prints_the_contract_fields():
    r = _bench("--config", "c1", "--steps", "5", "--warmup", "2")
    base = json.load(open(os.path.join(ROOT, "BASELINE.json")))
    assert r["metric"] == base["metric"] and r["unit"] == "us/layer" and r["n_gpus"] == 1
    assert r["steps"] == 5 and r["warmup"] == 2 and r["higher_is_better"] is False and r["vs_baseline"] is None
    assert r["value"] > 0 and r["ms_per_step"] > 0 and r["data"] == "synthetic" and r["dtype"] == "bf16"
    assert r["config"]["workload"].startswith("c1")
    roof = r["roofline"]
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    cpu = r["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
    # the call-level fraction beside the kernel's, the graph-replayed figures, and this run's own
    # comparison with the oracle (index sets equal, outputs inside the stated tolerance)
    call = r["roofline_call"]
    assert call["bytes"] == roof["algorithmic_bytes_per_launch"] and call["us"] == r["value"]
    assert call["frac"] <= roof["frac"] + 1e-6
    assert r["graph_replay"]["sparse_attn_us"] > 0 and r["graph_replay"]["step_us"] > 0
    par = r["parity"]
    assert par["ok"] is True and par["index_sets_equal"] is True
    assert par["out_max_abs_err"] <= 1e-2 and par["out_mean_abs_err"] <= 1e-3
    assert r["library_version"] > 0
    rs = r["roofline_select"]                        # the selection's bytes over its kernels' and its call's time
    assert rs["bytes"] > 0 and rs["kernels_us"] > 0 and rs["call_us"] > 0 and 0 < rs["frac_call"] <= rs["frac_kernels"] < 1


def test_headline_configuration_carries_sweep_and_paper_budgets():
    """The default run (128K context, batch 4) with few steps and without the oracle leg: the 5%
    and 20% points of the sweep, the paper's own budgets and the 32K point are in the line."""
    r = _bench("--steps", "3", "--warmup", "1", "--no-cpu-baseline")
    assert set(r["sweep"]) == {"5%", "20%"}
    assert r["sweep"]["5%"]["budget_tokens"] == 6554 and r["sweep"]["20%"]["budget_tokens"] == 26215
    for pt in r["sweep"].values():
        assert pt["sparse_attn_us"] > 0 and pt["dense_attn_us"] > pt["sparse_attn_us"] and 0 < pt["split_kernel_frac"] < 1
    st = r["stacked_layers"]                       # eight layers' caches attended back to back, eager
    assert st["layers"] == 8 and st["sparse_attn_us_per_layer"] > 0 and 0 < st["call_frac"] < 1
    assert {"c3@256", "c3@512", "c3@4096"} <= set(r["paper_budgets"])
    assert any(k.startswith("c2@") for k in r["paper_budgets"])
    for pt in r["paper_budgets"].values():
        # (the graph-replayed figure of a call is a difference of two medians: present, not sign-checked)
        assert isinstance(pt["graph_replay"]["sparse_attn_us"], float) and pt["graph_replay"]["step_us"] > 0
        assert pt["select_us"] > 0 and pt["sparse_attn_us"] > 0


def test_fused_tail_option_and_other_modes():
    r = _bench("--config", "c1", "--steps", "3", "--warmup", "1", "--no-cpu-baseline", "--fused-tail")
    assert r["config"]["fused_tail"] is True and r["value"] > 0
    p = _bench("--config", "c1", "--prefill-blocks", "4", "--steps", "3", "--warmup", "1")
    assert p["unit"] == "us/block" and p["value"] > 0 and p["select_us"]["median"] > 0
    h = _bench("--headmap", "--steps", "3")
    assert h["unit"] == "ms" and h["value"] > 0 and h["planted_map_recovered"] is True
