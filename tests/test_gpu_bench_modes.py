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


def test_fused_tail_option_and_other_modes():
    r = _bench("--config", "c1", "--steps", "3", "--warmup", "1", "--no-cpu-baseline", "--fused-tail")
    assert r["config"]["fused_tail"] is True and r["value"] > 0
    p = _bench("--config", "c1", "--prefill-blocks", "4", "--steps", "3", "--warmup", "1")
    assert p["unit"] == "us/block" and p["value"] > 0 and p["select_us"]["median"] > 0
    h = _bench("--headmap", "--steps", "3")
    assert h["unit"] == "ms" and h["value"] > 0 and h["planted_map_recovered"] is True
