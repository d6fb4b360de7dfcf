"""bench.py's command line, as far as it can be checked without a GPU: more than one GPU is
refused with a message (this build runs on one GPU only), and the file parses."""
import ast
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_source_parses_and_names_the_metric():
    src = open(os.path.join(ROOT, "bench.py")).read()
    ast.parse(src)
    import json
    metric = json.load(open(os.path.join(ROOT, "BASELINE.json")))["metric"]
    assert f'METRIC = "{metric}"' in src
