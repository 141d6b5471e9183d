"""The native driver program: scheduler library + kernel library, no Python in the loop.
It checks the KV content of every request after each move itself (non-zero exit on any
difference); this test runs it and reads its summary."""
import json
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DRIVER = os.path.join(ROOT, "paper_2602_11530_amd", "serve_trace")


@pytest.mark.parametrize("args", [
    [],                                                                   # two instances under memory pressure
    ["--instances", "3", "--blocks", "120", "--requests", "40", "--layers", "3", "--seed", "7"],
])
def test_native_driver_serves_a_trace(device, args):
    assert os.path.exists(DRIVER), "run `python -m paper_2602_11530_amd.build` first"
    p = subprocess.run([DRIVER] + args, capture_output=True, text=True, timeout=300)
    print(p.stdout, p.stderr, flush=True)
    assert p.returncode == 0, p.stderr
    s = json.loads(p.stdout.strip().splitlines()[-1])
    assert s["ok"] and s["kv_checks"] >= s["requests"]
    assert s["offloads"] > 0 and s["reloads"] > 0
    assert s["migrations"] + s["migrations_via_host"] > 0
    assert 0 < s["worst_qoe"] <= 1 + 1e-12 and s["mean_ttft_s"] > 0


def test_native_driver_rejects_bad_sizes():
    p = subprocess.run([DRIVER, "--blocks", "10"], capture_output=True, text=True, timeout=60)
    assert p.returncode == 1 and "must fit" in p.stderr
