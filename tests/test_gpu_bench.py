"""bench.py end to end on a short workload: the JSON contract, and that the outputs of the timed
configuration are the ones compared with the oracle."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*extra):
    import torch  # noqa: F401  (paged in here, so that the child's import is not the first on a fresh box)
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "llama1b_down_b32_int4_perm",
           "--steps", "60", "--warmup", "10", *extra]
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=400, cwd=ROOT)
    assert res.returncode == 0, res.stderr[-2000:]
    return json.loads([l for l in res.stdout.splitlines() if l.startswith("{")][-1])


@pytest.mark.parametrize("extra", [(), ("--arranged",), ("--identity",)])
def test_bench_line_and_check(extra):
    r = _run(*extra)
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in r, key
    assert r["n_gpus"] == 1 and r["steps"] == 60 and r["warmup"] == 10 and r["vs_baseline"] is None
    assert r["config"]["workload"] == "llama1b_down_b32_int4_perm"
    rf = r["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-12 and 0 < rf["frac"] < 1
    assert r["cpu_baseline"]["kind"] == "oracle" and r["cpu_baseline"]["value"] > 0
    assert r["check"]["ok"] and r["check"]["mismatch_fail"] == 0 and r["check"]["elements"] > 0
    if not extra:
        assert "arranged_perm" in r["context"]
    lm = r["context"]["launch_model"]
    assert [pt[0] for pt in lm["points_rows_us"]] == [512, 1024, 1536, 2048] and all(pt[1] > 0 for pt in lm["points_rows_us"])
    assert lm["ns_per_row"] > 0
