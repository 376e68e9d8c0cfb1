"""bench.py end to end on a small workload: every option combination prints one JSON line with the
contract's fields."""
import json
import os
import subprocess
import sys

import pytest
import torch

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "c2_small", "--steps", "12",
                        "--warmup", "2", *args], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    return json.loads(lines[0])


def test_default_line_has_the_contract_fields():
    d = _bench("--cpu-seconds", "2")
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 12 and d["value"] > 0 and d["dtype"] == "f32"
    assert d["config"]["workload"] == "c2_small" and d["vs_baseline"] is None
    rf = d["roofline"]
    assert rf["bound"] == "mfma" and rf["unit"] == "TFLOP/s" and rf["peak"] == 157.3
    assert rf["frac"] == pytest.approx(rf["achieved"] / rf["peak"], rel=1e-3)
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0
    assert cb["value_one_thread"] > 0 and cb["legs"]["one_thread"]["threads"] == 1 and cb["cpu_model"] and cb["nproc"] >= 1
    assert d["secondary"] is None                    # only the default workload's line carries the second block
    assert set(d["variants"]) == {"shards4", "dynamic"}
    assert d["hbm_pass"]["ms"] > 0 and d["hbm_streams"]["dots"]["bytes"] > 0


@pytest.mark.parametrize("args", [
    ("--shards", "2"), ("--deps", "dynamic"), ("--deps", "dynamic", "--shards", "2"), ("--deps", "none", "--p-max", "50"),
    ("--priority", "uniform"), ("--loss", "logistic"), ("--kkt-tol", "1e-2", "--check-every", "4"),
    ("--graph-rounds", "4"), ("--tune", "gram_xcd_map=0"),
])
def test_option_combinations_run(args):
    d = _bench("--cpu-seconds", "0", "--no-variants", *args)
    assert d["value"] > 0 and d["steps"] >= 1 and d["objective_end"] < d["objective_start"]


def _run(*args):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    return [l for l in r.stdout.splitlines() if l.strip()]


def test_size_sweep_mode_prints_one_row_per_point():
    lines = _run("--sweep", "--sweep-rows", "3000", "--sweep-l-prime", "128", "600", "--sweep-rounds", "3")
    assert len(lines) == 3 and lines[0].split()[0] == "N"
    for l in lines[1:]:
        f = l.replace("|", " ").split()
        # N, L', gram us, TFLOP/s, frac, tile kernel, mask us | dots MB, us, GB/s, frac | residual us, GB/s, frac
        assert len(f) == 14 and int(f[0]) == 3000 and int(f[5]) == 128
        assert float(f[2]) > 0 and float(f[6]) > 0 and float(f[8]) > 0 and float(f[11]) > 0


def test_scheduler_comparison_mode_prints_one_line_per_scheduler():
    lines = _run("--compare-schedulers", "--workload", "c2_small", "--steps", "40", "--check-every", "20", "--p-max", "100")
    got = [json.loads(l) for l in lines]
    assert [g["scheduler"] for g in got] == ["strads", "strads-dynamic", "static-corr", "shotgun"]
    for g in got:
        tr = g["trajectory_round_ms_objective"]
        assert tr[0][0] == 0 and tr[-1][0] == 40 and tr[-1][2] < tr[0][2]
