"""The benchmark's command-line contract: one GPU only, one JSON line with the agreed fields."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_pass_planner_keeps_the_run_inside_its_budget():
    """--steps / --warmup are upper bounds under a wall-clock budget.  One pass has been run and timed
    when the plan is made; the plan never exceeds the request, never times fewer than one pass, gives
    timed passes priority over further warm-up passes, and what it adds fits the seconds left."""
    sys.path.insert(0, ROOT)
    import bench
    # the driver's command on the headline workload: a pass of about 25.5 s, 182 s left after the
    # first pass, the extra evented pass and the CPU baseline have been set aside
    assert bench.plan_passes(20, 5, 25.5, 182.0) == (1, 7)
    assert bench.plan_passes(20, 5, 25.5, 10.0) == (1, 1)       # nothing more fits: still one timed pass
    assert bench.plan_passes(20, 5, 25.5, -30.0) == (1, 1)
    assert bench.plan_passes(20, 5, 1.0, 300.0) == (5, 20)      # a fast workload runs what was asked for
    assert bench.plan_passes(5, 1, 25.5, 1000.0) == (1, 5)
    assert bench.plan_passes(3, 2, 10.0, 55.0) == (2, 3)        # timed passes first, then a second warm-up
    assert bench.plan_passes(1, 0, 25.0, 500.0) == (0, 1)       # no warm-up: the first pass is the timed one
    assert bench.plan_passes(5, 0, 25.0, 60.0) == (0, 3)
    for steps in (1, 5, 20):
        for warmup in (0, 1, 5):
            for pass_s in (0.01, 3.0, 25.5, 80.0):
                for avail in (-10.0, 0.0, 30.0, 200.0, 400.0):
                    w, k = bench.plan_passes(steps, warmup, pass_s, avail)
                    assert 1 <= k <= steps and min(warmup, 1) <= w <= warmup
                    fit = int(avail // pass_s) if avail > 0 else 0
                    must = 1 if warmup else 0          # after a warm-up pass one timed pass always follows
                    assert w + k - 1 <= max(fit, must), (steps, warmup, pass_s, avail, w, k)


def test_headline_plan_fits_the_drivers_ten_minutes():
    """With the default budget, a first pass of 25.5 s that ends 150 s into the run (a slow first
    import of torch included) and the reserves main() sets aside, the whole run stays well under the
    600 s the driver allows, and at least five passes are timed."""
    sys.path.insert(0, ROOT)
    import bench
    budget, first, at = 400.0, 25.5, 150.0
    reserve = 1.25 * first + 35.0 + 5.0
    w, k = bench.plan_passes(20, 5, first, budget - at - reserve)
    total = at + (w - 1 + k) * first + reserve
    assert k >= 5 and total <= 420.0


@pytest.mark.gpu
def test_bench_line_fields_on_the_tiny_workload():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "opt125m_layer_q4", "--steps", "2",
                        "--warmup", "1"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["vs_baseline"] is None
    assert d["unit"] == "tokens/s" and d["value"] > 0 and d["data"] == "synthetic"
    assert d["config"]["workload"] == "opt125m_layer_q4"
    rl = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic", "kernel"):
        assert key in rl, key
    assert rl["bound"] in ("hbm", "mfma") and 0 < rl["frac"] < 1.5
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1 and cb["sample"]
