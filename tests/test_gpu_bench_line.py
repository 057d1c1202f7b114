"""bench.py prints ONE JSON line with the fields its contract names; checked on a short run of
every workload (the oracle leg included for the headline, sized down by --steps)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COMMON = {"metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
          "scaling", "vs_baseline", "dtype", "data", "config", "roofline"}
ROOF = {"bound", "achieved", "peak", "unit", "frac", "traffic"}


def _run(*args):
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, check=True,
                         capture_output=True, text=True, timeout=600).stdout.strip().splitlines()
    lines = [l for l in out if l.startswith("{")]
    assert len(lines) == 1
    return json.loads(lines[0])


@pytest.mark.parametrize("args,bound,peak", [
    (("--workload", "cfg3", "--n", "8192", "--steps", "50", "--warmup", "5", "--profile-reps", "5"), "hbm", 8000.0),
    (("--workload", "cfg1", "--steps", "50", "--warmup", "5", "--no-cpu-baseline"), "hbm", 8000.0),
    (("--workload", "cfg4", "--n", "4096", "--steps", "5", "--warmup", "1", "--profile-reps", "2", "--no-cpu-baseline"), "alu", 78.6),
    (("--workload", "cfg5", "--n", "2048", "--steps", "5", "--warmup", "1", "--no-cpu-baseline"), "mfma", 157.3),
    (("--workload", "cfg5", "--n", "2048", "--dtype", "f64", "--steps", "5", "--warmup", "1", "--no-cpu-baseline"), "mfma", 78.6),
])
def test_bench_line(args, bound, peak):
    d = _run(*args)
    assert COMMON <= set(d) and ROOF <= set(d["roofline"])
    assert d["n_gpus"] == 1 and d["higher_is_better"] is True and d["vs_baseline"] is None
    assert d["data"] == "synthetic" and "workload" in d["config"] and "model" not in d["config"]
    assert d["value"] > 0 and d["ms_per_step"] > 0
    r = d["roofline"]
    assert r["bound"] == bound and r["peak"] == peak and 0 < r["frac"] < 1.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9
    if "--no-cpu-baseline" not in args:
        c = d["cpu_baseline"]
        assert c["kind"] == "oracle" and c["value"] > 0 and c["cores"] >= 1 and c["sample"]


def test_default_line_carries_the_other_four_configurations():
    """The driver's command: the headline (configuration 3) with `secondary` holding short runs of
    configurations 1, 2, 4, 5, each with its rate and the roofline of its dominant kernel."""
    d = _run("--steps", "20", "--warmup", "5")
    assert COMMON <= set(d) and d["config"]["n"] == 32768 and d["config"]["c"] == 8
    assert d["roofline"]["bound"] == "hbm" and d["roofline"]["frac"] > 0.8
    assert "profiles/" in d["roofline"]["traffic_source"]
    assert d["cpu_baseline"]["kind"] == "oracle"
    sec = d["secondary"]
    assert set(sec) == {"cfg1", "cfg2", "cfg4", "cfg5"}
    for name, bound in (("cfg1", "hbm"), ("cfg2", "hbm"), ("cfg4", "alu"), ("cfg5", "mfma")):
        e = sec[name]
        assert "error" not in e, e
        assert e["iterations_per_s"] > 0 and e["ms_per_step"] > 0 and name in e["workload"]
        r = e["roofline"]
        assert r["bound"] == bound and 0 < r["frac"] < 1.0 and r["kernel_ms"] > 0
        assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9
