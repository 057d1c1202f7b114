"""Host-side logic that needs no GPU: the input generators, the loader's refusal to run without
the built library, bench.py's one-GPU contract, and the rule that the product never touches the
oracle."""
import os
import re
import subprocess
import sys

import numpy as np
import pytest

from paper_2502_07021_amd import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("cfg,n,dtype,d", [(1, 64, np.float64, 2), (2, 96, np.float32, 3),
                                           (3, 128, np.float32, 8), (4, 80, np.float32, 16),
                                           (5, 72, np.float32, 2)])
def test_workload_recipe(cfg, n, dtype, d):
    w = workloads.make(cfg, n=n)
    assert w.n == n and w.d == d and w.dtype == np.dtype(dtype)
    assert w.x.shape == (n, d) and w.y.shape == (n, d) and w.x.dtype == dtype
    m = w.m
    assert w.a.shape == ((n,) if m == 1 else (n, m)) and w.a.dtype == dtype
    assert (w.a > 0).all() and (w.b > 0).all()
    # normalised in fp64 before the cast: sums are 1 up to the cast's rounding
    assert np.allclose(w.a.astype(np.float64).sum(axis=0), 1.0, rtol=0, atol=n * np.finfo(dtype).eps)
    assert np.allclose(w.b.astype(np.float64).sum(axis=0), 1.0, rtol=0, atol=n * np.finfo(dtype).eps)
    # seeded: the same call gives the same bytes, another seed does not
    w2 = workloads.make(cfg, n=n)
    assert all(np.array_equal(getattr(w, k), getattr(w2, k)) for k in "xyab")
    assert not np.array_equal(workloads.make(cfg, n=n, seed=1).x, w.x)


def test_full_size_configurations_are_the_published_ones():
    full = {1: (512, np.float64, 200, 1), 2: (8192, np.float32, 500, 1), 3: (32768, np.float32, 1000, 8)}
    for cfg, (n, dtype, iters, c) in full.items():
        w = workloads.make(cfg, n=8)          # tiny draw; the metadata is what is checked
        assert (w.iters, w.c, w.dtype) == (iters, c, np.dtype(dtype))
    assert workloads.make(4, n=8).tol == 1e-6 and workloads.make(4, n=8).iters == 2000
    w5 = workloads.make(5, n=8)
    assert w5.m == 64 and w5.iters == 300
    assert workloads.SEED_BASE * 10 + 3 == 202502073


def test_loader_refuses_to_run_without_the_library(monkeypatch):
    from paper_2502_07021_amd import api
    monkeypatch.setattr(api, "_lib", None)
    monkeypatch.setattr(api, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libfsk.so"))
    with pytest.raises(RuntimeError, match="is missing"):
        api.fsk_version()


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode != 0
    assert "one GPU" in r.stderr or "--gpus 1" in r.stderr
    assert r.stdout.strip() == ""


def test_product_never_touches_the_oracle():
    """Only tests/, smoke() and bench.py's cpu_baseline leg may use oracle/."""
    pkg = os.path.join(ROOT, "paper_2502_07021_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle\b", text, re.M), f
                assert "sinkhorn_oracle" not in text and "orc_" not in text, f
    bench = open(os.path.join(ROOT, "bench.py")).read()
    for m in re.finditer(r"^(\s*)import oracle\b", bench, re.M):
        assert len(m.group(1)) > 0          # only inside the cpu_baseline branches, never at module level
