#!/usr/bin/env python3
"""Benchmark of the Sinkhorn hot path on one MI355X.

Default workload (the metric's): configuration 3 -- n = 32768, fp32 dense K (4 GiB) built on the
GPU from seeded point clouds, row-partitioned into c = 8 blocks of 4096 rows, fused one-pass
flow.  A "step" is one Sinkhorn iteration (u-update then v-update over the whole of K).  Inputs
are resident in HBM before the timed region; the K build is setup and is not timed.

Prints ONE JSON line: iterations/s (metric), the roofline of the dominant kernel measured live
with HIP events on the launch stream, and the CPU oracle timed on this machine's host cores on a
bounded sample of the same workload.

The default run also times short fixed runs of the other four configurations and reports them
in a `secondary` object of the same line (rate, time per step, roofline of the dominant kernel);
`--workload cfg1|cfg2|cfg4|cfg5` prints a full line of its own for one of them.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X published HBM3E peak
PEAK_FP32_MFMA_TFLOPS = 157.3  # dense fp32 matrix peak
PEAK_FP64_MFMA_TFLOPS = 78.6   # dense fp64 matrix peak
PEAK_FMA_TFLOPS = 78.6         # 256 CU x 64 lanes x 2.4 GHz x 2 flop: one (unpacked fp32 or fp64) FMA per lane per clock
METRIC = "Sinkhorn iters/sec (Kv+K^Tu) at n=32768 fp32; achieved HBM GB/s vs peak"


def traffic_from_profile(name: str):
    """HBM bytes per launch of the dominant kernel from the committed counter summary, if any."""
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
    return float(m.group(1)) if m else None


def timed(fn):
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    fn()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def repeats(fn, steps, first_dt, n=5):
    """The timed region again, n - 1 more times: spread of the measurement (not used for `value`)."""
    ms = sorted([first_dt / steps * 1e3] + [timed(fn) / steps * 1e3 for _ in range(n - 1)])
    return {"runs": n, "median_ms_per_step": ms[len(ms) // 2], "min_ms_per_step": ms[0],
            "max_ms_per_step": ms[-1]}


def event_ms(fn):
    """Duration of fn's GPU work by HIP events recorded on the stream the library launches on."""
    import torch
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(); fn(); e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1)


# ------------------------------------------------------------------ dense (cfg 1, 2, 3)
def bench_dense(args, cfg):
    import numpy as np
    import torch
    from paper_2502_07021_amd import api, workloads

    w = workloads.make(cfg, n=args.n)
    n = w.n
    c = args.c if args.c is not None else w.c
    steps = args.steps if args.steps is not None else w.iters
    w.c = c
    td = torch.float64 if w.dtype == np.float64 else torch.float32
    esz = 8 if td == torch.float64 else 4
    dev = lambda t: torch.from_numpy(t).cuda()
    x, y, a, b = dev(w.x), dev(w.y), dev(w.a), dev(w.b)

    # setup (untimed): K on the GPU from the points
    opts = api.make_opts(n, td, c=c, max_iters=steps, flow=args.flow)
    K = torch.empty(n, n, dtype=td, device="cuda")
    api.fsk_kernel_from_points(opts, x, y, w.eps, w.normalise_by_max, K,
                               api.alloc_workspace(opts, api.FSK_MODE_SETUP, w.d))
    ws = api.alloc_workspace(opts, api.FSK_MODE_DENSE)
    u = torch.ones(n, dtype=td, device="cuda"); v = torch.ones(n, dtype=td, device="cuda")

    # one plain 1 GiB device copy: the known-size stream against which profiler byte
    # counters (FETCH_SIZE / WRITE_SIZE) of the same run are scaled
    cal_src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    api.fsk_bench_copy(cal_dst, cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    def run(iters, cc=c, wsp=ws):
        o = api.make_opts(n, td, c=cc, max_iters=iters, flow=args.flow)
        api.fsk_sinkhorn_dense(o, K, a, b, u, v, wsp)

    if args.warmup > 0:
        run(args.warmup)
    dt = timed(lambda: run(steps))
    if not bool(torch.isfinite(u).all() and torch.isfinite(v).all()):
        raise RuntimeError("non-finite scalings")

    # dominant kernel alone, same launch configuration, HIP events on the launch stream
    stream_ms, other_ms, launches = api.fsk_dense_profile(opts, K, a, b, u, v, ws, args.profile_reps)
    light = getattr(args, "light", False)      # a secondary entry of the default line
    spread = None if light else repeats(lambda: run(steps), steps, dt)
    # K read once per iteration (fused), twice (two-pass flows), or once per CALL (resident:
    # no HBM roofline applies; the figure below then only says how far from HBM-bound it is)
    alg_bytes = float(n) * n * esz * (2 if args.flow in (1, 2) else 1)
    achieved = alg_bytes / (stream_ms * 1e-3) / 1e9
    headline = cfg == 3 and args.flow == 0 and n == 32768 and c == 8
    if args.flow == 3:
        roofline_note = ("register-resident flow: one launch runs every iteration, K is read from "
                         "memory once per call; kernel_ms = launch time / iterations is barrier "
                         "latency, not bandwidth")
    roofline = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": achieved / PEAK_HBM_GBS,
                "traffic": traffic_from_profile("dense_fused_cfg3_pmc.txt") if headline
                else traffic_from_profile("dense_fused_cfg2_pmc.txt")
                if (cfg == 2 and args.flow == 0 and n == 8192 and c == 1) else None,
                "traffic_source": ("profiles/dense_fused_cfg3_pmc.txt" if headline else
                                   "profiles/dense_fused_cfg2_pmc.txt"
                                   if (cfg == 2 and args.flow == 0 and n == 8192 and c == 1) else None),
                "kernel": {0: "fused_kernel", 3: "resident_kernel"}.get(args.flow, "rowpass_kernel+colpartial_kernel"),
                "kernel_ms": stream_ms, "launches_per_step": launches,
                "algorithmic_bytes_per_step": alg_bytes, "other_kernels_ms": other_ms}
    if args.flow == 3:
        roofline["note"] = roofline_note

    if roofline["traffic_source"]:
        roofline["traffic_source"] += (": HBM bytes per launch from the committed rocprofv3 --pmc runs "
                                       "(FETCH_SIZE, WRITE_SIZE) of this command, not a counter of this run")
    extra = {}
    if c != 1 and not light:   # the same problem with c = 1 (the iterates the blocked run must reproduce)
        o1 = api.make_opts(n, td, c=1, max_iters=steps, flow=args.flow)
        ws1 = api.alloc_workspace(o1, api.FSK_MODE_DENSE)
        u.fill_(1.0); v.fill_(1.0)
        run(max(args.warmup, 1), 1, ws1)
        dt1 = timed(lambda: run(steps, 1, ws1))
        s1, _, _ = api.fsk_dense_profile(o1, K, a, b, u, v, ws1, args.profile_reps)
        extra = {"c1_iterations_per_s": steps / dt1, "c1_kernel_ms": s1,
                 "c1_kernel_GBps": alg_bytes / (s1 * 1e-3) / 1e9}

    laws = {1: "x,y~U[0,1]^2, C=|x-y|^2", 2: "x,y~N(0,I_3), C/max C", 3: "x~N(0,I_8), y~N(0.5,I_8), C/max C"}
    out = {
        "metric": METRIC if cfg == 3 else f"Sinkhorn iters/sec (Kv+K^Tu), cfg{cfg} n={n}",
        "value": steps / dt, "unit": "iterations/s", "n_gpus": 1, "steps": steps,
        "warmup": args.warmup, "ms_per_step": dt / steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f64" if esz == 8 else "f32",
        "data": "synthetic",
        "config": {"workload": f"cfg{cfg}: n={n} {'fp64' if esz == 8 else 'fp32'} dense K "
                               f"({n * n * esz / 2**20:.0f} MiB), {laws[cfg]}, eps={w.eps}, "
                               f"row-partitioned c={c} on one GPU, "
                               f"flow={['fused', 'two_pass', 'algorithm1', 'resident'][args.flow]}",
                   "n": n, "c": c, "eps": w.eps, "iterations": steps},
        "roofline": roofline,
    }
    if spread:
        out["repeats"] = spread
    out.update(extra)
    if not args.no_cpu_baseline:
        del K
        torch.cuda.empty_cache()
        import oracle
        t0 = time.perf_counter()
        Ko, _ = oracle.gibbs_from_points_f32(w.x, w.y, w.eps, w.normalise_by_max) if esz == 4 \
            else oracle.gibbs_from_points(w.x, w.y, w.eps, w.normalise_by_max)
        t_setup = time.perf_counter() - t0
        t0 = time.perf_counter()
        uo, vo = oracle.sinkhorn_blocked(Ko, w.a, w.b, 1, c, 1)
        t_one = time.perf_counter() - t0
        iters = int(max(1, min(steps, 15.0 // max(t_one, 1e-4))))   # about 15 s of CPU work
        t0 = time.perf_counter()
        oracle.sinkhorn_blocked(Ko, w.a, w.b, iters, c, 1, u0=uo, v0=vo)
        dto = time.perf_counter() - t0
        out["cpu_baseline"] = {
            "value": iters / dto, "unit": "iterations/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"{iters} full iterations at n={n} (c={c}, fp64 arithmetic on the stored K; "
                      f"oracle K build {t_setup:.1f} s not counted)"}
    return out


# ------------------------------------------------------------------ log domain (cfg 4)
def bench_log(args):
    import numpy as np
    import torch
    from paper_2502_07021_amd import api, workloads

    w = workloads.make(4, n=args.n)
    n, d = w.n, w.d
    steps = args.steps if args.steps is not None else 100
    dev = lambda t: torch.from_numpy(t).cuda()
    x, y, a, b = dev(w.x), dev(w.y), dev(w.a), dev(w.b)
    opts = api.make_opts(n, torch.float32, max_iters=steps)
    ws = api.alloc_workspace(opts, api.FSK_MODE_LOG, d)
    f = torch.zeros(n, device="cuda"); g = torch.zeros(n, device="cuda")

    def run(iters):
        api.fsk_sinkhorn_log_points(api.make_opts(n, torch.float32, max_iters=iters), x, y, w.eps,
                                    a, b, f, g, ws)

    run(max(args.warmup, 1))
    dt = timed(lambda: run(steps))
    ms = event_ms(lambda: run(args.profile_reps))       # 2 half-step launches per iteration
    launch_ms = ms / (2 * args.profile_reps)
    pairs = float(n) * n
    flops_per_pair = 2 * 16 + 4                          # 16 FMA (fp64) + add, max, exp2, add
    achieved = pairs * flops_per_pair / (launch_ms * 1e-3) / 1e12
    out = {
        "metric": f"Sinkhorn iters/sec (log-domain f,g updates), cfg4 n={n}",
        "value": steps / dt, "unit": "iterations/s", "n_gpus": 1, "steps": steps,
        "warmup": args.warmup, "ms_per_step": dt / steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32 (fp64 dot product)",
        "data": "synthetic",
        "config": {"workload": f"cfg4: n={n} log-domain, x,y~U[0,1]^{d} fp32, cost on the fly, "
                               f"eps={w.eps}, a=b=1/n, fixed {steps} iterations", "n": n, "d": d},
        "roofline": {"bound": "alu", "achieved": achieved, "peak": PEAK_FMA_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_FMA_TFLOPS, "traffic": None,
                     "kernel": "log_lse_kernel<16>", "kernel_ms": launch_ms,
                     "launches_per_step": 2, "pair_evaluations_per_s": pairs / (launch_ms * 1e-3),
                     "flops_per_pair": flops_per_pair,
                     "note": "kernel_ms = event-timed run / launches; includes the ~0.1% finalize kernels"},
    }
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        oracle.sinkhorn_log_points(w.x, w.y, w.eps, w.a, w.b, 1)
        t_one = time.perf_counter() - t0
        iters = int(max(1, min(steps, 12.0 // max(t_one, 1e-3))))          # about 12 s of CPU work
        t0 = time.perf_counter()
        oracle.sinkhorn_log_points(w.x, w.y, w.eps, w.a, w.b, iters)
        dto = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": iters / dto, "unit": "iterations/s", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": f"{iters} full iterations (f- and g-update against all {n} points) "
                                         f"from the cold start"}
    return out


# ------------------------------------------------------------------ batched (cfg 5)
def bench_batched(args):
    import numpy as np
    import torch
    from paper_2502_07021_amd import api, workloads

    w = workloads.make(5, n=args.n)
    n = w.n
    m = args.m if args.m is not None else w.m
    f64 = args.dtype == "f64"
    td, nd = (torch.float64, np.float64) if f64 else (torch.float32, np.float32)
    steps = args.steps if args.steps is not None else w.iters
    dev = lambda t: torch.from_numpy(np.ascontiguousarray(t.astype(nd))).cuda()
    if m == w.m:
        a_np, b_np = w.a, w.b
    else:                                                # the same Dirichlet(1) law at another m
        rng = np.random.default_rng(12345)
        a_np = rng.dirichlet(np.ones(n), size=m).T
        b_np = rng.dirichlet(np.ones(n), size=m).T
    x, y, A, B = dev(w.x), dev(w.y), dev(a_np), dev(b_np)
    opts = api.make_opts(n, td, m=m, max_iters=steps)
    K = torch.empty(n, n, dtype=td, device="cuda")
    api.fsk_kernel_from_points(opts, x, y, w.eps, False, K, None)
    ws = api.alloc_workspace(opts, api.FSK_MODE_BATCHED)
    U = torch.ones(n, m, dtype=td, device="cuda"); V = torch.ones(n, m, dtype=td, device="cuda")

    def run(iters):
        api.fsk_sinkhorn_batched(api.make_opts(n, td, m=m, max_iters=iters), K, A, B, U, V, ws)

    run(max(args.warmup, 1))
    dt = timed(lambda: run(steps))
    # as long as the timed region (the clock of the card settles only after some tens of
    # milliseconds of matrix-core work), and long enough to amortise the one-off K^T build
    reps = max(args.profile_reps, 50, min(steps, 1000))
    ms = event_ms(lambda: run(reps))
    launch_ms = ms / (2 * reps)                           # two products per iteration
    flops = 2.0 * n * n * m
    achieved = flops / (launch_ms * 1e-3) / 1e12
    peak = PEAK_FP64_MFMA_TFLOPS if f64 else PEAK_FP32_MFMA_TFLOPS
    out = {
        "metric": f"Sinkhorn iters/sec (multitarget K V, K^T U on MFMA), cfg5 n={n} m={m}",
        "value": steps / dt, "unit": "iterations/s", "n_gpus": 1, "steps": steps,
        "warmup": args.warmup, "ms_per_step": dt / steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"cfg5: n={n} {'fp64' if f64 else 'fp32'} dense K shared by m={m} "
                               f"Dirichlet(1) histogram pairs, x,y~U[0,1]^2, eps={w.eps}", "n": n, "m": m},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": peak,
                     "unit": "TFLOP/s", "frac": achieved / peak,
                     "traffic": traffic_from_profile("batched_mfma_f64_cfg5.txt" if f64 else "batched_mfma_cfg5.txt")
                     if (n == 16384 and m == 64) else None,
                     "traffic_source": (("profiles/batched_mfma_f64_cfg5.txt" if f64 else "profiles/batched_mfma_cfg5.txt")
                                        + ": committed rocprofv3 --pmc summary, not a counter of this run")
                     if (n == 16384 and m == 64) else None,
                     "kernel": ("batched_prod_f64_kernel" if f64 else "batched_prod_wide_kernel")
                               + " (both products)",
                     "kernel_ms": launch_ms, "launches_per_step": 2,
                     "note": "kernel_ms = event-timed run / product launches; includes the small reduce "
                             "kernels and 1/reps of the K^T build"},
        "histogram_iterations_per_s": steps * m / dt,
    }
    if not args.no_cpu_baseline:
        import oracle
        Ko, _ = oracle.gibbs_from_points(w.x, w.y, w.eps, False) if f64 \
            else oracle.gibbs_from_points_f32(w.x, w.y, w.eps, False)
        mo = min(m, 64)                                  # bounded sample: at most 64 columns
        Ao, Bo = np.ascontiguousarray(a_np[:, :mo]), np.ascontiguousarray(b_np[:, :mo])
        t0 = time.perf_counter()
        oracle.sinkhorn_batched(Ko, Ao, Bo, 1)
        t_one = time.perf_counter() - t0
        iters = int(max(1, min(steps, 12.0 // max(t_one, 1e-3))))          # about 12 s of CPU work
        t0 = time.perf_counter()
        oracle.sinkhorn_batched(Ko, Ao, Bo, iters)
        dto = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": iters / dto * mo / m, "unit": "iterations/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"{iters} full iterations at n={n} on {mo} of the {m} columns"
                                         + ("" if mo == m else ", scaled by columns")}
    return out


def secondary(args):
    """Short fixed runs of the other four configurations, for the default line's `secondary`."""
    import torch
    plan = (("cfg1", 1, 200, 20, 50), ("cfg2", 2, 500, 20, 128), ("cfg4", 4, 20, 2, 10), ("cfg5", 5, 300, 100, 50))
    keep = ("bound", "achieved", "peak", "unit", "frac", "kernel", "kernel_ms", "launches_per_step",
            "traffic", "traffic_source", "note")
    res = {}
    for name, cfg, steps, warmup, reps in plan:
        a2 = argparse.Namespace(**vars(args))
        a2.workload, a2.n, a2.c, a2.m, a2.dtype = name, None, None, None, "f32"
        a2.flow = 3 if cfg == 1 else 0
        a2.steps, a2.warmup, a2.profile_reps = steps, warmup, reps
        a2.no_cpu_baseline, a2.light = True, True
        try:
            d = bench_log(a2) if cfg == 4 else bench_batched(a2) if cfg == 5 else bench_dense(a2, cfg)
        except Exception as exc:      # a failed secondary must not take the headline with it
            res[name] = {"error": f"{type(exc).__name__}: {exc}"}
            continue
        res[name] = {"workload": d["config"]["workload"], "iterations_per_s": d["value"],
                     "ms_per_step": d["ms_per_step"], "steps": d["steps"], "warmup": d["warmup"],
                     "dtype": d["dtype"],
                     "roofline": {k: d["roofline"][k] for k in keep if d["roofline"].get(k) is not None}}
        torch.cuda.empty_cache()
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed iterations (default: the configuration's own count; cfg4: 100)")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg3", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--n", type=int, default=None, help="override the problem size (same law)")
    ap.add_argument("--c", type=int, default=None, help="row blocks (dense workloads)")
    ap.add_argument("--m", type=int, default=None, help="histogram pairs (cfg5; default 64)")
    ap.add_argument("--dtype", default="f32", choices=["f32", "f64"],
                    help="arithmetic of the cfg5 products (the dense workloads fix theirs)")
    ap.add_argument("--flow", type=int, default=None,
                    help="dense: 0 fused, 1 two-pass, 2 Algorithm 1, 3 register-resident "
                         "(default: 3 for cfg1, 0 otherwise)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help="headline run only: leave out the short runs of configurations 1, 2, 4, 5")
    ap.add_argument("--profile-reps", type=int, default=50)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives are part of it); "
              "use --gpus 1", file=sys.stderr)
        return 2
    import torch
    torch.cuda.set_device(0)
    headline = (args.workload == "cfg3" and args.n is None and args.c is None and args.flow is None)
    if args.flow is None:
        args.flow = 3 if args.workload == "cfg1" and args.n in (None, 512) else 0
    sec = None
    if headline and not args.no_secondary:
        sec = secondary(args)      # before the headline: its CPU leg would leave the GPU idle first
    if args.workload == "cfg4":
        out = bench_log(args)
    elif args.workload == "cfg5":
        out = bench_batched(args)
    else:
        out = bench_dense(args, int(args.workload[3]))
    if sec is not None:
        out["secondary"] = sec
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
