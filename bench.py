#!/usr/bin/env python3
"""Benchmark of the DPPF consensus round on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--call round|pull_push|...]
                    [--graph] [--no-per-config] [--no-cpu-baseline]

One "step" is one pass of the whole hot path over one batch of synthetic input: the fused
`dppf_round` (last local momentum-SGD step + replica average + distances + pull-push update)
over the M resident replicas of a ViT-B/16-sized parameter list.  Inputs are generated on the
host with the seeded recipe of `paper_2507_20424_amd.workloads`, uploaded once, and resident
in HBM before the timed region starts.  Prints ONE JSON line.

Besides the headline figure the line carries
  roofline           the kernel of the call that takes the most GPU time
  roofline_lowest    the kernel of the call that is furthest below the HBM roofline
  per_config         the fused round (and, where tau > 1, the configuration's whole period of tau - 1
                     stand-alone local steps + the fused round) on all five configurations
  cpu_baseline       the CPU oracle on one core; cpu_baseline_all_cores: the same on every host core
--graph captures one step in a HIP graph after the eager warm-up and times replays of it.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published peak
# algorithmic HBM bytes per replica-parameter (fp32): what the method itself must move
BYTES_PER_RP = {
    "step_reduce": 16.0,        # read x, v, g; write v (average and distances ride along)
    "step_update": 12.0,        # read x, v; write x
    "reduce": 4.0,              # read x
    "update": 8.0,              # read x, write x
    "local_step": 20.0,         # read x, v, g; write x, v
    "finalize": 0.0,
    "update_exact": 8.0,        # read x, write x (the sum of unit vectors is formed in registers)
    "seq_reduce": None,         # read x and x_C: 4 + 4/M
    "seq_update": None,         # read x and x_C, write x: 8 + 4/M
    "adamw_step": 28.0,         # read x, m1, m2, g; write x, m1, m2
    "adamw_reduce": 28.0,       # the same traffic, with the average and distances riding along
}
CALL_BYTES = {"round": 28.0, "pull_push": 12.0, "local_step": 20.0, "pull_push_exact": 12.0,
              "pull_then_push": None, "adamw_step": 28.0,       # None: depends on M or tau, see below
              "schedule": None, "round_adamw": 36.0}
CONFIG_ORDER = ["flat1m_M2", "resnet50_M4", "resnet101_M4", "vitb16_M4", "pyramidnet_M8"]


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2507_20424_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".h", ".hip")):
            with open(os.path.join(csrc, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(kernel: str, workload: str):
    """HBM bytes per launch from rocprofv3 counter runs, if they were taken on this very
    kernel source; None otherwise."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        table = json.load(f)
    if table.get("kernel_source_sha256_16") != kernel_source_hash():
        return None
    return table.get("bytes_per_launch", {}).get(f"{workload}:{kernel}")


def cpu_baseline(spec, inp, g_host, hyper, sample_cols: int, all_cores: bool):
    """The CPU oracle as it stands, timed on a bounded sample of the same workload (one local step
    + one round, float64).  One core: the first `sample_cols` coordinates of every worker.  All
    cores: every host core runs the same oracle call on its own slice of that many coordinates in
    total (each slice is treated as a whole model, so the distances are per slice -- the work per
    replica-parameter is the same)."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from oracle import dppf_oracle as O
    n = min(sample_cols, spec.d)
    x = np.stack([a[:n] for a in inp.x])
    v = np.stack([a[:n] for a in inp.v])
    g = np.stack([a[:n] for a in g_host])
    args = (hyper["lr"], hyper["mu"], hyper["wd"], hyper["pull"], hyper["push"])
    cores = os.cpu_count() or 1
    if all_cores:
        cores = min(cores, len(os.sched_getaffinity(0))) if hasattr(os, "sched_getaffinity") else cores
    times = []
    if not all_cores:
        for _ in range(3):           # the oracle returns new arrays and leaves its inputs alone
            t0 = time.perf_counter()
            O.dppf_round(x, v, g, *args)
            times.append(time.perf_counter() - t0)
        dt = min(times)
        return {"value": spec.M * n / dt, "unit": "replica-params/s", "cores": 1, "kind": "oracle",
                "sample": f"first {n} of d={spec.d} coordinates of all M={spec.M} workers, one local step + one "
                          f"round in float64 numpy, best of 3 runs: {dt:.1f} s"}
    bounds = [(n * k) // cores for k in range(cores + 1)]

    def one(k):
        a, b = bounds[k], bounds[k + 1]
        if b > a:
            O.dppf_round(x[:, a:b], v[:, a:b], g[:, a:b], *args)

    for _ in range(2):
        t0 = time.perf_counter()
        with ThreadPoolExecutor(cores) as pool:
            list(pool.map(one, range(cores)))
        times.append(time.perf_counter() - t0)
    dt = min(times)
    return {"value": spec.M * n / dt, "unit": "replica-params/s", "cores": cores, "nproc": os.cpu_count(),
            "kind": "oracle",
            "sample": f"the same {n} coordinates cut into {cores} slices, one thread per slice running the oracle's "
                      f"fused round on its slice (distances per slice), best of 2 runs: {dt:.1f} s"}


def kernel_table(recs, bytes_per_rp, n_rp):
    """Per-kernel averages of a list of (name, ms) timing records."""
    per_kernel = {}
    for name, ms in recs:
        per_kernel.setdefault(name, []).append(ms)
    out = {}
    for k, vv in per_kernel.items():
        avg = sum(vv) / len(vv)
        b = bytes_per_rp.get(k)
        gbs = b * n_rp / (avg * 1e-3) / 1e9 if b else None
        out[k] = {"launches": len(vv), "avg_ms": avg, "median_ms": sorted(vv)[len(vv) // 2], "min_ms": min(vv),
                  "GBps": gbs, "frac": gbs / HBM_PEAK_GBS if gbs else None}
    return out


def time_steps(step, steps, warmup, graph=False):
    """ms per step over `steps` back-to-back calls after `warmup` untimed ones (synchronised on both
    sides).  With graph=True one step is captured after the warm-up and its replays are timed."""
    import torch
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    if graph:
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            step()                       # the pointer tables are on the device before the capture starts
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=s):
                step()
            for _ in range(3):
                g.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                g.replay()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
        torch.cuda.current_stream().wait_stream(s)
        return 1e3 * dt / steps
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    return 1e3 * (time.perf_counter() - t0) / steps


def per_config_rows(dppf, W, steps, warmup, graph):
    """The fused round and the whole period on all five configurations.  Timing inputs come from
    the device's own generator at each configuration's scales (values do not change the traffic)."""
    import torch
    rows = []
    for name in CONFIG_ORDER:
        spec = W.SPECS[name]
        gen = torch.Generator(device="cuda")
        gen.manual_seed(spec.seed)

        def normal(n, scale):
            return torch.randn(n, device="cuda", generator=gen) * scale

        x0 = [normal(n, spec.sigma_x0) for n in spec.numel]
        spread = [spec.sigma_worker] * spec.M
        if spec.hetero_spread:           # log-uniform worker spreads in [1e-4, 1e-2]
            spread = (10.0 ** (-4.0 + 2.0 * torch.rand(spec.M, generator=torch.Generator().manual_seed(spec.seed)))).tolist()
        x = [[x0[t] + normal(n, spread[m]) for t, n in enumerate(spec.numel)] for m in range(spec.M)]
        del x0
        v = [[torch.zeros(n, device="cuda") for n in spec.numel] for _ in range(spec.M)]
        g = [[normal(n, spec.sigma_grad) for n in spec.numel] for _ in range(spec.M)]
        r = torch.zeros(spec.M, device="cuda")
        c = torch.zeros(spec.M, device="cuda")
        plan = dppf.Plan(spec.M, spec.numel)
        xt, vt, gt = dppf.PointerTable(x), dppf.PointerTable(v), dppf.PointerTable(g)
        f32 = lambda a: float(__import__("numpy").float32(a))  # noqa: E731
        lr, mu, wd, pull, push = f32(spec.lr), f32(spec.momentum), f32(spec.weight_decay), f32(spec.pull), f32(spec.push)

        def fused():
            plan.round(xt, vt, gt, lr, mu, wd, pull, push, r_out=r, c_out=c)

        def period():
            for _ in range(spec.tau - 1):
                plan.local_sgd_step(xt, vt, gt, lr, mu, wd)
            fused()

        n_rp = spec.M * spec.d
        k = max(5, min(steps, 30))
        ms_round = time_steps(fused, k, warmup)
        plan.timing_enable(True)
        for _ in range(k):
            fused()
        kernels = kernel_table(plan.timing_read(cap=8 * k + 8), BYTES_PER_RP, n_rp)
        plan.timing_enable(False)
        row = {"workload": name, "M": spec.M, "d": spec.d, "T": spec.T, "tau": spec.tau,
               "round_ms": ms_round, "round_replica_params_per_s": n_rp / (ms_round * 1e-3),
               "round_GBps": 28.0 * n_rp / (ms_round * 1e-3) / 1e9,
               "round_frac": 28.0 * n_rp / (ms_round * 1e-3) / 1e9 / HBM_PEAK_GBS,
               "kernels": {kk: {"avg_ms": vv["avg_ms"], "frac": vv["frac"]} for kk, vv in kernels.items()}}
        if graph:
            row["round_graph_ms"] = time_steps(fused, k, 2, graph=True)
        if spec.tau > 1:
            kp = max(3, min(steps, 10))
            ms_period = time_steps(period, kp, 2)
            bytes_period = (20.0 * (spec.tau - 1) + 28.0) * n_rp
            row.update({"period_ms": ms_period, "period_GBps": bytes_period / (ms_period * 1e-3) / 1e9,
                        "period_frac": bytes_period / (ms_period * 1e-3) / 1e9 / HBM_PEAK_GBS})
            if graph:
                row["period_graph_ms"] = time_steps(period, kp, 2, graph=True)
        torch.cuda.synchronize()
        assert torch.isfinite(r).all()
        rows.append(row)
        plan.close()
        del x, v, g, xt, vt, gt
        torch.cuda.empty_cache()
    return rows


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="vitb16_M4")
    ap.add_argument("--call", default="round", choices=sorted(CALL_BYTES))
    ap.add_argument("--workers", type=int, default=0,
                    help="override the workload's number of workers M (same list, same value scales)")
    ap.add_argument("--graph", action="store_true",
                    help="also time replays of a HIP graph that captured one step (headline and per-config rows)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch a plain 1 GiB copy (known size) so hardware counters can be scaled")
    ap.add_argument("--cpu-sample-cols", type=int, default=1_000_000_000)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU (the M workers are M replicas resident in one GPU's "
              "HBM); --gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2507_20424_amd import dppf, workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    spec = W.SPECS[args.workload]
    if args.workers > 0 and args.workers != spec.M:
        import dataclasses
        spec = dataclasses.replace(spec, name=f"{spec.name}_as_M{args.workers}", M=args.workers)
    f32 = lambda a: float(np.float32(a))  # noqa: E731
    hyper = dict(lr=f32(spec.lr), mu=f32(spec.momentum), wd=f32(spec.weight_decay), pull=f32(spec.pull),
                 push=f32(spec.push))
    inp = W.make_inputs(spec)
    g_host = inp.grads(0)

    def rows(arrays):     # one separately allocated device tensor per list entry, like a model's parameters
        out = []
        for a in arrays:
            out.append([torch.from_numpy(a[inp.offsets[t]:inp.offsets[t + 1]]).to("cuda") for t in range(spec.T)])
        return out

    x, v, g = rows(inp.x), rows(inp.v), rows(g_host)
    bytes_per_rp = dict(BYTES_PER_RP)
    bytes_per_rp["seq_reduce"] = 4.0 + 4.0 / spec.M
    bytes_per_rp["seq_update"] = 8.0 + 4.0 / spec.M
    call_bytes = dict(CALL_BYTES)
    call_bytes["pull_then_push"] = 12.0 + 8.0 / spec.M
    call_bytes["schedule"] = 20.0 * (spec.tau - 1) + 28.0     # tau-1 stand-alone steps + the fused round
    if args.call in ("adamw_step", "round_adamw"):
        m2 = rows(inp.v)
    if args.call == "pull_then_push":
        xc = [torch.from_numpy(inp.x[0][inp.offsets[t]:inp.offsets[t + 1]]).to("cuda") for t in range(spec.T)]
        xct = dppf.PointerTable(xc)
    r = torch.zeros(spec.M, device="cuda")
    c = torch.zeros(spec.M, device="cuda")
    plan = dppf.Plan(spec.M, spec.numel)
    xt, vt, gt = dppf.PointerTable(x), dppf.PointerTable(v), dppf.PointerTable(g)

    state = {"t": 0}
    m2t = dppf.PointerTable(m2) if args.call in ("adamw_step", "round_adamw") else None

    def step():
        if args.call == "round":
            plan.round(xt, vt, gt, hyper["lr"], hyper["mu"], hyper["wd"], hyper["pull"], hyper["push"], r_out=r,
                       c_out=c)
        elif args.call == "schedule":                        # the configuration's whole period
            for _ in range(spec.tau - 1):
                plan.local_sgd_step(xt, vt, gt, hyper["lr"], hyper["mu"], hyper["wd"])
            plan.round(xt, vt, gt, hyper["lr"], hyper["mu"], hyper["wd"], hyper["pull"], hyper["push"], r_out=r,
                       c_out=c)
        elif args.call == "pull_push":
            plan.pull_push_round(xt, hyper["pull"], hyper["push"], r_out=r, c_out=c)
        elif args.call == "pull_push_exact":
            plan.pull_push_round_exact(xt, hyper["pull"], hyper["push"] * spec.M, r_out=r, c_out=c)
        elif args.call == "pull_then_push":
            plan.pull_then_push(xt, xct, hyper["pull"], hyper["push"], "average", r_post_out=r)
        elif args.call == "adamw_step":
            state["t"] += 1
            plan.local_adamw_step(xt, vt, m2t, gt, 5e-4, 0.9, 0.999, 1e-8, 0.01, state["t"])
        elif args.call == "round_adamw":
            state["t"] += 1
            plan.round_adamw(xt, vt, m2t, gt, 5e-4, 0.9, 0.999, 1e-8, 0.01, state["t"], hyper["pull"],
                             hyper["push"], r_out=r, c_out=c)
        else:
            plan.local_sgd_step(xt, vt, gt, hyper["lr"], hyper["mu"], hyper["wd"])

    if args.copy_calibration:
        n_cal = 1 << 28                     # 1 GiB read + 1 GiB written per launch
        src = torch.ones(n_cal, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dppf.util_copy(dst, src, n_cal)
        torch.cuda.synchronize()
        del src, dst

    ms_per_step = time_steps(step, args.steps, args.warmup)
    n_rp = spec.M * spec.d
    value = n_rp / (ms_per_step * 1e-3)

    # per-kernel durations with HIP events on the launch stream, over the same number of steps
    plan.timing_enable(True)
    for _ in range(args.steps):
        step()
    kernels = kernel_table(plan.timing_read(cap=(8 + spec.tau) * args.steps + 8), bytes_per_rp, n_rp)
    plan.timing_enable(False)

    def roofline_of(name):
        k = kernels[name]
        return {"bound": "hbm", "kernel": name, "achieved": k["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": k["frac"], "traffic": measured_traffic(name, spec.name), "avg_kernel_ms": k["avg_ms"],
                "algorithmic_bytes_per_launch": bytes_per_rp[name] * n_rp}

    streaming = [k for k in kernels if kernels[k]["frac"]]
    dominant = max(streaming, key=lambda k: kernels[k]["avg_ms"] * kernels[k]["launches"])   # most GPU time in total
    lowest = min(streaming, key=lambda k: kernels[k]["frac"])
    torch.cuda.synchronize()
    assert torch.isfinite(r).all() and torch.isfinite(x[0][-1]).all()

    out = {
        "metric": "dppf_round_replica_params_per_s",
        "value": value,
        "unit": "replica-params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": spec.name, "call": f"dppf_{args.call}", "M": spec.M, "d": spec.d, "T": spec.T,
                   "replica_params": n_rp, "pull": hyper["pull"], "push": hyper["push"], "lr": hyper["lr"],
                   "momentum": hyper["mu"], "weight_decay": hyper["wd"]},
        "effective_GBps": call_bytes[args.call] * value / 1e9,
        "effective_frac_of_hbm_peak": call_bytes[args.call] * value / 1e9 / HBM_PEAK_GBS,
        "kernel_ms": {k: kk["avg_ms"] for k, kk in kernels.items()},
        "kernel_ms_median": {k: kk["median_ms"] for k, kk in kernels.items()},
        "kernel_ms_min": {k: kk["min_ms"] for k, kk in kernels.items()},
        "roofline": roofline_of(dominant),
        "roofline_lowest": roofline_of(lowest),
    }
    if args.graph:
        out["graph_replay_ms_per_step"] = time_steps(step, args.steps, 2, graph=True)
    plan.close()
    del x, v, g, xt, vt, gt
    torch.cuda.empty_cache()
    if not args.no_per_config:
        out["per_config"] = per_config_rows(dppf, W, args.steps, args.warmup, args.graph)
    if not args.no_cpu_baseline:
        cols = args.cpu_sample_cols
        out["cpu_baseline"] = cpu_baseline(spec, inp, g_host, hyper, cols, all_cores=False)
        out["cpu_baseline_all_cores"] = cpu_baseline(spec, inp, g_host, hyper, cols, all_cores=True)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
