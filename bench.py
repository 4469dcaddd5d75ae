#!/usr/bin/env python3
"""Benchmark of the DPPF consensus round on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--call round|pull_push|local_step]

One "step" is one pass of the whole hot path over one batch of synthetic input: the fused
`dppf_round` (last local momentum-SGD step + replica average + distances + pull-push update)
over the M resident replicas of a ViT-B/16-sized parameter list.  Inputs are generated on the
host with the seeded recipe of `paper_2507_20424_amd.workloads`, uploaded once, and resident
in HBM before the timed region starts.  Prints ONE JSON line.
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


def cpu_baseline(spec, inp, g_host, hyper, sample_cols: int):
    """The CPU oracle as it stands, timed on a bounded sample of the same workload: the first
    `sample_cols` coordinates of every worker (one local step + one round, float64).  Whatever
    --call is benchmarked, this leg always times the fused round's oracle."""
    import numpy as np
    from oracle import dppf_oracle as O
    n = min(sample_cols, spec.d)
    x = np.stack([a[:n] for a in inp.x])
    v = np.stack([a[:n] for a in inp.v])
    g = np.stack([a[:n] for a in g_host])
    times = []
    for _ in range(3):           # the oracle returns new arrays and leaves its inputs alone
        t0 = time.perf_counter()
        O.dppf_round(x, v, g, hyper["lr"], hyper["mu"], hyper["wd"], hyper["pull"], hyper["push"])
        times.append(time.perf_counter() - t0)
    dt = min(times)
    return {"value": spec.M * n / dt, "unit": "replica-params/s", "cores": 1, "kind": "oracle",
            "sample": f"first {n} of d={spec.d} coordinates of all M={spec.M} workers, one local step + one "
                      f"round in float64 numpy, best of 3 runs: {dt:.1f} s"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="vitb16_M4")
    ap.add_argument("--call", default="round", choices=sorted(CALL_BYTES))
    ap.add_argument("--no-cpu-baseline", action="store_true")
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

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps
    n_rp = spec.M * spec.d
    value = n_rp / (dt / args.steps)

    # per-kernel durations with HIP events on the launch stream, over the same number of steps
    plan.timing_enable(True)
    for _ in range(args.steps):
        step()
    recs = plan.timing_read(cap=(8 + spec.tau) * args.steps + 8)
    plan.timing_enable(False)
    per_kernel = {}
    for name, ms in recs:
        per_kernel.setdefault(name, []).append(ms)
    avg_ms = {k: sum(vv) / len(vv) for k, vv in per_kernel.items()}
    min_ms = {k: min(vv) for k, vv in per_kernel.items()}
    med_ms = {k: sorted(vv)[len(vv) // 2] for k, vv in per_kernel.items()}
    dominant = max(avg_ms, key=lambda k: avg_ms[k] * len(per_kernel[k]))     # most GPU time in total
    achieved = bytes_per_rp[dominant] * n_rp / (avg_ms[dominant] * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(dominant, spec.name),
                "avg_kernel_ms": avg_ms[dominant],
                "algorithmic_bytes_per_launch": bytes_per_rp[dominant] * n_rp}
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
        "kernel_ms": avg_ms,
        "kernel_ms_median": med_ms,
        "kernel_ms_min": min_ms,
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(spec, inp, g_host, hyper, args.cpu_sample_cols)
    plan.close()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
