"""Practical HBM bandwidth of the device for several read/write mixes.

    python -m paper_2507_20424_amd.ceiling [--total-gib 4] [--reps 10]

Runs the library's streaming probe (``dppf_util_stream_probe``) over a footprint far larger than
the last-level cache and prints, per mix, the best rate over 1, 2 and 8 resident blocks per CU,
once with the work split evenly over the blocks and once with the work handed out on demand.
These are the ceilings the DPPF kernels are compared with next to the 8 TB/s datasheet peak."""
from __future__ import annotations

import argparse
import json
import sys

MIXES = [(1, 0, False), (4, 0, False), (12, 0, False), (0, 1, False), (0, 4, False), (1, 1, False), (2, 1, False),
         (4, 4, False), (4, 4, True), (8, 4, False), (8, 4, True), (12, 4, False), (12, 4, True),
         (12, 8, False), (12, 8, True), (16, 8, True), (24, 8, True)]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--total-gib", type=float, default=4.0)
    ap.add_argument("--reps", type=int, default=10)
    args = ap.parse_args()
    import torch
    from paper_2507_20424_amd import dppf
    if not torch.cuda.is_available():
        print("ceiling: no GPU visible", file=sys.stderr)
        return 2
    total_floats = int(args.total_gib * (1 << 28))
    skew = 17_472                                   # floats; keeps streams off a common power-of-two stride
    buf = torch.zeros(total_floats + 32 * skew, dtype=torch.float32, device="cuda")
    rows = []
    for reads, writes, inplace in MIXES:
        streams = reads + (0 if inplace else writes)
        n = (total_floats // streams) // 16384 * 16384
        stride = n + skew
        moved = 4.0 * n * (reads + writes)
        best = {False: (0.0, 0), True: (0.0, 0)}
        for on_demand in (False, True):
            for bpc in (1, 2, 8):
                for _ in range(2):
                    dppf.util_stream_probe(buf, stride, n, reads, writes, inplace, bpc, on_demand)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(args.reps):
                    dppf.util_stream_probe(buf, stride, n, reads, writes, inplace, bpc, on_demand)
                e1.record()
                torch.cuda.synchronize()
                gbs = moved / (e0.elapsed_time(e1) / args.reps * 1e-3) / 1e9
                if gbs > best[on_demand][0]:
                    best[on_demand] = (gbs, bpc)
        rows.append({"reads": reads, "writes": writes, "inplace": inplace,
                     "GBps_even_split": round(best[False][0], 1), "blocks_per_cu_even_split": best[False][1],
                     "GBps_on_demand": round(best[True][0], 1), "blocks_per_cu_on_demand": best[True][1],
                     "footprint_GB": round(4.0 * n * streams / 1e9, 2)})
        print(f"R={reads:2d} W={writes:2d} {'in place' if inplace else '        '}  even split {best[False][0]:7.0f} GB/s "
              f"({100 * best[False][0] / 8000:.1f} %) at {best[False][1]} block(s)/CU;  on demand "
              f"{best[True][0]:7.0f} GB/s ({100 * best[True][0] / 8000:.1f} %) at {best[True][1]} block(s)/CU;  "
              f"footprint {4.0 * n * streams / 1e9:.2f} GB", flush=True)
    print(json.dumps({"probe": rows}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
