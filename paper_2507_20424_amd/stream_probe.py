"""HBM bandwidth of the device for several read/write mixes and two access orders.

    python -m paper_2507_20424_amd.stream_probe [--total-gib 4] [--reps 10] [--only all-at-once|grouped|offsets]

Runs the library's two streaming probes over a footprint far larger than the last-level cache.

* "all at once" (``dppf_util_stream_probe``): R read arrays and W written arrays, every array
  touched by every lane at once; per mix the best rate over 1, 2 and 8 resident blocks per CU,
  with the work split evenly over the blocks and with the work handed out on demand.
* "group by group" (``dppf_util_stream_probe_grouped``): the order the library's sweeps use -- one
  worker's arrays after the other inside a tile, each group's first array overwritten in place.
  It is the traffic of a sweep with none of its arithmetic, reductions or pointer tables, so it
  says how much of a sweep's time is the memory system's and how much the kernel's own.

Neither is an upper bound of the device: both are access patterns, measured."""
from __future__ import annotations

import argparse
import json
import sys

MIXES = [(1, 0, False), (4, 0, False), (12, 0, False), (0, 1, False), (0, 4, False), (1, 1, False), (2, 1, False),
         (4, 4, False), (4, 4, True), (8, 4, False), (8, 4, True), (12, 4, False), (12, 4, True),
         (12, 8, False), (12, 8, True), (16, 8, True), (24, 8, True)]

# (groups, reads per group, vectors per lane and array, groups requested ahead, the sweep it mimics)
GROUPED = [(2, 3, 4, 0, "sweep 1 of the fused round, M = 2 (as built)"),
           (4, 3, 4, 0, "sweep 1 of the fused round, M = 4 (as built)"),
           (4, 3, 4, 3, "same, all workers' loads requested ahead"),
           (4, 3, 2, 0, "same, two vectors per lane"),
           (4, 3, 8, 0, "same, eight vectors per lane"),
           (4, 2, 4, 0, "sweep 2 of the fused round, M = 4, no look-ahead"),
           (4, 2, 4, 3, "sweep 2 of the fused round, M = 4 (as built: it needs every worker before it can store)"),
           (4, 2, 8, 0, "same, eight vectors per lane"),
           (4, 1, 4, 0, "sweep 2 of the plain round, M = 4"),
           (8, 3, 2, 0, "sweep 1 of the fused round, M = 8, no look-ahead"),
           (8, 3, 2, 7, "sweep 1 of the fused round, M = 8 (as built)"),
           (8, 2, 2, 0, "sweep 2 of the fused round, M = 8, no look-ahead"),
           (8, 2, 2, 7, "sweep 2 of the fused round, M = 8 (as built)"),
           (16, 3, 2, 0, "sweep 1 of the fused round, M = 16, no look-ahead"),
           (16, 3, 2, 7, "sweep 1 of the fused round, M = 16 (as built)"),
           (16, 2, 2, 7, "sweep 2 of the fused round, M = 16, eight workers requested ahead")]

# Shapes that are also timed with the arrays at several distances from one another: the array
# length plus this many floats (--offsets).
OFFSET_SHAPES = [(4, 3, 4, 0), (8, 3, 2, 7), (16, 3, 2, 0), (16, 3, 2, 7)]
OFFSETS = [0, 256, 1024, 4096, 17_472, 65_536, 100_000, 1_048_576]


def _time(launch, reps: int) -> float:
    import torch
    for _ in range(2):
        launch()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        launch()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps * 1e-3


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--total-gib", type=float, default=4.0)
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--only", choices=["all-at-once", "grouped", "offsets"], default=None)
    args = ap.parse_args()
    import torch
    from paper_2507_20424_amd import dppf
    if not torch.cuda.is_available():
        print("stream_probe: no GPU visible", file=sys.stderr)
        return 2
    total_floats = int(args.total_gib * (1 << 28))
    skew = 17_472                                   # floats; keeps arrays off a common power-of-two stride
    buf = torch.zeros(total_floats + 64 * max(OFFSETS), dtype=torch.float32, device="cuda")
    rows, grouped_rows, offset_rows = [], [], []
    for reads, writes, inplace in (MIXES if args.only in (None, "all-at-once") else []):
        streams = reads + (0 if inplace else writes)
        n = (total_floats // streams) // 16384 * 16384
        stride = n + skew
        moved = 4.0 * n * (reads + writes)
        best = {False: (0.0, 0), True: (0.0, 0)}
        for on_demand in (False, True):
            for bpc in (1, 2, 8):
                secs = _time(lambda: dppf.util_stream_probe(buf, stride, n, reads, writes, inplace, bpc, on_demand),
                             args.reps)
                gbs = moved / secs / 1e9
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
    for groups, per_group, vectors, ahead, what in (GROUPED if args.only in (None, "grouped") else []):
        streams = groups * per_group
        n = (total_floats // streams) // 16384 * 16384
        stride = n + skew
        moved = 4.0 * n * groups * (per_group + 1)
        rates = {}
        for on_demand in (False, True):
            for bpc in (1, 2):
                secs = _time(lambda: dppf.util_stream_probe_grouped(buf, stride, n, groups, per_group, vectors, ahead,
                                                                    bpc, on_demand), args.reps)
                rates[(on_demand, bpc)] = moved / secs / 1e9
        grouped_rows.append({"groups": groups, "reads_per_group": per_group, "vectors": vectors, "ahead": ahead,
                             "mimics": what, "footprint_GB": round(4.0 * n * streams / 1e9, 2),
                             **{f"GBps_{'on_demand' if od else 'even_split'}_{bpc}_per_cu": round(v, 1)
                                for (od, bpc), v in rates.items()}})
        print(f"{groups:2d} groups x ({per_group} R + 1 W in place), {vectors} vectors/lane, {ahead} ahead:  "
              f"on demand {rates[(True, 1)]:6.0f} GB/s ({100 * rates[(True, 1)] / 8000:.1f} %) at 1 block/CU, "
              f"{rates[(True, 2)]:6.0f} at 2;  even split {rates[(False, 1)]:6.0f} at 1, {rates[(False, 2)]:6.0f} at 2"
              f"   [{what}]", flush=True)
    # the same order with the arrays at other distances from one another (on demand, 1 block per CU)
    for groups, per_group, vectors, ahead in (OFFSET_SHAPES if args.only in (None, "offsets") else []):
        streams = groups * per_group
        n = (total_floats // streams) // 16384 * 16384
        moved = 4.0 * n * groups * (per_group + 1)
        rates = []
        for off in OFFSETS:
            secs = _time(lambda: dppf.util_stream_probe_grouped(buf, n + off, n, groups, per_group, vectors, ahead, 1,
                                                                True), args.reps)
            rates.append(round(moved / secs / 1e9, 1))
        offset_rows.append({"groups": groups, "reads_per_group": per_group, "vectors": vectors, "ahead": ahead,
                            "array_floats": n, "offsets_floats": OFFSETS, "GBps": rates})
        print(f"{groups:2d} groups x ({per_group} R + 1 W in place), {vectors} vectors/lane, {ahead} ahead, arrays "
              f"{n} floats + offset apart:  " + "  ".join(f"+{o}: {r:.0f}" for o, r in zip(OFFSETS, rates)), flush=True)
    print(json.dumps({"probe": rows, "probe_grouped": grouped_rows, "probe_offsets": offset_rows}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
