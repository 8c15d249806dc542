"""Turns rocprofv3 CSV output into the short text tables kept under profiles/.

    python -m paper_2604_24088_amd.profile_summary [--stats DIR] [--fetch DIR] [--write DIR] [--pmc DIR ...]
                                                   [--elements N --block B --k K]

  --stats DIR   output directory of   rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o bench -- python3 bench.py ...
                -> per kernel: calls, average / minimum / maximum duration, share of the GPU time
  --fetch DIR   output directory of   rocprofv3 --pmc FETCH_SIZE --output-format csv -d DIR -o bench -- python3 bench.py ...
  --write DIR   the same with WRITE_SIZE
                -> per kernel: mean counter value per dispatch (KiB), scaled by what the same counter reads for the
                   plain copy kernel of known size (taco_debug_copy of 393216 KiB in bench.py), i.e. HBM bytes per launch
  --pmc DIR     output directory of any other   rocprofv3 --pmc <counters> ...   run: mean of every counter per kernel
  --elements / --block / --k   when given, the algorithmic bytes of compress, decompress, decompress_sum(k) and the fused
                call on a tensor of N elements are printed beside the traffic, with the ratio

Only the standard library is used; nothing here touches the GPU.
"""
import argparse
import collections
import csv
import glob
import os
import sys

COPY_KIB = 393216.0          # bench.py's copy yardstick moves 384 MiB each way (1 GiB tensors are cut to that size)


def short(name: str) -> str:
    return name.split("(")[0].replace("taco::", "").replace("void ", "").strip()


def find_csv(directory: str, suffix: str) -> str:
    hits = glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True)
    if not hits:
        raise SystemExit(f"no *{suffix} under {directory}")
    return sorted(hits)[0]


def kernel_stats(directory: str):
    rows = list(csv.DictReader(open(find_csv(directory, "kernel_stats.csv"))))
    out = []
    for r in rows:
        out.append((short(r["Name"]), int(r["Calls"]), float(r["AverageNs"]), int(float(r["MinNs"])), int(float(r["MaxNs"])),
                    float(r["Percentage"])))
    return sorted(out, key=lambda t: -t[5])


def counters(directory: str):
    """{(kernel, grid size, counter): (dispatches, mean value)}; kernels of one name are kept apart by grid size, which
    tells the k = 1 decode from the k = 8 one."""
    agg = collections.defaultdict(lambda: [0, 0.0])
    for r in csv.DictReader(open(find_csv(directory, "counter_collection.csv"))):
        key = (short(r["Kernel_Name"]), r.get("Grid_Size", ""), r["Counter_Name"])
        agg[key][0] += 1
        agg[key][1] += float(r["Counter_Value"])
    return {k: (n, v / n) for k, (n, v) in agg.items()}


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--stats")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--pmc", action="append", default=[])
    ap.add_argument("--elements", type=int, default=0)
    ap.add_argument("--block", type=int, default=128)
    ap.add_argument("--k", type=int, default=8)
    a = ap.parse_args()
    if a.stats:
        print("== kernel stats (rocprofv3 --kernel-trace --stats): calls, average / min / max duration in ns, share of GPU time")
        for name, calls, avg, mn, mx, pct in kernel_stats(a.stats):
            print(f"  {name:78s} calls={calls:5d} avg_ns={avg:10.1f} min_ns={mn:8d} max_ns={mx:8d} pct={pct:5.2f}")
        print()
    if a.fetch or a.write:
        print("== HBM traffic counters: mean per dispatch in KiB as the counter reports it, and scaled by the copy kernel "
              f"(which moves {COPY_KIB:.0f} KiB each way)")
        scaled = {}
        for label, directory in (("FETCH_SIZE", a.fetch), ("WRITE_SIZE", a.write)):
            if not directory:
                continue
            tab = counters(directory)
            copy = [v for (kname, _, c), v in tab.items() if kname == "copy_kernel" and c == label]
            factor = COPY_KIB / copy[0][1] if copy else float("nan")
            print(f"  {label}: scale factor from the copy kernel x {factor:.6f}")
            for (kname, grid, c), (n, mean) in sorted(tab.items()):
                if c != label:
                    continue
                print(f"    {kname:78s} grid={grid:>10s} dispatches={n:4d} mean={mean:12.1f}  scaled={mean * factor:12.1f} KiB")
                scaled.setdefault((kname, grid), {})[label] = mean * factor * 1024.0
        if a.elements:
            n, B, k = a.elements, a.block, a.k
            per = 1.0 + 8.0 / B
            alg = {"compress / decompress": (2.0 + per) * n, f"decompress_sum(k={k})": (k * per + 2.0) * n,
                   f"fused sum -> compress (k={k})": (k + 1) * per * n}
            print(f"  algorithmic bytes on {n} elements, block {B}: " + "; ".join(f"{w} {v:.0f}" for w, v in alg.items()))
            for (kname, grid), d in sorted(scaled.items()):
                if "FETCH_SIZE" in d and "WRITE_SIZE" in d:
                    total = d["FETCH_SIZE"] + d["WRITE_SIZE"]
                    near = min(alg.items(), key=lambda kv: abs(kv[1] - total))
                    print(f"    {kname:78s} grid={grid:>10s} fetch+write={total:14.0f} B = {total / near[1]:.5f} x {near[0]}")
        print()
    for directory in a.pmc:
        tab = counters(directory)
        names = sorted({c for (_, _, c) in tab})
        print(f"== counters from {os.path.basename(os.path.normpath(directory))}: mean per dispatch, summed over the chip")
        print("  " + " " * 78 + " " + "      grid " + " ".join(f"{c:>26s}" for c in names))
        for kname, grid in sorted({(kn, g) for (kn, g, _) in tab}):
            vals = " ".join(f"{tab.get((kname, grid, c), (0, float('nan')))[1]:26.1f}" for c in names)
            print(f"  {kname:78s} {grid:>10s} {vals}")
        print()
    if not (a.stats or a.fetch or a.write or a.pmc):
        ap.print_help()
        sys.exit(1)


if __name__ == "__main__":
    main()
