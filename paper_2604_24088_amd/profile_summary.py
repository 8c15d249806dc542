"""Turns rocprofv3 CSV output into the short text tables kept under profiles/.

    python -m paper_2604_24088_amd.profile_summary [--stats DIR] [--trace DIR] [--fetch DIR] [--write DIR] [--pmc DIR ...]
                                                   [--elements N --block B --k K]

  --stats DIR   output directory of   rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o bench -- python3 bench.py ...
                -> per kernel: calls, average / minimum / maximum duration, share of the GPU time
  --fetch DIR   output directory of   rocprofv3 --pmc FETCH_SIZE --output-format csv -d DIR -o bench -- python3 bench.py ...
  --write DIR   the same with WRITE_SIZE
                -> per kernel: mean counter value per dispatch (KiB), scaled by what the same counter reads for the
                   plain copy kernel of known size (taco_debug_copy of 393216 KiB in bench.py), i.e. HBM bytes per launch
  --pmc DIR     output directory of any other   rocprofv3 --pmc <counters> ...   run: mean of every counter per kernel
  --elements / --block / --k   when given, the algorithmic bytes of compress, decompress, decompress_sum(k) and the fused
                call on a tensor of N elements are printed beside the traffic, with the ratio; the stats section adds the
                compress kernel's algorithmic bytes over its average duration as a share of the 8000 GB/s HBM peak, the
                counter sections add, per kernel, the chip's busy cycles, the matrix cores' busy share and the vector
                instructions per tile of 2048 elements with their issue share
  --trace DIR   the same directory as --stats (it holds the kernel trace): per kernel, the median duration and the median idle gap
                before it, apart for launches that follow another kernel (as in a bench step) and launches that follow the same
                kernel (back-to-back runs); the gap is what HIP-event times between calls contain beside the kernel itself
  --bench FILE ...   JSON lines printed by bench.py (one file per run): one table row per run with the step and each
                call's time and share of the HBM peak (in step, back to back, memory-only yardstick), and with
                --workloads the per-configuration table of the default run

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


def trace_split(directory: str):
    """Median duration and preceding idle gap per kernel, split by whether the previous kernel on the device was the same one."""
    import statistics
    rows = list(csv.DictReader(open(find_csv(directory, "kernel_trace.csv"))))
    seq = sorted((int(r["Start_Timestamp"]), int(r["End_Timestamp"]), short(r["Kernel_Name"])) for r in rows)
    groups = collections.defaultdict(lambda: ([], []))
    for (s0, e0, n0), (s1, e1, n1) in zip(seq, seq[1:]):
        dur, gap = groups[(n1, n0 == n1)]
        dur.append(e1 - s1)
        gap.append(s1 - e0)
    print("== kernel trace: median duration (ns) by what ran before the launch, and the idle gaps before it (a launch that "
          "follows a HIP event record waits for the event's marker packet; launches that follow a kernel directly show no gap)")
    for (name, same), (dur, gap) in sorted(groups.items()):
        if len(dur) < 4:
            continue
        held = [g for g in gap if g > 1000]
        print(f"  {name:78s} after {'itself        ' if same else 'another kernel'} launches={len(dur):4d} "
              f"duration={statistics.median(dur):9.0f}  launches with a gap over 1 us: {len(held):4d}"
              + (f", their median gap {statistics.median(held):7.0f}" if held else ""))
    print()


def load_bench(path: str):
    import json
    for line in open(path):
        line = line.strip()
        if line.startswith("{"):
            return json.loads(line)
    raise SystemExit(f"no JSON line in {path}")


def bench_rows(paths, workloads: bool):
    """One row per bench.py run: us and share of the 8 TB/s HBM peak (algorithmic bytes / time) per call."""
    def cell(e):
        return f"{e['ms'] * 1e3:7.1f} {e['hbm_frac']:.3f}" if e else "      -     -"

    print("== bench.py runs: per call  us  share-of-HBM-peak;  step = ms per step and share for the whole step")
    print(f"  {'run':48s} {'step':>13s} | in step: {'compress':>13s} {'decompress':>13s} {'sum(k)':>13s} {'sum->compress':>13s} | "
          f"back to back: {'compress':>13s} {'decompress':>13s} {'sum(k)':>13s} | yardstick: {'compress':>13s} {'decompress':>13s} {'sum(k)':>13s} "
          f"{'sum->compress':>13s}")
    for path in paths:
        r = load_bench(path)
        c = r["config"]
        k = next((key.rsplit("_k", 1)[1] for key in r["calls"] if key.startswith("decompress_sum_k")), "?")
        tag = (f"{c['workload'].split(':')[0]} k={k} B={c['block']} {c['layout']} {c['impl']} fmt={c['format']} mode={c['mode']}"
               + (f" chunks={c['chunks_per_call']}x{c['streams']}" if c.get("chunks_per_call", 1) > 1 else "")
               + (" batch" if c.get("batched_calls") else "") + (" graph" if c.get("hip_graph") else ""))
        calls = list(r["calls"].values())
        b2b = list(r.get("calls_back_to_back", {}).values()) + [None] * 3
        mix = r.get("mix_yardstick", {})
        mixv = [mix.get("compress"), mix.get("decompress"),
                next((v for k, v in mix.items() if k.startswith("decompress_sum_k")), None),
                next((v for k, v in mix.items() if k.startswith("decompress_sum_compress")), None)]
        print(f"  {tag:48s} {r['ms_per_step']:7.4f} {r['hbm_frac_step']:.3f} |          {cell(calls[0])} {cell(calls[1])} {cell(calls[2])} "
              f"{cell(calls[3]) if len(calls) > 3 else cell(None)} |               {cell(b2b[0])} {cell(b2b[1])} {cell(b2b[2])} |            "
              f"{cell(mixv[0])} {cell(mixv[1])} {cell(mixv[2])} {cell(mixv[3])}")
        if workloads and "workloads" in r:
            print("  per configuration (steps rotate through `sets` buffer sets so that cache-sized tensors are still timed from HBM):")
            print(f"    {'workload':12s} {'shape':>16s} {'k':>2s} {'sets':>4s} {'ms/step':>8s} | in step (median): {'compress':>13s} {'decompress':>13s} "
                  f"{'sum(k)':>13s} | back to back: {'compress':>13s} {'decompress':>13s} {'sum(k)':>13s} | batched, per tensor: {'compress':>13s} "
                  f"{'decompress':>13s} {'sum(k)':>13s}")
            for name, e in r["workloads"].items():
                i = list(e["in_step_median"].values())
                b = list(e["back_to_back"].values())
                bt = e.get("batched", {})
                bt = [bt.get("compress"), bt.get("decompress"), next((v for k, v in bt.items() if k.startswith("decompress_sum_k")), None)]
                print(f"    {name:12s} {str(e['shape']):>16s} {e['payloads']:2d} {e['buffer_sets']:4d} {e['ms_per_step']:8.4f} |                   "
                      f"{cell(i[0])} {cell(i[1])} {cell(i[2])} |               {cell(b[0])} {cell(b[1])} {cell(b[2])} |                      "
                      f"{cell(bt[0])} {cell(bt[1])} {cell(bt[2])}")
        if r.get("calls_same_payload_k_times"):
            print("    one payload given k times (reads from cache): " +
                  ", ".join(f"{k} {v['ms'] * 1e3:.1f} us" for k, v in r["calls_same_payload_k_times"].items()))
        for key in ("cpu_baseline", "cpu_baseline_1thread"):
            if key in r:
                e = r[key]
                print(f"    {key}: {e['value']:.4f} {e['unit']} on {e['cores']} thread(s); {e['sample']}")
    print()


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--stats")
    ap.add_argument("--trace")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--pmc", action="append", default=[])
    ap.add_argument("--elements", type=int, default=0)
    ap.add_argument("--block", type=int, default=128)
    ap.add_argument("--k", type=int, default=8)
    ap.add_argument("--bench", nargs="*", default=[])
    ap.add_argument("--workloads", action="store_true")
    a = ap.parse_args()
    if a.bench:
        bench_rows(a.bench, a.workloads)
    if a.stats:
        print("== kernel stats (rocprofv3 --kernel-trace --stats): calls, average / min / max duration in ns, share of GPU time")
        rows = kernel_stats(a.stats)
        for name, calls, avg, mn, mx, pct in rows:
            print(f"  {name:78s} calls={calls:5d} avg_ns={avg:10.1f} min_ns={mn:8d} max_ns={mx:8d} pct={pct:5.2f}")
        if a.elements:
            per = 1.0 + 8.0 / a.block
            for name, calls, avg, mn, mx, pct in rows:
                if name.startswith("compress_"):
                    alg = (2.0 + per) * a.elements
                    print(f"  roofline check, {name}: {alg:.0f} algorithmic bytes / {avg / 1e3:.2f} us average = {alg / avg:.0f} GB/s = "
                          f"{alg / avg / 8000.0:.3f} of 8000 GB/s")
        print()
    if a.trace:
        trace_split(a.trace)
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
        for kname, grid in sorted({(kn, g) for (kn, g, _) in tab}):
            print(f"  {kname}  grid={grid}")
            cells = [f"{c} {tab[(kname, grid, c)][1]:.0f}" for c in names if (kname, grid, c) in tab]
            for i in range(0, len(cells), 4):
                print("      " + "   ".join(f"{x:38s}" for x in cells[i:i + 4]).rstrip())
            get = lambda c: tab.get((kname, grid, c), (0, 0.0))[1]
            busy = get("SQ_BUSY_CYCLES") / 32.0                 # the counter sums over the 32 shader engines
            if busy > 0 and get("SQ_VALU_MFMA_BUSY_CYCLES") > 0:
                mfma = get("SQ_VALU_MFMA_BUSY_CYCLES") / 1024.0  # per SIMD (256 compute units x 4)
                line = (f"      derived: busy cycles of the chip {busy / 1e3:.0f} k; matrix cores busy per SIMD {mfma / 1e3:.0f} k = "
                        f"{mfma / busy:.3f} of them")
                if a.elements and get("SQ_INSTS_VALU") > 0:
                    tiles = a.elements / 2048.0
                    valu = get("SQ_INSTS_VALU")
                    line += (f"; vector instructions per tile of 2048 elements {valu / tiles:.0f}, at four issue cycles each "
                             f"{valu / 1024.0 * 4 / 1e3:.0f} k cycles per SIMD = {valu / 1024.0 * 4 / busy:.2f}")
                print(line)
        print()
    if not (a.stats or a.trace or a.fetch or a.write or a.pmc or a.bench):
        ap.print_help()
        sys.exit(1)


if __name__ == "__main__":
    main()
