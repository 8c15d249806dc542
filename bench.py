#!/usr/bin/env python3
"""Throughput of the TACO fused FP8 compression operator on one MI355X.

One STEP is one pass of the whole hot path over one batch of synthetic input:
    k x taco_compress  ->  taco_decompress (payload 0)  ->  taco_decompress_sum (all k)
The headline is the `large_k8` workload (bf16 [16384, 12288], k = 8 payloads, block 128): the largest
single-GPU configuration, and the one whose buffers (3 GiB of inputs) cannot sit in the 256 MB
last-level cache.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` counts bf16-equivalent bytes: 2N per compressed tensor, 2N per
decompressed tensor, k*2N for decompress_sum (k tensors decoded); `value_out_basis` counts only bf16
bytes that really cross HBM; `hbm_frac_step` prices the ALGORITHMIC bytes of the whole step.
The timed region records two HIP events per step: one at its start and one after the compress group, after
decompress or after decompress_sum, in turn over the steps.  `calls` gives the compress launch time from
the first kind of step (the roofline's launch duration is its average) and the two decode calls as
differences of the medians of those intervals: no event sits between the kernels they cover.  A launch that
follows an event record waits about 6 us for the event's marker packet (the kernel trace shows the gap,
and kernel durations equal to the back-to-back ones); `calls_with_events_between_calls` and
`ms_per_step_with_events_between_calls` are the same steps run once more with events around every call.
`calls_back_to_back` times 16 launches of one call in a row, which is what a kernel
costs when the host's launch time is not in the way.  `workloads` carries the same two measurements for
every one of the five benchmark configurations (steps rotate through enough buffer sets to defeat the
last-level cache).  `mix_yardstick` times memory-only kernels (taco_debug_traffic) that move exactly the
bytes of each call and compute nothing: what the memory system gives that mix.  `calls_same_payload_k_times`
is the opposite cut: the decode calls with one payload given k times, so that the reads come from cache and
the time left is what the kernel needs for everything but HBM.
The roofline object prices the dominant kernel (compress) by its ALGORITHMIC bytes (3.0625 B per
element at block 128) over its average launch duration inside the timed region.
`cpu_baseline` / `cpu_baseline_1thread`: the CPU oracle, as it stands, on a stated sample of the same
workload with all host threads and with one.

Before the warm-up steps the step loop runs untimed for `--settle-ms` (default 60 ms): from a cold start
the GPU's power management runs the first two steps at boost clocks, then drops (the decode kernels run
up to 35 % slower around the third to fifth step) and needs about 25 steps to settle; `--cold-trace N`
prints that transient (per-step call times from a cold start) instead of the benchmark.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, vendor figure

# HBM traffic per launch of the dominant kernel measured with rocprofv3 --pmc (FETCH_SIZE and
# WRITE_SIZE runs, scaled by a copy kernel of known size); None until measured.  The summary
# the number comes from is committed under profiles/.
MEASURED_TRAFFIC_BYTES = {
    # fetch 393272 KiB + write 208896 KiB per compress launch: profiles/mfma_kernels_large_k8.txt
    ("large_k8", 128, "auto"): 616619620,
}

# Share of time the matrix cores are busy in the dominant kernel (SQ_VALU_MFMA_BUSY_CYCLES over SIMD-cycles,
# rocprofv3 --pmc run summarised in the same profile); the Hadamard rotation is an MFMA contraction there.
MEASURED_MFMA_BUSY = {("large_k8", 128, "auto"): 0.202}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="large_k8")
    ap.add_argument("--block", type=int, default=128)
    ap.add_argument("--impl", default="auto", choices=["auto", "butterfly", "mfma"])
    ap.add_argument("--layout", default="split", choices=["split", "interleaved"])
    ap.add_argument("--format", default="e4m3", choices=["e4m3", "e5m2", "int8"], help="code book (ablation variants)")
    ap.add_argument("--mode", type=int, default=7, help="bit mask of the method's stages: 1 rescale, 2 rotate, 4 post-scale")
    ap.add_argument("--chunk-mb", type=float, default=0.0,
                    help="issue every call in row chunks of about this many MB of bf16 (0 = whole tensor): the overlap "
                         "granularity of Section 4.4.2")
    ap.add_argument("--streams", type=int, default=1, help="streams the chunks are dealt to in turn (with --chunk-mb)")
    ap.add_argument("--batch", action="store_true",
                    help="use the batched entry points: the k compress calls of a step, and with --chunk-mb all chunks of a "
                         "call, go out as ONE launch each")
    ap.add_argument("--rotate", type=int, default=0,
                    help="buffer sets the steps rotate through (0 = as many as it takes, up to 64, for the sets to exceed "
                         "1 GiB together, so that workloads smaller than the 256 MB last-level cache are still timed from HBM)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the three parts of the step into HIP graphs and time their replays (takes the "
                         "host's launch cost out of chunked runs)")
    ap.add_argument("--settle-ms", type=float, default=60.0,
                    help="untimed run of the step loop before the warm-up steps, so that the GPU's clocks have settled")
    ap.add_argument("--cold-trace", type=int, default=0,
                    help="print the per-step call times of this many steps from a cold start and exit")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--payloads", type=int, default=0,
                    help="number of payloads k of the step (1..16) instead of the workload's own (beyond those the data repeats, in buffers of "
                         "their own).  "
                         "Implies --no-cpu-baseline and --no-workloads")
    ap.add_argument("--no-cache-fed", action="store_true",
                    help="skip the decode calls with one payload given k times (counter runs: their dispatches carry the same "
                         "kernel name and grid as the real ones)")
    ap.add_argument("--no-workloads", action="store_true", help="skip the per-configuration table (headline workload only)")
    ap.add_argument("--gen-threads", type=int, default=16)
    return ap.parse_args()


def oracle_step(w, block, rows):
    """One step's call mix on the first `rows` tokens of every payload, on the oracle; returns (seconds, results)."""
    from oracle import taco_ref
    from paper_2604_24088_amd import workloads as W
    xs = [W.generate_rows(w, i, 0, rows) for i in range(w.payloads)]
    n = rows * w.hidden
    t0 = time.perf_counter()
    enc = [taco_ref.compress(x, block=block) for x in xs]
    taco_ref.decompress(enc[0][0], enc[0][1], n, block=block)
    total = taco_ref.decompress_sum([e[0] for e in enc], [e[1] for e in enc], n, block=block)
    return time.perf_counter() - t0, enc, total


def cpu_baseline(w, block, rows, gpu=None):
    """The oracle, as it stands, on the first `rows` tokens of every payload, same call mix as a step.

    With `gpu` = (payloads, scales, params, taco module) of the split layout and rows = all tokens, what the oracle
    computed anyway is also compared with the GPU's results, over the whole benchmark tensors: every code and scale of
    every payload, and decompress_sum of the ORACLE's payloads on the GPU against the oracle's own sum."""
    import numpy as np
    from oracle import taco_ref
    dt, enc, total = oracle_step(w, block, rows)
    n = rows * w.hidden
    k = w.payloads
    bf16_bytes = (k + 1 + k) * 2 * n
    base = {"value": bf16_bytes / dt / 1e9, "unit": "GB/s", "cores": taco_ref.threads(), "kind": "oracle",
            "sample": f"first {rows} of {w.tokens} tokens of each of the {k} payloads, same call mix as one step "
                      f"({dt:.1f} s)"}
    if gpu is None or rows != w.tokens:
        return base, None
    import torch
    payloads, scales, params, taco = gpu

    def rank(c):                       # E4M3 codes in sign-magnitude order, +0 and -0 merged
        mag = (c & 0x7F).astype(np.int16)
        return np.where(c & 0x80, -mag, mag)

    off_one = off_more = 0
    worst = [0.0, 0.0]
    for i in range(k):
        d = np.abs(rank(payloads[i].cpu().numpy()) - rank(enc[i][0]))
        off_one += int((d == 1).sum())
        off_more += int((d > 1).sum())
        g, r = scales[i].cpu().numpy().astype(np.float64), enc[i][1].astype(np.float64)
        for c in range(2):
            nz = r[:, c] != 0
            worst[c] = max(worst[c], float(np.max(np.abs(g[nz, c] - r[nz, c]) / np.abs(r[nz, c]))))
    dev = payloads[0].device
    out = taco.taco_decompress_sum([torch.from_numpy(e[0]).to(dev) for e in enc], [torch.from_numpy(e[1]).to(dev) for e in enc],
                                   (rows, w.hidden), params)
    torch.cuda.synchronize()
    got = out.view(torch.int16).cpu().numpy().view(np.uint16).reshape(-1)
    f = lambda b: (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    ref = f(total)
    err = np.abs(f(got) - ref)
    # the parity rule of the tests: per element at most max(one bf16 ulp of the oracle's value, 1e-3 of its block's maximum)
    mag = np.abs(ref)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(mag, 2.0 ** -126))) - 7)
    block_max = np.repeat(mag.reshape(-1, block).max(axis=1), block)
    worst_tol = float(np.max(err / np.maximum(ulp, 1e-3 * block_max + 1e-300)))
    parity = {"scope": f"all {k} x {n} elements of the benchmark tensors, GPU against the CPU oracle",
              "codes_identical": 1.0 - (off_one + off_more) / (k * n), "codes_one_step_apart": off_one,
              "codes_further_apart": off_more, "alpha_max_rel_err": worst[0], "s_max_rel_err": worst[1],
              f"decompress_sum_k{k}_outputs_identical": float((got == total).mean()),
              f"decompress_sum_k{k}_max_err_over_tolerance": worst_tol,
              "tolerance": "per element max(1 bf16 ulp of the oracle's value, 1e-3 of the block's max)"}
    return base, parity


def cpu_baseline_one_thread(w, block, rows):
    from oracle import taco_ref
    before = taco_ref.threads()
    taco_ref.set_threads(1)
    try:
        dt, _, _ = oracle_step(w, block, rows)
    finally:
        taco_ref.set_threads(before)
    k, n = w.payloads, rows * w.hidden
    return {"value": (k + 1 + k) * 2 * n / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"first {rows} of {w.tokens} tokens of each of the {k} payloads, same call mix as one step ({dt:.1f} s)"}


class Bench:
    """Buffers and calls of one workload under one parameter set."""

    def __init__(self, args, name, params, taco, torch, W, rotate=0, chunk_mb=0.0, streams=1, graph=False, batch=False):
        import numpy as np
        self.taco, self.torch = taco, torch
        self.w = w = W.WORKLOADS[name]
        self.params, self.B = params, params.block
        self.k, self.n = (args.payloads or w.payloads), w.numel
        k, n, B = self.k, self.n, self.B
        dev = torch.device("cuda:0")
        self.interleaved = params.layout == taco.TACO_LAYOUT_INTERLEAVED
        host = np.empty((w.tokens, w.hidden), dtype=np.uint16)
        xs = []
        for i in range(k):
            W.generate(w, i % w.payloads, threads=args.gen_threads, out=host)    # --payloads beyond the workload's own repeat them
            xs.append(torch.from_numpy(host.view(np.int16)).to(dev).view(torch.bfloat16))
        del host
        if self.interleaved:
            payloads = [torch.empty(taco.taco_payload_bytes(n, B) + taco.taco_scales_bytes(n, B), dtype=torch.uint8, device=dev)
                        for _ in range(k)]
            scales = [None] * k
        else:
            payloads = [torch.empty(taco.taco_payload_bytes(n, B), dtype=torch.uint8, device=dev) for _ in range(k)]
            scales = [torch.empty((taco.taco_scales_bytes(n, B) // 8, 2), dtype=torch.float32, device=dev) for _ in range(k)]
        out1 = torch.empty((w.tokens, w.hidden), dtype=torch.bfloat16, device=dev)
        outk = torch.empty((w.tokens, w.hidden), dtype=torch.bfloat16, device=dev)
        # Buffer sets: copies of everything a step touches; step j works on set j mod R.
        set_bytes = sum(t.numel() * t.element_size() for t in xs + payloads + [t for t in scales if t is not None] + [out1, outk])
        self.n_sets = rotate if rotate > 0 else max(1, min(64, -(-(1 << 30) // set_bytes)))
        if graph:
            self.n_sets = 1                 # a captured graph replays on the buffers it was captured with
        self.sets = [(xs, payloads, scales, out1, outk)]
        for _ in range(self.n_sets - 1):
            self.sets.append(tuple([t.clone() if t is not None else None for t in group] if isinstance(group, list) else group.clone()
                                   for group in self.sets[0]))
        self.cur = self.sets[0]
        self.step_no = 0
        self.stream = torch.cuda.current_stream()
        # Row chunks (whole rows, so every chunk is a whole number of blocks and tiles when hidden is a multiple of
        # 2048) dealt to `streams` streams in turn; each call joins them back into `stream`.
        self.rows_per_chunk = w.tokens
        if chunk_mb > 0:
            self.rows_per_chunk = max(1, min(w.tokens, int(chunk_mb * (1 << 20)) // (2 * w.hidden)))
            assert (self.rows_per_chunk * w.hidden) % 2048 == 0, "chunks must be whole tiles"
        self.bounds = [(r, min(r + self.rows_per_chunk, w.tokens)) for r in range(0, w.tokens, self.rows_per_chunk)]
        self.side = [torch.cuda.Stream() for _ in range(streams)] if chunk_mb > 0 and streams > 1 and not batch else []
        self.batch = batch
        self.rec = (B + 8) if self.interleaved else B       # payload bytes per block
        self.bpr = w.hidden // B                            # blocks per row
        self.parts = [self.part_compress, self.part_decompress, self.part_sum]
        if graph:
            for part in self.parts:
                part()                      # first launches (module load) outside the capture
            torch.cuda.synchronize()
            graphs = []
            for part in self.parts:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    self.stream = torch.cuda.current_stream()        # the capturing stream: chunked() forks from and joins it
                    part()
                graphs.append(g)
            self.stream = torch.cuda.current_stream()
            self.parts = [g.replay for g in graphs]

    # ---- the three parts of a step --------------------------------------------------------------
    @staticmethod
    def rows_of(t, r0, r1, per_row):
        return None if t is None else t[r0 * per_row:r1 * per_row]

    def chunked(self, fn):
        """fn(r0, r1, stream) for every chunk; whole-tensor calls go straight to the stream."""
        if len(self.bounds) == 1:
            fn(0, self.w.tokens, self.stream)
            return
        for s_ in self.side:
            s_.wait_stream(self.stream)
        for c, (r0, r1) in enumerate(self.bounds):
            fn(r0, r1, self.side[c % len(self.side)] if self.side else self.stream)
        for s_ in self.side:
            self.stream.wait_stream(s_)

    def part_compress(self):
        xs, payloads, scales, _, _ = self.cur
        taco, rows_of, bpr, rec = self.taco, self.rows_of, self.bpr, self.rec
        if self.batch:
            # every chunk of every tensor in launches of at most TACO_MAX_BATCH items
            items = [(i, r0, r1) for i in range(self.k) for (r0, r1) in self.bounds]
            for a in range(0, len(items), taco.TACO_MAX_BATCH):
                part = items[a:a + taco.TACO_MAX_BATCH]
                taco.taco_compress_batch([xs[i][r0:r1] for i, r0, r1 in part], self.params,
                                         [rows_of(payloads[i], r0, r1, bpr * rec) for i, r0, r1 in part],
                                         [rows_of(scales[i], r0, r1, bpr) for i, r0, r1 in part], self.stream)
            return
        for i in range(self.k):
            self.chunked(lambda r0, r1, st, i=i: taco.taco_compress(xs[i][r0:r1], self.params, rows_of(payloads[i], r0, r1, bpr * rec),
                                                                    rows_of(scales[i], r0, r1, bpr), st))

    def decode(self, srcs_p, srcs_s, out):
        taco, rows_of, bpr, rec = self.taco, self.rows_of, self.bpr, self.rec
        if self.batch and len(self.bounds) > 1:
            kk = len(srcs_p)
            per = max(1, min(taco.TACO_MAX_BATCH, taco.TACO_MAX_BATCH_PAYLOADS // kk))
            for a in range(0, len(self.bounds), per):
                part = self.bounds[a:a + per]
                taco.taco_decompress_sum_batch([[rows_of(t, r0, r1, bpr * rec) for t in srcs_p] for r0, r1 in part],
                                               [[rows_of(t, r0, r1, bpr) for t in srcs_s] for r0, r1 in part],
                                               [out[r0:r1].shape for r0, r1 in part], self.params,
                                               [out[r0:r1] for r0, r1 in part], self.stream)
            return
        self.chunked(lambda r0, r1, st: taco.taco_decompress_sum([rows_of(t, r0, r1, bpr * rec) for t in srcs_p],
                                                                 [rows_of(t, r0, r1, bpr) for t in srcs_s],
                                                                 out[r0:r1].shape, self.params, out[r0:r1], st))

    def part_decompress(self):
        _, payloads, scales, out1, _ = self.cur
        self.decode(payloads[:1], scales[:1], out1)

    def part_sum(self):
        _, payloads, scales, _, outk = self.cur
        self.decode(payloads, scales, outk)

    def step(self, ev=None, split="all"):
        """ev: four events.  split = "all": recorded around each of the three parts.  split = 0, 1 or 2: only ev[0] at the
        start of the step and ev[1] after part `split` (compress group, decompress, decompress_sum)."""
        self.cur = self.sets[self.step_no % self.n_sets]
        self.step_no += 1
        for j, part in enumerate(self.parts):
            if ev and (split == "all" or j == 0):
                ev[j].record(self.stream)
            part()
            if ev and split == j:
                ev[1].record(self.stream)
        if ev and split == "all":
            ev[3].record(self.stream)

    # ---- measurements -------------------------------------------------------------------------
    def bytes_of(self):
        per_elem = 1.0 + 8.0 / self.B                    # payload bytes per element: code + two fp32 per block
        n, k = self.n, self.k
        return {"compress": (2.0 + per_elem) * n, "decompress": (per_elem + 2.0) * n, "sum": (k * per_elem + 2.0) * n,
                "fused": (k + 1) * per_elem * n}

    def settle(self, ms):
        """Untimed steps for about `ms` milliseconds of GPU time: lets the clocks settle."""
        if ms <= 0:
            return
        torch = self.torch
        t0 = time.perf_counter()
        while (time.perf_counter() - t0) * 1e3 < ms:
            for _ in range(8):
                self.step()
            torch.cuda.synchronize()

    def timed_steps(self, steps, warmup, split="rotate"):
        """Wall time of `steps` steps and the HIP-event times of their calls, [compress per launch, decompress, decompress_sum],
        one list each.

        A launch that follows an event record waits about 6 us for the event's marker packet (the kernel trace shows the idle
        gap), so events BETWEEN the calls of a step stretch the step and the calls behind them.  split = "rotate" therefore
        records two events per step only: one at its start and one after the compress group, after decompress or after
        decompress_sum, in turn over the steps; the times of the two decode calls are the differences of the medians of those
        intervals (first the compress group alone, then with decompress, then with both), with no marker between the kernels
        they cover.  split = "all" records events around every call of every step (the times then contain the gaps)."""
        torch, statistics_median = self.torch, statistics.median
        for _ in range(warmup):
            self.step()
        if steps < 6:
            split = "all"
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            self.step(events[s], split if split == "all" else s % 3)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        if split == "all":
            per = [[e[j].elapsed_time(e[j + 1]) for e in events] for j in range(3)]
            per[0] = [v / self.k for v in per[0]]        # per compress launch
            return wall, per
        upto = [[e[0].elapsed_time(e[1]) for s, e in enumerate(events) if s % 3 == j] for j in range(3)]
        m = [statistics_median(v) for v in upto]
        per = [[v / self.k for v in upto[0]], [m[1] - m[0]], [m[2] - m[1]]]
        return wall, per

    def back_to_back(self, fn, alg_bytes):
        """16 launches in a row (after 3 untimed), launch r on buffer set r mod R: no events or other kernels between."""
        torch = self.torch
        yev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        for r in range(3):
            fn(r, self.sets[r % self.n_sets])
        yev[0].record(self.stream)
        for r in range(16):
            fn(r, self.sets[r % self.n_sets])
        yev[1].record(self.stream)
        torch.cuda.synchronize()
        ms = yev[0].elapsed_time(yev[1]) / 16
        return {"ms": round(ms, 4), "moved_GBps": round(alg_bytes / ms / 1e6, 1),
                "hbm_frac": round(alg_bytes / ms / 1e6 / HBM_PEAK_GBPS, 4)}

    def back_to_back_calls(self):
        taco, p, k, st = self.taco, self.params, self.k, self.stream
        by = self.bytes_of()
        return {"compress": self.back_to_back(lambda r, S: taco.taco_compress(S[0][r % k], p, S[1][r % k], S[2][r % k], st), by["compress"]),
                # source payload r mod k, so that a launch does not find its input in the last-level cache
                "decompress": self.back_to_back(lambda r, S: taco.taco_decompress(S[1][r % k], S[2][r % k], S[3].shape, p, S[3], st),
                                                by["decompress"]),
                f"decompress_sum_k{k}": self.back_to_back(lambda r, S: taco.taco_decompress_sum(S[1], S[2], S[4].shape, p, S[4], st),
                                                          by["sum"])}

    def batched_calls(self):
        """The same calls through the batched entry points: ONE launch covers the tensors of up to 32 buffer sets (one ramp-up
        and one drain for all of them); the time is per tensor."""
        taco, p, k, st, torch = self.taco, self.params, self.k, self.stream, self.torch
        by = self.bytes_of()
        sets = self.sets[:max(1, min(self.n_sets, taco.TACO_MAX_BATCH // k, taco.TACO_MAX_BATCH_PAYLOADS // k))]
        R = len(sets)
        if R == 1 and k == 1:
            return {}

        def run(fn, count, alg_bytes):
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            for _ in range(2):
                fn()
            ev[0].record(st)
            for _ in range(8):
                fn()
            ev[1].record(st)
            torch.cuda.synchronize()
            ms = ev[0].elapsed_time(ev[1]) / 8 / count
            return {"tensors_per_launch": count, "ms": round(ms, 4), "moved_GBps": round(alg_bytes / ms / 1e6, 1),
                    "hbm_frac": round(alg_bytes / ms / 1e6 / HBM_PEAK_GBPS, 4)}

        xs = [x for S in sets for x in S[0]]
        pl = [x for S in sets for x in S[1]]
        sc = [x for S in sets for x in S[2]]
        out = {"compress": run(lambda: taco.taco_compress_batch(xs, p, pl, sc, st), len(xs), by["compress"])}
        if R > 1:
            out["decompress"] = run(lambda: taco.taco_decompress_sum_batch([[S[1][0]] for S in sets], [[S[2][0]] for S in sets],
                                                                          [S[3].shape for S in sets], p, [S[3] for S in sets], st),
                                    R, by["decompress"])
            out[f"decompress_sum_k{k}"] = run(lambda: taco.taco_decompress_sum_batch([S[1] for S in sets], [S[2] for S in sets],
                                                                                   [S[4].shape for S in sets], p, [S[4] for S in sets], st),
                                              R, by["sum"])
        return out

    def yardsticks(self):
        """Memory-only kernels with the traffic of each call (set layout: xs, payloads, scales, out1, outk; the bf16
        buffers serve as sources and sinks of the right sizes)."""
        taco, k, B, st = self.taco, self.k, self.B, self.stream
        chunks = (2048 + 8 * (2048 // B)) // 16           # 16-byte words of one tile's payload
        n_tiles = self.n // 2048
        if n_tiles == 0:
            return {}
        per = (1.0 + 8.0 / B) * n_tiles * 2048
        raw = 2.0 * n_tiles * 2048
        return {"compress": self.back_to_back(lambda r, S: taco.taco_debug_traffic([S[0][r % k]], 256, S[4], chunks, n_tiles, st), raw + per),
                "decompress": self.back_to_back(lambda r, S: taco.taco_debug_traffic([S[0][r % k]], chunks, S[3], 256, n_tiles, st), raw + per),
                f"decompress_sum_k{k}": self.back_to_back(lambda r, S: taco.taco_debug_traffic(S[0], chunks, S[3], 256, n_tiles, st),
                                                          k * per + raw),
                f"decompress_sum_compress_k{k}": self.back_to_back(lambda r, S: taco.taco_debug_traffic(S[0], chunks, S[3], chunks, n_tiles, st),
                                                                   (k + 1) * per)}

    def same_payload_calls(self):
        """decompress_sum and the fused call with payload 0 given k times: the reads then come from cache (an eighth of
        the HBM read traffic), so the time left is what the kernel needs for everything but HBM."""
        taco, p, k, st = self.taco, self.params, self.k, self.stream
        by = self.bytes_of()
        fp = self.torch.empty_like(self.sets[0][1][0])
        fs = self.torch.empty_like(self.sets[0][2][0]) if self.sets[0][2][0] is not None else None
        out = {f"decompress_sum_k{k}": self.back_to_back(lambda r, S: taco.taco_decompress_sum([S[1][0]] * k, [S[2][0]] * k, S[4].shape, p, S[4], st),
                                                           by["sum"]),
               f"decompress_sum_compress_k{k}": self.back_to_back(
                   lambda r, S: taco.taco_decompress_sum_compress([S[1][0]] * k, [S[2][0]] * k, S[4].shape, p, fp, fs, st), by["fused"])}
        for e in out.values():
            del e["moved_GBps"], e["hbm_frac"]           # the bytes do not cross HBM: only the time means something
        return out

    def fused_call(self):
        taco, torch, st = self.taco, self.torch, self.stream
        xs, payloads, scales, out1, outk = self.sets[0]
        fev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        fp = torch.empty_like(payloads[0])
        fs = torch.empty_like(scales[0]) if scales[0] is not None else None
        for _ in range(3):
            taco.taco_decompress_sum_compress(payloads, scales, outk.shape, self.params, fp, fs, st)
        fev[0].record(st)
        for _ in range(10):
            taco.taco_decompress_sum_compress(payloads, scales, outk.shape, self.params, fp, fs, st)
        fev[1].record(st)
        torch.cuda.synchronize()
        return fev[0].elapsed_time(fev[1]) / 10


def call_entry(ms, alg_bytes, bf16_bytes):
    return {"ms": round(ms, 4), "moved_GBps": round(alg_bytes / ms / 1e6, 1),
            "bf16_GBps": round(bf16_bytes / ms / 1e6, 1), "hbm_frac": round(alg_bytes / ms / 1e6 / HBM_PEAK_GBPS, 4)}


def workload_entry(b, steps, warmup, settle_ms):
    """In-step medians and back-to-back times of one workload (k compress + 1 decompress + 1 decompress_sum(k))."""
    b.settle(settle_ms)
    wall, per = b.timed_steps(steps, warmup)
    by, k, n = b.bytes_of(), b.k, b.n
    med = [statistics.median(v) for v in per]
    moved = k * by["compress"] + by["decompress"] + by["sum"]
    ms_step = wall * 1e3 / steps
    return {"shape": [b.w.tokens, b.w.hidden], "payloads": k, "buffer_sets": b.n_sets,
            "ms_per_step": round(ms_step, 4), "hbm_frac_step": round(moved / (ms_step * 1e6) / HBM_PEAK_GBPS, 4),
            "in_step_median": {"compress": call_entry(med[0], by["compress"], 2.0 * n),
                               "decompress": call_entry(med[1], by["decompress"], 2.0 * n),
                               f"decompress_sum_k{k}": call_entry(med[2], by["sum"], k * 2.0 * n)},
            "back_to_back": b.back_to_back_calls(), "batched": b.batched_calls()}


def cold_trace(args, taco, torch, W, params):
    """Per-step call times from a cold start: nothing is launched before the first traced step."""
    b = Bench(args, args.workload, params, taco, torch, W, rotate=args.rotate)
    torch.cuda.synchronize()
    _, per = b.timed_steps(args.cold_trace, 0, split="all")
    print(json.dumps({"cold_trace_us": {"workload": b.w.name, "block": b.B,
                                        "compress": [round(v * 1e3, 1) for v in per[0]],
                                        "decompress": [round(v * 1e3, 1) for v in per[1]],
                                        f"decompress_sum_k{b.k}": [round(v * 1e3, 1) for v in per[2]]}}))


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the operator is block-local, so it shards on any block "
              "boundary without an exchange, and nothing here uses a second device); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2604_24088_amd import taco
    from paper_2604_24088_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    from paper_2604_24088_amd import build as hip_build
    hip_build.ensure_built()   # the library that matches the sources on disk (built if missing or stale)
    taco.lib()                 # fails loudly if the HIP library cannot be loaded
    B = args.block
    impl = {"auto": taco.TACO_IMPL_AUTO, "butterfly": taco.TACO_IMPL_BUTTERFLY, "mfma": taco.TACO_IMPL_MFMA}[args.impl]
    layout = taco.TACO_LAYOUT_INTERLEAVED if args.layout == "interleaved" else taco.TACO_LAYOUT_SPLIT
    fmt = {"e4m3": taco.TACO_FORMAT_E4M3, "e5m2": taco.TACO_FORMAT_E5M2, "int8": taco.TACO_FORMAT_INT8}[args.format]
    params = taco.taco_default_params(block=B, impl=impl, layout=layout, mode=args.mode, fmt=fmt)
    variant = args.mode != taco.TACO_MODE_FULL or fmt != taco.TACO_FORMAT_E4M3
    on_mfma = args.impl != "butterfly" and args.mode in (6, 7)

    if args.payloads:
        if not 1 <= args.payloads <= taco.TACO_MAX_K:
            sys.exit(f"--payloads must be between 1 and {taco.TACO_MAX_K}")
        args.no_cpu_baseline = args.no_workloads = True
    if args.cold_trace > 0:
        cold_trace(args, taco, torch, W, params)
        return

    b = Bench(args, args.workload, params, taco, torch, W, rotate=args.rotate, chunk_mb=args.chunk_mb, streams=args.streams,
              graph=args.graph, batch=args.batch)
    w, k, n = b.w, b.k, b.n
    b.settle(args.settle_ms)
    wall, per = b.timed_steps(args.steps, args.warmup)                          # THE timed region (two events per step)
    wall_split, per_marked = b.timed_steps(args.steps, 0, split="all")           # the same steps again with events between all calls

    # ---- yardstick outside the timed region: plain copy of 1 GiB (reads 1 GiB, writes 1 GiB)
    xs = b.sets[0][0]
    stream = b.stream
    src = xs[0].view(torch.uint8)[: 1 << 30] if xs[0].numel() * 2 >= (1 << 30) else xs[0].view(torch.uint8)
    dst = torch.empty_like(src)
    cev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for _ in range(2):
        taco.taco_debug_copy(src, dst, stream)
    cev[0].record(stream)
    for _ in range(10):
        taco.taco_debug_copy(src, dst, stream)
    cev[1].record(stream)
    torch.cuda.synchronize()
    copy_gbps = 2.0 * src.numel() * 10 / (cev[0].elapsed_time(cev[1]) * 1e6)
    del dst

    mix = b.yardsticks()
    b2b = b.back_to_back_calls()
    t_fused = b.fused_call()
    same = b.same_payload_calls() if k > 1 and not args.no_cache_fed else {}

    ms_step = wall * 1e3 / args.steps
    t_comp_avg = sum(per[0]) / len(per[0])               # ms per compress launch, average over the timed region
    med_marked = [statistics.median(v) for v in per_marked]
    med = [statistics.median(v) for v in per]
    by = b.bytes_of()
    equiv = (k + 1 + k) * 2.0 * n                        # bf16-equivalent bytes per step
    real_bf16 = (k + 1 + 1) * 2.0 * n                    # bf16 bytes that cross HBM per step
    moved = k * by["compress"] + by["decompress"] + by["sum"]
    achieved = by["compress"] / t_comp_avg / 1e6
    il = args.layout == "interleaved"
    result = {
        "metric": "compress+decompress GB/s of bf16 input and % of HBM peak, 1×MI355X",
        "value": round(equiv / (ms_step * 1e6), 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "ms_per_step_with_events_between_calls": round(wall_split * 1e3 / args.steps, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "arithmetic": "bf16 and FP8 matrix-core operands (exact products), fp32 accumulation and block scalars",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: bf16 [{w.tokens}, {w.hidden}] x {k} payloads, block {B}, "
                               f"step = {k} compress + 1 decompress + 1 decompress_sum(k={k})",
                   "impl": args.impl, "block": B, "layout": args.layout,
                   "chunk_rows": b.rows_per_chunk if len(b.bounds) > 1 else None, "chunks_per_call": len(b.bounds),
                   "streams": max(len(b.side), 1), "hip_graph": bool(args.graph), "batched_calls": bool(args.batch),
                   "buffer_sets": b.n_sets, "format": args.format, "mode": args.mode, "settle_ms": args.settle_ms,
                   "library_build_id": taco.taco_build_id()},
        "value_out_basis": round(real_bf16 / (ms_step * 1e6), 1),
        "moved_GBps": round(moved / (ms_step * 1e6), 1),
        "hbm_frac_step": round(moved / (ms_step * 1e6) / HBM_PEAK_GBPS, 4),
        "copy_yardstick_GBps": round(copy_gbps, 1),
        "mix_yardstick": mix,
        "calls_back_to_back": b2b,
        "calls_same_payload_k_times": same,
        "calls": {"compress": call_entry(med[0], by["compress"], 2.0 * n),
                  "decompress": call_entry(med[1], by["decompress"], 2.0 * n),
                  f"decompress_sum_k{k}": call_entry(med[2], by["sum"], k * 2.0 * n),
                  f"decompress_sum_compress_k{k} (not in the step)": call_entry(t_fused, by["fused"], k * 2.0 * n)},
        "calls_with_events_between_calls": {"compress": call_entry(med_marked[0], by["compress"], 2.0 * n),
                                            "decompress": call_entry(med_marked[1], by["decompress"], 2.0 * n),
                                            f"decompress_sum_k{k}": call_entry(med_marked[2], by["sum"], k * 2.0 * n)},
        "roofline": {"kernel": (f"compress_mfma_kernel<{max(B // 128, 1)},{max(128 // B, 1)},{'true' if il else 'false'},"
                                f"{ {'e4m3': 0, 'e5m2': 1, 'int8': 2}[args.format] },{'false' if (args.mode & 6) == 6 else 'true'}>")
                     if on_mfma else f"compress_butterfly_kernel<{B}>",
                     "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, B, args.impl)) if not il and not variant else None,
                     "alg_bytes_per_launch": by["compress"], "avg_launch_ms": round(t_comp_avg, 4),
                     "mfma_busy_frac": MEASURED_MFMA_BUSY.get((w.name, B, args.impl)) if not il and not variant else None},
    }
    payloads0, scales0 = b.sets[0][1], b.sets[0][2]
    plain = not (variant or il or args.chunk_mb > 0 or args.graph or args.batch)
    if not args.no_workloads and plain:
        # the other benchmark configurations, each with its own buffers (freed before the next)
        table = {w.name: {"shape": [w.tokens, w.hidden], "payloads": k, "buffer_sets": b.n_sets, "ms_per_step": round(ms_step, 4),
                          "hbm_frac_step": result["hbm_frac_step"], "in_step_median": {kk: vv for kk, vv in result["calls"].items()
                                                                                      if "not in the step" not in kk},
                          "back_to_back": b2b, "batched": b.batched_calls()}}
        keep = (payloads0, scales0)
        del b, xs, src
        torch.cuda.empty_cache()
        for name in ("tiny", "gpt_rowpar", "qwen_act", "bwd_grad"):
            if name == w.name:
                continue
            other = Bench(args, name, params, taco, torch, W)
            table[name] = workload_entry(other, 30, 10, 20.0)
            del other
            torch.cuda.empty_cache()
        result["workloads"] = {name: table[name] for name in ("tiny", "gpt_rowpar", "qwen_act", "bwd_grad", "large_k8") if name in table}
        payloads0, scales0 = keep
    if not args.no_cpu_baseline and variant:
        print("bench.py: the CPU baseline is timed for the method itself (mode 7, E4M3) only; skipped", file=sys.stderr)
    if not args.no_cpu_baseline and not variant:
        gpu = (payloads0, scales0, params, taco) if (args.layout == "split" and impl != taco.TACO_IMPL_BUTTERFLY) else None
        result["cpu_baseline"], parity = cpu_baseline(w, B, rows=w.tokens, gpu=gpu)
        if parity is not None:
            result["parity_full_size"] = parity
        # one thread: 1/16 of the tokens, so that it takes about as long as the all-threads run on 16 cores
        result["cpu_baseline_1thread"] = cpu_baseline_one_thread(w, B, rows=max(64, w.tokens // 16))
    print(json.dumps(result))


if __name__ == "__main__":
    main()
