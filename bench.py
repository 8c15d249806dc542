#!/usr/bin/env python3
"""Throughput of the TACO fused FP8 compression operator on one MI355X.

One STEP is one pass of the whole hot path over one batch of synthetic input:
    k x taco_compress  ->  taco_decompress (payload 0)  ->  taco_decompress_sum (all k)
on the `large_k8` workload (bf16 [16384, 12288], k = 8 payloads, block 128): the largest
single-GPU configuration, and the one whose buffers (3 GiB of inputs) cannot sit in the
256 MB last-level cache.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` counts bf16-equivalent
bytes: 2N per compressed tensor, 2N per decompressed tensor, k*2N for decompress_sum
(k tensors decoded); `value_out_basis` counts only bf16 bytes that really cross HBM.
`calls` times each call inside the step (HIP events between the calls); `calls_back_to_back` times
16 launches of one call in a row, which is what a kernel costs when the host's launch time (6-9 us
per call through this binding) is not in the way: on the smaller workloads the two differ.
`mix_yardstick` times memory-only kernels (taco_debug_traffic) that move exactly the bytes of a
compress and of a decompress_sum call and compute nothing: what the memory system gives that mix.
The roofline object prices the dominant kernel (compress) by its ALGORITHMIC bytes
(3.0625 B per element at block 128) over its average launch duration, measured with
HIP events on the launch stream inside the timed region.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, vendor figure

# HBM traffic per launch of the dominant kernel measured with rocprofv3 --pmc (FETCH_SIZE and
# WRITE_SIZE runs, scaled by a copy kernel of known size); None until measured.  The summary
# the number comes from is committed under profiles/.
MEASURED_TRAFFIC_BYTES = {
    # fetch 393250 KiB + write 208896 KiB per compress launch: profiles/mfma_kernels_large_k8.txt
    ("large_k8", 128, "auto"): 616597437,
}


# Share of time the matrix cores are busy in the dominant kernel (SQ_VALU_MFMA_BUSY_CYCLES over SIMD-cycles,
# rocprofv3 --pmc run summarised in the same profile); the Hadamard rotation is an MFMA contraction there.
MEASURED_MFMA_BUSY = {("large_k8", 128, "auto"): 0.203}


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
    ap.add_argument("--rotate", type=int, default=0,
                    help="buffer sets the steps rotate through (0 = as many as it takes, up to 64, for the sets to exceed "
                         "1 GiB together, so that workloads smaller than the 256 MB last-level cache are still timed from HBM)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the three parts of the step into HIP graphs and time their replays (takes the "
                         "host's launch cost out of chunked runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--gen-threads", type=int, default=16)
    return ap.parse_args()


def cpu_baseline(w, block, rows, gpu=None):
    """The oracle, as it stands, on the first `rows` tokens of every payload, same call mix as a step.

    With `gpu` = (payloads, scales, params, taco module) of the split layout and rows = all tokens, what the oracle
    computed anyway is also compared with the GPU's results, over the whole benchmark tensors: every code and scale of
    every payload, and decompress_sum of the ORACLE's payloads on the GPU against the oracle's own sum."""
    import numpy as np
    from oracle import taco_ref
    from paper_2604_24088_amd import workloads as W
    xs = [W.generate_rows(w, i, 0, rows) for i in range(w.payloads)]
    n = rows * w.hidden
    t0 = time.perf_counter()
    enc = [taco_ref.compress(x, block=block) for x in xs]
    taco_ref.decompress(enc[0][0], enc[0][1], n, block=block)
    total = taco_ref.decompress_sum([e[0] for e in enc], [e[1] for e in enc], n, block=block)
    dt = time.perf_counter() - t0
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


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the operator is block-local, so it shards on any block "
              "boundary without an exchange, and nothing here uses a second device); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2604_24088_amd import taco
    from paper_2604_24088_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    from paper_2604_24088_amd import build as hip_build
    hip_build.ensure_built()   # load what is built; build only if nothing is
    taco.lib()                 # fails loudly if the HIP library cannot be loaded
    dev = torch.device("cuda:0")
    w = W.WORKLOADS[args.workload]
    k, n, B = w.payloads, w.numel, args.block
    impl = {"auto": taco.TACO_IMPL_AUTO, "butterfly": taco.TACO_IMPL_BUTTERFLY, "mfma": taco.TACO_IMPL_MFMA}[args.impl]
    layout = taco.TACO_LAYOUT_INTERLEAVED if args.layout == "interleaved" else taco.TACO_LAYOUT_SPLIT
    fmt = {"e4m3": taco.TACO_FORMAT_E4M3, "e5m2": taco.TACO_FORMAT_E5M2, "int8": taco.TACO_FORMAT_INT8}[args.format]
    params = taco.taco_default_params(block=B, impl=impl, layout=layout, mode=args.mode, fmt=fmt)
    variant = args.mode != taco.TACO_MODE_FULL or fmt != taco.TACO_FORMAT_E4M3

    # ---- synthetic inputs, resident in HBM
    host = np.empty((w.tokens, w.hidden), dtype=np.uint16)
    xs = []
    for i in range(k):
        W.generate(w, i, threads=args.gen_threads, out=host)
        xs.append(torch.from_numpy(host.view(np.int16)).to(dev).view(torch.bfloat16))
    del host
    if args.layout == "interleaved":
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
    n_sets = args.rotate if args.rotate > 0 else max(1, min(64, -(-(1 << 30) // set_bytes)))
    if args.graph:
        n_sets = 1                      # a captured graph replays on the buffers it was captured with
    sets = [(xs, payloads, scales, out1, outk)]
    for _ in range(n_sets - 1):
        sets.append(tuple([t.clone() if t is not None else None for t in group] if isinstance(group, list) else group.clone()
                          for group in sets[0]))
    step_no = 0
    stream = torch.cuda.current_stream()

    # Row chunks (whole rows, so every chunk is a whole number of blocks and tiles when hidden is a multiple of
    # 2048) dealt to `--streams` streams in turn; each call joins them back into `stream`.
    rows_per_chunk = w.tokens
    if args.chunk_mb > 0:
        rows_per_chunk = max(1, min(w.tokens, int(args.chunk_mb * (1 << 20)) // (2 * w.hidden)))
        assert (rows_per_chunk * w.hidden) % 2048 == 0, "chunks must be whole tiles"
    bounds = [(r, min(r + rows_per_chunk, w.tokens)) for r in range(0, w.tokens, rows_per_chunk)]
    side = [torch.cuda.Stream() for _ in range(args.streams)] if args.chunk_mb > 0 and args.streams > 1 else []
    rec = (B + 8) if args.layout == "interleaved" else B       # payload bytes per block

    def rows_of(t, r0, r1, per_row):
        return None if t is None else t[r0 * per_row:r1 * per_row]

    def chunked(fn):
        """fn(r0, r1, stream) for every chunk; whole-tensor calls go straight to `stream`."""
        if len(bounds) == 1:
            fn(0, w.tokens, stream)
            return
        for s_ in side:
            s_.wait_stream(stream)
        for c, (r0, r1) in enumerate(bounds):
            fn(r0, r1, side[c % len(side)] if side else stream)
        for s_ in side:
            stream.wait_stream(s_)

    bpr = w.hidden // B                                          # blocks per row

    def compress_rows(i):
        return lambda r0, r1, st: taco.taco_compress(xs[i][r0:r1], params, rows_of(payloads[i], r0, r1, bpr * rec),
                                                     rows_of(scales[i], r0, r1, bpr), st)

    def decode_rows(srcs_p, srcs_s, out):
        return lambda r0, r1, st: taco.taco_decompress_sum([rows_of(t, r0, r1, bpr * rec) for t in srcs_p],
                                                           [rows_of(t, r0, r1, bpr) for t in srcs_s],
                                                           out[r0:r1].shape, params, out[r0:r1], st)

    def part_compress():
        for i in range(k):
            chunked(compress_rows(i))

    def part_decompress():
        chunked(decode_rows(payloads[:1], scales[:1], out1))

    def part_sum():
        chunked(decode_rows(payloads, scales, outk))

    parts = [part_compress, part_decompress, part_sum]
    if args.graph:
        for part in parts:
            part()                      # first launches (module load) outside the capture
        torch.cuda.synchronize()
        graphs = []
        for part in parts:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                stream = torch.cuda.current_stream()        # the capturing stream: chunked() forks from and joins it
                part()
            graphs.append(g)
        stream = torch.cuda.current_stream()
        parts = [g.replay for g in graphs]

    def step(ev=None):
        nonlocal xs, payloads, scales, out1, outk, step_no
        xs, payloads, scales, out1, outk = sets[step_no % n_sets]
        step_no += 1
        for j, part in enumerate(parts):
            if ev:
                ev[j].record(stream)
            part()
        if ev:
            ev[3].record(stream)

    for _ in range(args.warmup):
        step()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(events[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # ---- yardstick outside the timed region: plain copy of 1 GiB (reads 1 GiB, writes 1 GiB)
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

    # ---- yardsticks outside the timed region: memory-only kernels with the traffic of compress (reads one
    # bf16 tensor, writes one payload) and of decompress_sum (reads k payloads, writes one bf16 tensor)
    chunks = (2048 + 8 * (2048 // B)) // 16           # 16-byte words of one tile's payload
    n_tiles = n // 2048
    per_elem_y = 1.0 + 8.0 / B

    def back_to_back(fn, alg_bytes):
        """16 launches in a row (after 3 untimed), launch r on buffer set r mod R: no events or other kernels between."""
        yev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        for r in range(3):
            fn(r, sets[r % n_sets])
        yev[0].record(stream)
        for r in range(16):
            fn(r, sets[r % n_sets])
        yev[1].record(stream)
        torch.cuda.synchronize()
        ms = yev[0].elapsed_time(yev[1]) / 16
        return {"ms": round(ms, 4), "moved_GBps": round(alg_bytes / ms / 1e6, 1),
                "hbm_frac": round(alg_bytes / ms / 1e6 / HBM_PEAK_GBPS, 4)}

    mix, b2b = {}, {}
    if n_tiles > 0:
        # set layout: (xs, payloads, scales, out1, outk); the bf16 buffers serve as sources and sinks of the right sizes
        mix = {"compress": back_to_back(lambda r, S: taco.taco_debug_traffic([S[0][r % k]], 256, S[4], chunks, n_tiles, stream),
                                        (2.0 + per_elem_y) * n_tiles * 2048),
               f"decompress_sum_k{k}": back_to_back(lambda r, S: taco.taco_debug_traffic(S[0], chunks, S[3], 256, n_tiles, stream),
                                                    (k * per_elem_y + 2.0) * n_tiles * 2048)}
    b2b = {"compress": back_to_back(lambda r, S: taco.taco_compress(S[0][r % k], params, S[1][r % k], S[2][r % k], stream),
                                    (2.0 + per_elem_y) * n),
           "decompress": back_to_back(lambda r, S: taco.taco_decompress(S[1][0], S[2][0], S[3].shape, params, S[3], stream),
                                      (2.0 + per_elem_y) * n),
           f"decompress_sum_k{k}": back_to_back(lambda r, S: taco.taco_decompress_sum(S[1], S[2], S[4].shape, params, S[4], stream),
                                                (k * per_elem_y + 2.0) * n)}

    # ---- outside the timed region: the fused decompress_sum -> compress call (reduce-scatter receive
    # side feeding the all-gather send side) on the same payloads
    fev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    fp = torch.empty_like(payloads[0])
    fs = torch.empty_like(scales[0]) if scales[0] is not None else None
    for _ in range(3):
        taco.taco_decompress_sum_compress(payloads, scales, outk.shape, params, fp, fs, stream)
    fev[0].record(stream)
    for _ in range(10):
        taco.taco_decompress_sum_compress(payloads, scales, outk.shape, params, fp, fs, stream)
    fev[1].record(stream)
    torch.cuda.synchronize()
    t_fused = fev[0].elapsed_time(fev[1]) / 10
    del fp, fs

    ms_step = wall * 1e3 / args.steps
    t_comp = sum(e[0].elapsed_time(e[1]) for e in events) / (args.steps * k)   # ms per compress launch
    t_dec = sum(e[1].elapsed_time(e[2]) for e in events) / args.steps
    t_sum = sum(e[2].elapsed_time(e[3]) for e in events) / args.steps

    per_elem = 1.0 + 8.0 / B                         # payload bytes per element: code + two fp32 per block
    bytes_comp = (2.0 + per_elem) * n                # algorithmic bytes of one compress launch
    bytes_dec = (per_elem + 2.0) * n
    bytes_sum = (k * per_elem + 2.0) * n
    equiv = (k + 1 + k) * 2.0 * n                    # bf16-equivalent bytes per step
    real_bf16 = (k + 1 + 1) * 2.0 * n                # bf16 bytes that cross HBM per step
    moved = k * bytes_comp + bytes_dec + bytes_sum

    def call(ms, alg_bytes, bf16_bytes):
        return {"ms": round(ms, 4), "moved_GBps": round(alg_bytes / ms / 1e6, 1),
                "bf16_GBps": round(bf16_bytes / ms / 1e6, 1), "hbm_frac": round(alg_bytes / ms / 1e6 / HBM_PEAK_GBPS, 4)}

    achieved = bytes_comp / t_comp / 1e6
    result = {
        "metric": "compress+decompress GB/s of bf16 input and % of HBM peak, 1\u00d7MI355X",
        "value": round(equiv / (ms_step * 1e6), 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: bf16 [{w.tokens}, {w.hidden}] x {k} payloads, block {B}, "
                               f"step = {k} compress + 1 decompress + 1 decompress_sum(k={k})",
                   "impl": args.impl, "block": B, "layout": args.layout,
                   "chunk_rows": rows_per_chunk if len(bounds) > 1 else None, "chunks_per_call": len(bounds),
                   "streams": max(len(side), 1), "hip_graph": bool(args.graph),
                   "buffer_sets": n_sets, "format": args.format, "mode": args.mode},
        "value_out_basis": round(real_bf16 / (ms_step * 1e6), 1),
        "moved_GBps": round(moved / (ms_step * 1e6), 1),
        "hbm_frac_step": round(moved / (ms_step * 1e6) / HBM_PEAK_GBPS, 4),
        "copy_yardstick_GBps": round(copy_gbps, 1),
        "mix_yardstick": mix,
        "calls_back_to_back": b2b,
        "calls": {"compress": call(t_comp, bytes_comp, 2.0 * n),
                  "decompress": call(t_dec, bytes_dec, 2.0 * n),
                  f"decompress_sum_k{k}": call(t_sum, bytes_sum, k * 2.0 * n),
                  f"decompress_sum_compress_k{k} (not in the step)": call(t_fused, (k + 1) * per_elem * n, k * 2.0 * n)},
        "roofline": {"kernel": (f"compress_mfma_kernel<{max(B // 128, 1)},{max(128 // B, 1)},1,"
                                f"{'true' if args.layout == 'interleaved' else 'false'},{1 if args.format == 'e5m2' else 0}>")
                     if args.impl != "butterfly" and args.mode in (6, 7) and args.format != "int8"
                     else f"compress_butterfly_kernel<{B}>",
                     "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, B, args.impl)) if args.layout == "split" and not variant else None,
                     "alg_bytes_per_launch": bytes_comp, "avg_launch_ms": round(t_comp, 4),
                     "mfma_busy_frac": MEASURED_MFMA_BUSY.get((w.name, B, args.impl)) if args.layout == "split" and not variant else None},
    }
    if not args.no_cpu_baseline and variant:
        print("bench.py: the CPU baseline is timed for the method itself (mode 7, E4M3) only; skipped", file=sys.stderr)
    if not args.no_cpu_baseline and not variant:
        gpu = (sets[0][1], sets[0][2], params, taco) if (args.layout == "split" and impl != taco.TACO_IMPL_BUTTERFLY
                                                         and not variant) else None
        result["cpu_baseline"], parity = cpu_baseline(w, B, rows=w.tokens, gpu=gpu)
        if parity is not None:
            result["parity_full_size"] = parity
    print(json.dumps(result))


if __name__ == "__main__":
    main()
