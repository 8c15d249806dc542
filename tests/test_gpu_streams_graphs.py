"""The entry points under the launch mechanisms a training loop uses: a side stream, several streams at
once, and HIP graph capture with replays.  Each case must give bit for bit what the same calls give on
the default stream (the kernels are deterministic: no atomics, fixed summation order)."""
import numpy as np
import pytest
import torch

from paper_2604_24088_amd import taco
from paper_2604_24088_amd import workloads as W

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _inputs(k, rows=96, seed_base=0):
    w = W.WORKLOADS["gpt_rowpar"]
    xs = [torch.from_numpy(W.generate_rows(w, 0, (seed_base + i) * rows, rows).view(np.int16)).to(DEV).view(torch.bfloat16)
          for i in range(k)]
    return xs


def _step(xs, params, stream=None):
    enc = [taco.taco_compress(x, params, stream=stream) for x in xs]
    pls, scs = [e[0] for e in enc], [e[1] for e in enc]
    one = taco.taco_decompress(pls[0], scs[0], xs[0].shape, params, stream=stream)
    total = taco.taco_decompress_sum(pls, scs, xs[0].shape, params, stream=stream)
    fp, fs = taco.taco_decompress_sum_compress(pls, scs, xs[0].shape, params, stream=stream)
    return pls, scs, one, total, fp, fs


def _same(a, b):
    if a is None or b is None:
        return a is b
    if isinstance(a, (list, tuple)):
        return all(_same(x, y) for x, y in zip(a, b))
    return torch.equal(a.view(torch.uint8), b.view(torch.uint8))


@pytest.mark.parametrize("layout", [taco.TACO_LAYOUT_SPLIT, taco.TACO_LAYOUT_INTERLEAVED])
@pytest.mark.parametrize("block,k", [(128, 8), (256, 3), (32, 6)])
def test_side_stream_matches_default_stream(block, k, layout):
    xs = _inputs(k)
    p = taco.taco_default_params(block=block, layout=layout)
    ref = _step(xs, p)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):          # allocations and launches both on `side`
        got = _step(xs, p, stream=side)
    side.synchronize()
    assert _same(got, ref)


def test_two_streams_at_once():
    """Independent tensors compressed and decoded on two streams whose work overlaps in time."""
    p = taco.taco_default_params(block=128)
    xa, xb = _inputs(4, rows=512, seed_base=0), _inputs(4, rows=512, seed_base=4)
    ref_a, ref_b = _step(xa, p), _step(xb, p)
    torch.cuda.synchronize()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    for _ in range(3):
        with torch.cuda.stream(sa):
            got_a = _step(xa, p, stream=sa)
        with torch.cuda.stream(sb):
            got_b = _step(xb, p, stream=sb)
        sa.synchronize()
        sb.synchronize()
        assert _same(got_a, ref_a) and _same(got_b, ref_b)


@pytest.mark.parametrize("block,k,layout", [(128, 8, taco.TACO_LAYOUT_SPLIT), (256, 2, taco.TACO_LAYOUT_INTERLEAVED),
                                            (64, 6, taco.TACO_LAYOUT_SPLIT)])
def test_graph_capture_and_replay(block, k, layout):
    """One step captured into a HIP graph (every call enqueues kernels only: no allocation, no memset, no
    synchronisation), replayed with new inputs copied into the captured buffers and eager work in between."""
    p = taco.taco_default_params(block=block, layout=layout)
    xs = _inputs(k, rows=100)                      # 100 x 4096 elements: whole tiles only
    n = xs[0].numel()
    tail = torch.zeros(3 * 4096 + 77, dtype=torch.bfloat16, device=DEV)   # a second shape with a ragged tail
    il = layout == taco.TACO_LAYOUT_INTERLEAVED
    nbytes = taco.taco_payload_bytes(n, block) + (taco.taco_scales_bytes(n, block) if il else 0)
    pls = [torch.empty(nbytes, dtype=torch.uint8, device=DEV) for _ in range(k)]
    scs = [None if il else torch.empty((taco.taco_scales_bytes(n, block) // 8, 2), dtype=torch.float32, device=DEV)
           for _ in range(k)]
    total = torch.empty_like(xs[0])
    fp = torch.empty_like(pls[0])
    fs = None if il else torch.empty_like(scs[0])
    tb = taco.taco_payload_bytes(tail.numel(), block) + (taco.taco_scales_bytes(tail.numel(), block) if il else 0)
    tp = torch.empty(tb, dtype=torch.uint8, device=DEV)
    ts = None if il else torch.empty((taco.taco_scales_bytes(tail.numel(), block) // 8, 2), dtype=torch.float32, device=DEV)
    tout = torch.empty_like(tail)

    def enqueue(stream=None):
        for i in range(k):
            taco.taco_compress(xs[i], p, pls[i], scs[i], stream=stream)
        taco.taco_decompress_sum(pls, scs, total.shape, p, out=total, stream=stream)
        taco.taco_decompress_sum_compress(pls, scs, total.shape, p, fp, fs, stream=stream)
        taco.taco_compress(tail, p, tp, ts, stream=stream)          # matrix-core kernel + tail kernel
        taco.taco_decompress(tp, ts, tail.shape, p, out=tout, stream=stream)

    outs = lambda: [t.clone() for t in pls + [s for s in scs if s is not None] + [total, fp, tp, tout] +
                    ([fs, ts] if not il else [])]
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue()                                   # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    with torch.cuda.graph(graph):
        enqueue()                                   # the binding launches on the current (capturing) stream
    rng = np.random.default_rng(11)
    for rep in range(4):
        for x in xs:                                # new data in the captured input buffers
            x.copy_(torch.from_numpy(rng.standard_normal(x.shape).astype(np.float32)).to(DEV) * (0.01 * (rep + 1)))
        tail.copy_(torch.from_numpy(rng.standard_normal(tail.shape).astype(np.float32)).to(DEV))
        enqueue()
        torch.cuda.synchronize()
        want = outs()
        for t in pls + [total, fp, tp, tout]:
            t.fill_(0x55 if t.dtype == torch.uint8 else 1.0)       # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert _same(outs(), want), f"replay {rep} differs from the eager run"


def test_prepared_calls_match_direct_calls():
    """A PreparedCall launches the same kernels on the same buffers; new contents in the same buffers are picked up."""
    k = 6
    p = taco.taco_default_params(block=256)
    xs = _inputs(k, rows=64)
    ref = _step(xs, p)
    pls = [torch.empty_like(t) for t in ref[0]]
    scs = [torch.empty_like(t) for t in ref[1]]
    total, fp, fs = torch.empty_like(ref[3]), torch.empty_like(ref[4]), torch.empty_like(ref[5])
    plans = [taco.prepare_compress(xs[i], p, pls[i], scs[i]) for i in range(k)]
    plans += [taco.prepare_decompress_sum(pls, scs, xs[0].shape, p, total),
              taco.prepare_decompress_sum_compress(pls, scs, xs[0].shape, p, fp, fs)]
    for rep in range(2):
        for plan in plans:
            plan()
        torch.cuda.synchronize()
        assert _same((pls, scs, total, fp, fs), (ref[0], ref[1], ref[3], ref[4], ref[5]))
        for x in xs:                                    # new contents, same addresses
            x.mul_(0.5)
        ref = _step(xs, p)
        torch.cuda.synchronize()
    with pytest.raises(ValueError):
        taco.prepare_compress(xs[0], p, pls[0][:-1], scs[0])
