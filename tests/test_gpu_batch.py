"""The batched entry points: several tensors (or chunks of one tensor) in ONE kernel.  Results must be
bit-identical to the single calls, which the other GPU tests hold against the oracle; one case is also
compared with the oracle directly."""
import numpy as np
import pytest
import torch

from paper_2604_24088_amd import taco
from paper_2604_24088_amd import workloads as W

import parity_util as P

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def to_dev(bits: np.ndarray) -> torch.Tensor:
    """bf16 bits -> device tensor of exactly that many elements (storage padded to 16 bytes)."""
    n = bits.size
    padded = np.concatenate([bits.reshape(-1), np.zeros((-n) % 8, dtype=np.uint16)])
    return torch.from_numpy(padded.view(np.int16)).to(DEV).view(torch.bfloat16)[:n]


def make(n, seed, scale=0.02):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(n) * scale
    x[rng.integers(0, n, max(n // 300, 1))] *= 30.0
    return W.float32_to_bf16_bits(x.astype(np.float32))


SIZES = [2048 * 5, 1, 2048 * 3 + 700, 127, 2048, 2048 * 17 + 1, 300, 2048 * 2 + 2047]


@pytest.mark.parametrize("block,layout,impl,mode,fmt", [
    (128, 0, taco.TACO_IMPL_AUTO, 7, 0), (128, 1, taco.TACO_IMPL_AUTO, 7, 0), (256, 0, taco.TACO_IMPL_AUTO, 7, 0),
    (32, 1, taco.TACO_IMPL_AUTO, 7, 0), (512, 0, taco.TACO_IMPL_AUTO, 6, 1), (64, 0, taco.TACO_IMPL_AUTO, 7, 2),
    (128, 0, taco.TACO_IMPL_BUTTERFLY, 7, 0), (256, 1, taco.TACO_IMPL_BUTTERFLY, 7, 0), (128, 0, taco.TACO_IMPL_AUTO, 4, 0)])
def test_compress_batch_equals_single_calls(oracle, block, layout, impl, mode, fmt):
    p = taco.taco_default_params(block=block, layout=layout, impl=impl, mode=mode, fmt=fmt)
    xs = [make(n, 100 + i) for i, n in enumerate(SIZES)]
    dx = [to_dev(x) for x in xs]
    bp, bs = taco.taco_compress_batch(dx, p)
    torch.cuda.synchronize()
    for i, x in enumerate(dx):
        sp, ss = taco.taco_compress(x, p)
        torch.cuda.synchronize()
        assert torch.equal(bp[i], sp), (i, SIZES[i])
        assert layout == 1 or torch.equal(bs[i], ss), (i, SIZES[i])
    # and one tensor of the batch against the oracle itself
    i = 5
    rp, rs, z = oracle.compress(xs[i], block=block, mode=mode, fmt=fmt, want_z=True)
    gp, gs = P.deinterleave(bp[i].cpu().numpy(), block) if layout else (bp[i].cpu().numpy(), bs[i].cpu().numpy())
    P.check_scales(gs, rs, "batch")
    P.check_codes(gp, rp, rs, block, "batch", fmt=fmt, z=z,
                  min_match=P.CODE_MATCH_MIN if mode & 2 else P.CODE_MATCH_MIN_UNROTATED)


def test_compress_batch_of_the_maximum_number_of_tensors():
    p = taco.taco_default_params()
    dx = [to_dev(make(2048 * (1 + i % 3) + 13 * i, 7 + i)) for i in range(taco.TACO_MAX_BATCH)]
    bp, bs = taco.taco_compress_batch(dx, p)
    torch.cuda.synchronize()
    for i, x in enumerate(dx):
        sp, ss = taco.taco_compress(x, p)
        torch.cuda.synchronize()
        assert torch.equal(bp[i], sp) and torch.equal(bs[i], ss), i
    with pytest.raises(ValueError, match="between 1 and 32"):
        taco.taco_compress_batch(dx + dx[:1], p)


@pytest.mark.parametrize("block,layout,impl,k,mode,fmt", [
    (128, 0, taco.TACO_IMPL_AUTO, 1, 7, 0), (128, 0, taco.TACO_IMPL_AUTO, 8, 7, 0), (128, 1, taco.TACO_IMPL_AUTO, 3, 7, 0),
    (256, 0, taco.TACO_IMPL_AUTO, 6, 7, 0), (32, 1, taco.TACO_IMPL_AUTO, 2, 7, 0), (512, 0, taco.TACO_IMPL_AUTO, 16, 7, 0),
    (64, 0, taco.TACO_IMPL_AUTO, 3, 7, 2), (128, 0, taco.TACO_IMPL_BUTTERFLY, 5, 7, 0), (128, 1, taco.TACO_IMPL_AUTO, 2, 4, 0)])
def test_decompress_sum_batch_equals_single_calls(oracle, block, layout, impl, k, mode, fmt):
    p = taco.taco_default_params(block=block, layout=layout, impl=impl, mode=mode, fmt=fmt)
    sizes = SIZES[:taco.TACO_MAX_BATCH_PAYLOADS // k][:6]
    payloads, scales, shapes, encs = [], [], [], []
    for t, n in enumerate(sizes):
        enc = [oracle.compress(make(n, 1000 * t + i, 0.02 * (i + 1)), block=block, mode=mode, fmt=fmt) for i in range(k)]
        encs.append(enc)
        if layout:
            payloads.append([torch.from_numpy(P.interleave(e[0], e[1], block)).to(DEV) for e in enc])
            scales.append(None)
        else:
            payloads.append([torch.from_numpy(e[0]).to(DEV) for e in enc])
            scales.append([torch.from_numpy(e[1]).to(DEV) for e in enc])
        shapes.append((n,))
    guards = [torch.zeros(n + ((-n) % 8) + 16, dtype=torch.bfloat16, device=DEV) for n in sizes]
    outs = taco.taco_decompress_sum_batch(payloads, scales, shapes, p, outs=[g[:n] for g, n in zip(guards, sizes)])
    torch.cuda.synchronize()
    for t, n in enumerate(sizes):
        single = taco.taco_decompress_sum(payloads[t], scales[t], (n,), p)
        torch.cuda.synchronize()
        assert torch.equal(outs[t], single), (t, n)
        assert torch.all(guards[t][n:] == 0), (t, n)              # nothing written past the tensor's end
    t = len(sizes) - 1
    ref, acc = oracle.decompress_sum([e[0] for e in encs[t]], [e[1] for e in encs[t]], sizes[t], block=block, mode=mode, fmt=fmt,
                                     want_sum=True)
    P.check_recon(outs[t].view(torch.int16).cpu().numpy().view(np.uint16), ref, block, "batch decode", min_exact=P.RECON_EXACT_MIN_SMALL, acc=acc)


@pytest.mark.parametrize("block,layout,impl,k,mode,fmt", [
    (128, 0, taco.TACO_IMPL_AUTO, 8, 7, 0), (128, 1, taco.TACO_IMPL_AUTO, 4, 7, 0), (256, 0, taco.TACO_IMPL_AUTO, 2, 7, 0),
    (32, 0, taco.TACO_IMPL_AUTO, 8, 7, 0), (512, 1, taco.TACO_IMPL_AUTO, 3, 7, 0), (64, 0, taco.TACO_IMPL_AUTO, 5, 7, 2),
    (128, 0, taco.TACO_IMPL_BUTTERFLY, 2, 7, 0), (128, 0, taco.TACO_IMPL_AUTO, 1, 6, 1)])
def test_fused_batch_equals_single_calls(oracle, block, layout, impl, k, mode, fmt):
    """taco_decompress_sum_compress_batch: every tensor's output is bit for bit that of the single fused call (which the
    parity tests hold against the oracle and against the two separate calls)."""
    p = taco.taco_default_params(block=block, layout=layout, impl=impl, mode=mode, fmt=fmt)
    sizes = SIZES[:taco.TACO_MAX_BATCH_PAYLOADS // k][:6]
    payloads, scales, shapes = [], [], []
    for t, n in enumerate(sizes):
        enc = [oracle.compress(make(n, 2000 * t + i, 0.02 * (i + 1)), block=block, mode=mode, fmt=fmt) for i in range(k)]
        if layout:
            payloads.append([torch.from_numpy(P.interleave(e[0], e[1], block)).to(DEV) for e in enc])
            scales.append(None)
        else:
            payloads.append([torch.from_numpy(e[0]).to(DEV) for e in enc])
            scales.append([torch.from_numpy(e[1]).to(DEV) for e in enc])
        shapes.append((n,))
    bp, bs = taco.taco_decompress_sum_compress_batch(payloads, scales, shapes, p)
    torch.cuda.synchronize()
    for t, n in enumerate(sizes):
        sp, ss = taco.taco_decompress_sum_compress(payloads[t], scales[t], (n,), p)
        torch.cuda.synchronize()
        assert torch.equal(bp[t], sp), (t, n)
        assert layout or torch.equal(bs[t], ss), (t, n)


def test_chunks_of_one_tensor_as_a_batch():
    """Row chunks of a tensor (the overlap granularity of Section 4.4.2) as the items of one batched call: the same
    bits as the whole-tensor call, written into the same buffers."""
    w = W.WORKLOADS["qwen_act"]
    rows, chunk_rows, B = 96, 16, 128                       # 16 x 5120 elements = 40 tiles per chunk
    x = to_dev(W.generate_rows(w, 0, 0, rows)).view(rows, w.hidden)
    p = taco.taco_default_params(block=B)
    whole_p, whole_s = taco.taco_compress(x, p)
    pl = torch.empty_like(whole_p)
    sc = torch.empty_like(whole_s)
    per_row = w.hidden // B
    chunks = [(r, r + chunk_rows) for r in range(0, rows, chunk_rows)]
    taco.taco_compress_batch([x[a:b] for a, b in chunks], p, [pl[a * w.hidden:b * w.hidden] for a, b in chunks],
                             [sc[a * per_row:b * per_row] for a, b in chunks])
    torch.cuda.synchronize()
    assert torch.equal(pl, whole_p) and torch.equal(sc, whole_s)
    whole = taco.taco_decompress_sum([pl, pl], [sc, sc], x.shape, p)
    out = torch.empty_like(whole)
    taco.taco_decompress_sum_batch([[pl[a * w.hidden:b * w.hidden]] * 2 for a, b in chunks],
                                   [[sc[a * per_row:b * per_row]] * 2 for a, b in chunks],
                                   [(b - a, w.hidden) for a, b in chunks], p, outs=[out[a:b] for a, b in chunks])
    torch.cuda.synchronize()
    assert torch.equal(out, whole)


def test_overlap_is_refused_on_real_buffers():
    n = 2048 * 4
    x = to_dev(make(n, 3))
    p = taco.taco_default_params()
    with pytest.raises(taco.TacoError, match="overlaps"):
        taco.taco_compress(x, p, x.view(torch.uint8)[:n], torch.empty((n // 128, 2), dtype=torch.float32, device=DEV))
    buf = torch.empty(2 * n, dtype=torch.uint8, device=DEV)       # a payload and the bf16 output that would overwrite it
    sc = torch.ones((n // 128, 2), dtype=torch.float32, device=DEV)
    with pytest.raises(taco.TacoError, match="overlaps"):
        taco.taco_decompress(buf[:n], sc, (n,), p, out=buf.view(torch.bfloat16))
    # inputs may repeat: the same payload twice is fine
    pl, sc = taco.taco_compress(x, p)
    out = taco.taco_decompress_sum([pl, pl], [sc, sc], (n,), p)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
