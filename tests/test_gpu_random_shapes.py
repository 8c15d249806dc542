"""Seeded sweep over random shapes, block sizes, payload counts, layouts and kernel families:
every entry point against the oracle on each case (small tensors, so whole-tile, leftover-block
and zero-padded-tail paths all occur)."""
import numpy as np
import pytest
import torch

from paper_2604_24088_amd import taco
from paper_2604_24088_amd import workloads as W

import parity_util as P

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def cases(count, seed, ks=(1, 1, 2, 3, 5, 8, 16), max_tiles=7):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        block = int(rng.choice([32, 64, 128, 256, 512]))
        tiles = int(rng.integers(0, max_tiles))
        n = tiles * 2048 + int(rng.integers(0, 2048)) + (1 if tiles == 0 else 0)
        k = int(rng.choice(ks))
        layout = int(rng.integers(0, 2))
        impl = int(rng.choice([taco.TACO_IMPL_AUTO, taco.TACO_IMPL_BUTTERFLY]))
        kind = int(rng.integers(0, 4))
        out.append((block, n, k, layout, impl, kind, int(rng.integers(1 << 30))))
    return out


def make_input(n, kind, rng):
    if kind == 0:
        x = rng.standard_normal(n) * 0.02
    elif kind == 1:
        x = rng.standard_t(3.0, n) * 0.01
    elif kind == 2:
        x = rng.standard_normal(n) * 1e-4
        x[rng.random(n) < 0.02] = 0.0
        x[rng.random(n) < 0.002] *= 1000.0
    else:
        x = rng.standard_normal(n) * 0.02
        x[rng.random(n) < 0.3] = 0.0
        x[: min(n, 600)] = 0.0                      # whole zero blocks
    return W.float32_to_bf16_bits(x.astype(np.float32))


# second set: payload counts that are multiples of the decode ring (the fused call's loop without conditional refills)
# and more tiles, so that a wave runs several rounds and the launch mixes that loop with the guarded last tile
@pytest.mark.parametrize("block,n,k,layout,impl,kind,seed", cases(60, 20260) + cases(40, 20261, ks=(4, 8, 12, 16), max_tiles=13))
def test_random_case(oracle, block, n, k, layout, impl, kind, seed):
    rng = np.random.default_rng(seed)
    what = f"B={block} n={n} k={k} layout={layout} impl={impl} kind={kind}"
    p = taco.taco_default_params(block=block, impl=impl, layout=layout)
    xs = [make_input(n, kind, rng) for _ in range(k)]
    enc = [oracle.compress(x, block=block) for x in xs]
    z0 = oracle.compress(xs[0], block=block, want_z=True)[2]
    pad8 = np.zeros((-n) % 8, dtype=np.uint16)
    # compress
    buf, sc = taco.taco_compress(torch.from_numpy(np.concatenate([xs[0], pad8]).view(np.int16)).to(DEV).view(torch.bfloat16)[:n], p)
    torch.cuda.synchronize()
    gp, gs = (P.deinterleave(buf.cpu().numpy(), block) if layout else (buf.cpu().numpy(), sc.cpu().numpy()))
    P.check_scales(gs, enc[0][1], what)
    # Sparse inputs (kind 3) leave rotated values that are sums of a handful of bf16 numbers, and their
    # ratios to the block maximum hit rounding ties exactly far more often than dense data does: the
    # share of identical codes is lower there, the one-code bound is not; z=z0 makes check_codes assert that
    # every differing code does sit on such a tie of the oracle's own Z / s.
    P.check_codes(gp, enc[0][0], enc[0][1], block, what, min_match=P.CODE_MATCH_MIN_SPARSE if kind == 3 else P.CODE_MATCH_MIN,
                  z=z0)
    # decompress_sum of the oracle's payloads
    if layout:
        dp = [torch.from_numpy(P.interleave(e[0], e[1], block)).to(DEV) for e in enc]
        ds = None
    else:
        dp = [torch.from_numpy(e[0]).to(DEV) for e in enc]
        ds = [torch.from_numpy(e[1]).to(DEV) for e in enc]
    guard = torch.zeros(n + ((-n) % 8) + 16, dtype=torch.bfloat16, device=DEV)
    out = taco.taco_decompress_sum(dp, ds, (n,), p, out=guard[:n])
    torch.cuda.synchronize()
    ref, acc = oracle.decompress_sum([e[0] for e in enc], [e[1] for e in enc], n, block=block, want_sum=True)
    P.check_recon(out.view(torch.int16).cpu().numpy().view(np.uint16), ref, block, what,
                  min_exact=P.RECON_EXACT_MIN_MIXED_SUM if k > 1 else P.RECON_EXACT_MIN_MIXED, acc=acc)
    assert torch.all(guard[n:] == 0), what
    # fused sum -> compress equals the two separate calls
    fb, fs = taco.taco_decompress_sum_compress(dp, ds, (n,), p)
    ub, us = taco.taco_compress(out, p)
    torch.cuda.synchronize()
    assert torch.equal(fb, ub), what
    assert layout or torch.equal(fs, us), what
