"""A tensor of more than 2^32 elements with a ragged tail: element and byte offsets past 32 bits in every
kernel (the benchmark tensors stop at 2 * 10^8 elements), two payloads summed, both layouts.

The input is drawn on the device (8.6 GB of bf16 would take minutes to generate and copy from the host);
the oracle runs on sampled tiles copied back, chosen to include the first tiles, the tiles on both sides
of element 2^32, the last whole tiles and the ragged tail.  As in the other full-size tests the decode
side is fed the ORACLE's payload at the sampled positions."""
import numpy as np
import pytest
import torch

from paper_2604_24088_amd import taco

import parity_util as P

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TILE = 2048
N = (1 << 32) + 5 * TILE + 77


def draw(seed: int) -> torch.Tensor:
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    x = torch.empty(N, dtype=torch.bfloat16, device=DEV)
    step = 1 << 28
    for a in range(0, N, step):
        b = min(a + step, N)
        x[a:b] = (torch.randn(b - a, generator=g, device=DEV) * 0.02).to(torch.bfloat16)
    x[(1 << 32) - 3:(1 << 32) + 3] *= 40.0          # outliers right at the 32-bit boundary
    return x


def bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("block,layout", [(128, taco.TACO_LAYOUT_SPLIT), (256, taco.TACO_LAYOUT_INTERLEAVED),
                                          (32, taco.TACO_LAYOUT_SPLIT)])
def test_more_than_2_to_32_elements(oracle, block, layout):
    il = layout == taco.TACO_LAYOUT_INTERLEAVED
    p = taco.taco_default_params(block=block, layout=layout)
    n_tiles = N // TILE
    rng = np.random.default_rng(block)
    edge = (1 << 32) // TILE
    tiles = np.unique(np.concatenate([rng.choice(n_tiles, 40, replace=False), [0, 1, edge - 2, edge - 1, edge, edge + 1,
                                                                              n_tiles - 2, n_tiles - 1]]))
    # element ranges checked: the sampled tiles and everything past the last whole tile
    ranges = [(int(t) * TILE, (int(t) + 1) * TILE) for t in tiles] + [(n_tiles * TILE, N)]
    rec = block + 8
    payloads, scales, ref = [], [], []
    for i in range(2):
        x = draw(100 + i)
        print(f"[B{block} layout {layout}] payload {i}: drawn", flush=True)
        pl, sc = taco.taco_compress(x.view(1, N), p)
        torch.cuda.synchronize()
        per = []
        for a, b in ranges:
            xs = bits(x[a:b])
            rp, rs, z = oracle.compress(xs, block=block, want_z=True)
            nb = rs.shape[0]
            b0 = a // block
            if il:
                raw = pl[b0 * rec:(b0 + nb) * rec].cpu().numpy()
                gp, gs = P.deinterleave(raw, block)
            else:
                gp = pl[b0 * block:(b0 + nb) * block].cpu().numpy()
                gs = sc[b0:b0 + nb].cpu().numpy()
            what = f"B{block} layout {layout} payload {i} elements [{a}, {b})"
            P.check_scales(gs, rs, what)
            P.check_codes(gp, rp, rs, block, what, z=z)
            # the oracle's payload goes in at the sampled positions for the decode below
            if il:
                pl[b0 * rec:(b0 + nb) * rec] = torch.from_numpy(P.interleave(rp, rs, block)).to(DEV)
            else:
                pl[b0 * block:(b0 + nb) * block] = torch.from_numpy(rp).to(DEV)
                sc[b0:b0 + nb] = torch.from_numpy(rs).to(DEV)
            per.append((rp, rs))
        del x
        payloads.append(pl)
        scales.append(sc)
        ref.append(per)
        print(f"[B{block} layout {layout}] payload {i}: compress parity ok on {len(ranges)} ranges", flush=True)
    out = taco.taco_decompress_sum(payloads, scales, (1, N), p)
    one = taco.taco_decompress(payloads[1], scales[1], (1, N), p)
    fp, fs = taco.taco_decompress_sum_compress(payloads, scales, (1, N), p)
    up, us = taco.taco_compress(out, p)
    torch.cuda.synchronize()
    assert torch.equal(fp, up) and (il or torch.equal(fs, us))
    for j, (a, b) in enumerate(ranges):
        want, acc = oracle.decompress_sum([ref[0][j][0], ref[1][j][0]], [ref[0][j][1], ref[1][j][1]], b - a, block=block,
                                          want_sum=True)
        small = b - a < 1000                       # the ragged tail: too few elements for a percentage
        P.check_recon(bits(out.view(-1)[a:b]), want, block, f"B{block} layout {layout} sum, elements [{a}, {b})",
                      min_exact=P.RECON_EXACT_MIN_SMALL if small else P.RECON_EXACT_MIN_MIXED_SUM, acc=acc)
        want1, acc1 = oracle.decompress_sum([ref[1][j][0]], [ref[1][j][1]], b - a, block=block, want_sum=True)
        P.check_recon(bits(one.view(-1)[a:b]), want1, block, f"B{block} layout {layout} decompress, elements [{a}, {b})",
                      min_exact=P.RECON_EXACT_MIN_SMALL if small else P.RECON_EXACT_MIN_MIXED, acc=acc1)
    assert torch.isfinite(out.view(-1)[-4096:].float()).all()
    print(f"[B{block} layout {layout}] decode parity ok", flush=True)
