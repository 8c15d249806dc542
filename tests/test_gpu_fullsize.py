"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(default parameters, kernel choice AUTO, whole tensor in one call).

The oracle cannot be run over gigabytes inside a test, so it is run on SAMPLED tiles (groups
of 16 consecutive blocks, including the first and the last of the tensor): blocks are
independent (Algorithm 1 loops over them in parallel), so the oracle's result for a block
does not depend on the rest of the tensor.

  compress         GPU output at the sampled tiles against the oracle on the same inputs.
  decompress(_sum) the sampled tiles of every payload are overwritten with the ORACLE's
                   payload and scales before the full-size GPU decode, so both sides decode
                   identical, oracle-made inputs; the rest of the payload is filler that keeps
                   the launch at full size.
"""
import numpy as np
import pytest
import torch

from paper_2604_24088_amd import taco
from paper_2604_24088_amd import workloads as W

import parity_util as P

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TILE = 2048            # elements handled by one wave iteration of the matrix-core kernels, any block size
N_SAMPLED_TILES = 96


def to_dev(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)


def sampled_tiles(n_tiles: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    pick = rng.choice(n_tiles, size=min(N_SAMPLED_TILES, n_tiles), replace=False)
    return np.unique(np.concatenate([pick, [0, 1, n_tiles - 2, n_tiles - 1]]))


def gather_tiles(flat: np.ndarray, tiles: np.ndarray, per_tile: int) -> np.ndarray:
    idx = (tiles[:, None] * per_tile + np.arange(per_tile)[None, :]).reshape(-1)
    return flat[idx]


@pytest.mark.parametrize("name,B", [("gpt_rowpar", 128), ("qwen_act", 128), ("bwd_grad", 128), ("large_k8", 128),
                                    ("gpt_rowpar", 256), ("qwen_act", 256), ("bwd_grad", 256), ("qwen_act", 512),
                                    ("gpt_rowpar", 64), ("bwd_grad", 32)])
def test_full_size_workload(oracle, name, B):
    w = W.WORKLOADS[name]
    n = w.numel
    n_tiles = n // TILE
    k = w.payloads
    tiles = sampled_tiles(n_tiles, w.seed)
    params = taco.taco_default_params(block=B)
    per_tile = TILE // B
    host = np.empty((w.tokens, w.hidden), dtype=np.uint16)
    payloads, scales, ref_payloads, ref_scales = [], [], [], []
    for i in range(k):
        W.generate(w, i, threads=16, out=host)
        print(f"[{name}/B{B}] payload {i}: generated", flush=True)
        xd = to_dev(host)
        pl, sc = taco.taco_compress(xd, params)
        torch.cuda.synchronize()
        del xd
        # --- compress parity on the sampled tiles
        x_s = gather_tiles(host.reshape(-1), tiles, TILE)
        rp, rs, z = oracle.compress(x_s, block=B, want_z=True)
        gp = gather_tiles(pl.cpu().numpy(), tiles, TILE)
        gs = gather_tiles(sc.cpu().numpy().reshape(-1), tiles, 2 * per_tile).reshape(-1, 2)
        worst_alpha, worst_s = P.check_scales(gs, rs, f"{name}/B{B}[{i}]")
        match = P.check_codes(gp, rp, rs, B, f"{name}/B{B}[{i}]", z=z)
        print(f"[{name}/B{B}] payload {i}: compress parity ok, {match:.6f} of sampled codes identical, "
              f"worst relative error alpha {worst_alpha:.2e}, s {worst_s:.2e}", flush=True)
        # --- patch the oracle's payload into the sampled tiles for the decode test
        idx_c = torch.from_numpy((tiles[:, None] * TILE + np.arange(TILE)[None, :]).reshape(-1)).to(DEV)
        idx_s = torch.from_numpy((tiles[:, None] * per_tile + np.arange(per_tile)[None, :]).reshape(-1)).to(DEV)
        pl[idx_c] = torch.from_numpy(rp).to(DEV)
        sc[idx_s] = torch.from_numpy(rs).to(DEV)
        payloads.append(pl)
        scales.append(sc)
        ref_payloads.append(rp)
        ref_scales.append(rs)
    # --- decode at full size
    out = taco.taco_decompress_sum(payloads, scales, (w.tokens, w.hidden), params)
    torch.cuda.synchronize()
    got = gather_tiles(out.view(torch.int16).cpu().numpy().view(np.uint16).reshape(-1), tiles, TILE)
    ref = oracle.decompress_sum(ref_payloads, ref_scales, tiles.size * TILE, block=B)
    exact = P.check_recon(got, ref, B, f"{name} decompress_sum k={k}",
                          min_exact=P.RECON_EXACT_MIN if k == 1 else P.RECON_EXACT_MIN_SUM)
    print(f"[{name}/B{B}] decompress_sum k={k}: parity ok, {exact:.6f} of sampled outputs identical", flush=True)
    if k == 1:
        out1 = taco.taco_decompress(payloads[0], scales[0], (w.tokens, w.hidden), params)
        torch.cuda.synchronize()
        assert torch.equal(out1, out)
    # --- fused decompress_sum -> compress at full size: no bit differs from the two separate calls,
    # and on the sampled tiles the blocks whose bf16 intermediate equals the oracle's meet the usual bar
    fp, fs = taco.taco_decompress_sum_compress(payloads, scales, (w.tokens, w.hidden), params)
    up, us = taco.taco_compress(out, params)
    torch.cuda.synchronize()
    assert torch.equal(fp, up) and torch.equal(fs, us)
    rp2, rs2 = oracle.compress(ref, block=B)
    same = np.all(got.reshape(-1, B) == ref.reshape(-1, B), axis=1)
    gp2 = gather_tiles(fp.cpu().numpy(), tiles, TILE).reshape(-1, B)
    gs2 = gather_tiles(fs.cpu().numpy().reshape(-1), tiles, 2 * per_tile).reshape(-1, 2)
    assert same.mean() >= 0.5
    P.check_scales(gs2[same], rs2[same], f"{name}/B{B} fused")
    m2 = P.check_codes(gp2[same], rp2.reshape(-1, B)[same], rs2[same], B, f"{name}/B{B} fused")
    print(f"[{name}/B{B}] fused sum->compress: identical to the two calls; {same.mean():.3f} of sampled blocks "
          f"have the oracle's intermediate, {m2:.6f} of their codes identical", flush=True)
    del fp, fs, up, us
    # --- properties that hold at any size, over the whole tensor
    sc_all = scales[0]
    assert torch.isfinite(sc_all).all() and (sc_all[:, 0] > 0).all() and (sc_all[:, 1] >= 0).all()
    codes = payloads[0].view(-1, B)
    assert not ((codes & 0x7F) == 0x7F).any()                                   # never NaN
    nonzero = sc_all[:, 1] > 0
    assert ((codes & 0x7F).max(dim=1).values[nonzero] == 0x7E).all()            # block max maps to Q_max
    assert torch.isfinite(out.float()).all()
