"""GPU parity over WHOLE benchmark tensors: every element of every configuration, not a sample.

For each of the five benchmark configurations (block 128; the Qwen-style tensor again at the
paper's optimum block 256; one tensor at each of the other block sizes) the GPU compresses the full tensor in the launch configuration bench.py
times (default parameters, kernel choice AUTO, one call per tensor) and the oracle compresses the same
bits; every code and every {alpha, s} record is compared.  The decode side is then fed the ORACLE's
payloads (so both sides decode identical bits): taco_decompress for one payload, taco_decompress_sum
for the configuration's k, every output element compared with the oracle's decode.

The oracle works through the tensor in row slabs (blocks are independent, Algorithm 1 loops over them
in parallel, so a slab that is a whole number of blocks gives the same result as the whole tensor);
the shares of identical codes / outputs are taken over the WHOLE tensor and held to the bars of
parity_util: codes >= 99.99 % identical, the rest one code away and on a rounding tie of the oracle's
own Z / s; scales within 1e-6; outputs within max(1 bf16 ulp, 1e-3 of the block maximum), and a
minimum share bit-identical."""
import numpy as np
import pytest
import torch

from paper_2604_24088_amd import taco
from paper_2604_24088_amd import workloads as W

import parity_util as P

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
SLAB_ELEMS = 1 << 23          # elements the oracle handles at a time (a multiple of every block size)


def to_dev(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)


def slabs(n: int):
    for a in range(0, n, SLAB_ELEMS):
        yield a, min(a + SLAB_ELEMS, n)


@pytest.mark.parametrize("name,B", [("tiny", 128), ("gpt_rowpar", 128), ("qwen_act", 128), ("bwd_grad", 128),
                                    ("qwen_act", 256), ("large_k8", 128),
                                    # the other block sizes on one whole tensor each
                                    ("gpt_rowpar", 32), ("gpt_rowpar", 64), ("gpt_rowpar", 512), ("bwd_grad", 256)])
def test_whole_tensor_parity(oracle, name, B):
    w = W.WORKLOADS[name]
    n, k = w.numel, w.payloads
    assert n % B == 0
    params = taco.taco_default_params(block=B)
    host = np.empty((w.tokens, w.hidden), dtype=np.uint16)
    ref_payloads, ref_scales = [], []
    differing = 0
    worst = [0.0, 0.0]
    for i in range(k):
        W.generate(w, i, threads=16, out=host)
        flat = host.reshape(-1)
        pl, sc = taco.taco_compress(to_dev(host), params)
        torch.cuda.synchronize()
        gp, gs = pl.cpu().numpy(), sc.cpu().numpy()
        del pl, sc
        rp_all = np.empty(n, dtype=np.uint8)
        rs_all = np.empty((n // B, 2), dtype=np.float32)
        for a, b in slabs(n):
            rp, rs, z = oracle.compress(flat[a:b], block=B, want_z=True)
            rp_all[a:b] = rp
            rs_all[a // B:b // B] = rs
            wa, ws = P.check_scales(gs[a // B:b // B], rs, f"{name}/B{B}[{i}] elements [{a}, {b})")
            worst = [max(worst[0], wa), max(worst[1], ws)]
            # min_match = 0: the share is taken over the whole tensor below; what is asserted per slab is that
            # no code is more than one step away and that every differing code sits on a tie of the oracle's Z / s
            match = P.check_codes(gp[a:b], rp, rs, B, f"{name}/B{B}[{i}] elements [{a}, {b})", min_match=0.0, z=z)
            differing += int(round((1.0 - match) * (b - a)))
        ref_payloads.append(rp_all)
        ref_scales.append(rs_all)
        print(f"[{name}/B{B}] payload {i}: compress compared on all {n} elements", flush=True)
    share = 1.0 - differing / (k * n)
    print(f"[{name}/B{B}] codes identical: {share:.8f} ({differing} of {k * n} one step apart, each on a rounding tie); "
          f"worst relative error alpha {worst[0]:.2e}, s {worst[1]:.2e}", flush=True)
    assert differing <= max(1, int((1.0 - P.CODE_MATCH_MIN) * k * n)), f"only {share:.6f} of codes identical"
    del host, gp, gs

    # ---- decode the ORACLE's payloads on the GPU
    dp = [torch.from_numpy(p).to(DEV) for p in ref_payloads]
    ds = [torch.from_numpy(s).to(DEV) for s in ref_scales]
    shape = (w.tokens, w.hidden)
    calls = [("decompress", [0])] + ([(f"decompress_sum k={k}", list(range(k)))] if k > 1 else [("decompress_sum k=1", [0])])
    outs = {}
    for what, idx in calls:
        if what == "decompress":
            out = taco.taco_decompress(dp[0], ds[0], shape, params)
        else:
            out = taco.taco_decompress_sum([dp[j] for j in idx], [ds[j] for j in idx], shape, params)
        torch.cuda.synchronize()
        got = out.view(torch.int16).cpu().numpy().view(np.uint16).reshape(-1)
        outs[what] = out
        identical = 0
        for a, b in slabs(n):
            ref, acc = oracle.decompress_sum([ref_payloads[j][a:b] for j in idx], [ref_scales[j][a // B:b // B] for j in idx],
                                             b - a, block=B, want_sum=True)
            # min_exact = 0: the share is taken over the whole tensor below
            exact = P.check_recon(got[a:b], ref, B, f"{name}/B{B} {what} elements [{a}, {b})", min_exact=0.0, acc=acc)
            identical += int(round(exact * (b - a)))
        share = identical / n
        need = P.RECON_EXACT_MIN if len(idx) == 1 else P.RECON_EXACT_MIN_SUM
        print(f"[{name}/B{B}] {what}: all {n} outputs within tolerance, {share:.6f} bit-identical", flush=True)
        assert share >= need, f"{what}: only {share:.6f} of outputs identical"
    if k == 1:
        assert torch.equal(outs["decompress"], outs["decompress_sum k=1"])
