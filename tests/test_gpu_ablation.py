"""GPU parity of the ablation variants (mode bit mask x code book) against the oracle, and the
reconstruction-error table they exist for."""
import numpy as np
import pytest
import torch

from paper_2604_24088_amd import taco
from paper_2604_24088_amd import workloads as W

import parity_util as P

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

VARIANTS = [(7, 0), (6, 0), (4, 0), (2, 0), (3, 0), (0, 0), (5, 0), (1, 0), (7, 1), (6, 1), (4, 1), (0, 1), (7, 2), (4, 2),
            (6, 2)]


def to_dev(bits):
    return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)


def bits_of(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("impl", [taco.TACO_IMPL_MFMA, taco.TACO_IMPL_BUTTERFLY])
@pytest.mark.parametrize("mode,fmt", VARIANTS)
@pytest.mark.parametrize("block", [128, 256, 32])
@pytest.mark.parametrize("name", ["tiny", "bwd_grad"])
def test_variant_parity(oracle, mode, fmt, block, name, impl):
    """Every mode x code book on both kernel families (the matrix-core kernels multiply by the identity where the
    variant has no rotation)."""
    w = W.WORKLOADS[name]
    x = W.generate_rows(w, 0, 0, 16 if name == "tiny" else 2)
    n = x.size
    p = taco.taco_default_params(block=block, mode=mode, fmt=fmt, impl=impl)
    payload, scales = taco.taco_compress(to_dev(x), p)
    torch.cuda.synchronize()
    rp, rs, z = oracle.compress(x, block=block, mode=mode, fmt=fmt, want_z=True)
    P.check_scales(scales.cpu().numpy(), rs, f"mode={mode} fmt={fmt}")
    # every differing code must sit on a rounding tie of the oracle's Z / s (z=z), whatever the share
    P.check_codes(payload.cpu().numpy(), rp, rs, block, f"mode={mode} fmt={fmt}", fmt=fmt,
                  min_match=P.CODE_MATCH_MIN if mode & 2 else P.CODE_MATCH_MIN_UNROTATED, z=z)
    ref = oracle.decompress(rp, rs, n, block=block, mode=mode, fmt=fmt)
    out = taco.taco_decompress(torch.from_numpy(rp).to(DEV), torch.from_numpy(rs).to(DEV), x.shape, p)
    torch.cuda.synchronize()
    P.check_recon(bits_of(out), ref, block, f"mode={mode} fmt={fmt}", min_exact=P.RECON_EXACT_MIN_SUM)


@pytest.mark.parametrize("mode,fmt", [(7, 1), (4, 0), (7, 2), (2, 0), (0, 1), (5, 2), (3, 0), (1, 0)])
@pytest.mark.parametrize("block", [128, 512, 64])
def test_variant_sum_and_layout(oracle, mode, fmt, block):
    """decompress_sum, the fused sum -> compress and the interleaved layout go through the same variant code."""
    rng = np.random.default_rng(mode * 10 + fmt)
    n = 2048 * 2 + 128 * 5 + 19
    xs = [W.float32_to_bf16_bits((rng.standard_normal(n) * 0.02 * (i + 1)).astype(np.float32)) for i in range(3)]
    enc = [oracle.compress(x, block=block, mode=mode, fmt=fmt) for x in xs]
    ref = oracle.decompress_sum([e[0] for e in enc], [e[1] for e in enc], n, block=block, mode=mode, fmt=fmt)
    p = taco.taco_default_params(block=block, mode=mode, fmt=fmt)
    dp = [torch.from_numpy(e[0]).to(DEV) for e in enc]
    ds = [torch.from_numpy(e[1]).to(DEV) for e in enc]
    out = taco.taco_decompress_sum(dp, ds, (n,), p)
    torch.cuda.synchronize()
    P.check_recon(bits_of(out), ref, block, f"sum mode={mode} fmt={fmt}", min_exact=P.RECON_EXACT_MIN_SUM)
    fp, fs = taco.taco_decompress_sum_compress(dp, ds, (n,), p)
    buf = torch.zeros(n + ((-n) % 8), dtype=torch.bfloat16, device=DEV)
    mid = taco.taco_decompress_sum(dp, ds, (n,), p, out=buf[:n])
    up, us = taco.taco_compress(mid, p)
    torch.cuda.synchronize()
    assert torch.equal(fp, up) and torch.equal(fs, us)
    il = taco.taco_default_params(block=block, mode=mode, fmt=fmt, layout=taco.TACO_LAYOUT_INTERLEAVED)
    padded = np.concatenate([xs[0], np.zeros((-n) % 8, dtype=np.uint16)])
    rec, _ = taco.taco_compress(to_dev(padded)[:n], il)
    sp, ss = taco.taco_compress(to_dev(padded)[:n], p)
    torch.cuda.synchronize()
    gp, gs = P.deinterleave(rec.cpu().numpy(), block)
    assert np.array_equal(gp, sp.cpu().numpy()) and np.array_equal(gs, ss.cpu().numpy())


@pytest.mark.parametrize("mode,fmt", [(7, 1), (6, 0), (6, 1), (7, 2), (6, 2), (4, 0), (0, 0), (2, 1), (5, 2), (3, 0)])
@pytest.mark.parametrize("block,layout", [(64, 0), (128, 1), (256, 0), (512, 1), (32, 0)])
def test_variants_on_the_matrix_cores(oracle, mode, fmt, block, layout):
    """Variants on the matrix-core kernels (impl = MFMA), every entry point against the oracle, k = 8 so that the
    two-waves-per-workgroup form runs too."""
    w = W.WORKLOADS["qwen_act"]
    k, rows = 8, 4                                       # 4 x 5120 elements = 10 tiles per payload
    xs = [W.generate_rows(w, 0, rows * i, rows) for i in range(k)]
    n = xs[0].size
    p = taco.taco_default_params(block=block, mode=mode, fmt=fmt, layout=layout, impl=taco.TACO_IMPL_MFMA)
    enc = [oracle.compress(x, block=block, mode=mode, fmt=fmt) for x in xs]
    z0 = oracle.compress(xs[0], block=block, mode=mode, fmt=fmt, want_z=True)[2]
    buf, sc = taco.taco_compress(to_dev(xs[0]), p)
    torch.cuda.synchronize()
    gp, gs = P.deinterleave(buf.cpu().numpy(), block) if layout else (buf.cpu().numpy(), sc.cpu().numpy())
    P.check_scales(gs, enc[0][1], f"mfma mode={mode} fmt={fmt}")
    P.check_codes(gp, enc[0][0], enc[0][1], block, f"mfma mode={mode} fmt={fmt}", fmt=fmt, z=z0,
                  min_match=P.CODE_MATCH_MIN if mode & 2 else P.CODE_MATCH_MIN_UNROTATED)
    if layout:
        dp, ds = [torch.from_numpy(P.interleave(e[0], e[1], block)).to(DEV) for e in enc], [None] * k
    else:
        dp, ds = [torch.from_numpy(e[0]).to(DEV) for e in enc], [torch.from_numpy(e[1]).to(DEV) for e in enc]
    ref = oracle.decompress_sum([e[0] for e in enc], [e[1] for e in enc], n, block=block, mode=mode, fmt=fmt)
    out = taco.taco_decompress_sum(dp, ds, xs[0].shape, p)
    one = taco.taco_decompress(dp[0], ds[0], xs[0].shape, p)
    fp, fs = taco.taco_decompress_sum_compress(dp, ds, xs[0].shape, p)
    up, us = taco.taco_compress(out, p)
    torch.cuda.synchronize()
    P.check_recon(bits_of(out), ref, block, f"mfma sum mode={mode} fmt={fmt}", min_exact=P.RECON_EXACT_MIN_SUM)
    P.check_recon(bits_of(one), oracle.decompress(enc[0][0], enc[0][1], n, block=block, mode=mode, fmt=fmt), block,
                  f"mfma decompress mode={mode} fmt={fmt}", min_exact=P.RECON_EXACT_MIN_SUM)
    assert torch.equal(fp, up) and (layout == 1 or torch.equal(fs, us))
    # the other family agrees with the same oracle, so the two agree with each other to the same bar
    pb = taco.taco_default_params(block=block, mode=mode, fmt=fmt, layout=layout, impl=taco.TACO_IMPL_BUTTERFLY)
    bb, bs = taco.taco_compress(to_dev(xs[0]), pb)
    torch.cuda.synchronize()
    bp, bsc = P.deinterleave(bb.cpu().numpy(), block) if layout else (bb.cpu().numpy(), bs.cpu().numpy())
    P.check_codes(bp, enc[0][0], enc[0][1], block, f"butterfly mode={mode} fmt={fmt}", fmt=fmt, z=z0,
                  min_match=P.CODE_MATCH_MIN if mode & 2 else P.CODE_MATCH_MIN_UNROTATED)


def test_error_report(oracle, capsys):
    """Relative L2 reconstruction error, GPU compress -> GPU decompress, per variant and workload (the
    numerical side of the paper's ablations on synthetic tensors); must agree with the oracle's."""
    cols = [("full", 7, 0), ("rot+DS", 6, 0), ("DS only", 4, 0), ("std Hadamard", 2, 0), ("ASH no DS", 3, 0),
            ("direct", 0, 0), ("full E5M2", 7, 1), ("ASH+INT8", 7, 2), ("DS-only INT8", 4, 2)]
    lines = ["workload      " + " ".join(f"{c[0]:>13s}" for c in cols)]
    for name in ["tiny", "gpt_rowpar", "qwen_act", "bwd_grad", "large_k8"]:
        w = W.WORKLOADS[name]
        x = W.generate_rows(w, 0, 0, 64)
        g = P.bf16_to_f64(x.reshape(-1))
        row = []
        for _, mode, fmt in cols:
            p = taco.taco_default_params(mode=mode, fmt=fmt)
            payload, scales = taco.taco_compress(to_dev(x), p)
            out = taco.taco_decompress(payload, scales, x.shape, p)
            torch.cuda.synchronize()
            err = np.linalg.norm(P.bf16_to_f64(bits_of(out).reshape(-1)) - g) / np.linalg.norm(g)
            rp, rs = oracle.compress(x, mode=mode, fmt=fmt)
            ro = oracle.decompress(rp, rs, x.size, mode=mode, fmt=fmt)
            ref_err = np.linalg.norm(P.bf16_to_f64(ro) - g) / np.linalg.norm(g)
            assert abs(err - ref_err) <= 0.01 * ref_err + 1e-6, (name, mode, fmt, err, ref_err)
            row.append(err)
        lines.append(f"{name:13s} " + " ".join(f"{v:13.5f}" for v in row))
    with capsys.disabled():
        print("\n" + "\n".join(lines))
