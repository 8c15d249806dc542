"""Pins for the oracle's receiver side (Algorithm 1, Eqs. recon_dequant .. recon_rescale),
the local reduction of k payloads (Section 4.4.2) and the end-to-end error bound that
follows from orthogonality of the rotation and the FP8 rounding bound of Section 3.3."""
import math

import numpy as np
import pytest
import scipy.linalg
import torch

from paper_2604_24088_amd import workloads as W

QMAX = 448.0


def vals(b):
    return W.bf16_bits_to_float32(b).astype(np.float64)


def lib_decode_table():
    return torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)


@pytest.mark.parametrize("B", [16, 128, 256])
def test_decode_against_library_recomputation(oracle, B):
    """Decode arbitrary (valid) codes and scales with library pieces: the framework's fp8 table,
    scipy's Hadamard matrix, numpy long double products, torch's fp32 -> bf16 rounding."""
    rng = np.random.default_rng(40 + B)
    M = 16
    codes = rng.integers(0, 256, M * B).astype(np.uint8)
    codes[(codes & 0x7F) == 0x7F] = 0x7E
    scales = np.stack([np.exp(rng.uniform(0, 8, M)), np.exp(rng.uniform(-9, -3, M))], axis=1).astype(np.float32)
    out, acc = oracle.decompress(codes, scales, M * B, block=B, want_sum=True)
    table = lib_decode_table().astype(np.longdouble)
    H = scipy.linalg.hadamard(B).astype(np.longdouble)
    for k in range(M):
        zhat = table[codes[k * B:(k + 1) * B]] * np.longdouble(float(scales[k, 1]))
        g = (H @ zhat) / np.sqrt(np.longdouble(B)) / np.longdouble(float(scales[k, 0]))
        assert np.allclose(acc[k * B:(k + 1) * B], g.astype(np.float64), rtol=1e-13, atol=1e-300)
    lib_bf16 = torch.from_numpy(acc.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().astype(np.uint16)
    assert np.array_equal(out, lib_bf16)


def test_decode_uses_transpose_free_symmetric_matrix(oracle):
    """A code vector with a single non-zero entry at i decodes to column i of H (= row i)."""
    B = 128
    for i in (1, 6, 100):
        codes = np.zeros(B, dtype=np.uint8)
        codes[i] = 0x38                                    # 1.0
        scales = np.array([[1.0, math.sqrt(B)]], dtype=np.float32)
        _, acc = oracle.decompress(codes, scales, B, block=B, want_sum=True)
        expect = np.array([(-1.0) ** bin(i & j).count("1") for j in range(B)])
        assert np.allclose(acc, expect * (float(scales[0, 1]) / math.sqrt(B)), rtol=1e-14)


@pytest.mark.parametrize("name,B", [("tiny", 128), ("tiny", 256), ("qwen_act", 128), ("bwd_grad", 128), ("gpt_rowpar", 64)])
def test_round_trip_error_bound_per_block(oracle, name, B):
    """Orthogonality gives ||G' - G|| = ||Zhat - Z|| / alpha.  Each normal code is within
    2^-4 relative of Z_i / s, each subnormal within 2^-10 absolute, and |Z|_2 ~ tau sqrt(B),
    so the per-block relative L2 error is at most 2^-4 + 2^-10 sqrt(B) s / |Z|_2 before the
    final bf16 rounding (2^-9 relative)."""
    w = W.WORKLOADS[name]
    x = W.generate_rows(w, 0, 0, 16 if name == "tiny" else 4)
    n = x.size
    payload, scales, z = oracle.compress(x, block=B, want_z=True)
    out, acc = oracle.decompress(payload, scales, n, block=B, want_sum=True)
    g = vals(x).reshape(-1, B)
    rec = acc.reshape(-1, B)
    z = z.reshape(-1, B)
    s = scales[:, 1].astype(np.float64)
    gn = np.linalg.norm(g, axis=1)
    nz = gn > 0
    rel = np.linalg.norm(rec - g, axis=1)[nz] / gn[nz]
    bound = 2.0 ** -4 + 2.0 ** -10 * math.sqrt(B) * s[nz] / np.linalg.norm(z, axis=1)[nz]
    assert np.all(rel <= bound * (1 + 1e-6))
    assert rel.mean() < 0.04                                # typical 3-bit-mantissa noise
    relb = np.linalg.norm(vals(out).reshape(-1, B) - g, axis=1)[nz] / gn[nz]
    assert np.all(relb <= bound + 2.0 ** -8)
    assert np.all(vals(out).reshape(-1, B)[~nz] == 0.0)


def test_sum_of_one_is_decompress(oracle):
    w = W.WORKLOADS["tiny"]
    x = W.generate_rows(w, 0, 0, 8)
    p, s = oracle.compress(x)
    assert np.array_equal(oracle.decompress(p, s, x.size), oracle.decompress_sum([p], [s], x.size))


@pytest.mark.parametrize("k", [2, 4, 8])
def test_sum_of_identical_payloads_scales(oracle, k):
    w = W.WORKLOADS["tiny"]
    x = W.generate_rows(w, 0, 0, 8)
    p, s = oracle.compress(x)
    _, one = oracle.decompress(p, s, x.size, want_sum=True)
    outk, acck = oracle.decompress_sum([p] * k, [s] * k, x.size, want_sum=True)
    if k == 2:
        assert np.array_equal(acck, 2 * one)                # one addition of equal terms is exact
    assert np.allclose(acck, k * one, rtol=4e-16 * k, atol=0)
    lib = torch.from_numpy(acck.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().astype(np.uint16)
    assert np.array_equal(outk, lib)
    assert np.allclose(W.bf16_bits_to_float32(outk), k * one, rtol=2.0 ** -8, atol=0)


def test_sum_is_sum_of_decodes(oracle):
    rng = np.random.default_rng(77)
    B, M, k = 128, 12, 5
    n = M * B
    ps, ss, parts = [], [], []
    for i in range(k):
        x = W.float32_to_bf16_bits((rng.standard_normal(n) * 0.02 * (i + 1)).astype(np.float32))
        p, s = oracle.compress(x, block=B)
        ps.append(p)
        ss.append(s)
        parts.append(oracle.decompress(p, s, n, block=B, want_sum=True)[1])
    out, acc = oracle.decompress_sum(ps, ss, n, block=B, want_sum=True)
    total = np.zeros(n)
    for part in parts:                                       # payload index ascending
        total += part
    assert np.array_equal(acc, total)
    # Any other order agrees to double rounding.
    assert np.allclose(acc, np.sum(parts[::-1], axis=0), rtol=0, atol=1e-15 * np.max(np.abs(parts)))
    # The sum stays close to the sum of the inputs (each term carries FP8 noise).
    assert np.allclose(vals(out), acc, rtol=2.0 ** -8, atol=0)             # one bf16 rounding


def test_sum_rejects_bad_arguments(oracle):
    p = np.zeros(128, dtype=np.uint8)
    s = np.zeros((1, 2), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.decompress_sum([p], [s], 128, block=100)
