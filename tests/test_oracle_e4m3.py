"""Pins for the oracle's FP8 E4M3 encode / decode (Eq. quantization, Eq. recon_dequant;
format of Section 2.3 / 3.3 with 4 exponent and 3 mantissa bits).

The decode table is pinned to an independent library (PyTorch's float8_e4m3fn CPU cast)
and to hand-derived landmark values; the encoder is pinned by round-tripping every code,
by the library cast over dense sweeps, by the tie rule at every midpoint and by the
saturation / underflow edges."""
import math
import os

import numpy as np
import pytest
import torch

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def lib_decode_table():
    t = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32)
    return t.numpy().astype(np.float64)


def test_decode_table_matches_library(oracle):
    ref = lib_decode_table()
    for c in range(256):
        v = oracle.e4m3_decode(c)
        if c in (0x7F, 0xFF):
            assert math.isnan(v) and math.isnan(ref[c])
        else:
            assert v == ref[c], hex(c)
            assert math.copysign(1.0, v) == (-1.0 if c & 0x80 else 1.0)


def test_decode_landmarks_golden(oracle):
    rows = [l.split() for l in open(os.path.join(GOLD, "e4m3_landmarks.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) >= 25
    for code, val in rows:
        assert oracle.e4m3_decode(int(code, 16)) == float(val), code


def test_format_extremes(oracle):
    finite = [oracle.e4m3_decode(c) for c in range(256) if c not in (0x7F, 0xFF)]
    assert max(finite) == 448.0 and min(finite) == -448.0          # Q_max, no infinities
    assert min(v for v in finite if v > 0) == 2.0 ** -9             # smallest subnormal
    assert all(math.isfinite(v) for v in finite)
    mags = [oracle.e4m3_decode(c) for c in range(0x7F)]
    assert all(b > a for a, b in zip(mags, mags[1:]))               # codes ordered by magnitude


def test_encode_inverts_decode(oracle):
    for c in range(256):
        if c in (0x7F, 0xFF):
            continue
        assert oracle.e4m3_encode(oracle.e4m3_decode(c)) == c, hex(c)
    assert oracle.e4m3_encode(float("nan")) & 0x7F == 0x7F


def test_encode_ties_to_even_at_every_midpoint(oracle):
    for c in range(0x7E):
        lo, hi = oracle.e4m3_decode(c), oracle.e4m3_decode(c + 1)
        mid = 0.5 * (lo + hi)                      # exact in double
        even = c if c % 2 == 0 else c + 1
        assert oracle.e4m3_encode(mid) == even, hex(c)
        assert oracle.e4m3_encode(-mid) == (even | 0x80)
        assert oracle.e4m3_encode(np.nextafter(mid, 0.0)) == c
        assert oracle.e4m3_encode(np.nextafter(mid, 1e9)) == c + 1


def test_encode_saturates_and_underflows(oracle):
    for v in (448.0, 449.0, 463.9, 464.0, 480.0, 1e9, float("inf")):
        assert oracle.e4m3_encode(v) == 0x7E
        assert oracle.e4m3_encode(-v) == 0xFE
    assert oracle.e4m3_encode(2.0 ** -10) == 0x00            # tie between 0 and 2^-9 -> even (0)
    assert oracle.e4m3_encode(np.nextafter(2.0 ** -10, 1.0)) == 0x01
    assert oracle.e4m3_encode(1e-30) == 0x00
    assert oracle.e4m3_encode(-1e-30) == 0x80               # sign survives underflow
    assert oracle.e4m3_encode(-0.0) == 0x80
    assert oracle.e4m3_encode(0.0) == 0x00


def test_encode_matches_library_cast_on_sweeps(oracle):
    """In range, PyTorch's float32 -> float8_e4m3fn cast rounds to nearest even too."""
    rng = np.random.default_rng(11)
    vals = np.concatenate([
        rng.uniform(-448.0, 448.0, 40000),
        rng.standard_normal(40000) * 3.0,
        rng.standard_normal(40000) * 0.02,
        np.exp(rng.uniform(math.log(2.0 ** -12), math.log(448.0), 40000)) * rng.choice([-1.0, 1.0], 40000),
    ]).astype(np.float32)
    lib = torch.from_numpy(vals).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    mine = np.array([oracle.e4m3_encode(float(v)) for v in vals], dtype=np.uint8)
    assert np.array_equal(mine, lib)


def test_encode_is_monotone(oracle):
    xs = np.linspace(-460.0, 460.0, 200001)
    dec = np.array([oracle.e4m3_decode(oracle.e4m3_encode(float(x))) for x in xs])
    assert np.all(np.diff(dec) >= 0)


def test_rounding_error_within_paper_ulp_bound(oracle):
    """Section 3.3: |e| <= 2^(floor(log2|x|) - m), m = 3; nearest rounding gives half of it
    in the normal range and 2^-10 absolute in the subnormal range."""
    rng = np.random.default_rng(5)
    xs = np.exp(rng.uniform(math.log(2.0 ** -9), math.log(447.0), 50000))
    for x in xs:
        err = abs(oracle.e4m3_decode(oracle.e4m3_encode(float(x))) - x)
        e = math.floor(math.log2(x))
        if x >= 2.0 ** -6:
            assert err <= 2.0 ** (e - 3)            # the paper's bound
            assert err <= 2.0 ** (e - 4)            # what nearest rounding actually gives
        else:
            assert err <= 2.0 ** -10


def test_bf16_rounding_matches_library(oracle):
    rng = np.random.default_rng(3)
    vals = np.concatenate([rng.standard_normal(20000), rng.standard_normal(20000) * 1e-4,
                           np.array([1.00390625, 1.01171875, 1.0 + 2.0 ** -9, -(1.0 + 3 * 2.0 ** -9)])])
    vals = vals.astype(np.float32)
    lib = torch.from_numpy(vals).to(torch.bfloat16).view(torch.int16).numpy().astype(np.uint16)
    mine = np.array([oracle.float_to_bf16(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(mine, lib)
