"""Comparison rules between the HIP path and the CPU oracle (used by the GPU parity tests
and by the smoke check).  Tolerances:

  scales  alpha, s    |gpu - ref| <= 1e-6 * |ref|  (fp32 values; s = 0 must match exactly)
  codes               identical on >= 99.99 % of elements (at most one differing code in samples
                      too small to resolve that), the rest at most one code away in
                      sign-magnitude order, +0 and -0 merged.  Where the block scale s
                      is zero the sign bit is unspecified.
  reconstruction      per element |gpu - ref| <= max(one bf16 ulp of ref, 1e-3 * max|ref| of
                      its block); max|gpu - ref| / max|ref| over the tensor at most one bf16 ulp
                      of the largest element (between 2^-8 and 2^-7 of it); and a minimum share of
                      bit-identical elements: 99.5 % for one
                      decoded payload, 99 % for sums of k payloads (k fp32 additions, with
                      cancellation), 90 % for synthetic random codes (18 binades inside a block).

The code rule follows from the arithmetic: the kernels compute Z/s in fp32 (relative error a
few 2^-24) while the oracle works in double, so only values within ~1e-7 relative of a
rounding boundary (spacing 2^-4 relative) can land on the neighbouring code: ~1e-5 of the
elements at most.  The reconstruction rule allows the one legal bf16 rounding flip (one ulp,
2^-8 to 2^-7 of the element) that the same fp32-vs-double difference can cause."""
import numpy as np

CODE_MATCH_MIN = 0.9999
SCALE_RTOL = 1e-6
RECON_RTOL = 1e-3
# Variants without the rotation quantise ratios of bf16 numbers, 448 g / max|g|: a large share of them sits
# EXACTLY on a rounding tie, which the last bit of the fp32 reciprocal (GPU) or of the stored fp32 scale
# (oracle) then breaks either way.  Both are one code apart; the identical share is lower.
CODE_MATCH_MIN_UNROTATED = 0.99
RECON_EXACT_MIN = 0.995
RECON_EXACT_MIN_SUM = 0.99
RECON_EXACT_MIN_RANDOM = 0.90


def code_rank(codes: np.ndarray, fmt: int = 0) -> np.ndarray:
    """Position of a code on its format's value axis: sign-magnitude order for the two FP8 formats
    (0 = E4M3, 1 = E5M2), the integer itself for INT8 (2)."""
    if fmt == 2:
        return codes.view(np.int8).astype(np.int32)
    c = codes.astype(np.int32)
    mag = c & 0x7F
    return np.where(c & 0x80, -mag, mag)


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def check_scales(gpu: np.ndarray, ref: np.ndarray, what: str = ""):
    gpu = gpu.reshape(-1, 2).astype(np.float64)
    ref = ref.reshape(-1, 2).astype(np.float64)
    assert gpu.shape == ref.shape, (gpu.shape, ref.shape)
    assert np.all(np.isfinite(gpu)), f"{what}: non-finite scale"
    worst_of = []
    for col, name in ((0, "alpha"), (1, "s")):
        g, r = gpu[:, col], ref[:, col]
        zero = r == 0.0
        assert np.all(g[zero] == 0.0), f"{what}: {name} must be zero where the oracle's is"
        rel = np.abs(g[~zero] - r[~zero]) / np.abs(r[~zero])
        worst = rel.max() if rel.size else 0.0
        assert worst <= SCALE_RTOL, f"{what}: {name} relative error {worst:.3e} > {SCALE_RTOL}"
        worst_of.append(worst)
    return tuple(worst_of)


def check_codes(gpu: np.ndarray, ref: np.ndarray, ref_scales: np.ndarray, block: int, what: str = "", fmt: int = 0,
                min_match: float = CODE_MATCH_MIN):
    gpu = gpu.reshape(-1, block)
    ref = ref.reshape(-1, block)
    assert gpu.shape == ref.shape, (gpu.shape, ref.shape)
    if fmt == 0:
        assert not np.any((gpu & 0x7F) == 0x7F), f"{what}: NaN code produced"
    elif fmt == 1:
        assert not np.any((gpu & 0x7F) >= 0x7C), f"{what}: infinity or NaN code produced"
    dist = np.abs(code_rank(gpu, fmt) - code_rank(ref, fmt))
    zero_blocks = ref_scales.reshape(-1, 2)[:, 1] == 0.0
    assert np.all(code_rank(gpu[zero_blocks], fmt) == 0), f"{what}: non-zero code in an all-zero block"
    match = float((dist == 0).mean())
    assert dist.max() <= 1, f"{what}: a code is {dist.max()} steps from the oracle's"
    # A sample of fewer than 10^4 codes cannot resolve 99.99 %: there a single off-by-one code is let through.
    allowed = max(1, int((1.0 - min_match) * dist.size))
    assert int((dist != 0).sum()) <= allowed, f"{what}: only {match:.6f} of codes identical"
    return match


def check_recon(gpu_bits: np.ndarray, ref_bits: np.ndarray, block: int, what: str = "",
                min_exact: float = RECON_EXACT_MIN):
    g = bf16_to_f64(gpu_bits.reshape(-1))
    r = bf16_to_f64(ref_bits.reshape(-1))
    assert g.shape == r.shape
    assert np.all(np.isfinite(g)), f"{what}: non-finite output"
    n = g.size
    pad = (-n) % block
    rp = np.concatenate([np.abs(r), np.zeros(pad)]).reshape(-1, block)
    block_max = np.repeat(rp.max(axis=1), block)[:n]
    # one bf16 ulp of the oracle value: 2^(floor(log2|r|) - 7)
    with np.errstate(divide="ignore"):
        ulp = np.where(r != 0.0, 2.0 ** (np.floor(np.log2(np.abs(r), where=r != 0, out=np.zeros_like(r))) - 7), 0.0)
    tol = np.maximum(ulp, RECON_RTOL * block_max)
    err = np.abs(g - r)
    bad = err > tol
    assert not bad.any(), f"{what}: {int(bad.sum())} elements off by more than one bf16 ulp / 1e-3 of block max"
    # one ulp is 2^(e-7) for an element in [2^e, 2^(e+1)): up to 2^-7 of it at the low end of a binade
    overall = err.max() / max(np.abs(r).max(), 1e-300)
    assert overall <= 2.0 ** -7, f"{what}: max error {overall:.3e} of the tensor's max"
    exact = float((err == 0).mean())
    assert exact >= min_exact, f"{what}: only {exact:.6f} of outputs identical"
    return exact


# ---- the interleaved payload layout: pure data movement, no arithmetic ---------------------------

def interleave(payload: np.ndarray, scales: np.ndarray, block: int) -> np.ndarray:
    """codes[M*B] + scales[M,2] -> M records of B + 8 bytes (B codes, float alpha, float s)."""
    m = payload.size // block
    rec = np.empty((m, block + 8), dtype=np.uint8)
    rec[:, :block] = payload.reshape(m, block)
    rec[:, block:] = np.ascontiguousarray(scales, dtype=np.float32).reshape(m, 2).view(np.uint8)
    return rec.reshape(-1)


def deinterleave(buf: np.ndarray, block: int):
    rec = buf.reshape(-1, block + 8)
    return np.ascontiguousarray(rec[:, :block]).reshape(-1), np.ascontiguousarray(rec[:, block:]).view(np.float32).reshape(-1, 2)
