"""Seeded synthetic inputs shaped like the tensor-parallel intermediate tensors the TACO
paper compresses (Section 3.1: values packed tightly around zero with a long tail;
Section 5.1: GPT and Qwen2.5 models under tensor parallelism).

This module holds input generation only: no step of the compression method lives here.
It serves both the HIP path and the CPU oracle, so the two sides see the same bits.

A tensor is produced in fixed chunks of CHUNK_ROWS rows; chunk c of payload i of
workload w is a pure function of (w.seed, i, c), so any row range can be regenerated
without producing the whole tensor (sampled parity at full size relies on this).
bf16 values are returned as uint16 bit patterns (numpy has no bf16 dtype).
"""
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

CHUNK_ROWS = 64
SEED_BASE = 0x7AC00000


@dataclass(frozen=True)
class Workload:
    name: str
    index: int            # 1-based position in the benchmark's list of configurations
    tokens: int
    hidden: int
    kind: str             # "gauss_outlier_channels" | "student_t" | "grad_sparse_spikes"
    sigma: float
    outlier_fraction: float = 0.0   # share of hidden channels scaled up
    outlier_scale: float = 1.0
    zero_prob: float = 0.0          # per-element probability of an exact zero
    spike_prob: float = 0.0         # per-element probability of a spike
    spike_scale: float = 1.0
    payloads: int = 1               # k: independently seeded tensors of this shape

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index

    @property
    def numel(self) -> int:
        return self.tokens * self.hidden


WORKLOADS = {
    "tiny": Workload("tiny", 1, 256, 1024, "gauss_outlier_channels", 0.02,
                     outlier_fraction=0.01, outlier_scale=50.0),
    "gpt_rowpar": Workload("gpt_rowpar", 2, 8192, 4096, "gauss_outlier_channels", 0.02,
                           outlier_fraction=0.005, outlier_scale=30.0),
    "qwen_act": Workload("qwen_act", 3, 16384, 5120, "student_t", 0.01),
    "bwd_grad": Workload("bwd_grad", 4, 8192, 8192, "grad_sparse_spikes", 1e-4,
                         zero_prob=1e-3, spike_prob=1e-5, spike_scale=1000.0),
    "large_k8": Workload("large_k8", 5, 16384, 12288, "gauss_outlier_channels", 0.02,
                         outlier_fraction=0.01, outlier_scale=30.0, payloads=8),
}


def float32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round binary32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_float32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def outlier_channels(w: Workload) -> np.ndarray:
    """Sorted indices of the hidden channels that carry outliers (same for every payload)."""
    count = int(round(w.outlier_fraction * w.hidden))
    if count == 0:
        return np.zeros(0, dtype=np.int64)
    rng = np.random.Generator(np.random.Philox(key=[w.seed, 0xC4A77E15]))
    return np.sort(rng.permutation(w.hidden)[:count]).astype(np.int64)


def _chunk(w: Workload, payload: int, chunk: int, channels: np.ndarray) -> np.ndarray:
    rows = min(CHUNK_ROWS, w.tokens - chunk * CHUNK_ROWS)
    rng = np.random.Generator(np.random.Philox(key=[w.seed + (payload << 32), chunk]))
    shape = (rows, w.hidden)
    if w.kind == "gauss_outlier_channels":
        x = rng.standard_normal(shape, dtype=np.float32) * np.float32(w.sigma)
        if channels.size:
            x[:, channels] *= np.float32(w.outlier_scale)
    elif w.kind == "student_t":
        # Student-t with 3 degrees of freedom has variance 3; rescale to std = sigma.
        x = rng.standard_t(3.0, size=shape).astype(np.float32) * np.float32(w.sigma / np.sqrt(3.0))
    elif w.kind == "grad_sparse_spikes":
        x = rng.standard_normal(shape, dtype=np.float32) * np.float32(w.sigma)
        u = rng.random(shape, dtype=np.float32)
        x[u < np.float32(w.spike_prob)] *= np.float32(w.spike_scale)
        x[u > np.float32(1.0 - w.zero_prob)] = np.float32(0.0)
    else:
        raise ValueError(w.kind)
    return float32_to_bf16_bits(x)


def generate_rows(w: Workload, payload: int, row_start: int, row_count: int) -> np.ndarray:
    """bf16 bits of rows [row_start, row_start + row_count) of payload `payload`: uint16[row_count, hidden]."""
    assert 0 <= payload < w.payloads and 0 <= row_start and row_start + row_count <= w.tokens
    channels = outlier_channels(w)
    out = np.empty((row_count, w.hidden), dtype=np.uint16)
    c0 = row_start // CHUNK_ROWS
    c1 = (row_start + row_count - 1) // CHUNK_ROWS
    for c in range(c0, c1 + 1):
        blk = _chunk(w, payload, c, channels)
        lo = max(row_start, c * CHUNK_ROWS)
        hi = min(row_start + row_count, c * CHUNK_ROWS + blk.shape[0])
        out[lo - row_start:hi - row_start] = blk[lo - c * CHUNK_ROWS:hi - c * CHUNK_ROWS]
    return out


def generate(w: Workload, payload: int = 0, threads: int = 8, out: np.ndarray = None) -> np.ndarray:
    """Whole tensor of one payload: uint16[tokens, hidden].  Chunks are filled by a thread pool
    (numpy's generators release the GIL); the result does not depend on `threads`."""
    assert 0 <= payload < w.payloads
    channels = outlier_channels(w)
    if out is None:
        out = np.empty((w.tokens, w.hidden), dtype=np.uint16)
    assert out.shape == (w.tokens, w.hidden) and out.dtype == np.uint16
    n_chunks = (w.tokens + CHUNK_ROWS - 1) // CHUNK_ROWS

    def fill(c):
        blk = _chunk(w, payload, c, channels)
        out[c * CHUNK_ROWS:c * CHUNK_ROWS + blk.shape[0]] = blk

    if threads <= 1:
        for c in range(n_chunks):
            fill(c)
    else:
        with ThreadPoolExecutor(max_workers=threads) as pool:
            list(pool.map(fill, range(n_chunks)))
    return out
