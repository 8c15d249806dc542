"""The seeded input generators: shapes and statistics of the benchmark's five configurations, determinism,
and the property the sampled full-size tests rely on (any row range regenerates the same bits)."""
import numpy as np
import pytest

from paper_2604_24088_amd import workloads as W


def test_shapes_and_payload_counts():
    got = {name: (w.tokens, w.hidden, w.payloads) for name, w in W.WORKLOADS.items()}
    assert got == {"tiny": (256, 1024, 1), "gpt_rowpar": (8192, 4096, 1), "qwen_act": (16384, 5120, 1),
                   "bwd_grad": (8192, 8192, 1), "large_k8": (16384, 12288, 8)}
    assert len({w.seed for w in W.WORKLOADS.values()}) == 5


def test_bf16_rounding_is_nearest_even():
    f = np.array([1.0, 1.00390625, 1.01171875, 1.0 + 2.0 ** -9, -3.0e38, 0.0, -0.0], dtype=np.float32)
    b = W.float32_to_bf16_bits(f)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: even mantissa (1.0) wins; 1 + 3*2^-8 ties up to 1 + 2^-6
    assert list(b[:4]) == [0x3F80, 0x3F80, 0x3F82, 0x3F80]
    assert b[5] == 0x0000 and b[6] == 0x8000
    back = W.bf16_bits_to_float32(b)
    assert np.all(np.abs(back[:5] - f[:5]) <= np.abs(f[:5]) * 2.0 ** -8)
    assert np.array_equal(W.float32_to_bf16_bits(back), b)            # bf16 values survive the round trip


@pytest.mark.parametrize("name", ["tiny", "qwen_act", "bwd_grad", "large_k8"])
def test_row_ranges_regenerate_the_same_bits(name):
    w = W.WORKLOADS[name]
    top = W.generate_rows(w, 0, 0, 200)
    assert top.shape == (200, w.hidden) and top.dtype == np.uint16
    assert np.array_equal(W.generate_rows(w, 0, 37, 101), top[37:138])           # straddles chunks of 64 rows
    assert np.array_equal(W.generate_rows(w, 0, 64, 64), top[64:128])
    assert np.array_equal(W.generate_rows(w, 0, 0, 200), top)                    # deterministic
    if w.payloads > 1:
        assert not np.array_equal(W.generate_rows(w, 1, 0, 64), top[:64])        # payloads are seeded apart


def test_whole_tensor_does_not_depend_on_thread_count():
    w = W.WORKLOADS["tiny"]
    a, b = W.generate(w, 0, threads=1), W.generate(w, 0, threads=8)
    assert np.array_equal(a, b) and np.array_equal(a[:200], W.generate_rows(w, 0, 0, 200))


def test_outlier_channels():
    for name, count, scale in [("tiny", 10, 50.0), ("gpt_rowpar", 20, 30.0), ("large_k8", 123, 30.0)]:
        w = W.WORKLOADS[name]
        ch = W.outlier_channels(w)
        assert ch.size == count and np.all(np.diff(ch) > 0) and ch.max() < w.hidden
        x = W.bf16_bits_to_float32(W.generate_rows(w, 0, 0, 256)).astype(np.float64)
        std = x.std(axis=0)
        rest = np.setdiff1d(np.arange(w.hidden), ch)
        assert abs(np.median(std[rest]) / 0.02 - 1.0) < 0.05
        assert abs(np.median(std[ch]) / (0.02 * scale) - 1.0) < 0.1
        if w.payloads > 1:                                                       # same channels in every payload
            y = W.bf16_bits_to_float32(W.generate_rows(w, 3, 0, 256)).astype(np.float64)
            assert np.all(y.std(axis=0)[ch] > 10 * 0.02)


def test_student_t_workload():
    w = W.WORKLOADS["qwen_act"]
    x = W.bf16_bits_to_float32(W.generate_rows(w, 0, 0, 512)).astype(np.float64).reshape(-1)
    assert w.hidden % 128 == 0 and (w.hidden & (w.hidden - 1)) != 0              # whole blocks, not a power of two
    # heavy tails: the variance estimate is noisy (nu = 3), the quartiles are not: 0.7649 sigma/sqrt(3) for t(3)
    q = np.quantile(np.abs(x), 0.5)
    assert abs(q / (0.7649 * 0.01 / np.sqrt(3.0)) - 1.0) < 0.02
    assert np.abs(x).max() > 20 * 0.01                                           # far tail present


def test_gradient_workload():
    w = W.WORKLOADS["bwd_grad"]
    x = W.bf16_bits_to_float32(W.generate_rows(w, 0, 0, 1024)).astype(np.float64).reshape(-1)
    assert abs((x == 0).mean() / 1e-3 - 1.0) < 0.1
    spikes = np.abs(x) > 0.01                                                    # 100 sigma: only the x1000 elements
    assert 0.3e-5 < spikes.mean() < 3e-5
    body = x[~spikes & (x != 0)]
    assert abs(body.std() / 1e-4 - 1.0) < 0.01
