"""Pins for the oracle's Hadamard matrix and orthonormal rotation (Eq. ash_rotation and the
identity H^T = H^-1 = H/sqrt(B) stated below it)."""
import os

import numpy as np
import pytest
import scipy.linalg

GOLD = os.path.join(os.path.dirname(__file__), "golden")
SIZES = [2, 4, 8, 16, 32, 64, 128, 256, 512]


def read_golden():
    mats, cur = {}, None
    for line in open(os.path.join(GOLD, "hadamard_small.txt")):
        line = line.strip()
        if not line or line[0] == "#":
            continue
        if line[0] == "H":
            cur = line
            mats[cur] = []
        else:
            mats[cur].append([float(t) for t in line.split()])
    return {k: np.array(v) for k, v in mats.items()}


def test_small_matrices_golden(oracle):
    g = read_golden()
    assert np.array_equal(oracle.hadamard_matrix(2), g["H2"])
    assert np.array_equal(oracle.hadamard_matrix(4), g["H4"])


@pytest.mark.parametrize("B", SIZES)
def test_matrix_matches_library_and_is_orthogonal(oracle, B):
    H = oracle.hadamard_matrix(B)
    assert np.array_equal(H, scipy.linalg.hadamard(B).astype(np.float64))   # natural order
    assert np.array_equal(H, H.T)
    assert np.all(H[0] == 1.0) and np.all(np.abs(H) == 1.0)
    assert np.array_equal(H @ H.T, B * np.eye(B))


@pytest.mark.parametrize("B", SIZES)
def test_kronecker_recursion(oracle, B):
    if B == 2:
        return
    H2 = oracle.hadamard_matrix(2)
    assert np.array_equal(oracle.hadamard_matrix(B), np.kron(H2, oracle.hadamard_matrix(B // 2)))


@pytest.mark.parametrize("B", SIZES)
def test_rotation_is_library_product_and_involution(oracle, B):
    rng = np.random.default_rng(B)
    x = rng.integers(-1000, 1000, B).astype(np.float64)
    y = oracle.rotate(x)
    assert np.allclose(y, scipy.linalg.hadamard(B) @ x / np.sqrt(B), rtol=1e-14, atol=1e-11)
    back = oracle.rotate(y)
    assert np.allclose(back, x, rtol=0, atol=1e-10)
    if round(np.sqrt(B)) ** 2 == B:          # sqrt(B) exact: integers round-trip exactly
        assert np.array_equal(back, x)
    assert np.isclose(np.dot(y, y), np.dot(x, x), rtol=1e-13)       # energy preserved


def test_rotation_of_basis_vectors(oracle):
    B = 128
    for j in (0, 1, 5, 64, 127):
        e = np.zeros(B)
        e[j] = 1.0
        y = oracle.rotate(e) * np.sqrt(B)
        expect = np.array([(-1.0) ** bin(i & j).count("1") for i in range(B)])
        assert np.allclose(y, expect, atol=1e-14)
    ones = oracle.rotate(np.ones(B))
    assert np.isclose(ones[0], np.sqrt(B)) and np.allclose(ones[1:], 0.0)
