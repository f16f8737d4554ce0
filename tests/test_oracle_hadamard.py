"""Pins for the oracle's randomised Hadamard rotation (Sec. 2.3, Sec. 3.3 Step 1)."""
import numpy as np
import pytest
from scipy.linalg import hadamard

from oracle import pvq_oracle as o


def _signs(n, seed):
    return np.random.default_rng(seed).integers(0, 2, size=n).astype(np.uint8)


@pytest.mark.parametrize("n", [1, 2, 8, 64, 1024])
def test_equals_the_hadamard_matrix_product(n):
    rng = np.random.default_rng(n)
    X = rng.standard_normal((5, n)).astype(np.float32)
    sg = _signs(n, 7)
    s = 1.0 - 2.0 * sg.astype(np.float64)
    H = hadamard(n).astype(np.float64) if n > 1 else np.ones((1, 1))
    want = (X.astype(np.float64) * s) @ H.T / np.sqrt(n)
    got = o.hadamard_rows(X, n, sg)
    assert np.allclose(got, want, rtol=0, atol=1e-5 * np.abs(want).max())
    # the inverse puts the signs behind the transform
    want_inv = (X.astype(np.float64) @ H.T / np.sqrt(n)) * s
    assert np.allclose(o.hadamard_rows(X, n, sg, signs_after=True), want_inv, rtol=0, atol=1e-5 * np.abs(want_inv).max())


def test_unit_vectors_give_the_rows_of_the_matrix_exactly():
    # e_j -> column j of H / sqrt(n): entries (-1)^popcount(i & j) / sqrt(n), exact in float32 for n = 4^m
    n = 256
    X = np.eye(n, dtype=np.float32)
    got = o.hadamard_rows(X, n)
    i, j = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    par = np.array([[bin(a & b).count("1") & 1 for b in range(n)] for a in range(n)])
    assert np.array_equal(got, ((1 - 2 * par) / 16.0).astype(np.float32))


def test_rotation_then_inverse_is_the_identity_and_norms_are_kept():
    rng = np.random.default_rng(3)
    X = (rng.standard_normal((7, 4096)) * 0.02).astype(np.float32)
    sg = _signs(4096, 11)
    Y = o.hadamard_rows(X, 4096, sg)
    assert np.allclose(np.linalg.norm(Y, axis=1), np.linalg.norm(X, axis=1), rtol=1e-5)
    back = o.hadamard_rows(Y, 4096, sg, signs_after=True)
    assert np.allclose(back, X, rtol=0, atol=2e-6 * np.abs(X).max() * 12)
    # spreading: a one-hot outlier ends up with equal magnitude everywhere
    E = np.zeros((1, 4096), dtype=np.float32); E[0, 123] = 5.0
    assert np.allclose(np.abs(o.hadamard_rows(E, 4096, sg)), 5.0 / 64.0)


def test_block_diagonal_on_lengths_that_are_not_powers_of_two():
    # 7 blocks of 512, as 28672 = 7 * 4096 in the model: blocks do not mix
    rng = np.random.default_rng(5)
    X = rng.standard_normal((3, 7 * 512)).astype(np.float32)
    sg = _signs(7 * 512, 13)
    Y = o.hadamard_rows(X, 512, sg)
    for b in range(7):
        sl = slice(b * 512, (b + 1) * 512)
        assert np.array_equal(Y[:, sl], o.hadamard_rows(np.ascontiguousarray(X[:, sl]), 512, sg[sl]))
    with pytest.raises(ValueError):
        o.hadamard_rows(X, 1024, sg)      # does not divide
    with pytest.raises(ValueError):
        o.hadamard_rows(X, 7 * 512, sg)   # not a power of two
