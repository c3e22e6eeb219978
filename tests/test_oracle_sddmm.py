"""Pins for the CPU checker's sampled dense-dense product X[i,j] = S[i,j] * A[i,k] * B[k,j] (no GPU needed)."""
import numpy as np
import pytest

import oracle
from gen import workloads as W, prng


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("K", [1, 7, 64])
def test_against_dense_numpy(dtype, K):
    w = W.uniform_random(23, 31, 200, dtype=dtype)
    A = prng.uniform_pm1(4, 1, 23 * K, dtype=dtype).reshape(23, K)
    B = prng.uniform_pm1(4, 2, K * 31, dtype=dtype).reshape(K, 31)
    X, mag = oracle.sddmm_coo(w.shape, w.rows, w.cols, w.vals, A, B)
    full = A.astype(np.float64) @ B.astype(np.float64)
    fullmag = np.abs(A.astype(np.float64)) @ np.abs(B.astype(np.float64))
    ref = w.vals.astype(np.float64) * full[w.rows, w.cols]
    refmag = np.abs(w.vals.astype(np.float64)) * fullmag[w.rows, w.cols]
    tol = 4e-16 if dtype == np.float64 else 1e-7
    assert X.dtype == dtype
    assert np.all(np.abs(X - ref) <= tol * refmag + 1e-300)
    assert np.allclose(mag, refmag, rtol=1e-12, atol=0)


def test_closed_forms_and_exact_integers():
    w = W.uniform_random(20, 20, 120)
    n = 20
    A = prng.uniform_pm1(4, 3, n * n).reshape(n, n)
    X, _ = oracle.sddmm_coo(w.shape, w.rows, w.cols, w.vals, A, np.eye(n))        # B = I: X = S .* A
    assert np.allclose(X, w.vals * A[w.rows, w.cols], rtol=2.3e-16, atol=0)
    X, _ = oracle.sddmm_coo(w.shape, w.rows, w.cols, w.vals, np.eye(n), A)        # A = I: X = S .* B
    assert np.allclose(X, w.vals * A[w.rows, w.cols], rtol=2.3e-16, atol=0)
    a, b = prng.uniform_pm1(4, 4, n), prng.uniform_pm1(4, 5, n)                   # K = 1: outer product, sampled
    X, mag = oracle.sddmm_coo(w.shape, w.rows, w.cols, np.ones(w.nnz), a.reshape(n, 1), b.reshape(1, n))
    assert np.allclose(X, a[w.rows] * b[w.cols], rtol=2.3e-16, atol=0)
    assert np.allclose(mag, np.abs(a[w.rows] * b[w.cols]), rtol=1e-15, atol=0)
    # small integers: exact whatever the order; a transposed A or B would not survive (non-symmetric)
    Ai = prng.small_ints(4, 6, n * 9).reshape(n, 9)
    Bi = prng.small_ints(4, 7, 9 * n).reshape(9, n)
    si = w.exact_values()
    X, _ = oracle.sddmm_coo(w.shape, w.rows, w.cols, si, Ai, Bi)
    assert np.array_equal(X, si * (Ai @ Bi)[w.rows, w.cols])
    assert not np.array_equal(X, si * (Ai @ Bi)[w.cols, w.rows])


def test_errors():
    with pytest.raises(oracle.OracleError) as e:
        oracle.sddmm_coo((3, 3), [0, 3], [0, 0], [1.0, 1.0], np.ones((3, 2)), np.ones((2, 3)))
    assert e.value.code == oracle.ERR_COORD_RANGE
