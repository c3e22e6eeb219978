"""Pins for the CPU checker's sparse x dense product (no GPU needed).

The product is pinned against numpy's dense matmul on small inputs, closed forms, exact
small-integer inputs, and the paper's encoding-independence check (Section 5.2: the result
may not depend on the sparsity annotation).
"""
import itertools
import numpy as np
import pytest

import oracle
from gen import workloads as W, prng


def _dense(w, vals=None):
    A = np.zeros(w.shape, dtype=np.float64)
    A[w.rows, w.cols] = w.vals if vals is None else vals
    return A


@pytest.mark.parametrize("N", [1, 3, 64])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_coo_product_against_dense_matmul(N, dtype):
    w = W.uniform_random(37, 53, 400, dtype=dtype)
    B = w.dense_operand(N)
    C, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, B)
    ref = _dense(w) @ B.astype(np.float64)
    refmag = np.abs(_dense(w)) @ np.abs(B.astype(np.float64))
    assert C.dtype == dtype
    tol = 4e-16 if dtype == np.float64 else 1e-7
    assert np.all(np.abs(C - ref) <= tol * refmag + 1e-300)
    assert np.allclose(mag, refmag, rtol=1e-12, atol=0)


def test_exact_integer_inputs_are_bit_exact():
    w = W.cfg2_powerlaw_csr(2000, 1500, cap=400)
    vals = w.exact_values()
    B = w.dense_operand(5, exact=True)
    C, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, vals, B)
    ref = _dense(w, vals) @ B            # every partial sum is an integer < 2^53: exact in any order
    assert np.array_equal(C, ref)
    assert np.array_equal(mag, np.abs(_dense(w, vals)) @ np.abs(B))


def test_closed_forms():
    n = 50
    idx = np.arange(n, dtype=np.int64)
    B = prng.uniform_pm1(3, 1, n * 4).reshape(n, 4)
    C, _ = oracle.matmul_coo((n, n), idx, idx, np.ones(n), B)           # A = I  =>  C = B
    assert np.array_equal(C, B)
    d = prng.uniform_pm1(3, 2, n)
    C, _ = oracle.matmul_coo((n, n), idx, idx, d, B)                     # diagonal A: row scaling
    assert np.allclose(C, d[:, None] * B, rtol=2.3e-16, atol=0)   # x87 product rounded twice: <= 1 ulp
    C, mag = oracle.matmul_coo((7, 9), [4], [6], [2.5], np.arange(18.0).reshape(9, 2))   # single entry
    ref = np.zeros((7, 2)); ref[4] = 2.5 * np.array([12.0, 13.0])
    assert np.array_equal(C, ref) and np.array_equal(mag, np.abs(ref))
    # B = unit columns e_k reads column k of A back out
    w = W.uniform_random(20, 12, 60)
    C, _ = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, np.eye(12))
    assert np.array_equal(C, _dense(w))
    # all-ones values and x: y[i] = row length
    y, _ = oracle.matmul_coo(w.shape, w.rows, w.cols, np.ones(w.nnz), np.ones(12))
    assert np.array_equal(y[:, 0], np.bincount(w.rows, minlength=20).astype(np.float64))


def test_accumulate_and_empty_rows():
    w = W.cfg4_hypersparse_dcsr(512, 512, frac=0.05, per_row=4)
    x = w.dense_operand(1)
    C0 = prng.uniform_pm1(9, 1, 512).reshape(512, 1)
    y, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, x)
    empty = np.bincount(w.rows, minlength=512) == 0
    assert np.all(y[empty] == 0.0) and np.all(mag[empty] == 0.0)
    ya, maga = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, x, accumulate=True, C=C0)
    assert np.array_equal(ya[empty], C0[empty])
    assert np.allclose(ya, C0 + y, rtol=0, atol=1e-15)
    assert np.allclose(maga, np.abs(C0) + mag, rtol=1e-15, atol=0)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_result_is_independent_of_the_encoding(dtype):
    """Section 5.2: every level-type combination, both orderings, several widths: same C."""
    w = W.cfg2_powerlaw_csr(300, 200, cap=64)
    w.vals = w.vals.astype(dtype)
    B = w.dense_operand(6).astype(dtype)
    ref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, B)
    for lt in itertools.product([0, 1], repeat=2):
        for order in [(0, 1), (1, 0)]:
            for pw, cw in [(0, 0), (32, 32), (16, 64), (64, 16)]:
                t = oracle.pack(lt, order, w.shape, [w.rows, w.cols], w.vals, pw, cw)
                C, mag2 = t.matmul(B)
                tol = 1e-18 if dtype == np.float64 else 0.0
                # extended-precision accumulation: any visiting order rounds to the same result here
                assert np.all(np.abs(C.astype(np.float64) - ref) <= 2.3e-16 * mag * (dtype == np.float64) + tol), (lt, order)
                assert np.allclose(mag2, mag, rtol=1e-13, atol=0)


def test_extended_precision_is_not_the_noise_source():
    """|C_checker - C_exact| must sit far below the 1e-12*mag budget; plain f64 in order may use more."""
    w = W.cfg2_powerlaw_csr(400, 4000, mean=400.0, sigma=0.5, cap=2000)
    x = w.dense_operand(1)
    y, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, x)
    from fractions import Fraction
    rows = np.argsort(-np.bincount(w.rows, minlength=400))[:5]          # the longest rows, exactly
    for i in rows:
        sel = np.nonzero(w.rows == i)[0]
        exact = sum(Fraction(float(w.vals[e])) * Fraction(float(x[w.cols[e], 0])) for e in sel)
        assert abs(Fraction(float(y[i, 0])) - exact) <= Fraction(1.2e-16) * Fraction(float(mag[i, 0]))
    yseq = oracle.matmul_coo_f64seq(w.shape, w.rows, w.cols, w.vals, x)
    assert np.all(np.abs(yseq - y) <= 1e-12 * mag)
    assert np.max(np.abs(yseq - y) / mag) > 1e-17                      # and the two do differ


def test_product_errors():
    with pytest.raises(oracle.OracleError) as e:
        oracle.matmul_coo((3, 3), [0, 3], [0, 0], [1.0, 1.0], np.ones(3))
    assert e.value.code == oracle.ERR_COORD_RANGE
