"""Pins for the CPU checker's sparse x sparse product with a sparse result (the SpMSpM kernel).  No GPU needed."""
import json
import os

import numpy as np
import pytest
import scipy.sparse

import oracle
from gen import workloads as W, prng

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def pair(m, k, n, nnz_a, nnz_b, dtype=np.float64, seed=0):
    return (W.uniform_random(m, k, nnz_a, dtype=dtype, seed=W.BASE_SEED + 300 + seed),
            W.uniform_random(k, n, nnz_b, dtype=dtype, seed=W.BASE_SEED + 400 + seed))


def dense(w):
    D = np.zeros(w.shape, dtype=np.float64)
    D[w.rows, w.cols] = w.vals
    return D


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_against_dense_numpy_values_and_structural_pattern(dtype):
    a, b = pair(37, 29, 41, 160, 170, dtype)
    ci, cj, cv, mag = oracle.spgemm_coo(a.shape, a.rows, a.cols, a.vals, b.shape, b.rows, b.cols, b.vals)
    pattern = ((dense(a) != 0).astype(np.int64) @ (dense(b) != 0).astype(np.int64)) > 0      # a pair of stored entries exists
    ii, jj = np.nonzero(pattern)                                                            # row-major order
    assert np.array_equal(ci, ii) and np.array_equal(cj, jj)
    ref = dense(a) @ dense(b)
    refmag = np.abs(dense(a)) @ np.abs(dense(b))
    tol = 4e-16 if dtype == np.float64 else 1e-7
    assert cv.dtype == dtype
    assert np.all(np.abs(cv - ref[ci, cj]) <= tol * refmag[ci, cj])
    assert np.allclose(mag, refmag[ci, cj], rtol=1e-12, atol=0)


def test_against_an_independent_sparse_library():
    a, b = pair(300, 200, 250, 3000, 2500)
    ci, cj, cv, _ = oracle.spgemm_coo(a.shape, a.rows, a.cols, a.vals, b.shape, b.rows, b.cols, b.vals)
    A = scipy.sparse.csr_matrix((a.vals, (a.rows, a.cols)), shape=a.shape)
    B = scipy.sparse.csr_matrix((b.vals, (b.rows, b.cols)), shape=b.shape)
    C = (A @ B).tocsr()
    C.sort_indices()
    C = C.tocoo()
    assert np.array_equal(ci, C.row) and np.array_equal(cj, C.col)
    assert np.allclose(cv, C.data, rtol=1e-13, atol=1e-15)


def test_closed_forms_and_kept_zeros():
    a, _ = pair(40, 40, 40, 300, 1)
    eye = np.arange(40)
    order = np.lexsort((a.cols, a.rows))
    # A . I = A and I . A = A, entry for entry
    for left in (True, False):
        if left:
            ci, cj, cv, _ = oracle.spgemm_coo((40, 40), eye, eye, np.ones(40), a.shape, a.rows, a.cols, a.vals)
        else:
            ci, cj, cv, _ = oracle.spgemm_coo(a.shape, a.rows, a.cols, a.vals, (40, 40), eye, eye, np.ones(40))
        assert np.array_equal(ci, a.rows[order]) and np.array_equal(cj, a.cols[order]) and np.array_equal(cv, a.vals[order])
    # diagonal scaling from the left: C = diag(d) . A
    d = prng.uniform_pm1(3, 1, 40)
    ci, cj, cv, mag = oracle.spgemm_coo((40, 40), eye, eye, d, a.shape, a.rows, a.cols, a.vals)
    assert np.allclose(cv, d[a.rows[order]] * a.vals[order], rtol=2.3e-16, atol=0)
    assert np.allclose(mag, np.abs(d[a.rows[order]] * a.vals[order]), rtol=2.3e-16, atol=0)
    # a sum that cancels and an explicit zero both stay stored: the workspace marks an element when it is first touched
    ci, cj, cv, mag = oracle.spgemm_coo((1, 2), [0, 0], [0, 1], np.array([1.0, -1.0]), (2, 2), [0, 1, 1], [0, 0, 1], np.array([2.0, 2.0, 0.0]))
    assert np.array_equal(ci, [0, 0]) and np.array_equal(cj, [0, 1]) and np.array_equal(cv, [0.0, 0.0])
    assert np.array_equal(mag, [4.0, 0.0])
    # row vector times column vector and the reverse: inner and outer product
    u, v = prng.uniform_pm1(3, 2, 6), prng.uniform_pm1(3, 3, 6)
    z, r = np.zeros(6, dtype=np.int64), np.arange(6)
    ci, cj, cv, _ = oracle.spgemm_coo((1, 6), z, r, u, (6, 1), r, z, v)
    assert len(ci) == 1 and abs(cv[0] - np.dot(u, v)) <= 4e-16 * np.dot(np.abs(u), np.abs(v))
    ci, cj, cv, _ = oracle.spgemm_coo((6, 1), r, z, u, (1, 6), z, r, v)
    assert np.array_equal(cv.reshape(6, 6), np.outer(u, v))


def test_exact_integers_any_order_of_the_triples():
    a, b = pair(60, 50, 70, 500, 600)
    va = prng.small_ints(5, 1, a.nnz)
    vb = prng.small_ints(5, 2, b.nnz)
    ref = oracle.spgemm_coo(a.shape, a.rows, a.cols, va, b.shape, b.rows, b.cols, vb)
    pa, pb = prng.permutation(5, 3, a.nnz), prng.permutation(5, 4, b.nnz)
    got = oracle.spgemm_coo(a.shape, a.rows[pa], a.cols[pa], va[pa], b.shape, b.rows[pb], b.cols[pb], vb[pb])
    for x, y in zip(ref, got):
        assert np.array_equal(x, y)
    Da, Db = np.zeros(a.shape), np.zeros(b.shape)
    Da[a.rows, a.cols] = va
    Db[b.rows, b.cols] = vb
    assert np.array_equal(ref[2], (Da @ Db)[ref[0], ref[1]])


def test_empty_operands_and_errors():
    e = np.zeros(0, dtype=np.int64)
    ci, cj, cv, mag = oracle.spgemm_coo((3, 4), e, e, np.zeros(0), (4, 5), [0], [0], np.ones(1))
    assert len(ci) == 0 and len(cv) == 0
    ci, _, _, _ = oracle.spgemm_coo((3, 4), [0], [1], np.ones(1), (4, 5), [2], [0], np.ones(1))     # no matching k
    assert len(ci) == 0
    with pytest.raises(oracle.OracleError) as err:
        oracle.spgemm_coo((3, 4), [0], [4], np.ones(1), (4, 5), [0], [0], np.ones(1))
    assert err.value.code == oracle.ERR_COORD_RANGE
    with pytest.raises(oracle.OracleError) as err:
        oracle.spgemm_coo((3, 4), [0], [0], np.ones(1), (4, 5), [4], [0], np.ones(1))
    assert err.value.code == oracle.ERR_COORD_RANGE


def test_density_of_the_product_as_the_paper_prints_it():
    """The paper's table gives the density of C for uniform random operands of density 0.01; the realised density of the
    checker's result on the same kind of input rounds to the printed figure (n = 8192 is left to the GPU-side test:
    the dense accumulator of the checker takes 1.7 GB there)."""
    fix = json.load(open(os.path.join(GOLDEN, "spmspm_density_table.json")))
    for row in fix["rows"]:
        n = row["n"]
        if n > 4096:
            continue
        a, b = pair(n, n, n, int(round(fix["density_ab"] * n * n)), int(round(fix["density_ab"] * n * n)), seed=n)
        ci, _, _, _ = oracle.spgemm_coo(a.shape, a.rows, a.cols, a.vals, b.shape, b.rows, b.cols, b.vals)
        rho = len(ci) / float(n * n)
        assert abs(rho - row["density_c"]) <= 0.006, (n, rho)
        assert abs(rho - (1.0 - (1.0 - fix["density_ab"] ** 2) ** n)) <= 0.002, (n, rho)   # 1 - (1 - rho^2)^n for independent entries
