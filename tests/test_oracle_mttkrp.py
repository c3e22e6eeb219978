"""Pins for the CPU checker's MTTKRP, A[i,j] = B[i,k,l] * D[l,j] * C[k,j] (Section 6.3).  No GPU needed."""
import numpy as np
import pytest

import oracle
from gen import workloads as W, prng


def _dense(w):
    T = np.zeros(w.shape, dtype=np.float64)
    T[w.ci, w.ck, w.cl] = w.vals
    return T


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("J", [1, 5, 42])
def test_against_einsum_on_the_dense_tensor(dtype, J):
    w = W.tensor3_uniform(7, 5, 9, 120, J=J, dtype=dtype)
    C, D = w.factors()
    A, mag = oracle.mttkrp_coo(w.shape, w.ci, w.ck, w.cl, w.vals, C, D)
    T = _dense(w)
    ref = np.einsum("ikl,lj,kj->ij", T, D.astype(np.float64), C.astype(np.float64))
    refmag = np.einsum("ikl,lj,kj->ij", np.abs(T), np.abs(D.astype(np.float64)), np.abs(C.astype(np.float64)))
    tol = 4e-16 if dtype == np.float64 else 1e-7
    assert A.dtype == dtype and A.shape == (7, J)
    assert np.all(np.abs(A - ref) <= tol * refmag + 1e-300)
    assert np.allclose(mag, refmag, rtol=1e-12, atol=0)


def test_matricized_form_with_the_khatri_rao_product():
    """A = B_(1) . (C khatri-rao D) with the mode-1 unfolding B_(1)[i, k*L + l]: K != L, so swapping the roles of C
    and D, or of k and l, cannot pass."""
    w = W.tensor3_uniform(6, 4, 11, 150, J=3)
    C, D = w.factors()
    I, K, L = w.shape
    kr = (C[:, None, :] * D[None, :, :]).reshape(K * L, 3)
    ref = _dense(w).reshape(I, K * L) @ kr
    A, _ = oracle.mttkrp_coo(w.shape, w.ci, w.ck, w.cl, w.vals, C, D)
    assert np.allclose(A, ref, rtol=0, atol=1e-13)


def test_closed_forms():
    I, K, L, J = 4, 3, 5, 2
    ii, kk, ll = [x.ravel() for x in np.meshgrid(np.arange(I), np.arange(K), np.arange(L), indexing="ij")]
    ones = np.ones(I * K * L)
    A, mag = oracle.mttkrp_coo((I, K, L), ii, kk, ll, ones, np.ones((K, J)), np.ones((L, J)))
    assert np.array_equal(A, np.full((I, J), float(K * L))) and np.array_equal(mag, A)
    # rank-one tensor u x v x w: A[i,j] = u[i] * (v . C[:,j]) * (w . D[:,j])
    u, v, x = prng.uniform_pm1(5, 1, I), prng.uniform_pm1(5, 2, K), prng.uniform_pm1(5, 3, L)
    C = prng.uniform_pm1(5, 4, K * J).reshape(K, J)
    D = prng.uniform_pm1(5, 5, L * J).reshape(L, J)
    A, _ = oracle.mttkrp_coo((I, K, L), ii, kk, ll, u[ii] * v[kk] * x[ll], C, D)
    assert np.allclose(A, np.outer(u, (v @ C) * (x @ D)), rtol=0, atol=1e-14)
    # one entry: a single product, in the paper's order of the factors
    A, mag = oracle.mttkrp_coo((I, K, L), [2], [1], [4], np.array([0.3]), C, D)
    ref = np.zeros((I, J))
    ref[2] = 0.3 * D[4] * C[1]
    assert np.allclose(A, ref, rtol=2.3e-16, atol=0) and np.allclose(mag, np.abs(ref), rtol=2.3e-16, atol=0)


def test_reduces_to_matrix_times_vector():
    """L = 1 and J = 1: A[i] = sum_k B[i,k,0] * C[k] * D[0], the checker's own matrix product up to the scalar."""
    w = W.uniform_random(30, 40, 300)
    x = prng.uniform_pm1(6, 1, 40)
    A, mag = oracle.mttkrp_coo((30, 40, 1), w.rows, w.cols, np.zeros(w.nnz, dtype=np.int64), w.vals, x.reshape(40, 1), np.array([[2.0]]))
    y, ymag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, x)
    assert np.allclose(A, 2.0 * y, rtol=4e-16, atol=0) and np.allclose(mag, 2.0 * ymag, rtol=4e-16, atol=0)


def test_exact_integers_any_order_and_accumulate():
    w = W.tensor3_uniform(9, 8, 7, 200, J=4)
    C, D = w.factors(exact=True)
    vals = w.exact_values()
    A, _ = oracle.mttkrp_coo(w.shape, w.ci, w.ck, w.cl, vals, C, D)
    p = prng.permutation(9, 1, w.nnz)
    A2, _ = oracle.mttkrp_coo(w.shape, w.ci[p], w.ck[p], w.cl[p], vals[p], C, D)
    assert np.array_equal(A, A2)
    T = np.zeros(w.shape)
    T[w.ci, w.ck, w.cl] = vals
    assert np.array_equal(A, np.einsum("ikl,lj,kj->ij", T, D, C))
    A0 = prng.small_ints(9, 2, 9 * 4).reshape(9, 4)
    A3, _ = oracle.mttkrp_coo(w.shape, w.ci, w.ck, w.cl, vals, C, D, accumulate=True, A=A0)
    assert np.array_equal(A3, A0 + A)


def test_errors_and_empty():
    C, D = np.ones((3, 2)), np.ones((4, 2))
    A, mag = oracle.mttkrp_coo((2, 3, 4), [], [], [], np.zeros(0), C, D)
    assert np.array_equal(A, np.zeros((2, 2))) and np.array_equal(mag, np.zeros((2, 2)))
    for bad in ([2], [0], [0]), ([0], [3], [0]), ([0], [0], [4]), ([-1], [0], [0]):
        with pytest.raises(oracle.OracleError) as e:
            oracle.mttkrp_coo((2, 3, 4), bad[0], bad[1], bad[2], np.ones(1), C, D)
        assert e.value.code == oracle.ERR_COORD_RANGE


def test_storage_walk_agrees_for_both_orders_of_the_experiment():
    """Packing under (dense, compressed, compressed) with either inner order and walking the storage back gives the
    same product: ties the rank-3 storage to the kernel's definition."""
    w = W.tensor3_slices(I=40, K=30, L=50, nnz=3000, k_mean=10, l_mean=20, J=6)
    C, D = w.factors()
    ref, mag = oracle.mttkrp_coo(w.shape, w.ci, w.ck, w.cl, w.vals, C, D)
    for order in [(0, 1, 2), (0, 2, 1)]:
        for lt in [(0, 1, 1), (1, 1, 1)]:
            P = oracle.pack(lt, order, w.shape, [w.ci, w.ck, w.cl], w.vals)
            (ci, ck, cl), vals = P.unpack()
            assert vals.shape[0] == w.nnz
            A, _ = oracle.mttkrp_coo(w.shape, ci, ck, cl, vals, C, D)
            assert np.all(np.abs(A - ref) <= 4e-16 * mag)
