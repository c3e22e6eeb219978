"""GPU MTTKRP (Section 6.3) against the CPU checker, through the C ABI.

Tolerance as for the other products: 1e-12 (f64) / 1e-5 (f32) times the sum of the absolute values of the terms of an
output element; small-integer inputs bit for bit.  The rank-3 storage the kernel walks is compared with the checker's
bit for bit first.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_04305_amd as sp
from gen import workloads as W, prng
from gpu_util import say, dev, gpu_pack, assert_storage_equal, assert_product_close, DEV

pytestmark = pytest.mark.gpu

ORDERS = [(0, 1, 2), (0, 2, 1)]
LEVELS = [(0, 1, 1), (1, 1, 1)]


def small_tensor(dtype=np.float64, J=42):
    # slices from 1 entry to several windows of the kernel, fibres from 1 to a few hundred entries
    return W.tensor3_slices(I=300, K=400, L=900, nnz=260_000, k_mean=60, l_mean=150, sigma=1.3, J=J, dtype=dtype)


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("lt", LEVELS)
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_mttkrp_formats_of_the_experiment(order, lt, dtype):
    w = small_tensor(dtype)
    C, D = w.factors()
    say("case mttkrp", order, lt, dtype.__name__, w.stats)
    B = gpu_pack(lt, order, w.shape, [w.ci, w.ck, w.cl], w.vals)
    assert_storage_equal(B, oracle.pack(lt, order, w.shape, [w.ci, w.ck, w.cl], w.vals, 32, 32))
    ref, mag = oracle.mttkrp_coo(w.shape, w.ci, w.ck, w.cl, w.vals, C, D)
    A = torch.full((w.shape[0], w.J), float("nan"), dtype=B.dtype, device=DEV)
    sp.sp_mttkrp(B, dev(C), dev(D), A)
    assert_product_close(A, ref, mag, dtype, "mttkrp")
    A2 = torch.full_like(A, float("nan"))
    sp.sp_mttkrp(B, dev(C), dev(D), A2)
    assert torch.equal(A, A2), "not reproducible"


@pytest.mark.parametrize("J", [1, 2, 3, 5, 8, 16, 31, 42, 64, 70, 128, 130, 200])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_mttkrp_widths(J, dtype):
    w = W.tensor3_slices(I=120, K=90, L=200, nnz=40_000, k_mean=25, l_mean=60, sigma=1.2, J=J, dtype=dtype)
    C, D = w.factors()
    say("case mttkrp J", J, dtype.__name__)
    ref, mag = oracle.mttkrp_coo(w.shape, w.ci, w.ck, w.cl, w.vals, C, D)
    for order in ORDERS:
        B = gpu_pack((0, 1, 1), order, w.shape, [w.ci, w.ck, w.cl], w.vals)
        A = sp.sp_mttkrp(B, dev(C), dev(D))
        assert_product_close(A, ref, mag, dtype, "mttkrp J=%d" % J)


def test_mttkrp_exact_integers_widths_64_accumulate_and_leading_dimensions():
    w = small_tensor(J=10)
    C, D = w.factors(exact=True)
    vals = w.exact_values()
    ref, _ = oracle.mttkrp_coo(w.shape, w.ci, w.ck, w.cl, vals, C, D)
    I, K, L = w.shape
    for pw, cw in [(32, 32), (64, 32), (32, 64), (64, 64)]:
        for order in ORDERS:
            say("case mttkrp exact", pw, cw, order)
            B = gpu_pack((0, 1, 1), order, w.shape, [w.ci, w.ck, w.cl], vals, pw, cw)
            A = sp.sp_mttkrp(B, dev(C), dev(D))
            assert np.array_equal(A.cpu().numpy(), ref)
    # accumulate into a wider buffer; factor matrices with padding columns (odd leading dimensions: the scalar path)
    B = gpu_pack((0, 1, 1), (0, 1, 2), w.shape, [w.ci, w.ck, w.cl], vals)
    Cw = torch.full((K, 13), 99.0, dtype=torch.float64, device=DEV)
    Dw = torch.full((L, 11), 99.0, dtype=torch.float64, device=DEV)
    Cw[:, :10] = dev(C)
    Dw[:, :10] = dev(D)
    A0 = prng.small_ints(8, 1, I * 15).reshape(I, 15)
    Aw = dev(A0)
    sp.sp_mttkrp(B, Cw[:, :10], Dw[:, :10], Aw[:, :10], accumulate=True)
    exp = A0.copy()
    exp[:, :10] += ref
    assert np.array_equal(Aw.cpu().numpy(), exp)
    # overwrite: rows of empty slices become zero, the padding columns stay
    Aw = torch.full((I, 15), 7.0, dtype=torch.float64, device=DEV)
    sp.sp_mttkrp(B, Cw[:, :10], Dw[:, :10], Aw[:, :10])
    exp = np.full((I, 15), 7.0)
    exp[:, :10] = ref
    assert np.array_equal(Aw.cpu().numpy(), exp)


def test_mttkrp_one_slice_longer_than_many_windows_and_empty_slices():
    # every entry in slice 5 of 9: the carries of one slice span all windows; the other rows must come out zero
    n = 30_000
    _, lin = W.distinct_sorted_per_segment(W.BASE_SEED + 50, 1, np.array([n], dtype=np.int64), 700 * 800)
    p = prng.permutation(W.BASE_SEED + 50, 2, n)
    ck, cl = (lin // 800)[p], (lin % 800)[p]
    ci = np.full(n, 5, dtype=np.int64)
    vals = prng.uniform_pm1(W.BASE_SEED + 50, 3, n)
    C = prng.uniform_pm1(W.BASE_SEED + 50, 4, 700 * 42).reshape(700, 42)
    D = prng.uniform_pm1(W.BASE_SEED + 50, 5, 800 * 42).reshape(800, 42)
    ref, mag = oracle.mttkrp_coo((9, 700, 800), ci, ck, cl, vals, C, D)
    for lt in LEVELS:
        for order in ORDERS:
            say("case mttkrp one slice", lt, order)
            B = gpu_pack(lt, order, (9, 700, 800), [ci, ck, cl], vals)
            A = torch.full((9, 42), float("nan"), dtype=torch.float64, device=DEV)
            sp.sp_mttkrp(B, dev(C), dev(D), A)
            assert_product_close(A, ref, mag, np.float64, "one slice")
            assert np.all(A.cpu().numpy()[[0, 1, 2, 3, 4, 6, 7, 8]] == 0.0)


def test_mttkrp_factor_matrices_beyond_the_l2_size():
    """Inner factor matrices of more than 4 MB whose rows do not start on cache lines are gathered from a padded copy."""
    w = W.tensor3_slices(I=40, K=13000, L=13500, nnz=120_000, k_mean=300, l_mean=400, sigma=1.0, J=42)
    C, D = w.factors()
    ref, mag = oracle.mttkrp_coo(w.shape, w.ci, w.ck, w.cl, w.vals, C, D)
    Cd, Dd = dev(C), dev(D)
    for order in ORDERS:
        say("case mttkrp large factors", order)
        B = gpu_pack((0, 1, 1), order, w.shape, [w.ci, w.ck, w.cl], w.vals)
        A = sp.sp_mttkrp(B, Cd, Dd)
        assert_product_close(A, ref, mag, np.float64, "mttkrp large factors")
        A2 = sp.sp_mttkrp(B, Cd, Dd)                    # second call: the kept buffer is reused
        assert torch.equal(A, A2)
        # the caller's matrices are untouched
        assert np.array_equal(Cd.cpu().numpy(), C) and np.array_equal(Dd.cpu().numpy(), D)


def test_mttkrp_degenerate_and_unsupported():
    C = torch.ones((3, 4), dtype=torch.float64, device=DEV)
    D = torch.ones((5, 4), dtype=torch.float64, device=DEV)
    e = [np.zeros(0, dtype=np.int64)] * 3
    B = gpu_pack((0, 1, 1), (0, 1, 2), (2, 3, 5), e, np.zeros(0))
    A = torch.full((2, 4), 3.0, dtype=torch.float64, device=DEV)
    sp.sp_mttkrp(B, C, D, A)
    assert torch.equal(A, torch.zeros_like(A))
    one = gpu_pack((0, 1, 1), (0, 1, 2), (2, 3, 5), [np.array([1]), np.array([2]), np.array([4])], np.array([2.5]))
    A = sp.sp_mttkrp(one, C, D)
    assert np.array_equal(A.cpu().numpy(), np.array([[0.0] * 4, [2.5] * 4]))
    for lt, order in [((0, 0, 1), (0, 1, 2)), ((0, 1, 0), (0, 1, 2)), ((0, 1, 1), (1, 0, 2)), ((1, 1, 1), (2, 1, 0))]:
        T = gpu_pack(lt, order, (2, 3, 5), [np.array([1]), np.array([2]), np.array([4])], np.array([2.5]))
        with pytest.raises(sp.SpError) as err:
            sp.sp_mttkrp(T, C, D)
        assert err.value.code == 10           # SP_ERR_UNSUPPORTED
        # the paper's remedy: convert to a supported format, then multiply
        T2 = sp.sp_convert(T, sp.sp_encode((0, 1, 1), (0, 1, 2), 32, 32))
        assert np.array_equal(sp.sp_mttkrp(T2, C, D).cpu().numpy(), np.array([[0.0] * 4, [2.5] * 4]))
    M = gpu_pack((0, 1), (0, 1), (4, 4), [np.array([1]), np.array([2])], np.array([1.0]))
    with pytest.raises(sp.SpError) as err:
        sp.sp_mttkrp(M, C, D)
    assert err.value.code == 2                # SP_ERR_RANK
