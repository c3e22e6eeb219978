"""GPU sampled dense-dense product against the CPU checker, through the C ABI.

The GPU returns one value per stored position in storage order; the expected values are the checker's per-triple
results packed by the checker under the same encoding.  Tolerance as for the products: 1e-12 (f64) / 1e-5 (f32) times
|s| * sum|a*b| per entry; small-integer inputs bit for bit.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_04305_amd as sp
from gen import workloads as W, prng
from gpu_util import say, dev, gpu_pack, tol_for, DEV

pytestmark = pytest.mark.gpu


def expected(w, lt, A, B, vals=None):
    vals = w.vals if vals is None else vals
    x, mag = oracle.sddmm_coo(w.shape, w.rows, w.cols, vals, A, B)
    xs = oracle.pack(lt, (0, 1), w.shape, [w.rows, w.cols], x, 32, 32).values
    ms = oracle.pack(lt, (0, 1), w.shape, [w.rows, w.cols], mag, 32, 32).values
    return xs, ms


@pytest.mark.parametrize("lt", [(0, 1), (1, 1)])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("K", [1, 2, 7, 16, 64, 100, 128])
def test_sddmm(lt, dtype, K):
    w = W.cfg2_powerlaw_csr(3000, 2500, cap=900)
    w.vals = w.vals.astype(dtype)
    m, n = w.shape
    A = prng.uniform_pm1(6, 1, m * K, dtype=dtype).reshape(m, K)
    B = prng.uniform_pm1(6, 2, K * n, dtype=dtype).reshape(K, n)
    say("case sddmm", lt, dtype.__name__, "K", K)
    S = gpu_pack(lt, (0, 1), w.shape, [w.rows, w.cols], w.vals)
    xs, ms = expected(w, lt, A, B)
    for transposed in (False, True):
        Bd = dev(np.ascontiguousarray(B.T)) if transposed else dev(B)
        X = torch.full((w.nnz,), float("nan"), dtype=S.dtype, device=DEV)
        sp.sp_sddmm(S, dev(A), Bd, X, b_is_transposed=transposed)
        err = np.abs(X.cpu().numpy().astype(np.float64) - xs.astype(np.float64))
        assert np.all(err <= tol_for(dtype) * ms), (transposed, float(np.max(err / np.maximum(ms, 1e-300))))


def test_sddmm_exact_integers_and_mostly_empty_rows():
    w = W.cfg4_hypersparse_dcsr(1 << 15, 1 << 12, frac=0.03, per_row=40)       # CSR with mostly empty rows too
    m, n = w.shape
    K = 24
    A = prng.small_ints(6, 3, m * K).reshape(m, K)
    B = prng.small_ints(6, 4, K * n).reshape(K, n)
    si = w.exact_values()
    for lt in [(0, 1), (1, 1)]:
        say("case sddmm exact", lt)
        S = gpu_pack(lt, (0, 1), w.shape, [w.rows, w.cols], si)
        xs, _ = expected(w, lt, A, B, vals=si)
        X = sp.sp_sddmm(S, dev(A), dev(B))
        assert np.array_equal(X.cpu().numpy(), xs)


def test_sddmm_errors_and_degenerate():
    w = W.uniform_random(50, 40, 300)
    S = gpu_pack((0, 1), (1, 0), w.shape, [w.rows, w.cols], w.vals)            # column-major: not on this path
    with pytest.raises(sp.SpError) as e:
        sp.sp_sddmm(S, torch.ones((50, 4), dtype=torch.float64, device=DEV), torch.ones((4, 40), dtype=torch.float64, device=DEV))
    assert e.value.code == oracle.ERR_UNSUPPORTED
    S = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals)
    L = sp.load_library()
    A = torch.ones((50, 4), dtype=torch.float64, device=DEV)
    B = torch.ones((4, 40), dtype=torch.float64, device=DEV)
    X = torch.empty(300, dtype=torch.float64, device=DEV)
    assert L.sp_sddmm(S._h, A.data_ptr(), 3, B.data_ptr(), 40, 0, 4, X.data_ptr(), None) == oracle.ERR_SHAPE
    assert L.sp_sddmm(S._h, A.data_ptr(), 4, B.data_ptr(), 39, 0, 4, X.data_ptr(), None) == oracle.ERR_SHAPE
    z = np.zeros(0, dtype=np.int64)
    E = gpu_pack((0, 1), (0, 1), (50, 40), [z, z], np.zeros(0))
    assert sp.sp_sddmm(E, A, B).numel() == 0


def test_sddmm_with_64_bit_coordinates():
    w = W.cfg2_powerlaw_csr(3000, 2500, cap=900)
    m, n = w.shape
    K = 32
    A = prng.uniform_pm1(6, 8, m * K).reshape(m, K)
    B = prng.uniform_pm1(6, 9, K * n).reshape(K, n)
    x, mag = oracle.sddmm_coo(w.shape, w.rows, w.cols, w.vals, A, B)
    for pw, cw in [(32, 64), (64, 64)]:
        say("case sddmm 64-bit crd", pw, cw)
        S = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals, pw, cw)
        xs = oracle.pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], x, pw, cw).values
        ms = oracle.pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], mag, pw, cw).values
        X = sp.sp_sddmm(S, dev(A), dev(B))
        assert np.all(np.abs(X.cpu().numpy() - xs) <= 1e-12 * ms)
