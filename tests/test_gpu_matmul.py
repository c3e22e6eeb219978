"""GPU sparse x dense products against the CPU checker, element by element, through the C ABI.

Tolerance (stated with the target): |C_gpu - C_ref| <= 1e-12 * sum|a*b| for f64, 1e-5 * sum|a*b| for f32;
exact-integer inputs must match bit for bit whatever the summation order.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_04305_amd as sp
from gen import workloads as W, prng
from gpu_util import say, dev, gpu_pack, assert_product_close, DEV

pytestmark = pytest.mark.gpu


def run(A, w, B, accumulate=False, C0=None, vals=None):
    m = w.shape[0]
    Bn = np.ascontiguousarray(B, dtype=w.dtype).reshape(w.shape[1], -1)
    N = Bn.shape[1]
    if C0 is None:
        C = torch.full((m, N), float("nan"), dtype=A.dtype, device=DEV)      # overwrite mode must not read C
    else:
        C = dev(np.ascontiguousarray(C0, dtype=w.dtype).reshape(m, N))
    sp.sp_matmul(A, dev(Bn), C, accumulate=accumulate)
    ref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals if vals is None else vals, Bn, accumulate, C0)
    torch.cuda.synchronize()
    return C, ref, mag


SPMV_CASES = [
    ("cfg1 full", lambda: W.cfg1_uniform_csr()),
    ("cfg2 scaled, rows cross several blocks", lambda: W.cfg2_powerlaw_csr(40000, 30000, mean=24.0, cap=9000)),
    ("long rows only", lambda: W.cfg2_powerlaw_csr(64, 20000, mean=6000.0, sigma=0.3, cap=15000)),
    ("ragged tail, one block and a bit", lambda: W.cfg2_powerlaw_csr(300, 500, mean=8.0, cap=200)),
    ("many empty rows as CSR", lambda: W.cfg4_hypersparse_dcsr(1 << 17, 1 << 17, frac=0.02, per_row=40)),
]


@pytest.mark.parametrize("name,maker", SPMV_CASES)
@pytest.mark.parametrize("kernel", [0, 1, 2])
@pytest.mark.parametrize("widths", [(32, 32), (64, 64)])
def test_csr_spmv(name, maker, kernel, widths):
    w = maker()
    say("case spmv", name, "kernel", kernel, widths, w.stats)
    A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals, *widths)
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, kernel)
    x = w.dense_operand(1)
    y, ref, mag = run(A, w, x)
    assert_product_close(y, ref, mag, w.dtype, name)
    y0 = prng.uniform_pm1(5, 5, w.shape[0])
    y, ref, mag = run(A, w, x, accumulate=True, C0=y0)
    assert_product_close(y, ref, mag, w.dtype, name + " accumulate")


WIDE_CASES = [
    ("wide, 3 column panels", lambda: W.cfg2_powerlaw_csr(50000, 600000, mean=24.0, cap=9000)),
    ("wide, rows crossing several blocks inside a panel", lambda: W.cfg2_powerlaw_csr(64, 600000, mean=20000.0, sigma=0.3, cap=60000)),
    ("wide, many empty rows", lambda: W.cfg4_hypersparse_dcsr(1 << 19, 1 << 19, frac=0.05, per_row=40)),
]


@pytest.mark.parametrize("name,maker", WIDE_CASES)
@pytest.mark.parametrize("widths", [(32, 32), (64, 64)])
def test_csr_spmv_column_segmented(name, maker, widths):
    """Kernel 3 (x gathered from L2-sized column panels; rows that cross blocks are completed from per-block carries in
    block order, no atomics: the same bits on every call)."""
    w = maker()
    say("case segmented spmv", name, widths, w.stats)
    A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals, *widths)
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, 3)
    x = w.dense_operand(1)
    y, ref, mag = run(A, w, x)
    assert_product_close(y, ref, mag, w.dtype, name)
    y0 = prng.uniform_pm1(5, 5, w.shape[0])
    y, ref, mag = run(A, w, x, accumulate=True, C0=y0)
    assert_product_close(y, ref, mag, w.dtype, name + " accumulate")
    # exact integers: the order of the additions cannot matter
    vals = w.exact_values()
    A2 = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], vals, *widths)
    sp.sp_tensor_tune(A2, sp.SP_TUNE_SPMV_KERNEL, 3)
    y, ref, mag = run(A2, w, w.dense_operand(1, exact=True), vals=vals)
    assert np.array_equal(y.cpu().numpy(), ref)


def test_csr_spmv_column_segmented_empty_first_panel_and_fallback():
    w = W.cfg2_powerlaw_csr(20000, 300000, mean=10.0, cap=2000)
    w.cols = w.cols + 300000            # every entry in the upper panels of a 600000-column matrix
    w.shape = (20000, 600000)
    say("case segmented, empty first panel")
    A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals)
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, 3)
    y, ref, mag = run(A, w, w.dense_operand(1))
    assert_product_close(y, ref, mag, w.dtype, "empty first panel")
    say("case segmented, x too small for panels")
    w2 = W.cfg2_powerlaw_csr(3000, 3000, cap=500)
    A2 = gpu_pack((0, 1), (0, 1), w2.shape, [w2.rows, w2.cols], w2.vals)
    sp.sp_tensor_tune(A2, sp.SP_TUNE_SPMV_KERNEL, 3)
    with pytest.raises(sp.SpError) as e:
        sp.sp_matmul(A2, dev(w2.dense_operand(1)), torch.empty(3000, dtype=torch.float64, device=DEV))
    assert e.value.code == oracle.ERR_UNSUPPORTED


BINNED_CASES = SPMV_CASES + WIDE_CASES + [
    ("one entry", lambda: W.uniform_random(5, 9, 1)),
    ("last panel and last row block ragged", lambda: W.cfg2_powerlaw_csr(2048 * 3 + 1, 8192 * 2 + 1, mean=30.0, cap=5000)),
]


@pytest.mark.parametrize("name,maker", BINNED_CASES)
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_csr_spmv_binned(name, maker, dtype):
    """Kernel 4: entries regrouped by (column panel, row block), products through an LDS slice of x, sums in an LDS slice
    of y with atomic adds: within tolerance, and bit for bit on exact integers."""
    w = maker()
    w.vals = w.vals.astype(dtype)
    w.dtype = dtype
    widths = (32, 32) if dtype is np.float64 else (64, 32)
    say("case binned spmv", name, dtype.__name__, w.stats)
    A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals, *widths)
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, 4)
    x = w.dense_operand(1).astype(dtype)
    y, ref, mag = run(A, w, x)
    assert_product_close(y, ref, mag, dtype, name)
    y0 = prng.uniform_pm1(5, 5, w.shape[0]).astype(dtype)
    y, ref, mag = run(A, w, x, accumulate=True, C0=y0)
    assert_product_close(y, ref, mag, dtype, name + " accumulate")
    if dtype is np.float64:
        vals = w.exact_values()
        A2 = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], vals, *widths)
        sp.sp_tensor_tune(A2, sp.SP_TUNE_SPMV_KERNEL, 4)
        y, ref, mag = run(A2, w, w.dense_operand(1, exact=True), vals=vals)
        assert np.array_equal(y.cpu().numpy(), ref)


def test_csr_spmv_binned_random_shapes():
    """Seeded random shapes and fills for kernel 4: from a single bucket to hundreds, buckets that are empty, last panel and
    last row block of every raggedness, CSR and DCSR, both value types; small integers, so every sum is exact."""
    rng = np.random.default_rng(4305)
    for it in range(24):
        m = int(rng.integers(1, 9000))
        n = int(rng.integers(1, 70000))
        nnz = int(min(m * n, rng.integers(1, 60000)))
        lt = (int(rng.integers(0, 2)), 1)
        dtype = np.float64 if it % 2 == 0 else np.float32
        w = W.uniform_random(m, n, nnz, dtype=dtype, seed=W.BASE_SEED + 700 + it)
        vals = prng.small_ints(11, it, nnz, dtype=dtype)
        x = prng.small_ints(12, it, n, dtype=dtype).reshape(n, 1)
        say("case binned random", it, (m, n), nnz, lt, dtype.__name__)
        A = gpu_pack(lt, (0, 1), w.shape, [w.rows, w.cols], vals, 32, 32)
        sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, 4)
        ref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, vals, x)
        y = torch.full((m,), float("nan"), dtype=A.dtype, device=DEV)
        try:
            sp.sp_matmul(A, dev(x[:, 0].copy()), y)
        except sp.SpError as e:                      # more buckets than entries (+ 4096): refused, not wrong
            assert e.code == oracle.ERR_UNSUPPORTED
            assert -(-n // 8192) * -(-m // 2048) > nnz + 4096 or lt[0] == 1
            continue
        assert np.array_equal(y.cpu().numpy().astype(np.float64), ref[:, 0])


def test_csr_spmv_binned_padding_is_inert():
    """The binned copy pads every bucket to a multiple of 8 entries.  The padding must give exactly 0 whatever x holds: with
    infinities and NaNs in some columns, the rows that store none of those columns stay finite and exact."""
    w = W.cfg2_powerlaw_csr(5000, 40000, mean=10.0, cap=700)
    vals = prng.small_ints(21, 1, w.nnz)
    A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], vals)
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, 4)
    x = prng.small_ints(22, 2, w.shape[1])
    bad_cols = np.array([0, 1, 8191, 8192, 16384, 39999])          # first and last columns of panels among them
    xb = x.copy()
    xb[bad_cols] = [np.inf, np.nan, -np.inf, np.nan, np.inf, np.nan]
    y = torch.full((w.shape[0],), 7.0, dtype=torch.float64, device=DEV)
    sp.sp_matmul(A, dev(xb), y)
    ref, _ = oracle.matmul_coo(w.shape, w.rows, w.cols, vals, x.reshape(-1, 1))
    touched = np.zeros(w.shape[0], dtype=bool)
    touched[w.rows[np.isin(w.cols, bad_cols)]] = True
    got = y.cpu().numpy()
    assert touched.any() and not touched.all()
    assert np.array_equal(got[~touched], ref[~touched, 0])
    assert not np.isfinite(got[touched]).all()


def test_csr_spmv_binned_strides_and_refusals():
    w = W.cfg2_powerlaw_csr(3000, 20000, mean=12.0, cap=900)
    A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals)
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, 4)
    say("case binned, strided x and y")
    x = w.dense_operand(1)
    xs = torch.zeros((20000, 3), dtype=torch.float64, device=DEV)
    xs[:, 0] = dev(x[:, 0].copy())
    ys = torch.full((3000, 2), -7.0, dtype=torch.float64, device=DEV)
    sp.sp_matmul(A, xs, ys, N=1, ldb=3, ldc=2)
    ref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, x)
    assert_product_close(ys[:, 0].contiguous(), ref, mag, np.float64, "strided binned spmv")
    assert torch.all(ys[:, 1] == -7.0)
    say("case binned, a huge and mostly empty matrix: only the non-empty rows are binned")
    T = gpu_pack((0, 1), (0, 1), (1 << 22, 1 << 22), [w.rows, w.cols], w.vals)
    sp.sp_tensor_tune(T, sp.SP_TUNE_SPMV_KERNEL, 4)
    xb = prng.uniform_pm1(5, 9, 1 << 22)
    yb = torch.full((1 << 22,), float("nan"), dtype=torch.float64, device=DEV)
    sp.sp_matmul(T, dev(xb), yb)
    ref, mag = oracle.matmul_coo((1 << 22, 1 << 22), w.rows, w.cols, w.vals, xb.reshape(-1, 1))
    assert_product_close(yb, ref, mag, np.float64, "huge and mostly empty")
    say("case binned, empty / bucket table larger than the tensor")
    for lt, shape, coords, vals in [
        ((0, 1), (50, 60), [np.zeros(0, dtype=np.int64)] * 2, np.zeros(0)),
        ((0, 1), (3000, 1 << 26), [w.rows[:200], w.cols[:200]], w.vals[:200]),     # 8192 column panels for 200 entries
    ]:
        T = gpu_pack(lt, (0, 1), shape, coords, vals)
        sp.sp_tensor_tune(T, sp.SP_TUNE_SPMV_KERNEL, 4)
        if len(vals) == 0:                                # nothing stored: nothing to bin, the product is zero
            y = torch.full((shape[0],), float("nan"), dtype=torch.float64, device=DEV)
            try:
                sp.sp_matmul(T, torch.ones(shape[1], dtype=torch.float64, device=DEV), y)
                assert torch.all(y == 0)
            except sp.SpError as e:
                assert e.code == oracle.ERR_UNSUPPORTED
            continue
        with pytest.raises(sp.SpError) as e:
            sp.sp_matmul(T, torch.ones(shape[1], dtype=torch.float64, device=DEV), torch.empty(shape[0], dtype=torch.float64, device=DEV))
        assert e.value.code == oracle.ERR_UNSUPPORTED


@pytest.mark.parametrize("kernel", [0, 1, 2, 3, 4])
def test_csr_spmv_long_run_of_empty_rows(kernel):
    """Most rows hold entries, but 100,000 consecutive ones hold none (and, for the column-segmented copy, a whole column
    panel is empty): one window of the streaming kernels must not be left to walk over all of them."""
    w = W.cfg2_powerlaw_csr(200000, 300000, mean=10.0, cap=2000)
    w.rows = w.rows + 100000
    w.cols = w.cols + 300000
    w.shape = (300000, 600000)
    say("case long run of empty rows, kernel", kernel)
    A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals)
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, kernel)
    x = w.dense_operand(1)
    y, ref, mag = run(A, w, x)
    assert_product_close(y, ref, mag, w.dtype, "empty run")
    assert torch.all(y[:100000] == 0)
    y0 = prng.uniform_pm1(5, 5, w.shape[0])
    y, ref, mag = run(A, w, x, accumulate=True, C0=y0)
    assert_product_close(y, ref, mag, w.dtype, "empty run, accumulate")


@pytest.mark.parametrize("kernel", [1, 2])
def test_exact_integer_inputs_bit_exact(kernel):
    w = W.cfg2_powerlaw_csr(30000, 30000, mean=20.0, cap=7000)
    vals = w.exact_values()
    say("case exact ints kernel", kernel)
    A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], vals)
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, kernel)
    x = w.dense_operand(1, exact=True)
    y, ref, mag = run(A, w, x, vals=vals)
    assert np.array_equal(y.cpu().numpy(), ref)
    # all-ones: y[i] = row length = pos[i+1] - pos[i]
    ones = np.ones(w.nnz)
    A1 = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], ones)
    sp.sp_tensor_tune(A1, sp.SP_TUNE_SPMV_KERNEL, kernel)
    y = torch.empty(w.shape[0], dtype=torch.float64, device=DEV)
    sp.sp_matmul(A1, dev(np.ones(w.shape[1])), y)
    pos = sp.sp_pos(A1, 1).cpu().numpy()
    assert np.array_equal(y.cpu().numpy(), np.diff(pos).astype(np.float64))


@pytest.mark.parametrize("kernel", [1, 2])
def test_spmv_is_reproducible_run_to_run(kernel):
    w = W.cfg2_powerlaw_csr(30000, 30000, mean=20.0, cap=7000)
    A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals)
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, kernel)
    x = dev(w.dense_operand(1))
    ys = []
    for _ in range(3):
        y = torch.empty(w.shape[0], dtype=torch.float64, device=DEV)
        sp.sp_matmul(A, x, y)
        ys.append(y.cpu().numpy())
    assert np.array_equal(ys[0], ys[1]) and np.array_equal(ys[0], ys[2])


@pytest.mark.parametrize("N", [2, 3, 4, 6, 8, 12, 16, 32, 42, 64, 70, 100, 128, 130, 256, 260])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_csr_spmm(N, dtype):
    w = W.cfg3_powerlaw_csr_spmm(6000, 5000, N=N, cap=2500)
    w.vals = w.vals.astype(dtype)
    w.dtype = dtype
    say("case spmm N", N, dtype.__name__)
    A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals)
    B = w.dense_operand(N)
    C, ref, mag = run(A, w, B)
    assert_product_close(C, ref, mag, dtype, "spmm")
    C0 = prng.uniform_pm1(5, 6, w.shape[0] * N).reshape(-1, N)
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPMM_KERNEL, 1)          # one column per lane, whatever N is
    C, ref, mag = run(A, w, B)
    assert_product_close(C, ref, mag, dtype, "spmm, one column per lane")
    pieces = (N * np.dtype(dtype).itemsize) // 16 if (N * np.dtype(dtype).itemsize) % 16 == 0 else 0
    for kernel in (2, 3):                                     # 16-byte loads, a wave per row / cut by entries: only some N
        sp.sp_tensor_tune(A, sp.SP_TUNE_SPMM_KERNEL, kernel)
        if (pieces in (1, 2, 4, 8, 16, 32, 64)) if kernel == 2 else (1 <= pieces <= 64):
            C, ref, mag = run(A, w, B)
            assert_product_close(C, ref, mag, dtype, "spmm, 16-byte loads, kernel %d" % kernel)
            C, ref, mag = run(A, w, B, accumulate=True, C0=C0)
            assert_product_close(C, ref, mag, dtype, "spmm accumulate, kernel %d" % kernel)
        else:
            with pytest.raises(sp.SpError) as e:
                run(A, w, B)
            assert e.value.code == oracle.ERR_UNSUPPORTED
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPMM_KERNEL, 0)
    C0 = prng.uniform_pm1(5, 6, w.shape[0] * N).reshape(-1, N)
    C, ref, mag = run(A, w, B, accumulate=True, C0=C0)
    assert_product_close(C, ref, mag, dtype, "spmm accumulate")


@pytest.mark.parametrize("N", [1, 5])
@pytest.mark.parametrize("widths", [(32, 32), (64, 32)])
def test_csr_with_mostly_empty_rows(N, widths):
    """A CSR tensor whose rows are mostly empty is multiplied through the list of its non-empty rows; the accessors
    still hand out the plain CSR arrays."""
    w = W.cfg4_hypersparse_dcsr(1 << 16, 1 << 16, frac=0.03, per_row=50)
    say("case csr mostly empty", N, widths, w.stats)
    A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals, *widths)
    ref = oracle.pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals, *widths)
    from gpu_util import assert_storage_equal
    assert_storage_equal(A, ref)
    B = w.dense_operand(N)
    for kernel in (0, 1, 2):
        sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, kernel)
        C, cref, mag = run(A, w, B)
        assert_product_close(C, cref, mag, w.dtype, "mostly empty csr")
        C0 = prng.uniform_pm1(5, 11, w.shape[0] * N).reshape(-1, N)
        C, cref, mag = run(A, w, B, accumulate=True, C0=C0)
        assert_product_close(C, cref, mag, w.dtype, "mostly empty csr accumulate")
        untouched = torch.from_numpy(np.bincount(w.rows, minlength=w.shape[0]) == 0).to(DEV)
        assert torch.equal(C[untouched], dev(C0)[untouched])


@pytest.mark.parametrize("lt", [(0, 1), (1, 1)])
def test_spmm_cut_by_entries_long_rows_and_exact(lt):
    """Rows much longer than a block's window (several carries per row), empty rows between them, CSR and DCSR."""
    w = W.cfg2_powerlaw_csr(400, 30000, mean=3000.0, sigma=1.0, cap=25000)
    w.rows = w.rows * 3                     # two empty rows after every row
    w.shape = (1200, 30000)
    vals = w.exact_values()
    say("case spmm windows", lt, w.stats)
    A = gpu_pack(lt, (0, 1), w.shape, [w.rows, w.cols], vals)
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPMM_KERNEL, 3)
    B = w.dense_operand(8, exact=True)
    C, ref, mag = run(A, w, B, vals=vals)
    assert np.array_equal(C.cpu().numpy(), ref)
    A2 = gpu_pack(lt, (0, 1), w.shape, [w.rows, w.cols], w.vals)
    B2 = w.dense_operand(32)
    for kernel in (0, 3):
        sp.sp_tensor_tune(A2, sp.SP_TUNE_SPMM_KERNEL, kernel)
        C, ref, mag = run(A2, w, B2)
        assert_product_close(C, ref, mag, w.dtype, "spmm windows")
        C0 = prng.uniform_pm1(5, 12, w.shape[0] * 32).reshape(-1, 32)
        C, ref, mag = run(A2, w, B2, accumulate=True, C0=C0)
        assert_product_close(C, ref, mag, w.dtype, "spmm windows accumulate")


def test_leading_dimensions():
    w = W.cfg3_powerlaw_csr_spmm(3000, 2000, N=5, cap=500)
    A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals)
    B = w.dense_operand(5)
    Bp = torch.full((2000, 9), float("nan"), dtype=torch.float64, device=DEV)
    Bp[:, :5] = dev(B)
    Cp = torch.full((3000, 7), -7.0, dtype=torch.float64, device=DEV)
    say("case leading dimensions")
    sp.sp_matmul(A, Bp, Cp, N=5, ldb=9, ldc=7)
    ref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, B)
    assert_product_close(Cp[:, :5].contiguous(), ref, mag, np.float64, "ld")
    assert torch.all(Cp[:, 5:] == -7.0)
    # SpMV on a strided x and y
    xs = torch.zeros((2000, 3), dtype=torch.float64, device=DEV)
    xs[:, 0] = dev(B[:, 0].copy())
    ys = torch.full((3000, 2), -7.0, dtype=torch.float64, device=DEV)
    for kernel in (1, 2):
        sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, kernel)
        sp.sp_matmul(A, xs, ys, N=1, ldb=3, ldc=2)
        ref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, B[:, :1].copy())
        assert_product_close(ys[:, 0].contiguous(), ref, mag, np.float64, "strided spmv")
        assert torch.all(ys[:, 1] == -7.0)


@pytest.mark.parametrize("lt", [(1, 1), (0, 1)])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_spmv_binned_over_stored_rows(lt, dtype):
    """Kernel 4 where not every row is stored: DCSR, and CSR that carries the list of its non-empty rows.  Rows are
    binned by their position among the stored ones; the others must come out as zero (overwrite) or untouched (accumulate)."""
    w = W.cfg4_hypersparse_dcsr(1 << 18, 1 << 18)
    w.vals = w.vals.astype(dtype)
    w.dtype = dtype
    say("case binned over stored rows", lt, dtype.__name__, w.stats)
    A = gpu_pack(lt, (0, 1), w.shape, [w.rows, w.cols], w.vals, 32, 64 if dtype is np.float32 else 32)
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, 4)
    x = w.dense_operand(1).astype(dtype)
    y, ref, mag = run(A, w, x)
    assert_product_close(y, ref, mag, dtype, "binned, stored rows")
    assert torch.all(y[torch.from_numpy(mag[:, 0] == 0).to(DEV)] == 0)
    y0 = prng.uniform_pm1(5, 7, w.shape[0]).astype(dtype)
    y, ref, mag = run(A, w, x, accumulate=True, C0=y0)
    assert_product_close(y, ref, mag, dtype, "binned, stored rows, accumulate")
    untouched = torch.from_numpy(np.bincount(w.rows, minlength=w.shape[0]) == 0).to(DEV)
    assert torch.equal(y[untouched, 0], dev(y0)[untouched])


@pytest.mark.parametrize("kernel", [1, 2])
@pytest.mark.parametrize("N", [1, 4])
def test_dcsr(kernel, N):
    w = W.cfg4_hypersparse_dcsr(1 << 18, 1 << 18)
    say("case dcsr kernel", kernel, "N", N, w.stats)
    A = gpu_pack((1, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals)
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, kernel)
    B = w.dense_operand(N)
    C, ref, mag = run(A, w, B)                       # overwrite: rows that are not stored must come out as zero
    assert_product_close(C, ref, mag, w.dtype, "dcsr")
    assert torch.all(C[torch.from_numpy(mag[:, 0] == 0).to(DEV)] == 0)
    C0 = prng.uniform_pm1(5, 7, w.shape[0] * N).reshape(-1, N)
    C, ref, mag = run(A, w, B, accumulate=True, C0=C0)
    assert_product_close(C, ref, mag, w.dtype, "dcsr accumulate")
    untouched = torch.from_numpy(np.bincount(w.rows, minlength=w.shape[0]) == 0).to(DEV)
    assert torch.equal(C[untouched], dev(C0)[untouched])     # accumulate touches stored rows only


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("lt", [(0, 1), (1, 1)])
@pytest.mark.parametrize("N", [1, 32, 40])
def test_column_major(mode, lt, N):
    w = W.cfg5_zipf_csc_spmm(30000, 30000, N=N, cap=6000)
    say("case csc mode", mode, lt, "N", N, w.stats)
    A = gpu_pack(lt, (1, 0), w.shape, [w.rows, w.cols], w.vals)
    sp.sp_tensor_tune(A, sp.SP_TUNE_CSC_MODE, mode)
    B = w.dense_operand(N)
    C, ref, mag = run(A, w, B)
    assert_product_close(C, ref, mag, w.dtype, "csc")
    C0 = prng.uniform_pm1(5, 8, w.shape[0] * N, dtype=np.float32).reshape(-1, N)
    C, ref, mag = run(A, w, B, accumulate=True, C0=C0)
    assert_product_close(C, ref, mag, w.dtype, "csc accumulate")
    # exact integers: the atomic order cannot matter
    vals = w.exact_values()
    A2 = gpu_pack(lt, (1, 0), w.shape, [w.rows, w.cols], vals)
    sp.sp_tensor_tune(A2, sp.SP_TUNE_CSC_MODE, mode)
    Bx = w.dense_operand(N, exact=True)
    C, ref, mag = run(A2, w, Bx, vals=vals)
    assert np.array_equal(C.cpu().numpy(), ref)


def test_result_is_independent_of_the_encoding():
    """The paper's own check (Section 5.2): the same COO under every annotation (4 level-type pairs x 2 orderings x
    widths) gives the same C."""
    w = W.cfg2_powerlaw_csr(1500, 1200, cap=700)
    for N in (1, 6, 40):
        B = w.dense_operand(N)
        ref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, B)
        C0 = prng.uniform_pm1(5, 9, w.shape[0] * N).reshape(-1, N)
        refa, maga = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, B, True, C0)
        for lt in [(0, 0), (0, 1), (1, 0), (1, 1)]:
            for order in [(0, 1), (1, 0)]:
                for pw, cw in [(32, 32), (64, 32), (32, 64), (0, 0)]:
                    say("case encoding", lt, order, pw, cw, "N", N)
                    A = gpu_pack(lt, order, w.shape, [w.rows, w.cols], w.vals, pw, cw)
                    C = torch.full((w.shape[0], N), float("nan"), dtype=torch.float64, device=DEV)
                    sp.sp_matmul(A, dev(B), C)
                    assert_product_close(C, ref, mag, np.float64, str((lt, order, pw, cw)))
                    C = dev(C0)
                    sp.sp_matmul(A, dev(B), C, accumulate=True)
                    assert_product_close(C, refa, maga, np.float64, str((lt, order, pw, cw)) + " accumulate")


def test_sparse_state_space_200_configurations():
    """Section 5.2's loop: 4 level-type pairs x 2 orderings x 5 pointer widths x 5 index widths = 200 ways of
    storing one matrix; every one must hold the checker's arrays bit for bit and give the same SpMM result."""
    from gpu_util import assert_storage_equal
    w = W.uniform_random(40, 50, 100)
    B = w.dense_operand(3)
    ref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, B)
    Bd = dev(B)
    count = 0
    for lt in [(0, 0), (0, 1), (1, 0), (1, 1)]:
        for order in [(0, 1), (1, 0)]:
            for pw in [0, 8, 16, 32, 64]:
                for cw in [0, 8, 16, 32, 64]:
                    A = gpu_pack(lt, order, w.shape, [w.rows, w.cols], w.vals, pw, cw)
                    assert_storage_equal(A, oracle.pack(lt, order, w.shape, [w.rows, w.cols], w.vals, pw, cw))
                    C = torch.full((40, 3), float("nan"), dtype=torch.float64, device=DEV)
                    sp.sp_matmul(A, Bd, C)
                    assert_product_close(C, ref, mag, np.float64, str((lt, order, pw, cw)))
                    count += 1
    assert count == 200
    say("case width overflow")
    w2 = W.uniform_random(40, 300, 200)
    for pw, cw in [(8, 32), (32, 8)]:          # 200 entries do not fit a signed 8-bit pointer; column 299 no 8-bit index
        with pytest.raises(sp.SpError) as e:
            gpu_pack((0, 1), None, w2.shape, [w2.rows, w2.cols], w2.vals, pw, cw)
        assert e.value.code == oracle.ERR_WIDTH
    A = gpu_pack((1, 1), (1, 0), w2.shape, [w2.rows, w2.cols], w2.vals, 16, 16)     # CSC-like, 16-bit: transposed copy inside
    C = torch.empty((40, 2), dtype=torch.float64, device=DEV)
    sp.sp_matmul(A, dev(w2.dense_operand(2)), C)
    ref2, mag2 = oracle.matmul_coo(w2.shape, w2.rows, w2.cols, w2.vals, w2.dense_operand(2))
    assert_product_close(C, ref2, mag2, np.float64, "16-bit DCSC")


def test_dense_inner_levels_row_band_shape():
    """The paper's SpMV experiment shape (Section 6.2): the first rows full, the rest empty, under CSR, DCSR and the
    compressed-then-dense format, f64 and f32."""
    for dtype, n, band in ((np.float64, 2048, 100), (np.float32, 2048, 100), (np.float64, 5000, 37), (np.float32, 6148, 3)):
        w = W.row_band(n, band)
        w.vals = w.vals.astype(dtype)
        w.dtype = dtype
        x = w.dense_operand(1)
        ref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, x)
        for lt in [(0, 1), (1, 1), (1, 0), (0, 0)]:
            say("case row band", lt, dtype.__name__)
            A = gpu_pack(lt, (0, 1), w.shape, [w.rows, w.cols], w.vals)
            y = torch.full((w.shape[0],), float("nan"), dtype=A.dtype, device=DEV)
            sp.sp_matmul(A, dev(x[:, 0].copy()), y)
            assert_product_close(y, ref, mag, dtype, "row band " + str(lt))
            assert torch.all(y[band:] == 0)
            y0 = prng.uniform_pm1(5, 10, w.shape[0], dtype=dtype)
            refa, maga = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, x, True, y0)
            ya = dev(y0)
            sp.sp_matmul(A, dev(x[:, 0].copy()), ya, accumulate=True)
            assert_product_close(ya, refa, maga, dtype, "row band accumulate " + str(lt))


def test_degenerate_products():
    z = np.zeros(0, dtype=np.int64)
    for lt, order in [((0, 1), (0, 1)), ((1, 1), (0, 1)), ((0, 1), (1, 0))]:
        say("case nnz=0", lt, order)
        A = gpu_pack(lt, order, (50, 60), [z, z], np.zeros(0))
        C = torch.full((50, 3), float("nan"), dtype=torch.float64, device=DEV)
        sp.sp_matmul(A, torch.ones((60, 3), dtype=torch.float64, device=DEV), C)
        assert torch.all(C == 0)
    idx = np.arange(100, dtype=np.int64)
    A = gpu_pack((0, 1), None, (100, 100), [idx, idx], np.ones(100))      # identity: C = B exactly
    B = dev(prng.uniform_pm1(1, 1, 700).reshape(100, 7))
    C = torch.empty((100, 7), dtype=torch.float64, device=DEV)
    sp.sp_matmul(A, B, C)
    assert torch.equal(C, B)
    with pytest.raises(sp.SpError) as e:
        sp.sp_matmul(A, B, C, N=7, ldb=3, ldc=7)
    assert e.value.code == oracle.ERR_SHAPE


def test_spmm_with_64_bit_coordinates_takes_64_bit_row_offsets():
    """crd in 64 bits: the kernels cut by entries then keep 64-bit byte offsets of the rows of B (the variant meant for
    operands of 4 GB and more, exercised here at a small size)."""
    w = W.cfg3_powerlaw_csr_spmm(5000, 4000, N=16, cap=2000)
    B = w.dense_operand(16)
    for pw, cw in [(32, 64), (64, 64)]:
        say("case spmm 64-bit crd", pw, cw)
        A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals, pw, cw)
        for kernel in (3, 0):
            sp.sp_tensor_tune(A, sp.SP_TUNE_SPMM_KERNEL, kernel)
            C, ref, mag = run(A, w, B)
            assert_product_close(C, ref, mag, w.dtype, "spmm 64-bit crd")
