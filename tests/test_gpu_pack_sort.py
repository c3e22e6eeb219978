"""The storage builder's two sorts against the CPU checker, bit for bit: the most-significant-digit-first sort forced on
small inputs that reach each of its paths (several LDS chunks, a chunk that does not fit the LDS, keys narrower than its two
passes), and the builder's own choice on inputs of a million entries and more, even and skewed."""
import numpy as np
import pytest

import oracle
import paper_2202_04305_amd as sp
from gen import workloads as W, prng
from gpu_util import say, gpu_pack, assert_storage_equal

pytestmark = pytest.mark.gpu
SEED = 20220204


@pytest.fixture
def msd_first():
    sp.sp_pack_sort_mode(2)
    yield
    sp.sp_pack_sort_mode(0)


def distinct_pairs(seed, m, n, nnz):
    """nnz distinct (row, col) pairs below (m, n), in a scrambled order."""
    lin = np.unique(prng.below(seed, 1, int(nnz * 1.3) + 8, m * n))
    lin = lin[prng.permutation(seed, 2, lin.size)][:nnz]
    return (lin // n).astype(np.int64), (lin % n).astype(np.int64)


def both(lt, order, shape, coords, vals, what):
    say("case", what, "shape", shape, "entries", len(vals))
    ref = oracle.pack(lt, order, shape, coords, vals, 32, 32)
    A = gpu_pack(lt, order, shape, coords, vals, 32, 32)
    assert_storage_equal(A, ref)
    return A


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("lt,order", [((0, 1), (0, 1)), ((1, 1), (0, 1)), ((0, 1), (1, 0))])
def test_forced_on_small_inputs_of_every_key_width(msd_first, dtype, lt, order):
    for (m, n, nnz) in [(3, 4, 1), (4, 4, 9), (20, 30, 333), (200, 250, 20000), (3000, 3100, 50000), (1 << 18, 1 << 19, 40000)]:
        r, c = distinct_pairs(SEED + m, m, n, nnz)
        v = prng.uniform_pm1(SEED + n, 3, r.size, dtype)
        both(lt, order, (m, n), [r, c], v, "forced msd %s %s" % (lt, order))


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("width", [25000, 1 << 20])
def test_forced_with_rows_too_long_for_the_lds(msd_first, dtype, width):
    """Rows of 9000 to 20000 entries between ordinary ones: their chunks go through device memory, with two to four key
    digits that differ inside a chunk (odd and even numbers of hops between the buffers)."""
    m, n = 1 << 16, 1 << 20
    rows, cols = [], []
    for i, (row, length) in enumerate([(5, 20000), (4097, 9000), (m - 1, 15000)]):
        cc = np.unique(prng.below(SEED + i, 4, length * 3, width))
        assert cc.size >= length
        cc = cc[prng.permutation(SEED + i, 12, cc.size)][:length]
        rows.append(np.full(cc.size, row, dtype=np.int64))
        cols.append(cc.astype(np.int64))
    r0, c0 = distinct_pairs(SEED + 9, m, n, 30000)
    keep = ~np.isin(r0, [5, 4097, m - 1])
    r = np.concatenate(rows + [r0[keep]])
    c = np.concatenate(cols + [c0[keep]])
    p = prng.permutation(SEED + 11, 5, r.size)
    r, c = r[p], c[p]
    v = prng.uniform_pm1(SEED + 12, 6, r.size, dtype)
    A = both((0, 1), (0, 1), (m, n), [r, c], v, "forced msd, long rows, width %d" % width)
    assert sp.sp_tensor_info(A).maxSegment == 20000


def test_forced_rank3_and_input_errors(msd_first):
    I, K, L = 40, 50, 60
    lin = np.unique(prng.below(SEED, 7, 30000, I * K * L))
    lin = lin[prng.permutation(SEED, 8, lin.size)]
    ci, ck, cl = lin // (K * L), (lin // L) % K, lin % L
    v = prng.uniform_pm1(SEED, 9, lin.size, np.float64)
    for lt, order in [((1, 1, 1), (0, 1, 2)), ((0, 1, 1), (2, 0, 1)), ((1, 0, 1), (1, 2, 0))]:
        say("case rank 3", lt, order)
        ref = oracle.pack(lt, order, (I, K, L), [ci, ck, cl], v, 32, 32)
        A = gpu_pack(lt, order, (I, K, L), [ci, ck, cl], v, 32, 32)
        assert_storage_equal(A, ref)
    # an entry given twice, a coordinate out of range: the same errors as with the other sort
    r, c = distinct_pairs(SEED + 1, 300, 300, 5000)
    v = prng.uniform_pm1(SEED, 10, r.size + 1, np.float64)
    with pytest.raises(sp.SpError) as e:
        gpu_pack((0, 1), (0, 1), (300, 300), [np.append(r, r[17]), np.append(c, c[17])], v)
    assert e.value.code == 7
    with pytest.raises(sp.SpError) as e:
        gpu_pack((0, 1), (0, 1), (300, 300), [np.append(r, 300), np.append(c, 0)], v)
    assert e.value.code == 6


def test_forced_sums_of_duplicates_keep_their_order(msd_first):
    """Sparse addition and the sparse product add up entries with equal coordinates after the sort, in input order: the
    results stay bit-identical to the checker's under the other sort."""
    import test_gpu_add
    import test_gpu_spgemm
    test_gpu_add.test_add_matrices_in_every_pair_of_compressed_formats(np.float32)
    test_gpu_spgemm.test_spgemm_result_formats_widths_and_dtypes(np.float32, "dcsr")


@pytest.mark.parametrize("maker,name", [
    (lambda: W.cfg2_powerlaw_csr(1 << 17, 1 << 20, cap=9000), "lognormal rows, 2M entries"),
    (lambda: W.cfg5_zipf_csc_spmm(1 << 17, 1 << 17, cap=50000), "Zipf columns, 2M entries"),
    (lambda: W.cfg4_hypersparse_dcsr(1 << 22, 1 << 22), "hypersparse, 1.3M entries"),
])
@pytest.mark.parametrize("mode", [0, 2])
def test_a_million_entries_and_more(maker, name, mode):
    """mode 0: the builder's own choice (even input: most significant digit first; skewed: the other sort); mode 2: most
    significant digit first also on the skewed input, whose heavy columns then take the slow path."""
    w = maker()
    say("case", name, "mode", mode, w.stats)
    ref = oracle.pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], w.vals, 32, 32)
    sp.sp_pack_sort_mode(mode)
    try:
        A = gpu_pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], w.vals, 32, 32)
    finally:
        sp.sp_pack_sort_mode(0)
    assert_storage_equal(A, ref)
