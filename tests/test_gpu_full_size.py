"""The benchmark configurations at their full sizes, in the launch configuration bench.py times.

The storage arrays of all five configurations are compared with the CPU checker's bit for bit, and every product on
every element: to the tolerance for the seeded values, and bit for bit for small-integer values (sums that are exact in
any order).  The rank-3 tensor of the MTTKRP experiment is compared on whole slices picked by size and by seed (the
checker needs 14 s per product of that tensor on one core; its storage through invariants).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_04305_amd as sp
from gen import workloads as W, prng
from gpu_util import say, dev, gpu_pack, assert_storage_equal, assert_product_close, DEV

pytestmark = pytest.mark.gpu

_cache = {}


def workload(name):
    if name not in _cache:
        _cache.clear()                     # one full-size workload in host memory at a time
        say("generating", name)
        _cache[name] = {"cfg2": W.cfg2_powerlaw_csr, "cfg4": W.cfg4_hypersparse_dcsr, "cfg5": W.cfg5_zipf_csc_spmm}[name]()
        say(_cache[name].stats)
    return _cache[name]


def check_storage_invariants(A, w):
    """pos[0] = 0, pos monotone, pos[last] = len(crd), crd in range and strictly increasing inside each segment."""
    info = sp.sp_tensor_info(A)
    P = 1
    for l in range(2):
        size = w.shape[info.dimOrdering[l]]
        if info.levelTypes[l] == 0:
            P *= size
            continue
        pos, crd = sp.sp_pos(A, l).long(), sp.sp_crd(A, l).long()
        assert pos.numel() == P + 1 and int(pos[0]) == 0 and int(pos[-1]) == crd.numel()
        assert bool(torch.all(pos[1:] >= pos[:-1]))
        assert bool(torch.all((crd >= 0) & (crd < size)))
        inner = torch.ones(crd.numel(), dtype=torch.bool, device=DEV)
        starts = pos[:-1][pos[:-1] < crd.numel()]
        inner[starts] = False
        assert bool(torch.all((crd[1:] > crd[:-1]) | ~inner[1:]))
        P = crd.numel()
    assert info.nvalues == P


def sampled_rows_product(w, rows_pick, B):
    """(C_ref, mag) for the picked rows only, from the sub-COO holding exactly those rows."""
    sel = np.isin(w.rows, rows_pick)
    remap = -np.ones(w.shape[0], dtype=np.int64)
    remap[rows_pick] = np.arange(len(rows_pick))
    return oracle.matmul_coo((len(rows_pick), w.shape[1]), remap[w.rows[sel]], w.cols[sel], w.vals[sel], B)


def test_cfg2_pack_and_spmv_full_size():
    w = workload("cfg2")
    say("case cfg2 full: pack")
    A = gpu_pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], w.vals, 32, 32)
    ref = oracle.pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], w.vals, 32, 32)
    assert_storage_equal(A, ref)
    del ref
    x = w.dense_operand(1)
    yref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, x)
    xd = dev(x[:, 0].copy())
    for kernel in (0, 4, 2, 3, 1):         # 0 = what bench.py times (the binned kernel at this size)
        say("case cfg2 full: spmv kernel", kernel)
        sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, kernel)
        y = torch.full((w.shape[0],), float("nan"), dtype=torch.float64, device=DEV)
        sp.sp_matmul(A, xd, y)
        assert_product_close(y, yref, mag, np.float64, "cfg2 kernel %d" % kernel)
    # closed form at full size: all-ones values and x give the row lengths, exactly
    say("case cfg2 full: row lengths")
    A1 = gpu_pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], np.ones(w.nnz), 32, 32)
    y = torch.empty(w.shape[0], dtype=torch.float64, device=DEV)
    sp.sp_matmul(A1, torch.ones(w.shape[1], dtype=torch.float64, device=DEV), y)
    assert torch.equal(y, (sp.sp_pos(A1, 1)[1:] - sp.sp_pos(A1, 1)[:-1]).double())


def test_automatic_spmv_kernel_follows_the_column_pattern():
    """Two matrices of the size class where the automatic choice looks at the columns: nine diagonals (every gather falls
    next to the previous one: the streaming kernel stays, bit for bit the same sums as with tune value 2) and the scattered
    1M x 1M matrix (the binned kernel: same sums as with tune value 4 up to their order, so only to rounding)."""
    n = 600_000
    say("case automatic kernel: nine diagonals")
    i = np.repeat(np.arange(n, dtype=np.int64), 9)
    j = i + np.tile(np.arange(-4, 5, dtype=np.int64), n)
    keep = (j >= 0) & (j < n)
    i, j = i[keep], j[keep]
    v = prng.uniform_pm1(17, 1, len(i))
    x = prng.uniform_pm1(17, 2, n)
    yref, mag = oracle.matmul_coo((n, n), i, j, v, x.reshape(n, 1))
    ys = {}
    for kernel in (0, 2):
        A = gpu_pack((0, 1), (0, 1), (n, n), [i, j], v, 32, 32)
        sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, kernel)
        y = torch.full((n,), float("nan"), dtype=torch.float64, device=DEV)
        sp.sp_matmul(A, dev(x), y)
        assert_product_close(y, yref, mag, np.float64, "diagonals, kernel %d" % kernel)
        ys[kernel] = y
    assert torch.equal(ys[0], ys[2])
    say("case automatic kernel: scattered columns")
    w = workload("cfg2")
    x = w.dense_operand(1)
    ys = {}
    for kernel in (0, 2):
        A = gpu_pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], w.vals, 32, 32)
        sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, kernel)
        y = torch.empty(w.shape[0], dtype=torch.float64, device=DEV)
        sp.sp_matmul(A, dev(x[:, 0].copy()), y)
        ys[kernel] = y
    assert not torch.equal(ys[0], ys[2])                     # another kernel, another order of the additions
    assert float((ys[0] - ys[2]).abs().max()) < 1e-9


def full_product_both_ways(w, A, N, dtype, what):
    """Every element of C = A.B against the checker: the workload's own values to the tolerance, then small integers
    (values of A replaced through a second pack with the same coordinates) bit for bit."""
    tdt = torch.float64 if dtype == np.float64 else torch.float32
    B = w.dense_operand(N)
    say("case", what, "full: product,", N, "columns, every element")
    C = torch.full((w.shape[0], N), float("nan"), dtype=tdt, device=DEV)
    sp.sp_matmul(A, dev(B), C)
    ref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, B)
    assert_product_close(C, ref, mag, dtype, what + ", every element")
    del ref, mag
    say("case", what, "full: small integers, bit for bit")
    vals = w.exact_values()
    Bx = w.dense_operand(N, exact=True)
    Ax = gpu_pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], vals, 32, 32)
    C.fill_(float("nan"))
    sp.sp_matmul(Ax, dev(Bx), C)
    ref, _ = oracle.matmul_coo(w.shape, w.rows, w.cols, vals, Bx)
    assert np.array_equal(C.cpu().numpy(), ref), what + ": exact integers differ"
    Ax.free()


def test_cfg3_spmm_full_size_every_element():
    w = workload("cfg2")
    A = gpu_pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], w.vals, 32, 32)
    full_product_both_ways(w, A, 64, np.float64, "cfg3")


def test_cfg4_dcsr_full_size():
    w = workload("cfg4")
    say("case cfg4 full: pack")
    A = gpu_pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], w.vals, 32, 32)
    ref = oracle.pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], w.vals, 32, 32)
    assert_storage_equal(A, ref)
    x = w.dense_operand(1)
    yref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, x)
    say("case cfg4 full: spmv overwrite")
    y = torch.full((w.shape[0],), float("nan"), dtype=torch.float64, device=DEV)
    sp.sp_matmul(A, dev(x[:, 0].copy()), y)
    assert_product_close(y, yref, mag, np.float64, "cfg4")
    say("case cfg4 full: spmv accumulate")
    y0 = prng.uniform_pm1(3, 3, w.shape[0])
    yref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, x, True, y0)
    y = dev(y0)
    sp.sp_matmul(A, dev(x[:, 0].copy()), y, accumulate=True)
    assert_product_close(y, yref, mag, np.float64, "cfg4 accumulate")


def test_cfg5_csc_full_size():
    w = workload("cfg5")
    say("case cfg5 full: pack, storage bit for bit")
    A = gpu_pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], w.vals, 32, 32)
    check_storage_invariants(A, w)
    ref = oracle.pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], w.vals, 32, 32)
    assert_storage_equal(A, ref)
    del ref
    full_product_both_ways(w, A, 32, np.float32, "cfg5")


def test_full_size_mttkrp_both_storage_orders():
    """The 12092 x 9184 x 28818 tensor with 76.9M entries and 42 columns (the shape of the paper's MTTKRP experiment):
    sampled output rows (the heaviest slices, the lightest, and seeded others), each computed by the checker from
    exactly the entries of its slice; the rank-3 storage through its invariants and the same slices' values."""
    say("generating mttkrp tensor")
    w = W.tensor3_slices()
    say(w.stats)
    C, D = w.factors()
    I = w.shape[0]
    per_slice = np.bincount(w.ci, minlength=I)
    order_by_size = np.argsort(per_slice, kind="stable")
    sample = np.unique(np.concatenate([order_by_size[:20], order_by_size[-6:], prng.below(W.BASE_SEED + 70, 1, 120, I)]))
    sel = np.isin(w.ci, sample)
    say("checker on", int(sel.sum()), "entries of", sample.size, "slices")
    ref, mag = oracle.mttkrp_coo(w.shape, w.ci[sel], w.ck[sel], w.cl[sel], w.vals[sel], C, D)
    coords = [dev(c) for c in (w.ci, w.ck, w.cl)]
    vals = dev(w.vals)
    for order in [(0, 1, 2), (0, 2, 1)]:
        say("case full-size mttkrp", order)
        B = sp.sp_pack(sp.sp_encode((0, 1, 1), order, 32, 32), w.shape, coords, vals)
        info = sp.sp_tensor_info(B)
        assert info.nvalues == w.nnz
        pos1, pos2 = sp.sp_pos(B, 1).long(), sp.sp_pos(B, 2).long()
        crd1, crd2 = sp.sp_crd(B, 1).long(), sp.sp_crd(B, 2).long()
        assert pos1.numel() == I + 1 and int(pos1[0]) == 0 and int(pos1[-1]) == crd1.numel() == pos2.numel() - 1
        assert int(pos2[0]) == 0 and int(pos2[-1]) == crd2.numel() == w.nnz
        assert bool(torch.all(pos1[1:] >= pos1[:-1])) and bool(torch.all(pos2[1:] > pos2[:-1]))     # no empty fibre
        assert bool(torch.all((crd1 >= 0) & (crd1 < w.shape[order[1]]))) and bool(torch.all((crd2 >= 0) & (crd2 < w.shape[order[2]])))
        got_per_slice = (pos2[pos1[1:]] - pos2[pos1[:-1]]).cpu().numpy()
        assert np.array_equal(got_per_slice, per_slice)
        A = torch.full((I, w.J), float("nan"), dtype=torch.float64, device=DEV)
        sp.sp_mttkrp(B, dev(C), dev(D), A)
        Ah = A.cpu().numpy()
        err = np.abs(Ah[sample] - ref[sample])
        assert np.all(err <= 1e-12 * mag[sample]), float(np.max(err / np.maximum(mag[sample], 1e-300)))
        assert np.all(Ah[per_slice == 0] == 0.0) and not np.isnan(Ah).any()
        B.free()


@pytest.mark.parametrize("m", [300_000, 1_500_000])
def test_pack_and_multiply_hundreds_of_millions_of_entries(m):
    """Well above the benchmark sizes, up to 1.5 billion entries (the builder takes fewer than 2^31): rows of exactly 1,000
    entries, given in an order scrambled by a multiplicative permutation (made on the device: no host generator needed
    at this size).  Every array of the result is known in closed form; the product with a vector of ones gives the row
    sums."""
    k, n = 1_000, 4_096
    N = m * k
    free_bytes, total_bytes = torch.cuda.mem_get_info()
    if total_bytes < 150 * N:              # a smaller card than the MI355X this is written for (288 GB): cannot hold the case at all
        pytest.skip("needs a device with %d GB of memory" % (150 * N >> 30))
    assert free_bytes >= 150 * N, "the device has the memory for this case but %d GB of it are in use" % ((total_bytes - free_bytes) >> 30)
    e = torch.arange(N, dtype=torch.int64, device=DEV)
    src = (e * 1_000_003) % N                          # a bijection of [0, N): gcd(1000003, N) = 1
    del e
    rows = src // k
    cols = (src % k) * 4 + (rows % 4)                  # distinct inside a row, ascending with src % k
    vals = (src % 1024).to(torch.float64)              # small integers: sums are exact
    say("packing", N, "entries")
    for pw, cw in ([(32, 32), (64, 64)] if m <= 300_000 else [(32, 32)]):
        A = sp.sp_pack(sp.sp_encode((0, 1), (0, 1), pw, cw), (m, n), [rows, cols], vals)
        info = sp.sp_tensor_info(A)
        assert info.nvalues == N and info.maxSegment == k
        pos, crd, v = sp.sp_pos(A, 1), sp.sp_crd(A, 1), sp.sp_values(A)
        assert bool(torch.equal(pos.long(), torch.arange(m + 1, dtype=torch.int64, device=DEV) * k))
        want = torch.arange(N, dtype=torch.int64, device=DEV)              # storage order = the unscrambled order
        assert bool(torch.equal(crd.long(), (want % k) * 4 + ((want // k) % 4)))
        assert bool(torch.equal(v, (want % 1024).to(torch.float64)))
        y = torch.full((m,), float("nan"), dtype=torch.float64, device=DEV)
        sp.sp_matmul(A, torch.ones(n, dtype=torch.float64, device=DEV), y)
        assert bool(torch.equal(y, (want % 1024).to(torch.float64).view(m, k).sum(dim=1)))
        del want, pos, crd, v
        A.free()
