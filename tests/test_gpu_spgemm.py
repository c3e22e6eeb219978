"""GPU sparse x sparse product with a sparse result (the SpMSpM kernel) against the CPU checker, through the C ABI.

C's pos / crd must equal, bit for bit, the storage the checker packs from its own product; the values are within
1e-12 (f64) / 1e-5 (f32) times the sum of the absolute values of an element's terms; small-integer inputs bit for bit.
"""
import json
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2202_04305_amd as sp
from gen import workloads as W, prng
from gpu_util import say, gpu_pack, tol_for

pytestmark = pytest.mark.gpu

ENC = {"csr": ((0, 1), (0, 1)), "dcsr": ((1, 1), (0, 1)), "csc": ((0, 1), (1, 0)), "dcsc": ((1, 1), (1, 0))}


def pair(m, k, n, nnz_a, nnz_b, dtype=np.float64, seed=0):
    return (W.uniform_random(m, k, nnz_a, dtype=dtype, seed=W.BASE_SEED + 500 + seed),
            W.uniform_random(k, n, nnz_b, dtype=dtype, seed=W.BASE_SEED + 600 + seed))


def check(C, fmt, shape, ref, dtype, exact=False, pw=32, cw=32):
    ci, cj, cv, mag = ref
    lt, order = ENC[fmt]
    P = oracle.pack(lt, order, shape, [ci, cj], cv, pw, cw)
    M = oracle.pack(lt, order, shape, [ci, cj], mag.astype(cv.dtype), pw, cw)
    info = sp.sp_tensor_info(C)
    assert tuple(info.shape[:2]) == tuple(shape) and info.nvalues == len(ci) and info.nnz == len(ci)
    for l in range(2):
        if P.pos[l] is None:
            continue
        gp, gc = sp.sp_pos(C, l).cpu().numpy(), sp.sp_crd(C, l).cpu().numpy()
        assert gp.dtype == P.pos[l].dtype and np.array_equal(gp, P.pos[l]), "pos[%d]" % l
        assert gc.dtype == P.crd[l].dtype and np.array_equal(gc, P.crd[l]), "crd[%d]" % l
    gv = sp.sp_values(C).cpu().numpy()
    assert gv.dtype == cv.dtype
    if exact:
        assert np.array_equal(gv, P.values)
    else:
        err = np.abs(gv.astype(np.float64) - P.values.astype(np.float64))
        tol = tol_for(dtype) * M.values.astype(np.float64) * (1.0 + 1e-6) + (1e-30 if dtype == np.float64 else 1e-37)
        assert np.all(err <= tol), float(np.max(err / np.maximum(M.values.astype(np.float64), 1e-300)))


@pytest.mark.parametrize("fa", ["csr", "dcsr", "csc", "dcsc"])
@pytest.mark.parametrize("fb", ["csr", "dcsr", "csc", "dcsc"])
def test_spgemm_every_operand_format(fa, fb):
    a, b = pair(700, 500, 600, 9000, 8000)
    ref = oracle.spgemm_coo(a.shape, a.rows, a.cols, a.vals, b.shape, b.rows, b.cols, b.vals)
    say("case spgemm", fa, fb, "pairs ->", len(ref[0]), "entries")
    A = gpu_pack(*ENC[fa], a.shape, [a.rows, a.cols], a.vals)
    B = gpu_pack(*ENC[fb], b.shape, [b.rows, b.cols], b.vals)
    for fc in ["csr", "dcsc"] if fa == fb else ["csr"]:
        C = sp.sp_spgemm(A, B, sp.sp_encode(*ENC[fc], 32, 32))
        check(C, fc, (700, 600), ref, np.float64)
        C2 = sp.sp_spgemm(A, B, sp.sp_encode(*ENC[fc], 32, 32))
        assert torch.equal(sp.sp_values(C), sp.sp_values(C2)), "not reproducible"


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("fc", ["csr", "dcsr", "csc", "dcsc"])
def test_spgemm_result_formats_widths_and_dtypes(dtype, fc):
    a = W.cfg2_powerlaw_csr(3000, 2000, mean=6.0, cap=400)           # skewed rows on both sides
    b = W.cfg2_powerlaw_csr(2000, 2500, mean=5.0, cap=300, seed=W.BASE_SEED + 33)
    va, vb = a.vals.astype(dtype), b.vals.astype(dtype)
    ref = oracle.spgemm_coo(a.shape, a.rows, a.cols, va, b.shape, b.rows, b.cols, vb)
    say("case spgemm result", fc, dtype.__name__, len(ref[0]))
    for pw, cw in [(32, 32), (64, 64), (64, 32)]:
        A = gpu_pack((0, 1), (0, 1), a.shape, [a.rows, a.cols], va, pw, cw)
        B = gpu_pack((0, 1), (0, 1), b.shape, [b.rows, b.cols], vb, pw, cw)
        C = sp.sp_spgemm(A, B, sp.sp_encode(*ENC[fc], pw, cw))
        check(C, fc, (3000, 2500), ref, dtype, pw=pw, cw=cw)


def test_spgemm_exact_integers_kept_zeros_and_chained_product():
    a, b = pair(400, 300, 350, 5000, 4000)
    va, vb = prng.small_ints(7, 1, a.nnz), prng.small_ints(7, 2, b.nnz)       # zeros among them: they stay stored
    ref = oracle.spgemm_coo(a.shape, a.rows, a.cols, va, b.shape, b.rows, b.cols, vb)
    assert (ref[2] == 0.0).any()
    A = gpu_pack(*ENC["csr"], a.shape, [a.rows, a.cols], va)
    B = gpu_pack(*ENC["csr"], b.shape, [b.rows, b.cols], vb)
    C = sp.sp_spgemm(A, B, sp.sp_encode(*ENC["csr"], 32, 32))
    check(C, "csr", (400, 350), ref, np.float64, exact=True)
    # the result is an ordinary tensor: multiply it again, by a sparse matrix and by a dense vector
    c, _ = pair(350, 350, 10, 3000, 1)
    vc = prng.small_ints(7, 3, c.nnz, lo=-2, hi=2)
    ref2 = oracle.spgemm_coo((400, 350), ref[0], ref[1], ref[2], c.shape, c.rows, c.cols, vc)
    D = sp.sp_spgemm(C, gpu_pack(*ENC["csr"], c.shape, [c.rows, c.cols], vc), sp.sp_encode(*ENC["dcsr"], 32, 32))
    check(D, "dcsr", (400, 350), ref2, np.float64, exact=True)
    x = prng.small_ints(7, 4, 350)
    y = torch.zeros(400, dtype=torch.float64, device="cuda:0")
    sp.sp_matmul(C, torch.from_numpy(x).cuda(), y)
    yref, _ = oracle.matmul_coo((400, 350), ref[0], ref[1], ref[2], x)
    assert np.array_equal(y.cpu().numpy(), yref.ravel())


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("fa", ["csr", "dcsr"])
def test_spgemm_both_kernels(dtype, fa):
    """Kernel 1 (pairs through the storage builder), kernel 2 (a row of C at a time in an LDS workspace, four waves per row
    over a column-panel copy of B), kernel 3 (the same with one wave per row) and kernel 4 (sixteen waves per row; the automatic
    choice at 9000 columns) against the checker; widths 32 and 64; rows of A from empty to hundreds of entries, rows of B longer
    than a wave."""
    a = W.cfg2_powerlaw_csr(2500, 1800, mean=8.0, cap=700)
    b = W.cfg2_powerlaw_csr(1800, 9000, mean=40.0, cap=3000, seed=W.BASE_SEED + 34)      # 9000 columns: near the LDS limit in f64
    va, vb = a.vals.astype(dtype), b.vals.astype(dtype)
    ref = oracle.spgemm_coo(a.shape, a.rows, a.cols, va, b.shape, b.rows, b.cols, vb)
    for pw, cw in [(32, 32), (64, 64)]:
        A = gpu_pack(*ENC[fa], a.shape, [a.rows, a.cols], va, pw, cw)
        B = gpu_pack(*ENC["csr"], b.shape, [b.rows, b.cols], vb, pw, cw)
        enc = sp.sp_encode(*ENC["csr"], pw, cw)
        for kernel in (1, 2, 3, 4, 5, 0):
            say("case spgemm kernels", dtype.__name__, fa, pw, "kernel", kernel, len(ref[0]))
            sp.sp_tensor_tune(A, sp.SP_TUNE_SPGEMM_KERNEL, kernel)
            C = sp.sp_spgemm(A, B, enc)
            check(C, "csr", (2500, 9000), ref, dtype, pw=pw, cw=cw)
            C2 = sp.sp_spgemm(A, B, enc)
            if kernel != 5:                                        # kernel 5 adds in an order that depends on timing
                assert torch.equal(sp.sp_values(C), sp.sp_values(C2)), "not reproducible"


def test_spgemm_workspace_kernel_limits_and_exact_integers():
    a, b = pair(300, 200, 9100, 2500, 30000)
    A = gpu_pack(*ENC["csr"], a.shape, [a.rows, a.cols], a.vals)
    B = gpu_pack(*ENC["csr"], b.shape, [b.rows, b.cols], b.vals)
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPGEMM_KERNEL, 2)
    with pytest.raises(sp.SpError) as err:           # a row of 9100 f64 does not fit the workspace
        sp.sp_spgemm(A, B, sp.sp_encode(*ENC["csr"], 32, 32))
    assert err.value.code == 10
    with pytest.raises(sp.SpError) as err:           # nor does the workspace kernel write a column-major result
        sp.sp_spgemm(A, gpu_pack(*ENC["csr"], (200, 50), [np.array([1]), np.array([2])], np.array([1.0])), sp.sp_encode(*ENC["csc"], 32, 32))
    assert err.value.code == 10
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPGEMM_KERNEL, 0)
    ref = oracle.spgemm_coo(a.shape, a.rows, a.cols, a.vals, b.shape, b.rows, b.cols, b.vals)
    check(sp.sp_spgemm(A, B, sp.sp_encode(*ENC["csr"], 32, 32)), "csr", (300, 9100), ref, np.float64)     # automatic: the other kernel
    # small integers, zeros among them, through the workspace kernel: bit for bit, kept zeros included
    a, b = pair(400, 300, 350, 5000, 4000)
    va, vb = prng.small_ints(7, 1, a.nnz), prng.small_ints(7, 2, b.nnz)
    ref = oracle.spgemm_coo(a.shape, a.rows, a.cols, va, b.shape, b.rows, b.cols, vb)
    for fa in ("csr", "dcsr"):
        for kernel in (2, 3):
            A = gpu_pack(*ENC[fa], a.shape, [a.rows, a.cols], va)
            sp.sp_tensor_tune(A, sp.SP_TUNE_SPGEMM_KERNEL, kernel)
            C = sp.sp_spgemm(A, gpu_pack(*ENC["csr"], b.shape, [b.rows, b.cols], vb), sp.sp_encode(*ENC["csr"], 32, 32))
            check(C, "csr", (400, 350), ref, np.float64, exact=True)
    # widths that are no multiple of the panel width, and fewer columns than four panels of 64
    for n in (257, 300, 1000, 130):
        a, b = pair(200, 150, n, 2500, 3000, seed=n)
        ref = oracle.spgemm_coo(a.shape, a.rows, a.cols, a.vals, b.shape, b.rows, b.cols, b.vals)
        A = gpu_pack(*ENC["csr"], a.shape, [a.rows, a.cols], a.vals)
        B = gpu_pack(*ENC["csr"], b.shape, [b.rows, b.cols], b.vals)
        sp.sp_tensor_tune(A, sp.SP_TUNE_SPGEMM_KERNEL, 2)
        check(sp.sp_spgemm(A, B, sp.sp_encode(*ENC["csr"], 32, 32)), "csr", (200, n), ref, np.float64)
    # sixteen waves per row: from 1024 columns on (below, tune value 4 runs the four-wave kernel), ragged last panel, rows of A
    # longer than one batch of 64 entries, rows of B longer than a group's eight lanes inside one panel; small integers: bit for bit
    for n, nnza, nnzb in ((1024, 2500, 3000), (1500, 20000, 30000), (4100, 30000, 60000), (1000, 2500, 3000)):
        a, b = pair(200, 150, n, nnza, nnzb, seed=n + 1)
        va, vb = prng.small_ints(9, 1, a.nnz), prng.small_ints(9, 2, b.nnz)
        ref = oracle.spgemm_coo(a.shape, a.rows, a.cols, va, b.shape, b.rows, b.cols, vb)
        for fa in ("csr", "dcsr"):
            say("case spgemm sixteen waves", n, nnza, nnzb, fa)
            A = gpu_pack(*ENC[fa], a.shape, [a.rows, a.cols], va)
            B = gpu_pack(*ENC["csr"], b.shape, [b.rows, b.cols], vb)
            for kernel in (4, 5):                                  # 5: the entries of the row dealt out to the waves, any width
                sp.sp_tensor_tune(A, sp.SP_TUNE_SPGEMM_KERNEL, kernel)
                check(sp.sp_spgemm(A, B, sp.sp_encode(*ENC["csr"], 32, 32)), "csr", (200, n), ref, np.float64, exact=True)


def test_spgemm_degenerate_and_errors():
    e = np.zeros(0, dtype=np.int64)
    enc = sp.sp_encode(*ENC["csr"], 32, 32)
    A0 = gpu_pack(*ENC["csr"], (5, 6), [e, e], np.zeros(0))
    B1 = gpu_pack(*ENC["csr"], (6, 4), [np.array([2]), np.array([3])], np.array([2.0]))
    C = sp.sp_spgemm(A0, B1, enc)
    assert sp.sp_tensor_info(C).nvalues == 0 and np.array_equal(sp.sp_pos(C, 1).cpu().numpy(), np.zeros(6, dtype=np.int32))
    A1 = gpu_pack(*ENC["csr"], (5, 6), [np.array([4]), np.array([1])], np.array([3.0]))
    C = sp.sp_spgemm(A1, B1, enc)                     # no common k
    assert sp.sp_tensor_info(C).nvalues == 0
    A2 = gpu_pack(*ENC["dcsr"], (5, 6), [np.array([4]), np.array([2])], np.array([3.0]))
    C = sp.sp_spgemm(A2, B1, enc)
    assert np.array_equal(sp.sp_pos(C, 1).cpu().numpy(), [0, 0, 0, 0, 0, 1]) and np.array_equal(sp.sp_crd(C, 1).cpu().numpy(), [3])
    assert np.array_equal(sp.sp_values(C).cpu().numpy(), [6.0])
    with pytest.raises(sp.SpError) as err:
        sp.sp_spgemm(B1, B1, enc)                     # 6 x 4 times 6 x 4
    assert err.value.code == 8
    with pytest.raises(sp.SpError) as err:
        sp.sp_spgemm(A1, gpu_pack(*ENC["csr"], (6, 4), [np.array([2])] * 2, np.array([2.0], dtype=np.float32)), enc)
    assert err.value.code == 9
    with pytest.raises(sp.SpError) as err:
        sp.sp_spgemm(A1, gpu_pack((1, 0), (0, 1), (6, 4), [np.array([2])] * 2, np.array([2.0])), enc)
    assert err.value.code == 10
    with pytest.raises(sp.SpError) as err:           # 300 columns do not fit 8-bit coordinates
        sp.sp_spgemm(A1, gpu_pack(*ENC["csr"], (6, 300), [np.array([1]), np.array([299])], np.array([2.0])), sp.sp_encode(*ENC["csr"], 32, 8))
    assert err.value.code == 5


def test_spgemm_density_of_the_papers_table_rows():
    """n x n uniform random operands of density 0.01 (the experiment of Section 6.2): the whole result against the
    checker for the three smaller sizes, and the density of C as the paper prints it for all four."""
    fix = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "spmspm_density_table.json")))
    enc = sp.sp_encode(*ENC["csr"], 32, 32)
    for row in fix["rows"]:
        n = row["n"]
        nnz = int(round(fix["density_ab"] * n * n))
        a, b = pair(n, n, n, nnz, nnz, seed=n)
        say("case spgemm table row n =", n)
        A = gpu_pack(*ENC["csr"], a.shape, [a.rows, a.cols], a.vals)
        B = gpu_pack(*ENC["csr"], b.shape, [b.rows, b.cols], b.vals)
        C = sp.sp_spgemm(A, B, enc)
        info = sp.sp_tensor_info(C)
        rho = info.nvalues / float(n * n)
        assert abs(rho - row["density_c"]) <= 0.006, (n, rho)
        if n <= 4096:
            check(C, "csr", (n, n), oracle.spgemm_coo(a.shape, a.rows, a.cols, a.vals, b.shape, b.rows, b.cols, b.vals), np.float64)
        else:      # sampled rows: the checker computes exactly those rows from A's entries in them
            rows = np.unique(prng.below(W.BASE_SEED + 71, 1, 200, n))
            sel = np.isin(a.rows, rows)
            ci, cj, cv, mag = oracle.spgemm_coo(a.shape, a.rows[sel], a.cols[sel], a.vals[sel], b.shape, b.rows, b.cols, b.vals)
            pos = sp.sp_pos(C, 1).cpu().numpy().astype(np.int64)
            crd, val = sp.sp_crd(C, 1).cpu().numpy(), sp.sp_values(C).cpu().numpy()
            at = 0
            for r in rows:
                seg = slice(pos[r], pos[r + 1])
                k = int(np.searchsorted(ci, r, side="right")) - int(np.searchsorted(ci, r, side="left"))
                assert pos[r + 1] - pos[r] == k and np.array_equal(crd[seg], cj[at:at + k])
                assert np.all(np.abs(val[seg] - cv[at:at + k]) <= 1e-12 * mag[at:at + k])
                at += k
            assert at == len(ci)
