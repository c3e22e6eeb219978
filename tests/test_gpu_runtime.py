"""How the library behaves as a component: another stream than the default one, an allocator that runs dry, and the
products recorded into a HIP graph and replayed (every replay is checked against the eager result, with eager work and
synchronisations in between)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_04305_amd as sp
from paper_2202_04305_amd import binding
from gen import workloads as W, prng
from gpu_util import say, dev, gpu_pack, assert_storage_equal, assert_product_close, DEV

pytestmark = pytest.mark.gpu


def test_everything_on_a_stream_of_its_own():
    w = W.cfg2_powerlaw_csr(6000, 5000, cap=1500)
    B = w.dense_operand(8)
    t3 = W.tensor3_slices(I=60, K=50, L=80, nnz=9000, k_mean=12, l_mean=25, J=6)
    C3, D3 = t3.factors()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals)
        y = torch.empty(w.shape[0], dtype=torch.float64, device=DEV)
        C = torch.empty((w.shape[0], 8), dtype=torch.float64, device=DEV)
        sp.sp_matmul(A, dev(B[:, 0].copy()), y)
        sp.sp_matmul(A, dev(B), C)
        T = gpu_pack((0, 1, 1), (0, 1, 2), t3.shape, [t3.ci, t3.ck, t3.cl], t3.vals)
        M = sp.sp_mttkrp(T, dev(C3), dev(D3))
        S = sp.sp_spgemm(A, gpu_pack((0, 1), (0, 1), (5000, 300), *_coo(5000, 300, 4000)), sp.sp_encode((0, 1), (0, 1), 32, 32))
        nC = sp.sp_tensor_info(S).nvalues
    side.synchronize()
    assert_storage_equal(A, oracle.pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals, 32, 32))
    ref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, B)
    assert_product_close(C, ref, mag, np.float64, "spmm on a side stream")
    assert_product_close(y, ref[:, :1], mag[:, :1], np.float64, "spmv on a side stream")
    r3, m3 = oracle.mttkrp_coo(t3.shape, t3.ci, t3.ck, t3.cl, t3.vals, C3, D3)
    assert_product_close(M, r3, m3, np.float64, "mttkrp on a side stream")
    rows, cols, vals = _coo(5000, 300, 4000)[0][0], _coo(5000, 300, 4000)[0][1], _coo(5000, 300, 4000)[1]
    ci, _, _, _ = oracle.spgemm_coo(w.shape, w.rows, w.cols, w.vals, (5000, 300), rows, cols, vals)
    assert nC == len(ci)


def _coo(m, n, nnz):
    u = W.uniform_random(m, n, nnz, seed=W.BASE_SEED + 901)
    return [u.rows, u.cols], u.vals


class _MeteredAllocator(binding._TorchAllocator):
    """torch's allocator behind the callbacks, refusing every request after the first `budget` ones."""

    def __init__(self, device, budget):
        super().__init__(device)
        self.budget, self.asked = budget, 0

    def _alloc(self, nbytes, ctx):
        self.asked += 1
        if self.asked > self.budget:
            return None
        return super()._alloc(nbytes, ctx)


@pytest.fixture(params=[0, 2], ids=["sort chosen", "most significant digit first"])
def sort_mode(request):
    """The storage builder's sort: its own choice (least significant digit first at these sizes), and the other one forced."""
    sp.sp_pack_sort_mode(request.param)
    yield request.param
    sp.sp_pack_sort_mode(0)


@pytest.mark.parametrize("fmt", [((0, 1), (0, 1)), ((1, 1), (1, 0)), ((0, 1, 1), (0, 2, 1))])
def test_allocator_running_dry_is_an_error_and_leaves_nothing_behind(fmt, sort_mode):
    lt, order = fmt
    if len(lt) == 2:
        w = W.cfg2_powerlaw_csr(3000, 2500, cap=500)
        shape, coords, vals = w.shape, [w.rows, w.cols], w.vals
    else:
        t3 = W.tensor3_slices(I=60, K=50, L=80, nnz=9000, k_mean=12, l_mean=25, J=6)
        shape, coords, vals = t3.shape, [t3.ci, t3.ck, t3.cl], t3.vals
    enc = sp.sp_encode(lt, order, 32, 32)
    cd, vd = [dev(c) for c in coords], dev(vals)
    ref = oracle.pack(lt, order, shape, coords, vals, 32, 32)
    budget, done = 0, False
    while not done:
        alloc = _MeteredAllocator(DEV, budget)
        try:
            T = sp.sp_pack(enc, shape, cd, vd, allocator=alloc)
            done = True
        except sp.SpError as e:
            assert e.code == 12, e                      # SP_ERR_ALLOC
            torch.cuda.synchronize()
            assert len(alloc.live) == 0, "budget %d: %d blocks still held after the failed call" % (budget, len(alloc.live))
            budget += 1
            assert budget < 400
    say("pack", fmt, "needs", budget, "allocations")
    assert_storage_equal(T, ref)
    held = len(alloc.live)
    T.free()
    assert len(alloc.live) == 0 and held > 0


def test_products_replayed_from_a_hip_graph():
    w = W.cfg2_powerlaw_csr(20000, 600000, cap=4000)       # x is 4.8 MB: three column panels for SpMV kernel 3
    Bh = w.dense_operand(16)
    x, Bd = dev(Bh[:, 0].copy()), dev(Bh)
    t3 = W.tensor3_slices(I=200, K=150, L=300, nnz=60000, k_mean=30, l_mean=60, J=42)
    C3, D3 = [dev(f) for f in t3.factors()]
    T = gpu_pack((0, 1, 1), (0, 1, 2), t3.shape, [t3.ci, t3.ck, t3.cl], t3.vals)
    for kernel in (1, 2, 3):
        say("case graph replay, SpMV kernel", kernel)
        A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals)
        sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, kernel)
        y, C, M = (torch.empty(w.shape[0], dtype=torch.float64, device=DEV), torch.empty((w.shape[0], 16), dtype=torch.float64, device=DEV),
                   torch.empty((200, 42), dtype=torch.float64, device=DEV))

        def products():
            sp.sp_matmul(A, x, y)
            sp.sp_matmul(A, Bd, C)
            sp.sp_mttkrp(T, C3, D3, M)

        products()                                     # the first call of a tensor builds what it keeps (no allocation later)
        torch.cuda.synchronize()
        eager = [t.clone() for t in (y, C, M)]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            products()
        for replay in range(4):
            for t in (y, C, M):
                t.fill_(float("nan"))
            scratch = torch.randn(1 << 20, device=DEV).sum()        # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for got, want in zip((y, C, M), eager):
                assert torch.equal(got, want), "replay %d differs from the eager result" % replay
            assert bool(torch.isfinite(scratch))
    ref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, Bh)
    assert_product_close(C, ref, mag, np.float64, "graph replay vs the checker")


def _binned_case():
    """Big enough, and scattered enough, for the automatic SpMV choice to take the copy binned by column panel and row
    block: at least 2^21 stored entries, x above 3 MB, 256 row blocks of 2048 rows, 32 entries per bucket on average."""
    return W.cfg2_powerlaw_csr(1 << 19, 1 << 19, mean=24.0, cap=4000)


@pytest.mark.parametrize("fmt", ["csr", "csc"])
def test_first_product_after_prepare_goes_into_a_hip_graph(fmt):
    """sp_prepare builds everything a product needs: the very first sp_matmul afterwards neither allocates nor
    synchronises, so it can be captured, and the handle reports that no product had to prepare anything."""
    w = _binned_case() if fmt == "csr" else W.cfg5_zipf_csc_spmm(1 << 15, 1 << 15)
    N = 8
    Bh = w.dense_operand(N)
    x, Bd = dev(Bh[:, 0].copy()), dev(Bh)
    A = gpu_pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], w.vals)
    assert sp.sp_tensor_info(A).spmvKernel == 0
    sp.sp_prepare(A, 1)
    sp.sp_prepare(A, N)
    info = sp.sp_tensor_info(A)
    say("case prepare then capture", fmt, "spmv kernel", info.spmvKernel, "derived bytes", info.derivedBytes, "storage", info.storageBytes)
    assert info.lazyPrepares == 0 and info.spmvKernel in (1, 2, 3, 4) and info.derivedBytes > 0
    if fmt == "csr":
        assert info.spmvKernel == 4
    y = torch.full((w.shape[0],), float("nan"), dtype=x.dtype, device=DEV)
    C = torch.full((w.shape[0], N), float("nan"), dtype=x.dtype, device=DEV)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):                      # the first products of this tensor
        sp.sp_matmul(A, x, y)
        sp.sp_matmul(A, Bd, C)
    assert sp.sp_tensor_info(A).lazyPrepares == 0
    ref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, Bh)
    for replay in range(3):
        y.fill_(float("nan")); C.fill_(float("nan"))
        scratch = torch.randn(1 << 20, device=DEV).sum()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert_product_close(C, ref, mag, w.dtype, "captured first SpMM, replay %d" % replay)
        assert_product_close(y, ref[:, :1], mag[:, :1], w.dtype, "captured first SpMV, replay %d" % replay)
        assert bool(torch.isfinite(scratch))
    sp.sp_prepare(A, N)                                # again: nothing to do
    assert sp.sp_tensor_info(A).derivedBytes == info.derivedBytes


def test_without_prepare_the_first_product_prepares_and_says_so():
    w = _binned_case()
    x = dev(w.dense_operand(1)[:, 0].copy())
    A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals)
    y = torch.empty(w.shape[0], dtype=torch.float64, device=DEV)
    for call in range(3):
        sp.sp_matmul(A, x, y)
    info = sp.sp_tensor_info(A)
    assert info.lazyPrepares == 1 and info.spmvKernel == 4
    sp.sp_tensor_tune(A, sp.SP_TUNE_SPMV_KERNEL, 2)    # another kernel is asked for: decided again, once
    assert sp.sp_tensor_info(A).spmvKernel == 0
    sp.sp_matmul(A, x, y); sp.sp_matmul(A, x, y)
    info = sp.sp_tensor_info(A)
    assert info.lazyPrepares == 2 and info.spmvKernel == 2


@pytest.mark.parametrize("maker,expect", [
    (lambda: W.cfg1_uniform_csr(), 1),                                           # small and even: lanes per row
    (lambda: W.cfg2_powerlaw_csr(20000, 20000, cap=3000), 2),                    # medium: the stream kernel
    (lambda: W.cfg2_powerlaw_csr(1 << 17, 1 << 17), 2),                          # 2 M entries but x is only 1 MB: still the stream kernel
    (lambda: W.cfg4_hypersparse_dcsr(1 << 21, 1 << 21), 2),                      # few stored rows: no binned copy
])
def test_automatic_spmv_choice_below_the_binned_threshold_is_reproducible(maker, expect):
    """The binned kernel adds a row's products in an order that depends on timing; every automatic choice below its
    size threshold (2^21 entries, x above 3 MB, 256 row blocks) must give the same bits on every call."""
    w = maker()
    A = gpu_pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], w.vals)
    x = dev(w.dense_operand(1)[:, 0].copy())
    sp.sp_prepare(A, 1)
    k = sp.sp_tensor_info(A).spmvKernel
    say("case automatic choice", w.shape, w.nnz, "-> kernel", k)
    assert k == expect
    first = None
    for call in range(4):
        y = torch.empty(w.shape[0], dtype=torch.float64, device=DEV)
        sp.sp_matmul(A, x, y)
        torch.cuda.synchronize()
        if first is None:
            first = y
        assert torch.equal(y, first), "call %d differs" % call
