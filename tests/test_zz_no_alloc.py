"""The entry point that allocates nothing (sp_matmul_noalloc): its result against sp_matmul's, bit for bit, on two calls
in a row, the second on a smaller input (the scratch inside the library keeps the first call's contents), plus the limit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_04305_amd as sp
from paper_2202_04305_amd import binding
from gen import workloads as W
from gpu_util import say, dev, gpu_pack, assert_product_close, DEV

pytestmark = pytest.mark.gpu


class _CountingAllocator(binding._TorchAllocator):
    def __init__(self, device):
        super().__init__(device)
        self.calls = 0

    def _alloc(self, nbytes, ctx):
        self.calls += 1
        return super()._alloc(nbytes, ctx)


def test_no_alloc_entry_point_matches_sp_matmul_on_two_calls_in_a_row():
    cases = [(W.cfg2_powerlaw_csr(200000, 150000, cap=20000), (0, 1), 16, np.float64),       # long rows cross many blocks
             (W.cfg4_hypersparse_dcsr(1 << 18, 1 << 18, frac=0.02, per_row=40), (1, 1), 8, np.float64)]   # smaller, DCSR: rows that are not stored
    for w, lt, N, dt in cases:
        say("case no-alloc", w.shape, w.nnz, lt, N)
        alloc = _CountingAllocator(DEV)
        enc = sp.sp_encode(lt, (0, 1), 32, 32)
        A = sp.sp_pack(enc, w.shape, [dev(w.rows), dev(w.cols)], dev(w.vals), allocator=alloc)
        Bh = w.dense_operand(N)
        Bd = dev(Bh)
        for accumulate in (False, True):
            C0 = torch.randn((w.shape[0], N), dtype=torch.float64, device=DEV)
            want = C0.clone()
            sp.sp_matmul(A, Bd, want, accumulate=accumulate)
            torch.cuda.synchronize()
            before = alloc.calls
            got = C0.clone()
            sp.sp_matmul_noalloc(A, Bd, got, accumulate=accumulate)
            torch.cuda.synchronize()
            assert alloc.calls == before, "the entry point went to the allocator"
            assert torch.equal(got, want), "differs from sp_matmul (accumulate=%s)" % accumulate
        ref, mag = oracle.matmul_coo(w.shape, w.rows, w.cols, w.vals, Bh)
        C = torch.full((w.shape[0], N), float("nan"), dtype=torch.float64, device=DEV)
        sp.sp_matmul_noalloc(A, Bd, C)
        assert_product_close(C, ref, mag, dt, "no-alloc entry point vs the checker")
        A.free()


def test_no_alloc_entry_point_rejects_what_it_cannot_do():
    w = W.cfg2_powerlaw_csr(300000, 1000, mean=30.0, cap=900)                  # 9 M entries: 8,800 blocks
    A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals)
    nb = -(-w.nnz // 1024)
    N = 256                                                                    # more than 64 16-byte pieces per row
    B, C = torch.zeros((w.shape[1], N), dtype=torch.float64, device=DEV), torch.zeros((w.shape[0], N), dtype=torch.float64, device=DEV)
    with pytest.raises(sp.SpError) as e:
        sp.sp_matmul_noalloc(A, B, C)
    assert e.value.code == 10
    N = 64                                                                     # the widest row the kernel takes in f64
    assert nb * N * 8 <= 16 << 20
    B64, C64 = torch.zeros((w.shape[1], N), dtype=torch.float64, device=DEV), torch.zeros((w.shape[0], N), dtype=torch.float64, device=DEV)
    sp.sp_matmul_noalloc(A, B64, C64)                                          # 4.6 MB of carries: fits
    w2 = W.cfg2_powerlaw_csr(1 << 20, 4096, mean=40.0, cap=2000)               # 42 M entries x 64 columns x 8 bytes = 21 MB of carries
    A2 = gpu_pack((0, 1), (0, 1), w2.shape, [w2.rows, w2.cols], w2.vals)
    assert -(-w2.nnz // 1024) * N * 8 > 16 << 20
    B2, C2 = torch.zeros((w2.shape[1], N), dtype=torch.float64, device=DEV), torch.zeros((w2.shape[0], N), dtype=torch.float64, device=DEV)
    with pytest.raises(sp.SpError) as e:
        sp.sp_matmul_noalloc(A2, B2, C2)
    assert e.value.code == 11                                                  # SP_ERR_TOO_LARGE
    Acsc = gpu_pack((0, 1), (1, 0), w.shape, [w.rows, w.cols], w.vals)
    with pytest.raises(sp.SpError) as e:
        sp.sp_matmul_noalloc(Acsc, B[:, :8].contiguous(), C[:, :8].contiguous())
    assert e.value.code == 10                                                  # column-major: SP_ERR_UNSUPPORTED
