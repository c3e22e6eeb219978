"""GPU element-wise sum of two sparse tensors (the example of Section 5.1) against the CPU checker, through the C ABI:
the storage of the result bit for bit (one IEEE addition per position that both operands store)."""
import itertools

import numpy as np
import pytest

import oracle
import paper_2202_04305_amd as sp
from gen import workloads as W, prng
from gpu_util import say, gpu_pack, assert_storage_equal
from test_oracle_add import two

pytestmark = pytest.mark.gpu


def reference(shape, enc_a, enc_b, enc_c, ca, va, cb, vb, pw=32, cw=32):
    """What the operands store (padding zeros of dense levels included) added by the checker, packed by the checker."""
    Pa = oracle.pack(enc_a[0], enc_a[1], shape, ca, va, pw, cw)
    Pb = oracle.pack(enc_b[0], enc_b[1], shape, cb, vb, pw, cw)
    (sa, xa), (sb, xb) = Pa.unpack(), Pb.unpack()
    coords, vals, _ = oracle.add_coo(shape, sa, xa.astype(va.dtype), sb, xb.astype(va.dtype))
    return oracle.pack(enc_c[0], enc_c[1], shape, coords, vals, pw, cw)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_add_matrices_in_every_pair_of_compressed_formats(dtype):
    shape = (700, 900)
    ca, va, cb, vb = two(shape, 40000, 50000, dtype)
    encs = [((0, 1), (0, 1)), ((1, 1), (0, 1)), ((0, 1), (1, 0)), ((1, 1), (1, 0))]
    for ea, eb in itertools.product(encs, repeat=2):
        ec = encs[(encs.index(ea) + encs.index(eb)) % 4]
        say("case add", ea, eb, "->", ec, dtype.__name__)
        A = gpu_pack(*ea, shape, ca, va)
        B = gpu_pack(*eb, shape, cb, vb)
        C = sp.sp_add(A, B, sp.sp_encode(*ec, 32, 32))
        assert_storage_equal(C, reference(shape, ea, eb, ec, ca, va, cb, vb))


def test_add_the_papers_example_format_and_other_ranks():
    # (compressed, dense) for all three tensors as in the paper's example: whole rows are stored, zeros included
    shape = (300, 64)
    ca, va, cb, vb = two(shape, 900, 700)
    cd = ((1, 0), (0, 1))
    C = sp.sp_add(gpu_pack(*cd, shape, ca, va), gpu_pack(*cd, shape, cb, vb), sp.sp_encode(*cd, 32, 32))
    assert_storage_equal(C, reference(shape, cd, cd, cd, ca, va, cb, vb))
    # a vector, a rank-3 tensor with mixed level types and orderings, 64-bit arrays
    for shape, ea, eb, ec in [((5000,), ((1,), (0,)), ((1,), (0,)), ((1,), (0,))),
                              ((30, 40, 50), ((0, 1, 1), (0, 1, 2)), ((1, 1, 1), (2, 0, 1)), ((1, 1, 1), (0, 2, 1))),
                              ((30, 40, 50), ((1, 0, 1), (1, 0, 2)), ((0, 1, 1), (0, 1, 2)), ((0, 1, 1), (0, 1, 2)))]:
        cells = int(np.prod(shape))
        ca, va, cb, vb = two(shape, cells // 10, cells // 8, seed=len(shape))
        say("case add rank", len(shape), ea, eb, ec)
        for pw, cw in [(32, 32), (64, 64)]:
            C = sp.sp_add(gpu_pack(*ea, shape, ca, va, pw, cw), gpu_pack(*eb, shape, cb, vb, pw, cw), sp.sp_encode(*ec, pw, cw))
            assert_storage_equal(C, reference(shape, ea, eb, ec, ca, va, cb, vb, pw, cw))


def test_add_cancellation_empty_operands_and_errors():
    shape = (50, 60)
    ca, va, cb, vb = two(shape, 400, 300)
    csr = ((0, 1), (0, 1))
    enc = sp.sp_encode(*csr, 32, 32)
    A, B = gpu_pack(*csr, shape, ca, va), gpu_pack(*csr, shape, cb, vb)
    Z = sp.sp_add(A, gpu_pack(*csr, shape, ca, -va), enc)                  # A + (-A): every position stays, value zero
    assert sp.sp_tensor_info(Z).nvalues == 400 and bool((sp.sp_values(Z) == 0).all())
    e = [np.zeros(0, dtype=np.int64)] * 2
    E = gpu_pack(*csr, shape, e, np.zeros(0))
    assert_storage_equal(sp.sp_add(A, E, enc), oracle.pack(*csr, shape, ca, va, 32, 32))
    assert_storage_equal(sp.sp_add(E, B, enc), oracle.pack(*csr, shape, cb, vb, 32, 32))
    assert sp.sp_tensor_info(sp.sp_add(E, E, enc)).nvalues == 0
    # the sum is an ordinary tensor: add again, C = (A + B) + A = 2A + B
    C2 = sp.sp_add(sp.sp_add(A, B, enc), A, enc)
    coords, vals, _ = oracle.add_coo(shape, *oracle.add_coo(shape, ca, va, cb, vb)[:2], ca, va)
    assert_storage_equal(C2, oracle.pack(*csr, shape, coords, vals, 32, 32))
    with pytest.raises(sp.SpError) as err:
        sp.sp_add(A, gpu_pack(*csr, (50, 61), cb, vb), enc)
    assert err.value.code == 8
    with pytest.raises(sp.SpError) as err:
        sp.sp_add(A, gpu_pack(*csr, shape, cb, vb.astype(np.float32)), enc)
    assert err.value.code == 9
    with pytest.raises(sp.SpError) as err:
        sp.sp_add(A, gpu_pack((1,), (0,), (50,), [ca[0][:1]], va[:1]), enc)
    assert err.value.code == 2
