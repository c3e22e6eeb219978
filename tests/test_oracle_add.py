"""Pins for the CPU checker's element-wise sum of two sparse tensors (the example of Section 5.1).  No GPU needed."""
import numpy as np
import pytest

import oracle
from gen import workloads as W, prng


def two(shape, na, nb, dtype=np.float64, seed=0):
    cells = int(np.prod(shape))
    _, la = W.distinct_sorted_per_segment(W.BASE_SEED + 700 + seed, 1, np.array([na], dtype=np.int64), cells)
    _, lb = W.distinct_sorted_per_segment(W.BASE_SEED + 710 + seed, 1, np.array([nb], dtype=np.int64), cells)
    pa, pb = prng.permutation(seed, 1, na), prng.permutation(seed, 2, nb)
    ca = [c[pa] for c in np.unravel_index(la, shape)]
    cb = [c[pb] for c in np.unravel_index(lb, shape)]
    return ca, prng.uniform_pm1(seed, 3, na, dtype=dtype), cb, prng.uniform_pm1(seed, 4, nb, dtype=dtype)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("shape", [(40,), (17, 23), (5, 6, 7)])
def test_against_dense_numpy(dtype, shape):
    cells = int(np.prod(shape))
    ca, va, cb, vb = two(shape, cells // 3, cells // 4, dtype)
    coords, vals, mag = oracle.add_coo(shape, ca, va, cb, vb)
    Da, Db = np.zeros(shape, dtype=dtype), np.zeros(shape, dtype=dtype)
    Da[tuple(ca)] = va
    Db[tuple(cb)] = vb
    Sa, Sb = np.zeros(shape, dtype=bool), np.zeros(shape, dtype=bool)
    Sa[tuple(ca)] = True
    Sb[tuple(cb)] = True
    want = np.nonzero(Sa | Sb)                                   # the union of the stored positions, lexicographic
    assert all(np.array_equal(c, w) for c, w in zip(coords, want))
    assert vals.dtype == dtype and np.array_equal(vals, (Da + Db)[want])          # one IEEE addition: bit for bit
    assert np.allclose(mag, (np.abs(Da.astype(np.float64)) + np.abs(Db.astype(np.float64)))[want], rtol=1e-15, atol=0)


def test_closed_forms():
    shape = (9, 11)
    ca, va, cb, vb = two(shape, 30, 40)
    # A + (-A): every position stays stored, with value zero
    coords, vals, _ = oracle.add_coo(shape, ca, va, ca, -va)
    assert vals.size == 30 and np.all(vals == 0.0)
    # commutative to the bit, whatever the order of the triples
    c1, v1, _ = oracle.add_coo(shape, ca, va, cb, vb)
    p = prng.permutation(3, 9, 40)
    c2, v2, _ = oracle.add_coo(shape, [c[p] for c in cb], vb[p], ca, va)
    assert all(np.array_equal(x, y) for x, y in zip(c1, c2)) and np.array_equal(v1, v2)
    # an empty operand: the other one, sorted
    e = [np.zeros(0, dtype=np.int64)] * 2
    c3, v3, _ = oracle.add_coo(shape, ca, va, e, np.zeros(0))
    order = np.lexsort((ca[1], ca[0]))
    assert np.array_equal(c3[0], ca[0][order]) and np.array_equal(c3[1], ca[1][order]) and np.array_equal(v3, va[order])
    # disjoint patterns: a plain merge
    c4, v4, _ = oracle.add_coo((4,), [np.array([0, 2])], np.array([1.0, 2.0]), [np.array([3, 1])], np.array([4.0, 3.0]))
    assert np.array_equal(c4[0], [0, 1, 2, 3]) and np.array_equal(v4, [1.0, 3.0, 2.0, 4.0])


def test_errors():
    with pytest.raises(oracle.OracleError) as e:
        oracle.add_coo((3, 3), [np.array([3]), np.array([0])], np.ones(1), [np.array([0]), np.array([0])], np.ones(1))
    assert e.value.code == oracle.ERR_COORD_RANGE
    with pytest.raises(oracle.OracleError) as e:
        oracle.add_coo((3, 3), [np.array([1, 1]), np.array([2, 2])], np.ones(2), [np.array([0]), np.array([0])], np.ones(1))
    assert e.value.code == oracle.ERR_DUPLICATE
