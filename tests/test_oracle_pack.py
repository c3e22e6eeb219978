"""Pins for the CPU checker's storage builder (no GPU needed).

Each test checks the checker against something other than itself: the arrays the paper
prints (Section 4.1), arrays rebuilt from an enumerated dense tensor by the definition,
storage invariants, and relations between encodings.
"""
import glob
import itertools
import json
import os
import numpy as np
import pytest

import oracle
from gen import workloads as W, prng

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
LT = {"dense": oracle.DENSE, "compressed": oracle.COMPRESSED}


def _load(name):
    return json.load(open(os.path.join(GOLDEN, name)))


def _coo_of(g):
    if "dense" in g:
        d = np.asarray(g["dense"], dtype=np.float64)
        idx = np.nonzero(d)[0]
        return [idx.astype(np.int64)], d[idx]
    coo = np.asarray(g["coo"], dtype=np.int64).reshape(len(g["values"]), len(g["shape"]))
    return [np.ascontiguousarray(coo[:, d]) for d in range(len(g["shape"]))], np.asarray(g["values"], dtype=np.float64)


def _storage_fixtures():
    """The fixtures that print a storage (the others under golden/ belong to other tests)."""
    names = []
    for p in sorted(glob.glob(os.path.join(GOLDEN, "*.json"))):
        with open(p) as f:
            if "level_types" in json.load(f):
                names.append(os.path.basename(p))
    return names


@pytest.mark.parametrize("name", _storage_fixtures())
@pytest.mark.parametrize("shuffle", [False, True])
def test_paper_worked_examples(name, shuffle):
    g = _load(name)
    coords, vals = _coo_of(g)
    if shuffle:  # the result may not depend on the order the entries arrive in
        p = prng.permutation(7, 1, len(vals))
        coords, vals = [c[p] for c in coords], vals[p]
    t = oracle.pack([LT[x] for x in g["level_types"]], g["dim_ordering"], g["shape"], coords, vals)
    for l in range(len(g["shape"])):
        if g["pos"][l] is None:
            assert t.pos[l] is None and t.crd[l] is None
        else:
            assert t.pos[l].tolist() == g["pos"][l], (name, l)
            assert t.crd[l].tolist() == g["crd"][l], (name, l)
    assert t.values.tolist() == [float(v) for v in g["values_out"]]


def _definition_pack(dense, level_types, order):
    """Rebuild pos/crd/values of a small dense tensor directly from the definition of the scheme:
    enumerate level coordinates in lexicographic order and keep, per compressed level, the distinct
    prefixes that lead to a nonzero."""
    rank = dense.ndim
    order = list(range(rank)) if order is None else list(order)
    T = np.transpose(dense, order)           # axes now in level order
    size = T.shape
    pos, crd = [None] * rank, [None] * rank
    parents = [()]                            # stored prefixes (level coords) at the level above
    for l in range(rank):
        children = []
        if level_types[l] == oracle.DENSE:
            for p in parents:
                children += [p + (k,) for k in range(size[l])]
        else:
            pl, cl = [0], []
            for p in parents:
                for k in range(size[l]):
                    sub = T[p + (k,)]
                    if np.any(sub != 0):
                        children.append(p + (k,))
                        cl.append(k)
                pl.append(len(cl))
            pos[l], crd[l] = pl, cl
        parents = children
    values = [float(T[p]) for p in parents]
    return pos, crd, values


@pytest.mark.parametrize("lt", list(itertools.product([oracle.DENSE, oracle.COMPRESSED], repeat=2)))
@pytest.mark.parametrize("order", [None, (0, 1), (1, 0)])
def test_rank2_against_definition(lt, order):
    rng = np.random.default_rng(5)
    for trial in range(6):
        m, n = rng.integers(1, 7, size=2)
        dense = np.where(rng.random((m, n)) < 0.35, rng.integers(1, 50, size=(m, n)).astype(np.float64), 0.0)
        if trial == 0:
            dense[:] = 0.0
        r, c = np.nonzero(dense)
        p = rng.permutation(len(r))
        t = oracle.pack(lt, order, (m, n), [r[p], c[p]], dense[r, c][p])
        pos, crd, values = _definition_pack(dense, lt, order)
        for l in range(2):
            if pos[l] is None:
                assert t.pos[l] is None
            else:
                assert t.pos[l].tolist() == pos[l] and t.crd[l].tolist() == crd[l]
        assert t.values.tolist() == values


@pytest.mark.parametrize("order", list(itertools.permutations(range(3))))
def test_rank3_against_definition(order):
    # dimOrdering[l] = dimension stored at level l: np.transpose(dense, order) puts that dimension at axis l
    rng = np.random.default_rng(11)
    for lt in itertools.product([oracle.DENSE, oracle.COMPRESSED], repeat=3):
        shape = tuple(rng.integers(1, 5, size=3))
        dense = np.where(rng.random(shape) < 0.3, rng.integers(1, 50, size=shape).astype(np.float64), 0.0)
        idx = np.nonzero(dense)
        t = oracle.pack(lt, order, shape, list(idx), dense[idx])
        pos, crd, values = _definition_pack(dense, lt, order)
        for l in range(3):
            if pos[l] is not None:
                assert t.pos[l].tolist() == pos[l] and t.crd[l].tolist() == crd[l]
        assert t.values.tolist() == values


def check_invariants(t, nnz_coo):
    """Storage invariants that hold for any input (Section 4.1)."""
    P = 1
    for l in range(t.rank):
        size = t.shape[(t.order or tuple(range(t.rank)))[l]]
        if t.pos[l] is None:
            P *= size
            continue
        pos, crd = t.pos[l].astype(np.int64), t.crd[l].astype(np.int64)
        assert len(pos) == P + 1 and pos[0] == 0 and pos[-1] == len(crd)
        assert np.all(np.diff(pos) >= 0)
        assert np.all((crd >= 0) & (crd < size)) if len(crd) else True
        inner = np.ones(len(crd), dtype=bool)
        inner[pos[:-1][pos[:-1] < len(crd)]] = False     # first child of each parent: no predecessor
        if len(crd) > 1:
            assert np.all((np.diff(crd) > 0) | ~inner[1:])
        P = len(crd)
    assert len(t.values) == P


@pytest.mark.parametrize("maker", [
    lambda: W.cfg1_uniform_csr(256, 256, 8),
    lambda: W.cfg2_powerlaw_csr(3000, 3000, cap=500),
    lambda: W.cfg4_hypersparse_dcsr(1 << 14, 1 << 14),
    lambda: W.cfg5_zipf_csc_spmm(2048, 2048, cap=300),
])
def test_invariants_and_roundtrip_on_workload_shapes(maker):
    w = maker()
    for lt, order in [(w.level_types, w.dim_ordering), ((1, 1), (1, 0)), ((0, 1), (0, 1)), ((1, 1), (0, 1))]:
        t = oracle.pack(lt, order, w.shape, [w.rows, w.cols], w.vals, 32, 32)
        check_invariants(t, w.nnz)
        (r, c), v = t.unpack()
        # unpack(pack(coo)) == coo sorted in level order
        k0, k1 = (r, c) if tuple(order) == (0, 1) else (c, r)
        key = k0 * max(w.shape) + k1
        assert np.all(np.diff(key) > 0)
        ref = np.lexsort((w.cols, w.rows)) if tuple(order) == (0, 1) else np.lexsort((w.rows, w.cols))
        assert np.array_equal(r, w.rows[ref]) and np.array_equal(c, w.cols[ref])
        assert np.array_equal(v, w.vals[ref].astype(np.float64))


def test_csc_is_csr_of_transpose_and_dcsr_is_csr_without_empty_rows():
    w = W.cfg4_hypersparse_dcsr(4096, 4096, frac=0.05, per_row=5)
    csr = oracle.pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals)
    csc_of_T = oracle.pack((0, 1), (1, 0), w.shape[::-1], [w.cols, w.rows], w.vals)
    assert np.array_equal(csr.pos[1], csc_of_T.pos[1]) and np.array_equal(csr.crd[1], csc_of_T.crd[1])
    assert np.array_equal(csr.values, csc_of_T.values)
    dcsr = oracle.pack((1, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals)
    lens = np.diff(csr.pos[1])
    assert np.array_equal(dcsr.crd[0], np.nonzero(lens)[0])
    assert dcsr.pos[0].tolist() == [0, int((lens > 0).sum())]
    keep = np.concatenate([[True], lens > 0])
    assert np.array_equal(dcsr.pos[1], csr.pos[1][keep])
    assert np.array_equal(dcsr.crd[1], csr.crd[1]) and np.array_equal(dcsr.values, csr.values)
    # against scipy's independent CSR builder
    import scipy.sparse as sp
    s = sp.coo_matrix((w.vals, (w.rows, w.cols)), shape=w.shape).tocsr()
    s.sort_indices()
    assert np.array_equal(csr.pos[1], s.indptr) and np.array_equal(csr.crd[1], s.indices)
    assert np.array_equal(csr.values, s.data)


def test_empty_and_explicit_zero_entries():
    t = oracle.pack((0, 1), None, (5, 7), [np.zeros(0, np.int64)] * 2, np.zeros(0))
    assert t.pos[1].tolist() == [0] * 6 and len(t.crd[1]) == 0 and len(t.values) == 0
    t = oracle.pack((1, 1), None, (5, 7), [np.zeros(0, np.int64)] * 2, np.zeros(0))
    assert t.pos[0].tolist() == [0, 0] and t.pos[1].tolist() == [0]
    # an explicit zero is a stored entry like any other (Section 2.1: explicit zeros are legal)
    t = oracle.pack((0, 1), None, (2, 3), [np.array([0, 1]), np.array([2, 1])], np.array([0.0, 4.0]))
    assert t.pos[1].tolist() == [0, 1, 2] and t.crd[1].tolist() == [2, 1] and t.values.tolist() == [0.0, 4.0]


def test_error_codes_and_precedence():
    r, c, v = np.array([0, 1]), np.array([1, 2]), np.array([1.0, 2.0])

    def code(*a, **k):
        with pytest.raises(oracle.OracleError) as e:
            oracle.pack(*a, **k)
        return e.value.code
    assert code((0, 1), None, (2, 3), [r, c], v, rank=0) == oracle.ERR_RANK
    assert code((0, 1) * 5, None, (2,) * 10, [r] * 10, v) == oracle.ERR_RANK
    assert code((0, 2), None, (2, 3), [r, c], v) == oracle.ERR_LEVEL_TYPE
    assert code((0, 1), (0, 0), (2, 3), [r, c], v) == oracle.ERR_ORDERING
    assert code((0, 1), (0, 2), (2, 3), [r, c], v) == oracle.ERR_ORDERING
    assert code((0, 1), None, (2, 3), [r, c], v, pos_width=12) == oracle.ERR_WIDTH
    assert code((0, 1), None, (2, 3), [r, c], v.astype(np.float16)) == oracle.ERR_DTYPE
    assert code((0, 1), None, (2, 3), [r, np.array([1, 3])], v) == oracle.ERR_COORD_RANGE
    assert code((0, 1), None, (2, 3), [np.array([-1, 1]), c], v) == oracle.ERR_COORD_RANGE
    assert code((0, 1), None, (2, 3), [np.array([1, 1]), np.array([2, 2])], v) == oracle.ERR_DUPLICATE
    # precedence: level type before ordering before width before range before duplicate
    assert code((0, 2), (0, 0), (2, 3), [r, c], v, pos_width=12) == oracle.ERR_LEVEL_TYPE
    assert code((0, 1), (0, 0), (2, 3), [r, c], v, pos_width=12) == oracle.ERR_ORDERING
    assert code((0, 1), None, (2, 3), [np.array([1, 1]), np.array([9, 9])], v) == oracle.ERR_COORD_RANGE
    # dense level sizes whose product overflows int64
    assert code((0, 0, 0), None, (1 << 30,) * 3, [r, r, r], v) == oracle.ERR_TOO_LARGE


def test_bit_widths():
    w = W.uniform_random(40, 300, 200)
    ref = oracle.pack((0, 1), None, w.shape, [w.rows, w.cols], w.vals)
    for pw, cw in itertools.product([0, 16, 32, 64], repeat=2):
        t = oracle.pack((0, 1), None, w.shape, [w.rows, w.cols], w.vals, pw, cw)
        assert t.pos[1].dtype.itemsize * 8 == (pw or 64) and t.crd[1].dtype.itemsize * 8 == (cw or 64)
        assert np.array_equal(t.pos[1], ref.pos[1]) and np.array_equal(t.crd[1], ref.crd[1])
    with pytest.raises(oracle.OracleError) as e:      # 200 stored entries do not fit a signed 8-bit pointer
        oracle.pack((0, 1), None, w.shape, [w.rows, w.cols], w.vals, 8, 32)
    assert e.value.code == oracle.ERR_WIDTH
    with pytest.raises(oracle.OracleError) as e:      # column 299 does not fit a signed 8-bit index
        oracle.pack((0, 1), None, w.shape, [w.rows, w.cols], w.vals, 32, 8)
    assert e.value.code == oracle.ERR_WIDTH
    ok = oracle.pack((0, 1), None, (40, 128), [w.rows[:100], w.cols[:100] % 128 * 0 + np.arange(100) % 128], w.vals[:100], 8, 8)
    assert ok.pos[1].dtype == np.int8 and ok.pos[1][-1] == 100
