"""GPU storage builder against the CPU checker: every pos / crd / values array bit-exact (through the C ABI)."""
import glob
import itertools
import json
import os
import numpy as np
import pytest
import torch

import oracle
import paper_2202_04305_amd as sp
from gen import workloads as W, prng
from gpu_util import say, dev, gpu_pack, assert_storage_equal

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
LT = {"dense": 0, "compressed": 1}


def _storage_fixtures():
    """The fixtures that print a storage (the others under golden/ belong to other tests)."""
    names = []
    for p in sorted(glob.glob(os.path.join(GOLDEN, "*.json"))):
        with open(p) as f:
            if "level_types" in json.load(f):
                names.append(os.path.basename(p))
    return names


@pytest.mark.parametrize("name", _storage_fixtures())
def test_paper_worked_examples(name):
    say("case", name)
    g = json.load(open(os.path.join(GOLDEN, name)))
    if "dense" in g:
        d = np.asarray(g["dense"], dtype=np.float64)
        coords, vals = [np.nonzero(d)[0].astype(np.int64)], d[np.nonzero(d)[0]]
    else:
        coo = np.asarray(g["coo"], dtype=np.int64).reshape(len(g["values"]), len(g["shape"]))
        coords, vals = [coo[:, k].copy() for k in range(len(g["shape"]))], np.asarray(g["values"], dtype=np.float64)
    p = prng.permutation(3, 1, len(vals))
    A = gpu_pack([LT[x] for x in g["level_types"]], g["dim_ordering"], g["shape"], [c[p] for c in coords], vals[p], 64, 64)
    for l in range(len(g["shape"])):
        if g["pos"][l] is not None:
            assert sp.sp_pos(A, l).cpu().tolist() == g["pos"][l]
            assert sp.sp_crd(A, l).cpu().tolist() == g["crd"][l]
    assert sp.sp_values(A).cpu().tolist() == [float(v) for v in g["values_out"]]


@pytest.mark.parametrize("lt", list(itertools.product([0, 1], repeat=2)))
@pytest.mark.parametrize("order", [(0, 1), (1, 0)])
def test_rank2_every_encoding_and_width(lt, order):
    w = W.cfg2_powerlaw_csr(700, 900, cap=300)
    for pw, cw in [(32, 32), (64, 32), (32, 64), (0, 0)]:
        say("case", lt, order, pw, cw)
        ref = oracle.pack(lt, order, w.shape, [w.rows, w.cols], w.vals, pw, cw)
        A = gpu_pack(lt, order, w.shape, [w.rows, w.cols], w.vals, pw, cw)
        assert_storage_equal(A, ref)
        info = sp.sp_tensor_info(A)
        assert info.nnz == w.nnz and info.nvalues == len(ref.values)


@pytest.mark.parametrize("order", [(0, 1, 2), (2, 0, 1), (1, 2, 0)])
def test_rank3(order):
    rng = np.random.default_rng(3)
    shape = (13, 7, 29)
    lin = rng.choice(int(np.prod(shape)), size=400, replace=False)
    coords = list(np.unravel_index(lin, shape))
    vals = rng.standard_normal(400)
    for lt in itertools.product([0, 1], repeat=3):
        say("case rank3", order, lt)
        ref = oracle.pack(lt, order, shape, coords, vals, 32, 32)
        A = gpu_pack(lt, order, shape, coords, vals, 32, 32)
        assert_storage_equal(A, ref)


@pytest.mark.parametrize("maker,name", [
    (lambda: W.cfg1_uniform_csr(), "cfg1 full"),
    (lambda: W.cfg2_powerlaw_csr(60000, 50000, cap=9000), "cfg2 scaled"),
    (lambda: W.cfg4_hypersparse_dcsr(1 << 18, 1 << 18), "cfg4 scaled"),
    (lambda: W.cfg5_zipf_csc_spmm(40000, 40000, cap=6000), "cfg5 scaled"),
])
def test_workload_shapes(maker, name):
    w = maker()
    say("case", name, w.stats)
    ref = oracle.pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], w.vals, 32, 32)
    A = gpu_pack(w.level_types, w.dim_ordering, w.shape, [w.rows, w.cols], w.vals, 32, 32)
    assert_storage_equal(A, ref)
    assert sp.sp_tensor_info(A).maxSegment == w.stats["max_len"]
    # back to the coordinate scheme: same entries, level order
    coords, vals = sp.sp_unpack(A)
    (r, c), v = ref.unpack()
    assert np.array_equal(coords[0].cpu().numpy(), r) and np.array_equal(coords[1].cpu().numpy(), c)
    assert np.array_equal(vals.cpu().numpy().astype(np.float64), v)


def test_unpack_with_padding_zeros():
    w = W.uniform_random(50, 30, 200)
    for lt, order in [((1, 0), (0, 1)), ((0, 0), (1, 0)), ((1, 0), (1, 0))]:
        say("case unpack", lt, order)
        A = gpu_pack(lt, order, w.shape, [w.rows, w.cols], w.vals)
        ref = oracle.pack(lt, order, w.shape, [w.rows, w.cols], w.vals, 32, 32)
        coords, vals = sp.sp_unpack(A)
        (r, c), v = ref.unpack()
        assert np.array_equal(coords[0].cpu().numpy(), r) and np.array_equal(coords[1].cpu().numpy(), c)
        assert np.array_equal(vals.cpu().numpy(), v)


def test_empty_tiny_and_explicit_zero():
    for lt in [(0, 1), (1, 1), (1, 0), (0, 0)]:
        say("case empty", lt)
        z = np.zeros(0, dtype=np.int64)
        ref = oracle.pack(lt, None, (5, 7), [z, z], np.zeros(0), 32, 32)
        A = gpu_pack(lt, None, (5, 7), [z, z], np.zeros(0), 32, 32)
        assert_storage_equal(A, ref)
    ref = oracle.pack((0, 1), None, (2, 3), [np.array([0, 1]), np.array([2, 1])], np.array([0.0, 4.0]), 32, 32)
    A = gpu_pack((0, 1), None, (2, 3), [np.array([0, 1]), np.array([2, 1])], np.array([0.0, 4.0]), 32, 32)
    assert_storage_equal(A, ref)
    one = gpu_pack((1, 1), (1, 0), (9, 9), [np.array([4]), np.array([6])], np.array([2.5], dtype=np.float32))
    assert_storage_equal(one, oracle.pack((1, 1), (1, 0), (9, 9), [np.array([4]), np.array([6])], np.array([2.5], dtype=np.float32), 32, 32))


def test_input_errors_match_the_checker():
    w = W.uniform_random(100, 100, 3000)
    rows, cols = w.rows.copy(), w.cols.copy()
    rows[1234], cols[1234] = rows[77], cols[77]
    say("case duplicate")
    with pytest.raises(sp.SpError) as e:
        gpu_pack((0, 1), None, w.shape, [rows, cols], w.vals)
    with pytest.raises(oracle.OracleError) as eo:
        oracle.pack((0, 1), None, w.shape, [rows, cols], w.vals)
    assert e.value.code == eo.value.code == oracle.ERR_DUPLICATE
    say("case range")
    cols = w.cols.copy()
    cols[5] = 100
    with pytest.raises(sp.SpError) as e:
        gpu_pack((0, 1), None, w.shape, [w.rows, cols], w.vals)
    assert e.value.code == oracle.ERR_COORD_RANGE
    rows = w.rows.copy()
    rows[9] = -1
    with pytest.raises(sp.SpError) as e:
        gpu_pack((1, 1), (1, 0), w.shape, [rows, w.cols], w.vals)
    assert e.value.code == oracle.ERR_COORD_RANGE
    say("case width")
    with pytest.raises(sp.SpError) as e:
        gpu_pack((0, 1), None, (4, 1 << 33), [np.array([0]), np.array([5])], np.array([1.0]), 32, 32)
    assert e.value.code == oracle.ERR_WIDTH
    with pytest.raises(sp.SpError) as e:
        gpu_pack((0, 0, 0), None, (1 << 30,) * 3, [np.array([0])] * 3, np.array([1.0]))
    assert e.value.code == oracle.ERR_TOO_LARGE
    # the library must still work after errors
    A = gpu_pack((0, 1), None, w.shape, [w.rows, w.cols], w.vals)
    assert_storage_equal(A, oracle.pack((0, 1), None, w.shape, [w.rows, w.cols], w.vals, 32, 32))


def test_convert_between_encodings():
    """The paper's convert operation (Section 4.2), through the coordinate scheme: the result must be what the checker
    packs from the checker's own unpacking of the source, for every pair of rank-2 encodings."""
    w = W.cfg2_powerlaw_csr(300, 200, cap=80)
    encs = [(lt, order) for lt in itertools.product([0, 1], repeat=2) for order in [(0, 1), (1, 0)]]
    for (lt_a, ord_a) in encs:
        A = gpu_pack(lt_a, ord_a, w.shape, [w.rows, w.cols], w.vals, 32, 64)
        ref_a = oracle.pack(lt_a, ord_a, w.shape, [w.rows, w.cols], w.vals, 32, 64)
        (r, c), v = ref_a.unpack()
        for (lt_b, ord_b) in encs:
            say("case convert", lt_a, ord_a, "->", lt_b, ord_b)
            Bt = sp.sp_convert(A, sp.sp_encode(lt_b, ord_b, 64, 32))
            assert_storage_equal(Bt, oracle.pack(lt_b, ord_b, w.shape, [r, c], v, 64, 32))
    # the allocator is shared by source and result: both stay usable after the other is freed
    A = gpu_pack((0, 1), (0, 1), w.shape, [w.rows, w.cols], w.vals)
    Bt = sp.sp_convert(A, sp.sp_encode((1, 1), (1, 0), 32, 32))
    A.free()
    assert_storage_equal(Bt, oracle.pack((1, 1), (1, 0), w.shape, [w.rows, w.cols], w.vals, 32, 32))


@pytest.fixture(params=[0, 2], ids=["sort chosen", "most significant digit first"])
def sort_mode(request):
    """The storage builder's sort: its own choice (least significant digit first at these sizes), and the other one forced."""
    sp.sp_pack_sort_mode(request.param)
    yield request.param
    sp.sp_pack_sort_mode(0)


def test_random_ranks_levels_orderings_and_widths(sort_mode):
    """Seeded random encodings of rank 1 to 6: any mix of level types, any ordering, pos / crd widths from 8 to 64 bits
    (whatever the sizes allow), several sort tiles of entries; the storage bit for bit, then back to coordinates.  Under
    either sort of the builder."""
    rng = np.random.default_rng(220204305)
    done = 0
    while done < 48:
        rank = int(rng.integers(1, 7))
        shape = tuple(int(x) for x in rng.integers(1, [200, 90, 40, 12, 8, 6][rank - 1] + 1, size=rank))
        cells = int(np.prod(shape))
        nnz = int(min(cells, rng.integers(1, 30000)))
        lt = tuple(int(x) for x in rng.integers(0, 2, size=rank))
        order = tuple(int(x) for x in rng.permutation(rank))
        pw, cw = int(rng.choice([8, 16, 32, 64, 0])), int(rng.choice([8, 16, 32, 64, 0]))
        lin = rng.choice(cells, size=nnz, replace=False)
        coords = [c.astype(np.int64) for c in np.unravel_index(lin, shape)]
        vals = rng.standard_normal(nnz)
        try:
            ref = oracle.pack(lt, order, shape, coords, vals, pw, cw)
        except oracle.OracleError as e:
            assert e.code == oracle.ERR_WIDTH          # the drawn widths cannot hold this tensor: the GPU must say the same
            with pytest.raises(sp.SpError) as err:
                gpu_pack(lt, order, shape, coords, vals, pw, cw)
            assert err.value.code == oracle.ERR_WIDTH
            continue
        say("case random", rank, shape, lt, order, pw, cw, nnz)
        A = gpu_pack(lt, order, shape, coords, vals, pw, cw)
        assert_storage_equal(A, ref)
        gc, gv = sp.sp_unpack(A)
        rc, rv = ref.unpack()
        assert all(np.array_equal(g.cpu().numpy(), r) for g, r in zip(gc, rc)) and np.array_equal(gv.cpu().numpy(), rv)
        done += 1
