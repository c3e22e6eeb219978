"""Seeded synthetic workloads with the shapes of the five benchmark configurations.

Every workload is a COO matrix (int64 rows/cols in a seeded shuffled order, values in
the configuration's dtype), the level-type encoding it is meant to be packed under, and
a recipe for the dense operand B.  Sizes are parameters so that tests can take the same
distributions at sizes a CPU checker finishes in seconds; the defaults are the full
configurations.  Nothing here multiplies or packs anything: it only draws inputs.
"""
from dataclasses import dataclass, field
import numpy as np
from . import prng

BASE_SEED = 2202043050

DENSE, COMPRESSED = 0, 1


@dataclass
class Workload:
    name: str
    shape: tuple            # (m, n) of A
    level_types: tuple      # per level
    dim_ordering: tuple     # dim_ordering[l] = dimension stored at level l
    dtype: type             # np.float64 / np.float32
    rows: np.ndarray        # int64, shuffled order
    cols: np.ndarray
    vals: np.ndarray
    N: int                  # columns of B (1 = SpMV)
    seed: int
    stats: dict = field(default_factory=dict)

    @property
    def nnz(self):
        return int(self.rows.shape[0])

    def dense_operand(self, N=None, exact=False):
        """B, row-major n x N, U[-1,1) (or small integers when `exact`)."""
        N = self.N if N is None else N
        n = self.shape[1]
        if exact:
            b = prng.small_ints(self.seed, 77, n * N, dtype=self.dtype)
        else:
            b = prng.uniform_pm1(self.seed, 7, n * N, dtype=self.dtype)
        return b.reshape(n, N)

    def exact_values(self):
        """Small-integer values with A's pattern: every product and partial sum is exact."""
        return prng.small_ints(self.seed, 78, self.nnz, dtype=self.dtype)


def distinct_sorted_per_segment(seed, stream, seg_len, bound):
    """For each segment s draw seg_len[s] distinct integers of [0, bound), ascending.

    Returns (seg_id, value), both int64 of length sum(seg_len), ordered by (segment, value).
    Draw-all / sort / redraw-the-duplicates until none are left; segments longer than
    bound/2 take a seeded permutation's prefix instead (small cases only).
    """
    seg_len = np.asarray(seg_len, dtype=np.int64)
    assert seg_len.min(initial=0) >= 0 and seg_len.max(initial=0) <= bound
    S = seg_len.shape[0]
    big = np.nonzero(seg_len * 2 > bound)[0]
    small_len = seg_len.copy()
    small_len[big] = 0
    total = int(small_len.sum())
    seg = np.repeat(np.arange(S, dtype=np.int64), small_len)
    key = seg * bound + prng.below(seed, stream, total, bound)
    used = total
    while True:
        key.sort()
        dup = np.nonzero(key[1:] == key[:-1])[0] + 1
        if dup.size == 0:
            break
        key[dup] = (key[dup] // bound) * bound + prng.below(seed, stream, dup.size, bound, offset=used)
        used += dup.size
    if big.size:
        extra = []
        for s in big:
            p = prng.permutation(seed, stream + 1000003 + int(s), bound)[: seg_len[s]]
            extra.append(int(s) * bound + np.sort(p))
        key = np.sort(np.concatenate([key] + extra))
    return key // bound, key % bound


def _finish(name, cfg_id, shape, lt, order, dtype, seg_is_row, seg, inner, N, seed):
    nnz = seg.shape[0]
    vals = prng.uniform_pm1(seed, 3, nnz, dtype=dtype)
    perm = prng.permutation(seed, 5, nnz)
    rows, cols = (seg, inner) if seg_is_row else (inner, seg)
    nseg = shape[0] if seg_is_row else shape[1]
    lens = np.bincount(seg, minlength=nseg)
    stats = {
        "nnz": int(nnz),
        "segments": int(nseg),
        "empty_segments": int((lens == 0).sum()),
        "min_len": int(lens.min()) if nseg else 0,
        "median_len": float(np.median(lens)) if nseg else 0.0,
        "max_len": int(lens.max()) if nseg else 0,
    }
    return Workload(name, tuple(shape), tuple(lt), tuple(order), dtype,
                    np.ascontiguousarray(rows[perm]), np.ascontiguousarray(cols[perm]),
                    np.ascontiguousarray(vals[perm]), N, seed, stats)


def cfg1_uniform_csr(m=4096, n=4096, per_row=8, seed=BASE_SEED + 1):
    """CSR SpMV, exactly `per_row` distinct sorted columns per row, f64."""
    seg, col = distinct_sorted_per_segment(seed, 1, np.full(m, per_row, dtype=np.int64), n)
    return _finish("cfg1_csr_spmv_uniform8", 1, (m, n), (DENSE, COMPRESSED), (0, 1), np.float64,
                   True, seg, col, 1, seed)


def lognormal_lengths(seed, m, mean=16.0, sigma=1.5, lo=1, hi=20000):
    mu = np.log(mean) - 0.5 * sigma * sigma
    z = prng.normal(seed, 11, m)
    return np.clip(np.rint(np.exp(mu + sigma * z)), lo, hi).astype(np.int64)


def cfg2_powerlaw_csr(m=1 << 20, n=1 << 20, mean=16.0, sigma=1.5, cap=20000, N=1, seed=BASE_SEED + 2,
                      name="cfg2_csr_spmv_lognormal"):
    """CSR, lognormal row lengths (mean 16, sigma 1.5, clipped to [1, cap]), f64."""
    cap = min(cap, n)
    lens = lognormal_lengths(seed, m, mean, sigma, 1, cap)
    seg, col = distinct_sorted_per_segment(seed, 1, lens, n)
    return _finish(name, 2, (m, n), (DENSE, COMPRESSED), (0, 1), np.float64, True, seg, col, N, seed)


def cfg3_powerlaw_csr_spmm(m=1 << 20, n=1 << 20, N=64, cap=20000, seed=BASE_SEED + 2):
    """SpMM: the same A as configuration 2 (same seed), B with N columns."""
    return cfg2_powerlaw_csr(m, n, N=N, cap=cap, seed=seed, name="cfg3_csr_spmm_lognormal")


def cfg4_hypersparse_dcsr(m=1 << 23, n=1 << 23, frac=0.01, per_row=32, seed=BASE_SEED + 4):
    """DCSR SpMV: `frac` of the rows non-empty (uniform choice), `per_row` entries each, f64."""
    R = max(1, int(round(frac * m)))
    _, live = distinct_sorted_per_segment(seed, 2, np.array([R], dtype=np.int64), m)
    seg, col = distinct_sorted_per_segment(seed, 1, np.full(R, per_row, dtype=np.int64), n)
    return _finish("cfg4_dcsr_spmv_hypersparse", 4, (m, n), (COMPRESSED, COMPRESSED), (0, 1), np.float64,
                   True, live[seg], col, 1, seed)


def zipf_rank_size_lengths(nseg, total, s=1.2, cap=50000):
    """L_r = min(cap, round(c * r^-s)), r = 1..nseg, with c bisected so that sum(L) ~= total."""
    r = np.arange(1, nseg + 1, dtype=np.float64) ** (-s)
    lo, hi = 0.0, float(total) * 64.0 + 64.0
    for _ in range(200):
        c = 0.5 * (lo + hi)
        if np.minimum(cap, np.rint(c * r)).sum() < total:
            lo = c
        else:
            hi = c
    return np.minimum(cap, np.rint(hi * r)).astype(np.int64)


def cfg5_zipf_csc_spmm(m=1 << 21, n=1 << 21, N=32, per_col_mean=16, cap=50000, seed=BASE_SEED + 5):
    """CSC SpMM in f32: column lengths follow a rank-size Zipf(1.2) law capped at `cap`."""
    cap = min(cap, m)
    lens_by_rank = zipf_rank_size_lengths(n, per_col_mean * n, 1.2, cap)
    col_of_rank = prng.permutation(seed, 9, n)
    lens = np.zeros(n, dtype=np.int64)
    lens[col_of_rank] = lens_by_rank
    seg, row = distinct_sorted_per_segment(seed, 1, lens, m)
    return _finish("cfg5_csc_spmm_zipf_f32", 5, (m, n), (DENSE, COMPRESSED), (1, 0), np.float32,
                   False, seg, row, N, seed)


def uniform_random(m, n, nnz, dtype=np.float64, seed=BASE_SEED + 99, lt=(DENSE, COMPRESSED), order=(0, 1), N=1):
    """`nnz` distinct coordinates uniform over an m x n matrix (small test inputs)."""
    _, lin = distinct_sorted_per_segment(seed, 1, np.array([nnz], dtype=np.int64), m * n)
    return _finish("uniform_random", 0, (m, n), lt, order, dtype, True, lin // n, lin % n, N, seed)


def row_band(n=8192, dense_rows=1000, seed=BASE_SEED + 6, lt=(DENSE, COMPRESSED)):
    """The shape of the paper's SpMV experiment: the first `dense_rows` rows full, the rest empty."""
    seg = np.repeat(np.arange(dense_rows, dtype=np.int64), n)
    col = np.tile(np.arange(n, dtype=np.int64), dense_rows)
    return _finish("row_band", 6, (n, n), lt, (0, 1), np.float64, True, seg, col, 1, seed)


# ---------------------------------------------------------------------------------------
# rank 3: a synthetic stand-in for the knowledge-base tensor of the paper's MTTKRP experiment
# ---------------------------------------------------------------------------------------
@dataclass
class Tensor3Workload:
    name: str
    shape: tuple            # (I, K, L)
    dtype: type
    ci: np.ndarray          # int64 coordinates per dimension, seeded shuffled order
    ck: np.ndarray
    cl: np.ndarray
    vals: np.ndarray
    J: int                  # columns of the factor matrices
    seed: int
    stats: dict = field(default_factory=dict)

    @property
    def nnz(self):
        return int(self.vals.shape[0])

    def factors(self, J=None, exact=False):
        """(C, D): K x J and L x J row-major, U[-1,1) (or small integers when `exact`)."""
        J = self.J if J is None else J
        _, K, L = self.shape
        if exact:
            return (prng.small_ints(self.seed, 81, K * J, lo=-3, hi=3, dtype=self.dtype).reshape(K, J),
                    prng.small_ints(self.seed, 82, L * J, lo=-3, hi=3, dtype=self.dtype).reshape(L, J))
        return (prng.uniform_pm1(self.seed, 8, K * J, dtype=self.dtype).reshape(K, J),
                prng.uniform_pm1(self.seed, 9, L * J, dtype=self.dtype).reshape(L, J))

    def exact_values(self):
        return prng.small_ints(self.seed, 83, self.nnz, lo=-3, hi=3, dtype=self.dtype)


def _distinct_sorted_var(seed, stream, seg_len, bounds):
    """As distinct_sorted_per_segment with a bound of its own per segment (each seg_len[s] <= bounds[s] / 2)."""
    seg_len = np.asarray(seg_len, dtype=np.int64)
    bounds = np.asarray(bounds, dtype=np.int64)
    assert np.all(seg_len * 2 <= bounds) or seg_len.size == 0
    S = seg_len.shape[0]
    top = int(bounds.max(initial=1))
    seg = np.repeat(np.arange(S, dtype=np.int64), seg_len)
    total = seg.shape[0]
    b = bounds[seg]
    key = seg * top + np.minimum((prng.uniform01(seed, stream, total) * b).astype(np.int64), b - 1)
    used = total
    while True:
        key.sort()
        dup = np.nonzero(key[1:] == key[:-1])[0] + 1
        if dup.size == 0:
            break
        sd = key[dup] // top
        bd = bounds[sd]
        key[dup] = sd * top + np.minimum((prng.uniform01(seed, stream, dup.size, offset=used) * bd).astype(np.int64), bd - 1)
        used += dup.size
    return key // top, key % top


def tensor3_slices(I=12092, K=9184, L=28818, nnz=76_879_419, J=42, k_mean=500.0, l_mean=1500.0, sigma=1.0,
                   dtype=np.float64, seed=BASE_SEED + 7, name="mttkrp_tensor3"):
    """I x K x L tensor with the shape, entry count and output width of the paper's MTTKRP experiment.

    Slice i touches a pool of a_i of the K and b_i of the L coordinates (lognormal sizes, seeded choices) and stores a
    uniform sample of that a_i x b_i grid; one density for all slices, set so that the total comes to about `nnz`.
    Both fibre families, (i,k,:) and (i,:,l), therefore have lengths that grow with the slice: the structure the two
    storage orders of the experiment walk."""
    mu_k = np.log(k_mean) - 0.5 * sigma * sigma
    mu_l = np.log(l_mean) - 0.5 * sigma * sigma
    a = np.clip(np.rint(np.exp(mu_k + sigma * prng.normal(seed, 21, I))), 2, max(2, K // 2)).astype(np.int64)
    b = np.clip(np.rint(np.exp(mu_l + sigma * prng.normal(seed, 22, I))), 2, max(2, L // 2)).astype(np.int64)
    cells = a * b
    rho = min(0.45, nnz / float(cells.sum()))
    cnt = np.clip(np.rint(rho * cells), 1, cells // 2).astype(np.int64)
    kseg, kval = distinct_sorted_per_segment(seed, 23, a, K)          # pools, ascending per slice
    lseg, lval = distinct_sorted_per_segment(seed, 24, b, L)
    koff = np.concatenate(([0], np.cumsum(a)))
    loff = np.concatenate(([0], np.cumsum(b)))
    si, cell = _distinct_sorted_var(seed, 25, cnt, cells)
    bi = b[si]
    ck = kval[koff[si] + cell // bi]
    cl = lval[loff[si] + cell % bi]
    n = si.shape[0]
    vals = prng.uniform_pm1(seed, 3, n, dtype=dtype)
    perm = prng.permutation(seed, 5, n)
    fib = np.nonzero(np.concatenate(([True], (si[1:] != si[:-1]) | (ck[1:] != ck[:-1]))))[0]
    flen = np.diff(np.concatenate((fib, [n])))
    stats = {"nnz": int(n), "slices": int(I), "fibres_ik": int(fib.shape[0]), "mean_fibre_ik": float(flen.mean()) if n else 0.0,
             "max_fibre_ik": int(flen.max(initial=0)), "max_slice": int(cnt.max(initial=0)), "median_slice": float(np.median(cnt))}
    return Tensor3Workload(name, (I, K, L), dtype, np.ascontiguousarray(si[perm]), np.ascontiguousarray(ck[perm]),
                           np.ascontiguousarray(cl[perm]), np.ascontiguousarray(vals[perm]), J, seed, stats)


def tensor3_uniform(I, K, L, nnz, J=5, dtype=np.float64, seed=BASE_SEED + 98):
    """Small uniform random rank-3 tensor (distinct coordinates), for tests."""
    _, lin = distinct_sorted_per_segment(seed, 26, np.array([nnz], dtype=np.int64), I * K * L)
    perm = prng.permutation(seed, 5, nnz)
    lin = lin[perm]
    vals = prng.uniform_pm1(seed, 3, nnz, dtype=dtype)
    return Tensor3Workload("tensor3_uniform", (I, K, L), dtype, lin // (K * L), (lin // L) % K, lin % L, vals, J, seed,
                           {"nnz": int(nnz)})
