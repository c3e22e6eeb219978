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
