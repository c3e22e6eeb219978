"""ctypes front end of the CPU checker in oracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the bench's
CPU-baseline leg.  The GPU package never imports this module and this module never
imports the GPU package.  The checker is compiled with gcc on first use.
"""
import ctypes
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_LIB_SANITIZED = os.path.join(_HERE, "liboracle_sanitized.so")

OK, ERR_NULL, ERR_RANK, ERR_LEVEL_TYPE, ERR_ORDERING, ERR_WIDTH, ERR_COORD_RANGE, ERR_DUPLICATE, \
    ERR_SHAPE, ERR_DTYPE, ERR_UNSUPPORTED, ERR_TOO_LARGE, ERR_ALLOC = range(13)
DENSE, COMPRESSED = 0, 1
F32, F64 = 0, 1

_lib = None


def build(force=False):
    """Compile oracle.c into liboracle.so (plain gcc, -O2, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def build_sanitized():
    """The same source under gcc's address and undefined-behaviour sanitizers (host code only; any finding aborts).  A
    process that loads it must have been started with the sanitizer runtime preloaded (see tests/test_oracle_sanitizers.py)."""
    tmp = _LIB_SANITIZED + ".tmp%d" % os.getpid()
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-Wall", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-o", tmp, _SRC, "-lm"])
    os.replace(tmp, _LIB_SANITIZED)
    return _LIB_SANITIZED


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(_LIB_SANITIZED if os.environ.get("ORACLE_SANITIZED") == "1" else build())
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        L.oracle_pack.restype = ci
        L.oracle_pack.argtypes = [ci, vp, vp, ci, ci, vp, i64, vp, vp, ci, ctypes.POINTER(vp)]
        L.oracle_tensor_free.restype = None
        L.oracle_tensor_free.argtypes = [vp]
        for f in ("oracle_pos_len", "oracle_crd_len"):
            getattr(L, f).restype = i64
            getattr(L, f).argtypes = [vp, ci]
        L.oracle_values_len.restype = i64
        L.oracle_values_len.argtypes = [vp]
        for f in ("oracle_get_pos", "oracle_get_crd"):
            getattr(L, f).restype = None
            getattr(L, f).argtypes = [vp, ci, vp]
        L.oracle_get_values.restype = None
        L.oracle_get_values.argtypes = [vp, vp]
        L.oracle_unpack.restype = i64
        L.oracle_unpack.argtypes = [vp, vp, vp]
        L.oracle_matmul_coo.restype = ci
        L.oracle_matmul_coo.argtypes = [i64, i64, i64, vp, vp, vp, ci, vp, i64, i64, vp, i64, ci, vp]
        L.oracle_matmul_storage.restype = ci
        L.oracle_matmul_storage.argtypes = [vp, vp, i64, i64, vp, i64, ci, vp]
        L.oracle_sddmm_coo.restype = ci
        L.oracle_sddmm_coo.argtypes = [i64, i64, i64, i64, vp, vp, vp, ci, vp, i64, vp, i64, vp, vp]
        L.oracle_spgemm_coo.restype = i64
        L.oracle_spgemm_coo.argtypes = [i64, i64, i64, i64, vp, vp, vp, i64, vp, vp, vp, ci, vp, vp, vp, vp]
        L.oracle_mttkrp_coo.restype = ci
        L.oracle_mttkrp_coo.argtypes = [i64, i64, i64, i64, i64, vp, vp, vp, vp, ci, vp, i64, vp, i64, vp, i64, ci, vp]
        L.oracle_matmul_coo_f64seq.restype = ci
        L.oracle_matmul_coo_f64seq.argtypes = [i64, i64, vp, vp, vp, vp, i64, i64, vp, i64]
        _lib = L
    return _lib


class OracleError(Exception):
    def __init__(self, code):
        super().__init__("oracle status %d" % code)
        self.code = code


def _dt(dtype):
    dtype = np.dtype(dtype)
    if dtype == np.float32:
        return F32
    if dtype == np.float64:
        return F64
    raise OracleError(ERR_DTYPE)


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


_INT = {8: np.int8, 16: np.int16, 32: np.int32, 64: np.int64, 0: np.int64}


class Packed:
    """A packed tensor held by the checker: .pos[l] / .crd[l] (None for dense levels), .values."""

    def __init__(self, handle, rank, level_types, order, shape, pw, cw, dtype):
        self._h = handle
        self.rank, self.level_types, self.order, self.shape, self.dtype = rank, level_types, order, shape, np.dtype(dtype)
        L = lib()
        self.pos, self.crd = [], []
        for l in range(rank):
            n = L.oracle_pos_len(handle, l)
            if n < 0:
                self.pos.append(None)
                self.crd.append(None)
                continue
            p = np.empty(n, dtype=_INT[pw])
            L.oracle_get_pos(handle, l, _ptr(p))
            c = np.empty(L.oracle_crd_len(handle, l), dtype=_INT[cw])
            L.oracle_get_crd(handle, l, _ptr(c))
            self.pos.append(p)
            self.crd.append(c)
        self.values = np.empty(L.oracle_values_len(handle), dtype=self.dtype)
        L.oracle_get_values(handle, _ptr(self.values))

    def __del__(self):
        if getattr(self, "_h", None):
            lib().oracle_tensor_free(self._h)
            self._h = None

    def unpack(self):
        """(coords[d] ..., values as f64) for every stored position, storage order."""
        n = self.values.shape[0]
        coords = [np.empty(n, dtype=np.int64) for _ in range(self.rank)]
        arr = (ctypes.c_void_p * self.rank)(*[c.ctypes.data for c in coords])
        vals = np.empty(n, dtype=np.float64)
        got = lib().oracle_unpack(self._h, arr, _ptr(vals))
        assert got == n
        return coords, vals

    def matmul(self, B, accumulate=False, C=None):
        """(C, mag) by walking the storage (rank 2)."""
        B = np.ascontiguousarray(B, dtype=self.dtype)
        if B.ndim == 1:
            B = B.reshape(-1, 1)
        m, N = self.shape[0], B.shape[1]
        Cout = np.zeros((m, N), dtype=self.dtype) if C is None else np.array(C, dtype=self.dtype).reshape(m, N).copy()
        mag = np.zeros((m, N), dtype=np.float64)
        st = lib().oracle_matmul_storage(self._h, _ptr(B), N, max(N, 1), _ptr(Cout), max(N, 1), int(accumulate), _ptr(mag))
        if st != OK:
            raise OracleError(st)
        return Cout, mag


def pack(level_types, dim_ordering, shape, coords, values, pos_width=0, crd_width=0, rank=None, dtype=None):
    """Pack COO (coords[d] = int64 array per dimension) under an encoding.  Raises OracleError(code)."""
    rank = len(shape) if rank is None else rank
    lt = np.asarray(level_types, dtype=np.int32)
    order = None if dim_ordering is None else np.asarray(dim_ordering, dtype=np.int32)
    shp = np.asarray(shape, dtype=np.int64)
    coords = [np.ascontiguousarray(c, dtype=np.int64) for c in coords]
    values = np.ascontiguousarray(values) if dtype is None else np.ascontiguousarray(values, dtype=dtype)
    nnz = int(values.shape[0])
    try:
        dt = _dt(values.dtype)
    except OracleError:
        dt = -1
    arr = (ctypes.c_void_p * max(len(coords), 1))(*[c.ctypes.data for c in coords])
    h = ctypes.c_void_p()
    st = lib().oracle_pack(rank, _ptr(lt), None if order is None else _ptr(order), pos_width, crd_width,
                           _ptr(shp), nnz, arr, _ptr(values), dt, ctypes.byref(h))
    if st != OK:
        raise OracleError(st)
    return Packed(h, rank, tuple(int(x) for x in lt), None if order is None else tuple(int(x) for x in order),
                  tuple(int(x) for x in shp), pos_width, crd_width, values.dtype)


def matmul_coo(shape, rows, cols, vals, B, accumulate=False, C=None):
    """(C, mag): C = A.B (or C += A.B) by the plain definition over the COO triples in the given order."""
    m, n = shape
    vals = np.ascontiguousarray(vals)
    dt = _dt(vals.dtype)
    B = np.ascontiguousarray(B, dtype=vals.dtype)
    if B.ndim == 1:
        B = B.reshape(-1, 1)
    N = B.shape[1]
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    Cout = np.zeros((m, N), dtype=vals.dtype) if C is None else np.array(C, dtype=vals.dtype).reshape(m, N).copy()
    mag = np.zeros((m, N), dtype=np.float64)
    st = lib().oracle_matmul_coo(m, n, rows.shape[0], _ptr(rows), _ptr(cols), _ptr(vals), dt, _ptr(B), N, max(N, 1),
                                 _ptr(Cout), max(N, 1), int(accumulate), _ptr(mag))
    if st != OK:
        raise OracleError(st)
    return Cout, mag


def matmul_coo_f64seq(shape, rows, cols, vals, B):
    m, n = shape
    B = np.ascontiguousarray(B, dtype=np.float64)
    if B.ndim == 1:
        B = B.reshape(-1, 1)
    N = B.shape[1]
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    vals = np.ascontiguousarray(vals, dtype=np.float64)
    C = np.zeros((m, N), dtype=np.float64)
    lib().oracle_matmul_coo_f64seq(m, rows.shape[0], _ptr(rows), _ptr(cols), _ptr(vals), _ptr(B), N, N, _ptr(C), N)
    return C


def sddmm_coo(shape, rows, cols, svals, A, B):
    """(X, mag) per COO triple, caller's order: X = s * (A @ B)[i, j] with A (m, K) and B (K, n) row-major."""
    m, n = shape
    svals = np.ascontiguousarray(svals)
    dt = _dt(svals.dtype)
    A = np.ascontiguousarray(A, dtype=svals.dtype)
    B = np.ascontiguousarray(B, dtype=svals.dtype)
    K = A.shape[1]
    assert A.shape == (m, K) and B.shape == (K, n)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    X = np.zeros(rows.shape[0], dtype=svals.dtype)
    mag = np.zeros(rows.shape[0], dtype=np.float64)
    st = lib().oracle_sddmm_coo(m, n, K, rows.shape[0], _ptr(rows), _ptr(cols), _ptr(svals), dt, _ptr(A), max(K, 1), _ptr(B),
                                max(n, 1), _ptr(X), _ptr(mag))
    if st != OK:
        raise OracleError(st)
    return X, mag


def mttkrp_coo(shape, ci, ck, cl, bvals, C, D, accumulate=False, A=None):
    """(A, mag): A[i,j] = sum_{k,l} B[i,k,l] * D[l,j] * C[k,j] over the COO triples of B (shape I x K x L), C (K, J)
    and D (L, J) row-major, by the plain definition."""
    I, K, L = shape
    bvals = np.ascontiguousarray(bvals)
    dt = _dt(bvals.dtype)
    C = np.ascontiguousarray(C, dtype=bvals.dtype)
    D = np.ascontiguousarray(D, dtype=bvals.dtype)
    J = C.shape[1]
    assert C.shape == (K, J) and D.shape == (L, J)
    ci = np.ascontiguousarray(ci, dtype=np.int64)
    ck = np.ascontiguousarray(ck, dtype=np.int64)
    cl = np.ascontiguousarray(cl, dtype=np.int64)
    Aout = np.zeros((I, J), dtype=bvals.dtype) if A is None else np.array(A, dtype=bvals.dtype).reshape(I, J).copy()
    mag = np.zeros((I, J), dtype=np.float64)
    st = lib().oracle_mttkrp_coo(I, K, L, J, ci.shape[0], _ptr(ci), _ptr(ck), _ptr(cl), _ptr(bvals), dt, _ptr(C), max(J, 1),
                                 _ptr(D), max(J, 1), _ptr(Aout), max(J, 1), int(accumulate), _ptr(mag))
    if st != OK:
        raise OracleError(st)
    return Aout, mag


def spgemm_coo(shape_a, ra, ca, va, shape_b, rb, cb, vb):
    """(rows, cols, vals, mag) of C = A.B for two sparse matrices given as COO triples, in row-major order: every (i, j)
    for which a pair A[i,k], B[k,j] of stored entries exists, by the plain definition."""
    m, kdim = shape_a
    k2, n = shape_b
    assert kdim == k2
    va = np.ascontiguousarray(va)
    dt = _dt(va.dtype)
    vb = np.ascontiguousarray(vb, dtype=va.dtype)
    ra, ca, rb, cb = [np.ascontiguousarray(x, dtype=np.int64) for x in (ra, ca, rb, cb)]
    args = (m, kdim, n, ra.shape[0], _ptr(ra), _ptr(ca), _ptr(va), rb.shape[0], _ptr(rb), _ptr(cb), _ptr(vb), dt)
    cnt = lib().oracle_spgemm_coo(*args, None, None, None, None)
    if cnt < 0:
        raise OracleError(int(-cnt))
    ci, cj = np.empty(cnt, dtype=np.int64), np.empty(cnt, dtype=np.int64)
    cv, mag = np.empty(cnt, dtype=va.dtype), np.empty(cnt, dtype=np.float64)
    got = lib().oracle_spgemm_coo(*args, _ptr(ci), _ptr(cj), _ptr(cv), _ptr(mag))
    assert got == cnt
    return ci, cj, cv, mag


def add_coo(shape, coords_a, vals_a, coords_b, vals_b):
    """(coords, vals, mag) of C = A + B element by element (the example of Section 5.1): C stores every position that A
    or B stores; where both do, the two values are added once in the operands' dtype, so the result is exact to the
    last bit whatever the order.  Positions come out in lexicographic order of the original dimensions."""
    va = np.ascontiguousarray(vals_a)
    vb = np.ascontiguousarray(vals_b, dtype=va.dtype)
    _dt(va.dtype)
    ca = [np.ascontiguousarray(c, dtype=np.int64) for c in coords_a]
    cb = [np.ascontiguousarray(c, dtype=np.int64) for c in coords_b]
    for c, n in zip(ca + cb, list(shape) * 2):
        if c.size and (c.min() < 0 or c.max() >= n):
            raise OracleError(ERR_COORD_RANGE)
    ka = np.ravel_multi_index(ca, shape) if va.size else np.zeros(0, dtype=np.int64)
    kb = np.ravel_multi_index(cb, shape) if vb.size else np.zeros(0, dtype=np.int64)
    if np.unique(ka).size != ka.size or np.unique(kb).size != kb.size:
        raise OracleError(ERR_DUPLICATE)
    keys, inv = np.unique(np.concatenate([ka, kb]), return_inverse=True)
    out = np.zeros(keys.size, dtype=va.dtype)
    mag = np.zeros(keys.size, dtype=np.float64)
    out[inv[:ka.size]] = va                                  # every position at most once per operand
    hit = np.zeros(keys.size, dtype=bool)
    hit[inv[:ka.size]] = True
    ib = inv[ka.size:]
    both = hit[ib]
    out[ib[both]] = out[ib[both]] + vb[both]                 # one addition, in dtype
    out[ib[~both]] = vb[~both]
    mag[inv[:ka.size]] = np.abs(va.astype(np.float64))
    mag[ib] += np.abs(vb.astype(np.float64))
    coords = [c.astype(np.int64) for c in np.unravel_index(keys, shape)] if keys.size else [np.zeros(0, dtype=np.int64) for _ in shape]
    return coords, out, mag
