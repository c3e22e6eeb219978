"""ctypes binding of libspmi.so.  Same names as the C ABI; argument marshalling only."""
import ctypes
import os

import torch

from . import build as _build

SP_DENSE, SP_COMPRESSED = 0, 1
SP_F32, SP_F64 = 0, 1
SP_TUNE_SPMV_KERNEL, SP_TUNE_CSC_MODE, SP_TUNE_SPMM_KERNEL, SP_TUNE_PROFILE, SP_TUNE_SPGEMM_KERNEL = 1, 2, 3, 4, 5
SP_MAX_RANK = 8

STATUS_NAMES = ["SP_OK", "SP_ERR_NULL", "SP_ERR_RANK", "SP_ERR_LEVEL_TYPE", "SP_ERR_ORDERING", "SP_ERR_WIDTH",
                "SP_ERR_COORD_RANGE", "SP_ERR_DUPLICATE", "SP_ERR_SHAPE", "SP_ERR_DTYPE", "SP_ERR_UNSUPPORTED",
                "SP_ERR_TOO_LARGE", "SP_ERR_ALLOC", "SP_ERR_HIP"]

EXPORTS = ["sp_encode", "sp_encoding_free", "sp_pack", "sp_tensor_free", "sp_prepare", "sp_matmul", "sp_matmul_noalloc", "sp_pos", "sp_crd", "sp_values",
           "sp_unpack", "sp_convert", "sp_sddmm", "sp_mttkrp", "sp_spgemm", "sp_add", "sp_tensor_info", "sp_tensor_tune", "sp_profile_read", "sp_stream_copy", "sp_stream_read", "sp_pack_sort_mode", "sp_status_str", "sp_last_hip_error"]

_ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p)
_FREE_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p)


class SpInfo(ctypes.Structure):
    _fields_ = [("rank", ctypes.c_int), ("levelTypes", ctypes.c_int * SP_MAX_RANK), ("dimOrdering", ctypes.c_int * SP_MAX_RANK),
                ("posWidth", ctypes.c_int), ("crdWidth", ctypes.c_int), ("dtype", ctypes.c_int),
                ("shape", ctypes.c_int64 * SP_MAX_RANK), ("nnz", ctypes.c_int64), ("nvalues", ctypes.c_int64),
                ("maxSegment", ctypes.c_int64), ("storageBytes", ctypes.c_int64), ("derivedBytes", ctypes.c_int64),
                ("spmvKernel", ctypes.c_int), ("lazyPrepares", ctypes.c_int)]


class SpError(RuntimeError):
    def __init__(self, code, what=""):
        name = STATUS_NAMES[code] if 0 <= code < len(STATUS_NAMES) else str(code)
        extra = ""
        if code == 13 and _lib is not None:
            extra = " (hipError %d)" % _lib.sp_last_hip_error()
        super().__init__("%s%s %s" % (name, extra, what))
        self.code = code


_lib = None


def load_library():
    """Loads libspmi.so; builds it first when there is none or when a source or header is newer than it.  Fails loudly
    when it can neither be loaded nor built: there is no other path."""
    global _lib
    if _lib is not None:
        return _lib
    if _build.is_stale():
        _build.build()
    L = ctypes.CDLL(_build.LIB)
    vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    L.sp_encode.restype = ci
    L.sp_encode.argtypes = [ci, vp, vp, ci, ci, ctypes.POINTER(vp)]
    L.sp_encoding_free.restype = None
    L.sp_encoding_free.argtypes = [vp]
    L.sp_pack.restype = ci
    L.sp_pack.argtypes = [vp, vp, i64, vp, vp, ci, _ALLOC_FN, _FREE_FN, vp, vp, ctypes.POINTER(vp)]
    L.sp_tensor_free.restype = None
    L.sp_tensor_free.argtypes = [vp]
    L.sp_matmul.restype = ci
    L.sp_matmul.argtypes = [vp, vp, i64, i64, vp, i64, ci, vp]
    L.sp_matmul_noalloc.restype = ci
    L.sp_matmul_noalloc.argtypes = [vp, vp, i64, i64, vp, i64, ci, vp]
    L.sp_prepare.restype = ci
    L.sp_prepare.argtypes = [vp, i64, vp]
    for f in (L.sp_pos, L.sp_crd):
        f.restype = ci
        f.argtypes = [vp, ci, ctypes.POINTER(vp), ctypes.POINTER(i64)]
    L.sp_values.restype = ci
    L.sp_values.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(i64)]
    L.sp_unpack.restype = ci
    L.sp_unpack.argtypes = [vp, vp, vp, vp]
    L.sp_add.restype = ci
    L.sp_add.argtypes = [vp, vp, vp, vp, ctypes.POINTER(vp)]
    L.sp_spgemm.restype = ci
    L.sp_spgemm.argtypes = [vp, vp, vp, vp, ctypes.POINTER(vp)]
    L.sp_mttkrp.restype = ci
    L.sp_mttkrp.argtypes = [vp, vp, i64, vp, i64, i64, vp, i64, ci, vp]
    L.sp_sddmm.restype = ci
    L.sp_sddmm.argtypes = [vp, vp, i64, vp, i64, ci, i64, vp, vp]
    L.sp_convert.restype = ci
    L.sp_convert.argtypes = [vp, vp, vp, ctypes.POINTER(vp)]
    L.sp_tensor_info.restype = ci
    L.sp_tensor_info.argtypes = [vp, ctypes.POINTER(SpInfo)]
    L.sp_tensor_tune.restype = ci
    L.sp_tensor_tune.argtypes = [vp, ci, i64]
    L.sp_profile_read.restype = ci
    L.sp_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
    L.sp_stream_copy.restype = ci
    L.sp_stream_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    L.sp_pack_sort_mode.restype = ci
    L.sp_pack_sort_mode.argtypes = [ci]
    L.sp_stream_read.restype = ci
    L.sp_stream_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    L.sp_status_str.restype = ctypes.c_char_p
    L.sp_status_str.argtypes = [ci]
    L.sp_last_hip_error.restype = ci
    L.sp_last_hip_error.argtypes = []
    _lib = L
    return L


def _check(code, what=""):
    if code != 0:
        raise SpError(code, what)


def _stream_ptr():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


class _TorchAllocator:
    """Backs the library's allocator callbacks with torch's caching allocator (uint8 tensors kept alive by address)."""

    def __init__(self, device):
        self.device = device
        self.live = {}
        self.alloc_cb = _ALLOC_FN(self._alloc)
        self.free_cb = _FREE_FN(self._free)

    def _alloc(self, nbytes, _ctx):
        try:
            t = torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=self.device)
        except Exception:          # out of memory: the library turns NULL into SP_ERR_ALLOC
            return None
        self.live[t.data_ptr()] = t
        return t.data_ptr()

    def _free(self, ptr, _ctx):
        self.live.pop(ptr, None)


class Encoding:
    def __init__(self, handle, rank):
        self._h, self.rank = handle, rank

    def __del__(self):
        if self._h and _lib is not None:
            _lib.sp_encoding_free(self._h)
            self._h = None


class Tensor:
    def __init__(self, handle, allocator, dtype, device):
        self._h, self._allocator, self.dtype, self.device = handle, allocator, dtype, device

    def free(self):
        if self._h and _lib is not None:
            _lib.sp_tensor_free(self._h)
            self._h = None

    def __del__(self):
        self.free()


def sp_encode(level_types, dim_ordering=None, pos_width=0, crd_width=0, rank=None):
    L = load_library()
    rank = len(level_types) if rank is None else rank
    lt = (ctypes.c_int * max(len(level_types), 1))(*[int(x) for x in level_types])
    order = None
    if dim_ordering is not None:
        order = (ctypes.c_int * max(len(dim_ordering), 1))(*[int(x) for x in dim_ordering])
    h = ctypes.c_void_p()
    _check(L.sp_encode(rank, lt, order, pos_width, crd_width, ctypes.byref(h)), "in sp_encode")
    return Encoding(h, rank)


def _dt(t):
    if t.dtype == torch.float64:
        return SP_F64
    if t.dtype == torch.float32:
        return SP_F32
    return -1


def sp_pack(enc, shape, coords, values, allocator=None):
    """coords: one int64 device tensor per dimension; values: device tensor (f32/f64).  allocator: an object with
    alloc_cb / free_cb (ctypes callbacks) that outlives the tensor; default: torch's caching allocator."""
    L = load_library()
    assert values.is_cuda and all(c.is_cuda and c.dtype == torch.int64 and c.is_contiguous() for c in coords)
    assert values.is_contiguous()
    nnz = int(values.shape[0])
    shp = (ctypes.c_int64 * max(len(shape), 1))(*[int(s) for s in shape])
    carr = (ctypes.c_void_p * max(len(coords), 1))(*[c.data_ptr() for c in coords])
    allocator = allocator or _TorchAllocator(values.device)
    h = ctypes.c_void_p()
    code = L.sp_pack(enc._h, shp, nnz, carr, values.data_ptr(), _dt(values), allocator.alloc_cb, allocator.free_cb, None,
                     _stream_ptr(), ctypes.byref(h))
    _check(code, "in sp_pack")
    return Tensor(h, allocator, values.dtype, values.device)


def sp_prepare(A, N=1):
    """The inspector step: builds and keeps whatever a product of A with N columns needs (synchronises)."""
    L = load_library()
    _check(L.sp_prepare(A._h, int(N), _stream_ptr()), "in sp_prepare")
    return A


def sp_matmul(A, B, C, accumulate=False, N=None, ldb=None, ldc=None):
    """C = A.B (or C += A.B).  B: (n, N) or (n,), C: (m, N) or (m,), row-major device tensors of A's dtype."""
    L = load_library()
    assert B.is_cuda and C.is_cuda and B.dtype == A.dtype and C.dtype == A.dtype
    if N is None:
        N = 1 if B.dim() == 1 else int(B.shape[1])
    if ldb is None:
        ldb = 1 if B.dim() == 1 else int(B.stride(0))
    if ldc is None:
        ldc = 1 if C.dim() == 1 else int(C.stride(0))
    _check(L.sp_matmul(A._h, B.data_ptr(), N, ldb, C.data_ptr(), ldc, int(bool(accumulate)), _stream_ptr()), "in sp_matmul")
    return C


def sp_matmul_noalloc(A, B, C, accumulate=False):
    """sp_matmul through the entry point that allocates nothing (SpMM of a CSR / DCSR tensor, scratch inside the library)."""
    L = load_library()
    assert B.is_cuda and C.is_cuda and B.dtype == A.dtype and C.dtype == A.dtype and B.dim() == 2 and C.dim() == 2
    _check(L.sp_matmul_noalloc(A._h, B.data_ptr(), int(B.shape[1]), int(B.stride(0)), C.data_ptr(), int(C.stride(0)), int(bool(accumulate)),
                               _stream_ptr()), "in sp_matmul_noalloc")
    return C


_INT = {8: torch.int8, 16: torch.int16, 32: torch.int32, 64: torch.int64}


def sp_tensor_info(A):
    L = load_library()
    info = SpInfo()
    _check(L.sp_tensor_info(A._h, ctypes.byref(info)))
    return info


def _view(A, ptr, length, dtype):
    """Borrowed torch view of an array the library allocated through the tensor's allocator (valid until A is freed)."""
    if length == 0:
        return torch.empty(0, dtype=dtype, device=A.device)
    owner = A._allocator.live[ptr]
    return owner[: length * torch.empty(0, dtype=dtype).element_size()].view(dtype)


def sp_pos(A, level):
    """pos[level] as a borrowed device tensor (int32/int64)."""
    L = load_library()
    p, n = ctypes.c_void_p(), ctypes.c_int64()
    _check(L.sp_pos(A._h, level, ctypes.byref(p), ctypes.byref(n)), "in sp_pos")
    return _view(A, p.value, n.value, _INT[sp_tensor_info(A).posWidth])


def sp_crd(A, level):
    L = load_library()
    p, n = ctypes.c_void_p(), ctypes.c_int64()
    _check(L.sp_crd(A._h, level, ctypes.byref(p), ctypes.byref(n)), "in sp_crd")
    return _view(A, p.value, n.value, _INT[sp_tensor_info(A).crdWidth])


def sp_values(A):
    L = load_library()
    p, n = ctypes.c_void_p(), ctypes.c_int64()
    _check(L.sp_values(A._h, ctypes.byref(p), ctypes.byref(n)), "in sp_values")
    return _view(A, p.value, n.value, A.dtype)


def sp_unpack(A):
    """(coords per dimension, values): every stored position in storage order, as device tensors."""
    L = load_library()
    info = sp_tensor_info(A)
    n = info.nvalues
    coords = [torch.empty(n, dtype=torch.int64, device=A.device) for _ in range(info.rank)]
    vals = torch.empty(n, dtype=A.dtype, device=A.device)
    carr = (ctypes.c_void_p * info.rank)(*[c.data_ptr() for c in coords])
    _check(L.sp_unpack(A._h, carr, vals.data_ptr(), _stream_ptr()), "in sp_unpack")
    return coords, vals


def sp_sddmm(S, A, B, X=None, b_is_transposed=False):
    """X[p] = S.values[p] * (A @ B)[i, j] for every stored position p = (i, j) of S.  A: (m, K); B: (K, n), or (n, K) when
    b_is_transposed.  Returns X (storage order)."""
    L = load_library()
    assert A.is_cuda and B.is_cuda and A.dtype == S.dtype and B.dtype == S.dtype and A.dim() == 2 and B.dim() == 2
    K = int(A.shape[1])
    if X is None:
        X = torch.empty(sp_tensor_info(S).nvalues, dtype=S.dtype, device=S.device)
    _check(L.sp_sddmm(S._h, A.data_ptr(), int(A.stride(0)), B.data_ptr(), int(B.stride(0)), int(bool(b_is_transposed)), K,
                      X.data_ptr(), _stream_ptr()), "in sp_sddmm")
    return X


def sp_mttkrp(B, C, D, A=None, accumulate=False):
    """A[i,j] = sum_{k,l} B[i,k,l] * D[l,j] * C[k,j] for a packed rank-3 tensor B.  C: (K, J), D: (L, J); returns A (I, J)."""
    L = load_library()
    assert C.is_cuda and D.is_cuda and C.dtype == B.dtype and D.dtype == B.dtype and C.dim() == 2 and D.dim() == 2
    assert C.shape[1] == D.shape[1] and C.stride(1) == 1 and D.stride(1) == 1
    J = int(C.shape[1])
    info = sp_tensor_info(B)
    if A is None:
        assert not accumulate
        A = torch.empty((info.shape[0], J), dtype=B.dtype, device=B.device)
    assert A.is_cuda and A.dtype == B.dtype and A.shape == (info.shape[0], J) and (J == 0 or A.stride(1) == 1)
    _check(L.sp_mttkrp(B._h, C.data_ptr(), int(C.stride(0)), D.data_ptr(), int(D.stride(0)), J,
                       A.data_ptr(), int(A.stride(0)), int(bool(accumulate)), _stream_ptr()), "in sp_mttkrp")
    return A


def sp_convert(A, enc):
    """A new tensor with A's stored entries under another encoding."""
    h = ctypes.c_void_p()
    _check(load_library().sp_convert(A._h, enc._h, _stream_ptr(), ctypes.byref(h)), "in sp_convert")
    return Tensor(h, A._allocator, A.dtype, A.device)


def sp_spgemm(A, B, enc):
    """C = A.B for two packed sparse matrices, as a new tensor under `enc` (it lives in A's allocator)."""
    h = ctypes.c_void_p()
    _check(load_library().sp_spgemm(A._h, B._h, enc._h, _stream_ptr(), ctypes.byref(h)), "in sp_spgemm")
    return Tensor(h, A._allocator, A.dtype, A.device)


def sp_add(A, B, enc):
    """C = A + B element by element, as a new tensor under `enc` (it lives in A's allocator)."""
    h = ctypes.c_void_p()
    _check(load_library().sp_add(A._h, B._h, enc._h, _stream_ptr(), ctypes.byref(h)), "in sp_add")
    return Tensor(h, A._allocator, A.dtype, A.device)


def sp_tensor_tune(A, key, value):
    _check(load_library().sp_tensor_tune(A._h, key, value), "in sp_tensor_tune")


def sp_profile_read(A):
    """(total milliseconds, launches) of the main kernels recorded since the last read."""
    ms, n = ctypes.c_double(), ctypes.c_int64()
    _check(load_library().sp_profile_read(A._h, ctypes.byref(ms), ctypes.byref(n)), "in sp_profile_read")
    return ms.value, n.value


def sp_stream_copy(dst, src):
    nbytes = src.numel() * src.element_size()
    _check(load_library().sp_stream_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream_ptr()), "in sp_stream_copy")


def sp_stream_read(src, sink):
    nbytes = src.numel() * src.element_size()
    _check(load_library().sp_stream_read(src.data_ptr(), nbytes, sink.data_ptr(), _stream_ptr()), "in sp_stream_read")


def sp_pack_sort_mode(mode):
    """0 = the storage builder chooses its sort, 1 = least significant digit first, 2 = most significant digit first."""
    _check(load_library().sp_pack_sort_mode(int(mode)), "in sp_pack_sort_mode")
