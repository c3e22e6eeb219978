"""Run by tests/test_api_host_sanitizers.py in a child process that has the AddressSanitizer runtime preloaded: drives the
host-only paths of the C ABI (argument validation, descriptors, status strings, error paths that end before or at the first
device call) through the library built with its host code under ASan + UBSan.  Any sanitizer report aborts the process.
argv[1] = path of the sanitized library."""
import ctypes
import sys

L = ctypes.CDLL(sys.argv[1])
ci, vp, i64 = ctypes.c_int, ctypes.c_void_p, ctypes.c_int64
L.sp_status_str.restype = ctypes.c_char_p
L.sp_status_str.argtypes = [ci]
L.sp_encode.argtypes = [ci, ctypes.POINTER(ci), ctypes.POINTER(ci), ci, ci, ctypes.POINTER(vp)]
L.sp_encoding_free.argtypes = [vp]
L.sp_encoding_free.restype = None
L.sp_pack.argtypes = [vp, ctypes.POINTER(i64), i64, ctypes.POINTER(vp), vp, ci, vp, vp, vp, vp, ctypes.POINTER(vp)]
L.sp_pack_sort_mode.argtypes = [ci]
checks = 0


def expect(got, want, what):
    global checks
    checks += 1
    if got != want:
        print("FAIL %s: status %d, expected %d" % (what, got, want), flush=True)
        sys.exit(1)


def ints(v):
    return (ci * len(v))(*v) if v is not None else None


def encode(lt, order=None, pw=32, cw=32, rank=None):
    out = vp()
    st = L.sp_encode(len(lt) if rank is None else rank, ints(lt), ints(order), pw, cw, ctypes.byref(out))
    return st, out


for code in range(-3, 20):
    assert L.sp_status_str(code)
# descriptors: every rank, both level types, orderings, widths; then every way to get it wrong
handles = []
for rank in range(1, 9):
    for pw, cw in ((0, 0), (8, 16), (32, 64), (64, 32)):
        st, h = encode([(l + rank) % 2 for l in range(rank)], list(reversed(range(rank))), pw, cw)
        expect(st, 0, "encode rank %d" % rank)
        handles.append(h)
expect(encode([0, 1], rank=0)[0], 2, "rank 0")
expect(encode([0] * 9)[0], 2, "rank 9")
expect(encode([0, 7])[0], 3, "level type 7")
expect(encode([0, -1])[0], 3, "level type -1")
expect(encode([0, 1], [0, 0])[0], 4, "ordering repeats")
expect(encode([0, 1], [0, 2])[0], 4, "ordering out of range")
expect(encode([0, 1], [-1, 0])[0], 4, "ordering negative")
expect(encode([0, 1], None, 12, 32)[0], 5, "width 12")
expect(encode([0, 1], None, 32, 128)[0], 5, "width 128")
expect(L.sp_encode(2, None, None, 32, 32, ctypes.byref(vp())), 1, "null level types")
expect(L.sp_encode(2, ints([0, 1]), None, 32, 32, None), 1, "null out")
# sp_pack: everything it rejects before it touches the device
st, enc = encode([0, 1])
shape = (i64 * 2)(4, 5)
out = vp()
null_coords = (vp * 2)(None, None)
expect(L.sp_pack(None, shape, 0, null_coords, None, 1, None, None, None, None, ctypes.byref(out)), 1, "pack: null encoding")
expect(L.sp_pack(enc, None, 0, null_coords, None, 1, None, None, None, None, ctypes.byref(out)), 1, "pack: null shape")
expect(L.sp_pack(enc, shape, 0, null_coords, None, 1, None, None, None, None, None), 1, "pack: null out")
expect(L.sp_pack(enc, shape, 3, null_coords, None, 1, None, None, None, None, ctypes.byref(out)), 1, "pack: entries without arrays")
expect(L.sp_pack(enc, shape, 0, null_coords, None, 7, None, None, None, None, ctypes.byref(out)), 9, "pack: dtype 7")
expect(L.sp_pack(enc, shape, -1, null_coords, None, 1, None, None, None, None, ctypes.byref(out)), 8, "pack: negative count")
neg = (i64 * 2)(4, -5)
expect(L.sp_pack(enc, neg, 0, null_coords, None, 1, None, None, None, None, ctypes.byref(out)), 8, "pack: negative size")
huge = (i64 * 2)(1 << 40, 1 << 40)
st, dd = encode([0, 0])
expect(L.sp_pack(dd, huge, 0, null_coords, None, 1, None, None, None, None, ctypes.byref(out)), 11, "pack: 2^80 dense positions")
L.sp_encoding_free(dd)
# the hooks and the calls that take a tensor: null handles
expect(L.sp_pack_sort_mode(3), 10, "sort mode 3")
expect(L.sp_pack_sort_mode(-1), 10, "sort mode -1")
expect(L.sp_pack_sort_mode(0), 0, "sort mode 0")
for name, nargs in (("sp_tensor_info", 2), ("sp_values", 3), ("sp_pos", 4), ("sp_crd", 4), ("sp_prepare", 3), ("sp_matmul", 8),
                    ("sp_matmul_noalloc", 8), ("sp_unpack", 4), ("sp_convert", 4), ("sp_profile_read", 3)):
    f = getattr(L, name)
    f.argtypes = [vp] * nargs
    expect(f(*([None] * nargs)), 1, name + " with null arguments")
L.sp_encoding_free(enc)
for h in handles:
    L.sp_encoding_free(h)
L.sp_encoding_free(None)
print("host paths ok: %d checks" % checks, flush=True)
