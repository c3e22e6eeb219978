"""Helpers for the GPU parity tests: move a workload to the device, pack it through the C ABI, compare with the checker."""
import sys
import numpy as np
import torch

import paper_2202_04305_amd as sp
import oracle

DEV = torch.device("cuda:0")


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def gpu_pack(lt, order, shape, coords, vals, pw=32, cw=32):
    enc = sp.sp_encode(lt, order, pw, cw)
    return sp.sp_pack(enc, shape, [dev(np.asarray(c, dtype=np.int64)) for c in coords], dev(vals))


def assert_storage_equal(A, ref):
    """pos / crd / values of a GPU tensor against the checker's, bit for bit."""
    info = sp.sp_tensor_info(A)
    for l in range(info.rank):
        if ref.pos[l] is None:
            continue
        gp, gc = sp.sp_pos(A, l).cpu().numpy(), sp.sp_crd(A, l).cpu().numpy()
        assert gp.dtype == ref.pos[l].dtype and gc.dtype == ref.crd[l].dtype
        assert np.array_equal(gp, ref.pos[l]), "pos[%d]" % l
        assert np.array_equal(gc, ref.crd[l]), "crd[%d]" % l
    gv = sp.sp_values(A).cpu().numpy()
    assert gv.dtype == ref.values.dtype
    assert gv.tobytes() == ref.values.tobytes(), "values"


def tol_for(dtype):
    return 1e-12 if np.dtype(dtype) == np.float64 else 1e-5


def assert_product_close(Cgpu, Cref, mag, dtype, what=""):
    """|C_gpu - C_ref| <= tol * sum|a*b| per element; elements with mag == 0 must be exactly zero."""
    Cg = Cgpu.detach().cpu().numpy().reshape(Cref.shape).astype(np.float64)
    err = np.abs(Cg - Cref.astype(np.float64))
    bad = err > tol_for(dtype) * mag
    assert not bad.any(), "%s: %d elements outside tolerance, worst err/mag %.3e" % (
        what, int(bad.sum()), float(np.max(err[bad] / np.maximum(mag[bad], 1e-300))))
