// Sparse times sparse with a sparse result, C[i,j] = sum_k A[i,k] * B[k,j] (arXiv 2202.04305, Sections 4.2 and 4.4: the
// SpMSpM kernel, whose generated loop walks A row by row, expands a row of C into a dense workspace and compresses it
// back in index order).  An entry (i,j) of C is stored when a pair A[i,k], B[k,j] of stored entries exists.
//
// On the GPU the insertion is done for all rows at once with the storage builder: every pair becomes one
// (key, product) record, key = the position of (i,j) in C's level order, and the builder's stable radix sort, a pass
// that adds up records of equal key in sorted order, and its level sweep produce C under any encoding.  The records
// are written in the order of A's stored entries and, inside one entry, of B's row, so the sum of an element of C
// runs over k in A's storage order: for a row-major A exactly the order of the paper's loop, and the same bits on
// every call.  Cost: 16 bytes per pair, written once and sorted; no per-row workspace, no atomics, no limit on n.
#include "spmi_internal.h"

namespace {

constexpr int kThreads = 256;

// pairs[p] = stored entries in row k = cols[p] of B; bstart[p] = where that row begins in B's crd / values.
// B is row-major with a compressed inner level; its outer level is dense (pos0 = nullptr) or compressed.
template <typename PT, typename CT>
__global__ __launch_bounds__(kThreads) void spgemm_count_kernel(const int64_t *__restrict__ cols, int64_t na, const PT *__restrict__ bpos0,
                                                                const CT *__restrict__ bcrd0, int64_t nrows0, const PT *__restrict__ bpos1,
                                                                unsigned long long *__restrict__ pairs, int64_t *__restrict__ bstart)
{
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p > na) return;
    if (p == na) { pairs[p] = 0; return; }          // sentinel: after the exclusive scan it holds the total
    const int64_t k = cols[p];
    int64_t q = k;
    if (bcrd0) {                                    // compressed outer level: look the row up
        int64_t lo = 0, hi = nrows0;
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if ((int64_t)bcrd0[mid] < k) lo = mid + 1; else hi = mid;
        }
        q = (lo < nrows0 && (int64_t)bcrd0[lo] == k) ? lo : -1;
    }
    if (q < 0) { pairs[p] = 0; bstart[p] = 0; return; }
    const int64_t a = (int64_t)bpos1[q], b = (int64_t)bpos1[q + 1];
    pairs[p] = (unsigned long long)(b - a);
    bstart[p] = a;
}

// A wave per stored entry of A: one record per entry of B's row.  key = c0 * size1 + c1 with (c0, c1) = (i, j) for a
// row-major C and (j, i) for a column-major one.
template <typename CT, typename VT>
__global__ __launch_bounds__(kThreads) void spgemm_expand_kernel(const int64_t *__restrict__ rows, const VT *__restrict__ avals, int64_t na,
                                                                 const unsigned long long *__restrict__ off, const int64_t *__restrict__ bstart,
                                                                 const CT *__restrict__ bcrd1, const VT *__restrict__ bvals,
                                                                 int c_is_row_major, uint64_t size1, uint64_t *__restrict__ keys,
                                                                 VT *__restrict__ payload)
{
    const int lane = threadIdx.x & 63;
    const int64_t p = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (p >= na) return;
    const int64_t o = (int64_t)off[p], len = (int64_t)off[p + 1] - o;
    if (len == 0) return;
    const uint64_t i = (uint64_t)rows[p];
    const VT a = avals[p];
    const int64_t bs = bstart[p];
    for (int64_t t = lane; t < len; t += 64) {
        const uint64_t j = (uint64_t)bcrd1[bs + t];
        keys[o + t] = c_is_row_major ? i * size1 + j : j * size1 + i;
        payload[o + t] = a * bvals[bs + t];
    }
}

template <typename PT, typename CT, typename VT>
sp_status spgemm_t(const sp_tensor *A, const sp_tensor *Br, const sp_encoding *encC, hipStream_t st, sp_tensor **out)
{
    sp_mem mem{A->alloc, A->free_, A->ctx};
    sp_scratch tmp(mem);
    const int64_t na = A->nvalues;
    const int64_t shapeC[2] = {A->shape[0], Br->shape[1]};
    const size_t cnt = (size_t)(na > 0 ? na : 1);
    int64_t *rows = (int64_t *)tmp.get(cnt * 8), *cols = (int64_t *)tmp.get(cnt * 8);
    VT *avals = (VT *)tmp.get(cnt * sizeof(VT));
    unsigned long long *off = (unsigned long long *)tmp.get((cnt + 1) * 8);
    int64_t *bstart = (int64_t *)tmp.get(cnt * 8);
    if (!rows || !cols || !avals || !off || !bstart) return SP_ERR_ALLOC;
    int64_t total = 0;
    if (na > 0 && Br->nvalues > 0) {
        int64_t *coords[2] = {rows, cols};
        SP_TRY(sp_unpack(A, coords, avals, st));
        const bool outer_compressed = Br->enc.lt[0] == SP_COMPRESSED;
        hipLaunchKernelGGL((spgemm_count_kernel<PT, CT>), dim3((unsigned)ceil_div(na + 1, kThreads)), dim3(kThreads), 0, st,
                           (const int64_t *)cols, na, (const PT *)Br->pos[0], outer_compressed ? (const CT *)Br->crd[0] : (const CT *)nullptr,
                           outer_compressed ? Br->ncrd[0] : 0, (const PT *)Br->pos[1], off, bstart);
        SP_HIP(hipGetLastError());
        SP_TRY(spmi_exclusive_scan(off, na + 1, 64, tmp, st));
        unsigned long long htotal = 0;
        SP_HIP(hipMemcpyAsync(&htotal, off + na, 8, hipMemcpyDeviceToHost, st));
        SP_HIP(hipStreamSynchronize(st));
        if (htotal >= ((unsigned long long)1 << 31)) return SP_ERR_TOO_LARGE;
        total = (int64_t)htotal;
    }
    uint64_t *keys = (uint64_t *)tmp.get((size_t)(total > 0 ? total : 1) * 8);
    VT *payload = (VT *)tmp.get((size_t)(total > 0 ? total : 1) * sizeof(VT));
    if (!keys || !payload) return SP_ERR_ALLOC;
    if (total > 0) {
        const int c_is_row_major = encC->perm[0] == 0;
        const uint64_t size1 = (uint64_t)(c_is_row_major ? shapeC[1] : shapeC[0]);
        hipLaunchKernelGGL((spgemm_expand_kernel<CT, VT>), dim3((unsigned)ceil_div(na, kThreads / 64)), dim3(kThreads), 0, st,
                           (const int64_t *)rows, (const VT *)avals, na, (const unsigned long long *)off, (const int64_t *)bstart,
                           (const CT *)Br->crd[1], (const VT *)Br->values, c_is_row_major, size1, keys, payload);
        SP_HIP(hipGetLastError());
    }
    return spmi_pack_keys(encC, shapeC, (sp_dtype)A->dtype, A->alloc, A->free_, A->ctx, total, keys, payload, tmp, st, out);
}

}  // namespace

extern "C" sp_status sp_spgemm(const sp_tensor *A, const sp_tensor *B, const sp_encoding *encC, void *stream, sp_tensor **C)
{
    if (!A || !B || !encC || !C) return SP_ERR_NULL;
    *C = nullptr;
    if (A->enc.rank != 2 || B->enc.rank != 2 || encC->rank != 2) return SP_ERR_RANK;
    if (A->shape[1] != B->shape[0]) return SP_ERR_SHAPE;
    if (A->dtype != B->dtype) return SP_ERR_DTYPE;
    hipStream_t st = (hipStream_t)stream;
    // B is read by rows: row-major with a compressed inner level as it is, column-major through its cached row-major copy
    const sp_tensor *Br = B;
    if (B->enc.lt[1] != SP_COMPRESSED) return SP_ERR_UNSUPPORTED;
    if (B->enc.perm[0] != 0) {
        SP_TRY(spmi_build_transposed(const_cast<sp_tensor *>(B), st));
        Br = B->transposed;
    }
    const int pw = Br->enc.pw, cw = Br->enc.cw;
#define SPMI_GO(PT, CT)                                                                                        \
    return A->dtype == SP_F64 ? spgemm_t<PT, CT, double>(A, Br, encC, st, C) : spgemm_t<PT, CT, float>(A, Br, encC, st, C)
    if (pw == 32 && cw == 32) SPMI_GO(int32_t, int32_t);
    if (pw == 32) SPMI_GO(int32_t, int64_t);
    if (cw == 32) SPMI_GO(int64_t, int32_t);
    SPMI_GO(int64_t, int64_t);
#undef SPMI_GO
}
