// C ABI entry points that are not the storage builder: the encoding attribute, the product's
// dispatch, the pointers / indices / values accessors (arXiv 2202.04305, Sections 4.1 and 4.2).
#include "spmi_internal.h"

thread_local int g_last_hip_error = 0;

extern "C" int sp_last_hip_error(void) { return g_last_hip_error; }

extern "C" const char *sp_status_str(sp_status status)
{
    int s;                                             // any integer may arrive: read it as one, not as the enumeration
    memcpy(&s, &status, sizeof(s));
    switch (s) {
    case SP_OK: return "ok";
    case SP_ERR_NULL: return "null pointer";
    case SP_ERR_RANK: return "bad rank";
    case SP_ERR_LEVEL_TYPE: return "bad level type";
    case SP_ERR_ORDERING: return "dimension ordering is not a permutation";
    case SP_ERR_WIDTH: return "bad or too narrow bit width";
    case SP_ERR_COORD_RANGE: return "coordinate out of range";
    case SP_ERR_DUPLICATE: return "duplicate coordinate";
    case SP_ERR_SHAPE: return "bad shape or leading dimension";
    case SP_ERR_DTYPE: return "bad dtype";
    case SP_ERR_UNSUPPORTED: return "not supported on the GPU path";
    case SP_ERR_TOO_LARGE: return "too large";
    case SP_ERR_ALLOC: return "allocation failed";
    case SP_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" sp_status sp_encode(int rank, const sp_level_type *levelTypes, const int *dimOrdering, int posWidth, int crdWidth,
                               sp_encoding **out)
{
    if (!levelTypes || !out) return SP_ERR_NULL;
    *out = nullptr;
    if (rank < 1 || rank > SP_MAX_RANK) return SP_ERR_RANK;
    // the caller's array may hold any integer: it is read as integers, not as the enumeration (whose other values C++ may not load)
    static_assert(sizeof(sp_level_type) == sizeof(int), "level types travel as ints");
    int lt[SP_MAX_RANK];
    for (int l = 0; l < rank; ++l) {
        memcpy(&lt[l], (const char *)levelTypes + (size_t)l * sizeof(int), sizeof(int));
        if (lt[l] != (int)SP_DENSE && lt[l] != (int)SP_COMPRESSED) return SP_ERR_LEVEL_TYPE;
    }
    bool seen[SP_MAX_RANK] = {false};
    for (int l = 0; l < rank; ++l) {
        const int d = dimOrdering ? dimOrdering[l] : l;
        if (d < 0 || d >= rank || seen[d]) return SP_ERR_ORDERING;
        seen[d] = true;
    }
    auto ok = [](int w) { return w == 0 || w == 8 || w == 16 || w == 32 || w == 64; };
    if (!ok(posWidth) || !ok(crdWidth)) return SP_ERR_WIDTH;
    sp_encoding *e = new sp_encoding();
    memset(e, 0, sizeof(*e));
    e->rank = rank;
    for (int l = 0; l < rank; ++l) {
        e->lt[l] = lt[l];
        e->perm[l] = dimOrdering ? dimOrdering[l] : l;
    }
    e->pw_store = posWidth ? posWidth : 64;
    e->cw_store = crdWidth ? crdWidth : 64;
    e->pw = e->pw_store < 32 ? 32 : e->pw_store;       // 8- and 16-bit arrays are kept next to 32-bit working copies
    e->cw = e->cw_store < 32 ? 32 : e->cw_store;
    *out = e;
    return SP_OK;
}

extern "C" void sp_encoding_free(sp_encoding *enc) { delete enc; }

extern "C" sp_status sp_pos(const sp_tensor *t, int level, const void **ptr, int64_t *len)
{
    if (!t || !ptr || !len) return SP_ERR_NULL;
    if (level < 0 || level >= t->enc.rank) return SP_ERR_RANK;
    if (t->enc.lt[level] != SP_COMPRESSED) return SP_ERR_LEVEL_TYPE;
    *ptr = t->pos_narrow[level] ? t->pos_narrow[level] : t->pos[level];
    *len = t->npos[level];
    return SP_OK;
}

extern "C" sp_status sp_crd(const sp_tensor *t, int level, const void **ptr, int64_t *len)
{
    if (!t || !ptr || !len) return SP_ERR_NULL;
    if (level < 0 || level >= t->enc.rank) return SP_ERR_RANK;
    if (t->enc.lt[level] != SP_COMPRESSED) return SP_ERR_LEVEL_TYPE;
    *ptr = t->crd_narrow[level] ? t->crd_narrow[level] : t->crd[level];
    *len = t->ncrd[level];
    return SP_OK;
}

extern "C" sp_status sp_values(const sp_tensor *t, const void **ptr, int64_t *len)
{
    if (!t || !ptr || !len) return SP_ERR_NULL;
    *ptr = t->values;
    *len = t->nvalues;
    return SP_OK;
}

extern "C" sp_status sp_tensor_info(const sp_tensor *t, sp_info *info)
{
    if (!t || !info) return SP_ERR_NULL;
    memset(info, 0, sizeof(*info));
    info->rank = t->enc.rank;
    int64_t bytes = t->nvalues * (t->dtype == SP_F64 ? 8 : 4);
    for (int l = 0; l < t->enc.rank; ++l) {
        info->levelTypes[l] = t->enc.lt[l];
        info->dimOrdering[l] = t->enc.perm[l];
        info->shape[l] = t->shape[l];
        if (t->enc.lt[l] == SP_COMPRESSED) bytes += t->npos[l] * (t->enc.pw_store / 8) + t->ncrd[l] * (t->enc.cw_store / 8);
    }
    info->posWidth = t->enc.pw_store;
    info->crdWidth = t->enc.cw_store;
    info->dtype = t->dtype;
    info->nnz = t->nnz;
    info->nvalues = t->nvalues;
    info->maxSegment = t->max_segment;
    info->storageBytes = bytes;
    // what the handle keeps beyond the paper's storage: tables, regrouped copies, scratch
    const int64_t v = t->dtype == SP_F64 ? 8 : 4;
    int64_t extra = (t->rowblocks.nblocks + t->nz_rowblocks.nblocks) * (4 + v) + (int64_t)t->dense_partial_bytes + (int64_t)t->spmm_carry_bytes +
                    (int64_t)t->sddmm_bt_bytes + (int64_t)t->mttkrp_carry_bytes + (int64_t)t->mttkrp_pad_bytes[0] + (int64_t)t->mttkrp_pad_bytes[1];
    if (t->nz_pos) extra += t->nz_rows * (t->enc.cw / 8) + (t->nz_rows + 1) * (t->enc.pw / 8);
    if (t->bins) extra += t->bins->np * (2 * v + 4) + t->bins->np / 8 * 4 + ((int64_t)t->bins->panels + t->bins->rowblocks + 2) * 8;
    const sp_tensor *copies[2] = {t->segments ? t->segments->seg : nullptr, t->transposed};
    for (const sp_tensor *c : copies)
        if (c) {
            sp_info ci;
            (void)sp_tensor_info(c, &ci);
            extra += ci.storageBytes + ci.derivedBytes;
        }
    if (t->segments) extra += (int64_t)t->segments->panels * t->segments->nrows * v;
    info->derivedBytes = extra;
    const sp_tensor *prod = t->transposed ? t->transposed : t;       // the tensor whose kernels a product of `t` runs
    info->spmvKernel = prod->plan_spmv;
    info->lazyPrepares = t->lazy_prepares + (t->transposed ? t->transposed->lazy_prepares : 0);
    return SP_OK;
}

extern "C" sp_status sp_tensor_tune(sp_tensor *t, int key, int64_t value)
{
    if (!t) return SP_ERR_NULL;
    switch (key) {
    case SP_TUNE_SPMV_KERNEL:
        if (value < 0 || value > 4) return SP_ERR_UNSUPPORTED;
        t->tune_spmv = (int)value;
        t->plan_spmv = 0;                                // decided again by sp_prepare or the next product (copies already built are kept)
        if (t->transposed) { t->transposed->tune_spmv = (int)value; t->transposed->plan_spmv = 0; }
        return SP_OK;
    case SP_TUNE_CSC_MODE:
        if (value < 0 || value > 2) return SP_ERR_UNSUPPORTED;
        t->tune_csc = (int)value;
        return SP_OK;
    case SP_TUNE_PROFILE:
        if (value != 0 && value != 1) return SP_ERR_UNSUPPORTED;
        if (value && !t->prof_events) t->prof_events = new std::vector<hipEvent_t>();
        t->profile = (int)value;
        if (t->transposed) return sp_tensor_tune(t->transposed, key, value);
        return SP_OK;
    case SP_TUNE_SPGEMM_KERNEL:
        if (value < 0 || value > 5) return SP_ERR_UNSUPPORTED;
        t->tune_spgemm = (int)value;
        return SP_OK;
    case SP_TUNE_SPMM_KERNEL:
        if (value < 0 || value > 3) return SP_ERR_UNSUPPORTED;
        t->tune_spmm = (int)value;
        if (t->transposed) t->transposed->tune_spmm = (int)value;
        return SP_OK;
    }
    return SP_ERR_UNSUPPORTED;
}

extern "C" sp_status sp_profile_read(sp_tensor *t, double *ms_total, int64_t *launches)
{
    if (!t || !ms_total || !launches) return SP_ERR_NULL;
    *ms_total = 0.0;
    *launches = 0;
    sp_tensor *src = (t->transposed && t->transposed->prof_events && !t->transposed->prof_events->empty()) ? t->transposed : t;
    if (!src->prof_events) return SP_OK;
    std::vector<hipEvent_t> &ev = *src->prof_events;
    sp_status s = SP_OK;
    for (size_t i = 0; i + 1 < ev.size(); i += 2) {
        float ms = 0.f;
        if (hipEventSynchronize(ev[i + 1]) != hipSuccess || hipEventElapsedTime(&ms, ev[i], ev[i + 1]) != hipSuccess) s = SP_ERR_HIP;
        else { *ms_total += (double)ms; *launches += 1; }
        (void)hipEventDestroy(ev[i]);
        (void)hipEventDestroy(ev[i + 1]);
    }
    ev.clear();
    return s;
}

// Row-major copy of a column-major tensor, through the coordinate scheme (the paper's route for
// conversions, Section 4.2).  Built on first use and kept by the handle.
sp_status spmi_build_transposed(const sp_tensor *A, hipStream_t st)
{
    if (A->transposed) return SP_OK;
    sp_mem mem{A->alloc, A->free_, A->ctx};
    sp_status s = SP_OK;
    sp_tensor *T = nullptr;
    {
        sp_scratch tmp(mem);
        const size_t cnt = (size_t)(A->nvalues > 0 ? A->nvalues : 1);
        int64_t *rows = (int64_t *)tmp.get(cnt * 8);
        int64_t *cols = (int64_t *)tmp.get(cnt * 8);
        void *vals = tmp.get(cnt * 8);
        if (!rows || !cols || !vals) return SP_ERR_ALLOC;
        int64_t *coords[2] = {rows, cols};
        SP_TRY(sp_unpack(A, coords, vals, st));
        sp_encoding enc = A->enc;
        enc.perm[0] = 0; enc.perm[1] = 1;
        enc.pw_store = enc.pw; enc.cw_store = enc.cw;     // an internal copy: working widths only
        const int64_t *ccoords[2] = {rows, cols};
        s = sp_pack(&enc, A->shape, A->nvalues, ccoords, vals, (sp_dtype)A->dtype, A->alloc, A->free_, A->ctx, st, &T);
    }
    if (s != SP_OK) return s;
    T->tune_spmv = A->tune_spmv;
    T->tune_spmm = A->tune_spmm;
    T->lazy_prepares = 0;
    if (A->profile) (void)sp_tensor_tune(T, SP_TUNE_PROFILE, 1);
    A->transposed = T;
    return SP_OK;
}

extern "C" sp_status sp_convert(const sp_tensor *from, const sp_encoding *to, void *stream, sp_tensor **out)
{
    if (!from || !to || !out) return SP_ERR_NULL;
    *out = nullptr;
    if (to->rank != from->enc.rank) return SP_ERR_RANK;
    hipStream_t st = (hipStream_t)stream;
    sp_mem mem{from->alloc, from->free_, from->ctx};
    sp_scratch tmp(mem);
    const int rank = from->enc.rank;
    const size_t cnt = (size_t)(from->nvalues > 0 ? from->nvalues : 1);
    int64_t *coords[SP_MAX_RANK] = {nullptr};
    for (int d = 0; d < rank; ++d) {
        coords[d] = (int64_t *)tmp.get(cnt * 8);
        if (!coords[d]) return SP_ERR_ALLOC;
    }
    void *vals = tmp.get(cnt * 8);
    if (!vals) return SP_ERR_ALLOC;
    SP_TRY(sp_unpack(from, coords, vals, st));
    return sp_pack(to, from->shape, from->nvalues, (const int64_t *const *)coords, vals, (sp_dtype)from->dtype, from->alloc,
                   from->free_, from->ctx, st, out);
}

// C = A + B element by element: the stored positions of both go through the storage builder as one list of
// (key, value) records, A's first; the builder's stable sort brings the two records of a position both store next to
// each other and its summation pass adds them (a + b, one addition).
extern "C" sp_status sp_add(const sp_tensor *A, const sp_tensor *B, const sp_encoding *encC, void *stream, sp_tensor **C)
{
    if (!A || !B || !encC || !C) return SP_ERR_NULL;
    *C = nullptr;
    const int rank = A->enc.rank;
    if (B->enc.rank != rank || encC->rank != rank) return SP_ERR_RANK;
    for (int d = 0; d < rank; ++d) if (A->shape[d] != B->shape[d]) return SP_ERR_SHAPE;
    if (A->dtype != B->dtype) return SP_ERR_DTYPE;
    const int64_t na = A->nvalues, nb = B->nvalues, n = na + nb;
    if (n >= ((int64_t)1 << 31)) return SP_ERR_TOO_LARGE;
    hipStream_t st = (hipStream_t)stream;
    sp_mem mem{A->alloc, A->free_, A->ctx};
    sp_scratch tmp(mem);
    const size_t cnt = (size_t)(n > 0 ? n : 1), vsz = A->dtype == SP_F64 ? 8 : 4;
    int64_t *coords[SP_MAX_RANK] = {nullptr};
    for (int d = 0; d < rank; ++d) {
        coords[d] = (int64_t *)tmp.get(cnt * 8);
        if (!coords[d]) return SP_ERR_ALLOC;
    }
    char *vals = (char *)tmp.get((cnt * vsz + 15) & ~(size_t)15);
    uint64_t *keys = (uint64_t *)tmp.get(cnt * 8);
    int *flags = (int *)tmp.get(64);
    if (!vals || !keys || !flags) return SP_ERR_ALLOC;
    SP_TRY(sp_unpack(A, coords, vals, st));
    int64_t *second[SP_MAX_RANK] = {nullptr};
    for (int d = 0; d < rank; ++d) second[d] = coords[d] + na;
    SP_TRY(sp_unpack(B, second, vals + (size_t)na * vsz, st));
    // a handle with C's level order and sizes, only to make the keys by
    sp_tensor *shaped = nullptr;
    int key_bits = 0;
    SP_TRY(spmi_new_tensor(encC, A->shape, (sp_dtype)A->dtype, A->alloc, A->free_, A->ctx, false, &shaped, &key_bits));
    sp_status s = spmi_fill_zero(flags, 64, st);
    if (s == SP_OK) s = spmi_make_keys(shaped, (const int64_t *const *)coords, n, keys, flags, st);
    delete shaped;
    SP_TRY(s);
    return spmi_pack_keys(encC, A->shape, (sp_dtype)A->dtype, A->alloc, A->free_, A->ctx, n, keys, vals, tmp, st, C);
}

extern "C" sp_status sp_matmul(const sp_tensor *A, const void *B, int64_t N, int64_t ldb, void *C, int64_t ldc, int accumulate,
                               void *stream)
{
    if (!A) return SP_ERR_NULL;
    if (A->enc.rank != 2) return SP_ERR_RANK;
    if (N < 0 || ldb < N || ldc < N || ldb < 1 || ldc < 1) return SP_ERR_SHAPE;
    const int64_t m = A->shape[0], n = A->shape[1];
    if (N == 0 || m == 0) return SP_OK;
    if (!C || (!B && n > 0)) return SP_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    if (A->tables_pending) { ++A->lazy_prepares; SP_TRY(spmi_ensure_tables(A, st)); }
    if (A->enc.lt[1] != SP_COMPRESSED) return spmi_matmul_dense_inner(A, B, N, ldb, C, ldc, accumulate, st);
    if (A->enc.perm[0] == 0) return spmi_matmul_rowmajor(A, B, N, ldb, C, ldc, accumulate, st);
    int mode = A->tune_csc ? A->tune_csc : 2;
    if (mode == 1) return spmi_matmul_colmajor_scatter(A, B, N, ldb, C, ldc, accumulate, st);
    if (!A->transposed) { ++A->lazy_prepares; SP_TRY(spmi_build_transposed(A, st)); }
    return spmi_matmul_rowmajor(A->transposed, B, N, ldb, C, ldc, accumulate, st);
}

extern "C" sp_status sp_prepare(sp_tensor *A, int64_t N, void *stream)
{
    if (!A) return SP_ERR_NULL;
    if (A->enc.rank != 2) return SP_ERR_RANK;
    if (N < 0) return SP_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    if (N == 0 || A->shape[0] == 0) return SP_OK;
    SP_TRY(spmi_ensure_tables(A, st));
    sp_status s = SP_OK;
    if (A->enc.lt[1] != SP_COMPRESSED) s = spmi_prepare_dense_inner(A, N, st);
    else if (A->enc.perm[0] == 0) s = spmi_prepare_rowmajor(A, N, st);
    else if ((A->tune_csc ? A->tune_csc : 2) == 2) {
        s = spmi_build_transposed(A, st);
        if (s == SP_OK) s = spmi_prepare_rowmajor(A->transposed, N, st);
    }
    SP_TRY(s);
    SP_HIP(hipStreamSynchronize(st));
    return SP_OK;
}

// ---- plain streaming copy: the bandwidth yardstick ----------------------------------------
__global__ __launch_bounds__(256) void stream_copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src, size_t n16)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n16; i += stride) dst[i] = src[i];
}

extern "C" sp_status sp_stream_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src) return SP_ERR_NULL;
    if (bytes % 16) return SP_ERR_SHAPE;
    const size_t n16 = bytes / 16;
    if (n16 == 0) return SP_OK;
    size_t nb = (n16 + 255) / 256;
    if (nb > 256 * 32) nb = 256 * 32;
    hipLaunchKernelGGL(stream_copy_kernel, dim3((unsigned)nb), dim3(256), 0, (hipStream_t)stream, (uint4 *)dst, (const uint4 *)src, n16);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

// ---- plain streaming read: the read-only bandwidth yardstick --------------------------------
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4 *__restrict__ src, size_t n16, unsigned *__restrict__ sink)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    unsigned acc = 0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < n16; i += stride) { const uint4 a = src[i]; acc ^= a.x ^ a.y ^ a.z ^ a.w; }
    if (acc == 0x9e3779b9u) *sink = acc;               // practically never: keeps the loads alive
}

extern "C" sp_status sp_stream_read(const void *src, size_t bytes, void *sink, void *stream)
{
    if (!src || !sink) return SP_ERR_NULL;
    if (bytes % 16) return SP_ERR_SHAPE;
    const size_t n16 = bytes / 16;
    if (n16 == 0) return SP_OK;
    size_t nb = (n16 + 255) / 256;
    if (nb > 256 * 32) nb = 256 * 32;
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)nb), dim3(256), 0, (hipStream_t)stream, (const uint4 *)src, n16, (unsigned *)sink);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

extern "C" sp_status sp_pack_sort_mode(int mode)
{
    if (mode < 0 || mode > 2) return SP_ERR_UNSUPPORTED;
    g_pack_sort_mode.store(mode, std::memory_order_relaxed);
    return SP_OK;
}
