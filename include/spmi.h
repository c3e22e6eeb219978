/* spmi: sparse x dense products under per-level dense/compressed storage, for AMD MI355X (gfx950).
 *
 * C ABI of the library.  Plain pointers and sizes only; every pointer is marked HOST or
 * DEVICE.  No call throws; every call returns an sp_status.  There is no global state
 * other than what a handle owns.  All GPU work is enqueued on the HIP stream the caller
 * passes (void* = hipStream_t, NULL = the null stream).
 *
 * Vocabulary follows arXiv 2202.04305: a rank-d tensor is stored level by level; level l
 * holds dimension dimOrdering[l]; a level is "dense" (nothing stored, child position =
 * parent * size + coordinate) or "compressed" (arrays pointers[l] and indices[l], called
 * pos and crd here), and one values array holds the stored entries (Section 4.1).
 */
#ifndef SPMI_H
#define SPMI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SP_OK = 0,
    SP_ERR_NULL = 1,         /* a required pointer is NULL                                  */
    SP_ERR_RANK = 2,         /* rank outside [1, SP_MAX_RANK], or a rank-2 call on another rank */
    SP_ERR_LEVEL_TYPE = 3,   /* level type not dense/compressed; pos/crd asked of a dense level */
    SP_ERR_ORDERING = 4,     /* dimOrdering is not a permutation                            */
    SP_ERR_WIDTH = 5,        /* width not in {0,8,16,32,64}, or a stored value does not fit */
    SP_ERR_COORD_RANGE = 6,  /* a coordinate is < 0 or >= its dimension's size              */
    SP_ERR_DUPLICATE = 7,    /* the same coordinate tuple appears twice                     */
    SP_ERR_SHAPE = 8,        /* negative size, ld < N, and the like                         */
    SP_ERR_DTYPE = 9,
    SP_ERR_UNSUPPORTED = 10, /* valid request with no GPU path yet                          */
    SP_ERR_TOO_LARGE = 11,   /* position count or linearised key overflows 63 bits, nnz >= 2^31 */
    SP_ERR_ALLOC = 12,       /* the allocator returned NULL                                 */
    SP_ERR_HIP = 13          /* a HIP runtime call failed (sp_last_hip_error has the code)  */
} sp_status;

typedef enum { SP_DENSE = 0, SP_COMPRESSED = 1 } sp_level_type;
typedef enum { SP_F32 = 0, SP_F64 = 1 } sp_dtype;
#define SP_MAX_RANK 8

typedef struct sp_encoding sp_encoding;   /* HOST, immutable                                */
typedef struct sp_tensor sp_tensor;       /* HOST handle that owns DEVICE arrays            */

/* Device-memory allocator the library uses for everything it allocates (storage arrays and
 * temporaries).  alloc returns a DEVICE pointer aligned to >= 256 bytes or NULL; free_
 * releases one.  Both are called from the thread that calls into the library.  free_ may be
 * called while kernels that use the block are still queued on the stream of that call, so the
 * allocator must be stream-ordered with respect to it (torch's caching allocator is, for the
 * stream that was current at allocation).  Pass NULL for both to use hipMalloc / hipFree. */
typedef void *(*sp_alloc_fn)(size_t bytes, void *ctx);
typedef void (*sp_free_fn)(void *ptr, void *ctx);

/* The encoding attribute (Section 4.1: per-dimension level types, dimension ordering, bit
 * widths).  levelTypes: HOST array of `rank` entries, by level.  dimOrdering: HOST array,
 * dimOrdering[l] = dimension stored at level l (the result list of the paper's affine map
 * read left to right); NULL = identity.  posWidth / crdWidth: bits of the pos and crd
 * arrays: 8, 16, 32, 64, or 0 = "native" = 64; the arrays hold signed integers.  (For 8 and
 * 16 bits the tensor keeps 32-bit working copies for its kernels next to the narrow arrays
 * it hands out.)  Checks run in the order rank, level type, ordering, width; *out is written only
 * on SP_OK and is released with sp_encoding_free. */
sp_status sp_encode(int rank, const sp_level_type *levelTypes, const int *dimOrdering,
                    int posWidth, int crdWidth, sp_encoding **out);
void sp_encoding_free(sp_encoding *enc);

/* Build the storage from coordinate-scheme input (Section 4.2: tensors are materialised and
 * converted through an intermediate coordinate scheme; Section 4.1 defines the arrays built).
 *   shape   HOST  `rank` sizes by original dimension.
 *   nnz     number of entries, in any order, zero-based coordinates, no tuple twice.
 *   coords  HOST array of `rank` DEVICE pointers; coords[d][e] = coordinate of entry e in
 *           dimension d (structure of arrays, int64).
 *   values  DEVICE, nnz elements of `dt`.  Explicit zeros are kept as stored entries.
 * The inputs are read, never kept.  The tensor owns its arrays; they are obtained from
 * `alloc` and released through `free_` by sp_tensor_free (the callbacks and ctx must stay
 * valid until then).  The call synchronises the stream (level sizes and the input checks
 * come back to the host).  Errors, in this order: NULL, shape, TOO_LARGE, COORD_RANGE,
 * DUPLICATE, WIDTH; on error nothing is left allocated and *out is NULL. */
sp_status sp_pack(const sp_encoding *enc, const int64_t *shape, int64_t nnz,
                  const int64_t *const *coords, const void *values, sp_dtype dt,
                  sp_alloc_fn alloc, sp_free_fn free_, void *ctx, void *stream, sp_tensor **out);
void sp_tensor_free(sp_tensor *t);

/* The inspector step of the products below (Section 6.2 measures the matrix-times-vector and SpMM kernels on tensors
 * that were read and packed beforehand; what a kernel needs beyond the packed storage is prepared here, once, outside
 * the products).  For a product of `A` with a dense operand of N columns it decides which kernel will run (for N = 1
 * it measures, in one pass over the innermost crd array, how scattered the columns are), builds the copy of the
 * entries that kernel reads (row-major copy of a column-major tensor; for a large matrix with scattered columns
 * a copy regrouped by column panel and row block), and allocates the scratch the kernel uses.  Everything is obtained
 * from the tensor's allocator and kept by the handle until sp_tensor_free; sp_tensor_info reports its size (derivedBytes)
 * and the choice (spmvKernel).  Synchronises `stream`.  Calling it again with the same N is a no-op; a larger N
 * grows the scratch; sp_tensor_tune with a kernel key makes the next sp_prepare (or product) decide again.
 * After sp_prepare(A, N), sp_matmul(A, .., N' <= N columns ..) neither allocates nor synchronises, so it may be recorded
 * into a HIP graph from its first call on.  Errors: NULL, RANK (not rank 2), SHAPE (N < 0), UNSUPPORTED (a kernel forced
 * with sp_tensor_tune cannot run on this tensor), ALLOC, HIP. */
sp_status sp_prepare(sp_tensor *A, int64_t N, void *stream);

/* C[i,j] = sum_k A[i,k] * B[k,j] (Section 1, the SpMM kernel; Section 6.2, matrix times vector
 * is the case N = 1), A a packed rank-2 tensor of shape m x n.
 *   B  DEVICE, row-major n x N with leading dimension ldb >= N, A's dtype.
 *   C  DEVICE, row-major m x N with leading dimension ldc >= N, A's dtype.
 *   accumulate = 0: C is overwritten (rows of A without stored entries become zero);
 *   accumulate = 1: C += A.B and rows without stored entries are not touched.
 * Enqueues on `stream` and returns without synchronising or allocating, provided sp_prepare(A, N) ran before.
 * Without it the product still works: whatever sp_prepare would have built is built by the first product that needs
 * it (that call then allocates and synchronises `stream`), and sp_tensor_info counts such calls in lazyPrepares, so
 * a caller can assert that its loop ran without any.  The handle's derived state is a cache that a product may fill
 * in although it takes the handle as const: a handle must not be used by two host threads at the same time, and the
 * scratch it holds is shared by all products on it, so products of one tensor that run concurrently on different
 * streams race.  B and C must not overlap.  Summation order inside a row is unspecified (floating-point reassociation,
 * Section 5.2); whether it is the same from call to call depends on the kernel (see SP_TUNE_SPMV_KERNEL). */
sp_status sp_matmul(const sp_tensor *A, const void *B, int64_t N, int64_t ldb,
                    void *C, int64_t ldc, int accumulate, void *stream);

/* sp_matmul for callers that cannot allocate device memory or have it allocated on their behalf: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and result as sp_matmul, for a
 * row-major tensor with a compressed innermost level (CSR, DCSR) and N >= 2 columns with N * element size a multiple of
 * 16 and at most 64 such 16-byte pieces per row, B, C and their leading dimensions 16-byte aligned (the product cut by
 * stored entries; SP_ERR_UNSUPPORTED otherwise, also for a tensor whose tables a product would still have to build).
 * The per-block partial rows that kernel keeps between its two launches live in a fixed array of 16 MiB inside the
 * library's code object on each GPU instead of a buffer from the tensor's allocator: the call needs
 * (stored entries / 1024, rounded up) * N * element size bytes of it and returns SP_ERR_TOO_LARGE beyond 16 MiB.  It calls no
 * allocator, neither the tensor's nor HIP's, and does not synchronise.  All calls on one GPU share that array: calls that
 * overlap on one GPU (different streams, different tensors) race; stream-ordered calls do not.  Results are the same
 * bits as sp_matmul's with SP_TUNE_SPMM_KERNEL 0 or 3. */
sp_status sp_matmul_noalloc(const sp_tensor *A, const void *B, int64_t N, int64_t ldb,
                            void *C, int64_t ldc, int accumulate, void *stream);

/* The paper's pointers / indices / values operations (Section 4.2): borrowed DEVICE
 * pointers, valid until sp_tensor_free.  `level` is a storage level, not a dimension.  *len is in
 * elements of the tensor's pos / crd width (sp_tensor_info) or dtype. */
sp_status sp_pos(const sp_tensor *t, int level, const void **ptr, int64_t *len);
sp_status sp_crd(const sp_tensor *t, int level, const void **ptr, int64_t *len);
sp_status sp_values(const sp_tensor *t, const void **ptr, int64_t *len);

/* Back to the coordinate scheme (Section 4.2: the intermediate form every conversion passes through; it is the first
 * half of the paper's convert operation, whose second half is sp_pack): every stored position in storage order
 * (padding zeros of a dense level under a compressed one included), coordinates in the original dimension order.
 * coords: HOST array of `rank` DEVICE int64 arrays, each with room for sp_values' length (sp_tensor_info: nvalues) entries;
 * values: DEVICE array of the tensor's dtype, same length.  The number of entries written is that length: nothing comes
 * back to the host, so the call is asynchronous. */
sp_status sp_unpack(const sp_tensor *t, int64_t *const *coords, void *values, void *stream);

/* Sampled dense-dense product X[i,j] = S[i,j] * sum_k A[i,k] * B[k,j] (Section 6.2, the SDDMM kernel of the
 * state-space experiment).  X has S's pattern: the result is one value per stored position of S, in storage order
 * (the order of sp_values), so it can stand in for S's values array.
 *   S  packed rank-2 tensor m x n, row-major with a compressed innermost level (CSR or DCSR); other encodings
 *      give SP_ERR_UNSUPPORTED (convert first).
 *   A  DEVICE, m x K row-major, leading dimension lda >= K, S's dtype.
 *   B  DEVICE, S's dtype: K x n row-major with ldb >= n as in the paper's formula (b_is_transposed = 0; the library
 *      transposes it into scratch from the tensor's allocator on every call), or already n x K row-major with
 *      ldb >= K (b_is_transposed = 1).
 *   X  DEVICE, as many elements as sp_values reports, S's dtype.
 * Enqueues on `stream`; does not synchronise when the allocator is stream-ordered (see sp_alloc_fn). */
sp_status sp_sddmm(const sp_tensor *S, const void *A, int64_t lda, const void *B, int64_t ldb, int b_is_transposed,
                   int64_t K, void *X, void *stream);

/* Matricized tensor times Khatri-Rao product A[i,j] = sum_{k,l} B[i,k,l] * D[l,j] * C[k,j] (Section 6.3, the MTTKRP
 * kernel), B a packed rank-3 tensor of shape I x K x L.
 *   B  stored with dimension i at the outermost level (dense or compressed) and two compressed inner levels in
 *      either order of k and l: the two formats of the paper's experiment and their all-compressed variants.
 *      Other encodings give SP_ERR_UNSUPPORTED (convert first).
 *   C  DEVICE, K x J row-major, leading dimension ldc >= J, B's dtype.
 *   D  DEVICE, L x J row-major, leading dimension ldd >= J, B's dtype.
 *   A  DEVICE, I x J row-major, leading dimension lda >= J, B's dtype; must not overlap C or D.
 *   accumulate = 0: A is overwritten (slices of B without stored entries become zero rows); 1: A += the product.
 * Enqueues on `stream`; does not synchronise when the allocator is stream-ordered (the first call on a tensor
 * allocates a small table and a scratch buffer through it).  Results are bit-reproducible from call to call. */
sp_status sp_mttkrp(const sp_tensor *B, const void *C, int64_t ldc, const void *D, int64_t ldd, int64_t J,
                    void *A, int64_t lda, int accumulate, void *stream);

/* Sparse times sparse with a sparse result: C[i,j] = sum_k A[i,k] * B[k,j] (Section 4.2, the SpMSpM kernel; Section 4.4
 * describes the generated loop with its workspace; Section 6.2 measures it).  A: packed rank-2 tensor m x k of any
 * encoding; B: packed k x n with a compressed inner level (CSR, DCSR as they are; CSC, DCSC through a row-major copy
 * that the tensor builds on first use and keeps); a B with a dense inner level gives SP_ERR_UNSUPPORTED (convert
 * first).  *C is a new tensor m x n under `encC` with A's dtype and allocator: it stores every (i,j) for which a pair of
 * stored entries A[i,k], B[k,j] exists, whatever the sum comes to, and each sum runs over k in A's storage order, so
 * the result is the same bits on every call (unless SP_TUNE_SPGEMM_KERNEL 5 was asked for).  Synchronises like sp_pack.  Errors: NULL, RANK, SHAPE (inner sizes
 * differ), DTYPE (A and B differ), TOO_LARGE (2^31 or more pairs), WIDTH (C does not fit encC's widths), ALLOC, HIP. */
sp_status sp_spgemm(const sp_tensor *A, const sp_tensor *B, const sp_encoding *encC, void *stream, sp_tensor **C);

/* Element-wise sum C = A + B of two packed tensors of the same shape and dtype, any rank and encodings (the example of
 * Section 5.1).  *C is a new tensor under `encC` with A's allocator that stores every position A or B stores (padding
 * zeros of dense levels and explicit zeros included, a sum that comes to zero too); where both store a position the
 * two values are added once.  Synchronises like sp_pack.  Errors: NULL, RANK, SHAPE (shapes differ), DTYPE,
 * TOO_LARGE (2^31 or more stored positions together), WIDTH (C does not fit encC's widths), ALLOC, HIP. */
sp_status sp_add(const sp_tensor *A, const sp_tensor *B, const sp_encoding *encC, void *stream, sp_tensor **C);

/* The paper's convert operation between two sparse encodings (Section 4.2: conversions go through an intermediate
 * coordinate scheme, which avoids one converter per pair of formats).  Every stored position of `from` (explicit and
 * padding zeros included) becomes a stored entry of the new tensor, which has `from`'s shape, dtype and allocator and
 * the encoding `to` (same rank).  Synchronises like sp_pack; `from` is left untouched. */
sp_status sp_convert(const sp_tensor *from, const sp_encoding *to, void *stream, sp_tensor **out);

typedef struct {
    int rank;
    int levelTypes[SP_MAX_RANK];
    int dimOrdering[SP_MAX_RANK];
    int posWidth, crdWidth;          /* resolved: 8, 16, 32 or 64 */
    int dtype;
    int64_t shape[SP_MAX_RANK];
    int64_t nnz;                     /* entries given to sp_pack */
    int64_t nvalues;                 /* length of the values array */
    int64_t maxSegment;              /* longest innermost pos segment (rank 2: longest row/column) */
    int64_t storageBytes;            /* pos + crd + values */
    int64_t derivedBytes;            /* what the handle keeps beyond that: tables, regrouped copies, scratch (see sp_prepare) */
    int spmvKernel;                  /* the SpMV kernel a product with one column runs (values of SP_TUNE_SPMV_KERNEL); 0 = not decided yet */
    int lazyPrepares;                /* products that had to build, allocate or decide something first (0 when sp_prepare covered them) */
} sp_info;
sp_status sp_tensor_info(const sp_tensor *t, sp_info *info /* HOST */);

/* Kernel choice for sp_matmul on this tensor, for A/B measurements.  key/value pairs:
 *   SP_TUNE_SPMV_KERNEL: 0 = automatic, 1 = lanes-per-row, 2 = streaming over the CSR arrays (bit-reproducible),
 *                        3 = streaming over a column-segmented copy (built and kept on first use; CSR only),
 *                        4 = two streaming passes over a copy binned by column panel and row block, gathers and
 *                        adds inside the LDS (built and kept on first use; CSR only; the order in which a row's
 *                        products are added varies from call to call: results agree to rounding, not bit for bit)
 *   SP_TUNE_SPMM_KERNEL: 0 = automatic, 1 = one column per lane, 2 = 16 bytes of a row of B per lane, a wave per row,
 *                        3 = the same cut by stored entries instead of rows (2 and 3 need N a multiple
 *                        of 16 / element size and B, C rows 16-byte aligned; 2 takes 1, 2, 4, ... 64 such vectors
 *                        per row, 3 any number up to 64)
 *   SP_TUNE_CSC_MODE:    0 = automatic, 1 = scatter with atomics, 2 = via a cached transpose
 *   SP_TUNE_SPGEMM_KERNEL (set on the left operand of sp_spgemm): 0 = automatic, 1 = pairs expanded, sorted and added
 *                        up by the storage builder (any sizes and encodings), 2 = a row of C at a time in an LDS
 *                        workspace (CSR / DCSR operands and a CSR result with one pos / crd width, rows of C that
 *                        fit the LDS; SP_ERR_UNSUPPORTED otherwise), four waves per row over a column-panel copy
 *                        of B that B builds on first use and keeps, 3 = the same workspace with one wave per row
 *                        and no copy of B, 4 = the same with sixteen waves per row (sixteen column panels, B read in place; results
 *                        of 1024 columns or more, else as 2; the automatic choice from 8192 columns on), 5 = sixteen
 *                        waves per row with the entries of the row of A dealt out to them instead of the columns:
 *                        the fastest (0.38 ms against 0.45 ms on the 8192 x 8192 product of Section 6.2), but the
 *                        waves add into one workspace in an order that depends on timing, so the values of C agree
 *                        from call to call only to rounding; never chosen automatically
 * Unknown keys or values give SP_ERR_UNSUPPORTED. */
enum { SP_TUNE_SPMV_KERNEL = 1, SP_TUNE_CSC_MODE = 2, SP_TUNE_SPMM_KERNEL = 3, SP_TUNE_SPGEMM_KERNEL = 5 };   /* 4: see spmi_bench.h */
sp_status sp_tensor_tune(sp_tensor *t, int key, int64_t value);

const char *sp_status_str(sp_status s);
int sp_last_hip_error(void);          /* hipError_t of the last SP_ERR_HIP on this thread */

#ifdef __cplusplus
}
#endif
#endif /* SPMI_H */
