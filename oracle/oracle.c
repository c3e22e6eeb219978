/* CPU checker for the sparse storage scheme and the sparse x dense product.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the GPU library includes, links or calls this
 * file, and this file uses nothing of the GPU library.  It is deliberately plain and
 * slow: one thread, no blocking, no fusion, extended-precision accumulators.
 *
 * What it follows (arXiv 2202.04305):
 *   - Section 4.1 "Sparse Tensor Attributes and Types": a tensor of rank d is stored as
 *     per-level arrays pointers[l] / indices[l] (called pos / crd here) plus one values
 *     array; each level is "dense" or "compressed"; a dimension ordering says which
 *     dimension each level stores; pointer and index bit widths may be narrowed.  The
 *     five worked examples of that section (sparse vector, CSR, compressed-dense, DCSC,
 *     triply compressed 3-D tensor) fix what the arrays must contain.
 *   - Section 1 / Section 4.2: the kernel C[i,j] = A[i,k] * B[k,j] with only A sparse
 *     (SpMM; SpMV when B has one column).  The sparse code computes exactly this plain
 *     definition while skipping structural zeros, so the checker is the definition.
 *
 * Parity pins (tests/test_oracle_*.py): the paper's printed arrays, storage invariants,
 * brute-force dense products on tiny inputs, closed forms, exact-integer inputs, and the
 * paper's own encoding-independence check (Section 5.2).  Unpinned conventions, stated
 * in the design notes: the direction of dimOrdering for rank >= 3 permutations that are
 * not their own inverse, duplicates being an error, and width 0 meaning 64 bits.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#include <float.h>

#define OR_MAX_RANK 8

enum {
    OR_OK = 0, OR_ERR_NULL = 1, OR_ERR_RANK = 2, OR_ERR_LEVEL_TYPE = 3, OR_ERR_ORDERING = 4,
    OR_ERR_WIDTH = 5, OR_ERR_COORD_RANGE = 6, OR_ERR_DUPLICATE = 7, OR_ERR_SHAPE = 8,
    OR_ERR_DTYPE = 9, OR_ERR_UNSUPPORTED = 10, OR_ERR_TOO_LARGE = 11, OR_ERR_ALLOC = 12
};
enum { OR_DENSE = 0, OR_COMPRESSED = 1 };
enum { OR_F32 = 0, OR_F64 = 1 };

typedef struct {
    int rank;
    int lt[OR_MAX_RANK];        /* level type of level l */
    int perm[OR_MAX_RANK];      /* perm[l] = dimension stored at level l */
    int pw, cw;                 /* widths in bits, already resolved (0 -> 64) */
    int dtype;
    int64_t shape[OR_MAX_RANK]; /* by dimension */
    int64_t size[OR_MAX_RANK];  /* by level: size[l] = shape[perm[l]] */
    int64_t *pos[OR_MAX_RANK];  /* NULL for dense levels */
    int64_t npos[OR_MAX_RANK];
    int64_t *crd[OR_MAX_RANK];
    int64_t ncrd[OR_MAX_RANK];
    double *values;             /* f32 inputs are held widened: exact both ways */
    int64_t nvalues;
} oracle_tensor;

void oracle_tensor_free(oracle_tensor *t)
{
    if (!t) return;
    for (int l = 0; l < OR_MAX_RANK; ++l) { free(t->pos[l]); free(t->crd[l]); }
    free(t->values);
    free(t);
}

static int width_ok(int w) { return w == 0 || w == 8 || w == 16 || w == 32 || w == 64; }

static int fits(int64_t v, int w)
{
    if (w >= 64) return 1;
    return v <= (((int64_t)1 << (w - 1)) - 1);
}

/* --- lexicographic stable merge sort of entry ids by their level coordinates ---------- */
typedef struct { const int64_t *lc; int rank; } sort_ctx;

static int tuple_less(const sort_ctx *c, int64_t a, int64_t b)
{
    const int64_t *pa = c->lc + a * c->rank, *pb = c->lc + b * c->rank;
    for (int l = 0; l < c->rank; ++l) {
        if (pa[l] < pb[l]) return 1;
        if (pa[l] > pb[l]) return 0;
    }
    return 0;
}

static void msort(const sort_ctx *c, int64_t *a, int64_t *tmp, int64_t lo, int64_t hi)
{
    if (hi - lo < 2) return;
    int64_t mid = lo + (hi - lo) / 2;
    msort(c, a, tmp, lo, mid);
    msort(c, a, tmp, mid, hi);
    int64_t i = lo, j = mid, k = lo;
    while (i < mid && j < hi) {
        /* take from the right run only when it is strictly smaller: stable */
        if (tuple_less(c, a[j], a[i])) tmp[k++] = a[j++]; else tmp[k++] = a[i++];
    }
    while (i < mid) tmp[k++] = a[i++];
    while (j < hi) tmp[k++] = a[j++];
    memcpy(a + lo, tmp + lo, (size_t)(hi - lo) * sizeof(int64_t));
}

/* Build the storage of Section 4.1 from COO.  coords[d][e] = coordinate of entry e in
 * dimension d (original dimension order).  Validation order: null, rank, level type,
 * ordering, width, shape, coordinate range, duplicate. */
int oracle_pack(int rank, const int *levelTypes, const int *dimOrdering, int posWidth, int crdWidth,
                const int64_t *shape, int64_t nnz, const int64_t *const *coords, const void *values,
                int dtype, oracle_tensor **out)
{
    if (!levelTypes || !shape || !out || (nnz > 0 && (!coords || !values))) return OR_ERR_NULL;
    *out = NULL;
    if (rank < 1 || rank > OR_MAX_RANK) return OR_ERR_RANK;
    for (int l = 0; l < rank; ++l)
        if (levelTypes[l] != OR_DENSE && levelTypes[l] != OR_COMPRESSED) return OR_ERR_LEVEL_TYPE;
    int seen[OR_MAX_RANK] = {0};
    for (int l = 0; l < rank; ++l) {
        int d = dimOrdering ? dimOrdering[l] : l;
        if (d < 0 || d >= rank || seen[d]) return OR_ERR_ORDERING;
        seen[d] = 1;
    }
    if (!width_ok(posWidth) || !width_ok(crdWidth)) return OR_ERR_WIDTH;
    if (dtype != OR_F32 && dtype != OR_F64) return OR_ERR_DTYPE;
    if (nnz < 0) return OR_ERR_SHAPE;
    for (int d = 0; d < rank; ++d) if (shape[d] < 0) return OR_ERR_SHAPE;
    for (int d = 0; d < rank && nnz > 0; ++d) if (!coords[d]) return OR_ERR_NULL;
    for (int d = 0; d < rank; ++d)
        for (int64_t e = 0; e < nnz; ++e)
            if (coords[d][e] < 0 || coords[d][e] >= shape[d]) return OR_ERR_COORD_RANGE;

    oracle_tensor *t = (oracle_tensor *)calloc(1, sizeof(oracle_tensor));
    if (!t) return OR_ERR_ALLOC;
    t->rank = rank; t->dtype = dtype;
    t->pw = posWidth ? posWidth : 64;
    t->cw = crdWidth ? crdWidth : 64;
    for (int l = 0; l < rank; ++l) {
        t->lt[l] = levelTypes[l];
        t->perm[l] = dimOrdering ? dimOrdering[l] : l;
        t->shape[l] = shape[l];
    }
    for (int l = 0; l < rank; ++l) t->size[l] = shape[t->perm[l]];

    /* level coordinates, entry-major so that one comparison touches one cache line */
    int64_t *lc = (int64_t *)malloc((size_t)(nnz > 0 ? nnz : 1) * rank * sizeof(int64_t));
    int64_t *ord = (int64_t *)malloc((size_t)(nnz > 0 ? nnz : 1) * sizeof(int64_t));
    int64_t *tmp = (int64_t *)malloc((size_t)(nnz > 0 ? nnz : 1) * sizeof(int64_t));
    int64_t *parent = (int64_t *)malloc((size_t)(nnz > 0 ? nnz : 1) * sizeof(int64_t));
    if (!lc || !ord || !tmp || !parent) { free(lc); free(ord); free(tmp); free(parent); oracle_tensor_free(t); return OR_ERR_ALLOC; }
    for (int64_t e = 0; e < nnz; ++e) {
        for (int l = 0; l < rank; ++l) lc[e * rank + l] = coords[t->perm[l]][e];
        ord[e] = e;
    }
    sort_ctx sc = { lc, rank };
    msort(&sc, ord, tmp, 0, nnz);
    int status = OR_OK;
    for (int64_t s = 1; s < nnz && status == OR_OK; ++s)
        if (!tuple_less(&sc, ord[s - 1], ord[s])) status = OR_ERR_DUPLICATE;

    /* walk the levels; parent[s] = position of sorted entry s at the level above */
    int64_t P = 1;
    for (int64_t s = 0; s < nnz; ++s) parent[s] = 0;
    for (int l = 0; l < rank && status == OR_OK; ++l) {
        int64_t sz = t->size[l];
        if (t->lt[l] == OR_DENSE) {
            if (sz != 0 && P > INT64_MAX / sz) { status = OR_ERR_TOO_LARGE; break; }
            for (int64_t s = 0; s < nnz; ++s) parent[s] = parent[s] * sz + lc[ord[s] * rank + l];
            P *= sz;
        } else {
            int64_t *pos = (int64_t *)calloc((size_t)P + 1, sizeof(int64_t));
            int64_t *crd = (int64_t *)malloc((size_t)(nnz > 0 ? nnz : 1) * sizeof(int64_t));
            if (!pos || !crd) { free(pos); free(crd); status = OR_ERR_ALLOC; break; }
            int64_t nchild = 0, prev_parent = -1, prev_c = -1;
            for (int64_t s = 0; s < nnz; ++s) {
                int64_t c = lc[ord[s] * rank + l];
                if (s == 0 || parent[s] != prev_parent || c != prev_c) {
                    crd[nchild++] = c;
                    pos[parent[s] + 1] += 1;          /* count, shifted by one for the prefix sum */
                }
                prev_parent = parent[s]; prev_c = c;
                parent[s] = nchild - 1;
            }
            for (int64_t p = 0; p < P; ++p) pos[p + 1] += pos[p];
            t->pos[l] = pos; t->npos[l] = P + 1;
            t->crd[l] = crd; t->ncrd[l] = nchild;
            if (!fits(nchild, t->pw) || (sz > 0 && !fits(sz - 1, t->cw))) { status = OR_ERR_WIDTH; break; }
            P = nchild;
        }
    }
    if (status == OR_OK) {
        t->values = (double *)calloc((size_t)(P > 0 ? P : 1), sizeof(double));
        t->nvalues = P;
        if (!t->values) status = OR_ERR_ALLOC;
        else for (int64_t s = 0; s < nnz; ++s) {
            int64_t e = ord[s];
            t->values[parent[s]] = dtype == OR_F32 ? (double)((const float *)values)[e] : ((const double *)values)[e];
        }
    }
    free(lc); free(ord); free(tmp); free(parent);
    if (status != OR_OK) { oracle_tensor_free(t); return status; }
    *out = t;
    return OR_OK;
}

/* --- accessors ------------------------------------------------------------------------ */
int64_t oracle_pos_len(const oracle_tensor *t, int l) { return (l >= 0 && l < t->rank && t->pos[l]) ? t->npos[l] : -1; }
int64_t oracle_crd_len(const oracle_tensor *t, int l) { return (l >= 0 && l < t->rank && t->pos[l]) ? t->ncrd[l] : -1; }
int64_t oracle_values_len(const oracle_tensor *t) { return t->nvalues; }
int oracle_pos_width(const oracle_tensor *t) { return t->pw; }
int oracle_crd_width(const oracle_tensor *t) { return t->cw; }

static void narrow_copy(const int64_t *src, int64_t n, int w, void *dst)
{
    for (int64_t i = 0; i < n; ++i) {
        switch (w) {
        case 8:  ((int8_t *)dst)[i] = (int8_t)src[i]; break;
        case 16: ((int16_t *)dst)[i] = (int16_t)src[i]; break;
        case 32: ((int32_t *)dst)[i] = (int32_t)src[i]; break;
        default: ((int64_t *)dst)[i] = src[i]; break;
        }
    }
}
/* copies in the tensor's own bit width (signed) */
void oracle_get_pos(const oracle_tensor *t, int l, void *dst) { narrow_copy(t->pos[l], t->npos[l], t->pw, dst); }
void oracle_get_crd(const oracle_tensor *t, int l, void *dst) { narrow_copy(t->crd[l], t->ncrd[l], t->cw, dst); }
void oracle_get_values(const oracle_tensor *t, void *dst)
{
    for (int64_t i = 0; i < t->nvalues; ++i) {
        if (t->dtype == OR_F32) ((float *)dst)[i] = (float)t->values[i];
        else ((double *)dst)[i] = t->values[i];
    }
}

/* --- generic level walk: visits every stored position in storage order ---------------- */
typedef void (*visit_fn)(void *ctx, const int64_t *dimcoord, double v);

static void walk(const oracle_tensor *t, int l, int64_t p, int64_t *dimcoord, visit_fn f, void *ctx)
{
    if (l == t->rank) { f(ctx, dimcoord, t->values[p]); return; }
    if (t->lt[l] == OR_DENSE) {
        for (int64_t k = 0; k < t->size[l]; ++k) {
            dimcoord[t->perm[l]] = k;
            walk(t, l + 1, p * t->size[l] + k, dimcoord, f, ctx);
        }
    } else {
        for (int64_t q = t->pos[l][p]; q < t->pos[l][p + 1]; ++q) {
            dimcoord[t->perm[l]] = t->crd[l][q];
            walk(t, l + 1, q, dimcoord, f, ctx);
        }
    }
}

typedef struct { int rank; int64_t **coords; double *vals; int64_t n; } unpack_ctx;
static void unpack_visit(void *c_, const int64_t *dc, double v)
{
    unpack_ctx *c = (unpack_ctx *)c_;
    for (int d = 0; d < c->rank; ++d) c->coords[d][c->n] = dc[d];
    c->vals[c->n] = v;
    c->n++;
}
/* Every stored position (padding zeros of dense-under-compressed levels included), in
 * storage order, with coordinates in the original dimension order.  Arrays must hold
 * oracle_values_len() entries; values come back as f64. */
int64_t oracle_unpack(const oracle_tensor *t, int64_t **coords, double *vals)
{
    unpack_ctx c = { t->rank, coords, vals, 0 };
    int64_t dc[OR_MAX_RANK];
    walk(t, 0, 0, dc, unpack_visit, &c);
    return c.n;
}

/* --- the product ---------------------------------------------------------------------- */
#if LDBL_MANT_DIG < 64
#error "the checker wants an extended-precision long double (x87)"
#endif

static double ldB(const void *B, int dtype, int64_t idx)
{
    return dtype == OR_F32 ? (double)((const float *)B)[idx] : ((const double *)B)[idx];
}

static int finish_product(long double *acc, int64_t m, int64_t N, void *C, int64_t ldc, int dtype)
{
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < N; ++j) {
            if (dtype == OR_F32) ((float *)C)[i * ldc + j] = (float)acc[i * N + j];
            else ((double *)C)[i * ldc + j] = (double)acc[i * N + j];
        }
    return OR_OK;
}

static long double *start_product(int64_t m, int64_t N, const void *C, int64_t ldc, int dtype, int accumulate, double *mag)
{
    size_t cnt = (size_t)(m * N > 0 ? m * N : 1);
    long double *acc = (long double *)malloc(cnt * sizeof(long double));
    if (!acc) return NULL;
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < N; ++j) {
            acc[i * N + j] = accumulate ? (long double)ldB(C, dtype, i * ldc + j) : 0.0L;
            if (mag) mag[i * N + j] = accumulate ? fabs(ldB(C, dtype, i * ldc + j)) : 0.0;
        }
    return acc;
}

/* C[i,j] (+)= sum over the COO triples, in the caller's order, of a * B[k,j]; accumulators
 * are long double, rounded once at the end.  mag[i*N+j] = sum |a * B[k,j]| (+ |C_in| when
 * accumulating): the scale the parity tolerance is stated against.  mag may be NULL. */
int oracle_matmul_coo(int64_t m, int64_t n, int64_t nnz, const int64_t *rows, const int64_t *cols,
                      const void *vals, int dtype, const void *B, int64_t N, int64_t ldb,
                      void *C, int64_t ldc, int accumulate, double *mag)
{
    if ((nnz > 0 && (!rows || !cols || !vals)) || (N > 0 && n > 0 && !B) || (N > 0 && m > 0 && !C)) return OR_ERR_NULL;
    if (m < 0 || n < 0 || N < 0 || ldb < N || ldc < N) return OR_ERR_SHAPE;
    for (int64_t e = 0; e < nnz; ++e)
        if (rows[e] < 0 || rows[e] >= m || cols[e] < 0 || cols[e] >= n) return OR_ERR_COORD_RANGE;
    long double *acc = start_product(m, N, C, ldc, dtype, accumulate, mag);
    if (!acc) return OR_ERR_ALLOC;
    for (int64_t e = 0; e < nnz; ++e) {
        int64_t i = rows[e], k = cols[e];
        long double a = (long double)ldB(vals, dtype, e);
        for (int64_t j = 0; j < N; ++j) {
            long double prod = a * (long double)ldB(B, dtype, k * ldb + j);
            acc[i * N + j] += prod;
            if (mag) mag[i * N + j] += (double)fabsl(prod);
        }
    }
    finish_product(acc, m, N, C, ldc, dtype);
    free(acc);
    return OR_OK;
}

typedef struct { long double *acc; double *mag; const void *B; int dtype; int64_t N, ldb; } mm_ctx;
static void mm_visit(void *c_, const int64_t *dc, double v)
{
    mm_ctx *c = (mm_ctx *)c_;
    int64_t i = dc[0], k = dc[1];
    for (int64_t j = 0; j < c->N; ++j) {
        long double prod = (long double)v * (long double)ldB(c->B, c->dtype, k * c->ldb + j);
        c->acc[i * c->N + j] += prod;
        if (c->mag) c->mag[i * c->N + j] += (double)fabsl(prod);
    }
}
/* The same product, computed by walking pos/crd/values of a packed rank-2 tensor under
 * whatever encoding it has: ties the storage semantics to the product. */
int oracle_matmul_storage(const oracle_tensor *t, const void *B, int64_t N, int64_t ldb,
                          void *C, int64_t ldc, int accumulate, double *mag)
{
    if (!t) return OR_ERR_NULL;
    if (t->rank != 2) return OR_ERR_RANK;
    int64_t m = t->shape[0];
    if (N < 0 || ldb < N || ldc < N) return OR_ERR_SHAPE;
    long double *acc = start_product(m, N, C, ldc, t->dtype, accumulate, mag);
    if (!acc) return OR_ERR_ALLOC;
    mm_ctx c = { acc, mag, B, t->dtype, N, ldb };
    int64_t dc[OR_MAX_RANK];
    walk(t, 0, 0, dc, mm_visit, &c);
    finish_product(acc, m, N, C, ldc, t->dtype);
    free(acc);
    return OR_OK;
}

/* Plain-f64 sequential product in the caller's order (no extended precision): used by a
 * test that shows the extended-precision result is not the noise source. */
int oracle_matmul_coo_f64seq(int64_t m, int64_t nnz, const int64_t *rows, const int64_t *cols,
                             const double *vals, const double *B, int64_t N, int64_t ldb, double *C, int64_t ldc)
{
    for (int64_t i = 0; i < m; ++i) for (int64_t j = 0; j < N; ++j) C[i * ldc + j] = 0.0;
    for (int64_t e = 0; e < nnz; ++e)
        for (int64_t j = 0; j < N; ++j) C[rows[e] * ldc + j] += vals[e] * B[cols[e] * ldb + j];
    return OR_OK;
}

/* Sampled dense-dense product (Section 6.2, last experiment): X[i,j] = S[i,j] * sum_k A[i,k] * B[k,j], computed
 * only where S stores an entry.  S comes as COO triples; X and mag are per triple, in the caller's order.  A is m x K
 * and B is K x n, both row-major.  Inner sums in long double, rounded once; mag = |s| * sum_k |A[i,k] * B[k,j]|. */
int oracle_sddmm_coo(int64_t m, int64_t n, int64_t K, int64_t nnz, const int64_t *rows, const int64_t *cols,
                     const void *svals, int dtype, const void *A, int64_t lda, const void *B, int64_t ldb,
                     void *X, double *mag)
{
    if (nnz > 0 && (!rows || !cols || !svals || !X)) return OR_ERR_NULL;
    if (K > 0 && nnz > 0 && (!A || !B)) return OR_ERR_NULL;
    if (m < 0 || n < 0 || K < 0 || lda < K || ldb < n) return OR_ERR_SHAPE;
    for (int64_t e = 0; e < nnz; ++e)
        if (rows[e] < 0 || rows[e] >= m || cols[e] < 0 || cols[e] >= n) return OR_ERR_COORD_RANGE;
    for (int64_t e = 0; e < nnz; ++e) {
        const int64_t i = rows[e], j = cols[e];
        long double acc = 0.0L, macc = 0.0L;
        for (int64_t k = 0; k < K; ++k) {
            const long double prod = (long double)ldB(A, dtype, i * lda + k) * (long double)ldB(B, dtype, k * ldb + j);
            acc += prod;
            macc += fabsl(prod);
        }
        const long double s = (long double)ldB(svals, dtype, e);
        if (dtype == OR_F32) ((float *)X)[e] = (float)(s * acc); else ((double *)X)[e] = (double)(s * acc);
        if (mag) mag[e] = (double)(fabsl(s) * macc);
    }
    return OR_OK;
}

/* Matricized tensor times Khatri-Rao product (Section 6.3): A[i,j] = sum_{k,l} B[i,k,l] * D[l,j] * C[k,j] for a
 * rank-3 tensor B of shape I x K x L given as COO triples (any order), C of K x J and D of L x J, both row-major.
 * Plain definition: one pass over the triples, every term formed and added in long double, rounded once at the
 * end; mag[i,j] = sum of the terms' absolute values.  With accumulate != 0 the sums start from A's contents. */
int oracle_mttkrp_coo(int64_t I, int64_t K, int64_t L, int64_t J, int64_t nnz, const int64_t *ci, const int64_t *ck,
                      const int64_t *cl, const void *bvals, int dtype, const void *C, int64_t ldc, const void *D,
                      int64_t ldd, void *A, int64_t lda, int accumulate, double *mag)
{
    if (nnz > 0 && (!ci || !ck || !cl || !bvals)) return OR_ERR_NULL;
    if (I > 0 && J > 0 && !A) return OR_ERR_NULL;
    if (nnz > 0 && J > 0 && (!C || !D)) return OR_ERR_NULL;
    if (I < 0 || K < 0 || L < 0 || J < 0 || ldc < J || ldd < J || lda < J) return OR_ERR_SHAPE;
    if (dtype != OR_F32 && dtype != OR_F64) return OR_ERR_DTYPE;
    for (int64_t e = 0; e < nnz; ++e)
        if (ci[e] < 0 || ci[e] >= I || ck[e] < 0 || ck[e] >= K || cl[e] < 0 || cl[e] >= L) return OR_ERR_COORD_RANGE;
    if (I == 0 || J == 0) return OR_OK;
    long double *acc = (long double *)calloc((size_t)(I * J), sizeof(long double));
    long double *macc = (long double *)calloc((size_t)(I * J), sizeof(long double));
    if (!acc || !macc) { free(acc); free(macc); return OR_ERR_ALLOC; }
    if (accumulate)
        for (int64_t i = 0; i < I; ++i)
            for (int64_t j = 0; j < J; ++j) acc[i * J + j] = (long double)ldB(A, dtype, i * lda + j);
    for (int64_t e = 0; e < nnz; ++e) {
        const int64_t i = ci[e], k = ck[e], l = cl[e];
        const long double b = (long double)ldB(bvals, dtype, e);
        for (int64_t j = 0; j < J; ++j) {
            const long double term = b * (long double)ldB(D, dtype, l * ldd + j) * (long double)ldB(C, dtype, k * ldc + j);
            acc[i * J + j] += term;
            macc[i * J + j] += fabsl(term);
        }
    }
    for (int64_t i = 0; i < I; ++i)
        for (int64_t j = 0; j < J; ++j) {
            if (dtype == OR_F32) ((float *)A)[i * lda + j] = (float)acc[i * J + j];
            else ((double *)A)[i * lda + j] = (double)acc[i * J + j];
            if (mag) mag[i * J + j] = (double)macc[i * J + j];
        }
    free(acc);
    free(macc);
    return OR_OK;
}

/* Sparse times sparse with a sparse result (Sections 4.2 and 4.4, the SpMSpM kernel): C[i,j] = sum_k A[i,k] * B[k,j]
 * with A (m x kdim) and B (kdim x n) given as COO triples in any order.  The result is what the paper's row-wise
 * loop with a workspace inserts: an entry (i,j) is stored as soon as one pair A[i,k], B[k,j] of stored entries
 * exists, whatever its sum comes to (explicit zeros and cancellations stay stored).  Plain definition on a dense
 * m x n accumulator in long double (this is a checker for moderate sizes: 25 bytes per element of C), every pair
 * taken in the order of A's triples, then of B's triples within row k; each sum is rounded once at the end.
 * Output in row-major lexicographic order: first call with ci = NULL to get the count, then with arrays of that
 * length.  mag[e] = sum of |a * b| over the pairs of entry e. */
int64_t oracle_spgemm_coo(int64_t m, int64_t kdim, int64_t n, int64_t nnzA, const int64_t *ra, const int64_t *ca,
                          const void *va, int64_t nnzB, const int64_t *rb, const int64_t *cb, const void *vb, int dtype,
                          int64_t *ci, int64_t *cj, void *cv, double *mag)
{
    if ((nnzA > 0 && (!ra || !ca || !va)) || (nnzB > 0 && (!rb || !cb || !vb))) return -OR_ERR_NULL;
    if (m < 0 || kdim < 0 || n < 0) return -OR_ERR_SHAPE;
    if (dtype != OR_F32 && dtype != OR_F64) return -OR_ERR_DTYPE;
    for (int64_t e = 0; e < nnzA; ++e)
        if (ra[e] < 0 || ra[e] >= m || ca[e] < 0 || ca[e] >= kdim) return -OR_ERR_COORD_RANGE;
    for (int64_t e = 0; e < nnzB; ++e)
        if (rb[e] < 0 || rb[e] >= kdim || cb[e] < 0 || cb[e] >= n) return -OR_ERR_COORD_RANGE;
    if (m == 0 || n == 0) return 0;
    if ((long double)m * (long double)n > 268435456.0L) return -OR_ERR_TOO_LARGE;
    /* B's triples grouped by row k, keeping their order: start[k] .. start[k+1] index into `by_row` */
    int64_t *start = (int64_t *)calloc((size_t)kdim + 2, sizeof(int64_t));
    int64_t *by_row = (int64_t *)malloc((size_t)(nnzB > 0 ? nnzB : 1) * sizeof(int64_t));
    long double *acc = (long double *)calloc((size_t)(m * n), sizeof(long double));
    double *macc = (double *)calloc((size_t)(m * n), sizeof(double));
    unsigned char *filled = (unsigned char *)calloc((size_t)(m * n), 1);
    if (!start || !by_row || !acc || !macc || !filled) { free(start); free(by_row); free(acc); free(macc); free(filled); return -OR_ERR_ALLOC; }
    for (int64_t e = 0; e < nnzB; ++e) start[rb[e] + 2]++;
    for (int64_t k = 0; k < kdim; ++k) start[k + 2] += start[k + 1];
    for (int64_t e = 0; e < nnzB; ++e) by_row[start[rb[e] + 1]++] = e;      /* afterwards start[k+1] = end of row k */
    for (int64_t e = 0; e < nnzA; ++e) {
        const int64_t i = ra[e], k = ca[e];
        const long double a = (long double)ldB(va, dtype, e);
        for (int64_t t = start[k]; t < start[k + 1]; ++t) {
            const int64_t eb = by_row[t], j = cb[eb];
            const long double prod = a * (long double)ldB(vb, dtype, eb);
            acc[i * n + j] += prod;
            macc[i * n + j] += (double)fabsl(prod);
            filled[i * n + j] = 1;
        }
    }
    int64_t count = 0;
    for (int64_t x = 0; x < m * n; ++x)
        if (filled[x]) {
            if (ci) {
                ci[count] = x / n;
                cj[count] = x % n;
                if (dtype == OR_F32) ((float *)cv)[count] = (float)acc[x]; else ((double *)cv)[count] = (double)acc[x];
                if (mag) mag[count] = macc[x];
            }
            ++count;
        }
    free(start); free(by_row); free(acc); free(macc); free(filled);
    return count;
}
