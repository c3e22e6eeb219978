/* A client of the library written in plain C (compiled with gcc, not hipcc): includes the public header as C, lets the
 * library use its default allocator (hipMalloc / hipFree: NULL callbacks), and checks a few tiny cases whose expected
 * results are worked out here by the plain definitions on small integers (exact in floating point).
 * Prints "c client ok" and returns 0 when everything matches. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <hip/hip_runtime_api.h>
#include "spmi.h"

#define CHECK(cond)                                                          \
    do {                                                                     \
        if (!(cond)) {                                                       \
            printf("c client: line %d: check failed: %s\n", __LINE__, #cond); \
            return 1;                                                        \
        }                                                                    \
    } while (0)
#define HIP(call) CHECK((call) == hipSuccess)
#define SP(call)                                                                              \
    do {                                                                                      \
        sp_status s__ = (call);                                                               \
        if (s__ != SP_OK) {                                                                   \
            printf("c client: line %d: %s (hip %d)\n", __LINE__, sp_status_str(s__), sp_last_hip_error()); \
            return 1;                                                                         \
        }                                                                                     \
    } while (0)

static void *to_device(const void *host, size_t bytes)
{
    void *d = NULL;
    if (hipMalloc(&d, bytes ? bytes : 16) != hipSuccess) return NULL;
    if (host && bytes && hipMemcpy(d, host, bytes, hipMemcpyHostToDevice) != hipSuccess) return NULL;
    return d;
}

int main(void)
{
    /* ---- a 4 x 5 matrix, 7 entries given out of order, stored as CSR with 32-bit arrays -------------------------- */
    enum { M = 4, N = 5, NNZ = 7 };
    const int64_t rows[NNZ] = {3, 0, 2, 0, 3, 2, 3};
    const int64_t cols[NNZ] = {4, 1, 0, 3, 0, 2, 2};
    const double vals[NNZ] = {7, 1, 3, 2, 5, 4, 6};
    const int32_t want_pos[M + 1] = {0, 2, 2, 4, 7};
    const int32_t want_crd[NNZ] = {1, 3, 0, 2, 0, 2, 4};
    const double want_val[NNZ] = {1, 2, 3, 4, 5, 6, 7};
    const sp_level_type csr[2] = {SP_DENSE, SP_COMPRESSED};
    sp_encoding *enc = NULL;
    SP(sp_encode(2, csr, NULL, 32, 32, &enc));
    const sp_level_type bad[2] = {SP_DENSE, (sp_level_type)7};
    sp_encoding *none = NULL;
    CHECK(sp_encode(2, bad, NULL, 32, 32, &none) == SP_ERR_LEVEL_TYPE && none == NULL);
    CHECK(sp_status_str(SP_ERR_DUPLICATE) != NULL && strlen(sp_status_str(SP_ERR_DUPLICATE)) > 0);

    int64_t *drows = (int64_t *)to_device(rows, sizeof(rows)), *dcols = (int64_t *)to_device(cols, sizeof(cols));
    double *dvals = (double *)to_device(vals, sizeof(vals));
    CHECK(drows && dcols && dvals);
    const int64_t shape[2] = {M, N};
    const int64_t *coords[2] = {drows, dcols};
    sp_tensor *A = NULL;
    SP(sp_pack(enc, shape, NNZ, coords, dvals, SP_F64, NULL, NULL, NULL, NULL, &A));

    const void *p = NULL;
    int64_t len = 0;
    int32_t got_pos[M + 1], got_crd[NNZ];
    double got_val[NNZ];
    SP(sp_pos(A, 1, &p, &len));
    CHECK(len == M + 1);
    HIP(hipMemcpy(got_pos, p, sizeof(got_pos), hipMemcpyDeviceToHost));
    SP(sp_crd(A, 1, &p, &len));
    CHECK(len == NNZ);
    HIP(hipMemcpy(got_crd, p, sizeof(got_crd), hipMemcpyDeviceToHost));
    SP(sp_values(A, &p, &len));
    CHECK(len == NNZ);
    HIP(hipMemcpy(got_val, p, sizeof(got_val), hipMemcpyDeviceToHost));
    CHECK(memcmp(got_pos, want_pos, sizeof(want_pos)) == 0);
    CHECK(memcmp(got_crd, want_crd, sizeof(want_crd)) == 0);
    CHECK(memcmp(got_val, want_val, sizeof(want_val)) == 0);
    CHECK(sp_pos(A, 0, &p, &len) == SP_ERR_LEVEL_TYPE);           /* level 0 is dense */

    sp_info info;
    SP(sp_tensor_info(A, &info));
    CHECK(info.rank == 2 && info.nnz == NNZ && info.nvalues == NNZ && info.posWidth == 32 && info.maxSegment == 3);

    /* ---- C = A.B for one and two columns, and C += A.B --------------------------------------------------------- */
    double B[N * 2], want_C[M * 2], got_C[M * 2];
    for (int k = 0; k < N; ++k) { B[2 * k] = k + 1; B[2 * k + 1] = -(double)k; }
    memset(want_C, 0, sizeof(want_C));
    for (int e = 0; e < NNZ; ++e)
        for (int j = 0; j < 2; ++j) want_C[rows[e] * 2 + j] += vals[e] * B[cols[e] * 2 + j];
    double *dB = (double *)to_device(B, sizeof(B)), *dC = (double *)to_device(NULL, sizeof(got_C));
    CHECK(dB && dC);
    SP(sp_matmul(A, dB, 2, 2, dC, 2, 0, NULL));
    HIP(hipDeviceSynchronize());
    HIP(hipMemcpy(got_C, dC, sizeof(got_C), hipMemcpyDeviceToHost));
    CHECK(memcmp(got_C, want_C, sizeof(want_C)) == 0);
    SP(sp_matmul(A, dB, 2, 2, dC, 2, 1, NULL));                   /* accumulate: twice the product */
    HIP(hipDeviceSynchronize());
    HIP(hipMemcpy(got_C, dC, sizeof(got_C), hipMemcpyDeviceToHost));
    for (int i = 0; i < M * 2; ++i) CHECK(got_C[i] == 2 * want_C[i]);
    SP(sp_matmul(A, dB, 1, 2, dC, 2, 0, NULL));                   /* one column of B with its leading dimension: SpMV */
    HIP(hipDeviceSynchronize());
    HIP(hipMemcpy(got_C, dC, sizeof(got_C), hipMemcpyDeviceToHost));
    for (int i = 0; i < M; ++i) CHECK(got_C[2 * i] == want_C[2 * i]);
    CHECK(sp_matmul(A, dB, 2, 1, dC, 2, 0, NULL) == SP_ERR_SHAPE);  /* ldb < N */

    /* ---- the same entry twice is an error and leaves nothing behind ------------------------------------------- */
    {
        const int64_t r2[2] = {1, 1}, c2[2] = {2, 2};
        const double v2[2] = {1, 1};
        int64_t *dr = (int64_t *)to_device(r2, sizeof(r2)), *dc = (int64_t *)to_device(c2, sizeof(c2));
        double *dv = (double *)to_device(v2, sizeof(v2));
        const int64_t *cc[2] = {dr, dc};
        sp_tensor *D = (sp_tensor *)1;
        CHECK(sp_pack(enc, shape, 2, cc, dv, SP_F64, NULL, NULL, NULL, NULL, &D) == SP_ERR_DUPLICATE && D == NULL);
        HIP(hipFree(dr)); HIP(hipFree(dc)); HIP(hipFree(dv));
    }

    /* ---- C = A.At with a sparse result: (A.At)[i][j] = sum_k A[i][k] * A[j][k] ------------------------------- */
    {
        const int64_t tshape[2] = {N, M};
        const int64_t *tcoords[2] = {dcols, drows};               /* the transpose is the same triples with the roles swapped */
        sp_tensor *At = NULL, *P = NULL;
        SP(sp_pack(enc, tshape, NNZ, tcoords, dvals, SP_F64, NULL, NULL, NULL, NULL, &At));
        SP(sp_spgemm(A, At, enc, NULL, &P));
        double dense[M][M];
        int stored[M][M], count = 0;
        memset(dense, 0, sizeof(dense));
        memset(stored, 0, sizeof(stored));
        for (int a = 0; a < NNZ; ++a)
            for (int b = 0; b < NNZ; ++b)
                if (cols[a] == cols[b]) { dense[rows[a]][rows[b]] += vals[a] * vals[b]; stored[rows[a]][rows[b]] = 1; }
        for (int i = 0; i < M; ++i) for (int j = 0; j < M; ++j) count += stored[i][j];
        sp_info pi;
        SP(sp_tensor_info(P, &pi));
        CHECK(pi.nvalues == count && pi.shape[0] == M && pi.shape[1] == M);
        int32_t ppos[M + 1], pcrd[M * M];
        double pval[M * M];
        SP(sp_pos(P, 1, &p, &len));
        HIP(hipMemcpy(ppos, p, sizeof(ppos), hipMemcpyDeviceToHost));
        SP(sp_crd(P, 1, &p, &len));
        HIP(hipMemcpy(pcrd, p, (size_t)count * 4, hipMemcpyDeviceToHost));
        SP(sp_values(P, &p, &len));
        HIP(hipMemcpy(pval, p, (size_t)count * 8, hipMemcpyDeviceToHost));
        int at = 0;
        for (int i = 0; i < M; ++i) {
            CHECK(ppos[i] == at);
            for (int j = 0; j < M; ++j)
                if (stored[i][j]) { CHECK(pcrd[at] == j && pval[at] == dense[i][j]); ++at; }
        }
        CHECK(ppos[M] == at && at == count);
        sp_tensor_free(P);
        sp_tensor_free(At);
    }

    /* ---- a 2 x 3 x 4 tensor of ones on its full grid: MTTKRP with factors of ones gives K * L everywhere ------- */
    {
        enum { I3 = 2, K3 = 3, L3 = 4, J3 = 6, N3 = I3 * K3 * L3 };
        int64_t ci[N3], ck[N3], cl[N3];
        double ones[N3], fk[K3 * J3], fl[L3 * J3], out[I3 * J3];
        for (int e = 0; e < N3; ++e) { ci[e] = e / (K3 * L3); ck[e] = (e / L3) % K3; cl[e] = e % L3; ones[e] = 1.0; }
        for (int x = 0; x < K3 * J3; ++x) fk[x] = 1.0;
        for (int x = 0; x < L3 * J3; ++x) fl[x] = 1.0;
        const sp_level_type dss[3] = {SP_DENSE, SP_COMPRESSED, SP_COMPRESSED};
        sp_encoding *e3 = NULL;
        SP(sp_encode(3, dss, NULL, 32, 32, &e3));
        int64_t *di = (int64_t *)to_device(ci, sizeof(ci)), *dk = (int64_t *)to_device(ck, sizeof(ck)), *dl = (int64_t *)to_device(cl, sizeof(cl));
        double *dv = (double *)to_device(ones, sizeof(ones)), *dfk = (double *)to_device(fk, sizeof(fk)), *dfl = (double *)to_device(fl, sizeof(fl));
        double *dout = (double *)to_device(NULL, sizeof(out));
        CHECK(di && dk && dl && dv && dfk && dfl && dout);
        const int64_t shape3[3] = {I3, K3, L3};
        const int64_t *c3[3] = {di, dk, dl};
        sp_tensor *T = NULL;
        SP(sp_pack(e3, shape3, N3, c3, dv, SP_F64, NULL, NULL, NULL, NULL, &T));
        SP(sp_mttkrp(T, dfk, J3, dfl, J3, J3, dout, J3, 0, NULL));
        HIP(hipDeviceSynchronize());
        HIP(hipMemcpy(out, dout, sizeof(out), hipMemcpyDeviceToHost));
        for (int x = 0; x < I3 * J3; ++x) CHECK(out[x] == (double)(K3 * L3));
        sp_tensor_free(T);
        sp_encoding_free(e3);
        HIP(hipFree(di)); HIP(hipFree(dk)); HIP(hipFree(dl)); HIP(hipFree(dv)); HIP(hipFree(dfk)); HIP(hipFree(dfl)); HIP(hipFree(dout));
    }

    sp_tensor_free(A);
    sp_encoding_free(enc);
    HIP(hipFree(drows)); HIP(hipFree(dcols)); HIP(hipFree(dvals)); HIP(hipFree(dB)); HIP(hipFree(dC));
    printf("c client ok\n");
    return 0;
}
