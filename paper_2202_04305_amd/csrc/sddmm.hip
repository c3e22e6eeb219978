// Sampled dense-dense product X[i,j] = S[i,j] * sum_k A[i,k] * B[k,j] (arXiv 2202.04305, Section 6.2: the kernel of
// the state-space search experiment).  X has S's sparsity pattern, so the result is one value per stored position
// of S, in storage order: no insertion into a sparse output is needed.
//
// Per stored entry (i, j) the kernel needs row i of A and column j of B.  B is K x n row-major in the paper's
// formula, so a column is a stride-n walk; it is transposed once per call into an n x K scratch (unless the caller
// already holds it that way), after which every entry reads one contiguous row of K values, exactly as the SpMM
// kernel reads rows of its dense operand.  A wave takes one stored row of S: the row of A sits in registers, LR
// lanes cover one row of the transposed B with 16-byte loads, 64 / LR entries go side by side, and a short
// shuffle reduction over the LR lanes finishes each dot product.
#include "spmi_internal.h"

namespace {

constexpr int kThreads = 256;

template <typename VT>
__global__ __launch_bounds__(256) void transpose_kernel(const VT *__restrict__ B, int64_t K, int64_t n, int64_t ldb,
                                                        VT *__restrict__ Bt, int64_t ldt)
{
    __shared__ VT tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;          // 32 x 8 threads
    const int64_t j0 = (int64_t)blockIdx.x * 32, k0 = (int64_t)blockIdx.y * 32;
#pragma unroll
    for (int r = ty; r < 32; r += 8)
        if (k0 + r < K && j0 + tx < n) tile[r][tx] = B[(k0 + r) * ldb + j0 + tx];
    __syncthreads();
#pragma unroll
    for (int r = ty; r < 32; r += 8)
        if (j0 + r < n && k0 + tx < K) Bt[(j0 + r) * ldt + k0 + tx] = tile[tx][r];
}

// 16-byte loads: K = LR * (16 / sizeof(VT)), rows of A and of the transposed B 16-byte aligned.
// Work is cut by stored entries, not by rows: block w owns the entries [w*T, (w+1)*T) (T and the table `rowblk` of
// the row holding every T-th entry are the stream SpMV's), its waves take the rows that meet that window in turn
// and each handles the part of its row inside the window.  A row of 20,000 entries is thus spread over 20 blocks
// instead of being walked by one wave; no results need combining because every entry has its own output.
// The window's values of S and, instead of its coordinates, the byte offsets of the rows of the transposed B that they
// select are first copied into LDS with coalesced loads, so
// that the loop over the entries does its index arithmetic on small window-relative integers and every gather address
// is a wave-uniform base plus a lane offset (OT: 32 bits when the matrix is below 4 GB).
template <typename PT, typename CT, typename VT, int LR, typename OT>
__global__ __launch_bounds__(kThreads) void sddmm_windows_vec_kernel(const PT *__restrict__ pos, const CT *__restrict__ crd,
                                                                     const VT *__restrict__ sval, const CT *__restrict__ rowid,
                                                                     const int32_t *__restrict__ rowblk, int64_t nrows, int64_t nnz,
                                                                     const VT *__restrict__ A, int64_t lda,
                                                                     const VT *__restrict__ Bt, int64_t ldt, VT *__restrict__ X)
{
    constexpr int V = 16 / sizeof(VT);
    constexpr int S = 64 / LR;
    constexpr int U = S >= 4 ? 2 : 4;
    constexpr int T = (int)kSpmiStreamT;
    typedef VT vec_t __attribute__((ext_vector_type(V)));
    __shared__ OT s_off[T];
    __shared__ VT s_val[T];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int jl = lane % LR, sl = lane / LR;
    const int64_t s = (int64_t)blockIdx.x * T;
    const int64_t e = s + T < nnz ? s + T : nnz;
    const int ne = (int)(e - s);
    const OT brow = (OT)(ldt * (int64_t)sizeof(VT));
    for (int i = threadIdx.x; i < ne; i += kThreads) {
        s_off[i] = (OT)crd[s + i] * brow;
        s_val[i] = sval[s + i];
    }
    const int64_t lo = rowblk[blockIdx.x], hi = rowblk[blockIdx.x + 1];
    const int64_t last = hi < nrows ? hi : nrows - 1;
    __syncthreads();
    const char *Bb = (const char *)Bt;
    const OT colb = (OT)(jl * V * (int)sizeof(VT));
    VT *Xw = X + s;                                   // this window's part of the result
    int slot[U];
#pragma unroll
    for (int u = 0; u < U; ++u) slot[u] = sl + u * S;
    for (int64_t r = lo + wave; r <= last; r += kThreads / 64) {
        const int64_t pa = (int64_t)pos[r], pb = (int64_t)pos[r + 1];
        const int a = (int)((pa > s ? pa : s) - s), b = (int)((pb < e ? pb : e) - s);
        if (b <= a) continue;                         // wave-uniform
        const int64_t i = rowid ? (int64_t)rowid[r] : r;
        const vec_t av = *(const vec_t *)(A + i * lda + jl * V);
        // the step count is the same for every lane of the wave, so the shuffles run with all lanes active;
        // entries past the end are clamped and their result dropped
        for (int p0 = a; p0 < b; p0 += U * S) {
            vec_t bv[U];
            int pp[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                pp[u] = p0 + slot[u];
                const int pc = pp[u] < b ? pp[u] : b - 1;
                bv[u] = *(const vec_t *)(Bb + (s_off[pc] + colb));
            }
            VT dot[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                dot[u] = 0;
#pragma unroll
                for (int ee = 0; ee < V; ++ee) dot[u] += av[ee] * bv[u][ee];
            }
            if (LR >= U) {
                // The U sums are reduced together: each of the first log2(U) exchange steps halves the number of sums
                // a lane carries (a lane keeps the half its bit selects and hands the other half over), the remaining
                // steps finish the one sum left.  U - 1 + log2(LR / U) shuffles instead of U * log2(LR); sum u ends
                // complete in the lanes whose top bits of jl are u.
                int m = LR / 2;
#pragma unroll
                for (int n = U; n > 1; n >>= 1) {
                    const bool upper = (jl & m) != 0;
#pragma unroll
                    for (int k = 0; k < n / 2; ++k) {
                        const VT send = upper ? dot[k] : dot[k + n / 2];
                        const VT keep = upper ? dot[k + n / 2] : dot[k];
                        dot[k] = keep + __shfl_xor(send, m, 64);
                    }
                    m >>= 1;
                }
#pragma unroll
                for (; m >= 1; m >>= 1) dot[0] += __shfl_xor(dot[0], m, 64);
                constexpr int G = LR / U > 0 ? LR / U : 1;      // lanes that end with the same sum
                const int u = jl / G;
                int mine = pp[0];
#pragma unroll
                for (int k = 1; k < U; ++k) mine = u == k ? pp[k] : mine;
                if (jl % G == 0 && mine < b) Xw[mine] = s_val[mine] * dot[0];
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) {
#pragma unroll
                    for (int d = LR / 2; d >= 1; d >>= 1) dot[u] += __shfl_xor(dot[u], d, 64);
                    if (jl == 0 && pp[u] < b) Xw[pp[u]] = s_val[pp[u]] * dot[u];
                }
            }
        }
    }
}

// any K: CG lanes per entry, each striding over k
template <typename PT, typename CT, typename VT, int CG>
__global__ __launch_bounds__(kThreads) void sddmm_rows_kernel(const PT *__restrict__ pos, const CT *__restrict__ crd,
                                                              const VT *__restrict__ sval, const CT *__restrict__ rowid, int64_t nrows,
                                                              const VT *__restrict__ A, int64_t lda, const VT *__restrict__ Bt,
                                                              int64_t ldt, int64_t K, VT *__restrict__ X)
{
    constexpr int S = 64 / CG;
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (r >= nrows) return;
    const int jl = lane % CG, sl = lane / CG;
    const int64_t a = (int64_t)pos[r], b = (int64_t)pos[r + 1];
    if (a == b) return;
    const int64_t i = rowid ? (int64_t)rowid[r] : r;
    const int64_t steps = (b - a + S - 1) / S;
    for (int64_t t = 0; t < steps; ++t) {
        const int64_t p = a + t * S + sl;
        const int64_t pc = p < b ? p : b - 1;
        const int64_t j = (int64_t)crd[pc];
        VT dot = 0;
        for (int64_t k = jl; k < K; k += CG) dot += A[i * lda + k] * Bt[j * ldt + k];
#pragma unroll
        for (int d = CG / 2; d >= 1; d >>= 1) dot += __shfl_xor(dot, d, 64);
        if (jl == 0 && p < b) X[p] = sval[p] * dot;
    }
}

inline unsigned grid_for(int64_t n, int64_t per_block) { return (unsigned)(n > 0 ? ceil_div(n, per_block) : 1); }

template <typename PT, typename CT, typename VT>
sp_status sddmm_t(const sp_tensor *S, const VT *A, int64_t lda, const VT *B, int64_t ldb, int b_is_transposed, int64_t K, VT *X,
                  hipStream_t st)
{
    const PT *pos = (const PT *)S->pos[1];
    const CT *crd = (const CT *)S->crd[1];
    const VT *sval = (const VT *)S->values;
    const CT *rowid = S->enc.lt[0] == SP_COMPRESSED ? (const CT *)S->crd[0] : nullptr;
    int64_t nrows = S->npos[1] - 1;
    const sp_rowblocks *rowblocks = &S->rowblocks;
    if (!rowid && S->nz_pos) { pos = (const PT *)S->nz_pos; rowid = (const CT *)S->nz_rowid; nrows = S->nz_rows; rowblocks = &S->nz_rowblocks; }
    const int64_t n = S->shape[1];
    if (S->nvalues == 0 || nrows == 0) return SP_OK;
    if (K == 0) return spmi_fill_zero(X, (size_t)S->nvalues * sizeof(VT), st);   // X was allocated by the caller: exact size, 4-byte multiple

    sp_mem mem{S->alloc, S->free_, S->ctx};
    constexpr int64_t V = 16 / sizeof(VT);
    const VT *Bt = B;
    int64_t ldt = ldb;
    if (!b_is_transposed) {
        ldt = (K + V - 1) / V * V;                         // rows of the scratch start 16-byte aligned
        // the transposed operand lives in scratch the tensor keeps and grows on demand: only a call that needs more than any
        // call before it allocates (and then waits for the stream, since the old block may still be read)
        const size_t need = (size_t)(n > 0 ? n : 1) * ldt * sizeof(VT);
        if (S->sddmm_bt_bytes < need) {
            if (S->sddmm_bt) { SP_HIP(hipStreamSynchronize(st)); mem.put(S->sddmm_bt); S->sddmm_bt = nullptr; S->sddmm_bt_bytes = 0; }
            S->sddmm_bt = mem.get((need + 255) & ~(size_t)255);
            if (!S->sddmm_bt) return SP_ERR_ALLOC;
            S->sddmm_bt_bytes = need;
        }
        VT *scratch = (VT *)S->sddmm_bt;
        hipLaunchKernelGGL(transpose_kernel<VT>, dim3(grid_for(n, 32), grid_for(K, 32)), dim3(256), 0, st, B, K, n, ldb, scratch, ldt);
        SP_HIP(hipGetLastError());
        Bt = scratch;
    }
    {
        sp_prof_scope prof(S, st);
        const int64_t lr = K / V;
        const bool vec = rowblocks->start && K % V == 0 && (lr == 1 || lr == 2 || lr == 4 || lr == 8 || lr == 16 || lr == 32 || lr == 64) && lda % V == 0 &&
                         ldt % V == 0 && (uintptr_t)A % 16 == 0 && (uintptr_t)Bt % 16 == 0;
        const bool small = sizeof(CT) == 4 && (uint64_t)n * (uint64_t)ldt * sizeof(VT) < ((uint64_t)1 << 32);      // 32-bit byte offsets into the transposed B (64-bit coordinates keep 64-bit offsets)
        const dim3 grid(grid_for(nrows, kThreads / 64));
        if (vec) {
#define SPMI_SDDMM_VEC_O(LR, OT)                                                                                              \
    hipLaunchKernelGGL((sddmm_windows_vec_kernel<PT, CT, VT, LR, OT>), dim3((unsigned)rowblocks->nblocks), dim3(kThreads), 0, st, pos, crd, \
                       sval, rowid, (const int32_t *)rowblocks->start, nrows, S->ncrd[1], A, lda, Bt, ldt, X)
#define SPMI_SDDMM_VEC(LR)                              \
    do {                                                \
        if (small) SPMI_SDDMM_VEC_O(LR, uint32_t);      \
        else SPMI_SDDMM_VEC_O(LR, uint64_t);            \
    } while (0)
            if (lr == 1) SPMI_SDDMM_VEC(1);
            else if (lr == 2) SPMI_SDDMM_VEC(2);
            else if (lr == 4) SPMI_SDDMM_VEC(4);
            else if (lr == 8) SPMI_SDDMM_VEC(8);
            else if (lr == 16) SPMI_SDDMM_VEC(16);
            else if (lr == 32) SPMI_SDDMM_VEC(32);
            else SPMI_SDDMM_VEC(64);
#undef SPMI_SDDMM_VEC
#undef SPMI_SDDMM_VEC_O
        } else {
#define SPMI_SDDMM(CG)                                                                                                        \
    hipLaunchKernelGGL((sddmm_rows_kernel<PT, CT, VT, CG>), grid, dim3(kThreads), 0, st, pos, crd, sval, rowid, nrows, A, lda, Bt, ldt, \
                       K, X)
            if (K > 32) SPMI_SDDMM(64);
            else if (K > 8) SPMI_SDDMM(32);
            else if (K > 2) SPMI_SDDMM(8);
            else SPMI_SDDMM(2);
#undef SPMI_SDDMM
        }
        SP_HIP(hipGetLastError());
    }
    return SP_OK;
}

}  // namespace

extern "C" sp_status sp_sddmm(const sp_tensor *S, const void *A, int64_t lda, const void *B, int64_t ldb, int b_is_transposed,
                              int64_t K, void *X, void *stream)
{
    if (!S) return SP_ERR_NULL;
    if (S->enc.rank != 2) return SP_ERR_RANK;
    const int64_t n = S->shape[1];
    if (K < 0 || lda < K || (b_is_transposed ? ldb < K : ldb < n)) return SP_ERR_SHAPE;
    if (S->nvalues > 0 && (!X || (K > 0 && (!A || !B)))) return SP_ERR_NULL;
    if (S->enc.perm[0] != 0 || S->enc.lt[1] != SP_COMPRESSED) return SP_ERR_UNSUPPORTED;   // row-major with a compressed inner level
    hipStream_t st = (hipStream_t)stream;
    SP_TRY(spmi_ensure_tables(S, st));
    const int pw = S->enc.pw, cw = S->enc.cw;
#define SPMI_GO(PT, CT)                                                                                                       \
    return S->dtype == SP_F64 ? sddmm_t<PT, CT, double>(S, (const double *)A, lda, (const double *)B, ldb, b_is_transposed, K, (double *)X, st) \
                              : sddmm_t<PT, CT, float>(S, (const float *)A, lda, (const float *)B, ldb, b_is_transposed, K, (float *)X, st)
    if (pw == 32 && cw == 32) SPMI_GO(int32_t, int32_t);
    if (pw == 32) SPMI_GO(int32_t, int64_t);
    if (cw == 32) SPMI_GO(int64_t, int32_t);
    SPMI_GO(int64_t, int64_t);
#undef SPMI_GO
}
