// Matricized tensor times Khatri-Rao product A[i,j] = sum_{k,l} B[i,k,l] * D[l,j] * C[k,j] (arXiv 2202.04305,
// Section 6.3) for a packed rank-3 tensor B whose outermost level stores dimension i (dense or compressed) and whose
// two inner levels are compressed, in either order of k and l (the two formats of the paper's experiment).
//
// Call "mid" the factor matrix indexed by the level-1 coordinate and "inner" the one indexed by the level-2
// coordinate.  For a level-1 fibre f (one pair of level-0 position and level-1 coordinate m) the sum factors as
//     A[i,:] += mid[m,:] .* sum_{p in fibre f} values[p] * inner[crd2[p],:]
// so the hot loop is the SpMM loop over the entries of a fibre (a gather of rows of `inner`), one elementwise product
// per fibre, and a running sum per slice i.  Both factor matrices are small next to B (megabytes) and live in cache;
// B's crd2 / values stream from HBM once.
//
// Work is cut by stored entries: wave w owns the entries [w*TW, (w+1)*TW) and walks the fibres that meet that window,
// each clipped to it.  LR lanes cover the J columns (16-byte loads when J allows) and S = 64 / LR entries go side by
// side; the S partial sums meet only when a slice ends.  The part of a slice that began in an earlier window goes to
// carry[w] (J values); a second kernel adds the carries to A in window order; everything else is written to A
// directly.  No atomics: results are bit-reproducible.
#include "spmi_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int64_t kTW = 512;                  // stored entries per wave

__global__ __launch_bounds__(kThreads) void zero_rows_kernel(char *__restrict__ A, int64_t rows, int64_t row_bytes, int64_t ld_bytes)
{
    const int64_t words = row_bytes / 4;      // element sizes are 4 or 8
    const int64_t total = rows * words;
    for (int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x; t < total; t += (int64_t)gridDim.x * kThreads)
        *(uint32_t *)(A + (t / words) * ld_bytes + (t % words) * 4) = 0u;
}

// wfib[w] = level-1 fibre holding entry w*TW, wslc[w] = level-0 position holding that fibre (largest index whose
// pos entry is <= the target: empty slices are skipped by construction)
template <typename PT>
__global__ __launch_bounds__(kThreads) void mttkrp_windows_table_kernel(const PT *__restrict__ pos1, int64_t nslc,
                                                                        const PT *__restrict__ pos2, int64_t nfib, int64_t nwin,
                                                                        int32_t *__restrict__ wfib, int32_t *__restrict__ wslc)
{
    const int64_t w = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (w >= nwin) return;
    const int64_t s = w * kTW;
    int64_t lo = 0, hi = nfib - 1;            // pos2[lo] <= s always (pos2[0] = 0)
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if ((int64_t)pos2[mid] <= s) lo = mid; else hi = mid - 1;
    }
    const int64_t f = lo;
    lo = 0; hi = nslc - 1;
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if ((int64_t)pos1[mid] <= f) lo = mid; else hi = mid - 1;
    }
    wfib[w] = (int32_t)f;
    wslc[w] = (int32_t)lo;
}

template <typename VT, int V>
struct vec_of { typedef VT type __attribute__((ext_vector_type(V))); };

// grid = (windows / waves per block, column tiles of 64 * V columns)
template <typename PT, typename CT, typename VT, int V, int U>
__global__ __launch_bounds__(kThreads) void mttkrp_windows_kernel(const PT *__restrict__ pos1, const CT *__restrict__ crd0,
                                                                  const CT *__restrict__ crd1, const PT *__restrict__ pos2,
                                                                  const CT *__restrict__ crd2, const VT *__restrict__ val,
                                                                  const int32_t *__restrict__ wfib, const int32_t *__restrict__ wslc,
                                                                  int64_t nwin, int64_t nfib, int64_t nnz,
                                                                  const VT *__restrict__ M, int64_t ldm, const VT *__restrict__ X,
                                                                  int64_t ldx, VT *__restrict__ A, int64_t lda,
                                                                  VT *__restrict__ carry, int64_t J, int accumulate)
{
    typedef typename vec_of<VT, V>::type vec_t;
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * kWaves + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if (w >= nwin) return;
    const int64_t j0 = (int64_t)blockIdx.y * 64 * V;
    const int64_t jw = J - j0 < 64 * V ? J - j0 : 64 * V;          // columns of this tile (a multiple of V)
    const int LR = (int)(jw / V);                                  // lanes per row, 1..64
    const int S = 64 / LR;                                         // entries side by side
    const int jl = lane % LR, sl = lane / LR;
    const bool live = sl < S;
    const int64_t col = j0 + (int64_t)jl * V;
    const int64_t s = w * kTW;
    const int64_t e = s + kTW < nnz ? s + kTW : nnz;
    int64_t f = wfib[w], q = wslc[w];
    int64_t qend = (int64_t)pos1[q + 1];
    bool cont = (int64_t)pos2[(int64_t)pos1[q]] < s;               // the first slice began in an earlier window
    vec_t acc = (vec_t)(0);

    auto flush = [&](int64_t slice) {
        vec_t r = acc;
        for (int g = 1; g < S; ++g) {
#pragma unroll
            for (int c = 0; c < V; ++c) r[c] += __shfl(acc[c], jl + g * LR, 64);
        }
        if (sl == 0) {
            if (cont) *(vec_t *)(carry + w * J + col) = r;
            else {
                const int64_t i = crd0 ? (int64_t)crd0[slice] : slice;
                vec_t *dst = (vec_t *)(A + i * lda + col);
                *dst = accumulate ? *dst + r : r;
            }
        }
        cont = false;
        acc = (vec_t)(0);
    };

    int64_t pa = (int64_t)pos2[f];
    while (pa < e) {                                               // wave-uniform throughout
        const int64_t pb = (int64_t)pos2[f + 1];
        if (f >= qend) {
            flush(q);
            do { ++q; qend = (int64_t)pos1[q + 1]; } while (f >= qend);
        }
        const int64_t a = pa > s ? pa : s, b = pb < e ? pb : e;
        const vec_t c = *(const vec_t *)(M + (int64_t)crd1[f] * ldm + col);
        vec_t t[U];
#pragma unroll
        for (int u = 0; u < U; ++u) t[u] = (vec_t)(0);
        for (int64_t p0 = a; p0 < b; p0 += (int64_t)S * U) {
            int64_t l[U];
            VT v[U];
            vec_t xv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t pp = p0 + sl + (int64_t)u * S;
                const bool in = live && pp < b;
                l[u] = (int64_t)crd2[in ? pp : a];
                v[u] = in ? val[pp] : (VT)0;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) xv[u] = *(const vec_t *)(X + l[u] * ldx + col);
#pragma unroll
            for (int u = 0; u < U; ++u) t[u] += v[u] * xv[u];
        }
#pragma unroll
        for (int u = 1; u < U; ++u) t[0] += t[u];
        acc += c * t[0];
        ++f;
        pa = pb;
        if (f >= nfib) break;
    }
    flush(q);
}

// A wave per window boundary: the first boundary a slice crosses adds all of that slice's carries, in window order.
template <typename PT, typename CT, typename VT>
__global__ __launch_bounds__(kThreads) void mttkrp_fixup_kernel(const PT *__restrict__ pos1, const CT *__restrict__ crd0,
                                                                const PT *__restrict__ pos2, const int32_t *__restrict__ wslc,
                                                                int64_t nwin, int64_t J, const VT *__restrict__ carry,
                                                                VT *__restrict__ A, int64_t lda)
{
    const int lane = threadIdx.x & 63;
    const int64_t b = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6) + 1;
    if (b >= nwin) return;
    const int64_t q = wslc[b];
    const int64_t start = (int64_t)pos2[(int64_t)pos1[q]];
    if (start >= b * kTW || start < (b - 1) * kTW) return;        // not crossed here, or crossed earlier already
    const int64_t i = crd0 ? (int64_t)crd0[q] : q;
    int64_t last = b;
    while (last + 1 < nwin && wslc[last + 1] == q) ++last;
    for (int64_t j = lane; j < J; j += 64) {
        VT sum = 0;
        for (int64_t bb = b; bb <= last; ++bb) sum += carry[bb * J + j];
        A[i * lda + j] += sum;
    }
}

template <typename PT, typename CT, typename VT>
sp_status mttkrp_t(const sp_tensor *B, const VT *M, int64_t ldm, const VT *X, int64_t ldx, int64_t J, VT *A, int64_t lda,
                   int accumulate, hipStream_t st)
{
    const int64_t I = B->shape[0];
    if (I == 0 || J == 0) return SP_OK;
    if (!accumulate) {
        hipLaunchKernelGGL(zero_rows_kernel, dim3((unsigned)(ceil_div(I * J, kThreads) < 2048 ? ceil_div(I * J, kThreads) : 2048)),
                           dim3(kThreads), 0, st, (char *)A, I, J * (int64_t)sizeof(VT), lda * (int64_t)sizeof(VT));
        SP_HIP(hipGetLastError());
    }
    const int64_t nnz = B->nvalues;
    if (nnz == 0) return SP_OK;
    const PT *pos1 = (const PT *)B->pos[1], *pos2 = (const PT *)B->pos[2];
    const CT *crd0 = (const CT *)B->crd[0], *crd1 = (const CT *)B->crd[1], *crd2 = (const CT *)B->crd[2];
    const int64_t nslc = B->npos[1] - 1, nfib = B->npos[2] - 1;
    const int64_t nwin = ceil_div(nnz, kTW);
    sp_tensor *Bt = const_cast<sp_tensor *>(B);
    sp_mem mem{B->alloc, B->free_, B->ctx};
    if (!Bt->mttkrp_windows) {
        Bt->mttkrp_windows = mem.get((size_t)nwin * 8);
        if (!Bt->mttkrp_windows) return SP_ERR_ALLOC;
        int32_t *wfib = (int32_t *)Bt->mttkrp_windows, *wslc = wfib + nwin;
        hipLaunchKernelGGL(mttkrp_windows_table_kernel<PT>, dim3((unsigned)ceil_div(nwin, kThreads)), dim3(kThreads), 0, st, pos1, nslc,
                           pos2, nfib, nwin, wfib, wslc);
        SP_HIP(hipGetLastError());
    }
    const size_t need = (size_t)nwin * J * sizeof(VT);
    if (Bt->mttkrp_carry_bytes < need) {
        if (Bt->mttkrp_carry) { SP_HIP(hipStreamSynchronize(st)); mem.put(Bt->mttkrp_carry); Bt->mttkrp_carry = nullptr; Bt->mttkrp_carry_bytes = 0; }
        Bt->mttkrp_carry = mem.get((need + 255) & ~(size_t)255);
        if (!Bt->mttkrp_carry) return SP_ERR_ALLOC;
        Bt->mttkrp_carry_bytes = need;
    }
    const int32_t *wfib = (const int32_t *)B->mttkrp_windows, *wslc = wfib + nwin;
    constexpr int VV = 16 / sizeof(VT);
    const bool vec = J % VV == 0 && ldm % VV == 0 && ldx % VV == 0 && lda % VV == 0 && (uintptr_t)M % 16 == 0 && (uintptr_t)X % 16 == 0 &&
                     (uintptr_t)A % 16 == 0 && (uintptr_t)B->mttkrp_carry % 16 == 0;
    {
        sp_prof_scope prof(B, st);
        const unsigned gx = (unsigned)ceil_div(nwin, kWaves);
#define SPMI_MTTKRP(V, U)                                                                                                              \
    hipLaunchKernelGGL((mttkrp_windows_kernel<PT, CT, VT, V, U>), dim3(gx, (unsigned)ceil_div(J, 64 * V)), dim3(kThreads), 0, st, pos1, crd0, \
                       crd1, pos2, crd2, (const VT *)B->values, wfib, wslc, nwin, nfib, nnz, M, ldm, X, ldx, A, lda,                    \
                       (VT *)B->mttkrp_carry, J, accumulate)
        const int64_t lanes = vec ? J / VV : J;                 // lanes a row of the (first) column tile takes
        const bool few_side_by_side = 64 / (lanes < 64 ? lanes : 64) < 4;
        if (vec) {
            if (few_side_by_side) SPMI_MTTKRP(VV, 4);
            else SPMI_MTTKRP(VV, 2);
        } else {
            if (few_side_by_side) SPMI_MTTKRP(1, 4);
            else SPMI_MTTKRP(1, 2);
        }
#undef SPMI_MTTKRP
        SP_HIP(hipGetLastError());
    }
    if (nwin > 1) {
        hipLaunchKernelGGL((mttkrp_fixup_kernel<PT, CT, VT>), dim3((unsigned)ceil_div(nwin - 1, kWaves)), dim3(kThreads), 0, st, pos1, crd0,
                           pos2, wslc, nwin, J, (const VT *)B->mttkrp_carry, A, lda);
        SP_HIP(hipGetLastError());
    }
    return SP_OK;
}

}  // namespace

extern "C" sp_status sp_mttkrp(const sp_tensor *B, const void *C, int64_t ldc, const void *D, int64_t ldd, int64_t J, void *A,
                               int64_t lda, int accumulate, void *stream)
{
    if (!B) return SP_ERR_NULL;
    if (B->enc.rank != 3) return SP_ERR_RANK;
    if (J < 0 || ldc < J || ldd < J || lda < J) return SP_ERR_SHAPE;
    if (J > 0 && B->shape[0] > 0 && !A) return SP_ERR_NULL;
    if (J > 0 && B->nvalues > 0 && (!C || !D)) return SP_ERR_NULL;
    // dimension i outermost, both inner levels compressed; anything else: convert first
    if (B->enc.perm[0] != 0 || B->enc.lt[1] != SP_COMPRESSED || B->enc.lt[2] != SP_COMPRESSED) return SP_ERR_UNSUPPORTED;
    const bool k_first = B->enc.perm[1] == 1;
    const void *M = k_first ? C : D, *X = k_first ? D : C;
    const int64_t ldm = k_first ? ldc : ldd, ldx = k_first ? ldd : ldc;
    hipStream_t st = (hipStream_t)stream;
    const int pw = B->enc.pw, cw = B->enc.cw;
#define SPMI_GO(PT, CT)                                                                                                            \
    return B->dtype == SP_F64 ? mttkrp_t<PT, CT, double>(B, (const double *)M, ldm, (const double *)X, ldx, J, (double *)A, lda, accumulate, st) \
                              : mttkrp_t<PT, CT, float>(B, (const float *)M, ldm, (const float *)X, ldx, J, (float *)A, lda, accumulate, st)
    if (pw == 32 && cw == 32) SPMI_GO(int32_t, int32_t);
    if (pw == 32) SPMI_GO(int32_t, int64_t);
    if (cw == 32) SPMI_GO(int64_t, int32_t);
    SPMI_GO(int64_t, int64_t);
#undef SPMI_GO
}
