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
// carry[w] (J values); a second kernel adds a slice's carries to A in a fixed pattern; everything else is written to A
// directly.  No atomics: results are bit-reproducible.
#include "spmi_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
// stored entries per wave.  Measured on the 76.9 M-entry tensor with 42 columns: 512 -> 3.18 ms, 256 -> 2.21, 128 -> 1.97,
// 64 -> 2.15: with small windows fewer slices are in flight at a time and more of their factor rows are found in the L2.
constexpr int64_t kTW = 128;

__global__ __launch_bounds__(kThreads) void zero_rows_kernel(char *__restrict__ A, int64_t rows, int64_t row_bytes, int64_t ld_bytes)
{
    const int64_t words = row_bytes / 4;      // element sizes are 4 or 8
    const int64_t total = rows * words;
    for (int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x; t < total; t += (int64_t)gridDim.x * kThreads)
        *(uint32_t *)(A + (t / words) * ld_bytes + (t % words) * 4) = 0u;
}

// dst[r, 0..cols) = src[r, 0..cols) for a row-major matrix with other leading dimensions (16-byte pieces)
__global__ __launch_bounds__(kThreads) void repitch_rows_kernel(const char *__restrict__ src, int64_t src_ld_bytes, int64_t rows,
                                                                int64_t row_bytes, char *__restrict__ dst, int64_t dst_ld_bytes)
{
    const int64_t pieces = row_bytes / 16;
    const int64_t total = rows * pieces;
    for (int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x; t < total; t += (int64_t)gridDim.x * kThreads) {
        const int64_t r = t / pieces, c = t % pieces;
        *(uint4 *)(dst + r * dst_ld_bytes + c * 16) = *(const uint4 *)(src + r * src_ld_bytes + c * 16);
    }
}

// wfib[w] = level-1 fibre holding entry w*TW, wslc[w] = level-0 position holding that fibre (largest index whose
// pos entry is <= the target: empty slices are skipped by construction).  A window boundary w that is the first one
// its slice crosses (the slice begins inside window w - 1) is appended to `cross` (count in cross[-1]); the order of
// that list does not matter, every entry is an independent piece of work for the fix-up kernel.  An entry is the
// pair (w, last window that begins inside the same slice).
template <typename PT>
__global__ __launch_bounds__(kThreads) void mttkrp_windows_table_kernel(const PT *__restrict__ pos1, int64_t nslc,
                                                                        const PT *__restrict__ pos2, int64_t nfib, int64_t nwin,
                                                                        int32_t *__restrict__ wfib, int32_t *__restrict__ wslc,
                                                                        int32_t *__restrict__ cross)
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
    if (w >= 1) {
        const int64_t start = (int64_t)pos2[(int64_t)pos1[lo]];
        if (start < s && start >= s - kTW) {
            const int64_t end = (int64_t)pos2[(int64_t)pos1[lo + 1]];      // first entry past the slice
            const int64_t a = (end - 1) / kTW;                             // last window that begins inside the slice
            const int at = atomicAdd(&cross[-1], 1);
            cross[2 * at] = (int32_t)w;
            cross[2 * at + 1] = (int32_t)a;
        }
    }
}

template <typename VT, int V>
struct vec_of { typedef VT type __attribute__((ext_vector_type(V))); };

// grid = (windows / waves per block rounded up to a multiple of 8, column tiles of 64 * V columns).  Each wave first
// copies its window into LDS with coalesced loads that are all in flight together: the values, and instead of the
// coordinates the byte offsets of the rows they select (crd2 -> row of the inner factor, crd1 -> row of the mid
// factor, of type OT: 32 bits when both matrices are below 4 GB), plus the fibres' bounds relative to the window.
// The walk over the fibres afterwards does no index arithmetic beyond one add per gather.
template <typename PT, typename CT, typename VT, int V, int U, typename OT>
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
    __shared__ VT s_val[kWaves][kTW];
    __shared__ OT s_xoff[kWaves][kTW];
    __shared__ OT s_moff[kWaves][kTW + 1];      // at most TW + 1 fibres meet a window (the last may only touch its end)
    __shared__ int32_t s_off[kWaves][kTW + 2];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // Workgroups go to the 8 XCDs in turn, each with an L2 of its own.  Block b therefore takes the (b / 8)-th block of
    // the (b % 8)-th eighth of the windows: an XCD walks a contiguous range of entries, so the rows of the factor
    // matrices that a slice keeps coming back to are found in that XCD's L2.  (Only the mapping depends on this.)
    const int64_t per = gridDim.x / 8;
    const int64_t w = ((int64_t)(blockIdx.x % 8) * per + blockIdx.x / 8) * kWaves + wave;
    const bool active = w < nwin;
    const int64_t s = w * kTW;
    const int64_t e = s + kTW < nnz ? s + kTW : nnz;
    int64_t f0 = 0, q = 0, qend = 0;
    int nf = 0;
    bool cont = false;
    if (active) {
        f0 = wfib[w];
        q = wslc[w];
        nf = (int)((w + 1 < nwin ? (int64_t)wfib[w + 1] : nfib - 1) - f0) + 1;
        const OT xrow = (OT)(ldx * (int64_t)sizeof(VT)), mrow = (OT)(ldm * (int64_t)sizeof(VT));
        for (int64_t p = s + lane; p < e; p += 64) {
            s_xoff[wave][p - s] = (OT)crd2[p] * xrow;
            s_val[wave][p - s] = val[p];
        }
        for (int fi = lane; fi <= nf; fi += 64) {
            int64_t o = (int64_t)pos2[f0 + fi] - s;
            o = o < 0 ? 0 : o > e - s ? e - s : o;
            s_off[wave][fi] = (int32_t)o;
            if (fi < nf) s_moff[wave][fi] = (OT)crd1[f0 + fi] * mrow;
        }
        qend = (int64_t)pos1[q + 1];
        cont = (int64_t)pos2[(int64_t)pos1[q]] < s;                // the first slice began in an earlier window
    }
    __syncthreads();
    if (!active) return;
    const int64_t j0 = (int64_t)blockIdx.y * 64 * V;
    const int64_t jw = J - j0 < 64 * V ? J - j0 : 64 * V;          // columns of this tile (a multiple of V)
    const int LR = (int)(jw / V);                                  // lanes per row, 1..64
    const int S = 64 / LR;                                         // entries side by side
    const int jl = lane % LR, sl = lane / LR;
    const int64_t col = j0 + (int64_t)jl * V;
    const OT colb = (OT)(col * (int64_t)sizeof(VT));
    int slot[U];                                                   // this lane's place in a group of S * U entries
#pragma unroll
    for (int u = 0; u < U; ++u) slot[u] = sl < S ? sl + u * S : (1 << 24);   // lanes beyond LR * S never take an entry
    const char *Xb = (const char *)X, *Mb = (const char *)M;
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

    vec_t c_next = *(const vec_t *)(Mb + (s_moff[wave][0] + colb));
    int b = s_off[wave][0];
    for (int fi = 0; fi < nf; ++fi) {                              // wave-uniform throughout
        const vec_t c = c_next;
        const int a = b;
        b = s_off[wave][fi + 1];
        if (fi + 1 < nf) c_next = *(const vec_t *)(Mb + (s_moff[wave][fi + 1] + colb));
        if (b <= a) continue;                                      // only the last fibre, when it begins where the window ends
        const int64_t f = f0 + fi;
        if (f >= qend) {
            flush(q);
            do { ++q; qend = (int64_t)pos1[q + 1]; } while (f >= qend);
        }
        vec_t t[U];
#pragma unroll
        for (int u = 0; u < U; ++u) t[u] = (vec_t)(0);
        for (int p0 = a; p0 < b; p0 += S * U) {
            VT v[U];
            vec_t xv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (p0 + u * S < b) {                              // wave-uniform: no gather for a slot group past the fibre's end
                    const int pp = p0 + slot[u];
                    const int idx = pp < b ? pp : b - 1;
                    v[u] = s_val[wave][idx];
                    xv[u] = *(const vec_t *)(Xb + (s_xoff[wave][idx] + colb));
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (p0 + u * S < b) {
                    if (p0 + slot[u] < b) t[u] += v[u] * xv[u];
                }
            }
        }
#pragma unroll
        for (int u = 1; u < U; ++u) t[0] += t[u];
        acc += c * t[0];
    }
    flush(q);
}

// A block per listed window boundary (the first one a slice crosses): adds all of that slice's carries to A.  The
// carries are summed in a fixed pattern (four strided partial sums per column, combined in order), so the result is
// the same on every call.
constexpr int kFixThreads = 1024, kFixGroups = kFixThreads / 64;
template <typename CT, typename VT>
__global__ __launch_bounds__(kFixThreads) void mttkrp_fixup_kernel(const CT *__restrict__ crd0, const int32_t *__restrict__ wslc,
                                                                   const int32_t *__restrict__ cross, int64_t nwin, int64_t J,
                                                                   const VT *__restrict__ carry, VT *__restrict__ A, int64_t lda)
{
    __shared__ VT part[kFixGroups][64];
    if ((int)blockIdx.x >= cross[-1]) return;                      // block-uniform
    const int lane = threadIdx.x & 63, g = threadIdx.x >> 6;
    const int64_t b = cross[2 * blockIdx.x], last = cross[2 * blockIdx.x + 1];
    const int32_t q = wslc[b];
    const int64_t i = crd0 ? (int64_t)crd0[q] : (int64_t)q;
    for (int64_t jb = 0; jb < J; jb += 64) {                       // block-uniform
        const int64_t j = jb + lane;
        VT s0 = 0, s1 = 0, s2 = 0, s3 = 0;
        if (j < J) {
            int64_t bb = b + g;
            for (; bb + 3 * kFixGroups <= last; bb += 4 * kFixGroups) {
                s0 += carry[bb * J + j];
                s1 += carry[(bb + kFixGroups) * J + j];
                s2 += carry[(bb + 2 * kFixGroups) * J + j];
                s3 += carry[(bb + 3 * kFixGroups) * J + j];
            }
            for (; bb <= last; bb += kFixGroups) s0 += carry[bb * J + j];
        }
        part[g][lane] = (s0 + s1) + (s2 + s3);
        __syncthreads();
        if (g == 0 && j < J) {
            VT tot = part[0][lane];
#pragma unroll
            for (int k = 1; k < kFixGroups; ++k) tot += part[k][lane];
            A[i * lda + j] += tot;
        }
        __syncthreads();
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
    const sp_tensor *Bt = B;                    // the handle's scratch and tables are its cache (mutable members)
    sp_mem mem{B->alloc, B->free_, B->ctx};
    const int64_t ncross = nslc < nwin - 1 ? nslc : nwin - 1;        // a slice has at most one first crossing
    const size_t table_bytes = (size_t)(2 * nwin + 4 + (ncross > 0 ? 2 * ncross : 0)) * 4;
    if (!Bt->mttkrp_windows) {
        // the handle takes the table only once its build has been enqueued: a failure on the way leaves no half-built table behind
        void *table = mem.get(table_bytes);
        if (!table) return SP_ERR_ALLOC;
        int32_t *wfib = (int32_t *)table, *wslc = wfib + nwin, *cross = wslc + nwin + 4;
        sp_status built = spmi_fill_zero(wslc + nwin, 16, st);     // cross[-1] = 0: the length of the list
        if (built == SP_OK) {
            hipLaunchKernelGGL(mttkrp_windows_table_kernel<PT>, dim3((unsigned)ceil_div(nwin, kThreads)), dim3(kThreads), 0, st, pos1, nslc,
                               pos2, nfib, nwin, wfib, wslc, cross);
            if (hipGetLastError() != hipSuccess) built = SP_ERR_HIP;
        }
        if (built != SP_OK) { (void)hipStreamSynchronize(st); mem.put(table); return built; }
        Bt->mttkrp_windows = table;
    }
    const size_t need = (size_t)nwin * J * sizeof(VT);
    if (Bt->mttkrp_carry_bytes < need) {
        if (Bt->mttkrp_carry) { SP_HIP(hipStreamSynchronize(st)); mem.put(Bt->mttkrp_carry); Bt->mttkrp_carry = nullptr; Bt->mttkrp_carry_bytes = 0; }
        Bt->mttkrp_carry = mem.get((need + 255) & ~(size_t)255);
        if (!Bt->mttkrp_carry) return SP_ERR_ALLOC;
        Bt->mttkrp_carry_bytes = need;
    }
    const int32_t *wfib = (const int32_t *)B->mttkrp_windows, *wslc = wfib + nwin, *cross = wslc + nwin + 4;
    constexpr int VV = 16 / sizeof(VT);
    const bool vec = J % VV == 0 && ldm % VV == 0 && ldx % VV == 0 && lda % VV == 0 && (uintptr_t)M % 16 == 0 && (uintptr_t)X % 16 == 0 &&
                     (uintptr_t)A % 16 == 0 && (uintptr_t)B->mttkrp_carry % 16 == 0;
    // f32 with an even J that is no multiple of four (the 42 columns of the paper's experiment): 8-byte loads
    const bool half_vec = !vec && sizeof(VT) == 4 && J % 2 == 0 && ldm % 2 == 0 && ldx % 2 == 0 && lda % 2 == 0 && (uintptr_t)M % 8 == 0 &&
                          (uintptr_t)X % 8 == 0 && (uintptr_t)A % 8 == 0;
    const int64_t K = B->shape[1], L = B->shape[2];
    const int64_t rows_m = B->enc.perm[1] == 1 ? K : L, rows_x = B->enc.perm[1] == 1 ? L : K;
    // The inner factor is gathered a row per stored entry, the mid factor a row per fibre.  When such a matrix is
    // larger than an XCD's L2 and its rows do not start on 128-byte lines, a copy with rows padded to whole lines is
    // gathered from instead (a 336-byte row then touches 3 lines, not 3.6 on average); the copy is made on every call
    // into a buffer the tensor keeps.
    const int64_t row_bytes = J * (int64_t)sizeof(VT);
    for (int which = 0; which < 2; ++which) {
        const VT *&F = which == 0 ? X : M;
        int64_t &ldf = which == 0 ? ldx : ldm;
        const int64_t rows_f = which == 0 ? rows_x : rows_m;
        if (!(vec && rows_f * row_bytes > ((int64_t)4 << 20) && row_bytes % 128 != 0 &&
              (ldf * (int64_t)sizeof(VT) % 128 != 0 || (uintptr_t)F % 128 != 0)))
            continue;
        const int64_t ldp_bytes = (row_bytes + 127) / 128 * 128;
        const size_t want = (size_t)rows_f * (size_t)ldp_bytes;
        if (Bt->mttkrp_pad_bytes[which] < want) {
            if (Bt->mttkrp_pad[which]) {
                SP_HIP(hipStreamSynchronize(st));
                mem.put(Bt->mttkrp_pad[which]);
                Bt->mttkrp_pad[which] = nullptr;
                Bt->mttkrp_pad_bytes[which] = 0;
            }
            Bt->mttkrp_pad[which] = mem.get(want);
            if (!Bt->mttkrp_pad[which]) return SP_ERR_ALLOC;
            Bt->mttkrp_pad_bytes[which] = want;
        }
        const int64_t pieces = rows_f * (row_bytes / 16);
        hipLaunchKernelGGL(repitch_rows_kernel, dim3((unsigned)(ceil_div(pieces, kThreads) < 4096 ? ceil_div(pieces, kThreads) : 4096)), dim3(kThreads),
                           0, st, (const char *)F, ldf * (int64_t)sizeof(VT), rows_f, row_bytes, (char *)Bt->mttkrp_pad[which], ldp_bytes);
        SP_HIP(hipGetLastError());
        F = (const VT *)Bt->mttkrp_pad[which];
        ldf = ldp_bytes / (int64_t)sizeof(VT);
    }
    // byte offsets into the factor matrices fit 32 bits when both are below 4 GB
    const bool small = sizeof(CT) == 4 && (uint64_t)rows_m * (uint64_t)ldm * sizeof(VT) < ((uint64_t)1 << 32) &&
                       (uint64_t)rows_x * (uint64_t)ldx * sizeof(VT) < ((uint64_t)1 << 32);      // 64-bit coordinates keep 64-bit offsets
    {
        sp_prof_scope prof(B, st);
        const unsigned gx = (unsigned)(ceil_div(ceil_div(nwin, kWaves), 8) * 8);   // a multiple of 8: see the block mapping in the kernel
#define SPMI_MTTKRP(V, U, OT)                                                                                                          \
    hipLaunchKernelGGL((mttkrp_windows_kernel<PT, CT, VT, V, U, OT>), dim3(gx, (unsigned)ceil_div(J, 64 * V)), dim3(kThreads), 0, st, pos1, crd0, \
                       crd1, pos2, crd2, (const VT *)B->values, wfib, wslc, nwin, nfib, nnz, M, ldm, X, ldx, A, lda,                    \
                       (VT *)B->mttkrp_carry, J, accumulate)
#define SPMI_MTTKRP_V(V)                                                        \
    do {                                                                        \
        const int64_t lanes = J / V < 64 ? J / V : 64;                          \
        if (64 / lanes < 4) { if (small) SPMI_MTTKRP(V, 4, uint32_t); else SPMI_MTTKRP(V, 4, uint64_t); } \
        else { if (small) SPMI_MTTKRP(V, 2, uint32_t); else SPMI_MTTKRP(V, 2, uint64_t); }               \
    } while (0)
        if (vec) SPMI_MTTKRP_V(VV);
        else if (half_vec) SPMI_MTTKRP_V(2);
        else SPMI_MTTKRP_V(1);
#undef SPMI_MTTKRP_V
#undef SPMI_MTTKRP
        SP_HIP(hipGetLastError());
    }
    if (ncross > 0) {
        hipLaunchKernelGGL((mttkrp_fixup_kernel<CT, VT>), dim3((unsigned)ncross), dim3(kFixThreads), 0, st, crd0, wslc, cross, nwin, J,
                           (const VT *)B->mttkrp_carry, A, lda);
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
