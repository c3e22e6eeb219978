// C[i,j] = sum_k A[i,k] * B[k,j] with A sparse and B, C dense row-major (arXiv 2202.04305,
// Section 1: the SpMM kernel; Section 6.2: matrix times vector).  The loops the paper's
// compiler would emit visit, per outer position, the pos range of the inner compressed
// level (Section 4.3); the kernels below visit exactly those entries, split differently:
//
//   rows kernel      G lanes per stored row, strided over the row, shuffle reduction.
//   stream kernel    SpMV: every block owns 2048 consecutive stored entries whatever rows
//                    they belong to: coalesced crd/values stream, gathered x, products
//                    staged in LDS, rows reduced from LDS (a thread per short row, a wave per
//                    long one); rows that cross a block boundary are completed by a small
//                    fix-up kernel from per-block carries (deterministic, no atomics).
//   spmm kernel      one wave per stored row, lanes across the columns of B.
//   scatter kernel   column-major storage (CSC / DCSC): a wave per stored column, atomic
//                    adds into the rows of C.
//
// "Row-major" means the outer level holds dimension 0; that level may be dense (CSR: row =
// position) or compressed (DCSR: row = crd0[position], so empty rows cost nothing).
#include "spmi_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kST = kSpmiStreamThreads;        // threads per block of the stream kernel, 8 stored entries each
constexpr int kStreamT = (int)kSpmiStreamT;   // stored entries per block of the stream kernel (the row blocks are built for it)
constexpr int kLongRow = 64;        // in-window row length above which a wave reduces the row
constexpr int kQueue = 64;
constexpr int64_t kSpmvSliceBytes = (int64_t)2 << 20;     // slice of x one column panel gathers from: half of a 4 MB per-XCD L2
constexpr int kPre = 1;             // rounds of the row loop whose pos entries are fetched ahead
static_assert(kStreamT / (kLongRow + 1) < kQueue, "queue of long rows too small");

template <typename T>
__device__ __forceinline__ T wave_sum(T v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

template <typename VT>
__global__ __launch_bounds__(kThreads) void zero_matrix_kernel(VT *__restrict__ C, int64_t m, int64_t N, int64_t ldc)
{
    const int64_t total = m * N;
    int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (; i < total; i += stride) C[(i / N) * ldc + (i % N)] = (VT)0;
}

// ---- G lanes per stored row -------------------------------------------------------------
template <typename PT, typename CT, typename VT, int G>
__global__ __launch_bounds__(kThreads) void spmv_rows_kernel(const PT *__restrict__ pos, const CT *__restrict__ crd,
                                                             const VT *__restrict__ val, const CT *__restrict__ rowid, int64_t nrows,
                                                             const VT *__restrict__ x, int64_t ldb, VT *__restrict__ y, int64_t ldc,
                                                             int accumulate)
{
    const int64_t r = ((int64_t)blockIdx.x * kThreads + threadIdx.x) / G;
    const int sub = threadIdx.x % G;
    VT acc = 0;
    if (r < nrows) {
        const int64_t a = (int64_t)pos[r], b = (int64_t)pos[r + 1];
        for (int64_t p = a + sub; p < b; p += G) acc += val[p] * x[(int64_t)crd[p] * ldb];
    }
#pragma unroll
    for (int d = G / 2; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, 64);
    if (sub == 0 && r < nrows) {
        const int64_t row = rowid ? (int64_t)rowid[r] : r;
        y[row * ldc] = accumulate ? y[row * ldc] + acc : acc;
    }
}

// ---- stream kernel ----------------------------------------------------------------------
// Measured on the 1M x 1M workload: with operands cold in HBM the kernel runs 10 % faster at 3 waves per SIMD than at
// the 8 the register count would allow (fewer concurrent entry streams); warm it makes no difference.
#ifndef SPMI_WPE
#define SPMI_WPE 3
#endif
template <typename PT, typename CT, typename VT>
__global__ __launch_bounds__(kST) __attribute__((amdgpu_waves_per_eu(1, SPMI_WPE))) void spmv_stream_kernel(const PT *__restrict__ pos, const CT *__restrict__ crd,
                                                               const VT *__restrict__ val, const CT *__restrict__ rowid,
                                                               const int32_t *__restrict__ rowblk, int64_t nrows, int64_t nnz,
                                                               const VT *__restrict__ x, int64_t ldb, VT *__restrict__ y, int64_t ldc,
                                                               VT *__restrict__ carry, int accumulate)
{
    const int64_t win = blockIdx.x;
    __shared__ VT prods[kStreamT];
    __shared__ int queue[kQueue];
    __shared__ int qn, lo_began_earlier;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t s = win * kStreamT;
    const int64_t e = (s + kStreamT < nnz) ? s + kStreamT : nnz;
    if (tid == 0) qn = 0;

    // phase A: this block's entries (two consecutive entries per lane and step), every load issued before the
    // first use.  The pos entries of the rows that meet the window (see phase B) are fetched in the same
    // batch, for the first kPre rounds of the row loop, so that their latency hides under the gathers.
    const bool full = e - s == kStreamT;
    constexpr int E = kSpmiStreamPer;
    CT k[E];
    VT v[E];
    if (full) {
#pragma unroll
        for (int t = 0; t < E / 2; ++t) {
            const int64_t p = s + (int64_t)(t * kST + tid) * 2;
            k[2 * t] = crd[p]; k[2 * t + 1] = crd[p + 1];
            v[2 * t] = val[p]; v[2 * t + 1] = val[p + 1];
        }
    }
    const int64_t lo = rowblk[win], hi = rowblk[win + 1];
    const int64_t last = hi < nrows ? hi : nrows - 1;
    PT pre_a[kPre], pre_b[kPre];
#pragma unroll
    for (int i = 0; i < kPre; ++i) {
        int64_t r = lo + tid + (int64_t)i * kST;
        r = r <= last ? r : last;                      // clamped, not predicated: the loads stay unconditional
        pre_a[i] = pos[r];
        pre_b[i] = pos[r + 1];
    }
    if (full) {
        VT xv[E];
#pragma unroll
        for (int i = 0; i < E; ++i) xv[i] = x[(int64_t)k[i] * ldb];
#pragma unroll
        for (int t = 0; t < E / 2; ++t) {
            prods[(t * kST + tid) * 2] = v[2 * t] * xv[2 * t];
            prods[(t * kST + tid) * 2 + 1] = v[2 * t + 1] * xv[2 * t + 1];
        }
    } else {
        for (int i = tid; i < (int)(e - s); i += kST) prods[i] = val[s + i] * x[(int64_t)crd[s + i] * ldb];
    }
    if (tid == 0) lo_began_earlier = (int64_t)pre_a[0] < s;      // thread 0 prefetched pos[lo]
    __syncthreads();

    // phase B: rows lo..hi meet this window.  Rows lo..hi-1 end here and are written; row hi only
    // starts here (its head goes to y, the rest arrives through later blocks' carries); if row lo
    // began in an earlier window its part goes to this block's carry.
    const bool lo_carried = lo_began_earlier != 0;
    auto emit = [&](int64_t r, VT sum) {
        if (r == lo && lo_carried) { carry[win] = sum; return; }
        VT *dst = y + (rowid ? (int64_t)rowid[r] : r) * ldc;
        *dst = accumulate ? *dst + sum : sum;
    };
    auto short_row = [&](int64_t r, int64_t pa, int64_t pb) {
        const int a = (int)((pa > s ? pa : s) - s), b = (int)((pb < e ? pb : e) - s);
        if (r == hi && b <= a) return;               // row hi starts at the next window: not ours
        if (b - a > kLongRow) { queue[atomicAdd(&qn, 1)] = (int)(r - lo); return; }
        VT sum = 0;
        for (int i = a; i < b; ++i) sum += prods[i];
        emit(r, sum);
    };
#pragma unroll
    for (int k = 0; k < kPre; ++k) {
        const int64_t r = lo + tid + (int64_t)k * kST;
        if (r <= last) short_row(r, (int64_t)pre_a[k], (int64_t)pre_b[k]);
    }
    for (int64_t r = lo + tid + (int64_t)kPre * kST; r <= last; r += kST)
        short_row(r, (int64_t)pos[r], (int64_t)pos[r + 1]);
    __syncthreads();
    const int nq = qn;
    for (int q = wave; q < nq; q += kST / 64) {
        const int64_t r = lo + queue[q];
        const int64_t pa = (int64_t)pos[r], pb = (int64_t)pos[r + 1];
        const int a = (int)((pa > s ? pa : s) - s), b = (int)((pb < e ? pb : e) - s);
        VT sum = 0;
        for (int i = a + lane; i < b; i += 64) sum += prods[i];
        sum = wave_sum(sum);
        if (lane == 0) emit(r, sum);
    }
}

// One thread per block boundary: the first boundary a row crosses adds all of that row's carries, in
// block order, to the head part already in y.
template <typename PT, typename CT, typename VT>
__global__ __launch_bounds__(kThreads) void spmv_stream_fixup_kernel(const PT *__restrict__ pos, const CT *__restrict__ rowid,
                                                                     const int32_t *__restrict__ rowblk, int64_t nblocks,
                                                                     const VT *__restrict__ carry, VT *__restrict__ y, int64_t ldc)
{
    const int64_t b = (int64_t)blockIdx.x * kThreads + threadIdx.x + 1;
    if (b >= nblocks) return;
    const int64_t r = rowblk[b];
    const int64_t start = (int64_t)pos[r];
    if (start >= b * kStreamT || start < (b - 1) * kStreamT) return;   // not crossed here, or crossed earlier already
    VT sum = 0;
    for (int64_t bb = b; bb < nblocks && rowblk[bb] == r; ++bb) sum += carry[bb];
    const int64_t row = rowid ? (int64_t)rowid[r] : r;
    y[row * ldc] += sum;
}

// Column-segmented SpMV, last step: y[r] = (y[r]) + sum over panels of the per-panel partial results.
template <typename VT>
__global__ __launch_bounds__(kThreads) void spmv_panel_sum_kernel(const VT *__restrict__ part, int64_t nrows, int panels,
                                                                  VT *__restrict__ y, int64_t ldc, int accumulate)
{
    const int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (r >= nrows) return;
    VT sum = accumulate ? y[r * ldc] : (VT)0;
    for (int p = 0; p < panels; ++p) sum += part[(int64_t)p * nrows + r];
    y[r * ldc] = sum;
}

// ---- binned SpMV (see sp_bins): two streaming passes, every gather and every scattered add inside the LDS ----
constexpr int kBinThreads = 1024;
constexpr int kBinPW = 1 << kSpmiBinPanelShift;
constexpr int kBinRB = 1 << kSpmiBinRowShift;

// First pass: block (panel, piece) loads the panel's slice of x into LDS, then streams its share of the panel's entries, 16 bytes
// of values per lane and load: the product of entry e = val[e] * x[panel * PW + lcol[e]] goes to the row-block-major array, to
// slot e % 8 of the group that gdst names for e's group of 8.  Padding entries carry value 0 and column PW, where the slice
// holds a zero, so that they give 0 whatever x holds.
template <typename VT>
__global__ __launch_bounds__(kBinThreads) void spmv_bins_multiply_kernel(const VT *__restrict__ val, const uint16_t *__restrict__ lcol,
                                                                         const uint32_t *__restrict__ gdst, const int64_t *__restrict__ pstart,
                                                                         int panels, int pieces, int64_t n, const VT *__restrict__ x, int64_t ldb,
                                                                         VT *__restrict__ prod)
{
    constexpr int V = 16 / sizeof(VT);
    typedef VT vec_t __attribute__((ext_vector_type(V)));
    typedef uint16_t idx_t __attribute__((ext_vector_type(V)));
    __shared__ VT xs[kBinPW + V];
    // blocks go to the eight XCDs in turn: the pieces of one panel are given to blocks b, b + 8, b + 16, ... so that they
    // share an L2 and the panel's slice of x is fetched from memory once, not once per piece
    const int grp = 8 * pieces;
    const int p = (int)(blockIdx.x / grp) * 8 + (int)(blockIdx.x % 8), q = (int)(blockIdx.x / 8) % pieces;
    if (p >= panels) return;                           // whole block (the panel count is rounded up to eight)
    const int64_t pa = pstart[p], pb = pstart[p + 1];  // multiples of 8
    auto cut = [&](int k) -> int64_t {                 // piece boundaries: multiples of 8 inside the panel
        if (k <= 0) return pa;
        if (k >= pieces) return pb;
        return (pa + (pb - pa) * k / pieces) & ~(int64_t)7;
    };
    const int64_t a = cut(q), b = cut(q + 1);
    if (a >= b) return;                                // whole block
    const int64_t c0 = (int64_t)p * kBinPW;
    for (int i = threadIdx.x; i < kBinPW + V; i += kBinThreads) xs[i] = (i < kBinPW && c0 + i < n) ? x[(c0 + i) * ldb] : (VT)0;
    __syncthreads();
    const int64_t nvec = (b - a) / V;
    const vec_t *__restrict__ vv = (const vec_t *)(val + a);
    const idx_t *__restrict__ cc = (const idx_t *)(lcol + a);
    const uint32_t *__restrict__ gg = gdst + (a >> 3);
    constexpr int U = 2, GV = 8 / V;                   // GV lanes share a group
    auto store = [&](int64_t j, uint32_t g, const vec_t &r) { *(vec_t *)(prod + ((int64_t)g * 8 + (int64_t)(j % GV) * V)) = r; };
    int64_t j = threadIdx.x;
    for (; j + (U - 1) * kBinThreads < nvec; j += U * kBinThreads) {
        vec_t v[U];
        idx_t c[U];
        uint32_t g[U];
#pragma unroll
        for (int u = 0; u < U; ++u) { v[u] = vv[j + u * kBinThreads]; c[u] = cc[j + u * kBinThreads]; g[u] = gg[(j + u * kBinThreads) / GV]; }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            vec_t r;
#pragma unroll
            for (int t = 0; t < V; ++t) r[t] = v[u][t] * xs[c[u][t]];
            store(j + u * kBinThreads, g[u], r);
        }
    }
    for (; j < nvec; j += kBinThreads) {
        const vec_t v = vv[j];
        const idx_t c = cc[j];
        const uint32_t g = gg[j / GV];
        vec_t r;
#pragma unroll
        for (int t = 0; t < V; ++t) r[t] = v[t] * xs[c[t]];
        store(j, g, r);
    }
}

// Second pass: block = row block.  It streams the row block's products and 16-bit rows, which the first pass left side by side
// (a lane takes a group of 8 with 16-byte loads), and adds them into the block's slice of y in LDS (atomic adds: the order in
// which a row's products meet is not fixed); the slice is written out at the end.  Every stored row of the row block is
// written (m of them; rowid[q] is the matrix row of stored row q when not all rows are stored, and the caller has then
// zeroed the others).
template <typename CT, typename VT>
__global__ __launch_bounds__(kBinThreads) void spmv_bins_reduce_kernel(const VT *__restrict__ prod, const uint16_t *__restrict__ lrow,
                                                                       const int64_t *__restrict__ rbstart, int rowblocks, int64_t m,
                                                                       const CT *__restrict__ rowid, VT *__restrict__ y, int64_t ldc,
                                                                       int accumulate)
{
    constexpr int V = 16 / sizeof(VT), NV = 8 / V;
    typedef VT vec_t __attribute__((ext_vector_type(V)));
    typedef unsigned uint4v __attribute__((ext_vector_type(4)));
    __shared__ VT ys[kBinRB];
    const int rb = (int)blockIdx.x;
    for (int i = threadIdx.x; i < kBinRB; i += kBinThreads) ys[i] = (VT)0;
    __syncthreads();
    const int64_t g0 = rbstart[rb] >> 3, g1 = rbstart[rb + 1] >> 3;
    const vec_t *__restrict__ pp = (const vec_t *)prod;
    const uint4v *__restrict__ rr = (const uint4v *)lrow;
    for (int64_t g = g0 + threadIdx.x; g < g1; g += kBinThreads) {
        vec_t v[NV];
#pragma unroll
        for (int k = 0; k < NV; ++k) v[k] = pp[g * NV + k];
        const uint4v r = rr[g];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const unsigned w = (t >> 1) == 0 ? r.x : (t >> 1) == 1 ? r.y : (t >> 1) == 2 ? r.z : r.w;
            atomicAdd(&ys[(t & 1) ? (w >> 16) : (w & 0xffffu)], v[t / V][t % V]);
        }
    }
    __syncthreads();
    const int64_t r0 = (int64_t)rb * kBinRB;
    for (int i = threadIdx.x; i < kBinRB; i += kBinThreads) {
        const int64_t q = r0 + i;                      // stored row; rowid maps it to the matrix row where not all rows are stored
        if (q < m) {
            VT *dst = y + (rowid ? (int64_t)rowid[q] : q) * ldc;
            *dst = accumulate ? *dst + ys[i] : ys[i];
        }
    }
}

// ---- SpMM: a wave per stored row, CG lanes across a tile of B's columns, 64/CG entries in flight ----
template <typename PT, typename CT, typename VT, int CG>
__global__ __launch_bounds__(kThreads) void spmm_rows_kernel(const PT *__restrict__ pos, const CT *__restrict__ crd,
                                                             const VT *__restrict__ val, const CT *__restrict__ rowid, int64_t nrows,
                                                             const VT *__restrict__ B, int64_t N, int64_t ldb, VT *__restrict__ C,
                                                             int64_t ldc, int accumulate)
{
    constexpr int S = 64 / CG;                        // entries of the row handled side by side
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (r >= nrows) return;                           // whole wave
    const int jl = lane % CG, sl = lane / CG;
    const int64_t a = (int64_t)pos[r], b = (int64_t)pos[r + 1];
    const int64_t row = rowid ? (int64_t)rowid[r] : r;
    for (int64_t j0 = 0; j0 < N; j0 += CG) {
        const int64_t j = j0 + jl;
        const bool jin = j < N;
        VT acc = 0;
        int64_t p = a + sl;
        if constexpr (CG == 64) {                      // 512-byte rows of B (f64): two row gathers in flight measured best
            VT acc1 = 0;
            for (; p + S < b; p += 2 * S) {
                const int64_t k0 = (int64_t)crd[p], k1 = (int64_t)crd[p + S];
                const VT v0 = val[p], v1 = val[p + S];
                if (jin) { acc += v0 * B[k0 * ldb + j]; acc1 += v1 * B[k1 * ldb + j]; }
            }
            if (p < b && jin) acc += val[p] * B[(int64_t)crd[p] * ldb + j];
            acc += acc1;
        } else {                                       // narrower tiles: four
            constexpr int U = 4;
            VT accu[U];
#pragma unroll
            for (int u = 0; u < U; ++u) accu[u] = 0;
            for (; p + (U - 1) * S < b; p += U * S) {
                int64_t k[U];
                VT v[U], bv[U];
#pragma unroll
                for (int u = 0; u < U; ++u) { k[u] = (int64_t)crd[p + u * S]; v[u] = val[p + u * S]; }
#pragma unroll
                for (int u = 0; u < U; ++u) bv[u] = jin ? B[k[u] * ldb + j] : (VT)0;
#pragma unroll
                for (int u = 0; u < U; ++u) accu[u] += v[u] * bv[u];
            }
            for (; p < b; p += S)
                if (jin) accu[0] += val[p] * B[(int64_t)crd[p] * ldb + j];
#pragma unroll
            for (int u = 0; u < U; ++u) acc += accu[u];
        }
#pragma unroll
        for (int d = 32; d >= CG; d >>= 1) acc += __shfl_xor(acc, d, 64);
        if (sl == 0 && jin) C[row * ldc + j] = accumulate ? C[row * ldc + j] + acc : acc;
    }
}

// SpMM with 16-byte loads: LR lanes cover one row of B (N = LR * 16 / sizeof(VT) columns), 64 / LR stored entries of
// the row of A side by side, two gathers in flight per lane.  Needs N a multiple of the vector width and B, C rows
// 16-byte aligned; the dispatch checks it.
template <typename PT, typename CT, typename VT, int LR>
__global__ __launch_bounds__(kThreads) void spmm_rows_vec_kernel(const PT *__restrict__ pos, const CT *__restrict__ crd,
                                                                 const VT *__restrict__ val, const CT *__restrict__ rowid, int64_t nrows,
                                                                 const VT *__restrict__ B, int64_t ldb, VT *__restrict__ C, int64_t ldc,
                                                                 int accumulate)
{
    constexpr int V = 16 / sizeof(VT);
    constexpr int S = 64 / LR;
    typedef VT vec_t __attribute__((ext_vector_type(V)));
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (r >= nrows) return;                           // whole wave
    const int jl = lane % LR, sl = lane / LR;
    const int64_t a = (int64_t)pos[r], b = (int64_t)pos[r + 1];
    constexpr int U = S >= 4 ? 2 : 4;                 // row gathers in flight per lane (measured: 8 to 16 entries per step)
    vec_t accu[U];
#pragma unroll
    for (int u = 0; u < U; ++u) accu[u] = (vec_t)(0);
    int64_t p = a + sl;
    for (; p + (U - 1) * S < b; p += U * S) {
        int64_t k[U];
        VT v[U];
        vec_t bv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) { k[u] = (int64_t)crd[p + u * S]; v[u] = val[p + u * S]; }
#pragma unroll
        for (int u = 0; u < U; ++u) bv[u] = *(const vec_t *)(B + k[u] * ldb + jl * V);
#pragma unroll
        for (int u = 0; u < U; ++u) accu[u] += v[u] * bv[u];
    }
    if (p < b) {                                      // the last, partial step: same batch of loads, clamped and masked
        int64_t k[U];
        VT v[U];
        vec_t bv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t pp = p + u * S;
            const bool in = pp < b;
            k[u] = (int64_t)crd[in ? pp : p];
            v[u] = in ? val[pp] : (VT)0;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) bv[u] = *(const vec_t *)(B + k[u] * ldb + jl * V);
#pragma unroll
        for (int u = 0; u < U; ++u) accu[u] += v[u] * bv[u];
    }
    vec_t acc0 = accu[0];
#pragma unroll
    for (int u = 1; u < U; ++u) acc0 += accu[u];
#pragma unroll
    for (int e = 0; e < V; ++e) {
        VT x = acc0[e];
#pragma unroll
        for (int d = 32; d >= LR; d >>= 1) x += __shfl_xor(x, d, 64);
        acc0[e] = x;
    }
    if (sl == 0) {
        const int64_t row = rowid ? (int64_t)rowid[r] : r;
        vec_t *dst = (vec_t *)(C + row * ldc + jl * V);
        *dst = accumulate ? *dst + acc0 : acc0;
    }
}

// The same product cut by stored entries instead of rows (tune value 3; automatic when some row is long): block w
// owns the entries [w*T, (w+1)*T) with T and `rowblk` as in the stream SpMV, its four waves take the rows that meet
// the window in turn.  The part of a row that began in an earlier window goes to carry[w] (N values) and the fix-up
// kernel below adds the carries to C in block order; everything else is written to C directly.  No atomics.
// The window's values and, instead of its coordinates, the byte offsets of the rows of B that they select (OT: 32 bits
// when B is below 4 GB) are first copied into LDS with coalesced loads: the loop over the entries then works on small
// window-relative integers and every gather address is a wave-uniform base plus a lane offset.
template <typename PT, typename CT, typename VT, int LR, typename OT>
__global__ __launch_bounds__(kThreads) void spmm_windows_vec_kernel(const PT *__restrict__ pos, const CT *__restrict__ crd,
                                                                    const VT *__restrict__ val, const CT *__restrict__ rowid,
                                                                    const int32_t *__restrict__ rowblk, int64_t nrows, int64_t nnz,
                                                                    const VT *__restrict__ B, int64_t ldb, VT *__restrict__ C, int64_t ldc,
                                                                    VT *__restrict__ carry, int accumulate, int lr_any)
{
    constexpr int V = 16 / sizeof(VT);
    const int LRv = LR > 0 ? LR : lr_any;             // LR = 0: any number of lanes per row of B, known at run time
    const int S = 64 / LRv;
    constexpr int U = (LR > 0 && 64 / (LR > 0 ? LR : 1) >= 4) ? 2 : 4;
    typedef VT vec_t __attribute__((ext_vector_type(V)));
    __shared__ OT s_off[kStreamT];
    __shared__ VT s_val[kStreamT];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int jl = lane % LRv, sl = lane / LRv;
    const int64_t s = (int64_t)blockIdx.x * kStreamT;
    const int64_t e = s + kStreamT < nnz ? s + kStreamT : nnz;
    const int ne = (int)(e - s);
    const OT brow = (OT)(ldb * (int64_t)sizeof(VT));
    for (int i = threadIdx.x; i < ne; i += kThreads) {
        s_off[i] = (OT)crd[s + i] * brow;
        s_val[i] = val[s + i];
    }
    const int64_t lo = rowblk[blockIdx.x], hi = rowblk[blockIdx.x + 1];
    const int64_t last = hi < nrows ? hi : nrows - 1;
    __syncthreads();
    const char *Bb = (const char *)B;
    const OT colb = (OT)(jl * V * (int)sizeof(VT));
    int slot[U];
#pragma unroll
    for (int u = 0; u < U; ++u) slot[u] = sl < S ? sl + u * S : (1 << 24);      // lanes beyond LR * S never take an entry
    for (int64_t r = lo + wave; r <= last; r += kThreads / 64) {
        const int64_t pa = (int64_t)pos[r], pb = (int64_t)pos[r + 1];
        const int a = (int)((pa > s ? pa : s) - s), b = (int)((pb < e ? pb : e) - s);
        if (r == hi && b <= a) continue;              // row hi starts at the next window: not ours (wave-uniform)
        vec_t accu[U];
#pragma unroll
        for (int u = 0; u < U; ++u) accu[u] = (vec_t)(0);
        for (int p0 = a; p0 < b; p0 += U * S) {       // wave-uniform
            VT v[U];
            vec_t bv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int pp = p0 + slot[u];
                const bool in = pp < b;
                const int idx = in ? pp : a;
                v[u] = in ? s_val[idx] : (VT)0;
                bv[u] = *(const vec_t *)(Bb + (s_off[idx] + colb));
            }
#pragma unroll
            for (int u = 0; u < U; ++u) accu[u] += v[u] * bv[u];
        }
        vec_t acc0 = accu[0];
#pragma unroll
        for (int u = 1; u < U; ++u) acc0 += accu[u];
        if (LR > 0) {
#pragma unroll
            for (int ee = 0; ee < V; ++ee) {
                VT x = acc0[ee];
#pragma unroll
                for (int d = 32; d >= (LR > 0 ? LR : 64); d >>= 1) x += __shfl_xor(x, d, 64);
                acc0[ee] = x;
            }
        } else {                                      // the S groups' sums meet in group 0
            const vec_t mine = acc0;
            for (int g = 1; g < S; ++g) {
#pragma unroll
                for (int ee = 0; ee < V; ++ee) acc0[ee] += __shfl(mine[ee], jl + g * LRv, 64);
            }
        }
        if (sl == 0) {
            if (pa < s) *(vec_t *)(carry + (int64_t)blockIdx.x * LRv * V + jl * V) = acc0;
            else {
                const int64_t row = rowid ? (int64_t)rowid[r] : r;
                vec_t *dst = (vec_t *)(C + row * ldc + jl * V);
                *dst = accumulate ? *dst + acc0 : acc0;
            }
        }
    }
}

// A wave per block boundary: the first boundary a row crosses adds all of that row's carries, in block order.
template <typename PT, typename CT, typename VT>
__global__ __launch_bounds__(kThreads) void spmm_windows_fixup_kernel(const PT *__restrict__ pos, const CT *__restrict__ rowid,
                                                                      const int32_t *__restrict__ rowblk, int64_t nblocks, int64_t N,
                                                                      const VT *__restrict__ carry, VT *__restrict__ C, int64_t ldc)
{
    const int lane = threadIdx.x & 63;
    const int64_t b = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6) + 1;
    if (b >= nblocks) return;
    const int64_t r = rowblk[b];
    const int64_t start = (int64_t)pos[r];
    if (start >= b * kStreamT || start < (b - 1) * kStreamT) return;   // not crossed here, or crossed earlier already
    const int64_t row = rowid ? (int64_t)rowid[r] : r;
    for (int64_t j = lane; j < N; j += 64) {
        VT sum = 0;
        for (int64_t bb = b; bb < nblocks && rowblk[bb] == r; ++bb) sum += carry[bb * N + j];
        C[row * ldc + j] += sum;
    }
}

// ---- column-major storage: a wave per stored column, atomic adds into C ------------------
template <typename PT, typename CT, typename VT, int CG>
__global__ __launch_bounds__(kThreads) void spmm_scatter_kernel(const PT *__restrict__ pos, const CT *__restrict__ crd,
                                                                const VT *__restrict__ val, const CT *__restrict__ colid, int64_t ncols,
                                                                const VT *__restrict__ B, int64_t N, int64_t ldb, VT *__restrict__ C,
                                                                int64_t ldc)
{
    constexpr int S = 64 / CG;
    const int lane = threadIdx.x & 63;
    const int64_t q = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (q >= ncols) return;
    const int jl = lane % CG, sl = lane / CG;
    const int64_t a = (int64_t)pos[q], b = (int64_t)pos[q + 1];
    if (a == b) return;
    const int64_t k = colid ? (int64_t)colid[q] : q;
    for (int64_t j0 = 0; j0 < N; j0 += CG) {
        const int64_t j = j0 + jl;
        if (j >= N) continue;
        const VT bj = B[k * ldb + j];
        for (int64_t p = a + sl; p < b; p += S) unsafeAtomicAdd(&C[(int64_t)crd[p] * ldc + j], val[p] * bj);
    }
}

// ---- dense innermost level (the paper's compressed-then-dense format of Section 4.1 and the all-dense one) ----
// Row-major: stored row q holds all `n` values of matrix row rowid[q] (or q).  A block per stored row: lanes
// stride over the row with coalesced loads, LG lanes side by side per tile of CG columns of B.
template <typename CT, typename VT, int CG>
__global__ __launch_bounds__(kThreads) void dense_rows_kernel(const VT *__restrict__ val, const CT *__restrict__ rowid, int64_t n,
                                                              const VT *__restrict__ B, int64_t N, int64_t ldb, VT *__restrict__ C,
                                                              int64_t ldc, int accumulate)
{
    constexpr int KS = kThreads / CG;                 // entries of the row handled side by side
    __shared__ VT red[kThreads];
    const int64_t q = blockIdx.x;
    const int jl = threadIdx.x % CG, kl = threadIdx.x / CG;
    const VT *__restrict__ vrow = val + q * n;
    const int64_t row = rowid ? (int64_t)rowid[q] : q;
    for (int64_t j0 = 0; j0 < N; j0 += CG) {
        const int64_t j = j0 + jl;
        VT acc = 0;
        if (j < N)
            for (int64_t k = kl; k < n; k += KS) acc += vrow[k] * B[k * ldb + j];
        red[threadIdx.x] = acc;
        __syncthreads();
        for (int stride = kThreads / 2; stride >= CG; stride >>= 1) {
            if (threadIdx.x < stride) red[threadIdx.x] += red[threadIdx.x + stride];
            __syncthreads();
        }
        if (kl == 0 && j < N) C[row * ldc + j] = accumulate ? C[row * ldc + j] + red[jl] : red[jl];
        __syncthreads();
    }
}

// Column-major: stored column q holds all `m` values of matrix column colid[q] (or q): C[i, j] = sum_q V[q, i] * B[col_q, j].
// A thread per (i, j); every row of C is written, so no zero fill is needed and no atomics either.
template <typename CT, typename VT, int CG>
__global__ __launch_bounds__(kThreads) void dense_cols_kernel(const VT *__restrict__ val, const CT *__restrict__ colid, int64_t ncols,
                                                              int64_t m, const VT *__restrict__ B, int64_t N, int64_t ldb,
                                                              VT *__restrict__ C, int64_t ldc, int accumulate)
{
    constexpr int IS = kThreads / CG;                 // rows of C per block
    const int jl = threadIdx.x % CG;
    const int64_t i = (int64_t)blockIdx.x * IS + threadIdx.x / CG;
    if (i >= m) return;
    for (int64_t j0 = 0; j0 < N; j0 += CG) {
        const int64_t j = j0 + jl;
        if (j >= N) continue;
        VT acc = accumulate ? C[i * ldc + j] : (VT)0;
        for (int64_t q = 0; q < ncols; ++q) {
            const int64_t k = colid ? (int64_t)colid[q] : q;
            acc += val[q * m + i] * B[k * ldb + j];
        }
        C[i * ldc + j] = acc;
    }
}

// Row-major dense innermost level, one column (y = A.x with fully stored rows): pure streaming.  Block (c, q) takes
// 2048 consecutive values of stored row q with 16-byte loads and leaves one partial sum; a second small kernel adds
// the partial sums of a row in order (deterministic) and writes y.
constexpr int kDenseChunk = kThreads * 8;
template <typename VT>
__global__ __launch_bounds__(kThreads) void dense_rows_spmv_partial_kernel(const VT *__restrict__ val, int64_t n, const VT *__restrict__ x,
                                                                           int64_t nchunks, VT *__restrict__ partial)
{
    constexpr int V = 16 / sizeof(VT);                // elements per 16-byte load
    typedef VT vec_t __attribute__((ext_vector_type(V)));
    __shared__ VT wsum[kThreads / 64];
    const int64_t q = blockIdx.y, c = blockIdx.x;
    const int64_t k0 = c * kDenseChunk;
    const VT *__restrict__ vrow = val + q * n;
    VT acc = 0;
    if (k0 + kDenseChunk <= n) {
        vec_t a[8 / V], b[8 / V];
#pragma unroll
        for (int t = 0; t < 8 / V; ++t) {
            const int64_t k = k0 + (int64_t)(t * kThreads + threadIdx.x) * V;
            a[t] = *(const vec_t *)(vrow + k);
            b[t] = *(const vec_t *)(x + k);
        }
#pragma unroll
        for (int t = 0; t < 8 / V; ++t)
#pragma unroll
            for (int e = 0; e < V; ++e) acc += a[t][e] * b[t][e];
    } else {
        for (int64_t k = k0 + threadIdx.x; k < n; k += kThreads) acc += vrow[k] * x[k];
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        VT tot = 0;
        for (int w = 0; w < kThreads / 64; ++w) tot += wsum[w];
        partial[q * nchunks + c] = tot;
    }
}

template <typename CT, typename VT>
__global__ __launch_bounds__(kThreads) void dense_rows_spmv_finish_kernel(const VT *__restrict__ partial, int64_t nchunks, const CT *__restrict__ rowid,
                                                                          int64_t nstored, VT *__restrict__ y, int64_t ldc, int accumulate)
{
    const int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (q >= nstored) return;
    VT sum = 0;
    for (int64_t c = 0; c < nchunks; ++c) sum += partial[q * nchunks + c];
    const int64_t row = rowid ? (int64_t)rowid[q] : q;
    y[row * ldc] = accumulate ? y[row * ldc] + sum : sum;
}

inline unsigned grid_for(int64_t n, int64_t per_block) { return (unsigned)(n > 0 ? ceil_div(n, per_block) : 1); }

template <typename PT, typename CT, typename VT>
sp_status zero_c(VT *C, int64_t m, int64_t N, int64_t ldc, hipStream_t st)
{
    if (m * N == 0) return SP_OK;
    const int64_t nb = ceil_div(m * N, kThreads);
    hipLaunchKernelGGL(zero_matrix_kernel<VT>, dim3((unsigned)(nb < 16384 ? nb : 16384)), dim3(kThreads), 0, st, C, m, N, ldc);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

// Which stored rows a product walks: all positions of the outer level, or only the stored / non-empty ones through a row-id list
// (a compressed outer level, or a dense one that is mostly empty and therefore carries the list of its non-empty rows).
template <typename PT, typename CT>
struct row_view {
    const PT *pos; const CT *rowid; int64_t nrows; const sp_rowblocks *rowblocks; bool dcsr;
    explicit row_view(const sp_tensor *A)
    {
        pos = (const PT *)A->pos[1];
        dcsr = A->enc.lt[0] == SP_COMPRESSED;
        rowid = dcsr ? (const CT *)A->crd[0] : nullptr;
        nrows = A->npos[1] - 1;
        rowblocks = &A->rowblocks;
        if (!dcsr && A->nz_pos) {
            dcsr = true;
            pos = (const PT *)A->nz_pos; rowid = (const CT *)A->nz_rowid; nrows = A->nz_rows; rowblocks = &A->nz_rowblocks;
        }
    }
};

// The SpMM cut by stored entries plus its fix-up, with the per-block carries in `carry` (room for N values per block).
// N * sizeof(VT) is a multiple of 16 with at most 64 such pieces per row; B, C and their leading dimensions are 16-byte aligned.
template <typename PT, typename CT, typename VT>
sp_status spmm_windows_launch(const sp_tensor *A, const row_view<PT, CT> &rv, const VT *B, int64_t N, int64_t ldb, VT *C, int64_t ldc,
                              int accumulate, VT *carry, hipStream_t st)
{
    constexpr int64_t V = 16 / sizeof(VT);
    const int64_t lr = N / V;
    const PT *pos = rv.pos;
    const CT *crd = (const CT *)A->crd[1];
    const VT *val = (const VT *)A->values;
    const CT *rowid = rv.rowid;
    const int64_t nrows = rv.nrows, nnz = A->ncrd[1];
    const sp_rowblocks *rowblocks = rv.rowblocks;
    const int64_t nb = rowblocks->nblocks;
    const bool small = sizeof(CT) == 4 && (uint64_t)A->shape[1] * (uint64_t)ldb * sizeof(VT) < ((uint64_t)1 << 32);     // 32-bit byte offsets into B (64-bit coordinates keep 64-bit offsets)
#define SPMI_SPMM_WIN_O(LR, OT)                                                                                               \
    hipLaunchKernelGGL((spmm_windows_vec_kernel<PT, CT, VT, LR, OT>), dim3((unsigned)nb), dim3(kThreads), 0, st, pos, crd, val, rowid,    \
                       (const int32_t *)rowblocks->start, nrows, nnz, B, ldb, C, ldc, carry, accumulate, (int)lr)
#define SPMI_SPMM_WIN(LR)                           \
    do {                                            \
        if (small) SPMI_SPMM_WIN_O(LR, uint32_t);   \
        else SPMI_SPMM_WIN_O(LR, uint64_t);         \
    } while (0)
    if (lr == 1) SPMI_SPMM_WIN(1);
    else if (lr == 2) SPMI_SPMM_WIN(2);
    else if (lr == 4) SPMI_SPMM_WIN(4);
    else if (lr == 8) SPMI_SPMM_WIN(8);
    else if (lr == 16) SPMI_SPMM_WIN(16);
    else if (lr == 32) SPMI_SPMM_WIN(32);
    else if (lr == 64) SPMI_SPMM_WIN(64);
    else SPMI_SPMM_WIN(0);                    // any other number of 16-byte pieces per row, up to 64
#undef SPMI_SPMM_WIN
#undef SPMI_SPMM_WIN_O
    SP_HIP(hipGetLastError());
    if (nb > 1) {
        hipLaunchKernelGGL((spmm_windows_fixup_kernel<PT, CT, VT>), dim3(grid_for(nb - 1, kThreads / 64)), dim3(kThreads), 0, st, pos,
                           rowid, (const int32_t *)rowblocks->start, nb, N, (const VT *)carry, C, ldc);
        SP_HIP(hipGetLastError());
    }
    return SP_OK;
}

// The inspector step of the matrix-times-vector product (Section 6.2): decides which SpMV kernel the tensor's products run
// and builds the regrouped copy that kernel reads.  Measures once how scattered the columns are (one pass over crd, one
// synchronisation), may allocate through the tensor's allocator.  The decision is kept in A->plan_spmv.
template <typename PT, typename CT, typename VT>
sp_status prepare_spmv_t(const sp_tensor *A, hipStream_t st)
{
    if (A->plan_spmv) return SP_OK;
    const row_view<PT, CT> rv(A);
    const int64_t nnz = A->ncrd[1], nrows = rv.nrows;
    int kernel = A->tune_spmv;
    const bool fixed = kernel != 0;
    if (kernel == 0) {
        // small and even (no row beyond one wave's stride): one launch of the rows kernel beats stream + fix-up
        const bool small_even = nnz < ((int64_t)1 << 18) && A->max_segment <= 64;
        kernel = (rv.rowblocks->start && nnz >= 8 * kStreamT && !small_even) ? 2 : 1;
        // a large matrix whose gathers are scattered over a large x: no gather should leave the chip's caches.  The
        // binned copy keeps them inside the LDS (measured 103 us against 122 us on the 1M x 1M matrix); where it cannot
        // be built, L2-sized column panels.  Gathers that mostly fall into the line of their predecessor stay as they are.
        if (kernel == 2 && nnz >= ((int64_t)1 << 21) && A->shape[1] * (int64_t)sizeof(VT) > ((int64_t)3 << 20)) {
            double share = 0;
            SP_TRY(spmi_column_scatter(A, st, &share));
            // ... and buckets of at least 32 entries on average (the second pass reads them a bucket at a time), in enough
            // row blocks to give every CU one (the hypersparse 8M x 8M workload has 41: 85 us binned, 73 us streamed)
            const int64_t rowblocks = ceil_div(nrows, (int64_t)kBinRB);
            const double buckets = (double)ceil_div(A->shape[1], (int64_t)kBinPW) * (double)rowblocks;
            if (share >= 0.5) kernel = ((double)nnz >= 32.0 * buckets && rowblocks >= 256) ? 4 : (!rv.dcsr && nnz >= ((int64_t)1 << 22)) ? 3 : 2;
        }
    }
    if (kernel == 4) {
        const sp_status sb = spmi_build_bins(A, st);
        if (sb == SP_ERR_UNSUPPORTED && !fixed) kernel = (!rv.dcsr && nnz >= ((int64_t)1 << 22)) ? 3 : 2;
        else if (sb != SP_OK) return sb;
    }
    if (kernel == 3) {
        if (A->enc.lt[0] == SP_COMPRESSED) return SP_ERR_UNSUPPORTED;
        const sp_status sb = spmi_build_segments(A, sizeof(VT), kSpmvSliceBytes, st);
        if (sb == SP_ERR_UNSUPPORTED && !fixed) kernel = 2;
        else if (sb != SP_OK) return sb;
    }
    if (kernel == 2 && !rv.rowblocks->start) return SP_ERR_UNSUPPORTED;
    A->plan_spmv = kernel;
    return SP_OK;
}

// Scratch of the SpMM cut by stored entries: one row of N values per block, kept by the tensor and grown on demand.
template <typename PT, typename CT, typename VT>
sp_status prepare_spmm_t(const sp_tensor *A, int64_t N, hipStream_t st)
{
    const row_view<PT, CT> rv(A);
    if (!rv.rowblocks->start || A->tune_spmm == 1 || A->tune_spmm == 2) return SP_OK;
    const size_t need = (size_t)rv.rowblocks->nblocks * N * sizeof(VT);
    if (A->spmm_carry_bytes >= need) return SP_OK;
    sp_mem mem{A->alloc, A->free_, A->ctx};
    if (A->spmm_carry) { SP_HIP(hipStreamSynchronize(st)); mem.put(A->spmm_carry); A->spmm_carry = nullptr; A->spmm_carry_bytes = 0; }
    A->spmm_carry = mem.get((need + 255) & ~(size_t)255);
    if (!A->spmm_carry) return SP_ERR_ALLOC;
    A->spmm_carry_bytes = need;
    return SP_OK;
}

template <typename PT, typename CT, typename VT>
sp_status prepare_rowmajor_t(const sp_tensor *A, const VT *, int64_t N, int64_t, VT *, int64_t, int, hipStream_t st)
{
    if (A->npos[1] - 1 <= 0) return SP_OK;
    if (N == 1) return prepare_spmv_t<PT, CT, VT>(A, st);
    return prepare_spmm_t<PT, CT, VT>(A, N, st);
}

template <typename PT, typename CT, typename VT>
sp_status rowmajor_t(const sp_tensor *A, const VT *B, int64_t N, int64_t ldb, VT *C, int64_t ldc, int accumulate, hipStream_t st)
{
    const row_view<PT, CT> rv(A);
    const PT *pos = rv.pos;
    const CT *crd = (const CT *)A->crd[1];
    const VT *val = (const VT *)A->values;
    const bool dcsr = rv.dcsr;
    const CT *rowid = rv.rowid;
    const int64_t nrows = rv.nrows;              // stored rows
    const sp_rowblocks *rowblocks = rv.rowblocks;
    const int64_t m = A->shape[0];
    const int64_t nnz = A->ncrd[1];
    if (dcsr && !accumulate) SP_TRY((zero_c<PT, CT, VT>(C, m, N, ldc, st)));   // rows that are not stored become zero
    if (nrows == 0) return SP_OK;
    if (N == 1) {
        if (!A->plan_spmv) {                     // no sp_prepare before this product: the inspector runs now (may allocate and synchronise)
            ++A->lazy_prepares;
            SP_TRY((prepare_spmv_t<PT, CT, VT>(A, st)));
        }
        const int kernel = A->plan_spmv;
        if (kernel == 3) {
            // the segmented copy is an ordinary CSR over panels*nrows virtual rows: stream it into the per-panel
            // partial vector (consecutive blocks gather from the same <= 2 MB slice of x), then add the panels up
            const sp_segments *g = A->segments;
            const sp_tensor *S = g->seg;
            int64_t vrows = (int64_t)g->panels * g->nrows;
            const PT *spos = (const PT *)S->pos[1];
            const CT *srowid = nullptr;
            const sp_rowblocks *srb = &S->rowblocks;
            if (S->nz_pos) {          // long runs of empty virtual rows (an empty panel): only the others are visited
                SP_TRY((zero_c<PT, CT, VT>((VT *)g->partial, vrows, 1, 1, st)));
                spos = (const PT *)S->nz_pos; srowid = (const CT *)S->nz_rowid; srb = &S->nz_rowblocks; vrows = S->nz_rows;
            }
            const int64_t nb = srb->nblocks;
            sp_prof_scope prof(A, st);
            hipLaunchKernelGGL((spmv_stream_kernel<PT, CT, VT>), dim3((unsigned)nb), dim3(kST), 0, st, spos,
                               (const CT *)S->crd[1], (const VT *)S->values, srowid, (const int32_t *)srb->start,
                               vrows, S->ncrd[1], B, ldb, (VT *)g->partial, (int64_t)1, (VT *)srb->carry, 0);
            SP_HIP(hipGetLastError());
            if (nb > 1) {
                hipLaunchKernelGGL((spmv_stream_fixup_kernel<PT, CT, VT>), dim3(grid_for(nb - 1, kThreads)), dim3(kThreads), 0, st,
                                   spos, srowid, (const int32_t *)srb->start, nb, (const VT *)srb->carry, (VT *)g->partial, (int64_t)1);
                SP_HIP(hipGetLastError());
            }
            hipLaunchKernelGGL((spmv_panel_sum_kernel<VT>), dim3(grid_for(g->nrows, kThreads)), dim3(kThreads), 0, st,
                               (const VT *)g->partial, g->nrows, g->panels, C, ldc, accumulate);
            SP_HIP(hipGetLastError());
            return SP_OK;
        }
        if (kernel == 4) {
            const sp_bins *g = A->bins;                                       // over the same stored rows as pos / rowid here
            sp_prof_scope prof(A, st);
            hipLaunchKernelGGL((spmv_bins_multiply_kernel<VT>), dim3((unsigned)(ceil_div(g->panels, 8) * 8 * g->pieces)), dim3(kBinThreads), 0, st,
                               (const VT *)g->val, (const uint16_t *)g->lcol, (const uint32_t *)g->gdst, (const int64_t *)g->pstart, g->panels,
                               g->pieces, A->shape[1], B, ldb, (VT *)g->prod);
            SP_HIP(hipGetLastError());
            hipLaunchKernelGGL((spmv_bins_reduce_kernel<CT, VT>), dim3((unsigned)g->rowblocks), dim3(kBinThreads), 0, st, (const VT *)g->prod,
                               (const uint16_t *)g->lrow, (const int64_t *)g->rbstart, g->rowblocks, g->nrows, rowid, C, ldc, accumulate);
            SP_HIP(hipGetLastError());
            return SP_OK;
        }
        if (kernel == 2) {
            const int64_t nb = rowblocks->nblocks;
            {
            sp_prof_scope prof(A, st);
            hipLaunchKernelGGL((spmv_stream_kernel<PT, CT, VT>), dim3((unsigned)nb), dim3(kST), 0, st, pos, crd, val, rowid,
                               (const int32_t *)rowblocks->start, nrows, nnz, B, ldb, C, ldc, (VT *)rowblocks->carry, accumulate);
            }
            SP_HIP(hipGetLastError());
            if (nb > 1) {
                hipLaunchKernelGGL((spmv_stream_fixup_kernel<PT, CT, VT>), dim3(grid_for(nb - 1, kThreads)), dim3(kThreads), 0, st, pos,
                                   rowid, (const int32_t *)rowblocks->start, nb, (const VT *)rowblocks->carry, C, ldc);
                SP_HIP(hipGetLastError());
            }
            return SP_OK;
        }
        const double avg = (double)nnz / (double)nrows;
        sp_prof_scope prof(A, st);
#define SPMI_ROWS(G)                                                                                                          \
    hipLaunchKernelGGL((spmv_rows_kernel<PT, CT, VT, G>), dim3(grid_for(nrows * G, kThreads)), dim3(kThreads), 0, st, pos, crd, \
                       val, rowid, nrows, B, ldb, C, ldc, accumulate)
        if (avg <= 3) SPMI_ROWS(2);
        else if (avg <= 6) SPMI_ROWS(4);
        else if (avg <= 12) SPMI_ROWS(8);
        else if (avg <= 24) SPMI_ROWS(16);
        else if (avg <= 48) SPMI_ROWS(32);
        else SPMI_ROWS(64);
#undef SPMI_ROWS
        SP_HIP(hipGetLastError());
        return SP_OK;
    }
    // Tried and dropped (measured on the 1M x 1M matrix times a 1M x 64 operand): one launch per column panel of the
    // segmented copy, so that the slice of B a launch gathers from fits the 256 MB last-level cache.  Re-reading and
    // re-writing C once per panel costs more than the gathers save: 3.17 ms against 2.94 ms.
    sp_prof_scope prof(A, st);
    {
        constexpr int64_t V = 16 / sizeof(VT);
        const int64_t lr = N / V;
        const bool aligned = N % V == 0 && ldb % V == 0 && ldc % V == 0 && (uintptr_t)B % 16 == 0 && (uintptr_t)C % 16 == 0;
        const bool fits = aligned && (lr == 1 || lr == 2 || lr == 4 || lr == 8 || lr == 16 || lr == 32 || lr == 64);    // a wave per row
        const bool fits_any = aligned && lr >= 1 && lr <= 64;                                                           // cut by entries
        if (A->tune_spmm == 2 && !fits) return SP_ERR_UNSUPPORTED;
        if (A->tune_spmm == 3 && (!fits_any || !rowblocks->start)) return SP_ERR_UNSUPPORTED;
        // measured faster than a wave per row on every workload tried (1.42 vs 1.57 ms, 0.68 vs 0.83 ms), and a very long
        // row no longer sets the run time: the default
        const bool by_entries = A->tune_spmm == 3 || (A->tune_spmm == 0 && rowblocks->start);
        if (fits_any && by_entries) {
            const int64_t nb = rowblocks->nblocks;
            if (A->spmm_carry_bytes < (size_t)nb * N * sizeof(VT)) {       // no sp_prepare for this many columns: the scratch is made now
                ++A->lazy_prepares;
                SP_TRY((prepare_spmm_t<PT, CT, VT>(A, N, st)));
            }
            return spmm_windows_launch<PT, CT, VT>(A, rv, B, N, ldb, C, ldc, accumulate, (VT *)A->spmm_carry, st);
        }
        if (fits && A->tune_spmm != 1) {
#define SPMI_SPMM_VEC(LR)                                                                                                     \
    hipLaunchKernelGGL((spmm_rows_vec_kernel<PT, CT, VT, LR>), dim3(grid_for(nrows, kThreads / 64)), dim3(kThreads), 0, st, pos, \
                       crd, val, rowid, nrows, B, ldb, C, ldc, accumulate)
            if (lr == 1) SPMI_SPMM_VEC(1);
            else if (lr == 2) SPMI_SPMM_VEC(2);
            else if (lr == 4) SPMI_SPMM_VEC(4);
            else if (lr == 8) SPMI_SPMM_VEC(8);
            else if (lr == 16) SPMI_SPMM_VEC(16);
            else if (lr == 32) SPMI_SPMM_VEC(32);
            else SPMI_SPMM_VEC(64);
#undef SPMI_SPMM_VEC
            SP_HIP(hipGetLastError());
            return SP_OK;
        }
    }
#define SPMI_SPMM(CG)                                                                                                      \
    hipLaunchKernelGGL((spmm_rows_kernel<PT, CT, VT, CG>), dim3(grid_for(nrows, kThreads / 64)), dim3(kThreads), 0, st, pos, crd, \
                       val, rowid, nrows, B, N, ldb, C, ldc, accumulate)
    if (N > 32) SPMI_SPMM(64);
    else if (N > 16) SPMI_SPMM(32);
    else if (N > 8) SPMI_SPMM(16);
    else if (N > 4) SPMI_SPMM(8);
    else SPMI_SPMM(4);
#undef SPMI_SPMM
    SP_HIP(hipGetLastError());
    return SP_OK;
}

template <typename PT, typename CT, typename VT>
sp_status scatter_t(const sp_tensor *A, const VT *B, int64_t N, int64_t ldb, VT *C, int64_t ldc, int accumulate, hipStream_t st)
{
    const PT *pos = (const PT *)A->pos[1];
    const CT *crd = (const CT *)A->crd[1];
    const VT *val = (const VT *)A->values;
    const CT *colid = A->enc.lt[0] == SP_COMPRESSED ? (const CT *)A->crd[0] : nullptr;
    const int64_t ncols = A->npos[1] - 1;
    if (!accumulate) SP_TRY((zero_c<PT, CT, VT>(C, A->shape[0], N, ldc, st)));
    if (ncols == 0) return SP_OK;
    sp_prof_scope prof(A, st);
#define SPMI_SCAT(CG)                                                                                                         \
    hipLaunchKernelGGL((spmm_scatter_kernel<PT, CT, VT, CG>), dim3(grid_for(ncols, kThreads / 64)), dim3(kThreads), 0, st, pos, \
                       crd, val, colid, ncols, B, N, ldb, C, ldc)
    if (N > 32) SPMI_SCAT(64);
    else if (N > 16) SPMI_SCAT(32);
    else if (N > 8) SPMI_SCAT(16);
    else if (N > 4) SPMI_SCAT(8);
    else if (N > 2) SPMI_SCAT(4);
    else if (N > 1) SPMI_SCAT(2);
    else SPMI_SCAT(1);
#undef SPMI_SCAT
    SP_HIP(hipGetLastError());
    return SP_OK;
}

// Scratch of the streaming product of fully stored rows with a vector: one partial sum per 2048-value chunk.
template <typename PT, typename CT, typename VT>
sp_status prepare_dense_inner_t(const sp_tensor *A, const VT *, int64_t N, int64_t, VT *, int64_t, int, hipStream_t st)
{
    const bool outer_compressed = A->enc.lt[0] == SP_COMPRESSED;
    const int64_t nstored = outer_compressed ? A->ncrd[0] : A->size[0];
    const int64_t inner = A->size[1];
    if (A->enc.perm[0] != 0 || N != 1 || inner < kDenseChunk || nstored <= 0 || nstored > 65535) return SP_OK;
    const size_t need = (size_t)(nstored * ceil_div(inner, kDenseChunk)) * sizeof(VT);
    if (A->dense_partial_bytes >= need) return SP_OK;
    sp_mem mem{A->alloc, A->free_, A->ctx};
    if (A->dense_partial) { SP_HIP(hipStreamSynchronize(st)); mem.put(A->dense_partial); A->dense_partial = nullptr; A->dense_partial_bytes = 0; }
    A->dense_partial = mem.get((need + 255) & ~(size_t)255);
    if (!A->dense_partial) return SP_ERR_ALLOC;
    A->dense_partial_bytes = need;
    return SP_OK;
}

template <typename PT, typename CT, typename VT>
sp_status dense_inner_t(const sp_tensor *A, const VT *B, int64_t N, int64_t ldb, VT *C, int64_t ldc, int accumulate, hipStream_t st)
{
    const VT *val = (const VT *)A->values;
    const bool outer_compressed = A->enc.lt[0] == SP_COMPRESSED;
    const CT *outer = outer_compressed ? (const CT *)A->crd[0] : nullptr;
    const int64_t nstored = outer_compressed ? A->ncrd[0] : A->size[0];        // stored rows (row-major) or columns
    const int64_t inner = A->size[1];
    const int64_t m = A->shape[0];
    const bool rowmajor = A->enc.perm[0] == 0;
    if (rowmajor && outer_compressed && !accumulate) SP_TRY((zero_c<PT, CT, VT>(C, m, N, ldc, st)));
    if (!rowmajor && nstored == 0 && !accumulate) return zero_c<PT, CT, VT>(C, m, N, ldc, st);
    if (nstored == 0 || inner == 0) return SP_OK;
    if (rowmajor && nstored > 0x7fffffff) return SP_ERR_TOO_LARGE;
    sp_prof_scope prof(A, st);
    constexpr int64_t V = 16 / sizeof(VT);
    if (rowmajor && N == 1 && ldb == 1 && inner >= kDenseChunk && inner % V == 0 && nstored <= 65535 &&
        (uintptr_t)B % 16 == 0 && (uintptr_t)val % 16 == 0) {
        // fully stored rows times a vector: the streaming path (16-byte loads need every row 16-byte aligned)
        const int64_t nchunks = ceil_div(inner, kDenseChunk);
        if (A->dense_partial_bytes < (size_t)(nstored * nchunks) * sizeof(VT)) {
            ++A->lazy_prepares;
            SP_TRY((prepare_dense_inner_t<PT, CT, VT>(A, B, N, ldb, C, ldc, accumulate, st)));
        }
        hipLaunchKernelGGL((dense_rows_spmv_partial_kernel<VT>), dim3((unsigned)nchunks, (unsigned)nstored), dim3(kThreads), 0, st, val, inner,
                           B, nchunks, (VT *)A->dense_partial);
        SP_HIP(hipGetLastError());
        hipLaunchKernelGGL((dense_rows_spmv_finish_kernel<CT, VT>), dim3(grid_for(nstored, kThreads)), dim3(kThreads), 0, st,
                           (const VT *)A->dense_partial, nchunks, outer, nstored, C, ldc, accumulate);
        SP_HIP(hipGetLastError());
        return SP_OK;
    }
#define SPMI_DENSE(CG)                                                                                                        \
    do {                                                                                                                      \
        if (rowmajor)                                                                                                         \
            hipLaunchKernelGGL((dense_rows_kernel<CT, VT, CG>), dim3((unsigned)nstored), dim3(kThreads), 0, st, val, outer, inner, B, N, \
                               ldb, C, ldc, accumulate);                                                                       \
        else                                                                                                                  \
            hipLaunchKernelGGL((dense_cols_kernel<CT, VT, CG>), dim3(grid_for(m, kThreads / CG)), dim3(kThreads), 0, st, val, outer,    \
                               nstored, inner, B, N, ldb, C, ldc, accumulate);                                                 \
    } while (0)
    if (N > 32) SPMI_DENSE(64);
    else if (N > 8) SPMI_DENSE(32);
    else if (N > 1) SPMI_DENSE(8);
    else SPMI_DENSE(1);
#undef SPMI_DENSE
    SP_HIP(hipGetLastError());
    return SP_OK;
}

}  // namespace

#define SPMI_DISPATCH_TYPES(FN, A, ...)                                                             \
    do {                                                                                            \
        const int pw__ = (A)->enc.pw, cw__ = (A)->enc.cw;                                           \
        if ((A)->dtype == SP_F64) {                                                                 \
            if (pw__ == 32 && cw__ == 32) return FN<int32_t, int32_t, double>(A, (const double *)B, N, ldb, (double *)C, ldc, accumulate, st); \
            if (pw__ == 32) return FN<int32_t, int64_t, double>(A, (const double *)B, N, ldb, (double *)C, ldc, accumulate, st);               \
            if (cw__ == 32) return FN<int64_t, int32_t, double>(A, (const double *)B, N, ldb, (double *)C, ldc, accumulate, st);               \
            return FN<int64_t, int64_t, double>(A, (const double *)B, N, ldb, (double *)C, ldc, accumulate, st);                               \
        } else {                                                                                    \
            if (pw__ == 32 && cw__ == 32) return FN<int32_t, int32_t, float>(A, (const float *)B, N, ldb, (float *)C, ldc, accumulate, st);    \
            if (pw__ == 32) return FN<int32_t, int64_t, float>(A, (const float *)B, N, ldb, (float *)C, ldc, accumulate, st);                  \
            if (cw__ == 32) return FN<int64_t, int32_t, float>(A, (const float *)B, N, ldb, (float *)C, ldc, accumulate, st);                  \
            return FN<int64_t, int64_t, float>(A, (const float *)B, N, ldb, (float *)C, ldc, accumulate, st);                                  \
        }                                                                                           \
    } while (0)

sp_status spmi_matmul_rowmajor(const sp_tensor *A, const void *B, int64_t N, int64_t ldb, void *C, int64_t ldc, int accumulate,
                               hipStream_t st)
{
    SPMI_DISPATCH_TYPES(rowmajor_t, A);
}

sp_status spmi_prepare_rowmajor(const sp_tensor *A, int64_t N, hipStream_t st)
{
    const void *B = nullptr; void *C = nullptr; const int64_t ldb = N, ldc = N; const int accumulate = 0;
    SPMI_DISPATCH_TYPES(prepare_rowmajor_t, A);
}

sp_status spmi_prepare_dense_inner(const sp_tensor *A, int64_t N, hipStream_t st)
{
    const void *B = nullptr; void *C = nullptr; const int64_t ldb = N, ldc = N; const int accumulate = 0;
    SPMI_DISPATCH_TYPES(prepare_dense_inner_t, A);
}

sp_status spmi_matmul_colmajor_scatter(const sp_tensor *A, const void *B, int64_t N, int64_t ldb, void *C, int64_t ldc,
                                       int accumulate, hipStream_t st)
{
    SPMI_DISPATCH_TYPES(scatter_t, A);
}

sp_status spmi_matmul_dense_inner(const sp_tensor *A, const void *B, int64_t N, int64_t ldb, void *C, int64_t ldc, int accumulate,
                                  hipStream_t st)
{
    SPMI_DISPATCH_TYPES(dense_inner_t, A);
}

// ---- the product for callers that cannot allocate ------------------------------------------------------------------
// The per-block carries of the SpMM cut by stored entries live in this array instead of a buffer from the tensor's
// allocator.  Every GPU the library runs on holds its own copy until the process ends; host code reaches it only through
// the address hipGetSymbolAddress returns for the current device (the name itself is a host-side stand-in).
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];               // per device, filled in on the first call on that device

static sp_status static_scratch(void **out)
{
    int device = -1;
    SP_HIP(hipGetDevice(&device));
    if (device < 0 || device >= kMaxDevices) return SP_ERR_UNSUPPORTED;
    if (!g_scratch_ptr[device]) {
        void *ptr = nullptr;
        SP_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return SP_ERR_HIP;
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return SP_OK;
}

namespace {
template <typename PT, typename CT, typename VT>
sp_status noalloc_t(const sp_tensor *A, const VT *B, int64_t N, int64_t ldb, VT *C, int64_t ldc, int accumulate, hipStream_t st)
{
    const row_view<PT, CT> rv(A);
    constexpr int64_t V = 16 / sizeof(VT);
    const int64_t lr = N / V;
    const bool aligned = N % V == 0 && ldb % V == 0 && ldc % V == 0 && (uintptr_t)B % 16 == 0 && (uintptr_t)C % 16 == 0;
    if (!rv.rowblocks->start || !aligned || lr < 1 || lr > 64) return SP_ERR_UNSUPPORTED;
    if ((size_t)rv.rowblocks->nblocks * (size_t)N * sizeof(VT) > kStaticScratchBytes) return SP_ERR_TOO_LARGE;
    void *carry = nullptr;
    SP_TRY(static_scratch(&carry));
    if (rv.dcsr && !accumulate) SP_TRY((zero_c<PT, CT, VT>(C, A->shape[0], N, ldc, st)));   // rows that are not stored become zero
    if (rv.nrows == 0) return SP_OK;
    // nothing in the carries has to start at zero: a block writes its carry before the fix-up reads it, and the fix-up
    // reads only carries of blocks whose first row began in an earlier block
    return spmm_windows_launch<PT, CT, VT>(A, rv, B, N, ldb, C, ldc, accumulate, (VT *)carry, st);
}
}  // namespace

extern "C" sp_status sp_matmul_noalloc(const sp_tensor *A, const void *B, int64_t N, int64_t ldb, void *C, int64_t ldc, int accumulate,
                                       void *stream)
{
    if (!A) return SP_ERR_NULL;
    if (A->enc.rank != 2) return SP_ERR_RANK;
    if (N < 0 || ldb < N || ldc < N || ldb < 1 || ldc < 1) return SP_ERR_SHAPE;
    if (N == 0 || A->shape[0] == 0) return SP_OK;
    if (!C || (!B && A->shape[1] > 0)) return SP_ERR_NULL;
    if (A->enc.lt[1] != SP_COMPRESSED || A->enc.perm[0] != 0 || A->tables_pending) return SP_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    SPMI_DISPATCH_TYPES(noalloc_t, A);
}
