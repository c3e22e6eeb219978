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
//
// When a full row of C fits the LDS (72 KB: 9216 columns in f64) and the operands are CSR / DCSR with a CSR result,
// the paper's workspace itself is used instead, one wave per row of A with the workspace in LDS: a first kernel
// marks the columns a row reaches in an n-bit map and counts them, the counts are scanned into C's pos, and a second
// kernel adds the products into a dense row of n values (32 chunks of 64 entries of B requested at a time), then walks the bit map in column order and writes crd and
// values: the paper's expand / compress, with the sort of the added indices replaced by the ordered walk.  One wave
// owns a row and takes the pairs in a fixed order, so there are no atomics on values and the bits repeat.
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
    VT *payload = (VT *)tmp.get((((size_t)(total > 0 ? total : 1) * sizeof(VT)) + 15) & ~(size_t)15);   // the result may keep it as its values
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

// ---- a row of C at a time in an LDS workspace ---------------------------------------------------------------------
constexpr int64_t kWorkspaceBytes = 72 * 1024;          // dense row of C + its bit map; two such waves fit a CU's LDS

// *out = the last entry of a scanned pos array (the number of stored entries), sign-extended: a 32-bit count that wrapped
// stays negative
template <typename PT>
__global__ void spgemm_last_pos_kernel(const PT *__restrict__ last, long long *__restrict__ out) { *out = (long long)*last; }

// block = one stored row r of A, four waves that take the selected rows of B in turn (marking a column is an OR: the order
// does not matter).  count[i] = number of distinct columns the row reaches.
constexpr int kCountWaves = 4;
template <typename PT, typename CT>
__global__ __launch_bounds__(64 * kCountWaves) void spgemm_ws_count_kernel(const PT *__restrict__ apos, const CT *__restrict__ acrd,
                                                                           const CT *__restrict__ arowid, const PT *__restrict__ bpos,
                                                                           const CT *__restrict__ bcrd, int64_t n, PT *__restrict__ count)
{
    extern __shared__ uint32_t ws_bits[];
    __shared__ int partial[kCountWaves];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t r = blockIdx.x;
    const int64_t a0 = (int64_t)apos[r], a1 = (int64_t)apos[r + 1];
    if (a1 == a0) return;                                          // the whole block
    const int64_t words = (n + 31) >> 5;
    for (int64_t w = threadIdx.x; w < words; w += 64 * kCountWaves) ws_bits[w] = 0u;
    __syncthreads();
    for (int64_t g = a0; g < a1; g += 64) {
        const int64_t e = g + lane;
        int64_t b0 = 0, b1 = 0;
        if (e < a1) {
            const int64_t k = (int64_t)acrd[e];
            b0 = (int64_t)bpos[k];
            b1 = (int64_t)bpos[k + 1];
        }
        const int cnt = (int)(a1 - g < 64 ? a1 - g : 64);
        for (int x = wave; x < cnt; x += kCountWaves) {            // wave-uniform
            const int64_t s0 = __shfl(b0, x, 64), s1 = __shfl(b1, x, 64);
            for (int64_t t = s0 + lane; t < s1; t += 64) {
                const uint32_t j = (uint32_t)bcrd[t];
                atomicOr(&ws_bits[j >> 5], 1u << (j & 31));
            }
        }
    }
    __syncthreads();
    int c = 0;
    for (int64_t w = threadIdx.x; w < words; w += 64 * kCountWaves) c += __popc(ws_bits[w]);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) c += __shfl_xor(c, d, 64);
    if (lane == 0) partial[wave] = c;
    __syncthreads();
    if (threadIdx.x == 0) {
        int total = 0;
        for (int w = 0; w < kCountWaves; ++w) total += partial[w];
        count[arowid ? (int64_t)arowid[r] : r] = (PT)total;
    }
}

// block = one wave = one stored row r of A; LDS: n values, the n-bit map, then a short list of chunk descriptors.
// The rows of B that the row of A selects are cut into chunks of 64 entries (one per lane); U chunks are requested
// together, whichever rows they belong to, and then added in turn, so that only two waves per CU (the workspace
// fills the LDS) still keep many loads in flight.  The order of the additions to one element is fixed by the
// structure, not by timing.
constexpr int kChunkList = 64;             // one descriptor per lane
template <typename VT>
struct chunk_list {
    int64_t start[kChunkList];
    int32_t len[kChunkList];
    VT a[kChunkList];
};

// the value a given lane holds, as a wave-uniform value (lane index uniform)
__device__ inline int64_t uniform_i64(int64_t v, int src)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(uint64_t)v, src);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), src);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}
__device__ inline double uniform_val(double v, int src) { return __longlong_as_double(uniform_i64(__double_as_longlong(v), src)); }
__device__ inline float uniform_val(float v, int src) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src)); }

template <typename PT, typename CT, typename VT, int U>
__global__ __launch_bounds__(64) void spgemm_ws_numeric_kernel(const PT *__restrict__ apos, const CT *__restrict__ acrd,
                                                               const VT *__restrict__ aval, const CT *__restrict__ arowid,
                                                               const PT *__restrict__ bpos, const CT *__restrict__ bcrd,
                                                               const VT *__restrict__ bval, int64_t n, const PT *__restrict__ cpos,
                                                               CT *__restrict__ ccrd, VT *__restrict__ cval)
{
    extern __shared__ unsigned char ws_raw[];
    __shared__ chunk_list<VT> list;
    VT *acc = (VT *)ws_raw;
    uint32_t *bits = (uint32_t *)(ws_raw + (size_t)n * sizeof(VT));
    const int lane = threadIdx.x;
    const int64_t r = blockIdx.x;
    const int64_t a0 = (int64_t)apos[r], a1 = (int64_t)apos[r + 1];
    if (a1 == a0) return;
    const int64_t words = (n + 31) >> 5;
    for (int64_t j = lane; j < n; j += 64) acc[j] = (VT)0;
    for (int64_t w = lane; w < words; w += 64) bits[w] = 0u;
    __syncthreads();
    for (int64_t g = a0; g < a1; g += 64) {
        const int64_t e = g + lane;
        int64_t b0 = 0, b1 = 0;
        VT a = (VT)0;
        if (e < a1) {
            const int64_t k = (int64_t)acrd[e];
            a = aval[e];
            b0 = (int64_t)bpos[k];
            b1 = (int64_t)bpos[k + 1];
        }
        // chunks of this lane's row of B, numbered across the wave in lane order
        const int mine = (int)((b1 - b0 + 63) >> 6);
        int before = mine;                                         // inclusive scan over the lanes
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(before, d, 64);
            if (lane >= d) before += up;
        }
        const int total = __shfl(before, 63, 64);
        before -= mine;
        for (int w0 = 0; w0 < total; w0 += kChunkList) {           // wave-uniform: a window of the chunk numbering
            for (int c = 0; c < mine; ++c) {
                const int id = before + c - w0;
                if (id >= 0 && id < kChunkList) {
                    const int64_t s = b0 + (int64_t)c * 64;
                    list.start[id] = s;
                    list.len[id] = (int32_t)(b1 - s < 64 ? b1 - s : 64);
                    list.a[id] = a;
                }
            }
            __syncthreads();
            const int here = total - w0 < kChunkList ? total - w0 : kChunkList;
            // lane x keeps descriptor x in registers; the loop below reads them with readlane (no LDS round trip per chunk)
            const int64_t my_start = lane < here ? list.start[lane] : 0;
            const int my_len = lane < here ? list.len[lane] : 0;
            const VT my_a = lane < here ? list.a[lane] : (VT)0;
            for (int d0 = 0; d0 < here; d0 += U) {
                uint32_t j[U];
                VT p[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    j[u] = 0xffffffffu;
                    p[u] = (VT)0;
                    if (d0 + u < here) {                           // wave-uniform
                        // a wave-uniform base plus the lane: the address needs no vector arithmetic
                        const int64_t s0 = uniform_i64(my_start, d0 + u);
                        const CT *cp = bcrd + s0;
                        const VT *vp = bval + s0;
                        if (lane < __builtin_amdgcn_readlane(my_len, d0 + u)) {
                            j[u] = (uint32_t)cp[lane];
                            p[u] = vp[lane];
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (d0 + u < here && j[u] != 0xffffffffu) {
                        // LDS atomics without a return value: the LDS takes one wave's instructions in the order
                        // they were issued, so the additions to one element still happen in program order
                        atomicOr(&bits[j[u] >> 5], 1u << (j[u] & 31));
                        atomicAdd(&acc[j[u]], uniform_val(my_a, d0 + u) * p[u]);
                    }
                }
            }
            __syncthreads();
        }
    }
    __syncthreads();
    // the compress step: set bits in column order.  Row-relative 32-bit positions on wave-uniform row pointers.
    const int64_t row_at = (int64_t)cpos[arowid ? (int64_t)arowid[r] : r];
    CT *crow = ccrd + row_at;
    VT *vrow = cval + row_at;
    uint32_t base = 0;
    const uint32_t n32 = (uint32_t)n;
    const unsigned long long below = (1ull << lane) - 1ull;
    for (uint32_t j0 = 0; j0 < n32; j0 += 64) {
        const uint32_t j = j0 + lane;
        const bool set = j < n32 && ((bits[j >> 5] >> (j & 31)) & 1u);
        const unsigned long long mask = __ballot(set);
        if (set) {
            const uint32_t o = base + (uint32_t)__popcll(mask & below);
            crow[o] = (CT)j;
            vrow[o] = acc[j];
        }
        base += (uint32_t)__popcll(mask);
    }
}

// The same with four waves per row of A.  B is read from a copy cut into (at most) four column panels of 2^shift columns
// (a CSR over the virtual rows panel * kdim + k, built once per B and kept): wave w takes panel w, i.e. the columns
// [w << shift, (w + 1) << shift) of every row of B that the row of A selects.  The waves share one workspace but never
// an element of it, so no two waves ever add to the same value and the order of the additions to an element is still
// fixed by the structure.  Chunks are 32 entries, two per instruction (one per half-wave); each wave compresses its
// own columns.
constexpr int kPanelWaves = 4, kHalfChunk = 32, kPanelList = 64;
template <typename VT>
struct panel_lists {
    int64_t start[kPanelWaves][kPanelList];
    int32_t len[kPanelWaves][kPanelList];
    VT a[kPanelWaves][kPanelList];
};

template <typename PT, typename CT, typename VT, int U>
__global__ __launch_bounds__(64 * kPanelWaves) void spgemm_ws_numeric_panels_kernel(
    const PT *__restrict__ apos, const CT *__restrict__ acrd, const VT *__restrict__ aval, const CT *__restrict__ arowid,
    const PT *__restrict__ spos, const CT *__restrict__ scrd, const VT *__restrict__ sval, int64_t kdim, int shift, int64_t n,
    const PT *__restrict__ cpos, CT *__restrict__ ccrd, VT *__restrict__ cval)
{
    extern __shared__ unsigned char ws_raw[];
    __shared__ panel_lists<VT> lists;
    VT *acc = (VT *)ws_raw;
    uint32_t *bits = (uint32_t *)(ws_raw + (size_t)n * sizeof(VT));
    const int lane = threadIdx.x & 63, half = lane >> 5, hl = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t r = blockIdx.x;
    const int64_t a0 = (int64_t)apos[r], a1 = (int64_t)apos[r + 1];
    if (a1 == a0) return;                                          // the whole block
    const int64_t words = (n + 31) >> 5;
    for (int64_t j = threadIdx.x; j < n; j += 64 * kPanelWaves) acc[j] = (VT)0;
    for (int64_t w = threadIdx.x; w < words; w += 64 * kPanelWaves) bits[w] = 0u;
    __syncthreads();
    const int64_t col_lo = (int64_t)wave << shift;                 // this wave's columns: [col_lo, col_hi)
    const int64_t col_hi = col_lo + ((int64_t)1 << shift) < n ? col_lo + ((int64_t)1 << shift) : n;
    if (col_lo < n) {
        const PT *wpos = spos + (int64_t)wave * kdim;              // the pos entries of this wave's panel
        for (int64_t g = a0; g < a1; g += 64) {
            const int64_t e = g + lane;
            int64_t b0 = 0, b1 = 0;
            VT a = (VT)0;
            if (e < a1) {
                const int64_t k = (int64_t)acrd[e];
                a = aval[e];
                b0 = (int64_t)wpos[k];
                b1 = (int64_t)wpos[k + 1];
            }
            const int mine = (int)((b1 - b0 + kHalfChunk - 1) / kHalfChunk);
            int before = mine;                                     // inclusive scan over the lanes
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int up = __shfl_up(before, d, 64);
                if (lane >= d) before += up;
            }
            const int total = __shfl(before, 63, 64);
            before -= mine;
            for (int w0 = 0; w0 < total; w0 += kPanelList) {       // wave-uniform: a window of the chunk numbering
                for (int c = 0; c < mine; ++c) {
                    const int id = before + c - w0;
                    if (id >= 0 && id < kPanelList) {
                        const int64_t st = b0 + (int64_t)c * kHalfChunk;
                        lists.start[wave][id] = st;
                        lists.len[wave][id] = (int32_t)(b1 - st < kHalfChunk ? b1 - st : kHalfChunk);
                        lists.a[wave][id] = a;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                const int here = total - w0 < kPanelList ? total - w0 : kPanelList;
                for (int d0 = 0; d0 < here; d0 += 2 * U) {
                    uint32_t j[U];
                    VT p[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        j[u] = 0xffffffffu;
                        p[u] = (VT)0;
                        const int d = d0 + 2 * u + half;           // one descriptor per half-wave
                        if (d0 + 2 * u < here) {                   // wave-uniform
                            if (d < here && hl < lists.len[wave][d]) {
                                const int64_t t = lists.start[wave][d] + hl;
                                j[u] = (uint32_t)scrd[t];
                                p[u] = lists.a[wave][d] * sval[t];
                            }
                        }
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        if (d0 + 2 * u < here && j[u] != 0xffffffffu) {
                            atomicOr(&bits[j[u] >> 5], 1u << (j[u] & 31));
                            atomicAdd(&acc[j[u]], p[u]);
                        }
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }
    }
    __syncthreads();
    if (col_lo >= n) return;
    // the compress step for this wave's columns; its first output follows the set bits of the columns before
    int before_cols = 0;
    for (int64_t w = lane; w < (col_lo >> 5); w += 64) before_cols += __popc(bits[w]);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) before_cols += __shfl_xor(before_cols, d, 64);
    const int64_t row_at = (int64_t)cpos[arowid ? (int64_t)arowid[r] : r] + before_cols;
    CT *crow = ccrd + row_at;
    VT *vrow = cval + row_at;
    uint32_t base = 0;
    const unsigned long long below = (1ull << lane) - 1ull;
    for (uint32_t j0 = (uint32_t)col_lo; j0 < (uint32_t)col_hi; j0 += 64) {
        const uint32_t j = j0 + lane;
        const bool set = j < (uint32_t)col_hi && ((bits[j >> 5] >> (j & 31)) & 1u);
        const unsigned long long mask = __ballot(set);
        if (set) {
            const uint32_t o = base + (uint32_t)__popcll(mask & below);
            crow[o] = (CT)j;
            vrow[o] = acc[j];
        }
        base += (uint32_t)__popcll(mask);
    }
}

// bounds[k * (panels + 1) + p] = position of the first entry of row k of B whose column is >= p << shift (p = panels: the
// end of the row): where each column panel's share of the row starts, the row staying where it is.
template <typename PT, typename CT>
__global__ __launch_bounds__(256) void spgemm_panel_bounds_kernel(const PT *__restrict__ bpos, const CT *__restrict__ bcrd, int64_t kdim,
                                                                  int shift, int panels, uint32_t *__restrict__ bounds)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= kdim * (panels + 1)) return;
    const int64_t k = i / (panels + 1);
    const int p = (int)(i - k * (panels + 1));
    int64_t lo = (int64_t)bpos[k], hi = (int64_t)bpos[k + 1];
    const int64_t first = (int64_t)p << shift;
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if ((int64_t)bcrd[mid] < first) lo = mid + 1;
        else hi = mid;
    }
    bounds[i] = (uint32_t)lo;
}

// Sixteen waves per row of A, for wide rows of C: the same ownership of columns (wave w works on the columns of panel
// w and on its own part of the workspace, so the additions to an element keep a fixed order) with four times the waves
// in flight per CU.  B is read where it is, through the table of panel bounds inside each row (above): the sixteen
// shares of a row of B are neighbours in memory and the block's waves ask for them at about the same time, so a line
// is fetched once (with the regrouped copy that the four-wave kernel reads, every 40-byte share cost its own lines:
// 1.83 GB past the L2 per product).  A wave loads 64 entries of the row of A at once (one per lane, with the bounds
// of the selected row of B inside the wave's panel) and hands them out, 32 at a time through a small LDS table, to its
// eight groups of eight lanes, four entries per group in flight: a group walks its segment of the row of B eight
// entries at a time.  Measured on the 8192 x 8192 product of density 0.01 (348 us; 478 us with four waves): leaving the
// adds out changes nothing, the kernel waits for its many short loads (a panel's share of a row of B is five entries);
// 75 us of it are clearing the workspace, 50 us writing the row out.
constexpr int kWideWaves = 16, kWideGroup = 8, kWideStage = 32;
constexpr int64_t kWideMinColumns = 8192;               // from this many columns of C on the sixteen-wave kernel is the default
template <typename VT>
struct wide_entry {
    uint32_t b0, b1;      // the segment of the selected row of B inside the wave's panel (offsets into the panel copy)
    VT a;                 // the value of the entry of A
};

template <typename PT, typename CT, typename VT>
__global__ __launch_bounds__(64 * kWideWaves) void spgemm_ws_numeric_wide_kernel(
    const PT *__restrict__ apos, const CT *__restrict__ acrd, const VT *__restrict__ aval, const CT *__restrict__ arowid, int64_t arows,
    const uint32_t *__restrict__ bounds, const CT *__restrict__ scrd, const VT *__restrict__ sval, int shift, int64_t n,
    const PT *__restrict__ cpos, CT *__restrict__ ccrd, VT *__restrict__ cval)
{
    constexpr int G = kWideGroup, NG = 64 / G, U = 4;
    static_assert(NG * U == kWideStage, "one pass over the table hands out all of it");
    extern __shared__ unsigned char ws_raw[];
    __shared__ wide_entry<VT> table[kWideWaves][kWideStage];
    VT *acc = (VT *)ws_raw;
    uint32_t *bits = (uint32_t *)(ws_raw + (size_t)n * sizeof(VT));
    const int lane = threadIdx.x & 63, g = lane / G, gl = lane % G;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t words = (n + 31) >> 5;
    // The block keeps its workspace over all the rows it takes (r = blockIdx.x, + gridDim.x, ...): cleared once here, and
    // after every row each wave clears exactly what the row has touched in its columns while it writes them out.
    for (int64_t j = threadIdx.x; j < n; j += 64 * kWideWaves) acc[j] = (VT)0;
    for (int64_t w = threadIdx.x; w < words; w += 64 * kWideWaves) bits[w] = 0u;
    __syncthreads();
    const int64_t col_lo = (int64_t)wave << shift;                 // this wave's columns: [col_lo, col_hi), a multiple of 64 wide
    const int64_t col_hi = col_lo + ((int64_t)1 << shift) < n ? col_lo + ((int64_t)1 << shift) : n;
    const uint32_t *wbounds = bounds + wave;                       // this wave's panel in every row's kWideWaves + 1 bounds
    wide_entry<VT> *mine = table[wave];
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int64_t r = blockIdx.x; r < arows; r += gridDim.x) {
        const int64_t a0 = (int64_t)apos[r], a1 = (int64_t)apos[r + 1];
        if (a1 == a0) continue;                                    // the whole block
        if (col_lo < n) {
            for (int64_t g0 = a0; g0 < a1; g0 += 64) {
                const int64_t e = g0 + lane;
                wide_entry<VT> w;
                w.b0 = 0; w.b1 = 0; w.a = (VT)0;                   // lanes past the row hold empty segments
                if (e < a1) {
                    const int64_t k = (int64_t)acrd[e];
                    w.a = aval[e];
                    w.b0 = wbounds[k * (kWideWaves + 1)];
                    w.b1 = wbounds[k * (kWideWaves + 1) + 1];
                }
                const int cnt = (int)(a1 - g0 < 64 ? a1 - g0 : 64);   // wave-uniform
                for (int s0 = 0; s0 < cnt; s0 += kWideStage) {
                    if (lane >= s0 && lane < s0 + kWideStage) mine[lane - s0] = w;
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                    wide_entry<VT> seg[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) seg[u] = mine[u * NG + g];
                    uint32_t j[U];
                    VT p[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {                  // the first eight entries of each segment: all loads first
                        const uint32_t t = seg[u].b0 + (uint32_t)gl;
                        j[u] = 0xffffffffu;
                        p[u] = (VT)0;
                        if (t < seg[u].b1) { j[u] = (uint32_t)scrd[t]; p[u] = seg[u].a * sval[t]; }
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        if (j[u] != 0xffffffffu) {
                            atomicOr(&bits[j[u] >> 5], 1u << (j[u] & 31));
                            atomicAdd(&acc[j[u]], p[u]);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u)                    // what is left of longer segments
                        for (uint32_t t = seg[u].b0 + (uint32_t)(G + gl); __any(t < seg[u].b1); t += G)
                            if (t < seg[u].b1) {
                                const uint32_t jj = (uint32_t)scrd[t];
                                atomicOr(&bits[jj >> 5], 1u << (jj & 31));
                                atomicAdd(&acc[jj], seg[u].a * sval[t]);
                            }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the table is rewritten in the next pass
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                }
            }
        }
        __syncthreads();
        // the compress step for this wave's columns; its first output follows the set bits of the columns before
        if (col_lo < n) {
            int before_cols = 0;
            for (int64_t w = lane; w < (col_lo >> 5); w += 64) before_cols += __popc(bits[w]);
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) before_cols += __shfl_xor(before_cols, d, 64);
            const int64_t row_at = (int64_t)cpos[arowid ? (int64_t)arowid[r] : r] + before_cols;
            CT *crow = ccrd + row_at;
            VT *vrow = cval + row_at;
            uint32_t base = 0;
            for (uint32_t j0 = (uint32_t)col_lo; j0 < (uint32_t)col_hi; j0 += 64) {
                const uint32_t j = j0 + lane;
                const bool set = j < (uint32_t)col_hi && ((bits[j >> 5] >> (j & 31)) & 1u);
                const unsigned long long mask = __ballot(set);
                if (set) {
                    const uint32_t o = base + (uint32_t)__popcll(mask & below);
                    crow[o] = (CT)j;
                    vrow[o] = acc[j];
                    acc[j] = (VT)0;                                // clean for the block's next row
                }
                base += (uint32_t)__popcll(mask);
            }
        }
        __syncthreads();                                           // every wave has counted the bits before its columns
        if (col_lo < n)
            for (int64_t w = (col_lo >> 5) + lane; w < ((col_hi + 31) >> 5); w += 64) bits[w] = 0u;
        // no barrier needed here: until the next row's barrier only this wave touches these words again
    }
}

// Sixteen waves per row of A with the ENTRIES of the row dealt out instead of the columns: wave w takes entries
// w, w + 16, ... of the row of A, a half-wave walks one selected row of B, 32 entries at a time with contiguous loads
// (no column-panel copy of B, a sixth of the load requests of the kernel above).  All waves add into the one
// workspace, so the order in which the products of one element of C meet depends on timing: results agree to rounding,
// not bit for bit.  Persistent blocks and the clean-as-you-go workspace as above; wave w writes out columns
// [w * n / 16 rounded to 64, ...).
template <typename PT, typename CT, typename VT>
__global__ __launch_bounds__(64 * kWideWaves) void spgemm_ws_numeric_entries_kernel(
    const PT *__restrict__ apos, const CT *__restrict__ acrd, const VT *__restrict__ aval, const CT *__restrict__ arowid, int64_t arows,
    const PT *__restrict__ bpos, const CT *__restrict__ bcrd, const VT *__restrict__ bval, int64_t n,
    const PT *__restrict__ cpos, CT *__restrict__ ccrd, VT *__restrict__ cval)
{
    constexpr int W = kWideWaves, U = 2;
    extern __shared__ unsigned char ws_raw[];
    __shared__ wide_entry<VT> table[W][kWideStage];
    VT *acc = (VT *)ws_raw;
    uint32_t *bits = (uint32_t *)(ws_raw + (size_t)n * sizeof(VT));
    const int lane = threadIdx.x & 63, half = lane >> 5, hl = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t words = (n + 31) >> 5;
    for (int64_t j = threadIdx.x; j < n; j += 64 * W) acc[j] = (VT)0;
    for (int64_t w = threadIdx.x; w < words; w += 64 * W) bits[w] = 0u;
    __syncthreads();
    const int64_t span = ((n + W - 1) / W + 63) & ~(int64_t)63;     // columns a wave writes out: a multiple of 64
    const int64_t col_lo = (int64_t)wave * span < n ? (int64_t)wave * span : n;
    const int64_t col_hi = col_lo + span < n ? col_lo + span : n;
    wide_entry<VT> *mine = table[wave];
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int64_t r = blockIdx.x; r < arows; r += gridDim.x) {
        const int64_t a0 = (int64_t)apos[r], a1 = (int64_t)apos[r + 1];
        if (a1 == a0) continue;                                    // the whole block
        for (int64_t g0 = a0 + wave; g0 < a1; g0 += kWideStage * W) {      // 32 of this wave's entries at a time, one per lane of the lower half
            const int64_t e = g0 + (int64_t)lane * W;
            wide_entry<VT> w;
            w.b0 = 0; w.b1 = 0; w.a = (VT)0;                       // lanes past the row hold empty rows of B
            if (lane < kWideStage && e < a1) {
                const int64_t k = (int64_t)acrd[e];
                w.a = aval[e];
                w.b0 = (uint32_t)bpos[k];
                w.b1 = (uint32_t)bpos[k + 1];
            }
            if (lane < kWideStage) mine[lane] = w;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int64_t mine_left = (a1 - g0 + W - 1) / W;       // this wave's entries from g0 on
            const int cnt = (int)(mine_left < kWideStage ? mine_left : kWideStage);   // wave-uniform
            for (int s0 = 0; s0 < cnt; s0 += 2 * U) {              // U rows of B per half-wave in flight
                wide_entry<VT> seg[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int idx = s0 + 2 * u + half;
                    seg[u] = mine[idx < kWideStage ? idx : kWideStage - 1];
                    if (idx >= cnt) seg[u].b1 = seg[u].b0;
                }
                uint32_t j[U];
                VT p[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {                      // the first 32 entries of each row: all loads first
                    const uint32_t t = seg[u].b0 + (uint32_t)hl;
                    j[u] = 0xffffffffu;
                    p[u] = (VT)0;
                    if (t < seg[u].b1) { j[u] = (uint32_t)bcrd[t]; p[u] = seg[u].a * bval[t]; }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (j[u] != 0xffffffffu) {
                        atomicOr(&bits[j[u] >> 5], 1u << (j[u] & 31));
                        atomicAdd(&acc[j[u]], p[u]);
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u)                        // the rest of longer rows
                    for (uint32_t t = seg[u].b0 + (uint32_t)(32 + hl); __any(t < seg[u].b1); t += 32)
                        if (t < seg[u].b1) {
                            const uint32_t jj = (uint32_t)bcrd[t];
                            atomicOr(&bits[jj >> 5], 1u << (jj & 31));
                            atomicAdd(&acc[jj], seg[u].a * bval[t]);
                        }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the table is rewritten in the next batch
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        __syncthreads();
        if (col_lo < col_hi) {
            int before_cols = 0;
            for (int64_t w = lane; w < (col_lo >> 5); w += 64) before_cols += __popc(bits[w]);
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) before_cols += __shfl_xor(before_cols, d, 64);
            const int64_t row_at = (int64_t)cpos[arowid ? (int64_t)arowid[r] : r] + before_cols;
            CT *crow = ccrd + row_at;
            VT *vrow = cval + row_at;
            uint32_t base = 0;
            for (uint32_t j0 = (uint32_t)col_lo; j0 < (uint32_t)col_hi; j0 += 64) {
                const uint32_t j = j0 + lane;
                const bool set = j < (uint32_t)col_hi && ((bits[j >> 5] >> (j & 31)) & 1u);
                const unsigned long long mask = __ballot(set);
                if (set) {
                    const uint32_t o = base + (uint32_t)__popcll(mask & below);
                    crow[o] = (CT)j;
                    vrow[o] = acc[j];
                    acc[j] = (VT)0;                                // clean for the block's next row
                }
                base += (uint32_t)__popcll(mask);
            }
        }
        __syncthreads();                                           // every wave has counted the bits before its columns
        if (col_lo < col_hi)
            for (int64_t w = (col_lo >> 5) + lane; w < ((col_hi + 31) >> 5); w += 64) bits[w] = 0u;
        __syncthreads();                                           // any wave may mark any column of the next row
    }
}

template <typename PT, typename CT, typename VT>
sp_status spgemm_workspace_t(const sp_tensor *A, const sp_tensor *Br, const sp_encoding *encC, hipStream_t st, sp_tensor **out)
{
    const int64_t m = A->shape[0], n = Br->shape[1];
    const int64_t shapeC[2] = {m, n};
    sp_tensor *t = nullptr;
    int key_bits = 0;
    SP_TRY(spmi_new_tensor(encC, shapeC, (sp_dtype)A->dtype, A->alloc, A->free_, A->ctx, false, &t, &key_bits));
    sp_mem mem{A->alloc, A->free_, A->ctx};
    sp_status status = SP_OK;
    {
        sp_scratch tmp(mem);
        do {
            int *flags = (int *)tmp.get(64);
            if (!flags) { status = SP_ERR_ALLOC; break; }
            if ((status = spmi_fill_zero(flags, 64, st)) != SP_OK) break;
            const size_t pbytes = ((size_t)(m + 1) * sizeof(PT) + 15) & ~(size_t)15;
            t->pos[1] = mem.get(pbytes);
            t->npos[1] = m + 1;
            if (!t->pos[1]) { status = SP_ERR_ALLOC; break; }
            if ((status = spmi_fill_zero(t->pos[1], pbytes, st)) != SP_OK) break;
            const bool a_outer_compressed = A->enc.lt[0] == SP_COMPRESSED;
            const int64_t arows = a_outer_compressed ? A->ncrd[0] : m;
            const CT *arowid = a_outer_compressed ? (const CT *)A->crd[0] : nullptr;
            const size_t bits_bytes = (size_t)((n + 31) / 32) * 4;
            const size_t ws_bytes = (size_t)n * sizeof(VT) + bits_bytes;
            const bool work = arows > 0 && A->nvalues > 0 && Br->nvalues > 0 && n > 0;
            // sixteen waves per row for wide results (tune value 4 asks for them from 1024 columns on), else four
            const bool wide = A->tune_spgemm == 4 ? n >= kWideWaves * 64 : (A->tune_spgemm == 0 && n >= kWideMinColumns);
            if (work) {
                hipLaunchKernelGGL((spgemm_ws_count_kernel<PT, CT>), dim3((unsigned)arows), dim3(64 * kCountWaves), bits_bytes, st, (const PT *)A->pos[1],
                                   (const CT *)A->crd[1], arowid, (const PT *)Br->pos[1], (const CT *)Br->crd[1], n, (PT *)t->pos[1]);
                if (hipGetLastError() != hipSuccess) { status = SP_ERR_HIP; break; }
            }
            // the sixteen-wave kernel's table of panel bounds does not depend on the counts: enqueued here, ahead of the
            // synchronisation below, so that nothing but the allocation of C stands between that and the numeric kernel
            int pshift = 0;
            uint32_t *bounds = nullptr;
            if (work && wide) {
                while (((int64_t)kWideWaves << pshift) < n) ++pshift;       // the narrowest power of two with at most sixteen panels
                const int64_t kdim = Br->shape[0], nb = kdim * (kWideWaves + 1);
                bounds = (uint32_t *)tmp.get((size_t)nb * 4);
                if (!bounds) { status = SP_ERR_ALLOC; break; }
                hipLaunchKernelGGL((spgemm_panel_bounds_kernel<PT, CT>), dim3((unsigned)ceil_div(nb, 256)), dim3(256), 0, st, (const PT *)Br->pos[1],
                                   (const CT *)Br->crd[1], kdim, pshift, kWideWaves, bounds);
                if (hipGetLastError() != hipSuccess) { status = SP_ERR_HIP; break; }
            }
            if ((status = spmi_exclusive_scan(t->pos[1], m + 1, (int)sizeof(PT) * 8, tmp, st)) != SP_OK) break;
            // the longest row of C (the products choose kernels by it) comes back with the total, in one synchronisation
            if ((status = spmi_max_segment_async(t->pos[1], (int)sizeof(PT) * 8, m, (unsigned long long *)(flags + 4), st)) != SP_OK) break;
            // the total goes into the flags block next to the longest row: one copy to the host for both
            hipLaunchKernelGGL((spgemm_last_pos_kernel<PT>), dim3(1), dim3(1), 0, st, (const PT *)t->pos[1] + m, (long long *)(flags + 8));
            if (hipGetLastError() != hipSuccess) { status = SP_ERR_HIP; break; }
            long long back[6] = {0, 0, 0, 0, 0, 0};                // bytes 0..47 of the block: [2] = longest row, [4] = total
            if (hipMemcpyAsync(back, flags, sizeof(back), hipMemcpyDeviceToHost, st) != hipSuccess ||
                hipStreamSynchronize(st) != hipSuccess) { status = SP_ERR_HIP; break; }
            t->max_segment = (int64_t)back[2];
            const int64_t nnzc = (int64_t)back[4];
            if (nnzc < 0 || nnzc >= ((int64_t)1 << 31)) { status = SP_ERR_TOO_LARGE; break; }     // a 32-bit pos that wrapped shows as negative
            t->crd[1] = mem.get((((size_t)(nnzc > 0 ? nnzc : 1) * sizeof(CT)) + 15) & ~(size_t)15);
            t->values = mem.get((((size_t)(nnzc > 0 ? nnzc : 1) * sizeof(VT)) + 15) & ~(size_t)15);
            t->ncrd[1] = nnzc;
            t->nvalues = nnzc;
            t->nnz = nnzc;
            if (!t->crd[1] || !t->values) { status = SP_ERR_ALLOC; break; }
            // four waves per row when the column-panel copy of B can be had (it is built on the first product with this B)
            const sp_tensor *Bseg = nullptr;
            const int pwaves = kPanelWaves;
            if (nnzc == 0) bounds = nullptr;
            if (!bounds && work && nnzc > 0 && A->tune_spgemm != 3 && A->tune_spgemm != 5 && n >= 4 * 64) {
                while (((int64_t)pwaves << pshift) < n) ++pshift;           // the narrowest power of two with at most that many panels
                sp_status sb = spmi_build_segments(Br, 1, (int64_t)1 << pshift, st);
                if (sb == SP_OK && Br->segments && Br->segments->shift == pshift && Br->segments->panels <= pwaves) Bseg = Br->segments->seg;
                else if (sb != SP_OK && sb != SP_ERR_UNSUPPORTED) { status = sb; break; }
            }
            if (work && nnzc > 0 && A->tune_spgemm == 5) {
                auto kernel = spgemm_ws_numeric_entries_kernel<PT, CT, VT>;
                if (hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)ws_bytes) != hipSuccess) {
                    status = SP_ERR_HIP;
                    break;
                }
                const unsigned nblocks = (unsigned)(arows < 512 ? arows : 512);
                hipLaunchKernelGGL(kernel, dim3(nblocks), dim3(64 * kWideWaves), ws_bytes, st, (const PT *)A->pos[1], (const CT *)A->crd[1],
                                   (const VT *)A->values, arowid, arows, (const PT *)Br->pos[1], (const CT *)Br->crd[1], (const VT *)Br->values,
                                   n, (const PT *)t->pos[1], (CT *)t->crd[1], (VT *)t->values);
                if (hipGetLastError() != hipSuccess) { status = SP_ERR_HIP; break; }
            } else if (bounds) {
                auto kernel = spgemm_ws_numeric_wide_kernel<PT, CT, VT>;
                if (hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)ws_bytes) != hipSuccess) {
                    status = SP_ERR_HIP;
                    break;
                }
                // two blocks fit a CU's LDS: that many blocks, each taking every 512th row
                const unsigned wide_blocks = (unsigned)(arows < 512 ? arows : 512);
                hipLaunchKernelGGL(kernel, dim3(wide_blocks), dim3(64 * kWideWaves), ws_bytes, st, (const PT *)A->pos[1], (const CT *)A->crd[1],
                                   (const VT *)A->values, arowid, arows, (const uint32_t *)bounds, (const CT *)Br->crd[1], (const VT *)Br->values,
                                   pshift, n, (const PT *)t->pos[1], (CT *)t->crd[1], (VT *)t->values);
                if (hipGetLastError() != hipSuccess) { status = SP_ERR_HIP; break; }
            } else if (Bseg) {
                auto kernel = spgemm_ws_numeric_panels_kernel<PT, CT, VT, 8>;
                if (hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)ws_bytes) != hipSuccess) {
                    status = SP_ERR_HIP;
                    break;
                }
                hipLaunchKernelGGL(kernel, dim3((unsigned)arows), dim3(64 * kPanelWaves), ws_bytes, st, (const PT *)A->pos[1], (const CT *)A->crd[1],
                                   (const VT *)A->values, arowid, (const PT *)Bseg->pos[1], (const CT *)Bseg->crd[1], (const VT *)Bseg->values,
                                   Br->shape[0], pshift, n, (const PT *)t->pos[1], (CT *)t->crd[1], (VT *)t->values);
                if (hipGetLastError() != hipSuccess) { status = SP_ERR_HIP; break; }
            } else if (work && nnzc > 0) {
                auto kernel = spgemm_ws_numeric_kernel<PT, CT, VT, 32>;
                if (hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)ws_bytes) != hipSuccess) {
                    status = SP_ERR_HIP;
                    break;
                }
                hipLaunchKernelGGL(kernel, dim3((unsigned)arows), dim3(64), ws_bytes, st, (const PT *)A->pos[1], (const CT *)A->crd[1],
                                   (const VT *)A->values, arowid, (const PT *)Br->pos[1], (const CT *)Br->crd[1], (const VT *)Br->values, n,
                                   (const PT *)t->pos[1], (CT *)t->crd[1], (VT *)t->values);
                if (hipGetLastError() != hipSuccess) { status = SP_ERR_HIP; break; }
            }
            // the tables that only sp_matmul and sp_sddmm read (row blocks, non-empty rows) are built when one of them first
            // takes this tensor: a result that goes into another sparse product never needs them
            t->tables_pending = 1;
            if (hipStreamSynchronize(st) != hipSuccess) { status = SP_ERR_HIP; break; }
        } while (0);
        if (status != SP_OK) (void)hipStreamSynchronize(st);
    }
    return spmi_finish_pack(t, status, st, out);
}

// can the workspace kernels take this product?
static bool workspace_fits(const sp_tensor *A, const sp_tensor *Br, const sp_encoding *encC)
{
    const int64_t n = Br->shape[1];
    const size_t vsz = A->dtype == SP_F64 ? 8 : 4;
    return encC->lt[0] == SP_DENSE && encC->lt[1] == SP_COMPRESSED && encC->perm[0] == 0 &&        // C in CSR
           A->enc.perm[0] == 0 && A->enc.lt[1] == SP_COMPRESSED &&                                 // A in CSR or DCSR
           Br->enc.lt[0] == SP_DENSE &&                                                            // B's rows indexed directly
           A->enc.pw == Br->enc.pw && A->enc.cw == Br->enc.cw && encC->pw == A->enc.pw && encC->cw == A->enc.cw &&
           encC->pw_store >= 32 && encC->cw_store >= 32 &&
           (size_t)n * vsz + (size_t)((n + 31) / 32) * 4 <= (size_t)kWorkspaceBytes &&
           (unsigned __int128)A->shape[0] * (unsigned __int128)n < ((unsigned __int128)1 << 31);        // so that no 32-bit pos can wrap
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
        SP_TRY(spmi_build_transposed(B, st));
        Br = B->transposed;
    }
    const int pw = Br->enc.pw, cw = Br->enc.cw;
    const bool fits = workspace_fits(A, Br, encC);
    if (A->tune_spgemm >= 2 && !fits) return SP_ERR_UNSUPPORTED;
    if (fits && A->tune_spgemm != 1) {
#define SPMI_WS(PT, CT)                                                                                        \
    return A->dtype == SP_F64 ? spgemm_workspace_t<PT, CT, double>(A, Br, encC, st, C) : spgemm_workspace_t<PT, CT, float>(A, Br, encC, st, C)
        if (pw == 32 && cw == 32) SPMI_WS(int32_t, int32_t);
        if (pw == 32) SPMI_WS(int32_t, int64_t);
        if (cw == 32) SPMI_WS(int64_t, int32_t);
        SPMI_WS(int64_t, int64_t);
#undef SPMI_WS
    }
#define SPMI_GO(PT, CT)                                                                                        \
    return A->dtype == SP_F64 ? spgemm_t<PT, CT, double>(A, Br, encC, st, C) : spgemm_t<PT, CT, float>(A, Br, encC, st, C)
    if (pw == 32 && cw == 32) SPMI_GO(int32_t, int32_t);
    if (pw == 32) SPMI_GO(int32_t, int64_t);
    if (cw == 32) SPMI_GO(int64_t, int32_t);
    SPMI_GO(int64_t, int64_t);
#undef SPMI_GO
}
