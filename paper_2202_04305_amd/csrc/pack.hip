// Storage builder: coordinate scheme -> pos / crd / values per level (arXiv 2202.04305, Section 4.1).
//
// Steps, all on the GPU: linearise the level coordinates into one 64-bit key per entry,
// stable LSD radix sort of (key, entry id), adjacent-equal check for duplicates, then one
// sweep per level: a compressed level marks where a new (parent, coordinate) pair starts,
// prefix-sums the marks into child positions, counts children per parent and prefix-sums
// the counts into pos; a dense level only folds the coordinate into the position.  The
// values travel through the sort as the payload and are put in place last.  Only level sizes and the error flags travel to the host.
#include <algorithm>
#include "spmi_internal.h"

namespace {

constexpr int kThreads = 256;

// ---------------------------------------------------------------------------------------
// exclusive scan (reduce / recurse on tile sums / downsweep): no spinning on other blocks
// ---------------------------------------------------------------------------------------
constexpr int kScanItems = 8;
constexpr int kScanTile = kThreads * kScanItems;

template <typename T>
__global__ __launch_bounds__(kThreads) void scan_reduce_kernel(const T *__restrict__ data, int64_t n, T *__restrict__ sums)
{
    __shared__ T wsum[kThreads / 64];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    T s = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i)
        if (base + i < n) s += data[base + i];
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d, 64);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        T tot = 0;
        for (int w = 0; w < kThreads / 64; ++w) tot += wsum[w];
        sums[blockIdx.x] = tot;
    }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void scan_downsweep_kernel(T *__restrict__ data, int64_t n, const T *__restrict__ tile_base)
{
    __shared__ T wsum[kThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    T v[kScanItems];
    T s = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        v[i] = (base + i < n) ? data[base + i] : (T)0;
        s += v[i];
    }
    T incl = wave_inclusive_scan(s, lane);
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    T run = tile_base ? tile_base[blockIdx.x] : (T)0;
    for (int w = 0; w < wave; ++w) run += wsum[w];
    run += incl - s;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        if (base + i < n) data[base + i] = run;
        run += v[i];
    }
}

template <typename T>
sp_status exclusive_scan_t(T *data, int64_t n, sp_scratch &tmp, hipStream_t st)
{
    if (n <= 0) return SP_OK;
    const int64_t nt = ceil_div(n, kScanTile);
    if (nt == 1) {
        hipLaunchKernelGGL(scan_downsweep_kernel<T>, dim3(1), dim3(kThreads), 0, st, data, n, (const T *)nullptr);
        SP_HIP(hipGetLastError());
        return SP_OK;
    }
    T *sums = (T *)tmp.get((size_t)nt * sizeof(T));
    if (!sums) return SP_ERR_ALLOC;
    hipLaunchKernelGGL(scan_reduce_kernel<T>, dim3((unsigned)nt), dim3(kThreads), 0, st, (const T *)data, n, sums);
    SP_HIP(hipGetLastError());
    SP_TRY(exclusive_scan_t<T>(sums, nt, tmp, st));
    hipLaunchKernelGGL(scan_downsweep_kernel<T>, dim3((unsigned)nt), dim3(kThreads), 0, st, data, n, (const T *)sums);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

__global__ void fill_zero_kernel(uint32_t *p, size_t nwords)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < nwords; i += stride) p[i] = 0u;
}

// ---------------------------------------------------------------------------------------
// keys, levels, values
// ---------------------------------------------------------------------------------------
struct level_args {
    const int64_t *coord[SP_MAX_RANK];   // by level
    int64_t size[SP_MAX_RANK];
    int rank;
};

// The payload that travels with the key through the sort is the value itself (its bits), so that no gather by
// entry id is needed afterwards; the first pass of the sort reads it from the caller's array.
__global__ __launch_bounds__(kThreads) void make_keys_kernel(level_args a, int64_t nnz, uint64_t *__restrict__ keys, int *__restrict__ flags)
{
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= nnz) return;
    uint64_t key = 0;
    bool bad = false;
    for (int l = 0; l < a.rank; ++l) {
        const int64_t c = a.coord[l][e];
        bad |= (c < 0) | (c >= a.size[l]);
        key = key * (uint64_t)a.size[l] + (uint64_t)c;
    }
    keys[e] = bad ? 0 : key;
    if (bad) atomicOr(&flags[0], 1);
}

// The same, a block per tile of kSpmiMsdTile entries, filling in on the way what the most-significant-digit-first sort would
// otherwise read the keys for once more (sp_msd_plan): the tile's counts by the top digit and the sampled histogram.
__global__ __launch_bounds__(kThreads) void make_keys_counting_kernel(level_args a, int64_t nnz, uint64_t *__restrict__ keys, int *__restrict__ flags,
                                                                      sp_msd_plan plan)
{
    __shared__ uint32_t h[256];
    static_assert(kThreads == 256, "one thread per digit");
    h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t tile0 = (int64_t)blockIdx.x * kSpmiMsdTile;
    bool any_bad = false;
#pragma unroll 4
    for (int r = 0; r < kSpmiMsdTile / kThreads; ++r) {
        const int64_t e = tile0 + r * kThreads + threadIdx.x;
        if (e < nnz) {
            uint64_t key = 0;
            bool bad = false;
            for (int l = 0; l < a.rank; ++l) {
                const int64_t c = a.coord[l][e];
                bad |= (c < 0) | (c >= a.size[l]);
                key = key * (uint64_t)a.size[l] + (uint64_t)c;
            }
            if (bad) key = 0;
            any_bad |= bad;
            keys[e] = key;
            atomicAdd(&h[(uint32_t)(key >> plan.digit_shift) & 255u], 1u);
            if ((e & 63) == 0) atomicAdd(&plan.samp[(uint32_t)(key >> plan.samp_shift) & 0xffffu], 1u);
        }
    }
    if (any_bad) atomicOr(&flags[0], 1);
    __syncthreads();
    plan.ctr[(size_t)threadIdx.x * plan.tiles + blockIdx.x] = h[threadIdx.x];
}

__global__ __launch_bounds__(kThreads) void check_duplicates_kernel(const uint64_t *__restrict__ keys, int64_t nnz, int *__restrict__ flags)
{
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= 1 && e < nnz && keys[e] == keys[e - 1]) atomicOr(&flags[1], 1);
}

// Division of a key by a level's stride or size, which the host knows when it launches: a shift when the divisor is a
// power of two, a multiplication by the reciprocal in double plus a one-step correction while the dividend is below
// 2^52 (the estimate is then within one of the quotient), the hardware's 64-bit division otherwise.
struct divisor {
    uint64_t d;
    double inv;
    int shift;          // >= 0: d == 1 << shift
};

static divisor make_divisor(uint64_t d)
{
    divisor v;
    v.d = d;
    v.inv = 1.0 / (double)d;
    v.shift = -1;
    if ((d & (d - 1)) == 0) { v.shift = 0; while (((uint64_t)1 << v.shift) != d) ++v.shift; }
    return v;
}

__device__ inline uint64_t div_by(uint64_t x, const divisor &v)
{
    if (v.shift >= 0) return x >> v.shift;
    if (x < ((uint64_t)1 << 52)) {
        uint64_t q = (uint64_t)((double)x * v.inv);
        const int64_t r = (int64_t)(x - q * v.d);
        if (r < 0) --q;
        else if ((uint64_t)r >= v.d) ++q;
        return q;
    }
    return x / v.d;
}

// dense level: position = parent * size + coordinate
__global__ __launch_bounds__(kThreads) void dense_level_kernel(const uint64_t *__restrict__ keys, int64_t nnz, divisor stride,
                                                               divisor size, const uint64_t *__restrict__ parent_in,
                                                               uint64_t *__restrict__ parent_out)
{
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= nnz) return;
    const uint64_t pre = div_by(keys[e], stride);
    const uint64_t c = pre - div_by(pre, size) * size.d;
    parent_out[e] = (parent_in ? parent_in[e] : 0ull) * size.d + c;
}

// compressed level, step 1: mark[e] = 1 where the key prefix down to this level changes
__global__ __launch_bounds__(kThreads) void mark_children_kernel(const uint64_t *__restrict__ keys, int64_t nnz, divisor stride,
                                                                 uint32_t *__restrict__ mark)
{
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= nnz) return;
    mark[e] = (e == 0 || div_by(keys[e], stride) != div_by(keys[e - 1], stride)) ? 1u : 0u;
}

// compressed level, step 2: write crd, count children per parent (one add per run end, one
// subtract per run start: integer atomics, so the result does not depend on their order),
// and hand each entry its child position.  child_excl = exclusive scan of the marks, or
// nullptr on the innermost level, where every entry is its own child.  dup_flags (may be null): the duplicate check of the
// sorted keys, done here on the way when the builder has not run it yet.
template <typename PT, typename CT>
__global__ __launch_bounds__(kThreads) void emit_level_kernel(const uint64_t *__restrict__ keys, int64_t nnz, divisor stride,
                                                              divisor size, const uint32_t *__restrict__ child_excl,
                                                              const uint64_t *__restrict__ parent_in, uint64_t *__restrict__ parent_out,
                                                              PT *__restrict__ cnt, CT *__restrict__ crd, int *__restrict__ dup_flags)
{
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= nnz) return;
    const uint64_t key = keys[e], key_before = e > 0 ? keys[e - 1] : 0;
    if (dup_flags && e > 0 && key == key_before) atomicOr(&dup_flags[1], 1);      // an entry given twice (see check_duplicates_kernel)
    const uint64_t pre = div_by(key, stride);
    const uint64_t pre_before = e > 0 ? div_by(key_before, stride) : 0;
    const bool first = (e == 0) || (pre_before != pre);
    const uint64_t child = child_excl ? (uint64_t)child_excl[e] + (first ? 1u : 0u) - 1u : (uint64_t)e;
    const uint64_t up = div_by(pre, size);
    if (first) crd[child] = (CT)(pre - up * size.d);
    // position of the entry at the level above: carried in parent_in, or, while every level above is dense, simply
    // the key prefix down to that level (pre / size), which needs no array
    const uint64_t par = parent_in ? parent_in[e] : up;
    const bool head = (e == 0) || (parent_in ? parent_in[e - 1] : div_by(pre_before, size)) != par;
    const bool tail = (e == nnz - 1) || (parent_in ? parent_in[e + 1] : div_by(div_by(keys[e + 1], stride), size)) != par;
    typedef typename std::conditional<sizeof(PT) == 8, unsigned long long, unsigned int>::type UT;
    if (tail) atomicAdd((UT *)&cnt[par], (UT)(child + 1));
    if (head) atomicAdd((UT *)&cnt[par], (UT)(0) - (UT)child);
    if (parent_out) parent_out[e] = child;
}

template <typename P>
__global__ __launch_bounds__(kThreads) void place_values_kernel(const P *__restrict__ sorted, const uint64_t *__restrict__ position,
                                                                int64_t nnz, P *__restrict__ vout)
{
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= nnz) return;
    vout[position ? position[e] : (uint64_t)e] = sorted[e];
}

// longest pos segment: grid-stride maximum per thread, wave and block reduction, one atomic per block
template <typename PT>
__global__ __launch_bounds__(kThreads) void max_segment_kernel(const PT *__restrict__ pos, int64_t nseg, unsigned long long *__restrict__ out)
{
    __shared__ unsigned long long wmax[kThreads / 64];
    unsigned long long len = 0;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nseg; i += (int64_t)gridDim.x * kThreads) {
        const unsigned long long l = (unsigned long long)(pos[i + 1] - pos[i]);
        len = l > len ? l : len;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const unsigned long long o = __shfl_xor(len, d, 64);
        len = o > len ? o : len;
    }
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = len;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kThreads / 64; ++w) len = wmax[w] > len ? wmax[w] : len;
        if (len) atomicMax(out, len);
    }
}

// start[b] = row holding stored entry b*T (largest r with pos[r] <= b*T); block 0 starts at row 0 and the
// sentinel is the row count, so that leading and trailing empty rows belong to some block.
template <typename PT>
__global__ __launch_bounds__(kThreads) void rowblocks_kernel(const PT *__restrict__ pos, int64_t nrows, int64_t nblocks, int64_t T,
                                                             int32_t *__restrict__ start)
{
    const int64_t b = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (b > nblocks) return;
    if (b == 0) { start[0] = 0; return; }
    if (b == nblocks) { start[b] = (int32_t)nrows; return; }
    const int64_t target = b * T;
    int64_t lo = 0, hi = nrows;            // invariant: pos[lo] <= target; pos[hi] > target or hi == nrows
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)pos[mid] <= target) lo = mid; else hi = mid;
    }
    start[b] = (int32_t)lo;
}

template <typename ST, typename DT>
__global__ __launch_bounds__(kThreads) void narrow_kernel(const ST *__restrict__ src, int64_t n, DT *__restrict__ dst)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) dst[i] = (DT)src[i];
}

__global__ __launch_bounds__(kThreads) void virtual_rows_kernel(int64_t *__restrict__ rows, const int64_t *__restrict__ cols, int64_t n,
                                                                int shift, int64_t nrows)
{
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e < n) rows[e] += (cols[e] >> shift) * nrows;
}

template <typename PT, typename CT>
__global__ __launch_bounds__(kThreads) void unpack_kernel(int rank, level_args a /* coord[] unused */, const int *__restrict__ lt_perm,
                                                          const void *const *__restrict__ pos_arr, const void *const *__restrict__ crd_arr,
                                                          const int64_t *__restrict__ npos, int64_t nvalues, int64_t *const *__restrict__ out)
{
    const int64_t p0 = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p0 >= nvalues) return;
    int64_t p = p0;
    for (int l = rank - 1; l >= 0; --l) {
        const int lt = lt_perm[l], dim = lt_perm[SP_MAX_RANK + l];
        if (lt == SP_DENSE) {
            out[dim][p0] = p % a.size[l];
            p = p / a.size[l];
        } else {
            out[dim][p0] = (int64_t)((const CT *)crd_arr[l])[p];
            const PT *pos = (const PT *)pos_arr[l];
            int64_t lo = 0, hi = npos[l] - 1;       // largest q with pos[q] <= p  (q < npos-1 because pos[last] > p)
            while (hi - lo > 1) {
                const int64_t mid = (lo + hi) >> 1;
                if ((int64_t)pos[mid] <= p) lo = mid; else hi = mid;
            }
            p = lo;
        }
    }
}

inline unsigned blocks_for(int64_t n) { return (unsigned)(n > 0 ? ceil_div(n, kThreads) : 1); }

}  // namespace

// =========================================================================================
void *sp_mem::get(size_t bytes) const
{
    if (alloc) return alloc(bytes, ctx);
    void *p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) return nullptr;
    return p;
}
void sp_mem::put(void *p) const
{
    if (!p) return;
    if (free_) free_(p, ctx); else (void)hipFree(p);
}

sp_status spmi_fill_zero(void *p, size_t bytes, hipStream_t st)
{
    if (bytes == 0) return SP_OK;
    const size_t nwords = (bytes + 3) / 4;      // allocations are padded to 16 bytes by the callers
    const unsigned nb = (unsigned)(nwords / kThreads + 1 < 4096 ? nwords / kThreads + 1 : 4096);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(nb), dim3(kThreads), 0, st, (uint32_t *)p, nwords);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

sp_status spmi_exclusive_scan(void *data, int64_t n, int bits, sp_scratch &tmp, hipStream_t st)
{
    if (bits == 32) return exclusive_scan_t<uint32_t>((uint32_t *)data, n, tmp, st);
    return exclusive_scan_t<unsigned long long>((unsigned long long *)data, n, tmp, st);
}

static size_t pad16(size_t b) { return (b + 15) & ~(size_t)15; }

static sp_status build_rowblocks_for(const void *pos, int pw, int64_t nrows, int64_t nnz, const sp_mem &mem, sp_rowblocks *out,
                                     hipStream_t st)
{
    if (nrows >= ((int64_t)1 << 31) - 1) return SP_OK;    // the streaming kernel keeps 32-bit row ids
    const int64_t nb = ceil_div(nnz, kSpmiStreamT);
    if (nb == 0) return SP_OK;
    void *start = mem.get(pad16((size_t)(nb + 1) * 4));
    void *carry = mem.get(pad16((size_t)nb * 8));
    if (!start || !carry) { mem.put(start); mem.put(carry); return SP_ERR_ALLOC; }
    if (pw == 32)
        hipLaunchKernelGGL(rowblocks_kernel<int32_t>, dim3(blocks_for(nb + 1)), dim3(kThreads), 0, st, (const int32_t *)pos, nrows, nb,
                           kSpmiStreamT, (int32_t *)start);
    else
        hipLaunchKernelGGL(rowblocks_kernel<int64_t>, dim3(blocks_for(nb + 1)), dim3(kThreads), 0, st, (const int64_t *)pos, nrows, nb,
                           kSpmiStreamT, (int32_t *)start);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { mem.put(start); mem.put(carry); g_last_hip_error = (int)e; return SP_ERR_HIP; }
    out->start = start;
    out->carry = carry;
    out->nblocks = nb;
    return SP_OK;
}

sp_status spmi_build_rowblocks(const sp_tensor *t, hipStream_t st)
{
    // only for rank 2 with a compressed innermost level
    if (t->enc.rank != 2 || t->enc.lt[1] != SP_COMPRESSED || t->rowblocks.start) return SP_OK;
    sp_mem mem{t->alloc, t->free_, t->ctx};
    return build_rowblocks_for(t->pos[1], t->enc.pw, t->npos[1] - 1, t->ncrd[1], mem, &t->rowblocks, st);
}

// A dense outer level with mostly empty segments (a CSR matrix with mostly empty rows): keep the list of the
// non-empty ones and their pos entries, so that the product kernels visit stored rows only, as they do for a
// compressed outer level.  crd and values are shared with the tensor's own arrays.
template <typename PT>
__global__ __launch_bounds__(kThreads) void mark_nonempty_kernel(const PT *__restrict__ pos, int64_t nrows, uint32_t *__restrict__ mark)
{
    const int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (r < nrows) mark[r] = pos[r + 1] > pos[r] ? 1u : 0u;
}

template <typename PT, typename CT>
__global__ __launch_bounds__(kThreads) void compact_rows_kernel(const PT *__restrict__ pos, int64_t nrows, const uint32_t *__restrict__ excl,
                                                                int64_t nz_rows, CT *__restrict__ nz_rowid, PT *__restrict__ nz_pos)
{
    const int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (r > nrows) return;
    if (r == nrows) { nz_pos[nz_rows] = pos[nrows]; return; }
    if (pos[r + 1] > pos[r]) { nz_rowid[excl[r]] = (CT)r; nz_pos[excl[r]] = pos[r]; }
}

// out (zero before) = the largest number of rows that one window of the streaming kernels meets
__global__ __launch_bounds__(kThreads) void max_span_kernel(const int32_t *__restrict__ rowblk, int64_t nb, unsigned long long *__restrict__ out)
{
    const int64_t b = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    unsigned long long span = b < nb ? (unsigned long long)(rowblk[b + 1] - rowblk[b]) : 0ull;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) { const unsigned long long o = __shfl_xor(span, d, 64); span = o > span ? o : span; }
    if ((threadIdx.x & 63) == 0 && span) atomicMax(out, span);
}

// The list of non-empty rows is built in two steps so that its questions to the device can share one synchronisation
// with whatever else the caller reads back: enqueue (marks, their scan, the longest run of rows in one window; the
// answers land in the probe once the stream has been synchronised), then decide (and compact, when worth it).
struct nonempty_probe {
    int64_t nrows = 0;
    unsigned long long nz = 0, span = 0;
    bool active = false;
    // the answers come back inside the builder's 64-byte flags block (one copy to the host for everything):
    // ints 8-9 = the number of non-empty rows, ints 10-11 = the longest run, both as 64-bit values
    void take(const int *h) { memcpy(&nz, &h[8], 8); memcpy(&span, &h[10], 8); }
};

// *out += the number of rows that hold something: grid-stride count per thread, wave and block reduction, one atomic per block
template <typename PT>
__global__ __launch_bounds__(kThreads) void count_nonempty_kernel(const PT *__restrict__ pos, int64_t nrows, unsigned long long *__restrict__ out)
{
    __shared__ unsigned long long wsum[kThreads / 64];
    unsigned long long c = 0;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nrows; i += (int64_t)gridDim.x * kThreads) c += pos[i + 1] > pos[i] ? 1u : 0u;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) c += __shfl_xor(c, d, 64);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kThreads / 64; ++w) c += wsum[w];
        if (c) atomicAdd(out, c);
    }
}

// flags: the 64 zeroed device bytes of the build (see nonempty_probe for the slots used here)
static sp_status nonempty_enqueue(const sp_tensor *t, hipStream_t st, int *flags, nonempty_probe &q)
{
    if (t->enc.rank != 2 || t->enc.lt[0] != SP_DENSE || t->enc.lt[1] != SP_COMPRESSED) return SP_OK;
    const int64_t nrows = t->npos[1] - 1;
    if (nrows < 4096 || nrows >= ((int64_t)1 << 31) - 1 || t->ncrd[1] == 0) return SP_OK;
    const unsigned cnt_blocks = blocks_for(nrows) < 256u ? blocks_for(nrows) : 256u;
    if (t->enc.pw == 32)
        hipLaunchKernelGGL(count_nonempty_kernel<int32_t>, dim3(cnt_blocks), dim3(kThreads), 0, st, (const int32_t *)t->pos[1], nrows,
                           (unsigned long long *)(flags + 8));
    else
        hipLaunchKernelGGL(count_nonempty_kernel<int64_t>, dim3(cnt_blocks), dim3(kThreads), 0, st, (const int64_t *)t->pos[1], nrows,
                           (unsigned long long *)(flags + 8));
    SP_HIP(hipGetLastError());
    if (t->rowblocks.start) {
        hipLaunchKernelGGL(max_span_kernel, dim3(blocks_for(t->rowblocks.nblocks)), dim3(kThreads), 0, st, (const int32_t *)t->rowblocks.start,
                           t->rowblocks.nblocks, (unsigned long long *)(flags + 10));
        SP_HIP(hipGetLastError());
    }
    q.nrows = nrows; q.active = true;
    return SP_OK;
}

// after the stream has been synchronised; *launched = kernels were enqueued (they use a temporary of `tmp`: synchronise
// before it goes)
static sp_status nonempty_decide(const sp_tensor *t, sp_scratch &tmp, hipStream_t st, const nonempty_probe &q, bool *launched)
{
    *launched = false;
    if (!q.active) return SP_OK;
    const int64_t nrows = q.nrows;
    const int64_t nz = (int64_t)q.nz;
    // not worth it when at least half of the rows hold something, unless one window of the streaming kernels would have to walk
    // over a very long run of empty rows all by itself
    if (nz * 2 > nrows && q.span < 65536) return SP_OK;
    sp_mem mem{t->alloc, t->free_, t->ctx};
    const int ps = t->enc.pw / 8, cs = t->enc.cw / 8;
    void *rid = mem.get(pad16((size_t)(nz > 0 ? nz : 1) * cs));
    void *npos = mem.get(pad16((size_t)(nz + 1) * ps));
    uint32_t *mark = (uint32_t *)tmp.get((size_t)nrows * 4);
    if (!rid || !npos || !mark) { mem.put(rid); mem.put(npos); return SP_ERR_ALLOC; }
    *launched = true;
    if (t->enc.pw == 32)
        hipLaunchKernelGGL(mark_nonempty_kernel<int32_t>, dim3(blocks_for(nrows)), dim3(kThreads), 0, st, (const int32_t *)t->pos[1], nrows, mark);
    else
        hipLaunchKernelGGL(mark_nonempty_kernel<int64_t>, dim3(blocks_for(nrows)), dim3(kThreads), 0, st, (const int64_t *)t->pos[1], nrows, mark);
    sp_status ss = hipGetLastError() == hipSuccess ? spmi_exclusive_scan(mark, nrows, 32, tmp, st) : SP_ERR_HIP;
    if (ss != SP_OK) { mem.put(rid); mem.put(npos); return ss; }
#define SPMI_COMPACT(PT, CT)                                                                                                  \
    hipLaunchKernelGGL((compact_rows_kernel<PT, CT>), dim3(blocks_for(nrows + 1)), dim3(kThreads), 0, st, (const PT *)t->pos[1], nrows, \
                       (const uint32_t *)mark, nz, (CT *)rid, (PT *)npos)
    if (t->enc.pw == 32 && t->enc.cw == 32) SPMI_COMPACT(int32_t, int32_t);
    else if (t->enc.pw == 32) SPMI_COMPACT(int32_t, int64_t);
    else if (t->enc.cw == 32) SPMI_COMPACT(int64_t, int32_t);
    else SPMI_COMPACT(int64_t, int64_t);
#undef SPMI_COMPACT
    hipError_t e = hipGetLastError();
    sp_status s = e == hipSuccess ? build_rowblocks_for(npos, t->enc.pw, nz, t->ncrd[1], mem, &t->nz_rowblocks, st) : SP_ERR_HIP;
    if (s != SP_OK) { mem.put(rid); mem.put(npos); if (e != hipSuccess) g_last_hip_error = (int)e; return s; }
    t->nz_rowid = rid; t->nz_pos = npos; t->nz_rows = nz;
    return SP_OK;
}

static sp_status build_nonempty_rows(const sp_tensor *t, sp_scratch &tmp, hipStream_t st)
{
    int *flags = (int *)tmp.get(64);
    if (!flags) return SP_ERR_ALLOC;
    SP_TRY(spmi_fill_zero(flags, 64, st));
    nonempty_probe q;
    SP_TRY(nonempty_enqueue(t, st, flags, q));
    if (!q.active) return SP_OK;
    int h[16];
    SP_HIP(hipMemcpyAsync(h, flags, sizeof(h), hipMemcpyDeviceToHost, st));
    SP_HIP(hipStreamSynchronize(st));
    q.take(h);
    bool launched = false;
    return nonempty_decide(t, tmp, st, q, &launched);
}

// Column-segmented copy of a CSR tensor (see sp_segments): entries keyed by (panel, row, column) and packed
// again as a CSR over panels*nrows virtual rows, through the coordinate scheme like any other conversion.
static void free_segments(const sp_tensor *t)
{
    if (!t->segments) return;
    sp_mem mem{t->alloc, t->free_, t->ctx};
    mem.put(t->segments->partial);
    sp_tensor_free(t->segments->seg);
    delete t->segments;
    t->segments = nullptr;
}

// `slice_bytes`: how many bytes of the dense operand one panel may cover (a power-of-two number of its rows
// is taken).  The handle keeps one segmented copy; asking for another panel width rebuilds it.
sp_status spmi_build_segments(const sp_tensor *A, int64_t row_bytes, int64_t slice_bytes, hipStream_t st)
{
    if (A->enc.rank != 2 || A->enc.lt[0] != SP_DENSE || A->enc.lt[1] != SP_COMPRESSED || A->enc.perm[0] != 0) return SP_ERR_UNSUPPORTED;
    const int64_t nrows = A->shape[0], n = A->shape[1];
    const int vbytes = A->dtype == SP_F64 ? 8 : 4;
    int shift = 0;
    while (((int64_t)2 << shift) * row_bytes <= slice_bytes) ++shift;       // widest power-of-two panel within the budget
    if (A->segments && A->segments->shift == shift) return SP_OK;
    const int64_t panels = ceil_div(n, (int64_t)1 << shift);
    if (panels < 2 || panels * nrows >= ((int64_t)1 << 31) - 1) return SP_ERR_UNSUPPORTED;
    if (hipStreamSynchronize(st) != hipSuccess) return SP_ERR_HIP;          // an older copy may still be in use
    free_segments(A);
    sp_mem mem{A->alloc, A->free_, A->ctx};
    sp_tensor *S = nullptr;
    {
        sp_scratch tmp(mem);
        const size_t cnt = (size_t)(A->nvalues > 0 ? A->nvalues : 1);
        int64_t *rows = (int64_t *)tmp.get(cnt * 8);
        int64_t *cols = (int64_t *)tmp.get(cnt * 8);
        void *vals = tmp.get(cnt * 8);
        if (!rows || !cols || !vals) return SP_ERR_ALLOC;
        int64_t *coords[2] = {rows, cols};
        SP_TRY(sp_unpack(A, coords, vals, st));
        hipLaunchKernelGGL(virtual_rows_kernel, dim3(blocks_for(A->nvalues)), dim3(kThreads), 0, st, rows, (const int64_t *)cols,
                           A->nvalues, shift, nrows);
        SP_HIP(hipGetLastError());
        sp_encoding enc = A->enc;
        enc.pw_store = enc.pw; enc.cw_store = enc.cw;     // an internal copy: working widths only
        const int64_t shape[2] = {panels * nrows, n};
        const int64_t *ccoords[2] = {rows, cols};
        SP_TRY(sp_pack(&enc, shape, A->nvalues, ccoords, vals, (sp_dtype)A->dtype, A->alloc, A->free_, A->ctx, st, &S));
    }
    void *partial = mem.get(pad16((size_t)(panels * nrows) * vbytes));
    if (!partial) { sp_tensor_free(S); return SP_ERR_ALLOC; }
    sp_segments *g = new sp_segments();
    g->seg = S; g->panels = (int)panels; g->shift = shift; g->nrows = nrows; g->partial = partial;
    A->segments = g;
    return SP_OK;
}

// ---- how scattered the innermost coordinates are -------------------------------------------
template <typename CT>
__global__ __launch_bounds__(kThreads) void count_jumps_kernel(const CT *__restrict__ crd, int64_t n, unsigned long long *__restrict__ out)
{
    __shared__ unsigned int wsum[kThreads / 64];
    unsigned int mine = 0;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e + 1 < n; e += stride)
        mine += (uint64_t)((int64_t)crd[e + 1] - (int64_t)crd[e]) >= 16u ? 1u : 0u;      // a step back (next segment) counts as well
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) mine += __shfl_xor(mine, d, 64);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = mine;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned int tot = 0;
        for (int w = 0; w < kThreads / 64; ++w) tot += wsum[w];
        if (tot) atomicAdd(out, (unsigned long long)tot);
    }
}

sp_status spmi_column_scatter(const sp_tensor *A, hipStream_t st, double *share)
{
    const int last = A->enc.rank - 1;
    if (A->scatter < 0) {
        const int64_t n = A->enc.lt[last] == SP_COMPRESSED ? A->ncrd[last] : 0;
        if (n < 2) A->scatter = 0;
        else {
            sp_mem mem{A->alloc, A->free_, A->ctx};
            sp_scratch tmp(mem);
            unsigned long long *cnt = (unsigned long long *)tmp.get(64);
            if (!cnt) return SP_ERR_ALLOC;
            SP_TRY(spmi_fill_zero(cnt, 64, st));
            const unsigned nb = blocks_for(n) < 4096u ? blocks_for(n) : 4096u;
            if (A->enc.cw == 32)
                hipLaunchKernelGGL(count_jumps_kernel<int32_t>, dim3(nb), dim3(kThreads), 0, st, (const int32_t *)A->crd[last], n, cnt);
            else
                hipLaunchKernelGGL(count_jumps_kernel<int64_t>, dim3(nb), dim3(kThreads), 0, st, (const int64_t *)A->crd[last], n, cnt);
            SP_HIP(hipGetLastError());
            unsigned long long h = 0;
            SP_HIP(hipMemcpyAsync(&h, cnt, 8, hipMemcpyDeviceToHost, st));
            SP_HIP(hipStreamSynchronize(st));
            A->scatter = (double)h / (double)(n - 1);
        }
    }
    *share = A->scatter;
    return SP_OK;
}

// ---- binned copy (see sp_bins) ------------------------------------------------------------
static void free_bins(const sp_tensor *t)
{
    if (!t->bins) return;
    sp_mem mem{t->alloc, t->free_, t->ctx};
    mem.put(t->bins->val); mem.put(t->bins->prod); mem.put(t->bins->lcol); mem.put(t->bins->lrow); mem.put(t->bins->gdst);
    mem.put(t->bins->pstart); mem.put(t->bins->rbstart);
    delete t->bins;
    t->bins = nullptr;
}

// key = (((stored row << pshift) | column inside the panel) << pbits) | panel, pbits a multiple of 8.  The entries come in storage order (rows, then
// columns, ascending), so a STABLE sort by the low pbits alone (one pass for up to 256 panels) gives panel-major buckets with
// rows, then columns, ascending inside.  Block = 1024 consecutive entries: the rows they belong to are a short range of pos,
// found by two searches per block and then searched per entry inside the LDS (a search of all of pos per entry took 4x longer).
constexpr int kBinKeyTile = 1024, kBinKeyRows = 1024;
template <typename PT, typename CT>
__global__ __launch_bounds__(kThreads) void bin_keys_kernel(const PT *__restrict__ pos, int64_t nrows, const CT *__restrict__ crd, int64_t n,
                                                            int pshift, int pbits, uint64_t *__restrict__ keys)
{
    __shared__ int64_t s_row[2];
    __shared__ int64_t spos[kBinKeyRows];
    const int64_t e0 = (int64_t)blockIdx.x * kBinKeyTile, e1 = e0 + kBinKeyTile < n ? e0 + kBinKeyTile : n;
    auto row_of = [&](int64_t e, int64_t lo, int64_t hi) -> int64_t {      // last row q in [lo, hi] with pos[q] <= e (of empty rows the last one wins)
        while (lo < hi) {
            const int64_t mid = lo + (hi - lo + 1) / 2;
            if ((int64_t)pos[mid] <= e) lo = mid;
            else hi = mid - 1;
        }
        return lo;
    };
    if (threadIdx.x < 2) s_row[threadIdx.x] = row_of(threadIdx.x == 0 ? e0 : e1 - 1, 0, nrows - 1);
    __syncthreads();
    const int64_t r0 = s_row[0], r1 = s_row[1], nr = r1 - r0 + 1;
    const bool staged = nr <= kBinKeyRows;
    if (staged) for (int64_t i = threadIdx.x; i < nr; i += kThreads) spos[i] = (int64_t)pos[r0 + i];
    __syncthreads();
    for (int64_t e = e0 + threadIdx.x; e < e1; e += kThreads) {
        int64_t row;
        if (staged) {
            int64_t lo = 0, hi = nr - 1;
            while (lo < hi) {
                const int64_t mid = lo + (hi - lo + 1) / 2;
                if (spos[mid] <= e) lo = mid;
                else hi = mid - 1;
            }
            row = r0 + lo;
        } else {
            row = row_of(e, r0, r1);
        }
        const uint64_t c = (uint64_t)crd[e];
        keys[e] = (((((uint64_t)row) << pshift) | (c & (((uint64_t)1 << pshift) - 1))) << pbits) | (c >> pshift);
    }
}

// bucket (panel * rowblocks + row block) of a key; *row_out = its row
__device__ inline int64_t bin_bucket_of(uint64_t key, int pshift, int pbits, int rshift, int64_t rowblocks, uint64_t *row_out)
{
    const uint64_t p = key & (((uint64_t)1 << pbits) - 1);
    const uint64_t row = key >> (pbits + pshift);
    if (row_out) *row_out = row;
    return (int64_t)(p * (uint64_t)rowblocks + (row >> rshift));
}

// Padded bucket sizes (multiples of 8 entries) in both orders: pcnt[panel * rowblocks + rb] and rcnt[rb * panels + panel];
// one more element, zero, at the end of each, so that the exclusive scans also give the total.
__global__ __launch_bounds__(kThreads) void bin_padded_sizes_kernel(const int64_t *__restrict__ off, int64_t panels, int64_t rowblocks,
                                                                    uint64_t *__restrict__ pcnt, uint64_t *__restrict__ rcnt)
{
    const int64_t b = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t nbuckets = panels * rowblocks;
    if (b > nbuckets) return;
    if (b == nbuckets) { pcnt[b] = 0; rcnt[b] = 0; return; }
    const uint64_t sz = (uint64_t)((off[b + 1] - off[b] + 7) & ~(int64_t)7);
    const int64_t p = b / rowblocks, rb = b - p * rowblocks;
    pcnt[b] = sz;
    rcnt[rb * panels + p] = sz;
}

// From the sorted keys: every entry to its place in the padded panel-major arrays (value bits, column inside the panel) and
// in the padded row-block-major array of rows inside the row block.  The padding keeps what the arrays were filled with.
template <typename W>
__global__ __launch_bounds__(kThreads) void bin_place_kernel(const uint64_t *__restrict__ keys, const W *__restrict__ vals, int64_t n, int pshift,
                                                             int pbits, int rshift, int64_t panels, int64_t rowblocks,
                                                             const int64_t *__restrict__ off, const uint64_t *__restrict__ poff,
                                                             const uint64_t *__restrict__ roff, W *__restrict__ val,
                                                             uint16_t *__restrict__ lcol, uint16_t *__restrict__ lrow)
{
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= n) return;
    const uint64_t key = keys[e];
    uint64_t row;
    const int64_t b = bin_bucket_of(key, pshift, pbits, rshift, rowblocks, &row);
    const int64_t p = b / rowblocks, rb = b - p * rowblocks;
    const int64_t i = e - off[b];
    const uint64_t d = poff[b] + (uint64_t)i;
    val[d] = vals[e];
    lcol[d] = (uint16_t)((key >> pbits) & (((uint64_t)1 << pshift) - 1));
    lrow[roff[rb * panels + p] + (uint64_t)i] = (uint16_t)(row & (((uint64_t)1 << rshift) - 1));
}

// Thread = bucket: where each of its groups of 8 products goes in the row-block-major array (in groups); thread b < panels + 1
// and b < rowblocks + 1 also write where panel b / row block b start (in entries).
__global__ __launch_bounds__(kThreads) void bin_groups_kernel(int64_t panels, int64_t rowblocks, const uint64_t *__restrict__ poff,
                                                              const uint64_t *__restrict__ roff, uint32_t *__restrict__ gdst,
                                                              int64_t *__restrict__ pstart, int64_t *__restrict__ rbstart)
{
    const int64_t b = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t nbuckets = panels * rowblocks;
    if (b <= panels) pstart[b] = (int64_t)poff[b * rowblocks];
    if (b <= rowblocks) rbstart[b] = (int64_t)roff[b * panels];
    if (b >= nbuckets) return;
    const int64_t p = b / rowblocks, rb = b - p * rowblocks;
    const uint64_t g0 = poff[b] >> 3, g1 = poff[b + 1] >> 3, r0 = roff[rb * panels + p] >> 3;
    for (uint64_t g = g0; g < g1; ++g) gdst[g] = (uint32_t)(r0 + (g - g0));
}

__global__ __launch_bounds__(kThreads) void fill_u16_kernel(uint16_t *__restrict__ p, int64_t n, uint16_t v)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) p[i] = v;
}

// off[b] = number of entries in buckets before b (the bucket of a key never decreases along the sorted keys), for
// b = 0 .. nbuckets: a binary search per bucket, whatever the sizes of the buckets are.
__global__ __launch_bounds__(kThreads) void bin_offsets_kernel(const uint64_t *__restrict__ keys, int64_t n, int pshift, int pbits, int rshift,
                                                               int64_t rowblocks, int64_t nbuckets,
                                                               int64_t *__restrict__ off)
{
    const int64_t b = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (b > nbuckets) return;
    int64_t lo = 0, hi = n;                            // first entry whose bucket is >= b
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (bin_bucket_of(keys[mid], pshift, pbits, rshift, rowblocks, nullptr) < b) lo = mid + 1;
        else hi = mid;
    }
    off[b] = lo;
}

// Builds and keeps the binned copy of a row-major tensor with a compressed innermost level; no-op when it exists.
// Synchronises.  Rows are counted among the stored ones (all of them for CSR; the compressed outer level's for DCSR;
// the non-empty ones where the tensor carries their list), the caller maps them back.  SP_ERR_UNSUPPORTED for other
// encodings, for an empty tensor and when the bucket table would be larger than the tensor itself.
sp_status spmi_build_bins(const sp_tensor *A, hipStream_t st)
{
    if (A->bins) return SP_OK;
    if (A->enc.rank != 2 || A->enc.lt[1] != SP_COMPRESSED || A->enc.perm[0] != 0) return SP_ERR_UNSUPPORTED;
    const bool listed = A->enc.lt[0] == SP_DENSE && A->nz_pos;
    const void *pos = listed ? A->nz_pos : A->pos[1];
    const int64_t m = listed ? A->nz_rows : A->npos[1] - 1;          // stored rows
    const int64_t n = A->shape[1], nnz = A->ncrd[1];
    const int pshift = kSpmiBinPanelShift, rshift = kSpmiBinRowShift;
    const int64_t panels = ceil_div(n, (int64_t)1 << pshift), rowblocks = ceil_div(m, (int64_t)1 << rshift);
    if (nnz < 1 || m < 1 || panels > 0x7fffffff || rowblocks > 0x7fffffff) return SP_ERR_UNSUPPORTED;
    const unsigned __int128 nb128 = (unsigned __int128)panels * (unsigned __int128)rowblocks;
    if (nb128 > (unsigned __int128)nnz + 4096) return SP_ERR_UNSUPPORTED;
    const int64_t nbuckets = (int64_t)nb128;
    const int vbytes = A->dtype == SP_F64 ? 8 : 4;
    int pbits = 0, mbits = 0;
    while (((int64_t)1 << pbits) < panels) ++pbits;
    pbits = (pbits + 7) & ~7;                        // the sort works on whole 8-bit digits: the panel gets digits of its own
    while (mbits < 63 && ((int64_t)1 << mbits) < m) ++mbits;
    if (mbits + pshift + pbits > 63) return SP_ERR_UNSUPPORTED;
    sp_mem mem{A->alloc, A->free_, A->ctx};
    sp_bins *g = new sp_bins();
    A->bins = g;                                         // owned from here on: free_bins() releases whatever was allocated
    g->nnz = nnz; g->nrows = m; g->panels = (int)panels; g->rowblocks = (int)rowblocks;
    // pieces per panel in the first pass: about 32768 entries each, so that loading the slice of x stays a small part
    const int64_t per_panel = nnz / panels;
    g->pieces = (int)(per_panel / 32768 < 1 ? 1 : per_panel / 32768 > 64 ? 64 : per_panel / 32768);
    while (panels * g->pieces < 512 && per_panel / (2 * g->pieces) >= 4096) g->pieces *= 2;      // enough blocks for every CU
    sp_status status = SP_OK;
    auto build = [&]() -> sp_status {
        sp_scratch tmp(mem);
        uint64_t *keys = (uint64_t *)tmp.get((size_t)nnz * 8);
        int64_t *off = (int64_t *)tmp.get((size_t)(nbuckets + 1) * 8);
        uint64_t *poff = (uint64_t *)tmp.get((size_t)(nbuckets + 1) * 8), *roff = (uint64_t *)tmp.get((size_t)(nbuckets + 1) * 8);
        if (!keys || !off || !poff || !roff) return SP_ERR_ALLOC;
#define SPMI_BIN_KEYS(PT, CT)                                                                                                 \
    hipLaunchKernelGGL((bin_keys_kernel<PT, CT>), dim3((unsigned)ceil_div(nnz, kBinKeyTile)), dim3(kThreads), 0, st, (const PT *)pos, m,    \
                       (const CT *)A->crd[1], nnz, pshift, pbits, keys)
        if (A->enc.pw == 32 && A->enc.cw == 32) SPMI_BIN_KEYS(int32_t, int32_t);
        else if (A->enc.pw == 32) SPMI_BIN_KEYS(int32_t, int64_t);
        else if (A->enc.cw == 32) SPMI_BIN_KEYS(int64_t, int32_t);
        else SPMI_BIN_KEYS(int64_t, int64_t);
#undef SPMI_BIN_KEYS
        SP_HIP(hipGetLastError());
        uint64_t *sorted_keys = nullptr;
        const void *sorted_vals = nullptr;
        // stable, on the panel bits alone: one pass for up to 256 panels
        SP_TRY(spmi_radix_sort_pairs(keys, A->values, vbytes, nnz, pbits, tmp, st, &sorted_keys, &sorted_vals));
        hipLaunchKernelGGL(bin_offsets_kernel, dim3(blocks_for(nbuckets + 1)), dim3(kThreads), 0, st, (const uint64_t *)sorted_keys, nnz, pshift,
                           pbits, rshift, rowblocks, nbuckets, off);
        hipLaunchKernelGGL(bin_padded_sizes_kernel, dim3(blocks_for(nbuckets + 1)), dim3(kThreads), 0, st, (const int64_t *)off, panels, rowblocks,
                           poff, roff);
        SP_HIP(hipGetLastError());
        SP_TRY(spmi_exclusive_scan(poff, nbuckets + 1, 64, tmp, st));
        SP_TRY(spmi_exclusive_scan(roff, nbuckets + 1, 64, tmp, st));
        uint64_t total = 0;
        SP_HIP(hipMemcpyAsync(&total, poff + nbuckets, 8, hipMemcpyDeviceToHost, st));
        SP_HIP(hipStreamSynchronize(st));
        const int64_t np = (int64_t)total;                       // entries with every bucket padded to a multiple of 8
        if (np < nnz || np > nnz + 7 * nbuckets || (np >> 3) > 0xffffffffll) return SP_ERR_UNSUPPORTED;
        g->np = np;
        g->val = mem.get(pad16((size_t)np * vbytes));
        g->prod = mem.get(pad16((size_t)np * vbytes));
        g->lcol = (uint16_t *)mem.get(pad16((size_t)np * 2));
        g->lrow = (uint16_t *)mem.get(pad16((size_t)np * 2));
        g->gdst = (uint32_t *)mem.get(pad16((size_t)(np / 8) * 4));
        g->pstart = (int64_t *)mem.get(pad16((size_t)(panels + 1) * 8));
        g->rbstart = (int64_t *)mem.get(pad16((size_t)(rowblocks + 1) * 8));
        if (!g->val || !g->prod || !g->lcol || !g->lrow || !g->gdst || !g->pstart || !g->rbstart) return SP_ERR_ALLOC;
        // padding: value 0 times the zero that the first pass keeps behind its slice of x (column 2^pshift), added to row 0
        SP_TRY(spmi_fill_zero(g->val, pad16((size_t)np * vbytes), st));
        SP_TRY(spmi_fill_zero(g->lrow, pad16((size_t)np * 2), st));
        hipLaunchKernelGGL(fill_u16_kernel, dim3(blocks_for(np)), dim3(kThreads), 0, st, g->lcol, np, (uint16_t)((1 << pshift)));
        if (vbytes == 8)
            hipLaunchKernelGGL(bin_place_kernel<unsigned long long>, dim3(blocks_for(nnz)), dim3(kThreads), 0, st, (const uint64_t *)sorted_keys,
                               (const unsigned long long *)sorted_vals, nnz, pshift, pbits, rshift, panels, rowblocks, (const int64_t *)off,
                               (const uint64_t *)poff, (const uint64_t *)roff, (unsigned long long *)g->val, g->lcol, g->lrow);
        else
            hipLaunchKernelGGL(bin_place_kernel<uint32_t>, dim3(blocks_for(nnz)), dim3(kThreads), 0, st, (const uint64_t *)sorted_keys,
                               (const uint32_t *)sorted_vals, nnz, pshift, pbits, rshift, panels, rowblocks, (const int64_t *)off,
                               (const uint64_t *)poff, (const uint64_t *)roff, (uint32_t *)g->val, g->lcol, g->lrow);
        const int64_t most = std::max(nbuckets, std::max(panels, rowblocks) + 1);
        hipLaunchKernelGGL(bin_groups_kernel, dim3(blocks_for(most)), dim3(kThreads), 0, st, panels, rowblocks, (const uint64_t *)poff,
                           (const uint64_t *)roff, g->gdst, g->pstart, g->rbstart);
        SP_HIP(hipGetLastError());
        SP_HIP(hipStreamSynchronize(st));
        return SP_OK;
    };
    if (status == SP_OK) status = build();
    if (status != SP_OK) { (void)hipStreamSynchronize(st); free_bins(A); }
    return status;
}

static void release_tensor_arrays(sp_tensor *t)
{
    sp_mem mem{t->alloc, t->free_, t->ctx};
    for (int l = 0; l < SP_MAX_RANK; ++l) {
        mem.put(t->pos[l]); mem.put(t->crd[l]); mem.put(t->pos_narrow[l]); mem.put(t->crd_narrow[l]);
        t->pos[l] = t->crd[l] = t->pos_narrow[l] = t->crd_narrow[l] = nullptr;
    }
    mem.put(t->values); t->values = nullptr;
    mem.put(t->rowblocks.start); t->rowblocks.start = nullptr;
    mem.put(t->rowblocks.carry); t->rowblocks.carry = nullptr;
    mem.put(t->dense_partial); t->dense_partial = nullptr; t->dense_partial_bytes = 0;
    mem.put(t->spmm_carry); t->spmm_carry = nullptr; t->spmm_carry_bytes = 0;
    mem.put(t->sddmm_bt); t->sddmm_bt = nullptr; t->sddmm_bt_bytes = 0;
    mem.put(t->mttkrp_windows); t->mttkrp_windows = nullptr;
    mem.put(t->mttkrp_carry); t->mttkrp_carry = nullptr; t->mttkrp_carry_bytes = 0;
    for (int w = 0; w < 2; ++w) { mem.put(t->mttkrp_pad[w]); t->mttkrp_pad[w] = nullptr; t->mttkrp_pad_bytes[w] = 0; }
    mem.put(t->nz_rowid); mem.put(t->nz_pos); mem.put(t->nz_rowblocks.start); mem.put(t->nz_rowblocks.carry);
    t->nz_rowid = t->nz_pos = t->nz_rowblocks.start = t->nz_rowblocks.carry = nullptr;
}

extern "C" void sp_tensor_free(sp_tensor *t)
{
    if (!t) return;
    if (t->transposed) sp_tensor_free(t->transposed);
    free_segments(t);
    free_bins(t);
    release_tensor_arrays(t);
    if (t->prof_events) {
        for (hipEvent_t e : *t->prof_events) (void)hipEventDestroy(e);
        delete t->prof_events;
    }
    delete t;
}

// The same for the innermost level of a format whose levels above are all dense (CSR, CSC and their kin of any rank): every
// entry is its own child, its parent is the key divided by the level's size.  Four consecutive entries per thread, their keys
// and the two neighbours loaded once, the four coordinates written with one store.
template <typename PT, typename CT>
__global__ __launch_bounds__(kThreads) void emit_inner_kernel(const uint64_t *__restrict__ keys, int64_t nnz, divisor size, PT *__restrict__ cnt,
                                                              CT *__restrict__ crd, int *__restrict__ dup_flags)
{
    typedef unsigned long long u2 __attribute__((ext_vector_type(2)));
    typedef typename std::conditional<sizeof(PT) == 8, unsigned long long, unsigned int>::type UT;
    const int64_t e0 = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4;
    if (e0 >= nnz) return;
    uint64_t k[6];                                       // k[1..4] = the thread's keys, k[0] and k[5] the neighbours
    const bool whole = e0 + 4 <= nnz;
    if (whole) {
        const u2 a = *(const u2 *)(keys + e0), b = *(const u2 *)(keys + e0 + 2);
        k[1] = a[0]; k[2] = a[1]; k[3] = b[0]; k[4] = b[1];
    } else {
        for (int i = 0; i < 4; ++i) k[1 + i] = e0 + i < nnz ? keys[e0 + i] : 0;
    }
    k[0] = e0 > 0 ? keys[e0 - 1] : 0;
    k[5] = e0 + 4 < nnz ? keys[e0 + 4] : 0;
    uint64_t up[6];
#pragma unroll
    for (int i = 0; i < 6; ++i) up[i] = div_by(k[i], size);
    CT c[4];
    bool dup = false;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t e = e0 + i;
        c[i] = (CT)(k[1 + i] - up[1 + i] * size.d);
        if (e < nnz) {
            dup |= e > 0 && k[1 + i] == k[i];
            const bool head = e == 0 || up[i] != up[1 + i];
            const bool tail = e == nnz - 1 || up[2 + i] != up[1 + i];
            // children of a parent = (last child + 1) - first child: integer atomics, so the order does not matter
            if (head && tail) atomicAdd((UT *)&cnt[up[1 + i]], (UT)1);
            else if (tail) atomicAdd((UT *)&cnt[up[1 + i]], (UT)(e + 1));
            else if (head) atomicAdd((UT *)&cnt[up[1 + i]], (UT)0 - (UT)e);
        }
    }
    if (dup_flags && dup) atomicOr(&dup_flags[1], 1);
    if (whole && sizeof(CT) == 4) {
        typedef unsigned int u4 __attribute__((ext_vector_type(4)));
        *(u4 *)(crd + e0) = u4{(unsigned)c[0], (unsigned)c[1], (unsigned)c[2], (unsigned)c[3]};
    } else {
        for (int i = 0; i < 4; ++i) if (e0 + i < nnz) crd[e0 + i] = c[i];
    }
}

template <typename PT, typename CT>
static sp_status launch_emit(const uint64_t *keys, int64_t nnz, divisor stride, divisor size, const uint32_t *child_excl,
                             const uint64_t *pin, uint64_t *pout, void *cnt, void *crd, int *dup_flags, hipStream_t st)
{
    if (!child_excl && !pin && !pout && stride.d == 1)
        hipLaunchKernelGGL((emit_inner_kernel<PT, CT>), dim3(blocks_for((nnz + 3) / 4)), dim3(kThreads), 0, st, keys, nnz, size, (PT *)cnt, (CT *)crd,
                           dup_flags);
    else
        hipLaunchKernelGGL((emit_level_kernel<PT, CT>), dim3(blocks_for(nnz)), dim3(kThreads), 0, st, keys, nnz, stride, size, child_excl,
                           pin, pout, (PT *)cnt, (CT *)crd, dup_flags);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

// The tables a finished storage carries for the product kernels: longest innermost segment (kernel choice), the row
// blocks of the streaming kernels, the list of non-empty rows of a mostly empty CSR.  flags: 64 device bytes, the
// second half zero.  Synchronises.  input_flags (HOST int[2], may be null) receives flags[0..1], the input checks of
// the storage builder, read back together with the maximum; when one is set nothing more is built.
sp_status spmi_finish_tensor(sp_tensor *t, int *flags, sp_scratch &tmp, hipStream_t st, int *input_flags)
{
    const sp_encoding *enc = &t->enc;
    const int rank = enc->rank;
    const bool want_max = enc->lt[rank - 1] == SP_COMPRESSED && t->npos[rank - 1] > 1;
    if (want_max) {
        unsigned long long *mx = (unsigned long long *)(flags + 4);
        const int64_t nseg = t->npos[rank - 1] - 1;
        const unsigned seg_blocks = blocks_for(nseg) < 256u ? blocks_for(nseg) : 256u;      // one atomic per block, all to one address: few blocks
        if (enc->pw == 32)
            hipLaunchKernelGGL(max_segment_kernel<int32_t>, dim3(seg_blocks), dim3(kThreads), 0, st, (const int32_t *)t->pos[rank - 1], nseg, mx);
        else
            hipLaunchKernelGGL(max_segment_kernel<int64_t>, dim3(seg_blocks), dim3(kThreads), 0, st, (const int64_t *)t->pos[rank - 1], nseg, mx);
        SP_HIP(hipGetLastError());
    }
    // everything that can be enqueued before the host has to look at an answer: the row blocks and the questions of the
    // non-empty-rows list (all in bounds whatever the input checks say), then one synchronisation for all read-backs
    SP_TRY(spmi_build_rowblocks(t, st));
    nonempty_probe q;
    SP_TRY(nonempty_enqueue(t, st, flags, q));
    int h[16] = {0};
    if (want_max || input_flags || q.active) SP_HIP(hipMemcpyAsync(h, flags, sizeof(h), hipMemcpyDeviceToHost, st));
    SP_HIP(hipStreamSynchronize(st));
    q.take(h);
    if (input_flags) {
        input_flags[0] = h[0];
        input_flags[1] = h[1];
        if (h[0] || h[1]) return SP_OK;
    }
    unsigned long long hmx = 0;
    memcpy(&hmx, &h[4], 8);
    if (want_max) t->max_segment = (int64_t)hmx;
    bool launched = false;
    SP_TRY(nonempty_decide(t, tmp, st, q, &launched));
    if (launched) SP_HIP(hipStreamSynchronize(st));
    return SP_OK;
}

// *out (DEVICE, zero before the call) = the longest of the nseg segments of a pos array of width pw; enqueued only.
sp_status spmi_max_segment_async(const void *pos, int pw, int64_t nseg, unsigned long long *out, hipStream_t st)
{
    if (nseg <= 0) return SP_OK;
    const unsigned seg_blocks = blocks_for(nseg) < 256u ? blocks_for(nseg) : 256u;      // one atomic per block, all to one address: few blocks
    if (pw == 32) hipLaunchKernelGGL(max_segment_kernel<int32_t>, dim3(seg_blocks), dim3(kThreads), 0, st, (const int32_t *)pos, nseg, out);
    else hipLaunchKernelGGL(max_segment_kernel<int64_t>, dim3(seg_blocks), dim3(kThreads), 0, st, (const int64_t *)pos, nseg, out);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

sp_status spmi_ensure_tables(const sp_tensor *t, hipStream_t st)
{
    if (!t->tables_pending) return SP_OK;
    sp_mem mem{t->alloc, t->free_, t->ctx};
    sp_scratch tmp(mem);
    SP_TRY(spmi_build_rowblocks(t, st));
    SP_TRY(build_nonempty_rows(t, tmp, st));
    SP_HIP(hipStreamSynchronize(st));
    t->tables_pending = 0;
    return SP_OK;
}

// Everything after the keys exist: sort, duplicates (an error, or summed in sorted order when `sum_duplicates`), the
// level sweep, narrow copies, values, and the tables the product kernels want.  keys / payload: nnz entries in
// temporaries of `tmp` (the payload is the value's bits); flags: 64 zeroed bytes, flags[0] != 0 afterwards on the
// device means a coordinate was out of range.  t->size[] and t->enc are set.  On success t->nnz is the number of
// distinct entries.
template <typename VT>
__global__ __launch_bounds__(kThreads) void sum_runs_kernel(const uint64_t *__restrict__ keys, const VT *__restrict__ vals, int64_t n,
                                                            const uint32_t *__restrict__ head_excl, uint64_t *__restrict__ keys_out,
                                                            VT *__restrict__ vals_out)
{
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= n) return;
    const uint64_t k = keys[e];
    if (e > 0 && keys[e - 1] == k) return;            // not the head of its run
    VT sum = vals[e];
    for (int64_t x = e + 1; x < n && keys[x] == k; ++x) sum += vals[x];     // sorted order = the order the entries came in
    const uint32_t u = head_excl[e];
    keys_out[u] = k;
    vals_out[u] = sum;
}

__global__ __launch_bounds__(kThreads) void mark_heads_kernel(const uint64_t *__restrict__ keys, int64_t n, uint32_t *__restrict__ mark)
{
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e < n) mark[e] = (e == 0 || keys[e] != keys[e - 1]) ? 1u : 0u;
}

static sp_status pack_core(sp_tensor *t, int64_t nnz, uint64_t *keys, const void *payload, int key_bits, bool sum_duplicates, int *flags,
                           sp_scratch &tmp, const sp_mem &mem, hipStream_t st, const sp_msd_plan *plan = nullptr)
{
    const sp_encoding *enc = &t->enc;
    const int rank = enc->rank;
    const sp_dtype dt = (sp_dtype)t->dtype;
    const int vsz0 = dt == SP_F64 ? 8 : 4;
    const size_t cnt = (size_t)(nnz > 0 ? nnz : 1);
    uint64_t *parentA = nullptr, *parentB = nullptr;      // allocated when a level needs them
    uint32_t *child = (uint32_t *)tmp.get(cnt * 4);
    if (!child) return SP_ERR_ALLOC;
    if (nnz > 0) SP_TRY(spmi_sort_pairs(keys, payload, vsz0, nnz, key_bits, tmp, st, plan, &keys, &payload));
    // The duplicate check rides along with the first compressed level's kernel (it reads the same neighbouring keys); it
    // runs on its own only where no such kernel comes before its result is needed.
    bool dup_pending = !sum_duplicates && nnz > 0;
    auto run_dup_check = [&]() -> sp_status {
        if (!dup_pending) return SP_OK;
        dup_pending = false;
        hipLaunchKernelGGL(check_duplicates_kernel, dim3(blocks_for(nnz)), dim3(kThreads), 0, st, (const uint64_t *)keys, nnz, flags);
        SP_HIP(hipGetLastError());
        return SP_OK;
    };
    // The input checks (a coordinate out of range, an entry given twice) come back to the host with the last read-back
    // of the build, not here: a host synchronisation in the middle costs a tenth of a small pack.  Every kernel below stays
    // in bounds on such input (bad coordinates were replaced by 0 when the keys were made; equal keys only make equal
    // writes).  input_error() reads them early where another error would otherwise be reported in their place.
    auto input_error = [&]() -> sp_status {
        SP_TRY(run_dup_check());
        int h[2] = {0, 0};
        if (hipMemcpyAsync(h, flags, sizeof(h), hipMemcpyDeviceToHost, st) != hipSuccess || hipStreamSynchronize(st) != hipSuccess) return SP_ERR_HIP;
        return h[0] ? SP_ERR_COORD_RANGE : h[1] ? SP_ERR_DUPLICATE : SP_OK;
    };
    if (sum_duplicates && nnz > 1) {
        hipLaunchKernelGGL(mark_heads_kernel, dim3(blocks_for(nnz)), dim3(kThreads), 0, st, (const uint64_t *)keys, nnz, child);
        SP_HIP(hipGetLastError());
        SP_TRY(spmi_exclusive_scan(child, nnz, 32, tmp, st));
        uint32_t last_excl = 0;
        SP_HIP(hipMemcpyAsync(&last_excl, child + (nnz - 1), 4, hipMemcpyDeviceToHost, st));
        SP_HIP(hipStreamSynchronize(st));
        // the last entry is a head exactly when its exclusive count differs from that of a head before it: recount it
        uint64_t lastk[2] = {0, 0};
        SP_HIP(hipMemcpyAsync(lastk, keys + (nnz - 2), 16, hipMemcpyDeviceToHost, st));
        SP_HIP(hipStreamSynchronize(st));
        const int64_t distinct = (int64_t)last_excl + (lastk[0] != lastk[1] ? 1 : 0);
        if (distinct != nnz) {
            uint64_t *k2 = (uint64_t *)tmp.get((size_t)distinct * 8);
            void *v2 = tmp.get(pad16((size_t)distinct * vsz0));
            if (!k2 || !v2) return SP_ERR_ALLOC;
            if (dt == SP_F64)
                hipLaunchKernelGGL(sum_runs_kernel<double>, dim3(blocks_for(nnz)), dim3(kThreads), 0, st, (const uint64_t *)keys,
                                   (const double *)payload, nnz, (const uint32_t *)child, k2, (double *)v2);
            else
                hipLaunchKernelGGL(sum_runs_kernel<float>, dim3(blocks_for(nnz)), dim3(kThreads), 0, st, (const uint64_t *)keys,
                                   (const float *)payload, nnz, (const uint32_t *)child, k2, (float *)v2);
            SP_HIP(hipGetLastError());
            keys = k2;
            payload = v2;
            nnz = distinct;
        }
    }
    t->nnz = nnz;

    // level sweep
    const uint64_t *pin = nullptr;      // nullptr = the position at the level above is the key prefix (dense levels so far)
    bool dense_prefix = true;
    int which = 0;
    int64_t P = 1;
    for (int l = 0; l < rank; ++l) {
        uint64_t stride_u = 1;
        for (int k = l + 1; k < rank; ++k) stride_u *= (uint64_t)(t->size[k] > 0 ? t->size[k] : 1);
        const divisor stride = make_divisor(stride_u);
        const divisor size = make_divisor((uint64_t)(t->size[l] > 0 ? t->size[l] : 1));
        if (enc->lt[l] == SP_DENSE && dense_prefix) {
            P *= t->size[l];                  // nothing to compute: the position at this level is the key prefix
            continue;
        }
        const bool last_compressed = enc->lt[l] == SP_COMPRESSED && l == rank - 1;
        uint64_t *pout = nullptr;
        if (!last_compressed && nnz > 0) {
            uint64_t *&buf = which ? parentB : parentA;
            if (!buf) { buf = (uint64_t *)tmp.get(cnt * 8); if (!buf) return SP_ERR_ALLOC; }
            pout = buf;
        }
        if (enc->lt[l] == SP_DENSE) {
            if (nnz > 0) {
                hipLaunchKernelGGL(dense_level_kernel, dim3(blocks_for(nnz)), dim3(kThreads), 0, st, (const uint64_t *)keys, nnz,
                                   stride, size, pin, pout);
                SP_HIP(hipGetLastError());
            }
            P *= t->size[l];
        } else {
            int64_t nchild = nnz;
            const uint32_t *child_excl = nullptr;
            if (l != rank - 1 && nnz > 0) {
                hipLaunchKernelGGL(mark_children_kernel, dim3(blocks_for(nnz)), dim3(kThreads), 0, st, (const uint64_t *)keys, nnz, stride, child);
                SP_HIP(hipGetLastError());
                SP_TRY(spmi_exclusive_scan(child, nnz, 32, tmp, st));
                // children = exclusive[nnz-1] + mark[nnz-1]; the last mark is recomputed from the two last keys
                uint32_t last_excl = 0;
                uint64_t lastk[2] = {0, 0};
                SP_HIP(hipMemcpyAsync(&last_excl, child + (nnz - 1), 4, hipMemcpyDeviceToHost, st));
                const int64_t from = nnz >= 2 ? nnz - 2 : 0;
                SP_HIP(hipMemcpyAsync(lastk, keys + from, (size_t)(nnz - from) * 8, hipMemcpyDeviceToHost, st));
                SP_HIP(hipStreamSynchronize(st));
                const bool last_mark = nnz == 1 || (lastk[0] / stride_u != lastk[1] / stride_u);
                nchild = (int64_t)last_excl + (last_mark ? 1 : 0);
                child_excl = child;
            }
            if (enc->pw_store < 64 && nchild > (((int64_t)1 << (enc->pw_store - 1)) - 1)) {
                SP_TRY(input_error());
                return SP_ERR_WIDTH;
            }
            const size_t pbytes = pad16((size_t)(P + 1) * (enc->pw / 8));
            const size_t cbytes = pad16((size_t)(nchild > 0 ? nchild : 1) * (enc->cw / 8));
            t->pos[l] = mem.get(pbytes);
            t->crd[l] = mem.get(cbytes);
            t->npos[l] = P + 1;
            t->ncrd[l] = nchild;
            if (!t->pos[l] || !t->crd[l]) return SP_ERR_ALLOC;
            SP_TRY(spmi_fill_zero(t->pos[l], pbytes, st));
            if (nnz > 0) {
                if (enc->pw == 32 && enc->cw == 32) SP_TRY((launch_emit<int32_t, int32_t>(keys, nnz, stride, size, child_excl, pin, pout, t->pos[l], t->crd[l], dup_pending ? flags : nullptr, st)));
                else if (enc->pw == 32) SP_TRY((launch_emit<int32_t, int64_t>(keys, nnz, stride, size, child_excl, pin, pout, t->pos[l], t->crd[l], dup_pending ? flags : nullptr, st)));
                else if (enc->cw == 32) SP_TRY((launch_emit<int64_t, int32_t>(keys, nnz, stride, size, child_excl, pin, pout, t->pos[l], t->crd[l], dup_pending ? flags : nullptr, st)));
                else SP_TRY((launch_emit<int64_t, int64_t>(keys, nnz, stride, size, child_excl, pin, pout, t->pos[l], t->crd[l], dup_pending ? flags : nullptr, st)));
                dup_pending = false;
            }
            SP_TRY(spmi_exclusive_scan(t->pos[l], P + 1, enc->pw, tmp, st));
            P = nchild;
        }
        if (enc->lt[l] == SP_COMPRESSED) dense_prefix = false;
        if (nnz > 0 && !last_compressed) { pin = pout; which ^= 1; }
    }

    // 8- and 16-bit widths: the arrays handed out are narrowed copies of the 32-bit working arrays
    for (int l = 0; l < rank; ++l) {
        if (enc->lt[l] != SP_COMPRESSED) continue;
        if (enc->pw_store < 32) {
            t->pos_narrow[l] = mem.get(pad16((size_t)t->npos[l] * (enc->pw_store / 8)));
            if (!t->pos_narrow[l]) return SP_ERR_ALLOC;
            if (enc->pw_store == 8)
                hipLaunchKernelGGL((narrow_kernel<int32_t, int8_t>), dim3(blocks_for(t->npos[l])), dim3(kThreads), 0, st,
                                   (const int32_t *)t->pos[l], t->npos[l], (int8_t *)t->pos_narrow[l]);
            else
                hipLaunchKernelGGL((narrow_kernel<int32_t, int16_t>), dim3(blocks_for(t->npos[l])), dim3(kThreads), 0, st,
                                   (const int32_t *)t->pos[l], t->npos[l], (int16_t *)t->pos_narrow[l]);
        }
        if (enc->cw_store < 32) {
            t->crd_narrow[l] = mem.get(pad16((size_t)(t->ncrd[l] > 0 ? t->ncrd[l] : 1) * (enc->cw_store / 8)));
            if (!t->crd_narrow[l]) return SP_ERR_ALLOC;
            if (enc->cw_store == 8)
                hipLaunchKernelGGL((narrow_kernel<int32_t, int8_t>), dim3(blocks_for(t->ncrd[l])), dim3(kThreads), 0, st,
                                   (const int32_t *)t->crd[l], t->ncrd[l], (int8_t *)t->crd_narrow[l]);
            else
                hipLaunchKernelGGL((narrow_kernel<int32_t, int16_t>), dim3(blocks_for(t->ncrd[l])), dim3(kThreads), 0, st,
                                   (const int32_t *)t->crd[l], t->ncrd[l], (int16_t *)t->crd_narrow[l]);
        }
        SP_HIP(hipGetLastError());
    }

    // values: zero padding only where a dense level sits below a compressed one.  With a compressed innermost level the
    // sorted payload already is the values array: the tensor takes that buffer over when the sort (or the summation)
    // made it, and copies only when it still is the caller's own array.
    const size_t vsz = dt == SP_F64 ? 8 : 4;
    const size_t vbytes = pad16((size_t)(P > 0 ? P : 1) * vsz);
    t->nvalues = P;
    if (nnz > 0 && enc->lt[rank - 1] == SP_COMPRESSED && tmp.release((void *)payload)) {
        t->values = (void *)payload;
    } else {
        t->values = mem.get(vbytes);
        if (!t->values) return SP_ERR_ALLOC;
        if (P != nnz) SP_TRY(spmi_fill_zero(t->values, vbytes, st));
        if (nnz > 0) {
            // where each sorted entry's value goes: its own rank (innermost level compressed), the key itself (every
            // level dense), or the position carried down from the last compressed level
            const uint64_t *position = (enc->lt[rank - 1] == SP_COMPRESSED) ? nullptr : dense_prefix ? (const uint64_t *)keys : pin;
            if (dt == SP_F64)
                hipLaunchKernelGGL(place_values_kernel<unsigned long long>, dim3(blocks_for(nnz)), dim3(kThreads), 0, st,
                                   (const unsigned long long *)payload, position, nnz, (unsigned long long *)t->values);
            else
                hipLaunchKernelGGL(place_values_kernel<uint32_t>, dim3(blocks_for(nnz)), dim3(kThreads), 0, st,
                                   (const uint32_t *)payload, position, nnz, (uint32_t *)t->values);
            SP_HIP(hipGetLastError());
        }
    }
    SP_TRY(run_dup_check());
    int hf[2] = {0, 0};
    SP_TRY(spmi_finish_tensor(t, flags, tmp, st, sum_duplicates ? nullptr : hf));
    if (hf[0]) return SP_ERR_COORD_RANGE;
    if (hf[1]) return SP_ERR_DUPLICATE;
    return SP_OK;
}

// A new tensor handle with shape, sizes by level and the key width worked out; SP_ERR_TOO_LARGE / SP_ERR_WIDTH as sp_pack documents.
sp_status spmi_new_tensor(const sp_encoding *enc, const int64_t *shape, sp_dtype dt, sp_alloc_fn alloc, sp_free_fn free_, void *ctx,
                            bool entries_in_an_empty_dimension, sp_tensor **out, int *key_bits_out)
{
    const int rank = enc->rank;
    sp_tensor *t = new sp_tensor();
    memset(t, 0, sizeof(*t));
    t->enc = *enc; t->dtype = dt; t->alloc = alloc; t->free_ = free_; t->ctx = ctx;
    t->scatter = -1;
    // the linearised key and every dense position count must stay below 2^63
    unsigned __int128 prod = 1;
    for (int l = 0; l < rank; ++l) {
        t->shape[l] = shape[l];
        t->size[l] = shape[enc->perm[l]];
        prod *= (unsigned __int128)(t->size[l] > 0 ? t->size[l] : 1);
        if (prod >= ((unsigned __int128)1 << 63)) { delete t; return SP_ERR_TOO_LARGE; }
    }
    if (entries_in_an_empty_dimension) { delete t; return SP_ERR_COORD_RANGE; }
    for (int l = 0; l < rank; ++l)
        if (enc->lt[l] == SP_COMPRESSED && enc->cw_store < 64 && t->size[l] - 1 > (((int64_t)1 << (enc->cw_store - 1)) - 1)) {
            delete t;
            return SP_ERR_WIDTH;
        }
    int key_bits = 0;
    while (key_bits < 63 && ((unsigned __int128)1 << key_bits) < prod) ++key_bits;
    *key_bits_out = key_bits;
    *out = t;
    return SP_OK;
}

sp_status spmi_finish_pack(sp_tensor *t, sp_status status, hipStream_t st, sp_tensor **out)
{
    if (status == SP_ERR_HIP && g_last_hip_error == 0) g_last_hip_error = (int)hipGetLastError();
    if (status != SP_OK) { release_tensor_arrays(t); delete t; return status; }
    *out = t;
    return SP_OK;
}

extern "C" sp_status sp_pack(const sp_encoding *enc, const int64_t *shape, int64_t nnz, const int64_t *const *coords,
                             const void *values, sp_dtype dt, sp_alloc_fn alloc, sp_free_fn free_, void *ctx, void *stream,
                             sp_tensor **out)
{
    if (!enc || !shape || !out) return SP_ERR_NULL;
    *out = nullptr;
    if ((alloc == nullptr) != (free_ == nullptr)) return SP_ERR_NULL;
    if (nnz > 0 && (!coords || !values)) return SP_ERR_NULL;
    int dti;                                           // any integer may arrive: read it as one, not as the enumeration
    memcpy(&dti, &dt, sizeof(dti));
    if (dti != (int)SP_F32 && dti != (int)SP_F64) return SP_ERR_DTYPE;
    if (nnz < 0) return SP_ERR_SHAPE;
    const int rank = enc->rank;
    bool zero_dim = false;
    for (int d = 0; d < rank; ++d) {
        if (shape[d] < 0) return SP_ERR_SHAPE;
        if (shape[d] == 0) zero_dim = true;
        if (nnz > 0 && !coords[d]) return SP_ERR_NULL;
    }
    if (nnz >= ((int64_t)1 << 31)) return SP_ERR_TOO_LARGE;
    hipStream_t st = (hipStream_t)stream;
    sp_tensor *t = nullptr;
    int key_bits = 0;
    SP_TRY(spmi_new_tensor(enc, shape, dt, alloc, free_, ctx, zero_dim && nnz > 0, &t, &key_bits));
    sp_mem mem{alloc, free_, ctx};
    sp_status status = SP_OK;
    {
        sp_scratch tmp(mem);
        const size_t cnt = (size_t)(nnz > 0 ? nnz : 1);
        uint64_t *keys = (uint64_t *)tmp.get(cnt * 8);
        int *flags = (int *)tmp.get(64);
        sp_msd_plan plan;
        memset(&plan, 0, sizeof(plan));
        do {
            if (!keys || !flags) { status = SP_ERR_ALLOC; break; }
            if ((status = spmi_fill_zero(flags, 64, st)) != SP_OK) break;
            if (nnz > 0) {
                level_args la;
                memset(&la, 0, sizeof(la));
                la.rank = rank;
                for (int l = 0; l < rank; ++l) { la.coord[l] = coords[enc->perm[l]]; la.size[l] = t->size[l]; }
                if ((status = spmi_msd_plan(nnz, key_bits, tmp, st, &plan)) != SP_OK) break;
                if (plan.ctr)
                    hipLaunchKernelGGL(make_keys_counting_kernel, dim3(plan.tiles), dim3(kThreads), 0, st, la, nnz, keys, flags, plan);
                else
                    hipLaunchKernelGGL(make_keys_kernel, dim3(blocks_for(nnz)), dim3(kThreads), 0, st, la, nnz, keys, flags);
                if (hipGetLastError() != hipSuccess) { status = SP_ERR_HIP; break; }
            }
            status = pack_core(t, nnz, keys, values, key_bits, false, flags, tmp, mem, st, &plan);   // the values are the sort's payload
        } while (0);
        if (status != SP_OK) (void)hipStreamSynchronize(st);   // temporaries may still be in use by queued kernels
    }
    return spmi_finish_pack(t, status, st, out);
}

// keys[e] = the linearised key (level order of `t`, mixed radix over its level sizes) of the entry whose coordinate in
// dimension d is coords[d][e]; flags[0] is set when a coordinate is out of range.
sp_status spmi_make_keys(const sp_tensor *t, const int64_t *const *coords, int64_t n, uint64_t *keys, int *flags, hipStream_t st)
{
    if (n <= 0) return SP_OK;
    level_args la;
    memset(&la, 0, sizeof(la));
    la.rank = t->enc.rank;
    for (int l = 0; l < la.rank; ++l) { la.coord[l] = coords[t->enc.perm[l]]; la.size[l] = t->size[l]; }
    hipLaunchKernelGGL(make_keys_kernel, dim3(blocks_for(n)), dim3(kThreads), 0, st, la, n, keys, flags);
    SP_HIP(hipGetLastError());
    return SP_OK;
}

// The storage of a tensor whose entries are given as linearised keys (level order, mixed radix over the level sizes)
// with the value bits as payload; entries with equal keys are added up in the order they are given.
sp_status spmi_pack_keys(const sp_encoding *enc, const int64_t *shape, sp_dtype dt, sp_alloc_fn alloc, sp_free_fn free_, void *ctx,
                         int64_t n, uint64_t *keys, void *payload, sp_scratch &tmp, hipStream_t st, sp_tensor **out)
{
    *out = nullptr;
    if (n >= ((int64_t)1 << 31)) return SP_ERR_TOO_LARGE;
    sp_tensor *t = nullptr;
    int key_bits = 0;
    SP_TRY(spmi_new_tensor(enc, shape, dt, alloc, free_, ctx, false, &t, &key_bits));
    sp_mem mem{alloc, free_, ctx};
    int *flags = (int *)tmp.get(64);
    sp_status status = flags ? spmi_fill_zero(flags, 64, st) : SP_ERR_ALLOC;
    if (status == SP_OK) status = pack_core(t, n, keys, payload, key_bits, true, flags, tmp, mem, st);
    if (status != SP_OK) (void)hipStreamSynchronize(st);
    return spmi_finish_pack(t, status, st, out);
}

extern "C" sp_status sp_unpack(const sp_tensor *t, int64_t *const *coords, void *values, void *stream)
{
    if (!t || !coords || (!values && t->nvalues > 0)) return SP_ERR_NULL;
    const int rank = t->enc.rank;
    for (int d = 0; d < rank; ++d) if (!coords[d] && t->nvalues > 0) return SP_ERR_NULL;
    if (t->nvalues == 0) return SP_OK;
    hipStream_t st = (hipStream_t)stream;
    sp_mem mem{t->alloc, t->free_, t->ctx};
    // small descriptor tables for the kernel: level types + ordering, array pointers, pos lengths, outputs
    struct tables {
        int lt_perm[2 * SP_MAX_RANK];
        const void *pos[SP_MAX_RANK];
        const void *crd[SP_MAX_RANK];
        int64_t npos[SP_MAX_RANK];
        int64_t *out[SP_MAX_RANK];
    } h;
    memset(&h, 0, sizeof(h));
    level_args la;
    memset(&la, 0, sizeof(la));
    la.rank = rank;
    for (int l = 0; l < rank; ++l) {
        h.lt_perm[l] = t->enc.lt[l];
        h.lt_perm[SP_MAX_RANK + l] = t->enc.perm[l];
        h.pos[l] = t->pos[l]; h.crd[l] = t->crd[l]; h.npos[l] = t->npos[l];
        h.out[l] = coords[l];
        la.size[l] = t->size[l] > 0 ? t->size[l] : 1;
    }
    tables *d = (tables *)mem.get(sizeof(tables));
    if (!d) return SP_ERR_ALLOC;
    sp_status s = SP_OK;
    do {
        if (hipMemcpyAsync(d, &h, sizeof(h), hipMemcpyHostToDevice, st) != hipSuccess) { s = SP_ERR_HIP; break; }
        const unsigned nb = blocks_for(t->nvalues);
#define SPMI_UNPACK(PT, CT)                                                                                                   \
    hipLaunchKernelGGL((unpack_kernel<PT, CT>), dim3(nb), dim3(kThreads), 0, st, rank, la, (const int *)d->lt_perm,            \
                       (const void *const *)d->pos, (const void *const *)d->crd, (const int64_t *)d->npos, t->nvalues,        \
                       (int64_t *const *)d->out)
        if (t->enc.pw == 32 && t->enc.cw == 32) SPMI_UNPACK(int32_t, int32_t);
        else if (t->enc.pw == 32) SPMI_UNPACK(int32_t, int64_t);
        else if (t->enc.cw == 32) SPMI_UNPACK(int64_t, int32_t);
        else SPMI_UNPACK(int64_t, int64_t);
#undef SPMI_UNPACK
        if (hipGetLastError() != hipSuccess) { s = SP_ERR_HIP; break; }
        const size_t vsz = t->dtype == SP_F64 ? 8 : 4;
        if (hipMemcpyAsync(values, t->values, (size_t)t->nvalues * vsz, hipMemcpyDeviceToDevice, st) != hipSuccess) { s = SP_ERR_HIP; break; }
    } while (0);
    // the descriptor table is read by the queued kernel: wait before handing it back
    if (hipStreamSynchronize(st) != hipSuccess && s == SP_OK) s = SP_ERR_HIP;
    mem.put(d);
    return s;
}
