// Stable radix sorts of (key, payload) pairs for the storage builder (arXiv 2202.04305, Section 4.2: the entries of the
// coordinate scheme are brought into the level order of the target format before its arrays are built).  8-bit digits; one
// pair of kernels, a histogram per tile and a scatter that ranks keys inside a wave with ballots and sorts the tile in LDS
// before writing it, serves both orders of the digits.
//
// Least significant digit first: one such pass over all entries per 8 key bits.
//
// Most significant digit first: two passes split the entries by the top 16 bits of the key (256 buckets, then 256
// sub-buckets inside each bucket); what is left of the key is sorted inside the LDS, a block taking a run of consecutive
// sub-buckets of about a thousand entries.  Three reads and writes of the entries instead of one per 8 key bits.  Every
// pass keeps the input order of entries with equal digits, so this sort is stable as well, and duplicates are added up in
// the same order after either.
//
// Skew: a run of sub-buckets that does not fit the LDS is sorted by its block through device memory, slowly; the caller asks
// spmi_msd_sort_suits() first (a sampled histogram of the top 16 bits) and takes the other sort when that would be common.
#include "spmi_internal.h"

namespace {

#ifndef SPMI_SORT_T
#define SPMI_SORT_T 256
#endif
constexpr int kT = SPMI_SORT_T;               // threads of the partition kernels (at least 256: thread d also stands for digit d)
constexpr int kRounds = 16;
constexpr int kTile = kSpmiMsdTile;           // entries per tile of a partition pass
static_assert(kTile == kT * kRounds, "tile");
#ifndef SPMI_MSD_FE
#define SPMI_MSD_FE 8
#endif
constexpr int kFT = 256;                      // threads of the finishing kernel
constexpr int kFE = SPMI_MSD_FE;              // entries per thread in the LDS
constexpr int kCap = kFT * kFE;               // entries a block sorts inside the LDS
constexpr int kTarget = kCap / 2;             // a block takes the sub-buckets that start inside one stretch of this many entries
constexpr int kSub = 65536;                   // sub-buckets after two passes

// A partition pass works on segments (1 for the first pass, the 256 buckets for the second): segment b holds the entries
// [seg_start[b], seg_start[b+1]) and is cut into tiles of kTile entries, numbered from seg_tile[b].  Block = tile.  The count
// of digit d in tile j of segment b lives at ctr[256 * seg_tile[b] + d * tiles(b) + j]: one exclusive scan over the whole array
// then gives every (segment, digit, tile) its place in the output, which is ordered by segment, digit, tile.
struct tile_place { uint32_t lo, hi, ctr0, stride; bool any; };

__device__ __forceinline__ tile_place locate_tile(const uint32_t *__restrict__ seg_start, const uint32_t *__restrict__ seg_tile, int nseg)
{
    __shared__ tile_place s_place;
    if (threadIdx.x == 0) {
        tile_place p;
        const uint32_t t = blockIdx.x;
        p.any = t < seg_tile[nseg];
        if (p.any) {
            int lo = 0, hi = nseg;                      // largest b with seg_tile[b] <= t
            while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (seg_tile[mid] <= t) lo = mid; else hi = mid; }
            const uint32_t j = t - seg_tile[lo];
            p.stride = seg_tile[lo + 1] - seg_tile[lo];
            p.lo = seg_start[lo] + j * (uint32_t)kTile;
            const uint32_t end = seg_start[lo + 1];
            p.hi = p.lo + (uint32_t)kTile < end ? p.lo + (uint32_t)kTile : end;
            p.ctr0 = 256u * seg_tile[lo] + j;
        } else { p.lo = p.hi = p.ctr0 = p.stride = 0; }
        s_place = p;
    }
    __syncthreads();
    return s_place;
}

__global__ __launch_bounds__(kT) void partition_hist_kernel(const uint64_t *__restrict__ keys, const uint32_t *__restrict__ seg_start,
                                                      const uint32_t *__restrict__ seg_tile, int nseg, int shift, uint32_t *__restrict__ ctr)
{
    __shared__ uint32_t h[256];
    const tile_place p = locate_tile(seg_start, seg_tile, nseg);
    if (!p.any) return;
    if (threadIdx.x < 256) h[threadIdx.x] = 0;
    __syncthreads();
    if (p.hi - p.lo == (uint32_t)kTile && (p.lo & 1u) == 0) {     // a whole, 16-byte aligned tile: two keys per lane and load, all loads first
        typedef unsigned long long u2 __attribute__((ext_vector_type(2)));
        const u2 *__restrict__ kk = (const u2 *)(keys + p.lo);
        u2 k[kRounds / 2];
#pragma unroll
        for (int r = 0; r < kRounds / 2; ++r) k[r] = kk[r * kT + threadIdx.x];
#pragma unroll
        for (int r = 0; r < kRounds / 2; ++r) {
            atomicAdd(&h[(uint32_t)(k[r][0] >> shift) & 255u], 1u);
            atomicAdd(&h[(uint32_t)(k[r][1] >> shift) & 255u], 1u);
        }
    } else {
        for (uint32_t i = p.lo + threadIdx.x; i < p.hi; i += kT) atomicAdd(&h[(uint32_t)(keys[i] >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (threadIdx.x < 256) ctr[p.ctr0 + threadIdx.x * p.stride] = h[threadIdx.x];
}

// One tile of a partition pass: ranks inside the tile with ballots (tile order = wave, round, lane), the tile sorted by the
// digit in LDS, then written so that neighbouring threads write neighbouring addresses of one digit's run.
template <typename P>
__global__ __launch_bounds__(kT) void partition_scatter_kernel(const uint64_t *__restrict__ kin, const P *__restrict__ vin, uint64_t *__restrict__ kout,
                                                         P *__restrict__ vout, const uint32_t *__restrict__ seg_start,
                                                         const uint32_t *__restrict__ seg_tile, int nseg, int shift, const uint32_t *__restrict__ ctr)
{
    constexpr int W = kT / 64, PERW = kTile / W;
    __shared__ uint16_t wrun[W][256];                 // counts and slots inside a tile fit 16 bits
    __shared__ uint16_t wbase[W][256];
    __shared__ uint32_t gbase[256];
    __shared__ uint32_t wsum[4];
    __shared__ uint64_t stage[kTile];                 // the tile in sorted order: first the keys, then the payloads
    const tile_place p = locate_tile(seg_start, seg_tile, nseg);
    if (!p.any) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int in_tile = (int)(p.hi - p.lo);
    for (int i = tid; i < W * 256; i += kT) (&wrun[0][0])[i] = 0;
    uint64_t k[kRounds];
    P v[kRounds];
    uint32_t lpos[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int i = wave * PERW + r * 64 + lane;
        k[r] = i < in_tile ? kin[p.lo + i] : 0;
        v[r] = i < in_tile ? vin[p.lo + i] : 0;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const bool valid = wave * PERW + r * 64 + lane < in_tile;
        const uint32_t d = (uint32_t)(k[r] >> shift) & 255u;
        const uint64_t m = match_digit(d, valid);
        const uint32_t before = wrun[wave][d];
        lpos[r] = before + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
        if (valid && (m & ((1ull << lane) - 1ull)) == 0) wrun[wave][d] = (uint16_t)(before + (uint32_t)__popcll(m));
    }
    __syncthreads();
    {   // thread d < 256: tile count of digit d, exclusive scan over the digits, per-wave starts
        uint32_t c[W], tot = 0, incl = 0;
        if (tid < 256) {
#pragma unroll
            for (int w = 0; w < W; ++w) { c[w] = wrun[w][tid]; tot += c[w]; }
            incl = wave_inclusive_scan(tot, lane);
            if (lane == 63) wsum[wave] = incl;
        }
        __syncthreads();
        if (tid < 256) {
            uint32_t start = incl - tot;
            for (int w = 0; w < wave; ++w) start += wsum[w];
            gbase[tid] = ctr[p.ctr0 + tid * p.stride] - start;
#pragma unroll
            for (int w = 0; w < W; ++w) { wbase[w][tid] = (uint16_t)start; start += c[w]; }
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        if (wave * PERW + r * 64 + lane < in_tile) {
            const uint32_t d = (uint32_t)(k[r] >> shift) & 255u;
            lpos[r] += wbase[wave][d];                 // from here on: the entry's slot in the sorted tile
            stage[lpos[r]] = k[r];
        }
    }
    __syncthreads();
    uint32_t q[kRounds];                              // where the entry that sits in slot tid + j * kT goes
#pragma unroll
    for (int j = 0; j < kRounds; ++j) {
        const int slot = tid + j * kT;
        if (slot < in_tile) {
            const uint64_t key = stage[slot];
            q[j] = gbase[(uint32_t)(key >> shift) & 255u] + (uint32_t)slot;
            kout[q[j]] = key;
        }
    }
    __syncthreads();
    P *sval = (P *)stage;
#pragma unroll
    for (int r = 0; r < kRounds; ++r)
        if (wave * PERW + r * 64 + lane < in_tile) sval[lpos[r]] = v[r];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kRounds; ++j) {
        const int slot = tid + j * kT;
        if (slot < in_tile) vout[q[j]] = sval[slot];
    }
}

__global__ void one_segment_kernel(uint32_t *seg_start, uint32_t *seg_tile, uint32_t n)
{
    seg_start[0] = 0; seg_start[1] = n;
    seg_tile[0] = 0; seg_tile[1] = (n + kTile - 1) / kTile;
}

// The buckets of the first pass become the segments of the second: bucket b starts where digit b's first tile was placed.
__global__ __launch_bounds__(256) void buckets_to_segments_kernel(const uint32_t *__restrict__ ctr1, uint32_t tiles1, uint32_t n,
                                                               uint32_t *__restrict__ seg_start, uint32_t *__restrict__ seg_tile)
{
    __shared__ uint32_t start[257];
    __shared__ uint32_t wsum[4];
    const int b = threadIdx.x, lane = b & 63, wave = b >> 6;
    start[b] = ctr1[(uint32_t)b * tiles1];
    if (b == 0) start[256] = n;
    __syncthreads();
    const uint32_t tiles = (start[b + 1] - start[b] + kTile - 1) / kTile;
    const uint32_t incl = wave_inclusive_scan(tiles, lane);
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    uint32_t before = incl - tiles;
    for (int w = 0; w < wave; ++w) before += wsum[w];
    seg_start[b] = start[b];
    seg_tile[b] = before;
    if (b == 255) { seg_start[256] = n; seg_tile[256] = before + tiles; }
}

// Sub-bucket d of bucket b starts, after the second pass, at S(b, d) = the place of its first tile.  The finishing pass cuts the
// entries into chunks of whole sub-buckets: chunk k = the sub-buckets that start inside [k * kTarget, (k+1) * kTarget), so
// chunk_lo[k] = the first sub-bucket start at or after k * kTarget (n when there is none), for k = 0 .. nchunks.  Thread =
// sub-bucket (plus one for the end of the array): it writes chunk_lo[k] for the multiples of kTarget that lie after its
// predecessor's start and not after its own.
__global__ __launch_bounds__(256) void msd_chunks_kernel(const uint32_t *__restrict__ ctr2, const uint32_t *__restrict__ seg_start,
                                                         const uint32_t *__restrict__ seg_tile, uint32_t n, uint32_t nchunks,
                                                         uint32_t *__restrict__ chunk_lo)
{
    const uint32_t s = blockIdx.x * 256u + threadIdx.x;
    if (s > (uint32_t)kSub) return;
    auto start_of = [&](uint32_t sub) -> uint32_t {
        if (sub >= (uint32_t)kSub) return n;
        const uint32_t b = sub >> 8, d = sub & 255u;
        const uint32_t tiles = seg_tile[b + 1] - seg_tile[b];
        return tiles ? ctr2[256u * seg_tile[b] + d * tiles] : seg_start[b];
    };
    const uint32_t mine = start_of(s);
    uint32_t k = s == 0 ? 0u : start_of(s - 1) / (uint32_t)kTarget + 1u;
    const uint32_t k_last = s == (uint32_t)kSub ? nchunks : mine / (uint32_t)kTarget;
    for (; k <= k_last && k <= nchunks; ++k) chunk_lo[k] = mine;
}

// Ranks by one 8-bit digit the entries that a block of kFT threads holds in registers: wave w holds entries [w * perw,
// (w+1) * perw) of the tile, 64 per round, so tile order = wave, round, lane.  Afterwards the entry in (wave, r, lane) with
// digit d is number  wrel[wave * 256 + d] + lpos[r]  among the tile's entries of digit d (input order kept), digit d's run
// starts at dig[d] inside the sorted tile, and tot (thread d) is the tile's count of digit d.  Ends with a barrier.
template <int R>
__device__ __forceinline__ void rank_by_digit(const uint64_t (&k)[R], int rounds, uint32_t perw, uint32_t cnt, int shift, uint32_t *wrun,
                                              uint32_t *wrel, uint32_t *dig, uint32_t *wsum, uint32_t (&lpos)[R], uint32_t &tot)
{
    constexpr int W = kFT / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int w = 0; w < W; ++w) wrun[w * 256 + tid] = 0;
    __syncthreads();
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (r < rounds) {                                  // wave-uniform
            const bool valid = (uint32_t)wave * perw + (uint32_t)(r * 64 + lane) < cnt;
            const uint32_t d = (uint32_t)(k[r] >> shift) & 255u;
            const uint64_t m = match_digit(d, valid);
            const uint32_t before = wrun[wave * 256 + d];            // written by this wave only, in program order
            lpos[r] = before + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            if (valid && (m & ((1ull << lane) - 1ull)) == 0) wrun[wave * 256 + d] = before + (uint32_t)__popcll(m);
        }
    }
    __syncthreads();
    uint32_t c[W];
    tot = 0;
#pragma unroll
    for (int w = 0; w < W; ++w) { c[w] = wrun[w * 256 + tid]; tot += c[w]; }
    const uint32_t incl = wave_inclusive_scan(tot, lane);
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    uint32_t start = incl - tot;
    for (int w = 0; w < wave; ++w) start += wsum[w];
    dig[tid] = start;
    uint32_t rel = 0;
#pragma unroll
    for (int w = 0; w < W; ++w) { wrel[w * 256 + tid] = rel; rel += c[w]; }
    __syncthreads();
}

// The finishing pass.  Block k takes chunk k: a contiguous range of entries, sorted here by the whole key (stable, least
// significant digit first, digits in which no two keys of the range differ skipped) and written to the same range of the
// output.  kin/vin and kalt/valt are the same arrays: a range that does not fit the LDS is sorted through device memory,
// tile by tile, hopping between its part of these and its part of the output.
template <typename P>
__global__ __launch_bounds__(kFT) void msd_finish_kernel(const uint64_t *kin, const P *vin, uint64_t *kout, P *vout, uint64_t *kalt, P *valt,
                                                         const uint32_t *__restrict__ chunk_lo)
{
    constexpr int W = kFT / 64;
    __shared__ uint64_t skey[kCap];
    __shared__ P sval[kCap];
    __shared__ uint32_t wrun[W * 256];
    __shared__ uint32_t wrel[W * 256];
    __shared__ uint32_t dig[256];
    __shared__ uint32_t dstart[256];
    __shared__ uint32_t wsum[W];
    __shared__ unsigned long long s_or[W];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t lo = chunk_lo[blockIdx.x], hi = chunk_lo[blockIdx.x + 1];
    if (lo >= hi) return;
    const uint32_t cnt = hi - lo;
    const uint64_t k0 = kin[lo];
    uint64_t k[kFE];
    P v[kFE];
    uint32_t lpos[kFE];
    uint32_t tot;
    if (cnt <= (uint32_t)kCap) {
        const uint32_t perw = ((cnt + W * 64 - 1) / (W * 64)) * 64;
        const int rounds = (int)(perw / 64);                      // <= kFE
        unsigned long long diff = 0;
#pragma unroll
        for (int r = 0; r < kFE; ++r) {
            const uint32_t i = (uint32_t)wave * perw + (uint32_t)(r * 64 + lane);
            const bool valid = r < rounds && i < cnt;
            k[r] = valid ? kin[lo + i] : k0;
            v[r] = valid ? vin[lo + i] : (P)0;
            diff |= k[r] ^ k0;
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) diff |= __shfl_xor(diff, d, 64);
        if (lane == 0) s_or[wave] = diff;
        __syncthreads();
        diff = 0;
        for (int w = 0; w < W; ++w) diff |= s_or[w];
        for (int shift = 0; shift < 64; shift += 8) {
            if (((diff >> shift) & 255ull) == 0) continue;         // block-uniform
            rank_by_digit<kFE>(k, rounds, perw, cnt, shift, wrun, wrel, dig, wsum, lpos, tot);
#pragma unroll
            for (int r = 0; r < kFE; ++r) {
                if (r < rounds && (uint32_t)wave * perw + (uint32_t)(r * 64 + lane) < cnt) {
                    const uint32_t d = (uint32_t)(k[r] >> shift) & 255u;
                    const uint32_t slot = dig[d] + wrel[wave * 256 + d] + lpos[r];
                    skey[slot] = k[r];
                    sval[slot] = v[r];
                }
            }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < kFE; ++r) {
                const uint32_t i = (uint32_t)wave * perw + (uint32_t)(r * 64 + lane);
                if (r < rounds && i < cnt) { k[r] = skey[i]; v[r] = sval[i]; }
            }
            // the next writes to skey / sval come after the barriers of the next ranking
        }
#pragma unroll
        for (int r = 0; r < kFE; ++r) {
            const uint32_t i = (uint32_t)wave * perw + (uint32_t)(r * 64 + lane);
            if (r < rounds && i < cnt) { kout[lo + i] = k[r]; vout[lo + i] = v[r]; }
        }
        return;
    }
    // More entries than the LDS holds.  Slow (one block for the whole range); meant to be rare.
    unsigned long long diff = 0;
    for (uint32_t i = lo + tid; i < hi; i += kFT) diff |= kin[i] ^ k0;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) diff |= __shfl_xor(diff, d, 64);
    if (lane == 0) s_or[wave] = diff;
    __syncthreads();
    diff = 0;
    for (int w = 0; w < W; ++w) diff |= s_or[w];
    const uint64_t *src_k = kin;
    const P *src_v = vin;
    int hop = 0;
    for (int shift = 0; shift < 64; shift += 8) {
        if (((diff >> shift) & 255ull) == 0) continue;
        uint64_t *dst_k = (hop & 1) ? kalt : kout;
        P *dst_v = (hop & 1) ? valt : vout;
        ++hop;
        dstart[tid] = 0;
        __syncthreads();
        for (uint32_t i = lo + tid; i < hi; i += kFT) atomicAdd(&dstart[(uint32_t)(src_k[i] >> shift) & 255u], 1u);
        __syncthreads();
        {
            const uint32_t c = dstart[tid];
            const uint32_t incl = wave_inclusive_scan(c, lane);
            if (lane == 63) wsum[wave] = incl;
            __syncthreads();
            uint32_t start = incl - c;
            for (int w = 0; w < wave; ++w) start += wsum[w];
            dstart[tid] = lo + start;
        }
        for (uint32_t base = lo; base < hi; base += kCap) {      // tiles in order: the pass is stable
            const uint32_t tcnt = hi - base < (uint32_t)kCap ? hi - base : (uint32_t)kCap;
            const uint32_t perw = ((tcnt + W * 64 - 1) / (W * 64)) * 64;
            const int rounds = (int)(perw / 64);
#pragma unroll
            for (int r = 0; r < kFE; ++r) {
                const uint32_t i = (uint32_t)wave * perw + (uint32_t)(r * 64 + lane);
                const bool valid = r < rounds && i < tcnt;
                k[r] = valid ? src_k[base + i] : 0;
                v[r] = valid ? src_v[base + i] : (P)0;
            }
            rank_by_digit<kFE>(k, rounds, perw, tcnt, shift, wrun, wrel, dig, wsum, lpos, tot);   // its first barrier also orders dstart
#pragma unroll
            for (int r = 0; r < kFE; ++r) {
                if (r < rounds && (uint32_t)wave * perw + (uint32_t)(r * 64 + lane) < tcnt) {
                    const uint32_t d = (uint32_t)(k[r] >> shift) & 255u;
                    const uint32_t q = dstart[d] + wrel[wave * 256 + d] + lpos[r];
                    dst_k[q] = k[r];
                    dst_v[q] = v[r];
                }
            }
            __syncthreads();
            dstart[tid] += tot;
        }
        src_k = dst_k;
        src_v = dst_v;
        __syncthreads();                                          // the next pass reads what this one wrote (same workgroup)
    }
    if (src_k != kout) {                                          // no hop at all (every key equal), or an even number of them
        for (uint32_t i = lo + tid; i < hi; i += kFT) { kout[i] = src_k[i]; vout[i] = src_v[i]; }
    }
}

// Sampled histogram of the top 16 bits of the keys (one key in 64), and what it says about the finishing pass.
__global__ __launch_bounds__(256) void msd_sample_kernel(const uint64_t *__restrict__ keys, int64_t n, int shift, uint32_t *__restrict__ samp)
{
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 64;
    if (i < n) atomicAdd(&samp[(uint32_t)(keys[i] >> shift) & 0xffffu], 1u);
}

// out[0] = estimated number of entries in sub-buckets that alone overflow a finishing block, out[1] = estimated size of the
// largest sub-bucket.
__global__ __launch_bounds__(256) void msd_sample_summary_kernel(const uint32_t *__restrict__ samp, unsigned long long *__restrict__ out)
{
    unsigned long long heavy = 0, largest = 0;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < kSub; i += gridDim.x * 256) {
        const unsigned long long est = (unsigned long long)samp[i] * 64ull;
        if (est > (unsigned long long)(kCap - kTarget)) heavy += est;
        largest = est > largest ? est : largest;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        heavy += __shfl_xor(heavy, d, 64);
        const unsigned long long o = __shfl_xor(largest, d, 64);
        largest = o > largest ? o : largest;
    }
    if ((threadIdx.x & 63) == 0) {
        if (heavy) atomicAdd(&out[0], heavy);
        atomicMax(&out[1], largest);
    }
}

// Least significant digit first.  keys: n entries in a temporary of `tmp`, reordered freely; vals_in: n payloads, only read
// (it may be the caller's own array).  On return *keys_out / *vals_out point at the sorted arrays: temporaries of `tmp`, or
// the inputs when there was nothing to sort.
template <typename P>
sp_status lsd_sort_t(uint64_t *keys, const P *vals_in, int64_t n, int key_bits, sp_scratch &tmp, hipStream_t st, uint64_t **keys_out,
                     const P **vals_out)
{
    *keys_out = keys;
    *vals_out = vals_in;
    if (n <= 1 || key_bits <= 0) return SP_OK;
    if (n >= ((int64_t)1 << 32) - kTile) return SP_ERR_TOO_LARGE;
    const int passes = (key_bits + 7) / 8;
    const uint32_t n32 = (uint32_t)n, tiles = (n32 + kTile - 1) / kTile;
    const size_t vbytes = ((size_t)n * sizeof(P) + 15) & ~(size_t)15;
    uint64_t *kalt = (uint64_t *)tmp.get((size_t)n * 8);
    P *va = (P *)tmp.get(vbytes);
    P *vb = passes > 1 ? (P *)tmp.get(vbytes) : va;
    uint32_t *ctr = (uint32_t *)tmp.get((size_t)256 * tiles * 4);
    uint32_t *seg = (uint32_t *)tmp.get(16);                     // one segment: every entry
    if (!kalt || !va || !vb || !ctr || !seg) return SP_ERR_ALLOC;
    hipLaunchKernelGGL(one_segment_kernel, dim3(1), dim3(1), 0, st, seg, seg + 2, n32);
    uint64_t *kin = keys, *kout = kalt;
    const P *vin = vals_in;
    P *vout = va;
    for (int p = 0; p < passes; ++p) {
        const int shift = 8 * p;
        hipLaunchKernelGGL(partition_hist_kernel, dim3(tiles), dim3(kT), 0, st, (const uint64_t *)kin, (const uint32_t *)seg, (const uint32_t *)(seg + 2), 1, shift,
                           ctr);
        SP_HIP(hipGetLastError());
        SP_TRY(spmi_exclusive_scan(ctr, (int64_t)256 * tiles, 32, tmp, st));
        hipLaunchKernelGGL(partition_scatter_kernel<P>, dim3(tiles), dim3(kT), 0, st, (const uint64_t *)kin, vin, kout, vout, (const uint32_t *)seg,
                           (const uint32_t *)(seg + 2), 1, shift, (const uint32_t *)ctr);
        SP_HIP(hipGetLastError());
        uint64_t *tk = kin; kin = kout; kout = tk;
        vin = vout;
        vout = vout == va ? vb : va;
    }
    *keys_out = kin;
    *vals_out = vin;
    return SP_OK;
}

template <typename P>
sp_status msd_sort_t(uint64_t *keys, const P *vals_in, int64_t n, int key_bits, sp_scratch &tmp, hipStream_t st, uint32_t *ctr_ready,
                     uint64_t **keys_out, const P **vals_out)
{
    const uint32_t n32 = (uint32_t)n;
    const uint32_t tiles1 = (n32 + kTile - 1) / kTile, tiles2_max = tiles1 + 256;
    uint64_t *kb = (uint64_t *)tmp.get((size_t)n * 8);
    P *va = (P *)tmp.get(((size_t)n * sizeof(P) + 15) & ~(size_t)15);
    P *vb = (P *)tmp.get(((size_t)n * sizeof(P) + 15) & ~(size_t)15);
    const size_t ctr_words = (size_t)256 * tiles2_max;
    uint32_t *ctr = ctr_ready ? ctr_ready : (uint32_t *)tmp.get(ctr_words * 4);      // ctr_ready: the first pass's counts are in it already
    const uint32_t nchunks = n32 / (uint32_t)kTarget + 1;
    uint32_t *seg = (uint32_t *)tmp.get((size_t)(2 * 257 + 2 * 2 + nchunks + 1 + 8) * 4);
    if (!kb || !va || !vb || !ctr || !seg) return SP_ERR_ALLOC;
    uint32_t *seg_start1 = seg, *seg_tile1 = seg + 2, *seg_start2 = seg + 4, *seg_tile2 = seg + 4 + 257, *chunk_lo = seg + 4 + 2 * 257;
    const int shift1 = key_bits > 8 ? key_bits - 8 : 0, shift2 = key_bits > 16 ? key_bits - 16 : 0;
    // first pass: keys / vals_in -> kb / va
    hipLaunchKernelGGL(one_segment_kernel, dim3(1), dim3(1), 0, st, seg_start1, seg_tile1, n32);
    if (!ctr_ready)
        hipLaunchKernelGGL(partition_hist_kernel, dim3(tiles1), dim3(kT), 0, st, (const uint64_t *)keys, (const uint32_t *)seg_start1, (const uint32_t *)seg_tile1,
                           1, shift1, ctr);
    SP_HIP(hipGetLastError());
    SP_TRY(spmi_exclusive_scan(ctr, (int64_t)256 * tiles1, 32, tmp, st));
    hipLaunchKernelGGL(partition_scatter_kernel<P>, dim3(tiles1), dim3(kT), 0, st, (const uint64_t *)keys, vals_in, kb, va, (const uint32_t *)seg_start1,
                       (const uint32_t *)seg_tile1, 1, shift1, (const uint32_t *)ctr);
    hipLaunchKernelGGL(buckets_to_segments_kernel, dim3(1), dim3(256), 0, st, (const uint32_t *)ctr, tiles1, n32, seg_start2, seg_tile2);
    SP_HIP(hipGetLastError());
    // second pass: kb / va -> keys / vb.  Tiles past the last one of the last bucket do nothing; their counters stay zero.
    SP_TRY(spmi_fill_zero(ctr, ctr_words * 4, st));
    hipLaunchKernelGGL(partition_hist_kernel, dim3(tiles2_max), dim3(kT), 0, st, (const uint64_t *)kb, (const uint32_t *)seg_start2, (const uint32_t *)seg_tile2,
                       256, shift2, ctr);
    SP_HIP(hipGetLastError());
    SP_TRY(spmi_exclusive_scan(ctr, (int64_t)ctr_words, 32, tmp, st));
    hipLaunchKernelGGL(partition_scatter_kernel<P>, dim3(tiles2_max), dim3(kT), 0, st, (const uint64_t *)kb, (const P *)va, keys, vb,
                       (const uint32_t *)seg_start2, (const uint32_t *)seg_tile2, 256, shift2, (const uint32_t *)ctr);
    hipLaunchKernelGGL(msd_chunks_kernel, dim3(kSub / 256 + 1), dim3(256), 0, st, (const uint32_t *)ctr, (const uint32_t *)seg_start2,
                       (const uint32_t *)seg_tile2, n32, nchunks, chunk_lo);
    SP_HIP(hipGetLastError());
    // finishing pass: keys / vb -> kb / va (a range that does not fit the LDS also hops through its own part of keys / vb)
    hipLaunchKernelGGL(msd_finish_kernel<P>, dim3(nchunks), dim3(kFT), 0, st, (const uint64_t *)keys, (const P *)vb, kb, va, keys, vb,
                       (const uint32_t *)chunk_lo);
    SP_HIP(hipGetLastError());
    *keys_out = kb;
    *vals_out = va;
    return SP_OK;
}

}  // namespace

sp_status spmi_msd_plan(int64_t n, int key_bits, sp_scratch &tmp, hipStream_t st, sp_msd_plan *plan)
{
    memset(plan, 0, sizeof(*plan));
    const int mode = g_pack_sort_mode.load(std::memory_order_relaxed);
    if (mode == 1 || n < 1 || n >= ((int64_t)1 << 31)) return SP_OK;
    if (mode == 0 && (n < ((int64_t)1 << 20) || key_bits < 24)) return SP_OK;
    const uint32_t tiles1 = (uint32_t)((n + kTile - 1) / kTile);
    uint32_t *ctr = (uint32_t *)tmp.get((size_t)256 * (tiles1 + 256) * 4);
    uint32_t *samp = (uint32_t *)tmp.get((size_t)(kSub + 16) * 4);
    if (!ctr || !samp) return SP_ERR_ALLOC;
    SP_TRY(spmi_fill_zero(samp, (size_t)(kSub + 16) * 4, st));
    plan->ctr = ctr;
    plan->samp = samp;
    plan->tiles = tiles1;
    plan->digit_shift = key_bits > 8 ? key_bits - 8 : 0;
    plan->samp_shift = key_bits > 16 ? key_bits - 16 : 0;
    return SP_OK;
}

sp_status spmi_msd_sort_suits(const uint64_t *keys, int64_t n, int key_bits, sp_scratch &tmp, hipStream_t st, uint32_t *samp_ready, bool *suits)
{
    *suits = false;
    if (n < ((int64_t)1 << 20) || n >= ((int64_t)1 << 31) || key_bits < 24) return SP_OK;
    uint32_t *samp = samp_ready;
    if (!samp) {
        samp = (uint32_t *)tmp.get((size_t)(kSub + 16) * 4);
        if (!samp) return SP_ERR_ALLOC;
        SP_TRY(spmi_fill_zero(samp, (size_t)(kSub + 16) * 4, st));
        const int64_t samples = (n + 63) / 64;
        hipLaunchKernelGGL(msd_sample_kernel, dim3((unsigned)((samples + 255) / 256)), dim3(256), 0, st, keys, n, key_bits - 16, samp);
    }
    unsigned long long *summary = (unsigned long long *)(samp + kSub);       // zero so far
    hipLaunchKernelGGL(msd_sample_summary_kernel, dim3(64), dim3(256), 0, st, (const uint32_t *)samp, summary);
    SP_HIP(hipGetLastError());
    unsigned long long h[2] = {0, 0};
    SP_HIP(hipMemcpyAsync(h, summary, 16, hipMemcpyDeviceToHost, st));
    SP_HIP(hipStreamSynchronize(st));
    // a finishing block that gets more than it can hold in the LDS sorts its range alone through device memory: fine for a
    // tenth of the entries spread over many blocks, not for one block with a large share of them
    *suits = (double)h[0] <= 0.10 * (double)n && h[1] <= (unsigned long long)(8 * kCap);
    return SP_OK;
}

sp_status spmi_msd_sort_pairs(uint64_t *keys, const void *vals, int payload_bytes, int64_t n, int key_bits, sp_scratch &tmp, hipStream_t st,
                              uint32_t *ctr_ready, uint64_t **keys_out, const void **vals_out)
{
    if (payload_bytes == 4)
        return msd_sort_t<uint32_t>(keys, (const uint32_t *)vals, n, key_bits, tmp, st, ctr_ready, keys_out, (const uint32_t **)vals_out);
    return msd_sort_t<unsigned long long>(keys, (const unsigned long long *)vals, n, key_bits, tmp, st, ctr_ready, keys_out,
                                          (const unsigned long long **)vals_out);
}

std::atomic<int> g_pack_sort_mode{0};

sp_status spmi_radix_sort_pairs(uint64_t *keys, const void *vals, int payload_bytes, int64_t n, int key_bits, sp_scratch &tmp, hipStream_t st,
                                uint64_t **keys_out, const void **vals_out)
{
    if (payload_bytes == 4) return lsd_sort_t<uint32_t>(keys, (const uint32_t *)vals, n, key_bits, tmp, st, keys_out, (const uint32_t **)vals_out);
    return lsd_sort_t<unsigned long long>(keys, (const unsigned long long *)vals, n, key_bits, tmp, st, keys_out, (const unsigned long long **)vals_out);
}

sp_status spmi_sort_pairs(uint64_t *keys, const void *vals, int payload_bytes, int64_t n, int key_bits, sp_scratch &tmp, hipStream_t st,
                          const sp_msd_plan *plan, uint64_t **keys_out, const void **vals_out)
{
    const int mode = g_pack_sort_mode.load(std::memory_order_relaxed);
    uint32_t *ctr = plan ? plan->ctr : nullptr, *samp = plan ? plan->samp : nullptr;
    bool msd = false;
    if (mode == 2) msd = n >= 1 && n < ((int64_t)1 << 31);
    else if (mode == 0) SP_TRY(spmi_msd_sort_suits(keys, n, key_bits, tmp, st, samp, &msd));
    if (msd) return spmi_msd_sort_pairs(keys, vals, payload_bytes, n, key_bits, tmp, st, ctr, keys_out, vals_out);
    return spmi_radix_sort_pairs(keys, vals, payload_bytes, n, key_bits, tmp, st, keys_out, vals_out);
}
