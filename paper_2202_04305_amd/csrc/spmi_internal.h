// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <type_traits>
#include <atomic>
#include <vector>
#include "spmi.h"
#include "spmi_bench.h"

struct sp_encoding {
    int rank;
    int lt[SP_MAX_RANK];
    int perm[SP_MAX_RANK];   // perm[l] = dimension stored at level l
    int pw, cw;              // widths the kernels work on: 32 or 64
    int pw_store, cw_store;  // widths asked for (8, 16, 32, 64): what sp_pos / sp_crd hand out
};

// Row blocks of the streaming SpMV: block b covers rows [rowblk[b], rowblk[b+1]) of the
// outer level; built once at pack time from pos of the innermost level.
struct sp_rowblocks {
    void *start = nullptr;   // DEVICE int32[nblocks + 1]
    void *carry = nullptr;   // DEVICE value-typed[nblocks]: partial sums of rows that cross block boundaries
    int64_t nblocks = 0;
};

// Column-segmented copy for SpMV with a large x: the stored entries regrouped by column panel
// (panel = column >> shift), each panel a CSR over all rows, so that the x slice a panel gathers
// from stays in the per-XCD L2.  `seg` is a CSR tensor over panels*nrows virtual rows.
struct sp_segments {
    sp_tensor *seg = nullptr;
    int panels = 0, shift = 0;
    int64_t nrows = 0;
    void *partial = nullptr;          // DEVICE value-typed[panels * nrows]: per-panel results before they are added up
};

// Binned copy for SpMV with a large x and scattered columns: the stored entries regrouped into buckets (column panel
// of 2^pshift columns, row block of 2^rshift stored rows), panel-major, rows ascending inside a bucket.  Every entry keeps
// its value, its column inside the panel and its row inside the row block in 16 bits each.  The product runs in two
// streaming passes: one multiplies a panel's entries by the panel's slice of x held in LDS and writes the products in
// place (`prod`), the other adds a row block's products up in an LDS slice of y.  No gather ever leaves the LDS.
struct sp_bins {
    // Entries regrouped into buckets (column panel, row block), every bucket padded to a multiple of 8 entries (np in all).
    // Panel-major arrays (buckets of a panel side by side, rows ascending inside a bucket):
    void *val = nullptr;              // DEVICE value-typed[np]; padding 0
    uint16_t *lcol = nullptr;         // DEVICE [np]: column - panel * 2^pshift; padding 2^pshift
    uint32_t *gdst = nullptr;         // DEVICE [np / 8]: group of 8 entries -> its group in the row-block-major arrays
    int64_t *pstart = nullptr;        // DEVICE [panels + 1]: first entry of each panel
    // Row-block-major arrays (buckets of a row block side by side):
    void *prod = nullptr;             // DEVICE value-typed[np]: the products of the running call
    uint16_t *lrow = nullptr;         // DEVICE [np]: stored row - rowblock * 2^rshift; padding 0
    int64_t *rbstart = nullptr;       // DEVICE [rowblocks + 1]: first entry of each row block
    int64_t nnz = 0, np = 0, nrows = 0;   // entries, entries with padding, stored rows
    int panels = 0, rowblocks = 0, pieces = 0;
};


struct sp_tensor {
    sp_encoding enc;
    int dtype;
    int64_t shape[SP_MAX_RANK];
    int64_t size[SP_MAX_RANK];       // by level
    void *pos[SP_MAX_RANK];          // DEVICE, nullptr for dense levels
    int64_t npos[SP_MAX_RANK];
    void *crd[SP_MAX_RANK];
    int64_t ncrd[SP_MAX_RANK];
    void *pos_narrow[SP_MAX_RANK];   // DEVICE copies in 8 or 16 bits when such a width was asked for, else nullptr
    void *crd_narrow[SP_MAX_RANK];
    void *values;
    int64_t nvalues;
    int64_t nnz;
    int64_t max_segment;
    sp_alloc_fn alloc;
    sp_free_fn free_;
    void *ctx;
    // Derived state: tables, regrouped copies and scratch that the product kernels use.  None of it is part of the paper's
    // storage; sp_pack builds some of it, sp_prepare (or, lazily, the first product that needs it) the rest.  It is a cache
    // in the C++ sense, hence `mutable`: a product takes the handle as const and may still fill it in.
    mutable sp_rowblocks rowblocks;
    // a dense outer level whose segments are mostly empty: ids and pos entries of the non-empty ones (else nullptr)
    mutable void *nz_rowid, *nz_pos;
    mutable int64_t nz_rows;
    mutable sp_rowblocks nz_rowblocks;
    mutable sp_tensor *transposed;           // CSC/DCSC viewed through a row-major copy (owned)
    mutable sp_segments *segments;           // owned, built on first use
    mutable sp_bins *bins;                   // owned, built on first use
    mutable double scatter;                  // share of stored entries whose successor lies in another 128-byte line of x; < 0: not measured yet
    mutable void *dense_partial;             // DEVICE scratch of the dense-row SpMV (per-chunk partial sums), grown on demand
    mutable size_t dense_partial_bytes;
    mutable void *spmm_carry;                // DEVICE scratch of the SpMM cut by entries (N values per block), grown on demand
    mutable size_t spmm_carry_bytes;
    mutable void *sddmm_bt;                  // DEVICE scratch of the SDDMM: the transposed dense operand (n x K), grown on demand
    mutable size_t sddmm_bt_bytes;
    mutable void *mttkrp_windows;            // DEVICE int32[2 * windows]: fibre and slice holding the first entry of each window (rank 3)
    mutable void *mttkrp_carry;              // DEVICE scratch of the MTTKRP (J values per window), grown on demand
    mutable size_t mttkrp_carry_bytes;
    mutable void *mttkrp_pad[2];             // DEVICE scratch of the MTTKRP: inner / mid factor matrix with rows padded to whole cache lines
    mutable size_t mttkrp_pad_bytes[2];
    mutable int tables_pending;              // rowblocks / non-empty rows not built yet (a result of sp_spgemm): built on first use by a product
    mutable int plan_spmv;                   // SpMV kernel a product with one column runs (1..4); 0 = not decided yet (sp_prepare or the first product decides)
    mutable int lazy_prepares;               // how many products had to build, allocate or decide something first (none after sp_prepare)
    int tune_spmv, tune_csc, tune_spmm, tune_spgemm;
    int profile;
    std::vector<hipEvent_t> *prof_events;   // start/stop pairs, owned
};

extern thread_local int g_last_hip_error;

#define SP_HIP(call)                                            \
    do {                                                        \
        hipError_t e__ = (call);                                \
        if (e__ != hipSuccess) {                                \
            g_last_hip_error = (int)e__;                        \
            return SP_ERR_HIP;                                  \
        }                                                       \
    } while (0)

#define SP_TRY(call)                                            \
    do {                                                        \
        sp_status s__ = (call);                                 \
        if (s__ != SP_OK) return s__;                           \
    } while (0)

// Brackets the main kernel of a product with events when profiling is on.
struct sp_prof_scope {
    const sp_tensor *t; hipStream_t st; hipEvent_t stop = nullptr;
    sp_prof_scope(const sp_tensor *t_, hipStream_t st_) : t(t_), st(st_) {
        if (!t->profile || !t->prof_events) return;
        hipEvent_t a = nullptr;
        if (hipEventCreate(&a) != hipSuccess) return;
        if (hipEventCreate(&stop) != hipSuccess) { (void)hipEventDestroy(a); stop = nullptr; return; }
        (void)hipEventRecord(a, st);
        t->prof_events->push_back(a);
        t->prof_events->push_back(stop);
    }
    ~sp_prof_scope() { if (stop) (void)hipEventRecord(stop, st); }
};

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Device memory through the caller's allocator (or hipMalloc when none was given).
struct sp_mem {
    sp_alloc_fn alloc; sp_free_fn free_; void *ctx;
    void *get(size_t bytes) const;
    void put(void *p) const;
};

// A scope that frees its temporaries on exit.
struct sp_scratch {
    const sp_mem &mem;
    std::vector<void *> ptrs;
    explicit sp_scratch(const sp_mem &m) : mem(m) {}
    ~sp_scratch() { for (void *p : ptrs) mem.put(p); }
    void *get(size_t bytes) {
        void *p = mem.get(bytes ? bytes : 16);
        if (p) ptrs.push_back(p);
        return p;
    }
    // Takes a temporary out of the scope (its new owner frees it through the same allocator); false when p is not one.
    bool release(void *p) {
        for (size_t i = 0; i < ptrs.size(); ++i)
            if (ptrs[i] == p) { ptrs.erase(ptrs.begin() + (long)i); return true; }
        return false;
    }
};

// ---- device helpers shared by the sources ---------------------------------------------------
template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T v, int lane)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        T o = __shfl_up(v, d, 64);
        if (lane >= d) v += o;
    }
    return v;
}

// Lanes of the wave that hold the same 8-bit digit as this lane (among lanes with valid set).  Per bit: the lanes that agree
// with this one are ~(ballot ^ mine), `mine` being all ones or all zeros; m & ~(ballot ^ mine) is one three-input bit
// operation per 32-bit half (truth table 0x90 with m as the first input), five vector instructions per bit in all.
__device__ __forceinline__ uint64_t match_digit(uint32_t d, bool valid)
{
    const uint64_t v = __builtin_amdgcn_ballot_w64(valid);
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const int mine = __builtin_amdgcn_sbfe((int)d, b, 1);
        const uint64_t bb = __builtin_amdgcn_ballot_w64(mine != 0);
        lo = __builtin_amdgcn_bitop3_b32(lo, (uint32_t)bb, (uint32_t)mine, 0x90);
        hi = __builtin_amdgcn_bitop3_b32(hi, (uint32_t)(bb >> 32), (uint32_t)mine, 0x90);
    }
    return ((uint64_t)hi << 32) | lo;
}

// ---- pack.hip ----------------------------------------------------------------------------
// In-place exclusive prefix sum of n elements of width `bits` (32 or 64); data[n-1] afterwards
// holds the sum of the first n-1 inputs.
sp_status spmi_exclusive_scan(void *data, int64_t n, int bits, sp_scratch &tmp, hipStream_t st);
sp_status spmi_fill_zero(void *p, size_t bytes, hipStream_t st);
// ---- sort.hip ----
// Stable radix sort, least significant digit first, of (key, payload) pairs on the low `key_bits` bits taken as whole 8-bit
// digits (so ceil(key_bits / 8) * 8 bits decide), payload of 4 or 8 bytes.  keys: a temporary of `tmp`, overwritten; vals: only
// read.  *keys_out / *vals_out: where the sorted arrays are (temporaries of `tmp`, or the inputs themselves when there was
// nothing to sort).
sp_status spmi_radix_sort_pairs(uint64_t *keys, const void *vals, int payload_bytes, int64_t n, int key_bits, sp_scratch &tmp,
                                hipStream_t st, uint64_t **keys_out, const void **vals_out);
// The same sort (same arguments, same stability) with the most significant digits first: two passes over device memory, the
// rest inside the LDS.  Only for inputs that spmi_msd_sort_suits() accepted: enough entries, keys wide enough, and (from a
// sampled histogram of the top 16 key bits, samp_ready when the caller has it already; synchronises the stream) few entries
// in groups of equal top 16 key bits too large for the LDS, none of them huge.
//
// Whoever makes the keys can fill in, on the way, what the first pass would otherwise read them for (sp_msd_plan, empty when
// this sort is out of the question): for the tile e / kSpmiMsdTile of entry e, ctr[digit * tiles + tile] counts the entries
// whose digit is (key >> digit_shift) & 255 (every word written, zero included), and samp[(key >> samp_shift) & 0xffff]
// counts every 64th entry (e % 64 == 0; samp arrives zeroed).
#ifndef SPMI_SORT_T
#define SPMI_SORT_T 256
#endif
constexpr int kSpmiMsdTile = SPMI_SORT_T * 16;
struct sp_msd_plan { uint32_t *ctr, *samp; uint32_t tiles; int digit_shift, samp_shift; };
sp_status spmi_msd_plan(int64_t n, int key_bits, sp_scratch &tmp, hipStream_t st, sp_msd_plan *plan);
sp_status spmi_msd_sort_suits(const uint64_t *keys, int64_t n, int key_bits, sp_scratch &tmp, hipStream_t st, uint32_t *samp_ready, bool *suits);
sp_status spmi_msd_sort_pairs(uint64_t *keys, const void *vals, int payload_bytes, int64_t n, int key_bits, sp_scratch &tmp, hipStream_t st,
                              uint32_t *ctr_ready, uint64_t **keys_out, const void **vals_out);
// Whichever of the two suits (or the one that sp_pack_sort_mode() of the bench header forces); plan: null, or what
// spmi_msd_plan() handed out and the maker of the keys filled in.
sp_status spmi_sort_pairs(uint64_t *keys, const void *vals, int payload_bytes, int64_t n, int key_bits, sp_scratch &tmp, hipStream_t st,
                          const sp_msd_plan *plan, uint64_t **keys_out, const void **vals_out);
extern std::atomic<int> g_pack_sort_mode;
// ---- pack.hip ----
// The storage of a tensor whose n entries are given as linearised keys (level order, mixed radix over the level sizes)
// with the value bits as payload, both temporaries of `tmp`; entries with equal keys are added up in the order given.
sp_status spmi_pack_keys(const sp_encoding *enc, const int64_t *shape, sp_dtype dt, sp_alloc_fn alloc, sp_free_fn free_, void *ctx,
                         int64_t n, uint64_t *keys, void *payload, sp_scratch &tmp, hipStream_t st, sp_tensor **out);
sp_status spmi_build_rowblocks(const sp_tensor *t, hipStream_t st);
sp_status spmi_build_segments(const sp_tensor *A, int64_t row_bytes, int64_t slice_bytes, hipStream_t st);
#ifndef SPMI_BIN_PSHIFT
#define SPMI_BIN_PSHIFT 13
#endif
#ifndef SPMI_BIN_RSHIFT
#define SPMI_BIN_RSHIFT 11
#endif
constexpr int kSpmiBinPanelShift = SPMI_BIN_PSHIFT;          // columns per panel of the binned copy: 8192 (a 64 KB slice of an f64 x)
constexpr int kSpmiBinRowShift = SPMI_BIN_RSHIFT;            // rows per row block: 2048 (a 16 KB slice of an f64 y)
sp_status spmi_build_bins(const sp_tensor *A, hipStream_t st);
// How scattered the gathers of a product are: the share of stored entries of the innermost level whose successor is 16 or
// more coordinates away (or belongs to the next segment).  Measured once per tensor, then cached; synchronises the first time.
sp_status spmi_column_scatter(const sp_tensor *A, hipStream_t st, double *share);
#ifndef SPMI_ST
#define SPMI_ST 128
#endif
#ifndef SPMI_PER
#define SPMI_PER 8
#endif
constexpr int kSpmiStreamThreads = SPMI_ST;                  // threads per block of the stream kernel
constexpr int kSpmiStreamPer = SPMI_PER;                     // stored entries per thread (even)
constexpr int64_t kSpmiStreamT = kSpmiStreamThreads * kSpmiStreamPer;     // stored entries per block

// keys[e] = linearised key, in the level order of `shaped` (a tensor handle whose enc and size[] are set), of the entry
// with coordinates coords[d][e]; flags[0] != 0 afterwards on the device when a coordinate was out of range.
sp_status spmi_make_keys(const sp_tensor *shaped, const int64_t *const *coords, int64_t n, uint64_t *keys, int *flags, hipStream_t st);
// A new tensor handle with shape, sizes by level and the key width worked out (SP_ERR_TOO_LARGE, SP_ERR_WIDTH as sp_pack
// documents; `entries_in_an_empty_dimension` turns into SP_ERR_COORD_RANGE at its place in that order).
sp_status spmi_new_tensor(const sp_encoding *enc, const int64_t *shape, sp_dtype dt, sp_alloc_fn alloc, sp_free_fn free_, void *ctx,
                          bool entries_in_an_empty_dimension, sp_tensor **out, int *key_bits_out);
// The derived tables of a finished storage (see pack.hip); flags: 64 device bytes, the second half zero; input_flags: HOST
// int[2] that receives flags[0..1] (nothing more is built when one is set), or null.
sp_status spmi_finish_tensor(sp_tensor *t, int *flags, sp_scratch &tmp, hipStream_t st, int *input_flags);
// *out (DEVICE, zero before the call) = the longest of the nseg segments of a pos array of width pw; enqueued only.
sp_status spmi_max_segment_async(const void *pos, int pw, int64_t nseg, unsigned long long *out, hipStream_t st);
// Builds the tables a product kernel reads (row blocks, non-empty rows) when the tensor still lacks them; synchronises then.
sp_status spmi_ensure_tables(const sp_tensor *t, hipStream_t st);
// Hands the tensor out on SP_OK, releases everything it holds otherwise.
sp_status spmi_finish_pack(sp_tensor *t, sp_status status, hipStream_t st, sp_tensor **out);

// ---- api.hip -----------------------------------------------------------------------------
// Builds and keeps the row-major copy of a column-major tensor (A->transposed); no-op when it exists.
sp_status spmi_build_transposed(const sp_tensor *A, hipStream_t st);

// ---- matmul.hip --------------------------------------------------------------------------
sp_status spmi_matmul_rowmajor(const sp_tensor *A, const void *B, int64_t N, int64_t ldb,
                               void *C, int64_t ldc, int accumulate, hipStream_t st);
// Everything a product of a row-major tensor (compressed / dense innermost level) with N columns would otherwise build on
// first use: the kernel choice, regrouped copies, scratch.  May allocate and synchronise; a no-op when nothing is missing.
sp_status spmi_prepare_rowmajor(const sp_tensor *A, int64_t N, hipStream_t st);
sp_status spmi_prepare_dense_inner(const sp_tensor *A, int64_t N, hipStream_t st);
sp_status spmi_matmul_dense_inner(const sp_tensor *A, const void *B, int64_t N, int64_t ldb, void *C, int64_t ldc,
                                  int accumulate, hipStream_t st);
sp_status spmi_matmul_colmajor_scatter(const sp_tensor *A, const void *B, int64_t N, int64_t ldb,
                                       void *C, int64_t ldc, int accumulate, hipStream_t st);
