// microbenchmark: how fast one MI355X delivers whole rows of a dense row-major f64 matrix picked at random, which is what
// bounds SpMM, SDDMM and MTTKRP (one row of a dense operand per stored entry).  A wave takes consecutive row indices from
// a coalesced stream; LR lanes cover a row with one 16-byte load each, 64 / LR rows go side by side, 4 such gathers are
// in flight per lane; the loaded values are summed so that nothing is optimised away.  No sparse-matrix arithmetic.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstdint>
#include <vector>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("hip error %d at %d\n", (int)e, __LINE__); exit(1);} } while (0)

typedef double d2 __attribute__((ext_vector_type(2)));

// rows: cols doubles each (cols even), LR = cols / 2 lanes per row
__global__ __launch_bounds__(256) void row_gather_k(const int *__restrict__ idx, int64_t n, const double *__restrict__ table, int cols,
                                                    double *__restrict__ out)
{
    constexpr int U = 4;
    const int lane = threadIdx.x & 63;
    const int LR = cols / 2, S = 64 / LR;
    const int jl = lane % LR, sl = lane / LR;
    const bool live = sl < S;
    const int64_t per_wave = (int64_t)S * U * 8;                     // 8 rounds of U gathers
    const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t first = w * per_wave;
    d2 acc = (d2)(0);
    for (int r = 0; r < 8; ++r) {
        d2 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t p = first + ((int64_t)r * U + u) * S + sl;
            const int row = (live && p < n) ? idx[p] : idx[first < n ? first : 0];
            v[u] = *(const d2 *)(table + (int64_t)row * cols + jl * 2);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc += v[u];
    }
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = acc[0] + acc[1];
}

static uint64_t rng = 88172645463325252ull;
static inline uint64_t xs() { rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17; return rng; }

int main()
{
    const int64_t NMAX = 64ll << 20;
    std::vector<int> h(NMAX);
    int *idx; double *table, *out;
    const size_t table_bytes = 600ull << 20;
    CK(hipMalloc(&idx, NMAX * 4)); CK(hipMalloc(&table, table_bytes)); CK(hipMalloc(&out, NMAX * 8));
    CK(hipMemset(table, 0, table_bytes));
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    struct shape { int cols; int64_t n; } shapes[] = {{64, 16ll << 20}, {42, 64ll << 20}, {16, 64ll << 20}};
    for (auto sh : shapes) {
        const int64_t row_bytes = sh.cols * 8;
        for (double mb : {1.0, 3.0, 9.7, 32.0, 128.0, 537.0}) {
            const int64_t rows = (int64_t)(mb * 1048576.0 / row_bytes);
            for (int64_t i = 0; i < sh.n; ++i) h[i] = (int)(xs() % (uint64_t)rows);
            CK(hipMemcpy(idx, h.data(), sh.n * 4, hipMemcpyHostToDevice));
            const int S = 64 / (sh.cols / 2);
            const int64_t per_wave = (int64_t)S * 4 * 8;
            const int64_t waves = (sh.n + per_wave - 1) / per_wave;
            const unsigned blocks = (unsigned)((waves + 3) / 4);
            auto launch = [&] { hipLaunchKernelGGL(row_gather_k, dim3(blocks), dim3(256), 0, 0, idx, sh.n, table, sh.cols, out); };
            for (int i = 0; i < 3; ++i) launch();
            CK(hipEventRecord(e0));
            for (int i = 0; i < 10; ++i) launch();
            CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
            float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ms /= 10;
            printf("row %4ld B  table %7.1f MB  %9ld rows gathered  %9.1f us  %7.2f TB/s delivered  %6.2f G rows/s\n", (long)row_bytes, mb,
                   (long)sh.n, ms * 1e3, sh.n * (double)row_bytes / (ms * 1e-3) / 1e12, sh.n / (ms * 1e-3) / 1e9);
        }
    }
    return 0;
}
