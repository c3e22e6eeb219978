// microbenchmark: random gather throughput from a table of n doubles, and plain streaming
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstdint>
#include <vector>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("hip error %d at %d\n", (int)e, __LINE__); exit(1);} } while (0)

template <int PER>
__global__ __launch_bounds__(256) void gather_k(const int* __restrict__ idx, const double* __restrict__ x, double* __restrict__ out, int64_t n)
{
    int64_t base = ((int64_t)blockIdx.x * 256) * PER + threadIdx.x;
    int k[PER]; double s = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) k[i] = idx[base + i * 256];
#pragma unroll
    for (int i = 0; i < PER; ++i) s += x[k[i]];
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}
template <int PER>
__global__ __launch_bounds__(256) void stream_k(const int* __restrict__ idx, const double* __restrict__ val, double* __restrict__ out, int64_t n)
{
    int64_t base = ((int64_t)blockIdx.x * 256) * PER + threadIdx.x;
    double s = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) s += val[base + i * 256] * (double)idx[base + i * 256];
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}
// gather + stream (the SpMV phase A without reduction)
template <int PER>
__global__ __launch_bounds__(256) void spmv_a_k(const int* __restrict__ idx, const double* __restrict__ val, const double* __restrict__ x, double* __restrict__ out, int64_t n)
{
    int64_t base = ((int64_t)blockIdx.x * 256) * PER + threadIdx.x;
    int k[PER]; double v[PER]; double s = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) { k[i] = idx[base + i * 256]; v[i] = val[base + i * 256]; }
#pragma unroll
    for (int i = 0; i < PER; ++i) s += v[i] * x[k[i]];
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}
// float table gather (4-byte elements) to see if element size matters
template <int PER>
__global__ __launch_bounds__(256) void gatherf_k(const int* __restrict__ idx, const float* __restrict__ x, float* __restrict__ out, int64_t n)
{
    int64_t base = ((int64_t)blockIdx.x * 256) * PER + threadIdx.x;
    int k[PER]; float s = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) k[i] = idx[base + i * 256];
#pragma unroll
    for (int i = 0; i < PER; ++i) s += x[k[i]];
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}

static uint64_t rng = 88172645463325252ull;
static inline uint64_t xs() { rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17; return rng; }

int main()
{
    const int64_t N = 16 << 20;   // gathers
    std::vector<int> h(N);
    int *idx; double *x, *val, *out;
    CK(hipMalloc(&idx, N * 4)); CK(hipMalloc(&val, N * 8)); CK(hipMalloc(&out, N * 8));
    CK(hipMalloc(&x, (64 << 20) * 8ull));
    CK(hipMemset(x, 0, (64 << 20) * 8ull)); CK(hipMemset(val, 0, N * 8));
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    for (int64_t tab : {1ll << 14, 1ll << 17, 1ll << 18, 1ll << 19, 1ll << 20, 1ll << 21, 1ll << 23, 1ll << 25}) {
        for (int64_t i = 0; i < N; ++i) h[i] = (int)(xs() % tab);
        CK(hipMemcpy(idx, h.data(), N * 4, hipMemcpyHostToDevice));
        auto run = [&](const char* name, auto launch, double bytes) {
            for (int i = 0; i < 3; ++i) launch();
            CK(hipEventRecord(e0));
            for (int i = 0; i < 20; ++i) launch();
            CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
            float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ms /= 20;
            printf("table %8.2f MB  %-14s %8.1f us  %7.1f Ggather/s  %7.1f GB/s(alg)\n", tab * 8 / 1048576.0, name, ms * 1e3, N / (ms * 1e-3) / 1e9, bytes / (ms * 1e-3) / 1e9);
        };
        run("gather8 per8", [&] { hipLaunchKernelGGL(gather_k<8>, dim3(N / 2048), dim3(256), 0, 0, idx, x, out, N); }, N * 4.0);
        run("gather8 per16", [&] { hipLaunchKernelGGL(gather_k<16>, dim3(N / 4096), dim3(256), 0, 0, idx, x, out, N); }, N * 4.0);
        run("gather8 per4", [&] { hipLaunchKernelGGL(gather_k<4>, dim3(N / 1024), dim3(256), 0, 0, idx, x, out, N); }, N * 4.0);
        run("gather4 per8", [&] { hipLaunchKernelGGL(gatherf_k<8>, dim3(N / 2048), dim3(256), 0, 0, idx, (const float*)x, (float*)out, N); }, N * 4.0);
        run("spmvA per8", [&] { hipLaunchKernelGGL(spmv_a_k<8>, dim3(N / 2048), dim3(256), 0, 0, idx, val, x, out, N); }, N * 12.0);
    }
    {
        auto launch = [&] { hipLaunchKernelGGL(stream_k<8>, dim3(N / 2048), dim3(256), 0, 0, idx, val, out, N); };
        for (int i = 0; i < 3; ++i) launch();
        CK(hipEventRecord(e0));
        for (int i = 0; i < 20; ++i) launch();
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
        float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ms /= 20;
        printf("stream only (12 B/nnz): %.1f us  %.1f GB/s\n", ms * 1e3, N * 12.0 / (ms * 1e-3) / 1e9);
    }
    return 0;
}
