// microbenchmark: can one block hide bandwidth-bound streaming behind address-unit-bound gathering?  Some waves of every
// 1024-thread block stream (16 bytes of values + indices per lane, a gather from an LDS table, a 16-byte store: the first
// pass of the binned SpMV), the others gather 8-byte elements of a vector through the vector memory path (512 entries per
// wave and round, indices and values read coalesced, the gathers from 2 MB slices that stay in the L2: the column-segmented
// SpMV without its row logic).  Each role is timed alone and both together.  No sparse-matrix arithmetic beyond that.
// arguments: streamed entries, gathered entries, blocks.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <cstdint>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)
constexpr int PW = 8192;
typedef double d2 __attribute__((ext_vector_type(2)));
typedef uint16_t u2 __attribute__((ext_vector_type(2)));

// waves [0, SW): stream role over bin entries [ba, bb) of this block; waves [SW, 16): gather role over rest entries.
template <int SW>
__global__ __launch_bounds__(1024) void fused(const double *bval, const uint16_t *lcol, double *prod, int64_t nb_per_block,
                                              const double *rval, const int32_t *rcol, int64_t nr, const double *x, double *out, int mode)
{
    __shared__ double xs[PW];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    for (int i = tid; i < PW; i += 1024) xs[i] = x[i];
    __syncthreads();
    if (wave < SW) {
        if (!(mode & 1)) return;
        const int64_t a = (int64_t)blockIdx.x * nb_per_block, b = a + nb_per_block;
        const d2 *vv = (const d2 *)(bval + a);
        const u2 *cc = (const u2 *)(lcol + a);
        d2 *pp = (d2 *)(prod + a);
        const int64_t nvec = (b - a) / 2;
        constexpr int T = SW * 64;
        for (int64_t j = tid; j + T < nvec; j += 2 * T) {
            d2 v0 = vv[j], v1 = vv[j + T];
            u2 c0 = cc[j], c1 = cc[j + T];
            d2 r0, r1;
            r0[0] = v0[0] * xs[c0[0]]; r0[1] = v0[1] * xs[c0[1]];
            r1[0] = v1[0] * xs[c1[0]]; r1[1] = v1[1] * xs[c1[1]];
            pp[j] = r0; pp[j + T] = r1;
        }
    } else {
        if (!(mode & 2)) return;
        // windows of 512 entries per wave, strided over the whole grid so that all blocks are in the same region at a time
        const int gw = 16 - SW;
        const int64_t nwin = nr / 512;
        double acc = 0;
        for (int64_t w = (int64_t)blockIdx.x * gw + (wave - SW); w < nwin; w += (int64_t)gridDim.x * gw) {
            const int64_t s = w * 512;
            int32_t c[8]; double v[8], xv[8];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int64_t p = s + (int64_t)(t * 64 + lane) * 2;
                c[2 * t] = rcol[p]; c[2 * t + 1] = rcol[p + 1];
                v[2 * t] = rval[p]; v[2 * t + 1] = rval[p + 1];
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) xv[i] = x[c[i]];
#pragma unroll
            for (int i = 0; i < 8; ++i) acc += v[i] * xv[i];
        }
        out[(int64_t)blockIdx.x * 1024 + tid] = acc;
    }
}

int main(int argc, char **argv)
{
    const int64_t NB = argc > 1 ? atoll(argv[1]) : 5600000, NR = argc > 2 ? atoll(argv[2]) : 11200000;
    const int blocks = argc > 3 ? atoi(argv[3]) : 256;
    const int64_t n = 1 << 20, slice = 1 << 18;
    const int64_t nbpb = (NB / blocks) & ~(int64_t)3;
    std::vector<double> hv(NB > NR ? NB : NR);
    for (auto &v : hv) v = 1.0;
    std::vector<uint16_t> hl(NB);
    std::vector<int32_t> hc(NR);
    uint64_t s = 88172645463325252ull;
    auto rnd = [&]() { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return s; };
    for (auto &c : hl) c = (uint16_t)(rnd() % PW);
    const int64_t nslices = 3;
    for (int64_t i = 0; i < NR; ++i) hc[i] = (int32_t)((n - nslices * slice) + (i * nslices / NR) * slice + (int64_t)(rnd() % slice));
    double *bval, *prod, *rval, *x, *out; uint16_t *lcol; int32_t *rcol;
    CK(hipMalloc(&bval, NB * 8)); CK(hipMalloc(&prod, NB * 8)); CK(hipMalloc(&lcol, NB * 2));
    CK(hipMalloc(&rval, NR * 8)); CK(hipMalloc(&rcol, NR * 4)); CK(hipMalloc(&x, n * 8)); CK(hipMalloc(&out, (int64_t)blocks * 1024 * 8));
    CK(hipMemcpy(bval, hv.data(), NB * 8, hipMemcpyHostToDevice)); CK(hipMemcpy(rval, hv.data(), NR * 8, hipMemcpyHostToDevice));
    CK(hipMemcpy(lcol, hl.data(), NB * 2, hipMemcpyHostToDevice)); CK(hipMemcpy(rcol, hc.data(), NR * 4, hipMemcpyHostToDevice));
    CK(hipMemset(x, 0, n * 8));
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    auto run = [&](auto kern, const char *name) {
        for (int mode = 1; mode <= 3; ++mode) {
            for (int i = 0; i < 5; ++i) hipLaunchKernelGGL(kern, dim3(blocks), dim3(1024), 0, 0, bval, lcol, prod, nbpb, rval, rcol, NR, x, out, mode);
            CK(hipEventRecord(e0, 0));
            for (int i = 0; i < 50; ++i) hipLaunchKernelGGL(kern, dim3(blocks), dim3(1024), 0, 0, bval, lcol, prod, nbpb, rval, rcol, NR, x, out, mode);
            CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1));
            float ms; CK(hipEventElapsedTime(&ms, e0, e1));
            printf("%s mode %d (%s): %.1f us\n", name, mode, mode == 1 ? "stream waves only" : mode == 2 ? "gather waves only" : "both", ms / 50 * 1e3);
            fflush(stdout);
        }
    };
    printf("bin entries %lld, rest entries %lld, blocks %d\n", (long long)NB, (long long)NR, blocks);
    run(fused<8>, "8 stream + 8 gather waves");
    run(fused<4>, "4 stream + 12 gather waves");
    run(fused<12>, "12 stream + 4 gather waves");
    return 0;
}
