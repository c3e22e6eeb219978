// microbenchmark: does a buffer that one kernel wrote come back faster than HBM bandwidth when the next kernel reads it
// (the 256 MB last-level cache in front of the memory), with or without other data streamed in between?  Plain grid-stride
// kernels with 16-byte accesses; every kernel is timed with its own pair of HIP events (so small buffers include the
// launch gap).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstdint>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)
typedef double d2 __attribute__((ext_vector_type(2)));
__global__ __launch_bounds__(256) void wr(d2 *p, int64_t n, double v)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = (d2){v, v};
}
__global__ __launch_bounds__(256) void rd(const d2 *p, int64_t n, double *out)
{
    d2 acc = {0, 0};
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) acc += p[i];
    if (acc[0] + acc[1] == 1.2345) out[0] = acc[0];
}
int main()
{
    const int64_t MB = 1 << 20;
    d2 *P, *Q; double *out;
    CK(hipMalloc(&P, 256 * MB)); CK(hipMalloc(&Q, 2048 * MB)); CK(hipMalloc(&out, 64));
    CK(hipMemset(Q, 0, 2048 * MB)); CK(hipMemset(P, 0, 256 * MB));
    hipEvent_t ev[4]; for (auto &evt : ev) CK(hipEventCreate(&evt));
    const int G = 2048;
    for (int64_t S : {16, 32, 64, 128, 256}) for (int64_t T : {0, 64, 128, 256, 512}) {
        double tw = 0, tq = 0, tr = 0; int64_t qoff = 0; const int reps = 20;
        for (int it = 0; it < reps + 3; ++it) {
            CK(hipEventRecord(ev[0], 0));
            hipLaunchKernelGGL(wr, dim3(G), dim3(256), 0, 0, P, S * MB / 16, (double)it);
            CK(hipEventRecord(ev[1], 0));
            if (T) hipLaunchKernelGGL(rd, dim3(G), dim3(256), 0, 0, (const d2 *)((char *)Q + qoff * MB), T * MB / 16, out);
            CK(hipEventRecord(ev[2], 0));
            hipLaunchKernelGGL(rd, dim3(G), dim3(256), 0, 0, (const d2 *)P, S * MB / 16, out);
            CK(hipEventRecord(ev[3], 0)); CK(hipEventSynchronize(ev[3]));
            qoff = (qoff + T) % (2048 - 512);
            if (it < 3) continue;
            float a, b, c; CK(hipEventElapsedTime(&a, ev[0], ev[1])); CK(hipEventElapsedTime(&b, ev[1], ev[2])); CK(hipEventElapsedTime(&c, ev[2], ev[3]));
            tw += a; tq += b; tr += c;
        }
        printf("P %3lld MB, streamed between %3lld MB: write P %.2f TB/s, stream %.2f TB/s, read P back %.2f TB/s\n", (long long)S, (long long)T,
               S * MB / (tw / reps * 1e-3) / 1e12, T ? T * MB / (tq / reps * 1e-3) / 1e12 : 0.0, S * MB / (tr / reps * 1e-3) / 1e12);
        fflush(stdout);
    }
    return 0;
}
