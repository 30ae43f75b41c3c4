// Development probe, not part of libpreft.so: how much per-row contiguity does one load/store
// instruction need to stream a row tile at full speed?  No arithmetic: phase 1 reads the x rows of
// a 16-row tile, phase 2 reads and rewrites its y rows (the traffic shape of a LoRA apply).
// A workgroup of W wavefronts owns ROWS rows; wavefront w takes SEG-byte column chunks w, w+W, ...;
// one instruction covers RPI rows x SEG = 1024/RPI bytes, ROWS/RPI instructions cover the tile rows,
// G such groups (different column chunks) are in flight per wavefront.
// Build and run (standalone):
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         paper_2605_14217_amd/csrc/stream_probe.hip -o stream_probe && ./stream_probe
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstdint>
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)

template <int RPI, int G, int WAVES, int ROWS>
__global__ __launch_bounds__(WAVES * 64) void k_shape(const u32x4* __restrict__ x, u32x4* __restrict__ y, int T, int dv)
{
    constexpr int LPR = 64 / RPI;          // lanes per row = vectors per row segment
    constexpr int NI = ROWS / RPI;         // instructions to cover the tile rows for one segment
    __shared__ uint32_t red[WAVES];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row0 = blockIdx.x * ROWS;
    if (row0 >= T) return;
    const int nrows = min(ROWS, T - row0);
    const int sub = lane / LPR, cl = lane % LPR;
    const int nseg = dv / LPR;             // segments per row
    uint32_t s = 0;
    for (int seg = wave; seg + (G - 1) * WAVES < nseg; seg += WAVES * G) {
        u32x4 v[G][NI];
#pragma unroll
        for (int gq = 0; gq < G; ++gq)
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                int r = min(i * RPI + sub, nrows - 1);
                v[gq][i] = x[(size_t)(row0 + r) * dv + (seg + gq * WAVES) * LPR + cl];
            }
#pragma unroll
        for (int gq = 0; gq < G; ++gq)
#pragma unroll
            for (int i = 0; i < NI; ++i) s += v[gq][i][0] ^ v[gq][i][3];
    }
    s = __builtin_amdgcn_readfirstlane(s) & 1;
    if (lane == 0) red[wave] = s;
    __syncthreads();
    uint32_t add = 0;
    for (int w = 0; w < WAVES; ++w) add += red[w];
    for (int seg = wave; seg + (G - 1) * WAVES < nseg; seg += WAVES * G) {
        u32x4 v[G][NI];
#pragma unroll
        for (int gq = 0; gq < G; ++gq)
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                int r = min(i * RPI + sub, nrows - 1);
                v[gq][i] = y[(size_t)(row0 + r) * dv + (seg + gq * WAVES) * LPR + cl];
            }
#pragma unroll
        for (int gq = 0; gq < G; ++gq)
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                int r = min(i * RPI + sub, nrows - 1);
                v[gq][i][0] += add;
                y[(size_t)(row0 + r) * dv + (seg + gq * WAVES) * LPR + cl] = v[gq][i];
            }
    }
}

int main()
{
    const int T = 38411, d = 4096;
    const int dv = d * 2 / 16;
    const size_t n = (size_t)T * dv;
    const int NBUF = 3;
    u32x4 *x[NBUF], *y[NBUF];
    for (int i = 0; i < NBUF; ++i) { CK(hipMalloc(&x[i], n * 16)); CK(hipMalloc(&y[i], n * 16)); CK(hipMemset(x[i], 1, n * 16)); CK(hipMemset(y[i], 2, n * 16)); }
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    auto timeit = [&](const char* name, double bytes, auto launch) {
        for (int i = 0; i < 3; ++i) launch(i % NBUF);
        CK(hipDeviceSynchronize());
        const int iters = 12;
        CK(hipEventRecord(e0));
        for (int i = 0; i < iters; ++i) launch(i % NBUF);
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
        float ms; CK(hipEventElapsedTime(&ms, e0, e1));
        ms /= iters;
        printf("%-44s %8.1f us  %7.1f GB/s\n", name, ms * 1e3, bytes / ms / 1e6); fflush(stdout);
    };
    const double B = (double)n * 16;
    unsigned g16 = (T + 15) / 16, g32 = (T + 31) / 32;
#define RUN(RPI, G, W, ROWS, grid) timeit("shape RPI=" #RPI " G=" #G " W=" #W " rows=" #ROWS, 3 * B, [&](int b) { hipLaunchKernelGGL((k_shape<RPI, G, W, ROWS>), dim3(grid), dim3(W * 64), 0, 0, x[b], y[b], T, dv); })
    RUN(16, 1, 4, 16, g16); RUN(16, 2, 4, 16, g16); RUN(16, 4, 4, 16, g16); RUN(16, 8, 4, 16, g16);
    RUN(8, 1, 4, 16, g16);  RUN(8, 2, 4, 16, g16);  RUN(8, 4, 4, 16, g16);
    RUN(4, 1, 4, 16, g16);  RUN(4, 2, 4, 16, g16);  RUN(4, 4, 4, 16, g16);
    RUN(2, 1, 4, 16, g16);  RUN(2, 2, 4, 16, g16);
    RUN(1, 1, 4, 16, g16);  RUN(1, 2, 4, 16, g16);
    RUN(16, 4, 8, 16, g16); RUN(4, 2, 8, 16, g16); RUN(1, 1, 8, 16, g16);
    RUN(16, 2, 4, 32, g32); RUN(4, 1, 4, 32, g32); RUN(1, 1, 4, 32, g32) ;
    return 0;
}
