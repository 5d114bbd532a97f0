// Measurement only (stand-alone program, no part of the library): how fast rows of a matrix are
// fetched when the lanes of a wave read 16-byte pieces in the patterns the assignment kernels use -
// one row per lane, the fp64 and fp32 B-operand layouts (16 rows x 4 lane groups, 32 rows x 2),
// and row-contiguous - from a 1 GB array (HBM) and a 96 MB one (memory-side cache), 8 waves per SIMD.
// Build: hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops
//        row_fetch_bench.hip -o row_fetch_bench      (done by __graft_entry__.build())
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef float floatx4 __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("hip error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)

// MODE 0: lane l walks row (base + l): scattered, one row per lane
// MODE 1: 16 points x 4 groups: lane (n = l % 16, g = l / 16) reads piece 4*it + g of row base + n
// MODE 2: 32 points x 2 groups: lane (n = l % 32, g = l / 32) reads piece 2*it + g of row base + n
// MODE 3: row-contiguous: lane l reads piece it*64 + l of a block of rows laid end to end
template <int MODE>
__global__ __launch_bounds__(256) void fetch(const floatx4 *x, long nrows, int pieces, float *out)
{
    const int lane = threadIdx.x & 63;
    const long wave = ((long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const long nwaves = ((long)gridDim.x * blockDim.x) >> 6;
    floatx4 acc = {0, 0, 0, 0};
    constexpr int RPW = MODE == 0 ? 64 : (MODE == 1 ? 16 : (MODE == 2 ? 32 : 64));  // rows per wave step
    for (long r0 = wave * RPW; r0 + RPW <= nrows; r0 += nwaves * RPW) {
        if (MODE == 0) {
            const floatx4 *p = x + (r0 + lane) * pieces;
#pragma unroll 8
            for (int it = 0; it < pieces; ++it) acc += p[it];
        } else if (MODE == 1) {
            const floatx4 *p = x + (r0 + (lane & 15)) * pieces + (lane >> 4);
#pragma unroll 8
            for (int it = 0; it < pieces; it += 4) acc += p[it];
        } else if (MODE == 2) {
            const floatx4 *p = x + (r0 + (lane & 31)) * pieces + (lane >> 5);
#pragma unroll 8
            for (int it = 0; it < pieces; it += 2) acc += p[it];
        } else {
            const floatx4 *p = x + r0 * pieces + lane;
#pragma unroll 8
            for (int it = 0; it < pieces * 64; it += 64) acc += p[it];
        }
    }
    if (acc[0] + acc[1] + acc[2] + acc[3] == 12345.678f) out[0] = acc[0];
}

template <int MODE>
static void run(const floatx4 *x, long bytes, int rowbytes, float *out, const char *name)
{
    const int pieces = rowbytes / 16;
    const long nrows = bytes / rowbytes;
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    for (int i = 0; i < 3; ++i) hipLaunchKernelGGL(fetch<MODE>, dim3(2048), dim3(256), 0, 0, x, nrows, pieces, out);
    CK(hipEventRecord(e0));
    const int reps = 10;
    for (int i = 0; i < reps; ++i) hipLaunchKernelGGL(fetch<MODE>, dim3(2048), dim3(256), 0, 0, x, nrows, pieces, out);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    printf("%-34s row %5d B, %6.0f MB: %7.1f us  %6.2f TB/s\n", name, rowbytes, bytes / 1e6, ms / reps * 1e3, bytes / (ms / reps * 1e-3) / 1e12);
    fflush(stdout);
}

int main()
{
    const long big = 1L << 30, small = 96L << 20;  // HBM-sized and memory-side-cache-sized
    floatx4 *x; float *out;
    CK(hipMalloc(&x, big)); CK(hipMalloc(&out, 64));
    CK(hipMemset(x, 0, big));
    for (long bytes : {big, small})
        for (int rb : {128, 512, 4096}) {
            run<0>(x, bytes, rb, out, "one row per lane");
            run<1>(x, bytes, rb, out, "16 rows x 4 lane groups (fp64 B)");
            run<2>(x, bytes, rb, out, "32 rows x 2 lane groups (fp32 B)");
            run<3>(x, bytes, rb, out, "row-contiguous");
        }
    CK(hipFree(x)); CK(hipFree(out));
    return 0;
}
