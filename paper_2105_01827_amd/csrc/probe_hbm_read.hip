// Microbenchmark: what a kernel that only streams a large array out of HBM reaches on this part, for the two
// access shapes the multiply-accumulate of a one-input convolution can take over its encoded kernels
// (1.2 GB per 3x3 ResNet layer, read once):
//   linear   every workgroup walks a contiguous range with 16-byte loads per lane;
//   sliced   a wavefront owns `span` consecutive words of every polynomial of one row and walks the row's
//            polynomials (stride n words), 8- or 16-byte loads per lane: the multiply-accumulate's shape.
// Prints GB/s for each.  Build: hipcc --offload-arch=gfx950 -O3 -o probe_hbm_read probe_hbm_read.hip
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

typedef unsigned long long u64;

__global__ __launch_bounds__(256) void read_linear(const ulonglong2 *src, size_t per_block, u64 *out) {
    const ulonglong2 *p = src + (size_t)blockIdx.x * per_block;
    u64 s = 0;
    for (size_t k = threadIdx.x; k < per_block; k += 4 * 256) {
        ulonglong2 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = p[k + u * 256];      // per_block is a multiple of 1024
#pragma unroll
        for (int u = 0; u < 4; ++u) s += v[u].x ^ v[u].y;
    }
    if (s == 0x1234567) out[threadIdx.x] = s;                   // keeps the loads alive, practically never taken
}

// rows x terms polynomials of n words; workgroup = WAVES wavefronts on WAVES rows and the same slice of
// 64*VEC words; UNROLL terms in flight per wavefront.
template <int VEC, int WAVES, int UNROLL>
__global__ __launch_bounds__(64 * WAVES) void read_sliced(const u64 *src, int terms, int n, u64 *out) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t row = (size_t)blockIdx.y * WAVES + wave;
    const u64 *p = src + row * terms * n + ((size_t)blockIdx.x * 64 + lane) * VEC;
    u64 s = 0;
    for (int e = 0; e < terms; e += UNROLL) {
        u64 v[UNROLL][VEC];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            if (VEC == 2) {
                const ulonglong2 t = *reinterpret_cast<const ulonglong2 *>(p + (size_t)(e + u) * n);
                v[u][0] = t.x; v[u][VEC - 1] = t.y;
            } else {
                v[u][0] = p[(size_t)(e + u) * n];
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
#pragma unroll
            for (int k = 0; k < VEC; ++k) s += v[u][k];
    }
    if (s == 0x1234567) out[threadIdx.x] = s;
}

template <typename F>
double time_ms(F launch, int reps) {
    hipEvent_t e0, e1;
    hipEventCreate(&e0); hipEventCreate(&e1);
    launch();
    hipDeviceSynchronize();
    hipEventRecord(e0, 0);
    for (int r = 0; r < reps; ++r) launch();
    hipEventRecord(e1, 0);
    hipEventSynchronize(e1);
    float ms = 0;
    hipEventElapsedTime(&ms, e0, e1);
    return ms / reps;
}

int main() {
    const int n = 2048, rows = 128, terms = 576;                // 128 x 576 polynomials of 16 KiB = 1.2 GB
    const size_t words = (size_t)rows * terms * n, bytes = words * 8;
    u64 *d, *out;
    if (hipMalloc(&d, bytes) != hipSuccess || hipMalloc(&out, 4096) != hipSuccess) { std::printf("no device\n"); return 1; }
    hipMemset(d, 1, bytes);
    const int reps = 20;
    for (int blocks : {1024, 4096, 8192}) {
        const size_t per_block = words / 2 / blocks;
        const double ms = time_ms([&] { hipLaunchKernelGGL(read_linear, dim3(blocks), dim3(256), 0, 0, (const ulonglong2 *)d, per_block, out); }, reps);
        std::printf("linear, %5d workgroups of 256                     %7.1f GB/s\n", blocks, bytes / ms / 1e6);
    }
#define SLICED(VEC, WAVES, UNROLL)                                                                                   \
    {                                                                                                                \
        const dim3 grid(n / (64 * VEC), rows / WAVES);                                                               \
        const double ms = time_ms([&] { hipLaunchKernelGGL((read_sliced<VEC, WAVES, UNROLL>), grid, dim3(64 * WAVES), 0, 0, d, terms, n, out); }, reps); \
        std::printf("sliced, %d B/lane, %d rows/workgroup, %d terms in flight  %7.1f GB/s  (%u workgroups)\n", 8 * VEC, WAVES, UNROLL, \
                    bytes / ms / 1e6, grid.x * grid.y);                                                               \
    }
    SLICED(1, 4, 1) SLICED(1, 4, 4) SLICED(1, 4, 8) SLICED(1, 1, 8)
    SLICED(2, 4, 1) SLICED(2, 4, 4) SLICED(2, 4, 8) SLICED(2, 1, 4) SLICED(2, 1, 8) SLICED(2, 2, 8)
    std::printf("published HBM3E peak: 8000 GB/s\n");
    hipFree(d); hipFree(out);
    return 0;
}
