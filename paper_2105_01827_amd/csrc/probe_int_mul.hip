// Microbenchmark: issue rate of the 32-bit integer multiply instructions that the
// 64-bit modular arithmetic is built from (v_mul_lo_u32, v_mul_hi_u32,
// v_mad_u64_u32), against a full-rate 32-bit add.  Prints lane-operations per
// second for each.  Build: hipcc --offload-arch=gfx950 -O3 -o probe_int_mul probe_int_mul.hip
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

template <int OP>
__global__ __launch_bounds__(256) void chain(uint32_t *out, uint32_t seed, int iters) {
    // eight independent dependency chains per lane so the issue rate, not the latency, is measured
    uint32_t a[8];
    uint64_t w[8];
    for (int k = 0; k < 8; ++k) { a[k] = seed + threadIdx.x * 8 + k; w[k] = a[k]; }
    const uint32_t m = seed | 1u;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                // every operation feeds on another chain's value so that nothing folds at compile time
                if (OP == 0) a[k] = a[k] * a[(k + 1) & 7];                      // v_mul_lo_u32
                if (OP == 1) a[k] = __umulhi(a[k], a[(k + 1) & 7] | 0x80000000u);   // v_mul_hi_u32 (+ or)
                if (OP == 2) w[k] = (uint64_t)(uint32_t)w[k] * m + w[k];        // v_mad_u64_u32
                if (OP == 3) a[k] = a[k] + (a[(k + 1) & 7] ^ (uint32_t)i);      // v_add_u32 (+ xor)
            }
        }
    }
    uint32_t s = 0;
    for (int k = 0; k < 8; ++k) s += a[k] + (uint32_t)w[k] + (uint32_t)(w[k] >> 32);
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int OP>
double run(uint32_t *d, int blocks, int iters) {
    hipEvent_t e0, e1;
    hipEventCreate(&e0); hipEventCreate(&e1);
    hipLaunchKernelGGL(chain<OP>, dim3(blocks), dim3(256), 0, 0, d, 12345u, 16);
    hipDeviceSynchronize();
    hipEventRecord(e0, 0);
    hipLaunchKernelGGL(chain<OP>, dim3(blocks), dim3(256), 0, 0, d, 12345u, iters);
    hipEventRecord(e1, 0);
    hipEventSynchronize(e1);
    float ms = 0;
    hipEventElapsedTime(&ms, e0, e1);
    const double ops = (double)blocks * 256 * iters * 64;
    return ops / (ms * 1e-3);
}

int main() {
    const int blocks = 256 * 16, iters = 4096;
    uint32_t *d;
    if (hipMalloc(&d, sizeof(uint32_t) * blocks * 256) != hipSuccess) { std::printf("no device\n"); return 1; }
    const char *names[] = {"v_mul_lo_u32", "v_mul_hi_u32(+or)", "v_mad_u64_u32", "v_add_u32(+xor)"};
    double r[4] = {run<0>(d, blocks, iters), run<1>(d, blocks, iters), run<2>(d, blocks, iters), run<3>(d, blocks, iters)};
    for (int k = 0; k < 4; ++k) std::printf("%-20s %8.2f T lane-ops/s\n", names[k], r[k] / 1e12);
    std::printf("full-rate reference: 256 CU x 4 SIMD x 16 lanes x 2.4 GHz = %.2f T lane-ops/s\n", 256 * 4 * 16 * 2.4e9 / 1e12);
    hipFree(d);
    return 0;
}
