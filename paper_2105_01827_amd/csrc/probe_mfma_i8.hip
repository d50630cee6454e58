// Microbenchmark: issue rate of v_mfma_i32_16x16x64_i8 (the instruction of the convolution's matrix-core
// product) with 15 independent accumulators per wavefront, one and two wavefronts per SIMD.  Prints int8 TOP/s
// against the published dense peak.  Build: hipcc --offload-arch=gfx950 -O3 -o probe_mfma_i8 probe_mfma_i8.hip
#include <hip/hip_runtime.h>

#include <cstdio>

typedef int v4i __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void chain(v4i *out, int iters) {
    v4i s[15], a[8], b[8];
    for (int k = 0; k < 15; ++k) s[k] = v4i{0, 0, 0, 0};
    for (int k = 0; k < 8; ++k) {
        a[k] = v4i{(int)threadIdx.x + k, 1, 2, 3};
        b[k] = v4i{(int)threadIdx.x * 3 + k, 5, 6, 7};
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int v = 0; v < 8; ++v)
#pragma unroll
            for (int u = 0; u < 8; ++u) s[u + v] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[u], b[v], s[u + v], 0, 0, 0);
    }
    v4i r = s[0];
    for (int k = 1; k < 15; ++k) r += s[k];
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

int main() {
    v4i *d;
    const int max_blocks = 256 * 2;
    if (hipMalloc(&d, sizeof(v4i) * max_blocks * 256) != hipSuccess) { std::printf("no device\n"); return 1; }
    for (int per_cu : {1, 2}) {
        const int blocks = 256 * per_cu, iters = 2000;
        hipEvent_t e0, e1;
        (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
        hipLaunchKernelGGL(chain, dim3(blocks), dim3(256), 0, 0, d, 10);
        (void)hipDeviceSynchronize();
        (void)hipEventRecord(e0, 0);
        hipLaunchKernelGGL(chain, dim3(blocks), dim3(256), 0, 0, d, iters);
        (void)hipEventRecord(e1, 0);
        (void)hipEventSynchronize(e1);
        float ms = 0;
        (void)hipEventElapsedTime(&ms, e0, e1);
        const double mfmas = (double)blocks * 4 * iters * 64;        // per wavefront: 64 per iteration
        const double ops = mfmas * 16 * 16 * 64 * 2;
        std::printf("%d workgroup(s) of 4 wavefronts per CU: %.1f int8 TOP/s, %.1f cycles per MFMA per SIMD at 2.4 GHz\n", per_cu,
                    ops / (ms * 1e-3) / 1e12, (ms * 1e-3) * 2.4e9 / (mfmas / 1024.0));
    }
    std::printf("published dense int8 peak: 5000 TOP/s\n");
    (void)hipFree(d);
    return 0;
}
