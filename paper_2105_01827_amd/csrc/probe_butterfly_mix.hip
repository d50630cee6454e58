// Microbenchmark: issue rate of the instruction mix the Perm kernel's transforms are made of -- lazy forward
// butterflies (a 13-instruction multiplication by a constant with its precomputed quotient, one 64-bit add, one
// 64-bit subtract-and-add), with 1, 2 or 4 independent butterflies per thread and 2, 3 or 8 workgroups per
// compute unit (LDS padding sets the residency), no memory traffic.  Prints lane-operations per second.
// Build: hipcc --offload-arch=gfx950 -O3 -o probe_butterfly_mix probe_butterfly_mix.hip
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
typedef unsigned long long u64; typedef unsigned u32;
__device__ __forceinline__ u64 mad_u64(u32 a, u32 b, u64 c) { u64 r, carry; asm("v_mad_u64_u32 %0, %1, %2, %3, %4" : "=v"(r), "=s"(carry) : "v"(a), "v"(b), "v"(c)); return r; }
__device__ __forceinline__ u64 mul_u64(u32 a, u32 b) { u64 r, carry; asm("v_mad_u64_u32 %0, %1, %2, %3, 0" : "=v"(r), "=s"(carry) : "v"(a), "v"(b)); return r; }
__device__ __forceinline__ u64 mulhi64_dev(u64 y, u64 s) {
    const u32 y0 = (u32)y, y1 = (u32)(y >> 32), s0 = (u32)s, s1 = (u32)(s >> 32);
    const u64 B = mad_u64(y0, s1, (u64)__umulhi(y0, s0));
    u64 C, carry;
    asm("v_mad_u64_u32 %0, %1, %2, %3, %4" : "=v"(C), "=s"(carry) : "v"(y1), "v"(s0), "v"(B));
    u32 top;
    asm("v_cndmask_b32_e64 %0, 0, 1, %1" : "=v"(top) : "s"(carry));
    return mad_u64(y1, s1, ((u64)top << 32) | (u32)(C >> 32));
}
struct NegQ { u32 lo, hi; };
__device__ __forceinline__ u64 mul_const(u64 y, u64 w, u64 ws, NegQ nq) {
    const u64 h = mulhi64_dev(y, ws);
    const u32 y0 = (u32)y, y1 = (u32)(y >> 32), w0 = (u32)w, w1 = (u32)(w >> 32);
    const u32 h0 = (u32)h, h1 = (u32)(h >> 32);
    u64 u = mul_u64(y0, w1);
    u = mad_u64(y1, w0, u);
    u = mad_u64(h0, nq.hi, u);
    u = mad_u64(h1, nq.lo, u);
    u64 t = mul_u64(y0, w0);
    t = mad_u64(h0, nq.lo, t);
    u32 hi;
    asm("v_add_u32 %0, %1, %2" : "=v"(hi) : "v"((u32)(t >> 32)), "v"((u32)u));
    return ((u64)hi << 32) | (u32)t;
}
template <int ILP, int PAD>
__global__ __launch_bounds__(256) void k(u64 *out, u64 w, u64 ws, u32 nlo, u32 nhi, u64 q2, int iters) {
    __shared__ u64 pad[PAD];
    if (iters < 0) pad[threadIdx.x] = w;     // keeps the array alive
    NegQ nq{nlo, nhi};
    u64 x[ILP], y[ILP];
    for (int i = 0; i < ILP; ++i) { x[i] = threadIdx.x + i; y[i] = threadIdx.x * 3 + i; }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < ILP; ++i) {      // lazy forward butterfly: 17 instructions
                const u64 v = mul_const(y[i], w, ws, nq);
                y[i] = x[i] - v + q2;
                x[i] = x[i] + v;
            }
    }
    u64 s = 0;
    for (int i = 0; i < ILP; ++i) s += x[i] ^ y[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s + (iters < 0 ? pad[0] : 0);
}
template <int ILP, int PAD> void run(int wgs, const char *name) {
    const int iters = 20000;
    u64 *d; hipMalloc(&d, sizeof(u64) * 256 * 4096);
    const u64 q = 1152921500113727489ull, w = 123456789012345ull;
    const u64 ws = (u64)((((unsigned __int128)w) << 64) / q);
    const u64 neg = 0 - q;
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    float ms = 0;
    for (int rep = 0; rep < 3; ++rep) {
        hipEventRecord(e0);
        hipLaunchKernelGGL((k<ILP, PAD>), dim3(wgs), dim3(256), 0, 0, d, w, ws, (u32)neg, (u32)(neg >> 32), 2 * q, iters);
        hipEventRecord(e1); hipEventSynchronize(e1);
        hipEventElapsedTime(&ms, e0, e1);
    }
    const double ops = (double)wgs * 256 * iters * 4 * ILP * 17;
    printf("%s: ILP %d, %d workgroups: %.2f ms, %.2f T lane-ops/s (%.2f of 39.32)\n", name, ILP, wgs, ms, ops / ms / 1e9, ops / ms / 1e9 / 39.32);
    hipFree(d);
}
int main() {
    run<4, 6272>(768, "3 WG/CU (50 KB LDS each)");
    run<4, 8192>(512, "2 WG/CU (64 KB LDS each)");
    run<2, 6272>(768, "3 WG/CU");
    run<1, 6272>(768, "3 WG/CU");
    run<4, 64>(2048, "8 WG/CU");
    return 0;
}
