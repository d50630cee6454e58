// Rotate-and-accumulate kernel specialised for n = 2048 and q < 2^60.
//
// One 256-thread workgroup (four wavefronts) owns one polynomial; every thread
// keeps 8 coefficients in registers and runs radix-8 passes (three butterfly
// stages each) on them, so a 2048-point transform is 3 + 3 + 3 + 2 stages with
// only three exchanges through LDS.  The LDS image is padded by one word every
// 32 so that all exchange patterns are bank-conflict free, and two buffers
// alternate so that each exchange needs a single barrier.
//
// Index ownership of register k of thread t in each pass (bits of the
// coefficient index the pass works on):
//   forward:  A bits 8-10: t + 256k | B bits 5-7 | C bits 2-4 | D bits 0-1: 8t + k
//   inverse:  1 bits 0-2: 8t + k    | 2 bits 3-5 | 3 bits 6-8 | 4 bits 9-10: t + 256k
// so the inverse transform of c1 ends exactly where the forward transforms of
// its digits begin, and the digits never leave registers.
//
// Forward butterflies are fully lazy: no conditional subtraction at all except
// one (of 8q) after the seventh stage; values stay below 16q < 2^64.
#include <hip/hip_runtime.h>

#include "gala_internal.h"

namespace gala {
namespace {

constexpr int N = 2048, LOGN = 11, NT = 256, PER = 8;
constexpr int LDS_WORDS = N + N / 32;

__device__ __forceinline__ int pad(int i) { return i + (i >> 5); }
__device__ __forceinline__ int bitrev11(int v) { return (int)(__brev((unsigned)v) >> 21); }
__device__ __forceinline__ int galois_index11(int i, int gal) {
    const int e = ((2 * bitrev11(i) + 1) * gal) & (2 * N - 1);
    return bitrev11((e - 1) >> 1);
}

// x,y -> x + w*y, x - w*y + 2q  without any correction (bound grows by 2q per stage)
__device__ __forceinline__ void bf_fwd(u64 &x, u64 &y, const ulonglong2 t, u64 q, u64 q2) {
    const u64 v = mul_shoup_lazy(y, t.x, t.y, q);
    y = x - v + q2;
    x = x + v;
}
// x,y in [0,2q) -> x + y (below 2q), (x - y)*w (below 2q)
__device__ __forceinline__ void bf_inv(u64 &x, u64 &y, const ulonglong2 t, u64 q, u64 q2) {
    const u64 s = x + y, d = x - y + q2;
    x = csub(s, q2);
    y = mul_shoup_lazy(d, t.x, t.y, q);
}

// Radix-8 forward pass on the three index bits held in the register number
// (bit 2 of k first).  T = (n >> (B+3)) + (index >> (B+3)) selects the twiddles:
// tw[T], tw[2T..2T+1], tw[4T..4T+3].  FIRST = false skips the first stage (the
// last pass of the transform has only two stages).
template <bool FIRST, bool CORRECT>
__device__ __forceinline__ void fwd_pass(u64 (&a)[8], const ulonglong2 *__restrict__ tw, int T, u64 q, u64 q2) {
    if (FIRST) {
        const ulonglong2 t1 = tw[T];
#pragma unroll
        for (int k = 0; k < 4; ++k) bf_fwd(a[k], a[k + 4], t1, q, q2);
    }
    if (CORRECT) {   // seven stages done: everything is below 15q, bring it below 8q
        const u64 q8 = 4 * q2;
#pragma unroll
        for (int k = 0; k < 8; ++k) a[k] = csub(a[k], q8);
    }
    const ulonglong2 t2a = tw[2 * T], t2b = tw[2 * T + 1];
    bf_fwd(a[0], a[2], t2a, q, q2);
    bf_fwd(a[1], a[3], t2a, q, q2);
    bf_fwd(a[4], a[6], t2b, q, q2);
    bf_fwd(a[5], a[7], t2b, q, q2);
    const ulonglong2 *t4 = tw + 4 * T;
    bf_fwd(a[0], a[1], t4[0], q, q2);
    bf_fwd(a[2], a[3], t4[1], q, q2);
    bf_fwd(a[4], a[5], t4[2], q, q2);
    bf_fwd(a[6], a[7], t4[3], q, q2);
}
// Radix-8 inverse pass (bit 0 of k first), same twiddle addressing on the inverse table.
__device__ __forceinline__ void inv_pass(u64 (&a)[8], const ulonglong2 *__restrict__ tw, int T, u64 q, u64 q2) {
    const ulonglong2 *t4 = tw + 4 * T;
    bf_inv(a[0], a[1], t4[0], q, q2);
    bf_inv(a[2], a[3], t4[1], q, q2);
    bf_inv(a[4], a[5], t4[2], q, q2);
    bf_inv(a[6], a[7], t4[3], q, q2);
    const ulonglong2 t2a = tw[2 * T], t2b = tw[2 * T + 1];
    bf_inv(a[0], a[2], t2a, q, q2);
    bf_inv(a[1], a[3], t2a, q, q2);
    bf_inv(a[4], a[6], t2b, q, q2);
    bf_inv(a[5], a[7], t2b, q, q2);
    const ulonglong2 t1 = tw[T];
#pragma unroll
    for (int k = 0; k < 4; ++k) bf_inv(a[k], a[k + 4], t1, q, q2);
}

// store the 8 registers at index(k) = base | (k << shift), barrier, load index'(k) = base2 | (k << shift2)
template <int SH_OUT, int SH_IN>
__device__ __forceinline__ void exchange(u64 (&a)[8], u64 *buf, int base_out, int base_in) {
#pragma unroll
    for (int k = 0; k < 8; ++k) buf[pad(base_out | (k << SH_OUT))] = a[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 8; ++k) a[k] = buf[pad(base_in | (k << SH_IN))];
}

struct Tables2048 {
    const ulonglong2 *tw, *itw;   // (w, companion) pairs, forward and inverse
    ulonglong2 ninv, itw1n;       // n^-1 and itw[1]*n^-1 with companions
    Modulus mod;
};

// Forward transform of the 8 registers (ownership t + 256k, values below q); the result is left in
// LDS buffer `res` (natural index, padded), values below 16q.  LDS phases: other, res, other, res.
__device__ __forceinline__ void forward_to_lds(u64 (&a)[8], u64 *res, u64 *other, const Tables2048 &T, int tid) {
    const u64 q = T.mod.q, q2 = T.mod.q2;
    fwd_pass<true, false>(a, T.tw, 1, q, q2);                                        // bits 8-10
    exchange<8, 5>(a, other, tid, ((tid >> 5) << 8) | (tid & 31));
    fwd_pass<true, false>(a, T.tw, 8 + (tid >> 5), q, q2);                           // bits 5-7
    exchange<5, 2>(a, res, ((tid >> 5) << 8) | (tid & 31), ((tid >> 2) << 5) | (tid & 3));
    fwd_pass<true, true>(a, T.tw, 64 + (tid >> 2), q, q2);                           // bits 2-4
    exchange<2, 0>(a, other, ((tid >> 2) << 5) | (tid & 3), tid << 3);
    fwd_pass<false, false>(a, T.tw, 256 + tid, q, q2);                               // bits 0-1
#pragma unroll
    for (int k = 0; k < 8; ++k) res[pad((tid << 3) | k)] = a[k];
    __syncthreads();
}

// Inverse transform: registers hold index 8t + k (values below 2q) on entry and index t + 256k,
// canonical, on return.
__device__ __forceinline__ void inverse_in_regs(u64 (&a)[8], u64 *bufA, u64 *bufB, const Tables2048 &T, int tid) {
    const u64 q = T.mod.q, q2 = T.mod.q2;
    inv_pass(a, T.itw, 256 + tid, q, q2);                                            // bits 0-2
    exchange<0, 3>(a, bufA, tid << 3, ((tid >> 3) << 6) | (tid & 7));
    inv_pass(a, T.itw, 32 + (tid >> 3), q, q2);                                      // bits 3-5
    exchange<3, 6>(a, bufB, ((tid >> 3) << 6) | (tid & 7), ((tid >> 6) << 9) | (tid & 63));
    inv_pass(a, T.itw, 4 + (tid >> 6), q, q2);                                       // bits 6-8
    exchange<6, 8>(a, bufA, ((tid >> 6) << 9) | (tid & 63), tid);
    // bits 9-10 (register bits 1,2; register bit 0 is index bit 8), n^-1 folded into the last stage
    const ulonglong2 t2a = T.itw[2], t2b = T.itw[3];
    bf_inv(a[0], a[2], t2a, q, q2);
    bf_inv(a[1], a[3], t2a, q, q2);
    bf_inv(a[4], a[6], t2b, q, q2);
    bf_inv(a[5], a[7], t2b, q, q2);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const u64 x = a[k], y = a[k + 4];
        a[k] = mul_shoup(x + y, T.ninv.x, T.ninv.y, q);
        a[k + 4] = mul_shoup(x - y + q2, T.itw1n.x, T.itw1n.y, q);
    }
}

// below 16q -> canonical
__device__ __forceinline__ u64 reduce64(u64 x, const Modulus &m) {
    return csub(x - mulhi64(x, m.one_s) * m.q, m.q);
}

template <bool HAS_W>
__global__ __launch_bounds__(NT) void perm_accumulate_2048(PermJob job, Tables2048 T, int gadget_bits, int ndigits) {
    __shared__ u64 bufA[LDS_WORDS], bufB[LDS_WORDS];
    const int tid = threadIdx.x;
    const int item = blockIdx.x / job.nchunks, chunk = blockIdx.x % job.nchunks;
    const int g0 = (int)((long)chunk * job.G / job.nchunks), g1 = (int)((long)(chunk + 1) * job.G / job.nchunks);
    const u64 digit_mask = (1ull << gadget_bits) - 1;
    const size_t key_words = (size_t)ndigits * 2 * N;

    u64 sum0[PER], sum1[PER];   // running sums over the rotations of this chunk, lazy (below 16q)
#pragma unroll
    for (int k = 0; k < PER; ++k) sum0[k] = sum1[k] = 0;
    int lazy = 0;

    for (int g = g0; g < g1; ++g) {
        const u64 *c0 = job.ct_in + (size_t)item * job.in_item_stride + (size_t)g * job.in_g_stride;
        const u64 *c1 = c0 + N;
        const u64 *w = HAS_W ? job.w + (size_t)g * N : nullptr;
        const int gal = job.gal[g];
        if (lazy == 14) {
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                sum0[k] = reduce64(sum0[k], T.mod);
                sum1[k] = reduce64(sum1[k], T.mod);
            }
            lazy = 1;
        }
        ++lazy;
        if (gal == 1) {   // rotation by zero: ScMult and Add only
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                const int i = tid + k * NT;
                if (HAS_W) {
                    sum0[k] += mul_mod(c0[i], w[i], T.mod);
                    sum1[k] += mul_mod(c1[i], w[i], T.mod);
                } else {
                    sum0[k] += c0[i];
                    sum1[k] += c1[i];
                }
            }
            continue;
        }
        // LDS phases of one rotation: A B A (inverse), then B A B A per digit.  Consecutive phases use
        // different buffers, which is what lets each exchange do with one barrier; a rotation ends on
        // A and the next one starts on A, so that one boundary needs a barrier of its own.
        __syncthreads();
        const u64 *key = job.keys + (size_t)job.key_idx[g] * key_words;
        int src[PER];   // where the automorphism takes output index tid + 256k from
#pragma unroll
        for (int k = 0; k < PER; ++k) src[k] = galois_index11(tid + k * NT, gal);

        // ScMult of c1 (8 consecutive coefficients per thread), then the inverse transform
        u64 a[PER];
        {
            const ulonglong2 *c1v = reinterpret_cast<const ulonglong2 *>(c1 + 8 * tid);
            const ulonglong2 *wv = reinterpret_cast<const ulonglong2 *>(w + 8 * tid);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const ulonglong2 cv = c1v[k];
                if (HAS_W) {
                    const ulonglong2 ww = wv[k];
                    a[2 * k] = mul_mod(cv.x, ww.x, T.mod);
                    a[2 * k + 1] = mul_mod(cv.y, ww.y, T.mod);
                } else {
                    a[2 * k] = cv.x;
                    a[2 * k + 1] = cv.y;
                }
            }
        }
        inverse_in_regs(a, bufA, bufB, T, tid);
        u64 coef[PER];
#pragma unroll
        for (int k = 0; k < PER; ++k) coef[k] = a[k];

        u128 acc0[PER], acc1[PER];
        // the c0 part: permuted c0 (.) w
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            if (HAS_W) acc0[k] = (u128)c0[src[k]] * w[src[k]];
            else acc0[k] = c0[src[k]];
            acc1[k] = 0;
        }
        int terms = 1;
        for (int j = 0; j < ndigits; ++j) {
#pragma unroll
            for (int k = 0; k < PER; ++k) a[k] = (coef[k] >> (j * gadget_bits)) & digit_mask;
            forward_to_lds(a, bufA, bufB, T, tid);   // result in bufA
            const u64 *kb = key + (size_t)(2 * j) * N, *ka = kb + N;
            if (terms + 1 > 15) {   // products are below 2^124 here (digit transforms are below 16q)
#pragma unroll
                for (int k = 0; k < PER; ++k) {
                    acc0[k] = reduce128(acc0[k], T.mod);
                    acc1[k] = reduce128(acc1[k], T.mod);
                }
                terms = 1;
            }
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                const int i = tid + k * NT;
                const u64 d = bufA[pad(src[k])];
                acc0[k] += (u128)d * kb[i];
                acc1[k] += (u128)d * ka[i];
            }
            ++terms;
        }
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            sum0[k] += reduce128(acc0[k], T.mod);
            sum1[k] += reduce128(acc1[k], T.mod);
        }
    }
    u64 *out = job.partial + ((size_t)item * job.nchunks + chunk) * 2 * N;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int i = tid + k * NT;
        out[i] = reduce64(sum0[k], T.mod);
        out[N + i] = reduce64(sum1[k], T.mod);
    }
}

}  // namespace

int launch_perm_accumulate_2048(const gala_ctx *c, void *stream, const PermJob &job) {
    hipStream_t st = (hipStream_t)stream;
    Tables2048 T;
    T.tw = reinterpret_cast<const ulonglong2 *>(c->d_tw2);
    T.itw = reinterpret_cast<const ulonglong2 *>(c->d_tw2 + 2 * (size_t)N);
    T.ninv = make_ulonglong2(c->dev_q.ninv, c->dev_q.ninvs);
    T.itw1n = make_ulonglong2(c->dev_q.itw1n, c->dev_q.itw1ns);
    T.mod = c->dev_q.mod;
    const dim3 grid((unsigned)(job.items * job.nchunks));
    if (job.w)
        hipLaunchKernelGGL(perm_accumulate_2048<true>, grid, dim3(NT), 0, st, job, T, c->gadget_bits, c->ndigits);
    else
        hipLaunchKernelGGL(perm_accumulate_2048<false>, grid, dim3(NT), 0, st, job, T, c->gadget_bits, c->ndigits);
    return (int)hipGetLastError();
}

}  // namespace gala
