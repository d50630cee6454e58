// HIP kernels for gfx950: batched negacyclic transforms staged through LDS, the
// fused rotate-and-accumulate kernel (ScMult -> DecPerm -> HstPerm -> Add over
// the rotations of a layer), share generation, and the convolution's
// multiply-accumulate.  All arithmetic is unsigned 64-bit modulo a prime below
// 2^61; there is no floating point on this path.
#include <hip/hip_runtime.h>

#include <type_traits>

#include <cstdlib>

#include "gala_internal.h"

namespace gala {

namespace {

constexpr int kMaxPer = 8;   // coefficients owned by one thread (n <= kMaxPer * block size)

__device__ __forceinline__ int bitrev(int v, int bits) { return (int)(__brev((unsigned)v) >> (32 - bits)); }

// Index permutation of the Galois map X -> X^gal in the evaluation domain:
// position i holds the value at psi^(2 brev(i) + 1), and (a o gal)(x) = a(x^gal).
__device__ __forceinline__ int galois_index(int i, int gal, int logn, int n) {
    const int e = ((2 * bitrev(i, logn) + 1) * gal) & (2 * n - 1);
    return bitrev((e - 1) >> 1, logn);
}

// Forward transform of the n words in LDS; any input below 4q, output below 4q.
template <int NT>
__device__ void ntt_forward_lds(u64 *a, int n, int logn, const NttDev &T) {
    const u64 q = T.mod.q, q2 = T.mod.q2;
    for (int s = 0; s < logn; ++s) {
        const int tlog = logn - 1 - s, t = 1 << tlog, m = 1 << s;
        for (int b = threadIdx.x; b < (n >> 1); b += NT) {
            const int i = b >> tlog, j = (i << (tlog + 1)) | (b & (t - 1));
            u64 x = a[j], y = a[j + t];
            butterfly_fwd(x, y, T.tw[m + i], T.tws[m + i], q, q2);
            a[j] = x;
            a[j + t] = y;
        }
        __syncthreads();
    }
}
// Inverse transform in LDS; input below 2q, output canonical.
template <int NT>
__device__ void ntt_inverse_lds(u64 *a, int n, int logn, const NttDev &T) {
    const u64 q = T.mod.q, q2 = T.mod.q2;
    for (int s = 0; s < logn - 1; ++s) {
        const int t = 1 << s, m = n >> (s + 1);
        for (int b = threadIdx.x; b < (n >> 1); b += NT) {
            const int i = b >> s, j = (i << (s + 1)) | (b & (t - 1));
            u64 x = a[j], y = a[j + t];
            butterfly_inv(x, y, T.itw[m + i], T.itws[m + i], q, q2);
            a[j] = x;
            a[j + t] = y;
        }
        __syncthreads();
    }
    const int t = n >> 1;
    for (int b = threadIdx.x; b < t; b += NT) {
        const u64 x = a[b], y = a[b + t];
        a[b] = mul_shoup(x + y, T.ninv, T.ninvs, q);
        a[b + t] = mul_shoup(x - y + q2, T.itw1n, T.itw1ns, q);
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------
// batched transform (import / export / key upload): one workgroup per polynomial
// ---------------------------------------------------------------------------
template <int NT>
__global__ __launch_bounds__(NT) void ntt_kernel(const u64 *src, u64 *dst, int n, int logn, NttDev T, int inverse) {
    extern __shared__ u64 buf[];
    const size_t base = (size_t)blockIdx.x * n;
    for (int i = threadIdx.x; i < n; i += NT) buf[i] = src[base + i];
    __syncthreads();
    if (inverse) ntt_inverse_lds<NT>(buf, n, logn, T);
    else ntt_forward_lds<NT>(buf, n, logn, T);
    for (int i = threadIdx.x; i < n; i += NT) dst[base + i] = csub(csub(buf[i], T.mod.q2), T.mod.q);
}

__global__ void key_finish_kernel(u64 *pairs, const u64 *s_hat, int n, size_t total, Modulus mod) {
    const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= total) return;
    const size_t pair = id / n;
    const int i = (int)(id % n);
    u64 *t = pairs + pair * 2 * n, *a = t + n;
    t[i] = sub_mod(t[i], mul_mod(a[i], s_hat[i], mod), mod.q);
}

// companion of a constant w < q: floor(w * 2^64 / q), by 64 steps of binary long division
// (polys = 4: polynomials 2 and 3 of every group of four are constants modulo the second modulus).  The
// modulus differs from lane to lane; it is picked with a lane mask rather than a branch on purpose: hipcc 7.2
// kept a branchy `cond ? q_second : q_first` in scalar registers and gave every lane q_second.
__global__ void pair_pack_kernel(const u64 *src, u64 *dst, size_t count, u64 q_first, u64 q_second, int logn, int polys) {
    const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= count) return;
    const u64 second = polys == 4 ? 0 - (u64)((id >> (logn + 1)) & 1) : 0;   // all ones on polynomials 2, 3 of 4
    const u64 q = (q_first & ~second) | (q_second & second);
    const u64 w = src[id];
    u64 rem = w, quot = 0;
    for (int b = 0; b < 64; ++b) {
        rem <<= 1;                       // rem < q < 2^61, no overflow
        const bool ge = rem >= q;
        rem -= ge ? q : 0;
        quot = (quot << 1) | (ge ? 1 : 0);
    }
    dst[2 * id] = w;
    dst[2 * id + 1] = quot;
}

// ---------------------------------------------------------------------------
// rotate-and-accumulate
// ---------------------------------------------------------------------------
// SPECIAL: key switching with a special prime P.  Keys hold four polynomials per digit ((b, a) modulo q, then
// modulo P); the inner products run in both moduli; each sum modulo P goes back to coefficients r in [0,P) and
// the key switch contributes (t_q - r) / P.  Everything after the lift r -> r mod q is linear modulo q, so a
// workgroup adds the r of its rotations in the coefficient domain and transforms that sum once at the end;
// whatever is not divided by P (the c0 part, rotations by zero) enters the sums multiplied by P.
struct SpecialConst {
    u64 Pq, Pinv;   // P mod q and its inverse
};
template <int NT, bool SPECIAL>
__global__ __launch_bounds__(NT) void perm_accumulate_kernel(PermJob job, NttDev T, NttDev TP, SpecialConst sc, int n,
                                                             int logn, int gadget_bits, int ndigits) {
    extern __shared__ u64 buf[];
    const int tid = threadIdx.x;
    const int item = blockIdx.x / job.nchunks, chunk = blockIdx.x % job.nchunks;
    int g0, g1;
    chunk_range(chunk, job.nchunks, job.G, g0, g1);
    const u64 q = T.mod.q, q2 = T.mod.q2;
    const u64 digit_mask = (1ull << gadget_bits) - 1;
    constexpr int POLYS = SPECIAL ? 4 : 2;
    const size_t key_words = (size_t)ndigits * POLYS * n;

    u128 acc0[kMaxPer], acc1[kMaxPer];
    u64 R0[kMaxPer], R1[kMaxPer];   // SPECIAL: coefficient-domain sums (mod q) of the lifted remainders
#pragma unroll
    for (int k = 0; k < kMaxPer; ++k) {
        acc0[k] = acc1[k] = 0;
        R0[k] = R1[k] = 0;
    }
    int terms = 0;   // products (each below q^2 < 2^122) summed into the accumulators so far

    for (int g = g0; g < g1; ++g) {
        const u64 *c0 = job.ct_in + (size_t)item * job.in_item_stride +
                        (size_t)(job.in_g_index ? job.in_g_index[g] : g) * job.in_g_stride;
        const u64 *c1 = c0 + n;
        const u64 *w = job.w ? job.w + (size_t)g * n : nullptr;
        const int gal = job.gal[g];
        if (terms + ndigits + 1 > 60) {   // keep the 128-bit sums from overflowing
#pragma unroll
            for (int k = 0; k < kMaxPer; ++k) {
                acc0[k] = reduce128(acc0[k], T.mod);
                acc1[k] = reduce128(acc1[k], T.mod);
            }
            terms = 1;
        }
        if (gal == 1) {   // the rotation by zero: ScMult and Add only
#pragma unroll
            for (int k = 0; k < kMaxPer; ++k) {
                const int i = tid + k * NT;
                if (i < n) {
                    if (SPECIAL) {
                        acc0[k] += (u128)(w ? mul_mod(c0[i], w[i], T.mod) : c0[i]) * sc.Pq;
                        acc1[k] += (u128)(w ? mul_mod(c1[i], w[i], T.mod) : c1[i]) * sc.Pq;
                    } else if (w) {
                        acc0[k] += (u128)c0[i] * w[i];
                        acc1[k] += (u128)c1[i] * w[i];
                    } else {
                        acc0[k] += c0[i];
                        acc1[k] += c1[i];
                    }
                }
            }
            terms += 1;
            continue;
        }
        const u64 *key = job.keys + (size_t)job.key_idx[g] * key_words;
        // ScMult of c1, then DecPerm: back to coefficients, digits, forward again
        for (int k = 0; k < kMaxPer; ++k) {
            const int i = tid + k * NT;
            if (i < n) buf[i] = w ? mul_mod(c1[i], w[i], T.mod) : c1[i];
        }
        __syncthreads();
        ntt_inverse_lds<NT>(buf, n, logn, T);
        u64 coef[kMaxPer];
#pragma unroll
        for (int k = 0; k < kMaxPer; ++k) {
            const int i = tid + k * NT;
            coef[k] = i < n ? buf[i] : 0;
        }
        __syncthreads();
        u128 accP0[kMaxPer], accP1[kMaxPer];   // SPECIAL: this rotation's sums modulo P
#pragma unroll
        for (int k = 0; k < kMaxPer; ++k) accP0[k] = accP1[k] = 0;
        for (int j = 0; j < ndigits; ++j) {
#pragma unroll
            for (int k = 0; k < kMaxPer; ++k) {
                const int i = tid + k * NT;
                if (i < n) buf[i] = (coef[k] >> (j * gadget_bits)) & digit_mask;
            }
            __syncthreads();
            ntt_forward_lds<NT>(buf, n, logn, T);
            // HstPerm: automorphism as a gather, inner product with the key
            const u64 *kb = key + (size_t)(POLYS * j) * n, *ka = kb + n;
#pragma unroll
            for (int k = 0; k < kMaxPer; ++k) {
                const int i = tid + k * NT;
                if (i < n) {
                    const u64 d = csub(csub(buf[galois_index(i, gal, logn, n)], q2), q);
                    acc0[k] += (u128)d * kb[i];
                    acc1[k] += (u128)d * ka[i];
                }
            }
            __syncthreads();
            if (SPECIAL) {   // the same digit and gather modulo P
#pragma unroll
                for (int k = 0; k < kMaxPer; ++k) {
                    const int i = tid + k * NT;
                    if (i < n) buf[i] = (coef[k] >> (j * gadget_bits)) & digit_mask;
                }
                __syncthreads();
                ntt_forward_lds<NT>(buf, n, logn, TP);
                const u64 *kbP = kb + 2 * (size_t)n, *kaP = kbP + n;
#pragma unroll
                for (int k = 0; k < kMaxPer; ++k) {
                    const int i = tid + k * NT;
                    if (i < n) {
                        const u64 d = csub(csub(buf[galois_index(i, gal, logn, n)], TP.mod.q2), TP.mod.q);
                        accP0[k] += (u128)d * kbP[i];
                        accP1[k] += (u128)d * kaP[i];
                    }
                }
                __syncthreads();
            }
        }
        if (SPECIAL) {   // remainders modulo P back to coefficients, lifted to [0,P), reduced modulo q, summed
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (int k = 0; k < kMaxPer; ++k) {
                    const int i = tid + k * NT;
                    if (i < n) buf[i] = reduce128(h ? accP1[k] : accP0[k], TP.mod);
                }
                __syncthreads();
                ntt_inverse_lds<NT>(buf, n, logn, TP);
#pragma unroll
                for (int k = 0; k < kMaxPer; ++k) {
                    const int i = tid + k * NT;
                    if (i < n) {
                        const u64 r = buf[i] % q;
                        if (h) R1[k] = add_mod(R1[k], r, q); else R0[k] = add_mod(R0[k], r, q);
                    }
                }
                __syncthreads();
            }
        }
        // the c0 part of the rotated ciphertext
#pragma unroll
        for (int k = 0; k < kMaxPer; ++k) {
            const int i = tid + k * NT;
            if (i < n) {
                const int pi = galois_index(i, gal, logn, n);
                if (SPECIAL) acc0[k] += (u128)(w ? mul_mod(c0[pi], w[pi], T.mod) : c0[pi]) * sc.Pq;
                else if (w) acc0[k] += (u128)c0[pi] * w[pi];
                else acc0[k] += c0[pi];
            }
        }
        terms += ndigits + 1;
    }
    u64 *out = job.partial + ((size_t)item * job.slots + chunk) * 2 * n;
    if (SPECIAL) {   // out = (sum - transform(R)) / P
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            __syncthreads();
#pragma unroll
            for (int k = 0; k < kMaxPer; ++k) {
                const int i = tid + k * NT;
                if (i < n) buf[i] = h ? R1[k] : R0[k];
            }
            __syncthreads();
            ntt_forward_lds<NT>(buf, n, logn, T);
#pragma unroll
            for (int k = 0; k < kMaxPer; ++k) {
                const int i = tid + k * NT;
                if (i < n) {
                    const u64 x = csub(csub(buf[i], q2), q);
                    const u64 t = reduce128(h ? acc1[k] : acc0[k], T.mod);
                    out[h * n + i] = mul_mod(sub_mod(t, x, q), sc.Pinv, T.mod);
                }
            }
        }
        return;
    }
#pragma unroll
    for (int k = 0; k < kMaxPer; ++k) {
        const int i = tid + k * NT;
        if (i < n) {
            out[i] = reduce128(acc0[k], T.mod);
            out[n + i] = reduce128(acc1[k], T.mod);
        }
    }
}

// ---------------------------------------------------------------------------
// share generation: sum the partial ciphertexts of an item, subtract the mask
// ---------------------------------------------------------------------------
template <int NT>
__global__ __launch_bounds__(NT) void finalize_kernel(FinalizeJob job, NttDev Tq, NttDev Tp, const int *slot_to_idx,
                                                      int n, int logn, int pbits, u64 delta, u64 delta_s) {
    extern __shared__ u64 buf[];
    const int tid = threadIdx.x;
    const int item = blockIdx.x, b = item / job.nout, O = item % job.nout;
    const u64 q = Tq.mod.q, p = Tp.mod.q;
    if (job.r) {
        const int *row_ptr = job.mask.row_ptr + (size_t)O * (n + 1);
        const int *row_slots = job.mask.row_slots + (size_t)O * n;
        const int *row_rindex = job.mask.row_rindex + (size_t)O * n;
        const unsigned char *is_first = job.mask.is_first + (size_t)O * n;
        // every slot but the first of each real output is a draw from the mask stream
        for (int s = tid; s < n; s += NT) {
            u64 v = 0;
            if (!is_first[s]) v = draw_uniform(p, pbits, job.mask_seed, kStreamMask, ((u64)b << 32) + ((u64)O << 16) + (u64)s);
            buf[slot_to_idx[s]] = v;
        }
        __syncthreads();
        // the first slot absorbs r[t] minus the rest of its group
        const int nrows = job.mask.nrows[O];
        for (int t = tid; t < nrows; t += NT) {
            const int e0 = row_ptr[t], e1 = row_ptr[t + 1];
            if (e1 <= e0) continue;
            u64 sum = 0;
            for (int e = e0 + 1; e < e1; ++e) sum = add_mod(sum, buf[slot_to_idx[row_slots[e]]], p);
            u64 rv = job.r[(size_t)b * job.r_stride + row_rindex[t]];
            if (rv >= p) rv %= p;
            buf[slot_to_idx[row_slots[e0]]] = sub_mod(rv, sum, p);
        }
        __syncthreads();
        // encode: slots -> plaintext polynomial mod p -> delta * m mod q -> evaluation domain
        ntt_inverse_lds<NT>(buf, n, logn, Tp);
        for (int i = tid; i < n; i += NT) buf[i] = mul_shoup(buf[i], delta, delta_s, q);
        __syncthreads();
        ntt_forward_lds<NT>(buf, n, logn, Tq);
    }
    const u64 *part = job.partial + (size_t)item * job.slots * 2 * n;
    u64 *out = job.ct_out + (size_t)item * 2 * n;
    for (int i = tid; i < n; i += NT) {
        u64 s0 = 0, s1 = 0;
        for (int c = 0; c < job.nchunks; ++c) {
            s0 = add_mod(s0, part[(size_t)c * 2 * n + i], q);
            s1 = add_mod(s1, part[(size_t)c * 2 * n + n + i], q);
        }
        if (job.r) s0 = sub_mod(s0, csub(csub(buf[i], Tq.mod.q2), q), q);
        out[i] = s0;
        out[n + i] = s1;
    }
}

// ---------------------------------------------------------------------------
// Add, ScMult and plaintext operands on their own
// ---------------------------------------------------------------------------
// slots -> plaintext polynomial mod p -> lifted (mode 0: centred; mode 1: times delta) -> evaluation domain mod q
template <int NT>
__global__ __launch_bounds__(NT) void encode_plain_kernel(const u64 *slots, u64 *plain, NttDev Tq, NttDev Tp,
                                                          const int *slot_to_idx, int n, int logn, int mode, u64 delta,
                                                          u64 delta_s) {
    extern __shared__ u64 buf[];
    const int tid = threadIdx.x;
    const u64 q = Tq.mod.q, p = Tp.mod.q;
    const u64 *sl = slots + (size_t)blockIdx.x * n;
    for (int s = tid; s < n; s += NT) {
        const u64 v = sl[s];
        buf[slot_to_idx[s]] = v >= p ? v % p : v;
    }
    __syncthreads();
    ntt_inverse_lds<NT>(buf, n, logn, Tp);
    for (int i = tid; i < n; i += NT) {
        const u64 m = buf[i];
        buf[i] = mode ? mul_shoup(m, delta, delta_s, q) : (m > p / 2 ? q - (p - m) : m);
    }
    __syncthreads();
    ntt_forward_lds<NT>(buf, n, logn, Tq);
    u64 *out = plain + (size_t)blockIdx.x * n;
    for (int i = tid; i < n; i += NT) out[i] = csub(csub(buf[i], Tq.mod.q2), q);
}
// one thread per word of a ciphertext: op 0 ct + ct, 1 ct (.) plain, 2 ct - plain (c0 only), 3 ct + plain
__global__ void ct_op_kernel(int op, const u64 *a, const u64 *b, size_t b_stride, size_t words, int n, u64 *out, Modulus mod) {
    const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= words) return;
    const size_t item = id / (2 * (size_t)n);
    const int e = (int)(id % (2 * (size_t)n)), i = e % n;
    const u64 x = a[id];
    u64 r;
    if (op == 0) r = add_mod(x, b[item * b_stride + e], mod.q);
    else if (op == 1) r = mul_mod(x, b[item * b_stride + i], mod);
    else if (e >= n) r = x;
    else if (op == 2) r = sub_mod(x, b[item * b_stride + i], mod.q);
    else r = add_mod(x, b[item * b_stride + i], mod.q);
    out[id] = r;
}

// ---------------------------------------------------------------------------
// the client's steps, batched: one workgroup per ciphertext, internal (evaluation-domain) form
// ---------------------------------------------------------------------------
// ct = (-a s + e + delta m, a) (Sec. II-C(1)): m = the plaintext polynomial of the slots, a uniform, e Gaussian,
// everything drawn from the ciphertext's seed exactly as the host function does.
template <int NT>
__global__ __launch_bounds__(NT) void encrypt_kernel(const u64 *slots, const u64 *seeds, const u64 *s_hat, u64 *ct_out,
                                                     NttDev Tq, NttDev Tp, const int *slot_to_idx, GaussCdf cdf, int n,
                                                     int logn, int qbits, u64 delta, u64 delta_s) {
    extern __shared__ u64 buf[];
    const int tid = threadIdx.x;
    const u64 q = Tq.mod.q, p = Tp.mod.q, seed = seeds[blockIdx.x];
    const u64 *sl = slots + (size_t)blockIdx.x * n;
    u64 *c0 = ct_out + (size_t)blockIdx.x * 2 * n, *c1 = c0 + n;
    for (int s = tid; s < n; s += NT) {
        const u64 v = sl[s];
        buf[slot_to_idx[s]] = v >= p ? v % p : v;
    }
    __syncthreads();
    ntt_inverse_lds<NT>(buf, n, logn, Tp);
    u64 m[kMaxPer], a_hat[kMaxPer];
#pragma unroll
    for (int k = 0; k < kMaxPer; ++k) {
        const int i = tid + k * NT;
        m[k] = i < n ? buf[i] : 0;
    }
    __syncthreads();
    for (int i = tid; i < n; i += NT) buf[i] = draw_uniform(q, qbits, seed, kStreamCtA, (u64)i);
    __syncthreads();
    ntt_forward_lds<NT>(buf, n, logn, Tq);
#pragma unroll
    for (int k = 0; k < kMaxPer; ++k) {
        const int i = tid + k * NT;
        if (i < n) {
            a_hat[k] = csub(csub(buf[i], Tq.mod.q2), q);
            c1[i] = a_hat[k];
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kMaxPer; ++k) {
        const int i = tid + k * NT;
        if (i < n) {
            const int e = draw_gauss_cdf(cdf, seed, kStreamCtE, (u64)i);
            const u64 el = e >= 0 ? (u64)e : q - (u64)(-e);
            buf[i] = add_mod(el, mul_shoup(m[k], delta, delta_s, q), q);
        }
    }
    __syncthreads();
    ntt_forward_lds<NT>(buf, n, logn, Tq);
#pragma unroll
    for (int k = 0; k < kMaxPer; ++k) {
        const int i = tid + k * NT;
        if (i < n) c0[i] = sub_mod(csub(csub(buf[i], Tq.mod.q2), q), mul_mod(a_hat[k], s_hat[i], Tq.mod), q);
    }
}
// slots = decode(round(p (c0 + c1 s) / q) mod p).  The rounded quotient of t = p v + floor(q/2) by q comes from
// r = t mod q and the exact division (t - r) / q, which is the low word of (t - r) times q^-1 mod 2^64.
template <int NT>
__global__ __launch_bounds__(NT) void decrypt_kernel(const u64 *ct_in, const u64 *s_hat, u64 *slots, NttDev Tq, NttDev Tp,
                                                     const int *slot_to_idx, int n, int logn, u64 q_inv64) {
    extern __shared__ u64 buf[];
    const int tid = threadIdx.x;
    const u64 q = Tq.mod.q, p = Tp.mod.q;
    const u64 *c0 = ct_in + (size_t)blockIdx.x * 2 * n, *c1 = c0 + n;
    for (int i = tid; i < n; i += NT) buf[i] = add_mod(c0[i], mul_mod(c1[i], s_hat[i], Tq.mod), q);
    __syncthreads();
    ntt_inverse_lds<NT>(buf, n, logn, Tq);
    for (int i = tid; i < n; i += NT) {
        const u128 t = (u128)p * buf[i] + (q >> 1);
        const u64 r = reduce128(t, Tq.mod);
        const u64 quot = ((u64)t - r) * q_inv64;       // t - r is a multiple of q and the quotient is at most p
        buf[i] = quot >= p ? quot - p : quot;
    }
    __syncthreads();
    ntt_forward_lds<NT>(buf, n, logn, Tp);
    u64 *out = slots + (size_t)blockIdx.x * n;
    for (int s = tid; s < n; s += NT) out[s] = csub(csub(buf[slot_to_idx[s]], Tp.mod.q2), p);
}

// ---------------------------------------------------------------------------
// convolution: hoisted input rotations and the multiply-accumulate
// ---------------------------------------------------------------------------
template <int NT>
__global__ __launch_bounds__(NT) void decperm_kernel(const u64 *ct_in, u64 *digits, NttDev T, int n, int logn,
                                                     int gadget_bits, int ndigits) {
    extern __shared__ u64 buf[];
    const int tid = threadIdx.x;
    const u64 *c1 = ct_in + (size_t)blockIdx.x * 2 * n + n;
    u64 *out = digits + (size_t)blockIdx.x * ndigits * n;
    const u64 digit_mask = (1ull << gadget_bits) - 1;
    for (int i = tid; i < n; i += NT) buf[i] = c1[i];
    __syncthreads();
    ntt_inverse_lds<NT>(buf, n, logn, T);
    u64 coef[kMaxPer];
#pragma unroll
    for (int k = 0; k < kMaxPer; ++k) {
        const int i = tid + k * NT;
        coef[k] = i < n ? buf[i] : 0;
    }
    __syncthreads();
    for (int j = 0; j < ndigits; ++j) {
#pragma unroll
        for (int k = 0; k < kMaxPer; ++k) {
            const int i = tid + k * NT;
            if (i < n) buf[i] = (coef[k] >> (j * gadget_bits)) & digit_mask;
        }
        __syncthreads();
        ntt_forward_lds<NT>(buf, n, logn, T);
        for (int i = tid; i < n; i += NT) out[(size_t)j * n + i] = csub(csub(buf[i], T.mod.q2), T.mod.q);
        __syncthreads();
    }
}

__global__ void hstperm_taps_kernel(const u64 *ct_in, const u64 *digits, TermList terms, const u64 *keys, u64 *xrot,
                                    Modulus mod, int n, int logn, int ndigits) {
    const int b = blockIdx.x / terms.nterm, e = blockIdx.x % terms.nterm;
    const size_t c = (size_t)b * terms.nin + terms.ct[e];
    const u64 *c0 = ct_in + c * 2 * n, *c1 = c0 + n;
    const u64 *dig = digits + c * ndigits * n;
    u64 *out = xrot + (size_t)blockIdx.x * 2 * n;
    const int gal = terms.gal[e];
    if (gal == 1) {
        for (int i = threadIdx.x; i < n; i += blockDim.x) {
            out[i] = c0[i];
            out[n + i] = c1[i];
        }
        return;
    }
    const u64 *key = keys + (size_t)terms.key[e] * ndigits * 2 * n;
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        const int pi = galois_index(i, gal, logn, n);
        u128 a0 = c0[pi], a1 = 0;
        int terms = 0;
        for (int j = 0; j < ndigits; ++j) {
            const u64 d = dig[(size_t)j * n + pi];
            a0 += (u128)d * key[(size_t)(2 * j) * n + i];
            a1 += (u128)d * key[(size_t)(2 * j + 1) * n + i];
            if (++terms == 32) {
                a0 = reduce128(a0, mod);
                a1 = reduce128(a1, mod);
                terms = 0;
            }
        }
        out[i] = reduce128(a0, mod);
        out[n + i] = reduce128(a1, mod);
    }
}

// acc (128 bits in lo, hi) += x * w with ten instructions: four 32x32+64 multiply-adds (low, high and
// the two cross products) and six carry additions; written out because the compiler's own 128-bit
// multiply-accumulate spends a third of its instructions on register moves.
__device__ __forceinline__ void mac128(u64 &lo, u64 &hi, u64 x, u64 w) {
    const u32 x0 = (u32)x, x1 = (u32)(x >> 32), w0 = (u32)w, w1 = (u32)(w >> 32);
    u64 carry_lo, carry_mid, unused, mid;
    asm("v_mad_u64_u32 %0, %1, %2, %3, %4" : "=v"(lo), "=s"(carry_lo) : "v"(x0), "v"(w0), "v"(lo));
    asm("v_mad_u64_u32 %0, %1, %2, %3, %4" : "=v"(hi), "=s"(unused) : "v"(x1), "v"(w1), "v"(hi));
    asm("v_mad_u64_u32 %0, %1, %2, %3, 0" : "=v"(mid), "=s"(unused) : "v"(x0), "v"(w1));
    asm("v_mad_u64_u32 %0, %1, %2, %3, %4" : "=v"(mid), "=s"(carry_mid) : "v"(x1), "v"(w0), "v"(mid));
    // words 1..3 += mid, then the carry of the low product into word 2 and of the cross sum into word 3
    u32 a1 = (u32)(lo >> 32), a2 = (u32)hi, a3 = (u32)(hi >> 32);
    asm("v_add_co_u32 %0, vcc, %0, %3\n\t"
        "v_addc_co_u32 %1, vcc, %1, %4, vcc\n\t"
        "v_addc_co_u32 %2, vcc, 0, %2, vcc\n\t"
        "v_addc_co_u32_e64 %1, vcc, 0, %1, %5\n\t"
        "v_addc_co_u32 %2, vcc, 0, %2, vcc\n\t"
        "v_addc_co_u32_e64 %2, vcc, 0, %2, %6"
        : "+v"(a1), "+v"(a2), "+v"(a3)
        : "v"((u32)mid), "v"((u32)(mid >> 32)), "s"(carry_lo), "s"(carry_mid)
        : "vcc");
    lo = ((u64)a1 << 32) | (u32)lo;
    hi = ((u64)a3 << 32) | a2;
}

// Per coefficient the convolution's ScMult/Add step is a small dense product: (O,gam) x (I,tap) weights
// times (I,tap) x (input, polynomial) rotated ciphertext words.  One thread owns one coefficient and a
// TM x TN register tile of 128-bit sums, so each loaded word feeds TN (weights) or TM (inputs) products.
// nterm terms (the plan's active (input ciphertext, tap) pairs); groups = nout*cn; cols = 2*batch (input-major, c0 then c1).
// A workgroup is WM x WN wavefronts on the same 64 coefficients: the wavefronts of a row read the same
// weight words and those of a column the same input words, so those reads hit in the CU's vector cache.
// Segments (seg_ptr != nullptr, nseg of them): segment s owns the terms seg_terms[seg_ptr[s] .. seg_ptr[s+1]-1] and gets
// sums of its own, acc row (m, s) = m * nseg + s: the per-input-ciphertext sums that the output-rotation schedule of
// Sec. III-B(2) rotates one by one.  Without segments there is one sum per row over all terms.
template <int TM, int TN, int WM, int WN, int U>
__global__ __launch_bounds__(64 * WM * WN) void conv_mac_kernel(const u64 *w, const u64 *xrot, int cols, int groups,
                                                                int nterm, u64 *acc, Modulus mod, int n,
                                                                int flush_every, const int *seg_ptr, const int *seg_terms,
                                                                int nseg) {
    const int i = blockIdx.x * 64 + (threadIdx.x & 63);
    if (i >= n) return;
    const int wave = threadIdx.x >> 6;
    const int seg = seg_ptr ? (int)(blockIdx.y % (unsigned)nseg) : 0, by = seg_ptr ? (int)(blockIdx.y / (unsigned)nseg) : (int)blockIdx.y;
    const int e_begin = seg_ptr ? seg_ptr[seg] : 0, e_end = seg_ptr ? seg_ptr[seg + 1] : nterm;
    const int m0 = (by * WM + wave % WM) * TM, c0 = (blockIdx.z * WN + wave / WM) * TN;
    // rows / columns past the end repeat the last valid one; their sums are computed but not stored
    const u64 *wp[TM], *xp[TN];
#pragma unroll
    for (int a = 0; a < TM; ++a) wp[a] = w + (size_t)min(m0 + a, groups - 1) * nterm * n + i;
#pragma unroll
    for (int b = 0; b < TN; ++b) {
        const int col = min(c0 + b, cols - 1);          // col = 2*input + polynomial
        xp[b] = xrot + ((size_t)(col >> 1) * nterm * 2 + (col & 1)) * n + i;
    }
    u64 lo[TM][TN], hi[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) lo[a][b] = hi[a][b] = 0;
    // U terms per step, all their loads issued before the first product: a wavefront that waits for one load at
    // a time reaches about half of the memory rate that several loads in flight do.
    auto term = [&](int k) -> size_t { return (size_t)(seg_ptr ? seg_terms[k] : k); };
    int pending = 0, e = e_begin;
    for (; e + U <= e_end; e += U) {
        u64 wv[U][TM], xv[U][TN];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t et = term(e + u);
#pragma unroll
            for (int a = 0; a < TM; ++a) wv[u][a] = wp[a][et * n];
#pragma unroll
            for (int b = 0; b < TN; ++b) xv[u][b] = xp[b][et * 2 * n];
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b) mac128(lo[a][b], hi[a][b], xv[u][b], wv[u][a]);
        pending += U;
        if (pending + U > flush_every) {   // keep the 128-bit sums of products below q^2 from overflowing
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b) {
                    lo[a][b] = reduce128(hi[a][b], lo[a][b], mod);
                    hi[a][b] = 0;
                }
            pending = 1;
        }
    }
    for (; e < e_end; ++e) {               // fewer than U terms left: there is room for them (pending + U <= flush_every)
        u64 wv[TM], xv[TN];
        const size_t et = term(e);
#pragma unroll
        for (int a = 0; a < TM; ++a) wv[a] = wp[a][et * n];
#pragma unroll
        for (int b = 0; b < TN; ++b) xv[b] = xp[b][et * 2 * n];
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b) mac128(lo[a][b], hi[a][b], xv[b], wv[a]);
    }
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            const int m = m0 + a, col = c0 + b;
            if (m < groups && col < cols)
                acc[((((size_t)(col >> 1) * groups + m) * nseg + seg) * 2 + (col & 1)) * n + i] = reduce128(hi[a][b], lo[a][b], mod);
        }
}

// The same sums for a single input (two columns: c0 and c1), where the kernel is bound by streaming the encoded
// kernels out of HBM once.  A workgroup is 4 x KS wavefronts on the same 64 coefficients: four consecutive tiles
// of TM rows (their input words are shared through the vector cache) times KS slices of the terms, whose partial
// sums meet in LDS at the end.  The words of the next U terms are requested before the products of the current U
// terms are formed, so every wavefront keeps U*TM weight words in flight all the time.
template <int TM, int U, int KS>
__global__ __launch_bounds__(256 * KS) void conv_mac_stream_kernel(const u64 *w, const u64 *xrot, int groups, int nterm,
                                                                   u64 *acc, Modulus mod, int n, int flush_every) {
    __shared__ u64 part[KS > 1 ? (KS - 1) * 4 * TM * 2 * 64 : 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, r = wave & 3, ks = wave >> 2;
    const int i = min(blockIdx.x * 64 + lane, n - 1);          // lanes past the ring repeat the last coefficient
    const bool live = blockIdx.x * 64 + lane < n;
    const int m0 = (blockIdx.y * 4 + r) * TM;
    const int per = (nterm + KS * U - 1) / (KS * U) * U;       // terms per slice, a multiple of U
    const int e0 = min(ks * per, nterm), e1 = min(e0 + per, nterm);
    const u64 *wp[TM];
#pragma unroll
    for (int a = 0; a < TM; ++a) wp[a] = w + ((size_t)min(m0 + a, groups - 1) * nterm + e0) * n + i;
    const u64 *xp = xrot + (size_t)e0 * 2 * n + i;
    u64 lo[TM][2], hi[TM][2];
#pragma unroll
    for (int a = 0; a < TM; ++a) lo[a][0] = lo[a][1] = hi[a][0] = hi[a][1] = 0;
    const int nblk = (e1 - e0) / U;
    u64 wa[U][TM], xa[U][2], wb[U][TM], xb[U][2];
    auto load = [&](u64 (&wv)[U][TM], u64 (&xv)[U][2], int blk) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t e = (size_t)blk * U + u;
#pragma unroll
            for (int a = 0; a < TM; ++a) wv[u][a] = wp[a][e * n];
            xv[u][0] = xp[e * 2 * n];
            xv[u][1] = xp[e * 2 * n + n];
        }
    };
    int pending = 0;
    if (nblk > 0) load(wa, xa, 0);
    for (int k = 0; k < nblk; ++k) {
        load(wb, xb, min(k + 1, nblk - 1));         // the last step reads its own block again instead of branching
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int a = 0; a < TM; ++a) {
                mac128(lo[a][0], hi[a][0], xa[u][0], wa[u][a]);
                mac128(lo[a][1], hi[a][1], xa[u][1], wa[u][a]);
            }
        pending += U;
        if (pending + U > flush_every) {            // keep the 128-bit sums of products below q^2 from overflowing
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    lo[a][b] = reduce128(hi[a][b], lo[a][b], mod);
                    hi[a][b] = 0;
                }
            pending = 1;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int a = 0; a < TM; ++a) wa[u][a] = wb[u][a];
            xa[u][0] = xb[u][0];
            xa[u][1] = xb[u][1];
        }
    }
    for (int e = nblk * U; e < e1 - e0; ++e) {      // fewer than U terms left: pending + U <= flush_every holds
        const u64 x0 = xp[(size_t)e * 2 * n], x1 = xp[(size_t)e * 2 * n + n];
#pragma unroll
        for (int a = 0; a < TM; ++a) {
            const u64 wv = wp[a][(size_t)e * n];
            mac128(lo[a][0], hi[a][0], x0, wv);
            mac128(lo[a][1], hi[a][1], x1, wv);
        }
    }
    u64 sum[TM][2];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) sum[a][b] = reduce128(hi[a][b], lo[a][b], mod);
    if (KS > 1) {
        if (ks > 0) {
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b) part[((((ks - 1) * 4 + r) * TM + a) * 2 + b) * 64 + lane] = sum[a][b];
        }
        __syncthreads();
        if (ks > 0) return;
#pragma unroll
        for (int s2 = 1; s2 < KS; ++s2)
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    sum[a][b] = add_mod(sum[a][b], part[((((s2 - 1) * 4 + r) * TM + a) * 2 + b) * 64 + lane], mod.q);
    }
#pragma unroll
    for (int a = 0; a < TM; ++a)
        if (live && m0 + a < groups) {
            acc[((size_t)(m0 + a) * 2) * n + i] = sum[a][0];
            acc[((size_t)(m0 + a) * 2 + 1) * n + i] = sum[a][1];
        }
}

// Slot vectors of a convolution plan's encoded kernels (Sec. III-B(3)): polynomial (O, gamma, term) holds, at the
// slot of pixel (y,x) of channel position (h,kappa), the tap's kernel value between the input channel at that
// position and the output channel that kernel order gamma = (s,t) sends it to, or zero where the tap falls off
// the image or a channel does not exist.  One workgroup per polynomial.
__global__ void conv_weight_slots_kernel(const u64 *K, ConvGeom g, const int *term_ct, const int *term_tap, size_t first,
                                         u64 *slots) {
    const size_t id = first + blockIdx.x;
    const int e = (int)(id % g.nterm), gam = (int)(id / g.nterm % g.cn), O = (int)(id / g.nterm / g.cn);
    const int I = term_ct[e], tap = term_tap[e];
    const int gs = gam / g.hpos, gt = gam % g.hpos, dy = tap / g.k_w - g.k_h / 2, dx = tap % g.k_w - g.k_w / 2;
    const int half = g.n / 2;
    u64 *out = slots + (size_t)blockIdx.x * g.n;
    for (int s = threadIdx.x; s < g.n; s += blockDim.x) {
        const int h = s / half, k = s % half, kap = k / g.T, off = k % g.T, y = off / g.u_w, x = off % g.u_w;
        const int in_ch = I * g.cn + h * g.hpos + kap;
        const int okap = ((kap - gt) % g.hpos + g.hpos) % g.hpos;
        const int out_ch = O * g.cn + (h ^ gs) * g.hpos + okap;
        u64 v = 0;
        if (off < g.u_h * g.u_w && in_ch < g.c_i && out_ch < g.c_o && y + dy >= 0 && y + dy < g.u_h && x + dx >= 0 &&
            x + dx < g.u_w)
            v = K[((size_t)out_ch * g.c_i + in_ch) * g.k_h * g.k_w + tap] % g.p;
        out[s] = v;
    }
}

// Slot vectors of an FC plan's encoded weights ("encode-rowwise", Sec. III-A(3); also the diagonal vectors of the
// hybrid method, Sec. III-A(2)): vector g holds W[row][col] at slot s, with row = slot_row[(h, (k - shift*g) mod n/2)]
// (shift = 1: the vector is rotated left by g after the product; shift = 0: the input was rotated instead) and
// col = slot_col[s] (+ g mod col_period when the input was rotated); zero where row or column do not exist.
// One workgroup per vector.
__global__ void fc_weight_slots_kernel(const u64 *W, FcGeom g, const int *slot_row, u64 *slots) {
    const int gi = blockIdx.x, half = g.n / 2;
    u64 *out = slots + (size_t)gi * g.n;
    for (int s = threadIdx.x; s < g.n; s += blockDim.x) {
        const int h = s / half, k = s % half;
        int row, col;
        if (g.rotate_output) {      // GALA: row of the slot the value moves to, column of the slot it sits in
            row = slot_row[h * half + ((k - gi) % half + half) % half];
            col = g.big ? h * half + k : k % g.nip;
        } else {                    // hybrid: row of this slot, column of the input entry rotated into it
            row = slot_row[s];
            col = g.big ? h * half + (k + gi) % half : (k % g.nip + gi) % g.nip;
        }
        out[s] = (row >= 0 && row < g.n_o && col < g.n_i) ? W[(size_t)row * g.n_i + col] % g.p : 0;
    }
}

// The plaintext half of share generation: every output is the sum of its row's slots mod p (Sec. III-A(3); a
// convolution's rows are single slots).  One workgroup per slot vector; the row sums meet in LDS as plain integers.
__global__ void unpack_share_kernel(const u64 *slots, int nout, int n, u64 p, const int *slot_rowid, const int *row_rindex,
                                    const int *nrows, size_t out_stride, u64 *out) {
    extern __shared__ u64 lds[];
    unsigned long long *acc = reinterpret_cast<unsigned long long *>(lds);
    const int b = blockIdx.x / nout, O = blockIdx.x % nout;
    const u64 *v = slots + (size_t)blockIdx.x * n;
    for (int t = threadIdx.x; t < n; t += blockDim.x) acc[t] = 0;
    __syncthreads();
    for (int s = threadIdx.x; s < n; s += blockDim.x) {
        const int t = slot_rowid[(size_t)O * n + s];
        if (t >= 0) atomicAdd(&acc[t], (unsigned long long)(v[s] % p));
    }
    __syncthreads();
    for (int t = threadIdx.x; t < nrows[O]; t += blockDim.x) out[(size_t)b * out_stride + row_rindex[(size_t)O * n + t]] = acc[t] % p;
}

// Threads of the one-workgroup-per-polynomial kernels: every thread owns at most kMaxPer = 8 coefficients, so rings of
// 4096 and 8192 take 512 and 1024 threads (LDS image of n words: 32 and 64 KiB).
inline int block_threads(int n) { return n >= 8192 ? 1024 : n >= 4096 ? 512 : n >= 512 ? 256 : 64; }
// calls f with the thread count as a compile-time constant
template <class F>
inline void by_threads(int n, F f) {
    switch (block_threads(n)) {
        case 1024: f(std::integral_constant<int, 1024>{}); break;
        case 512: f(std::integral_constant<int, 512>{}); break;
        case 256: f(std::integral_constant<int, 256>{}); break;
        default: f(std::integral_constant<int, 64>{}); break;
    }
}
inline int last_error() { return (int)hipGetLastError(); }

}  // namespace

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
int launch_ntt_mod(const gala_ctx *c, void *stream, const u64 *src, u64 *dst, size_t count, int inverse, const NttDev &T) {
    if (!count) return 0;
    hipStream_t st = (hipStream_t)stream;
    const size_t lds = sizeof(u64) * c->n;
    by_threads(c->n, [&](auto nt) {
        constexpr int NT = decltype(nt)::value;
        hipLaunchKernelGGL(ntt_kernel<NT>, dim3((unsigned)count), dim3(NT), lds, st, src, dst, c->n, c->logn, T, inverse);
    });
    return last_error();
}
int launch_ntt(const gala_ctx *c, void *stream, const u64 *src, u64 *dst, size_t count, int inverse) {
    return launch_ntt_mod(c, stream, src, dst, count, inverse, c->dev_q);
}
int launch_encode_plain(const gala_ctx *c, void *stream, const u64 *slots, int count, int mode, u64 *plain) {
    if (!count) return 0;
    const size_t lds = sizeof(u64) * c->n;
    hipStream_t st = (hipStream_t)stream;
    by_threads(c->n, [&](auto nt) {
        constexpr int NT = decltype(nt)::value;
        hipLaunchKernelGGL(encode_plain_kernel<NT>, dim3((unsigned)count), dim3(NT), lds, st, slots, plain, c->dev_q, c->dev_p,
                           c->d_slot_to_idx, c->n, c->logn, mode, c->delta, c->delta_s);
    });
    return last_error();
}
int launch_ct_op(const gala_ctx *c, void *stream, int op, const u64 *a, const u64 *b, size_t b_stride, int count, u64 *out) {
    if (!count) return 0;
    const size_t words = (size_t)count * 2 * c->n;
    hipLaunchKernelGGL(ct_op_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, (hipStream_t)stream, op, a, b, b_stride,
                       words, c->n, out, c->dev_q.mod);
    return last_error();
}
int launch_conv_weight_slots(const gala_ctx *c, void *stream, const u64 *K, const ConvGeom &g, const int *term_ct,
                             const int *term_tap, size_t first, size_t count, u64 *slots) {
    if (!count) return 0;
    hipLaunchKernelGGL(conv_weight_slots_kernel, dim3((unsigned)count), dim3(block_threads(c->n)), 0, (hipStream_t)stream, K, g,
                       term_ct, term_tap, first, slots);
    return last_error();
}
int launch_fc_weight_slots(const gala_ctx *c, void *stream, const u64 *W, const FcGeom &g, const int *slot_row, int count,
                           u64 *slots) {
    if (count <= 0) return 0;
    hipLaunchKernelGGL(fc_weight_slots_kernel, dim3((unsigned)count), dim3(block_threads(c->n)), 0, (hipStream_t)stream, W, g,
                       slot_row, slots);
    return last_error();
}
int launch_unpack_share(const gala_ctx *c, void *stream, const u64 *slots, int count, int nout, const MaskLayoutDev &layout,
                        size_t out_stride, u64 *out) {
    if (count <= 0) return 0;
    hipLaunchKernelGGL(unpack_share_kernel, dim3((unsigned)((size_t)count * nout)), dim3(block_threads(c->n)), sizeof(u64) * c->n,
                       (hipStream_t)stream, slots, nout, c->n, c->p, layout.slot_rowid, layout.row_rindex, layout.nrows, out_stride,
                       out);
    return last_error();
}
int launch_encrypt(const gala_ctx *c, void *stream, const u64 *s_hat, const u64 *slots, const u64 *seeds, int count,
                   u64 *ct_out) {
    if (!count) return 0;
    if (uses_fast_perm(c)) return launch_encrypt_2048(c, stream, s_hat, slots, seeds, count, ct_out);
    GaussCdf cdf;
    for (int i = 0; i < 2 * kGaussBound; ++i) cdf.t[i] = gauss_cdf_table()[i];
    const size_t lds = sizeof(u64) * c->n;
    hipStream_t st = (hipStream_t)stream;
    by_threads(c->n, [&](auto nt) {
        constexpr int NT = decltype(nt)::value;
        hipLaunchKernelGGL(encrypt_kernel<NT>, dim3((unsigned)count), dim3(NT), lds, st, slots, seeds, s_hat, ct_out, c->dev_q,
                           c->dev_p, c->d_slot_to_idx, cdf, c->n, c->logn, c->qbits, c->delta, c->delta_s);
    });
    return last_error();
}
int launch_decrypt(const gala_ctx *c, void *stream, const u64 *s_hat, const u64 *ct_in, int count, u64 *slots) {
    if (!count) return 0;
    if (uses_fast_perm(c)) return launch_decrypt_2048(c, stream, s_hat, ct_in, count, slots);
    u64 inv = c->q;                                   // Newton's iteration for q^-1 mod 2^64 (q is odd)
    for (int i = 0; i < 6; ++i) inv *= 2 - c->q * inv;
    const size_t lds = sizeof(u64) * c->n;
    hipStream_t st = (hipStream_t)stream;
    by_threads(c->n, [&](auto nt) {
        constexpr int NT = decltype(nt)::value;
        hipLaunchKernelGGL(decrypt_kernel<NT>, dim3((unsigned)count), dim3(NT), lds, st, ct_in, s_hat, slots, c->dev_q, c->dev_p,
                           c->d_slot_to_idx, c->n, c->logn, inv);
    });
    return last_error();
}
int launch_key_finish(const gala_ctx *c, void *stream, u64 *pairs, const u64 *s_hat, size_t npairs, const Modulus &mod) {
    if (!npairs) return 0;
    const size_t total = npairs * c->n;
    hipLaunchKernelGGL(key_finish_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream, pairs,
                       s_hat, c->n, total, mod);
    return last_error();
}
__global__ void owner_order_2048_kernel(const ulonglong2 *src, ulonglong2 *dst) {
    const size_t base = (size_t)blockIdx.x * 2048;
    for (int j = threadIdx.x; j < 2048; j += blockDim.x) {
        const int t = j >> 3, k = j & 7;      // owner thread t, its k-th coefficient
        dst[base + (size_t)(t >> 6) * 512 + k * 64 + (t & 63)] = src[base + j];
    }
}
int launch_owner_order_2048(void *stream, const u64 *src, u64 *dst, size_t npolys) {
    if (!npolys) return 0;
    hipLaunchKernelGGL(owner_order_2048_kernel, dim3((unsigned)npolys), dim3(256), 0, (hipStream_t)stream,
                       reinterpret_cast<const ulonglong2 *>(src), reinterpret_cast<ulonglong2 *>(dst));
    return (int)hipGetLastError();
}
int launch_pair_pack(const gala_ctx *c, void *stream, const u64 *src, u64 *dst, size_t count, int polys) {
    if (!count) return 0;
    hipLaunchKernelGGL(pair_pack_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, (hipStream_t)stream, src,
                       dst, count, c->q, c->special, c->logn, polys);
    return last_error();
}
bool uses_fast_perm(const gala_ctx *c) {
    return c->n == 2048 && c->q < (1ull << 60) &&
           (!c->special || (c->special < (1ull << 60) && c->special < 2 * c->q));
}
int launch_perm_accumulate(const gala_ctx *c, void *stream, const PermJob &job) {
    if (job.items <= 0 || job.nchunks <= 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    const size_t lds = sizeof(u64) * c->n;
    const dim3 grid((unsigned)(job.items * job.nchunks));
    const bool timed = c->prof_which == 0 && (size_t)(2 * c->prof_used + 1) < c->prof_events.size();
    if (timed) (void)hipEventRecord((hipEvent_t)c->prof_events[2 * c->prof_used], st);
    if (uses_fast_perm(c) && !job.in_g_index) {   // the n = 2048 kernels take consecutive inputs only
        const int rc = launch_perm_accumulate_2048(c, stream, job);
        if (timed) (void)hipEventRecord((hipEvent_t)c->prof_events[2 * c->prof_used++ + 1], st);
        return rc;
    }
    const SpecialConst sc{c->Pq, c->Pinv};
    by_threads(c->n, [&](auto nt) {
        constexpr int NT = decltype(nt)::value;
        if (c->special)
            hipLaunchKernelGGL((perm_accumulate_kernel<NT, true>), grid, dim3(NT), lds, st, job, c->dev_q, c->dev_P, sc, c->n,
                               c->logn, c->gadget_bits, c->ndigits);
        else
            hipLaunchKernelGGL((perm_accumulate_kernel<NT, false>), grid, dim3(NT), lds, st, job, c->dev_q, c->dev_q, sc, c->n,
                               c->logn, c->gadget_bits, c->ndigits);
    });
    if (timed) (void)hipEventRecord((hipEvent_t)c->prof_events[2 * c->prof_used++ + 1], st);
    return last_error();
}
int launch_finalize(const gala_ctx *c, void *stream, const FinalizeJob &job) {
    if (job.items <= 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    const size_t lds = sizeof(u64) * c->n;
    by_threads(c->n, [&](auto nt) {
        constexpr int NT = decltype(nt)::value;
        hipLaunchKernelGGL(finalize_kernel<NT>, dim3(job.items), dim3(NT), lds, st, job, c->dev_q, c->dev_p,
                           c->d_slot_to_idx, c->n, c->logn, c->pbits, c->delta, c->delta_s);
    });
    return last_error();
}
int launch_perm_finalize(const gala_ctx *c, void *stream, const PermJob &job, const FinalizeJob &fin) {
    if (uses_fast_perm(c) && fin.r && job.slots > job.nchunks) return launch_perm_accumulate_2048_masked(c, stream, job, fin);
    if (job.in8_S) return (int)hipErrorInvalidValue;     // only the n = 2048 kernel reads blocks of eight
    const int rc = launch_perm_accumulate(c, stream, job);
    return rc ? rc : launch_finalize(c, stream, fin);
}
int launch_decperm(const gala_ctx *c, void *stream, const u64 *ct_in, size_t count, u64 *digits) {
    if (!count) return 0;
    hipStream_t st = (hipStream_t)stream;
    const size_t lds = sizeof(u64) * c->n;
    by_threads(c->n, [&](auto nt) {
        constexpr int NT = decltype(nt)::value;
        hipLaunchKernelGGL(decperm_kernel<NT>, dim3((unsigned)count), dim3(NT), lds, st, ct_in, digits, c->dev_q, c->n,
                           c->logn, c->gadget_bits, c->ndigits);
    });
    return last_error();
}
int launch_hstperm_taps(const gala_ctx *c, void *stream, const u64 *ct_in, const u64 *digits, int batch,
                        const TermList &terms, const u64 *keys, u64 *xrot) {
    if (batch <= 0 || terms.nterm <= 0) return 0;
    hipLaunchKernelGGL(hstperm_taps_kernel, dim3((unsigned)((size_t)batch * terms.nterm)), dim3(block_threads(c->n)), 0,
                       (hipStream_t)stream, ct_in, digits, terms, keys, xrot, c->dev_q.mod, c->n, c->logn, c->ndigits);
    return last_error();
}
int launch_conv_mac(const gala_ctx *c, void *stream, const u64 *w, const u64 *xrot, int batch, int nout, int cn,
                    int nterm, u64 *acc, const int *seg_ptr, const int *seg_terms, int nseg) {
    if (batch <= 0) return 0;
    if (!seg_ptr) nseg = 1;
    const int groups = nout * cn, cols = 2 * batch;
    // products are below q^2: 255 of them fit 128 bits when q < 2^60, 63 when q < 2^61
    const int flush_every = c->q < (1ull << 60) ? 255 : 63;
    hipStream_t st = (hipStream_t)stream;
    // The tile's width follows the number of (input, polynomial) columns; its height is halved until the launch
    // has a few workgroups per compute unit: with few columns the kernel is bound by streaming the encoded kernels
    // and needs the whole chip's loads in flight more than it needs reuse.  A single input (2 columns) has a
    // kernel of its own.
    const unsigned iblocks = (unsigned)((c->n + 63) / 64);
    auto wgs = [&](int tm, int tn, int wm, int wn) {
        return (size_t)iblocks * ((groups + tm * wm - 1) / (tm * wm)) * nseg * ((cols + tn * wn - 1) / (tn * wn));
    };
    const size_t enough = 1024;
#define GALA_MAC(TM, TN, WM, WN)                                                                                      \
    hipLaunchKernelGGL((conv_mac_kernel<TM, TN, WM, WN, 1>),                                                         \
                       dim3(iblocks, (unsigned)((groups + TM * WM - 1) / (TM * WM) * nseg), (unsigned)((cols + TN * WN - 1) / (TN * WN))), \
                       dim3(64 * WM * WN), 0, st, w, xrot, cols, groups, nterm, acc, c->dev_q.mod, c->n, flush_every, seg_ptr, seg_terms, nseg)
    if (cols <= 2 && !seg_ptr) {
        // one input: the streaming kernel, with the tallest row tile that still gives every compute unit a workgroup
        const size_t per_cu = 256;
#define GALA_MACS(TM, KS)                                                                                             \
    hipLaunchKernelGGL((conv_mac_stream_kernel<TM, 2, KS>), dim3(iblocks, (unsigned)((groups + TM * 4 - 1) / (TM * 4))), \
                       dim3(256 * KS), 0, st, w, xrot, groups, nterm, acc, c->dev_q.mod, c->n, flush_every)
        if (wgs(8, 2, 4, 1) >= per_cu) GALA_MACS(8, 2);
        else if (wgs(4, 2, 4, 1) >= per_cu) GALA_MACS(4, 2);
        else if (wgs(2, 2, 4, 1) >= per_cu) GALA_MACS(2, 1);
        else GALA_MACS(1, 1);
#undef GALA_MACS
    } else if (cols <= 4) {
        if (wgs(4, 4, 4, 1) >= enough) GALA_MAC(4, 4, 4, 1);
        else if (wgs(2, 4, 4, 1) >= enough) GALA_MAC(2, 4, 4, 1);
        else GALA_MAC(1, 4, 4, 1);
    } else {
        // wide tiles re-read the inputs once per row tile, so they give up height more reluctantly
        if (wgs(4, 8, 4, 2) >= enough / 2) GALA_MAC(4, 8, 4, 2);
        else if (wgs(2, 8, 4, 2) >= enough / 2) GALA_MAC(2, 8, 4, 2);
        else GALA_MAC(1, 8, 4, 2);
    }
#undef GALA_MAC
    return last_error();
}

}  // namespace gala
