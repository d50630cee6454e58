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

// ---- 64-bit modular primitives shaped for the gfx950 VALU ---------------------------------------
// v_mad_u64_u32 (32x32 + 64 -> 64 with carry-out) issues at the full VALU rate, so everything is built
// from it.  The compiler's own lowering of 64x64 products spends a quarter of its instructions on
// register moves; the sequences below are written out so that it cannot re-associate them.
// CM = true writes the multiply-adds in C instead: the compiler then knows the instruction and leaves out the wait
// state it puts after every inline-asm result, at the price of choosing the registers and the order itself.  The
// special-prime kernels are faster that way, the one-prime kernels are not.
template <bool CM = false>
__device__ __forceinline__ u64 mad_u64(u32 a, u32 b, u64 c) {
    if (CM) return (u64)a * b + c;
    u64 r, carry;
    asm("v_mad_u64_u32 %0, %1, %2, %3, %4" : "=v"(r), "=s"(carry) : "v"(a), "v"(b), "v"(c));
    return r;
}
template <bool CM = false>
__device__ __forceinline__ u64 mul_u64(u32 a, u32 b) {
    if (CM) return (u64)a * b;
    u64 r, carry;
    asm("v_mad_u64_u32 %0, %1, %2, %3, 0" : "=v"(r), "=s"(carry) : "v"(a), "v"(b));
    return r;
}
// high 64 bits of y*s in 6 instructions: with A1 = hi32(y0 s0), B = y0 s1 + A1 and
// S = y1 s0 + B (65 bits: C plus the carry-out), the result is y1 s1 + floor(S / 2^32).
template <bool CM = false>
__device__ __forceinline__ u64 mulhi64_dev(u64 y, u64 s) {
    const u32 y0 = (u32)y, y1 = (u32)(y >> 32), s0 = (u32)s, s1 = (u32)(s >> 32);
    const u64 B = mad_u64<CM>(y0, s1, (u64)__umulhi(y0, s0));
    u64 C, carry;
    asm("v_mad_u64_u32 %0, %1, %2, %3, %4" : "=v"(C), "=s"(carry) : "v"(y1), "v"(s0), "v"(B));
    u32 top;
    asm("v_cndmask_b32_e64 %0, 0, 1, %1" : "=v"(top) : "s"(carry));
    return mad_u64<CM>(y1, s1, ((u64)top << 32) | (u32)(C >> 32));
}
// negated modulus split in two VGPR words, set up once per kernel
struct NegQ { u32 lo, hi; };
// y*w mod q up to one extra q (a value in [0,2q)) for any 64-bit y, w a constant with companion ws:
// y*w - h*q = y*w + h*(-q) mod 2^64 as one chain for the low word and one for the high word.
// ADD: x is added to the product in the same instructions (the first multiply-add of the low chain takes it as its
// addend), so x + (y*w mod q) costs no more than the product; the sum is exact modulo 2^64.
template <bool CM = false, bool ADD = false>
__device__ __forceinline__ u64 mul_const(u64 y, u64 w, u64 ws, NegQ nq, u64 x = 0) {
    const u64 h = mulhi64_dev<CM>(y, ws);
    const u32 y0 = (u32)y, y1 = (u32)(y >> 32), w0 = (u32)w, w1 = (u32)(w >> 32);
    const u32 h0 = (u32)h, h1 = (u32)(h >> 32);
    u64 u = mul_u64<CM>(y0, w1);          // only the low word of this chain is used
    u = mad_u64<CM>(y1, w0, u);
    u = mad_u64<CM>(h0, nq.hi, u);
    u = mad_u64<CM>(h1, nq.lo, u);
    u64 t = ADD ? mad_u64<CM>(y0, w0, x) : mul_u64<CM>(y0, w0);
    t = mad_u64<CM>(h0, nq.lo, t);
    u32 hi;
    asm("v_add_u32 %0, %1, %2" : "=v"(hi) : "v"((u32)(t >> 32)), "v"((u32)u));
    return ((u64)hi << 32) | (u32)t;
}
// The same for y below 2^32 (a gadget digit): the quotient estimate floor(y*ws / 2^64) is the high word of
// y*ws1 + hi32(y*ws0) and fits one word, so five of the twelve instructions have nothing to do.  Same value as mul_const.
template <bool ADD = false>
__device__ __forceinline__ u64 mul_const_small(u32 y, u64 w, u64 ws, NegQ nq, u64 x = 0) {
    const u32 w0 = (u32)w, w1 = (u32)(w >> 32), s0 = (u32)ws, s1 = (u32)(ws >> 32);
    const u32 h = (u32)(mad_u64(y, s1, (u64)__umulhi(y, s0)) >> 32);
    u64 u = mul_u64(y, w1);
    u = mad_u64(h, nq.hi, u);
    u64 t = ADD ? mad_u64(y, w0, x) : mul_u64(y, w0);
    t = mad_u64(h, nq.lo, t);
    u32 hi;
    asm("v_add_u32 %0, %1, %2" : "=v"(hi) : "v"((u32)(t >> 32)), "v"((u32)u));
    return ((u64)hi << 32) | (u32)t;
}
// Two independent constant multiplications, written as three blocks of instructions instead of one statement per
// instruction.  The compiler cannot know that v_mad_u64_u32 forwards its result without a hazard, so it puts a
// wait state between an inline-asm statement and any statement that reads one of its results; inside a block
// there is none.  A block ends where the next step needs one half of a 64-bit result (halves cannot be named
// inside a block).  The two chains alternate, so no instruction reads the result of the one before it.  Carry-outs
// go to vcc except the one that is read through a scalar pair; each of the two carries that are used is read two
// wait states after the multiply-add that wrote it (the spacing the compiler itself keeps between a vector
// instruction that writes a scalar register and one that reads it).
// Measured, this form is 4.5 % faster where both constants already sit in registers (the packed convolution's
// key products), makes no difference in the transforms, and is a tenth slower where each product waits for its
// own loads (the Perm kernel's key products): only the first kind uses it.
__device__ __forceinline__ void mul_const2(u64 &ra, u64 &rb, u64 ya, const ulonglong2 ca, u64 yb, const ulonglong2 cb,
                                           NegQ nq) {
    const u32 a0 = (u32)ya, a1 = (u32)(ya >> 32), b0 = (u32)yb, b1 = (u32)(yb >> 32);
    const u32 wa0 = (u32)ca.x, wa1 = (u32)(ca.x >> 32), sa0 = (u32)ca.y, sa1 = (u32)(ca.y >> 32);
    const u32 wb0 = (u32)cb.x, wb1 = (u32)(cb.x >> 32), sb0 = (u32)cb.y, sb1 = (u32)(cb.y >> 32);
    const u64 A1a = __umulhi(a0, sa0), A1b = __umulhi(b0, sb0);
    u64 Ca, Cb, ua, ub, ta, tb, kb;   // C holds B, then C of mulhi64_dev
    u32 topa, topb;
    asm("v_mad_u64_u32 %[Ca], vcc, %[a0], %[sa1], %[A1a]\n\t"
        "v_mad_u64_u32 %[Cb], vcc, %[b0], %[sb1], %[A1b]\n\t"
        "v_mad_u64_u32 %[Ca], vcc, %[a1], %[sa0], %[Ca]\n\t"
        "v_mad_u64_u32 %[Cb], %[kb], %[b1], %[sb0], %[Cb]\n\t"
        "s_nop 0\n\t"
        "v_cndmask_b32_e64 %[topa], 0, 1, vcc\n\t"
        "v_cndmask_b32_e64 %[topb], 0, 1, %[kb]"
        : [Ca] "=&v"(Ca), [Cb] "=&v"(Cb), [topa] "=v"(topa), [topb] "=v"(topb), [kb] "=&s"(kb)
        : [a0] "v"(a0), [a1] "v"(a1), [b0] "v"(b0), [b1] "v"(b1), [sa0] "v"(sa0), [sa1] "v"(sa1), [sb0] "v"(sb0),
          [sb1] "v"(sb1), [A1a] "v"(A1a), [A1b] "v"(A1b)
        : "vcc");
    u64 ha = ((u64)topa << 32) | (u32)(Ca >> 32), hb = ((u64)topb << 32) | (u32)(Cb >> 32);
    asm("v_mad_u64_u32 %[ha], vcc, %[a1], %[sa1], %[ha]\n\t"
        "v_mad_u64_u32 %[hb], vcc, %[b1], %[sb1], %[hb]"
        : [ha] "+v"(ha), [hb] "+v"(hb)
        : [a1] "v"(a1), [sa1] "v"(sa1), [b1] "v"(b1), [sb1] "v"(sb1)
        : "vcc");
    asm("v_mad_u64_u32 %[ua], vcc, %[a0], %[wa1], 0\n\t"
        "v_mad_u64_u32 %[ub], vcc, %[b0], %[wb1], 0\n\t"
        "v_mad_u64_u32 %[ta], vcc, %[a0], %[wa0], 0\n\t"
        "v_mad_u64_u32 %[tb], vcc, %[b0], %[wb0], 0\n\t"
        "v_mad_u64_u32 %[ua], vcc, %[a1], %[wa0], %[ua]\n\t"
        "v_mad_u64_u32 %[ub], vcc, %[b1], %[wb0], %[ub]\n\t"
        "v_mad_u64_u32 %[ta], vcc, %[ha0], %[ql], %[ta]\n\t"
        "v_mad_u64_u32 %[tb], vcc, %[hb0], %[ql], %[tb]\n\t"
        "v_mad_u64_u32 %[ua], vcc, %[ha0], %[qh], %[ua]\n\t"
        "v_mad_u64_u32 %[ub], vcc, %[hb0], %[qh], %[ub]\n\t"
        "v_mad_u64_u32 %[ua], vcc, %[ha1], %[ql], %[ua]\n\t"
        "v_mad_u64_u32 %[ub], vcc, %[hb1], %[ql], %[ub]"
        : [ua] "=&v"(ua), [ub] "=&v"(ub), [ta] "=&v"(ta), [tb] "=&v"(tb)
        : [a0] "v"(a0), [a1] "v"(a1), [b0] "v"(b0), [b1] "v"(b1), [wa0] "v"(wa0), [wa1] "v"(wa1), [wb0] "v"(wb0),
          [wb1] "v"(wb1), [ha0] "v"((u32)ha), [ha1] "v"((u32)(ha >> 32)), [hb0] "v"((u32)hb), [hb1] "v"((u32)(hb >> 32)),
          [ql] "v"(nq.lo), [qh] "v"(nq.hi)
        : "vcc");
    u32 hia, hib;
    asm("v_add_u32 %0, %1, %2" : "=v"(hia) : "v"((u32)(ta >> 32)), "v"((u32)ua));
    asm("v_add_u32 %0, %1, %2" : "=v"(hib) : "v"((u32)(tb >> 32)), "v"((u32)ub));
    ra = ((u64)hia << 32) | (u32)ta;
    rb = ((u64)hib << 32) | (u32)tb;
}
struct U64Pair { u64 a, b; };
__device__ __forceinline__ U64Pair mul_const_pair(u64 ya, const ulonglong2 ca, u64 yb, const ulonglong2 cb, NegQ nq) {
    U64Pair r;
    mul_const2(r.a, r.b, ya, ca, yb, cb, nq);
    return r;
}
// x - c if x >= c else x, in 4 instructions (the borrow of the subtraction selects);
// needs x - c < 2^63 when x >= c, which holds for every use here (x < 2c, c <= 8q < 2^63).
__device__ __forceinline__ u64 csub_dev(u64 x, u64 c) {
    u32 r0, r1;
    asm("v_sub_co_u32 %0, vcc, %2, %4\n\tv_subb_co_u32 %1, vcc, %3, %5, vcc\n\t"
        "v_cndmask_b32 %0, %0, %2, vcc\n\tv_cndmask_b32 %1, %1, %3, vcc"
        : "=&v"(r0), "=&v"(r1)
        : "v"((u32)x), "v"((u32)(x >> 32)), "v"((u32)c), "v"((u32)(c >> 32))
        : "vcc");
    return ((u64)r1 << 32) | r0;
}

// x,y -> x + w*y, x - w*y + 2q  without any correction (bound grows by 2q per stage)
template <bool CM = false>
__device__ __forceinline__ void bf_fwd(u64 &x, u64 &y, const ulonglong2 t, NegQ nq, u64 q2) {
    const u64 s = mul_const<CM, true>(y, t.x, t.y, nq, x);      // x + w*y
    y = (x << 1) + q2 - s;                                      // x - w*y + 2q = 2x + 2q - (x + w*y)
    x = s;
}
// the forward butterfly when y is below 2^32
__device__ __forceinline__ void bf_fwd_small(u64 &x, u64 &y, const ulonglong2 t, NegQ nq, u64 q2) {
    const u64 s = mul_const_small<true>((u32)y, t.x, t.y, nq, x);
    y = (x << 1) + q2 - s;
    x = s;
}
// x, y -> x + y, (x - y + off)*w.  The sum is left uncorrected (its bound is the sum of the operands'), and `off`, a
// multiple of q above y's bound, keeps the difference non-negative.  The product is below 2q whatever comes in, so
// only the sums grow; a radix-8 pass lets them (2q -> 4q -> 8q -> 16q < 2^64) and corrects at its end.
template <bool CM = false>
__device__ __forceinline__ void bf_inv_lazy(u64 &x, u64 &y, const ulonglong2 t, NegQ nq, u64 off) {
    const u64 s = x + y, d = x - y + off;
    x = s;
    y = mul_const<CM>(d, t.x, t.y, nq);
}

// The seven constants one thread needs for a radix-8 pass on index bits B..B+2 are tw[T], tw[2T], tw[2T+1],
// tw[4T..4T+3] of the natural table order, with T = (n >> (B+3)) + (index >> (B+3)): "block" T.  A pass uses the
// blocks c .. 2c-1 of one level c (1, 8, 64, 256 forward; 256, 32, 4, 1 inverse).  The table is stored level by
// level with the constant's number before the block's: level c is [e][j] = constant e of block c + j.  Constant e
// of the 64 lanes of a wavefront is then 16 to 1024 contiguous bytes; stored block by block (128 bytes per block)
// the same load touched up to 64 different lines, and the twiddles were two thirds of all the lines the Perm
// kernel asked its vector cache for.
//
// Radix-8 forward pass on the three index bits held in the register number (bit 2 of k first).
// FIRST = false skips the first stage (the last pass of the transform has only two stages).
// The seven constants of a pass are fetched with tw_level() BEFORE the exchange that precedes the pass: a load
// cannot move across the exchange's barrier, and issued after it its latency is fully exposed, pass after pass.
struct Tw7 {
    ulonglong2 t[7];
};
// offset, in pairs, of level c inside a direction's table (levels 1, 4, 8, 32, 64, 256 in this order)
__device__ __forceinline__ constexpr int level_offset(int c) {
    return 7 * (c > 1 ? 1 : 0) + 7 * (c > 4 ? 4 : 0) + 7 * (c > 8 ? 8 : 0) + 7 * (c > 32 ? 32 : 0) + 7 * (c > 64 ? 64 : 0);
}
// constants of block COUNT + j: the level's start is uniform, j*16 a 32-bit offset
template <int COUNT>
__device__ __forceinline__ Tw7 tw_level(const ulonglong2 *__restrict__ table, unsigned j) {
    const char *level = reinterpret_cast<const char *>(table + level_offset(COUNT));
    const unsigned off = j * 16u;
    Tw7 w;
#pragma unroll
    for (int e = 0; e < 7; ++e) w.t[e] = *reinterpret_cast<const ulonglong2 *>(level + (size_t)(e * COUNT * 16) + off);
    return w;
}
// small_in (the same for every thread): all eight inputs are below 2^32, as gadget digits are; the first stage then
// multiplies with mul_const_small.
template <bool FIRST, bool CORRECT, bool CM = false>
__device__ __forceinline__ void fwd_pass(u64 (&a)[8], const Tw7 &w, NegQ q, u64 q2, bool small_in = false) {
    if (FIRST) {
        if (!CM && small_in) {
#pragma unroll
            for (int k = 0; k < 4; ++k) bf_fwd_small(a[k], a[k + 4], w.t[0], q, q2);
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) bf_fwd<CM>(a[k], a[k + 4], w.t[0], q, q2);
        }
    }
    if (CORRECT) {   // seven stages done: everything is below 15q, bring it below 8q
        const u64 q8 = 4 * q2;
#pragma unroll
        for (int k = 0; k < 8; ++k) a[k] = csub_dev(a[k], q8);
    }
    bf_fwd<CM>(a[0], a[2], w.t[1], q, q2);
    bf_fwd<CM>(a[1], a[3], w.t[1], q, q2);
    bf_fwd<CM>(a[4], a[6], w.t[2], q, q2);
    bf_fwd<CM>(a[5], a[7], w.t[2], q, q2);
    bf_fwd<CM>(a[0], a[1], w.t[3], q, q2);
    bf_fwd<CM>(a[2], a[3], w.t[4], q, q2);
    bf_fwd<CM>(a[4], a[5], w.t[5], q, q2);
    bf_fwd<CM>(a[6], a[7], w.t[6], q, q2);
}
// Radix-8 inverse pass (bit 0 of k first), same block layout on the inverse table.
template <bool CM = false>
__device__ __forceinline__ void inv_pass(u64 (&a)[8], const Tw7 &w, NegQ q, u64 q2) {
    // all eight below 2q on entry; bounds after each stage in the comments
    const u64 q4 = 2 * q2, q8 = 4 * q2;
    bf_inv_lazy<CM>(a[0], a[1], w.t[3], q, q2);
    bf_inv_lazy<CM>(a[2], a[3], w.t[4], q, q2);
    bf_inv_lazy<CM>(a[4], a[5], w.t[5], q, q2);
    bf_inv_lazy<CM>(a[6], a[7], w.t[6], q, q2);      // a0 a2 a4 a6 < 4q, the products a1 a3 a5 a7 < 2q
    bf_inv_lazy<CM>(a[0], a[2], w.t[1], q, q4);
    bf_inv_lazy<CM>(a[1], a[3], w.t[1], q, q2);
    bf_inv_lazy<CM>(a[4], a[6], w.t[2], q, q4);
    bf_inv_lazy<CM>(a[5], a[7], w.t[2], q, q2);      // a0 a4 < 8q, a1 a5 < 4q, a2 a3 a6 a7 < 2q
    bf_inv_lazy<CM>(a[0], a[4], w.t[0], q, q8);
    bf_inv_lazy<CM>(a[1], a[5], w.t[0], q, q4);
    bf_inv_lazy<CM>(a[2], a[6], w.t[0], q, q2);
    bf_inv_lazy<CM>(a[3], a[7], w.t[0], q, q2);      // a0 < 16q, a1 < 8q, a2 a3 < 4q, a4 .. a7 < 2q
    a[0] = csub_dev(csub_dev(csub_dev(a[0], q8), q4), q2);
    a[1] = csub_dev(csub_dev(a[1], q4), q2);
    a[2] = csub_dev(a[2], q2);
    a[3] = csub_dev(a[3], q2);
}

// Store the 8 registers at index(k) = base_out | (k << SH_OUT), barrier, load index(k) = base_in | (k << SH_IN).
// The bases have zeros in the three bits the register number fills, so the padded address of
// register k is pad(base) plus a compile-time offset.
template <int SH>
__device__ __forceinline__ constexpr int reg_offset(int k) { return (k << SH) + ((k << SH) >> 5); }
// LOCAL: every word a thread loads was stored by a thread of its own wavefront (both index sets lie in the
// wavefront's 512-word range of the buffer).  A wavefront's LDS instructions execute in order, so its loads see
// its stores without a workgroup barrier; the fences only keep the compiler from moving the loads up.  Four of
// the seven exchanges of an inverse + forward transform pair are of this kind: <5,2> and <2,0> move data inside
// groups of 32 and 4 lanes, <0,3> and <3,6> inside groups of 8 and 64; <8,5>, <6,8> and the final store of the
// forward transform cross wavefronts and keep the barrier.
template <int SH_OUT, int SH_IN, bool LOCAL = false>
__device__ __forceinline__ void exchange(u64 (&a)[8], u64 *buf, int base_out, int base_in) {
    u64 *po = buf + pad(base_out);
#pragma unroll
    for (int k = 0; k < 8; ++k) po[reg_offset<SH_OUT>(k)] = a[k];
    if (LOCAL) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    } else {
        __syncthreads();
    }
    const u64 *pi = buf + pad(base_in);
#pragma unroll
    for (int k = 0; k < 8; ++k) a[k] = pi[reg_offset<SH_IN>(k)];
}

struct Tables2048 {
    const ulonglong2 *tw, *itw;   // level-major (w, companion) pairs, forward and inverse (see tw_level)
    ulonglong2 ninv, itw1n;       // n^-1 and itw[1]*n^-1 with companions
    Modulus mod;
    NegQ nq;                      // 2^64 - q
};

// The thread id goes through an empty asm so that the address arithmetic of a transform is redone
// where it is used instead of being hoisted out of the rotation loop into long-lived registers.
__device__ __forceinline__ int fresh(int tid) {
    asm volatile("" : "+v"(tid));
    return tid;
}

// Forward transform of the 8 registers (ownership t + 256k, values below q); the result is left in
// LDS buffer `res` (natural index, padded), values below 16q.  LDS phases: other, res, other, res.
template <bool CM = false>
__device__ __forceinline__ void forward_to_lds(u64 (&a)[8], u64 *res, u64 *other, const Tables2048 &T, int tid_,
                                               bool small_in = false) {
    const int tid = fresh(tid_);
    const NegQ q = T.nq;
    const u64 q2 = T.mod.q2;
    Tw7 w = tw_level<1>(T.tw, 0);
    fwd_pass<true, false, CM>(a, w, q, q2, small_in);                                    // bits 8-10
    w = tw_level<8>(T.tw, (unsigned)tid >> 5);
    exchange<8, 5>(a, other, tid, ((tid >> 5) << 8) | (tid & 31));
    fwd_pass<true, false, CM>(a, w, q, q2);                                              // bits 5-7
    w = tw_level<64>(T.tw, (unsigned)tid >> 2);
    exchange<5, 2, true>(a, res, ((tid >> 5) << 8) | (tid & 31), ((tid >> 2) << 5) | (tid & 3));
    fwd_pass<true, true, CM>(a, w, q, q2);                                               // bits 2-4
    w = tw_level<256>(T.tw, (unsigned)tid);
    exchange<2, 0, true>(a, other, ((tid >> 2) << 5) | (tid & 3), tid << 3);
    fwd_pass<false, false, CM>(a, w, q, q2);                                             // bits 0-1
    u64 *po = res + pad(tid << 3);
#pragma unroll
    for (int k = 0; k < 8; ++k) po[k] = a[k];
    __syncthreads();
}

// Inverse transform: registers hold index 8t + k (values below 2q) on entry and index t + 256k,
// canonical, on return.
template <bool CM = false>
__device__ __forceinline__ void inverse_in_regs(u64 (&a)[8], u64 *bufA, u64 *bufB, const Tables2048 &T, int tid_) {
    const int tid = fresh(tid_);
    const NegQ q = T.nq;
    const u64 q2 = T.mod.q2;
    Tw7 w = tw_level<256>(T.itw, (unsigned)tid);
    inv_pass<CM>(a, w, q, q2);                                                           // bits 0-2
    w = tw_level<32>(T.itw, (unsigned)tid >> 3);
    exchange<0, 3, true>(a, bufA, tid << 3, ((tid >> 3) << 6) | (tid & 7));
    inv_pass<CM>(a, w, q, q2);                                                           // bits 3-5
    w = tw_level<4>(T.itw, (unsigned)tid >> 6);
    exchange<3, 6, true>(a, bufB, ((tid >> 3) << 6) | (tid & 7), ((tid >> 6) << 9) | (tid & 63));
    inv_pass<CM>(a, w, q, q2);                                                           // bits 6-8
    const ulonglong2 t2a = T.itw[1], t2b = T.itw[2];      // level 1: constants 1 and 2 of block 1
    exchange<6, 8>(a, bufA, ((tid >> 6) << 9) | (tid & 63), tid);
    // bits 9-10 (register bits 1,2; register bit 0 is index bit 8), n^-1 folded into the last stage
    bf_inv_lazy<CM>(a[0], a[2], t2a, q, q2);
    bf_inv_lazy<CM>(a[1], a[3], t2a, q, q2);
    bf_inv_lazy<CM>(a[4], a[6], t2b, q, q2);
    bf_inv_lazy<CM>(a[5], a[7], t2b, q, q2);         // the sums a0 a1 a4 a5 < 4q, the products a2 a3 a6 a7 < 2q
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const u64 x = a[k], y = a[k + 4];
        a[k] = csub_dev(mul_const<CM>(x + y, T.ninv.x, T.ninv.y, q), T.mod.q);
        a[k + 4] = csub_dev(mul_const<CM>(x - y + 2 * q2, T.itw1n.x, T.itw1n.y, q), T.mod.q);
    }
}

// below 16q -> canonical
__device__ __forceinline__ u64 reduce64(u64 x, const Modulus &m) {
    return csub(x - mulhi64(x, m.one_s) * m.q, m.q);
}

// Share generation inside the same launch: the workgroups after the last (item, chunk) pair build the
// negated mask of one output ciphertext each and store it as one more partial ciphertext.
struct MaskJob {
    int enabled;
    int nout;                   // output ciphertexts per batch element
    const u64 *r;               // batch x r_stride server shares mod p
    size_t r_stride;
    u64 mask_seed;
    MaskLayoutDev layout;
    const int *slot_to_idx;
    int pbits;
    ulonglong2 delta;           // delta = floor(q/p) and its companion mod q
    Tables2048 Tp;              // inverse-transform tables of the plaintext modulus
};

__device__ __forceinline__ void mask_role(const PermJob &job, const Tables2048 &T, const MaskJob &mj, int item,
                                          u64 *bufA, u64 *bufB) {
    const int tid = threadIdx.x;
    const int b = item / mj.nout, O = item % mj.nout;
    const u64 p = mj.Tp.mod.q, q = T.mod.q;
    const int *row_ptr = mj.layout.row_ptr + (size_t)O * (N + 1);
    const int *row_rindex = mj.layout.row_rindex + (size_t)O * N;
    const unsigned char *is_first = mj.layout.is_first + (size_t)O * N;
    // every slot but the first of each real output is a draw from the mask stream; values go to the
    // position the mod-p transform expects them at
    for (int s = tid; s < N; s += NT) {
        u64 v = 0;
        if (!is_first[s]) v = draw_uniform(p, mj.pbits, mj.mask_seed, kStreamMask, ((u64)b << 32) + ((u64)O << 16) + (u64)s);
        bufB[mj.slot_to_idx[s]] = v;
    }
    __syncthreads();
    // the first slot of every real row absorbs r minus the row's other slots.  The row sums are formed by all
    // threads: a thread adds up its strip of consecutive entries and flushes to the row's cell in LDS whenever the
    // row changes (plain integer sums of values below p: at most n of them, far from 64 bits).
    const int nrows = mj.layout.nrows[O];
    const int *entry_row = mj.layout.entry_row + (size_t)O * N, *entry_idx = mj.layout.entry_idx + (size_t)O * N;
    const int *first_idx = mj.layout.first_idx + (size_t)O * N;
    unsigned long long *rowsum = reinterpret_cast<unsigned long long *>(bufA);
    const int nent = row_ptr[nrows];
    const bool sums = nent > nrows;      // rows of a single slot (convolutions) have nothing to add up
    if (sums) {
        for (int t = tid; t < nrows; t += NT) rowsum[t] = 0;
        __syncthreads();
        int cur = -1;
        u64 acc = 0;
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int e = PER * tid + k;
            const int t = e < nent ? entry_row[e] : -1;
            if (t < 0) continue;
            if (t != cur) {
                if (cur >= 0) atomicAdd(&rowsum[cur], acc);
                cur = t;
                acc = 0;
            }
            acc += bufB[entry_idx[e]];
        }
        if (cur >= 0) atomicAdd(&rowsum[cur], acc);
        __syncthreads();
    }
    for (int t = tid; t < nrows; t += NT) {
        if (row_ptr[t + 1] <= row_ptr[t]) continue;
        u64 rv = mj.r[(size_t)b * mj.r_stride + row_rindex[t]];
        if (rv >= p) rv %= p;
        bufB[first_idx[t]] = sub_mod(rv, sums ? rowsum[t] % p : 0, p);
    }
    __syncthreads();
    // slots -> plaintext polynomial (inverse transform mod p) -> delta * m mod q -> evaluation domain mod q
    u64 a[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) a[k] = bufB[8 * tid + k];
    inverse_in_regs(a, bufA, bufB, mj.Tp, tid);        // LDS phases A B A; the reads of bufB above precede the first barrier
#pragma unroll
    for (int k = 0; k < PER; ++k) a[k] = csub_dev(mul_const(a[k], mj.delta.x, mj.delta.y, T.nq), q);
    forward_to_lds(a, bufA, bufB, T, tid);             // LDS phases B A B A, result in bufA (below 16q)
    u64 *out = job.partial + ((size_t)item * job.slots + job.nchunks) * 2 * N;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int i = tid + k * NT;
        const u64 m = reduce64(bufA[pad(i)], T.mod);
        out[i] = m ? q - m : 0;       // minus the mask on c0
        out[N + i] = 0;
    }
}

// Workgroup -> (item, chunk).  Consecutive workgroup ids go to the eight XCDs in turn, each with an L2 of its own.
// When the chunk count is a multiple of eight, chunk c is always given to XCD c % 8, so that an XCD only ever
// reads the keys and weights of its own chunks and they stay in its L2.
__device__ __forceinline__ void item_and_chunk(const PermJob &job, int &item, int &chunk) {
    const int w = blockIdx.x;
    if ((job.nchunks & 7) == 0) {
        const int per = job.nchunks >> 3, s = w >> 3;
        chunk = (w & 7) + 8 * (s % per);
        item = s / per;
    } else {
        item = w / job.nchunks;
        chunk = w % job.nchunks;
    }
}

// Every product on this path is a multiplication by a constant that carries its precomputed
// quotient (twiddles, encoded weights, key polynomials), so sums of products stay in 64-bit
// registers: each product is below 2q, a running sum is kept below 8q and may take four more
// products before one conditional subtraction of 8q.
// IN8: the inputs lie in blocks of eight coefficients (PermJob::in8_S), as the matrix-core product leaves them.
template <bool HAS_W, bool IN8 = false>
__global__ __launch_bounds__(NT) void perm_accumulate_2048(PermJob job, Tables2048 T, MaskJob mj, int gadget_bits,
                                                           int ndigits) {
    __shared__ u64 bufA[LDS_WORDS], bufB[LDS_WORDS];
    __shared__ u64 stash[N];   // each thread parks its 8 coefficients here between digits (private slots, no barrier)
    const int tid = threadIdx.x;
    if ((int)blockIdx.x >= job.items * job.nchunks) {   // only launched when mj.enabled
        mask_role(job, T, mj, (int)blockIdx.x - job.items * job.nchunks, bufA, bufB);
        return;
    }
    int item, chunk;
    item_and_chunk(job, item, chunk);
    int g0, g1;
    chunk_range(chunk, job.nchunks, job.G, g0, g1);
    const NegQ q = T.nq;
    const u64 q8 = 8 * T.mod.q;
    const u64 digit_mask = (1ull << gadget_bits) - 1;
    const size_t key_pairs = (size_t)ndigits * 2 * N;

    u64 sum0[PER], sum1[PER];   // running sums over the rotations of this chunk, below 8q between products
#pragma unroll
    for (int k = 0; k < PER; ++k) sum0[k] = sum1[k] = 0;

    for (int g = g0; g < g1; ++g) {
        const u64 *c0 = IN8 ? job.ct_in + (size_t)(item % job.in8_nout) * job.in8_o_stride + (size_t)(item / job.in8_nout) * 16 +
                                  (size_t)g * job.in_g_stride
                            : job.ct_in + (size_t)item * job.in_item_stride + (size_t)g * job.in_g_stride;
        const u64 *c1 = IN8 ? c0 + 8 : c0 + N;
        const size_t S = IN8 ? job.in8_S : 0;
        auto at = [&](const u64 *poly, int i) -> u64 { return IN8 ? poly[(size_t)(i >> 3) * S + (i & 7)] : poly[i]; };
        const ulonglong2 *w = HAS_W ? reinterpret_cast<const ulonglong2 *>(job.w2) + (size_t)g * N : nullptr;
        // middle of this wavefront's 8 KiB in the ownership-order copy: all eight loads are immediate offsets of it
        const char *wo = HAS_W ? reinterpret_cast<const char *>(w + (size_t)job.G * N) : nullptr;
        const unsigned wmid = ((unsigned)(fresh(tid) >> 6) * 512u + 256u + (unsigned)(tid & 63)) * 16u;
        const int gal = job.gal[g];
        if (gal == 1) {   // rotation by zero: ScMult and Add only
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                const int i = tid + k * NT;
                if (HAS_W) {
                    const ulonglong2 ww = w[i];
                    sum0[k] = csub_dev(mul_const<false, true>(c0[i], ww.x, ww.y, q, sum0[k]), q8);
                    sum1[k] = csub_dev(mul_const<false, true>(c1[i], ww.x, ww.y, q, sum1[k]), q8);
                } else {
                    sum0[k] = csub_dev(sum0[k] + at(c0, i), q8);
                    sum1[k] = csub_dev(sum1[k] + at(c1, i), q8);
                }
            }
            continue;
        }
        // LDS phases of one rotation: A B A (inverse), then B A B A per digit.  Consecutive phases use
        // different buffers, which is what lets each exchange do with one barrier; a rotation ends on
        // A and the next one starts on A, so that one boundary needs a barrier of its own.
        __syncthreads();
        const ulonglong2 *key = reinterpret_cast<const ulonglong2 *>(job.keys2) + (size_t)job.key_idx[g] * key_pairs;
        int src[PER];   // where the automorphism takes output index tid + 256k from
#pragma unroll
        for (int k = 0; k < PER; ++k) src[k] = galois_index11(tid + k * NT, gal);

        // ScMult of c1 (8 consecutive coefficients per thread), then the inverse transform
        u64 a[PER];
        {
            const ulonglong2 *c1v = reinterpret_cast<const ulonglong2 *>(IN8 ? c1 + (size_t)tid * S : c1 + 8 * tid);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const ulonglong2 cv = c1v[k];
                if (HAS_W) {     // the copy in ownership order: 64 lanes read 1 KiB of whole lines
                    const ulonglong2 wa = *reinterpret_cast<const ulonglong2 *>(wo + (wmid + (unsigned)((2 * k - 4) * 1024))),
                                     wb = *reinterpret_cast<const ulonglong2 *>(wo + (wmid + (unsigned)((2 * k - 3) * 1024)));
                    a[2 * k] = mul_const(cv.x, wa.x, wa.y, q);
                    a[2 * k + 1] = mul_const(cv.y, wb.x, wb.y, q);
                } else {
                    a[2 * k] = cv.x;
                    a[2 * k + 1] = cv.y;
                }
            }
        }
        inverse_in_regs(a, bufA, bufB, T, tid);
#pragma unroll
        for (int k = 0; k < PER; ++k) stash[tid + k * NT] = a[k];

        // the c0 part: permuted c0 (.) w
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            if (HAS_W) {
                const ulonglong2 ww = w[src[k]];
                sum0[k] = mul_const<false, true>(c0[src[k]], ww.x, ww.y, q, sum0[k]);
            } else {
                sum0[k] += at(c0, src[k]);
            }
        }
        int pending = 1;   // products added to sum0 since it was last brought below 8q
        for (int j = 0; j < ndigits; ++j) {
#pragma unroll
            for (int k = 0; k < PER; ++k) a[k] = (stash[tid + k * NT] >> (j * gadget_bits)) & digit_mask;
            // result in bufA, any 64-bit value below 16q.  The cheaper first stage for digits below 2^32 only where
            // the registers allow it: in the variants without weights it pushes the count past three workgroups per CU
            forward_to_lds(a, bufA, bufB, T, tid, HAS_W && gadget_bits <= 32);
            const ulonglong2 *kb = key + (size_t)(2 * j) * N, *ka = kb + N;
            if (pending == 4) {
#pragma unroll
                for (int k = 0; k < PER; ++k) {
                    sum0[k] = csub_dev(sum0[k], q8);
                    sum1[k] = csub_dev(sum1[k], q8);
                }
                pending = 0;
            }
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                const int i = tid + k * NT;
                const u64 d = bufA[pad(src[k])];
                const ulonglong2 b = kb[i], aa = ka[i];
                sum0[k] = mul_const<false, true>(d, b.x, b.y, q, sum0[k]);       // the sum rides on the product
                sum1[k] = mul_const<false, true>(d, aa.x, aa.y, q, sum1[k]);
            }
            ++pending;
        }
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            sum0[k] = csub_dev(sum0[k], q8);
            sum1[k] = csub_dev(sum1[k], q8);
        }
    }
    u64 *out = job.partial + ((size_t)item * job.slots + chunk) * 2 * N;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int i = tid + k * NT;
        out[i] = reduce64(sum0[k], T.mod);
        out[N + i] = reduce64(sum1[k], T.mod);
    }
}

// Hoisted rotations of the input ciphertexts (Sec. III-B: one DecPerm shared by all the taps of a kernel,
// then one HstPerm per tap), as two launches so that both fill the chip at small batches.
//
// DecPerm: one workgroup per (ciphertext, digit); each repeats the inverse transform of c1 and runs the
// forward transform of its digit.  digits[ct][j][i] holds lazy values (any 64-bit word below 16q), which is
// what the constant multiplications of the inner product accept.
constexpr int HOIST_DIGITS = 3;
__global__ __launch_bounds__(NT) void decperm_2048(const u64 *ct_in, u64 *digits, Tables2048 T, int gadget_bits,
                                                   int ndigits) {
    __shared__ u64 bufA[LDS_WORDS], bufB[LDS_WORDS];
    const int tid = threadIdx.x;
    const int ct = blockIdx.x / ndigits, j = blockIdx.x % ndigits;
    const u64 *c1 = ct_in + (size_t)ct * 2 * N + N;
    u64 a[PER];
    const ulonglong2 *c1v = reinterpret_cast<const ulonglong2 *>(c1 + 8 * tid);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const ulonglong2 cv = c1v[k];
        a[2 * k] = cv.x;
        a[2 * k + 1] = cv.y;
    }
    inverse_in_regs(a, bufA, bufB, T, tid);      // LDS phases A B A
    const u64 digit_mask = (1ull << gadget_bits) - 1;
#pragma unroll
    for (int k = 0; k < PER; ++k) a[k] = (a[k] >> (j * gadget_bits)) & digit_mask;
    forward_to_lds(a, bufA, bufB, T, tid, gadget_bits <= 32);       // LDS phases B A B A, ends on a barrier
    u64 *out = digits + ((size_t)ct * ndigits + j) * N;
#pragma unroll
    for (int k = 0; k < PER; ++k) out[tid + k * NT] = bufA[pad(tid + k * NT)];
}

// HstPerm: one workgroup per (ciphertext, tap).  c0 and the digits are read through the automorphism's index
// map straight from memory: the map sends every aligned block of 64 indices onto another such block, so a
// wavefront's gather still touches whole cache lines.  Output: xrot[ct][tap][c0|c1][i], canonical.
__global__ __launch_bounds__(NT) void hstperm_taps_2048(const u64 *ct_in, const u64 *digits, TermList terms,
                                                        const u64 *keys2, u64 *xrot, Tables2048 T, int ndigits) {
    const int tid = threadIdx.x;
    const int b = blockIdx.x / terms.nterm, e = blockIdx.x % terms.nterm;
    const size_t ct = (size_t)b * terms.nin + terms.ct[e];
    const u64 *c0 = ct_in + ct * 2 * N, *c1 = c0 + N;
    u64 *out = xrot + (size_t)blockIdx.x * 2 * N;
    const int gal = terms.gal[e];
    if (gal == 1) {
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int i = tid + k * NT;
            out[i] = c0[i];
            out[N + i] = c1[i];
        }
        return;
    }
    const NegQ q = T.nq;
    const u64 *dsrc = digits + ct * ndigits * N;
    const ulonglong2 *key = reinterpret_cast<const ulonglong2 *>(keys2) + (size_t)terms.key[e] * ndigits * 2 * N;
    // two batches of four coefficients keep the loads of a batch in flight together at a modest register count
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        constexpr int H = PER / 2;
        int idx[H], src[H];
        u64 s0[H], s1[H];
#pragma unroll
        for (int k = 0; k < H; ++k) {
            idx[k] = tid + (half * H + k) * NT;
            src[k] = galois_index11(idx[k], gal);
            s0[k] = c0[src[k]];
            s1[k] = 0;
        }
        for (int j = 0; j < ndigits; ++j) {
            const ulonglong2 *kb = key + (size_t)(2 * j) * N, *ka = kb + N;
            ulonglong2 b[H], aa[H];
            u64 d[H];
#pragma unroll
            for (int k = 0; k < H; ++k) {
                d[k] = dsrc[(size_t)j * N + src[k]];
                b[k] = kb[idx[k]];
                aa[k] = ka[idx[k]];
            }
#pragma unroll
            for (int k = 0; k < H; ++k) {
                s0[k] += mul_const(d[k], b[k].x, b[k].y, q);    // each product is below 2q: at most 7q in all
                s1[k] += mul_const(d[k], aa[k].x, aa[k].y, q);
            }
        }
#pragma unroll
        for (int k = 0; k < H; ++k) {
            out[idx[k]] = reduce64(s0[k], T.mod);
            out[N + idx[k]] = reduce64(s1[k], T.mod);
        }
    }
}

// HstPerm of all taps written straight into the column-operand image of the matrix-core multiply-accumulate
// (16-byte chunks [tile][kblock][lane][i][digit], lane = 16*(term block % 4) + column % 16, one balanced
// base-256 digit of 16 consecutive terms per chunk).  One thread owns one coefficient of one input and 16
// consecutive terms (input ciphertext, tap), so a chunk is assembled in registers and the eight digit
// chunks of a coefficient leave as 128 contiguous bytes.
typedef int v4i_t __attribute__((ext_vector_type(4)));
// ND: the number of digits when it is 3 (unrolled), else 0 (run-time loop).  ANY_ROT false: no term rotates, there
// are no keys and no digits to read.
template <int ND, bool ANY_ROT>
__global__ __launch_bounds__(NT) void hstperm_pack_2048(const u64 *ct_in, const u64 *digits, TermList terms, int kblocks,
                                                        const u64 *keys2, v4i_t *xl, Tables2048 T, int ndigits_rt, int batch) {
    // a workgroup is 64 coefficients x 4 inputs: its wavefronts read the same key words, which then come out of
    // the vector cache for three of them
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = blockIdx.x * 64 + lane, eb = blockIdx.y;
    const bool b_live = (int)blockIdx.z * 4 + wave < batch;
    const int b = min((int)blockIdx.z * 4 + wave, batch - 1);
    const int nterm = terms.nterm, ndigits = ND ? ND : ndigits_rt;
    const NegQ q = T.nq;
    const size_t key_pairs = (size_t)ndigits * 2 * N;
    // Terms come in (tap, input ciphertext) order, so the sixteen terms of a thread share their rotation in runs: the
    // automorphism's source index and the key pairs of the tap are fetched when the rotation changes (a decision all
    // lanes share), not per term; what differs from term to term is the input ciphertext, i.e. c0 and the digits at
    // the source index.  Terms of the central tap (no rotation) are copies.  A term past the end repeats the last
    // one and is zeroed.
    u64 D0[16], D1[16];     // balanced digits of the 16 terms' c0 and c1 values
    constexpr int KD = ND ? ND : 1;
    ulonglong2 kwb[KD], kwa[KD];
    const ulonglong2 *key = nullptr;
    int cur_gal = 0, src = i;
    bool ident = true;
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const int e = min(eb * 16 + t, nterm - 1);
        const bool live = eb * 16 + t < nterm;
        const int gal = terms.gal[e];
        if (gal != cur_gal) {          // the same for every lane
            cur_gal = gal;
            ident = gal == 1;
            src = ident ? i : galois_index11(i, gal);
            if (ANY_ROT && !ident) {
                key = reinterpret_cast<const ulonglong2 *>(keys2) + (size_t)terms.key[e] * key_pairs;
                if (ND) {
#pragma unroll
                    for (int j = 0; j < KD; ++j) {
                        kwb[j] = key[(size_t)(2 * j) * N + i];
                        kwa[j] = key[(size_t)(2 * j + 1) * N + i];
                    }
                }
            }
        }
        const size_t ct = (size_t)b * terms.nin + terms.ct[e];
        const u64 *c0 = ct_in + ct * 2 * N;
        u64 v0, v1;
        if (!ANY_ROT || ident) {
            v0 = c0[i];
            v1 = c0[N + i];
        } else {
            const u64 *dsrc = digits + ct * ndigits * N;
            u64 s0 = c0[src], s1 = 0;
            if (ND) {
#pragma unroll
                for (int j = 0; j < KD; ++j) {
                    const u64 d = dsrc[(size_t)j * N + src];
                    const U64Pair r = mul_const_pair(d, kwb[j], d, kwa[j], q);      // each product is below 2q: at most 7q in all
                    s0 += r.a;
                    s1 += r.b;
                }
            } else {
                for (int j = 0; j < ndigits; ++j) {
                    const u64 d = dsrc[(size_t)j * N + src];
                    const ulonglong2 wb = key[(size_t)(2 * j) * N + i], wa = key[(size_t)(2 * j + 1) * N + i];
                    s0 = mul_const<false, true>(d, wb.x, wb.y, q, s0);
                    s1 = mul_const<false, true>(d, wa.x, wa.y, q, s1);
                }
            }
            v0 = reduce64(s0, T.mod);
            v1 = reduce64(s1, T.mod);
        }
        if (!live) v0 = v1 = 0;
        const u64 k80 = 0x8080808080808080ull;   // bytes of x + 0x80..80 are the balanced digits plus 128
        D0[t] = (v0 + k80) ^ k80;
        D1[t] = (v1 + k80) ^ k80;
    }
    // A thread holds the eight 16-byte chunks of its coefficient (128 contiguous bytes); stored straight from
    // the registers, every store instruction would touch 64 different lines with 16 bytes each.  The chunks go
    // through LDS instead (row = lane, padded to 144 bytes), so that instruction k of a wavefront writes the
    // 1 KiB of coefficients 8k..8k+7.
    __shared__ v4i_t tr[NT / 64][64][9];
    const int kb = eb >> 2, g = eb & 3;
    const int i_wave = blockIdx.x * 64;
#pragma unroll
    for (int poly = 0; poly < 2; ++poly) {
        const int col = 2 * b + poly, row = g * 16 + (col & 15);
#pragma unroll
        for (int limb = 0; limb < 8; ++limb) {
            v4i_t c;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                u32 wd = 0;
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    wd |= (u32)(((poly ? D1[4 * w + t] : D0[4 * w + t]) >> (8 * limb)) & 0xff) << (8 * t);
                c[w] = (int)wd;
            }
            tr[wave][lane][limb] = c;
        }
        __syncthreads();
        v4i_t *dst = xl + ((((size_t)(col >> 4) * kblocks + kb) * 64 + row) * N + i_wave) * 8;
        if (b_live)
#pragma unroll
            for (int k = 0; k < 8; ++k) dst[64 * k + lane] = tr[wave][8 * k + (lane >> 3)][lane & 7];
        __syncthreads();
    }
}


// ---- the client's two steps with the radix-8 transforms (one workgroup per ciphertext) ------------------------
// ct = (-a s + e + delta m, a) (Sec. II-C(1)), bit for bit the any-n kernel: m = the plaintext polynomial of the
// slots, a uniform, e Gaussian, all drawn from the ciphertext's seed by coefficient index.
__global__ __launch_bounds__(NT) void encrypt_2048(const u64 *slots, const u64 *seeds, const u64 *s_hat, u64 *ct_out,
                                                   Tables2048 T, Tables2048 Tp, const int *slot_to_idx, GaussCdf cdf,
                                                   int qbits, ulonglong2 delta) {
    __shared__ u64 bufA[LDS_WORDS], bufB[LDS_WORDS];
    const int tid = threadIdx.x;
    const u64 q = T.mod.q, p = Tp.mod.q, seed = seeds[blockIdx.x];
    const u64 *sl = slots + (size_t)blockIdx.x * N;
    u64 *c0 = ct_out + (size_t)blockIdx.x * 2 * N, *c1 = c0 + N;
    for (int s = tid; s < N; s += NT) {
        const u64 v = sl[s];
        bufB[slot_to_idx[s]] = v >= p ? v % p : v;
    }
    __syncthreads();
    u64 a[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) a[k] = bufB[8 * tid + k];
    inverse_in_regs(a, bufA, bufB, Tp, tid);          // m, coefficient tid + 256k, canonical mod p
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int e = draw_gauss_cdf(cdf, seed, kStreamCtE, (u64)(tid + k * NT));
        const u64 el = e >= 0 ? (u64)e : q - (u64)(-e);
        a[k] = csub_dev(el + csub_dev(mul_const(a[k], delta.x, delta.y, T.nq), q), q);
    }
    forward_to_lds(a, bufA, bufB, T, tid);            // (e + delta m) in the evaluation domain, in bufA
    u64 t0[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) t0[k] = reduce64(bufA[pad(tid + k * NT)], T.mod);
#pragma unroll
    for (int k = 0; k < PER; ++k) a[k] = draw_uniform(q, qbits, seed, kStreamCtA, (u64)(tid + k * NT));
    forward_to_lds(a, bufA, bufB, T, tid);            // its first barrier comes after every read of bufA above
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int i = tid + k * NT;
        const u64 ah = reduce64(bufA[pad(i)], T.mod);
        c1[i] = ah;
        c0[i] = sub_mod(t0[k], mul_mod(ah, s_hat[i], T.mod), q);
    }
}
// slots = decode(round(p (c0 + c1 s) / q) mod p); the rounded quotient through the exact division by q (q^-1 mod 2^64).
__global__ __launch_bounds__(NT) void decrypt_2048(const u64 *ct_in, const u64 *s_hat, u64 *slots, Tables2048 T,
                                                   Tables2048 Tp, const int *slot_to_idx, u64 q_inv64) {
    __shared__ u64 bufA[LDS_WORDS], bufB[LDS_WORDS];
    const int tid = threadIdx.x;
    const u64 q = T.mod.q, p = Tp.mod.q;
    const u64 *c0 = ct_in + (size_t)blockIdx.x * 2 * N, *c1 = c0 + N;
    u64 a[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int i = 8 * tid + k;
        a[k] = add_mod(c0[i], mul_mod(c1[i], s_hat[i], T.mod), q);
    }
    inverse_in_regs(a, bufA, bufB, T, tid);           // c0 + c1 s, coefficient tid + 256k, canonical
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const u128 t = (u128)p * a[k] + (q >> 1);
        const u64 r = reduce128(t, T.mod);
        const u64 quot = ((u64)t - r) * q_inv64;      // t - r is a multiple of q and the quotient is at most p
        a[k] = quot >= p ? quot - p : quot;
    }
    forward_to_lds(a, bufA, bufB, Tp, tid);           // the slots' values at their transform positions, in bufA
    u64 *out = slots + (size_t)blockIdx.x * N;
    for (int s = tid; s < N; s += NT) out[s] = reduce64(bufA[pad(slot_to_idx[s])], Tp.mod);
}

// ---- key switching with a special prime P -------------------------------------------------------------
// Keys hold four polynomials per digit ((b, a) modulo q, then modulo P).  Per rotation the digits are
// transformed in both moduli and multiplied into sums modulo q and modulo P; the sums modulo P go back to
// coefficients r in [0,P), and the rotation contributes (t_q - r) / P.  After the lift r -> r mod q everything is
// linear modulo q, so the lifted remainders of a workgroup's rotations are added in the coefficient domain
// (R0, R1) and transformed once at the end; terms that are not divided by P (the c0 part, rotations by zero)
// enter the sums multiplied by P.  Needs P < 2^60 and P < 2q.
struct SpecialJob {
    Tables2048 TP;          // transform tables of P
    ulonglong2 Pq, Pinv;    // P mod q and P^-1 mod q with companions
};

// IN8: the inputs lie in blocks of eight coefficients (PermJob::in8_S), as the matrix-core product leaves them.
template <bool HAS_W, bool IN8 = false>
__global__ __launch_bounds__(NT, 2) void perm_accumulate_special_2048(PermJob job, Tables2048 T, SpecialJob S, MaskJob mj,
                                                                      int gadget_bits, int ndigits) {
    __shared__ u64 bufA[LDS_WORDS], bufB[LDS_WORDS];
    __shared__ u64 stash[N];
    // Sums of the lifted remainders (coefficient domain modulo q, canonical, index tid + 256k): 15 of a thread's 16
    // words live in LDS slots of its own (no barrier), which is what two workgroups per CU leave room for.
    __shared__ u64 Rl[15 * NT];
    const int tid = threadIdx.x;
    if ((int)blockIdx.x >= job.items * job.nchunks) {   // only launched when mj.enabled
        mask_role(job, T, mj, (int)blockIdx.x - job.items * job.nchunks, bufA, bufB);
        return;
    }
    int item, chunk;
    item_and_chunk(job, item, chunk);
    int g0, g1;
    chunk_range(chunk, job.nchunks, job.G, g0, g1);
    const NegQ q = T.nq, qP = S.TP.nq;
    const u64 q8 = 8 * T.mod.q, P8 = 8 * S.TP.mod.q;
    const u64 digit_mask = (1ull << gadget_bits) - 1;
    const size_t key_pairs = (size_t)ndigits * 4 * N;

    u64 sum0[PER], sum1[PER];   // evaluation domain modulo q, below 8q between products
    u64 Rlast = 0;              // the sixteenth word of the remainder sums
#pragma unroll
    for (int k = 0; k < PER; ++k) sum0[k] = sum1[k] = 0;
#pragma unroll
    for (int s = 0; s < 15; ++s) Rl[s * NT + tid] = 0;

    for (int g = g0; g < g1; ++g) {
        const u64 *c0 = IN8 ? job.ct_in + (size_t)(item % job.in8_nout) * job.in8_o_stride + (size_t)(item / job.in8_nout) * 16 +
                                  (size_t)g * job.in_g_stride
                            : job.ct_in + (size_t)item * job.in_item_stride + (size_t)g * job.in_g_stride;
        const u64 *c1 = IN8 ? c0 + 8 : c0 + N;
        const size_t S8 = IN8 ? job.in8_S : 0;
        auto at = [&](const u64 *poly, int i) -> u64 { return IN8 ? poly[(size_t)(i >> 3) * S8 + (i & 7)] : poly[i]; };
        const ulonglong2 *w = HAS_W ? reinterpret_cast<const ulonglong2 *>(job.w2) + (size_t)g * N : nullptr;
        const int gal = job.gal[g];
        if (gal == 1) {   // rotation by zero: ScMult and Add only, times P
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                const int i = tid + k * NT;
                u64 x0 = at(c0, i), x1 = at(c1, i);
                if (HAS_W) {
                    const ulonglong2 ww = w[i];
                    x0 = mul_const<true>(x0, ww.x, ww.y, q);
                    x1 = mul_const<true>(x1, ww.x, ww.y, q);
                }
                sum0[k] = csub_dev(sum0[k] + mul_const<true>(x0, S.Pq.x, S.Pq.y, q), q8);
                sum1[k] = csub_dev(sum1[k] + mul_const<true>(x1, S.Pq.x, S.Pq.y, q), q8);
            }
            continue;
        }
        __syncthreads();   // the previous rotation ended reading bufA, this one starts by writing it
        const ulonglong2 *key = reinterpret_cast<const ulonglong2 *>(job.keys2) + (size_t)job.key_idx[g] * key_pairs;
        int src[PER];
#pragma unroll
        for (int k = 0; k < PER; ++k) src[k] = galois_index11(tid + k * NT, gal);
        u64 a[PER];
        {
            const ulonglong2 *c1v = reinterpret_cast<const ulonglong2 *>(IN8 ? c1 + (size_t)tid * S8 : c1 + 8 * tid);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const ulonglong2 cv = c1v[k];
                if (HAS_W) {
                    const ulonglong2 wa = w[8 * tid + 2 * k], wb = w[8 * tid + 2 * k + 1];
                    a[2 * k] = mul_const<true>(cv.x, wa.x, wa.y, q);
                    a[2 * k + 1] = mul_const<true>(cv.y, wb.x, wb.y, q);
                } else {
                    a[2 * k] = cv.x;
                    a[2 * k + 1] = cv.y;
                }
            }
        }
        inverse_in_regs<true>(a, bufA, bufB, T, tid);
#pragma unroll
        for (int k = 0; k < PER; ++k) stash[tid + k * NT] = a[k];
        // the c0 part, times P
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            u64 x = at(c0, src[k]);
            if (HAS_W) {
                const ulonglong2 ww = w[src[k]];
                x = mul_const<true>(x, ww.x, ww.y, q);
            }
            sum0[k] += mul_const<true>(x, S.Pq.x, S.Pq.y, q);
        }
        int pending = 1, pendingP = 0;
        u64 tp0[PER], tp1[PER];   // this rotation's sums modulo P, below 8P between products
#pragma unroll
        for (int k = 0; k < PER; ++k) tp0[k] = tp1[k] = 0;
        for (int j = 0; j < ndigits; ++j) {
#pragma unroll
            for (int k = 0; k < PER; ++k) a[k] = (stash[tid + k * NT] >> (j * gadget_bits)) & digit_mask;
            forward_to_lds<true>(a, bufA, bufB, T, tid);
            const ulonglong2 *kb = key + (size_t)(4 * j) * N, *ka = kb + N;
            if (pending == 4) {
#pragma unroll
                for (int k = 0; k < PER; ++k) {
                    sum0[k] = csub_dev(sum0[k], q8);
                    sum1[k] = csub_dev(sum1[k], q8);
                }
                pending = 0;
            }
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                const int i = tid + k * NT;
                const u64 d = bufA[pad(src[k])];
                const ulonglong2 b = kb[i], aa = ka[i];
                sum0[k] += mul_const<true>(d, b.x, b.y, q);
                sum1[k] += mul_const<true>(d, aa.x, aa.y, q);
            }
            ++pending;
            // the same digit modulo P
#pragma unroll
            for (int k = 0; k < PER; ++k) a[k] = (stash[tid + k * NT] >> (j * gadget_bits)) & digit_mask;
            forward_to_lds<true>(a, bufA, bufB, S.TP, tid);
            const ulonglong2 *kbP = kb + 2 * (size_t)N, *kaP = kbP + N;
            if (pendingP == 4) {
#pragma unroll
                for (int k = 0; k < PER; ++k) {
                    tp0[k] = csub_dev(tp0[k], P8);
                    tp1[k] = csub_dev(tp1[k], P8);
                }
                pendingP = 0;
            }
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                const int i = tid + k * NT;
                const u64 d = bufA[pad(src[k])];
                const ulonglong2 b = kbP[i], aa = kaP[i];
                tp0[k] += mul_const<true>(d, b.x, b.y, qP);
                tp1[k] += mul_const<true>(d, aa.x, aa.y, qP);
            }
            ++pendingP;
        }
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            sum0[k] = csub_dev(sum0[k], q8);
            sum1[k] = csub_dev(sum1[k], q8);
        }
        // remainders modulo P: canonical, to the ownership the inverse transform starts from (through bufB, which
        // nobody reads any more), back to coefficients in [0,P), reduced modulo q and added up
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int k = 0; k < PER; ++k) bufB[pad(tid + k * NT)] = reduce64(h ? tp1[k] : tp0[k], S.TP.mod);
            __syncthreads();
            {
                const u64 *pi = bufB + pad(tid << 3);
#pragma unroll
                for (int k = 0; k < PER; ++k) a[k] = pi[k];
            }
            inverse_in_regs<true>(a, bufA, bufB, S.TP, tid);
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                const u64 r = csub_dev(a[k], T.mod.q);
                if (h && k == PER - 1) {
                    Rlast = csub_dev(Rlast + r, T.mod.q);
                } else {
                    u64 *slot = Rl + (h * PER + k) * NT + tid;
                    *slot = csub_dev(*slot + r, T.mod.q);
                }
            }
        }
    }
    // partial = (sum - transform(R)) / P
    u64 *out = job.partial + ((size_t)item * job.slots + chunk) * 2 * N;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        u64 a[PER];
#pragma unroll
        for (int k = 0; k < PER; ++k) a[k] = (h && k == PER - 1) ? Rlast : Rl[(h * PER + k) * NT + tid];
        forward_to_lds<true>(a, bufA, bufB, T, tid);
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int i = tid + k * NT;
            const u64 x = reduce64(bufA[pad(i)], T.mod);
            const u64 t = reduce64(h ? sum1[k] : sum0[k], T.mod);
            const u64 dlt = t >= x ? t - x : t + T.mod.q - x;
            out[h * N + i] = csub_dev(mul_const<true>(dlt, S.Pinv.x, S.Pinv.y, q), T.mod.q);
        }
    }
}

// ---- hoisted input rotations with a special prime ----------------------------------------------------------
// DecPerm: one workgroup per (ciphertext, digit, modulus); digits[ct][j][modulus][i], lazy values of that modulus.
__global__ __launch_bounds__(NT) void decperm_special_2048(const u64 *ct_in, u64 *digits, Tables2048 T, Tables2048 TP,
                                                           int gadget_bits, int ndigits) {
    __shared__ u64 bufA[LDS_WORDS], bufB[LDS_WORDS];
    const int tid = threadIdx.x;
    const int m = blockIdx.x & 1, j = (blockIdx.x >> 1) % ndigits, ct = (blockIdx.x >> 1) / ndigits;
    const u64 *c1 = ct_in + (size_t)ct * 2 * N + N;
    u64 a[PER];
    const ulonglong2 *c1v = reinterpret_cast<const ulonglong2 *>(c1 + 8 * tid);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const ulonglong2 cv = c1v[k];
        a[2 * k] = cv.x;
        a[2 * k + 1] = cv.y;
    }
    inverse_in_regs(a, bufA, bufB, T, tid);
    const u64 digit_mask = (1ull << gadget_bits) - 1;
#pragma unroll
    for (int k = 0; k < PER; ++k) a[k] = (a[k] >> (j * gadget_bits)) & digit_mask;
    if (m) forward_to_lds(a, bufA, bufB, TP, tid);
    else forward_to_lds(a, bufA, bufB, T, tid);
    u64 *out = digits + (((size_t)ct * ndigits + j) * 2 + m) * N;
#pragma unroll
    for (int k = 0; k < PER; ++k) out[tid + k * NT] = bufA[pad(tid + k * NT)];
}

// HstPerm: one workgroup per (ciphertext, tap): inner products in both moduli from the stored digits, the sums
// modulo P back to coefficients, lifted, reduced modulo q and transformed forward again, then
// out = (P c0(X^g) + t_b - NTT(r_b)) / P, (t_a - NTT(r_a)) / P.  Output: xrot[ct][tap][c0|c1][i], canonical.
__global__ __launch_bounds__(NT) void hstperm_special_2048(const u64 *ct_in, const u64 *digits, TermList terms,
                                                           const u64 *keys2, u64 *xrot, Tables2048 T, SpecialJob S,
                                                           int ndigits) {
    __shared__ u64 bufA[LDS_WORDS], bufB[LDS_WORDS];
    const int tid = threadIdx.x;
    const int b = blockIdx.x / terms.nterm, e = blockIdx.x % terms.nterm;
    const size_t ct = (size_t)b * terms.nin + terms.ct[e];
    const u64 *c0 = ct_in + ct * 2 * N, *c1 = c0 + N;
    u64 *out = xrot + (size_t)blockIdx.x * 2 * N;
    const int gal = terms.gal[e];
    if (gal == 1) {
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int i = tid + k * NT;
            out[i] = c0[i];
            out[N + i] = c1[i];
        }
        return;
    }
    const NegQ q = T.nq, qP = S.TP.nq;
    const u64 *dsrc = digits + ct * ndigits * 2 * N;
    const ulonglong2 *key = reinterpret_cast<const ulonglong2 *>(keys2) + (size_t)terms.key[e] * ndigits * 4 * N;
    int src[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) src[k] = galois_index11(tid + k * NT, gal);
    // The two output polynomials one after the other (the digits are read twice, out of the L2): half the sums
    // are alive at a time, and the products are formed four coefficients at a time so that no more than their
    // operands are in flight - the kernel fits three workgroups per CU instead of one.
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        u64 sum[PER], tp[PER];      // modulo q and modulo P, below 8 moduli (at most three digits)
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            sum[k] = h ? 0 : mul_const(c0[src[k]], S.Pq.x, S.Pq.y, q);
            tp[k] = 0;
        }
        for (int j = 0; j < ndigits; ++j) {
            const ulonglong2 *kq = key + (size_t)(4 * j + h) * N, *kP = key + (size_t)(4 * j + 2 + h) * N;
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                const int i = tid + k * NT;
                const u64 dq = dsrc[(size_t)(2 * j) * N + src[k]], dP = dsrc[(size_t)(2 * j + 1) * N + src[k]];
                const ulonglong2 wq = kq[i], wP = kP[i];
                sum[k] += mul_const(dq, wq.x, wq.y, q);
                tp[k] += mul_const(dP, wP.x, wP.y, qP);
                if (k == 3) __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        u64 a[PER];
        // LDS phases: B (ownership change), A B A (inverse), B A B A (forward), then reads of A
#pragma unroll
        for (int k = 0; k < PER; ++k) bufB[pad(tid + k * NT)] = reduce64(tp[k], S.TP.mod);
        __syncthreads();
        {
            const u64 *pi = bufB + pad(tid << 3);
#pragma unroll
            for (int k = 0; k < PER; ++k) a[k] = pi[k];
        }
        inverse_in_regs(a, bufA, bufB, S.TP, tid);
#pragma unroll
        for (int k = 0; k < PER; ++k) a[k] = csub_dev(a[k], T.mod.q);
        forward_to_lds(a, bufA, bufB, T, tid);
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int i = tid + k * NT;
            const u64 x = reduce64(bufA[pad(i)], T.mod);
            const u64 t = reduce64(sum[k], T.mod);
            const u64 dlt = t >= x ? t - x : t + T.mod.q - x;
            out[h * N + i] = csub_dev(mul_const(dlt, S.Pinv.x, S.Pinv.y, q), T.mod.q);
        }
    }
}

// out[item] = sum over the first `used` partial ciphertexts of the item (mod q).  A workgroup owns 64 consecutive
// words; its SG wavefronts each add every SG-th partial (independent loads, several in flight) and the SG sums
// meet in LDS: with one input and a few hundred partials a single thread per word would wait for them one by one.
template <int SG>
__global__ __launch_bounds__(64 * SG) void sum_partials_kernel(const u64 *partial, int slots, int used, u64 *out, size_t words,
                                                               u64 q) {
    __shared__ u64 red[SG][64];
    const int lane = threadIdx.x & 63, sg = threadIdx.x >> 6;
    const size_t id = (size_t)blockIdx.x * 64 + lane;          // words is a multiple of 2N, so of 64
    const size_t item = id / (2 * N), e = id % (2 * N);
    const u64 *src = partial + item * slots * 2 * N + e;
    u64 acc = 0;
#pragma unroll 4
    for (int s = sg; s < used; s += SG) acc = add_mod(acc, src[(size_t)s * 2 * N], q);
    red[sg][lane] = acc;
    __syncthreads();
    if (sg) return;
#pragma unroll
    for (int g = 1; g < SG; ++g) acc = add_mod(acc, red[g][lane], q);
    out[id] = acc;
}

// the same with one thread per word, for a handful of partials
__global__ void sum_few_partials_kernel(const u64 *partial, int slots, int used, u64 *out, size_t words, u64 q) {
    const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= words) return;
    const size_t item = id / (2 * N), e = id % (2 * N);
    const u64 *src = partial + item * slots * 2 * N + e;
    u64 acc = 0;
    for (int s = 0; s < used; ++s) acc = add_mod(acc, src[(size_t)s * 2 * N], q);
    out[id] = acc;
}

}  // namespace

static Tables2048 make_tables(const gala_ctx *c, const u64 *blocks, const NttDev &dev) {
    Tables2048 T;
    // the level-major tables follow the two block tables (512 blocks of 8 pairs each)
    const ulonglong2 *levels = reinterpret_cast<const ulonglong2 *>(blocks) + 2 * 8 * (size_t)512;
    T.tw = levels;
    T.itw = levels + 7 * (1 + 4 + 8 + 32 + 64 + 256);
    T.ninv = make_ulonglong2(dev.ninv, dev.ninvs);
    T.itw1n = make_ulonglong2(dev.itw1n, dev.itw1ns);
    T.mod = dev.mod;
    const u64 neg = 0 - dev.mod.q;
    T.nq.lo = (u32)neg;
    T.nq.hi = (u32)(neg >> 32);
    (void)c;
    return T;
}

static int launch_2048(const gala_ctx *c, void *stream, const PermJob &job, const MaskJob &mj) {
    hipStream_t st = (hipStream_t)stream;
    const Tables2048 T = make_tables(c, c->d_tw2, c->dev_q);
    const dim3 grid((unsigned)(job.items * job.nchunks + (mj.enabled ? job.items : 0)));
    if (c->special) {
        if (job.in8_S && job.w) return (int)hipErrorInvalidValue;
        SpecialJob S;
        S.TP = make_tables(c, c->d_tw2P, c->dev_P);
        S.Pq = make_ulonglong2(c->Pq, c->Pq_s);
        S.Pinv = make_ulonglong2(c->Pinv, c->Pinv_s);
        if (job.w)
            hipLaunchKernelGGL(perm_accumulate_special_2048<true>, grid, dim3(NT), 0, st, job, T, S, mj, c->gadget_bits, c->ndigits);
        else if (job.in8_S)
            hipLaunchKernelGGL((perm_accumulate_special_2048<false, true>), grid, dim3(NT), 0, st, job, T, S, mj, c->gadget_bits,
                               c->ndigits);
        else
            hipLaunchKernelGGL(perm_accumulate_special_2048<false>, grid, dim3(NT), 0, st, job, T, S, mj, c->gadget_bits, c->ndigits);
        return (int)hipGetLastError();
    }
    if (job.in8_S && job.w) return (int)hipErrorInvalidValue;
    if (job.w)
        hipLaunchKernelGGL(perm_accumulate_2048<true>, grid, dim3(NT), 0, st, job, T, mj, c->gadget_bits, c->ndigits);
    else if (job.in8_S)
        hipLaunchKernelGGL((perm_accumulate_2048<false, true>), grid, dim3(NT), 0, st, job, T, mj, c->gadget_bits, c->ndigits);
    else
        hipLaunchKernelGGL(perm_accumulate_2048<false>, grid, dim3(NT), 0, st, job, T, mj, c->gadget_bits, c->ndigits);
    return (int)hipGetLastError();
}

int launch_perm_accumulate_2048(const gala_ctx *c, void *stream, const PermJob &job) {
    MaskJob mj{};
    mj.enabled = 0;
    return launch_2048(c, stream, job, mj);
}

int launch_perm_accumulate_2048_masked(const gala_ctx *c, void *stream, const PermJob &job, const FinalizeJob &fin) {
    MaskJob mj{};
    mj.enabled = 1;
    mj.nout = fin.nout;
    mj.r = fin.r;
    mj.r_stride = fin.r_stride;
    mj.mask_seed = fin.mask_seed;
    mj.layout = fin.mask;
    mj.slot_to_idx = c->d_slot_to_idx;
    mj.pbits = c->pbits;
    mj.delta = make_ulonglong2(c->delta, c->delta_s);
    mj.Tp = make_tables(c, c->d_tw2p, c->dev_p);
    hipStream_t st = (hipStream_t)stream;
    const bool timed = c->prof_which == 0 && (size_t)(2 * c->prof_used + 1) < c->prof_events.size();
    if (timed) (void)hipEventRecord((hipEvent_t)c->prof_events[2 * c->prof_used], st);
    int rc = launch_2048(c, stream, job, mj);
    if (timed) (void)hipEventRecord((hipEvent_t)c->prof_events[2 * c->prof_used++ + 1], st);
    if (rc) return rc;
    const size_t words = (size_t)job.items * 2 * N;
    // many partials of few items: more wavefronts per word
    if (job.nchunks + 1 <= 8)
        hipLaunchKernelGGL(sum_few_partials_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st, job.partial, job.slots,
                           job.nchunks + 1, fin.ct_out, words, c->q);
    else if (job.nchunks + 1 > 64 && words / 64 < 2048)
        hipLaunchKernelGGL(sum_partials_kernel<16>, dim3((unsigned)(words / 64)), dim3(1024), 0, st, job.partial, job.slots,
                           job.nchunks + 1, fin.ct_out, words, c->q);
    else
        hipLaunchKernelGGL(sum_partials_kernel<4>, dim3((unsigned)(words / 64)), dim3(256), 0, st, job.partial, job.slots,
                           job.nchunks + 1, fin.ct_out, words, c->q);
    return (int)hipGetLastError();
}

bool uses_fast_hoist(const gala_ctx *c) { return uses_fast_perm(c) && c->ndigits <= HOIST_DIGITS; }
int launch_hoist_taps_2048(const gala_ctx *c, void *stream, const u64 *ct_in, int batch, const TermList &terms,
                           bool any_rotation, const u64 *keys2, u64 *digits, u64 *xrot) {
    if (batch <= 0 || terms.nterm <= 0) return 0;
    const size_t count = (size_t)batch * terms.nin;
    const Tables2048 T = make_tables(c, c->d_tw2, c->dev_q);
    hipStream_t st = (hipStream_t)stream;
    const dim3 per_term((unsigned)((size_t)batch * terms.nterm));
    if (c->special) {     // digits[ct][j][modulus][N]: twice the digit storage of the one-prime form
        SpecialJob S;
        S.TP = make_tables(c, c->d_tw2P, c->dev_P);
        S.Pq = make_ulonglong2(c->Pq, c->Pq_s);
        S.Pinv = make_ulonglong2(c->Pinv, c->Pinv_s);
        if (any_rotation) {
            hipLaunchKernelGGL(decperm_special_2048, dim3((unsigned)(count * c->ndigits * 2)), dim3(NT), 0, st, ct_in, digits,
                               T, S.TP, c->gadget_bits, c->ndigits);
            const int rc = (int)hipGetLastError();
            if (rc) return rc;
        }
        hipLaunchKernelGGL(hstperm_special_2048, per_term, dim3(NT), 0, st, ct_in, digits, terms, keys2, xrot, T, S, c->ndigits);
        return (int)hipGetLastError();
    }
    if (any_rotation) {
        hipLaunchKernelGGL(decperm_2048, dim3((unsigned)(count * c->ndigits)), dim3(NT), 0, st, ct_in, digits, T,
                           c->gadget_bits, c->ndigits);
        const int rc = (int)hipGetLastError();
        if (rc) return rc;
    }
    hipLaunchKernelGGL(hstperm_taps_2048, per_term, dim3(NT), 0, st, ct_in, digits, terms, keys2, xrot, T, c->ndigits);
    return (int)hipGetLastError();
}

// DecPerm (when any term rotates) followed by the HstPerm of every term, written as the column image
int launch_hstperm_pack_2048(const gala_ctx *c, void *stream, const u64 *ct_in, u64 *digits, int batch,
                             const TermList &terms, bool any_rotation, const u64 *keys2, u64 *xl) {
    if (batch <= 0 || terms.nterm <= 0) return 0;
    const Tables2048 T = make_tables(c, c->d_tw2, c->dev_q);
    hipStream_t st = (hipStream_t)stream;
    if (any_rotation) {
        hipLaunchKernelGGL(decperm_2048, dim3((unsigned)((size_t)batch * terms.nin * c->ndigits)), dim3(NT), 0, st, ct_in,
                           digits, T, c->gadget_bits, c->ndigits);
        const int rc = (int)hipGetLastError();
        if (rc) return rc;
    }
    const int eblocks = (terms.nterm + 15) / 16, kblocks = (terms.nterm + 63) / 64;
    const dim3 grid(N / 64, (unsigned)eblocks, (unsigned)((batch + 3) / 4));
    v4i_t *out = reinterpret_cast<v4i_t *>(xl);
    if (!any_rotation)
        hipLaunchKernelGGL((hstperm_pack_2048<0, false>), grid, dim3(NT), 0, st, ct_in, digits, terms, kblocks, keys2, out, T, c->ndigits, batch);
    else if (!keys2)
        return (int)hipErrorInvalidValue;
    else if (c->ndigits == 3)
        hipLaunchKernelGGL((hstperm_pack_2048<3, true>), grid, dim3(NT), 0, st, ct_in, digits, terms, kblocks, keys2, out, T, c->ndigits, batch);
    else
        hipLaunchKernelGGL((hstperm_pack_2048<0, true>), grid, dim3(NT), 0, st, ct_in, digits, terms, kblocks, keys2, out, T, c->ndigits, batch);
    return (int)hipGetLastError();
}

int launch_encrypt_2048(const gala_ctx *c, void *stream, const u64 *s_hat, const u64 *slots, const u64 *seeds, int count,
                        u64 *ct_out) {
    if (!count) return 0;
    GaussCdf cdf;
    for (int i = 0; i < 2 * kGaussBound; ++i) cdf.t[i] = gauss_cdf_table()[i];
    hipLaunchKernelGGL(encrypt_2048, dim3((unsigned)count), dim3(NT), 0, (hipStream_t)stream, slots, seeds, s_hat, ct_out,
                       make_tables(c, c->d_tw2, c->dev_q), make_tables(c, c->d_tw2p, c->dev_p), c->d_slot_to_idx, cdf, c->qbits,
                       make_ulonglong2(c->delta, c->delta_s));
    return (int)hipGetLastError();
}
int launch_decrypt_2048(const gala_ctx *c, void *stream, const u64 *s_hat, const u64 *ct_in, int count, u64 *slots) {
    if (!count) return 0;
    u64 inv = c->q;                                   // Newton's iteration for q^-1 mod 2^64 (q is odd)
    for (int i = 0; i < 6; ++i) inv *= 2 - c->q * inv;
    hipLaunchKernelGGL(decrypt_2048, dim3((unsigned)count), dim3(NT), 0, (hipStream_t)stream, ct_in, s_hat, slots,
                       make_tables(c, c->d_tw2, c->dev_q), make_tables(c, c->d_tw2p, c->dev_p), c->d_slot_to_idx, inv);
    return (int)hipGetLastError();
}

}  // namespace gala
