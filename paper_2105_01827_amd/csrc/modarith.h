// 64-bit modular arithmetic shared by the host and device halves of the library.
// Moduli are below 2^61 so that four times the modulus still fits a word
// ("lazy" residues in [0,4q) between butterflies).
#pragma once
#include <cstdint>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define GALA_HD __host__ __device__ __forceinline__
#else
#define GALA_HD inline
#endif

namespace gala {

using u32 = uint32_t;
using u64 = uint64_t;
using i64 = int64_t;
using u128 = unsigned __int128;

GALA_HD u64 mulhi64(u64 a, u64 b) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __umul64hi(a, b);
#else
    return (u64)(((u128)a * b) >> 64);
#endif
}

// a - q if a >= q (brings [0,2q) to [0,q))
GALA_HD u64 csub(u64 a, u64 q) { return a >= q ? a - q : a; }

// Multiplication by a constant w with companion ws = floor(w * 2^64 / q):
// returns a*w mod q up to one extra q, i.e. a value in [0,2q), for ANY 64-bit a.
GALA_HD u64 mul_shoup_lazy(u64 a, u64 w, u64 ws, u64 q) { return a * w - mulhi64(a, ws) * q; }
GALA_HD u64 mul_shoup(u64 a, u64 w, u64 ws, u64 q) { return csub(mul_shoup_lazy(a, w, ws, q), q); }

// What a kernel needs to know about a modulus (passed by value).
struct Modulus {
    u64 q;       // the modulus
    u64 q2;      // 2q
    u64 c64;     // 2^64 mod q
    u64 c64s;    // Shoup companion of c64
    u64 one_s;   // floor(2^64 / q): Shoup companion of the constant 1
};

// (hi*2^64 + lo) mod q for any 128-bit value, canonical result.
// hi*2^64 = hi * c64 (mod q); lo is reduced with the companion of 1.
GALA_HD u64 reduce128(u64 hi, u64 lo, const Modulus &m) {
    u64 a = mul_shoup_lazy(hi, m.c64, m.c64s, m.q);        // [0,2q)
    u64 b = lo - mulhi64(lo, m.one_s) * m.q;               // [0,2q)
    return csub(csub(a + b, m.q2), m.q);
}
GALA_HD u64 reduce128(u128 v, const Modulus &m) { return reduce128((u64)(v >> 64), (u64)v, m); }

// generic product of two residues
GALA_HD u64 mul_mod(u64 a, u64 b, const Modulus &m) { return reduce128((u128)a * b, m); }

GALA_HD u64 add_mod(u64 a, u64 b, u64 q) { return csub(a + b, q); }
GALA_HD u64 sub_mod(u64 a, u64 b, u64 q) { return a >= b ? a - b : a + q - b; }

// Forward (decimation-in-time) butterfly on lazy residues: x,y in [0,4q) -> [0,4q).
GALA_HD void butterfly_fwd(u64 &x, u64 &y, u64 w, u64 ws, u64 q, u64 q2) {
    u64 u = csub(x, q2);
    u64 t = mul_shoup_lazy(y, w, ws, q);
    x = u + t;
    y = u - t + q2;
}
// Inverse (decimation-in-frequency) butterfly: x,y in [0,2q) -> [0,2q).
GALA_HD void butterfly_inv(u64 &x, u64 &y, u64 w, u64 ws, u64 q, u64 q2) {
    u64 s = x + y;
    u64 d = x - y + q2;
    x = csub(s, q2);
    y = mul_shoup_lazy(d, w, ws, q);
}

// ---- counter-based generator used by every seeded sampler -----------------
GALA_HD u64 mix64(u64 z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
GALA_HD u64 rand64(u64 seed, u64 stream, u64 idx, u64 attempt) {
    u64 h = mix64(seed + 0x9E3779B97F4A7C15ull);
    h = mix64(h + stream);
    h = mix64(h + idx);
    return mix64(h + attempt);
}
enum : u64 { kStreamSk = 1, kStreamKskA = 2, kStreamKskE = 3, kStreamCtA = 4, kStreamCtE = 5, kStreamMask = 6,
             kStreamKskAP = 7 };

// uniform in [0,m): the top `bits` = bitlen(m) bits of a draw, redrawn while >= m
GALA_HD u64 draw_uniform(u64 m, int bits, u64 seed, u64 stream, u64 idx) {
    for (u64 t = 0;; ++t) {
        u64 v = rand64(seed, stream, idx, t) >> (64 - bits);
        if (v < m) return v;
    }
}

}  // namespace gala
