/*
 * GALA CPU oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, single-purpose C implementation of the server-side packed-HE
 * linear layers of GALA (arXiv 2105.01827): Add / ScMult / Perm (Sec. II-C(1)),
 * the row-encoding-share-RaS matrix-vector product (Sec. III-A(3)) and the
 * kernel-grouping convolution (Sec. III-B(3)).  Only tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it.  It shares no code with the HIP
 * library: every helper below is written here and used only here.
 *
 * Style: ciphertext polynomials always live in the COEFFICIENT domain, natural
 * order, canonical residues in [0,q).  The only "fast" primitive is the
 * evaluation/interpolation of a polynomial at the odd powers of a 2n-th root of
 * unity (a textbook twisted radix-2 FFT), used to multiply in Z_m[X]/(X^n+1);
 * it is pinned by tests against its O(n^2) definition and against schoolbook
 * negacyclic multiplication.  All modular products are (unsigned __int128) % m.
 *
 * Parity status: everything here is pinned by tests/test_oracle_*.py except the
 * seeded samplers (counter-based generator, ternary / uniform / discrete
 * Gaussian), which the paper does not define: their statistics and the Gaussian
 * threshold table are checked against the mathematics, but the exact bit
 * recipe is this build's own ("parity unpinned" by the paper).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef uint64_t u64;
typedef int64_t i64;
typedef unsigned __int128 u128;

/* ------------------------------------------------------------------ */
/* modular arithmetic, any modulus m < 2^63                            */
/* ------------------------------------------------------------------ */
static u64 addm(u64 a, u64 b, u64 m) { u64 s = a + b; return s >= m ? s - m : s; }
static u64 subm(u64 a, u64 b, u64 m) { return a >= b ? a - b : a + m - b; }
static u64 mulm(u64 a, u64 b, u64 m) { return (u64)(((u128)a * b) % m); }
static u64 powm(u64 b, u64 e, u64 m) {
    u64 r = 1 % m; b %= m;
    while (e) { if (e & 1) r = mulm(r, b, m); b = mulm(b, b, m); e >>= 1; }
    return r;
}
static u64 invm(u64 a, u64 m) { return powm(a, m - 2, m); } /* m prime */

/* ------------------------------------------------------------------ */
/* context                                                             */
/* ------------------------------------------------------------------ */
typedef struct {
    int n, logn;
    u64 q, p;
    int gadget_bits, ndigits;
    u64 delta;      /* floor(q/p); equals (q-1)/p when q = 1 mod p               */
    u64 psi;        /* a primitive 2n-th root of unity mod q (any one will do)    */
    u64 zeta;       /* the SMALLEST primitive 2n-th root of unity mod p (pinned)  */
    u64 *psi_pow;   /* psi^i,  i in [0,2n)                                        */
    u64 *zeta_pow;  /* zeta^i, i in [0,2n)                                        */
    u64 ninv_q, ninv_p;
    int *slot_exp;  /* slot s=(h,k) -> odd exponent e with value = m(zeta^e)      */
    /* optional special prime P for key switching (0 = keys live mod q only)       */
    u64 P;          /* prime, P = 1 mod 2n, P != q                                */
    u64 *psiP_pow;  /* powers of a primitive 2n-th root mod P                     */
    u64 ninv_P, Pinv_q, P_mod_q;
} orc_ctx;

static int ilog2(u64 v) { int l = 0; while ((1ull << l) < v) l++; return l; }
static int bitlen(u64 v) { int l = 0; while (v) { l++; v >>= 1; } return l; }

/* first primitive 2n-th root found by trying x = 2,3,4,...: c = x^((m-1)/2n) is
 * primitive iff c^n = -1. */
static u64 some_primitive_root(u64 m, int n) {
    for (u64 x = 2; x < m; x++) {
        u64 c = powm(x, (m - 1) / (2 * (u64)n), m);
        if (powm(c, (u64)n, m) == m - 1) return c;
    }
    return 0;
}
/* the primitive 2n-th roots are exactly c^e for odd e; take the least one */
static u64 smallest_primitive_root(u64 m, int n) {
    u64 c = some_primitive_root(m, n), c2 = mulm(c, c, m), best = c, cur = c;
    for (int e = 3; e < 2 * n; e += 2) { cur = mulm(cur, c2, m); if (cur < best) best = cur; }
    return best;
}

orc_ctx *orc_ctx_new(int n, u64 q, u64 p, int gadget_bits) {
    if (n < 4 || (n & (n - 1)) || q >> 62 || p >= q || gadget_bits < 1 || gadget_bits > 62) return NULL;
    if ((q - 1) % (2 * (u64)n) || (p - 1) % (2 * (u64)n)) return NULL;
    orc_ctx *c = calloc(1, sizeof *c);
    c->n = n; c->logn = ilog2(n); c->q = q; c->p = p;
    c->gadget_bits = gadget_bits;
    c->ndigits = (bitlen(q - 1) + gadget_bits - 1) / gadget_bits;
    c->delta = q / p;
    c->psi = some_primitive_root(q, n);
    c->zeta = smallest_primitive_root(p, n);
    c->psi_pow = malloc(sizeof(u64) * 2 * n);
    c->zeta_pow = malloc(sizeof(u64) * 2 * n);
    c->psi_pow[0] = 1; c->zeta_pow[0] = 1;
    for (int i = 1; i < 2 * n; i++) {
        c->psi_pow[i] = mulm(c->psi_pow[i - 1], c->psi, q);
        c->zeta_pow[i] = mulm(c->zeta_pow[i - 1], c->zeta, p);
    }
    c->ninv_q = invm(n, q); c->ninv_p = invm(n, p);
    /* slot (h,k): exponent 3^k for the first row, -3^k for the second (mod 2n) */
    c->slot_exp = malloc(sizeof(int) * n);
    int e = 1;
    for (int k = 0; k < n / 2; k++) {
        c->slot_exp[k] = e;
        c->slot_exp[n / 2 + k] = 2 * n - e;
        e = (int)(((long)e * 3) % (2 * n));
    }
    return c;
}
void orc_ctx_free(orc_ctx *c) {
    if (!c) return;
    free(c->psi_pow); free(c->zeta_pow); free(c->slot_exp); free(c->psiP_pow); free(c);
}
/* Switch key switching to the special-prime form: keys are generated modulo q*P with the
 * secret scaled by P, and every key switch ends with an exact division by P (see below). */
int orc_ctx_set_special(orc_ctx *c, u64 P) {
    if (!P || P == c->q || P >> 62 || (P - 1) % (2 * (u64)c->n)) return -1;
    c->P = P;
    u64 r = some_primitive_root(P, c->n);
    free(c->psiP_pow);
    c->psiP_pow = malloc(sizeof(u64) * 2 * c->n);
    c->psiP_pow[0] = 1;
    for (int i = 1; i < 2 * c->n; i++) c->psiP_pow[i] = mulm(c->psiP_pow[i - 1], r, P);
    c->ninv_P = invm(c->n, P);
    c->P_mod_q = P % c->q;
    c->Pinv_q = invm(c->P_mod_q, c->q);
    return 0;
}
/* polynomials per key digit: (b, a) mod q, and with a special prime also (b, a) mod P */
int orc_key_polys(const orc_ctx *c) { return c->P ? 4 : 2; }
int orc_ndigits(const orc_ctx *c) { return c->ndigits; }
u64 orc_delta(const orc_ctx *c) { return c->delta; }
u64 orc_zeta(const orc_ctx *c) { return c->zeta; }
u64 orc_psi(const orc_ctx *c) { return c->psi; }

/* ------------------------------------------------------------------ */
/* evaluation at the odd powers of a 2n-th root  (the only fast part)  */
/*   ev[k] = sum_i a[i] * root^{(2k+1) i}  (mod m),  k in [0,n)        */
/* ------------------------------------------------------------------ */
/* O(n^2) definition; rpow[i] = root^i, i in [0,2n) */
static void eval_odd_slow(const u64 *a, u64 *ev, int n, u64 m, const u64 *rpow) {
    for (int k = 0; k < n; k++) {
        u64 s = 0;
        for (int i = 0; i < n; i++)
            s = addm(s, mulm(a[i] % m, rpow[((long)(2 * k + 1) * i) % (2 * n)], m), m);
        ev[k] = s;
    }
}
static void interp_odd_slow(const u64 *ev, u64 *a, int n, u64 m, const u64 *rpow, u64 ninv) {
    /* a[i] = n^-1 * sum_k ev[k] * root^{-(2k+1) i} */
    for (int i = 0; i < n; i++) {
        u64 s = 0;
        for (int k = 0; k < n; k++) {
            long e = ((long)(2 * k + 1) * i) % (2 * n);
            s = addm(s, mulm(ev[k] % m, rpow[(2 * n - e) % (2 * n)], m), m);
        }
        a[i] = mulm(s, ninv, m);
    }
}
/* in-place cyclic radix-2 DFT of size n with omega = root^2 (sign=+1) or its
 * inverse (sign=-1): x[k] <- sum_i x[i] * omega^{ik} */
static void cyclic_dft(u64 *x, int n, u64 m, const u64 *rpow, int sign) {
    int logn = ilog2(n);
    for (int i = 0; i < n; i++) {           /* bit-reversal reordering */
        int r = 0;
        for (int b = 0; b < logn; b++) if (i >> b & 1) r |= 1 << (logn - 1 - b);
        if (r > i) { u64 t = x[i]; x[i] = x[r]; x[r] = t; }
    }
    for (int len = 2; len <= n; len <<= 1) {
        int half = len / 2, step = 2 * n / len;   /* omega_len^j = root^{j*step} */
        for (int s = 0; s < n; s += len)
            for (int j = 0; j < half; j++) {
                int e = (j * step) % (2 * n);
                u64 w = rpow[sign > 0 ? e : (2 * n - e) % (2 * n)];
                u64 u = x[s + j], v = mulm(x[s + j + half], w, m);
                x[s + j] = addm(u, v, m);
                x[s + j + half] = subm(u, v, m);
            }
    }
}
static void eval_odd(const u64 *a, u64 *ev, int n, u64 m, const u64 *rpow) {
    u64 *x = malloc(sizeof(u64) * n);
    for (int i = 0; i < n; i++) x[i] = mulm(a[i] % m, rpow[i], m);   /* twist by root^i */
    cyclic_dft(x, n, m, rpow, +1);
    memcpy(ev, x, sizeof(u64) * n);
    free(x);
}
static void interp_odd(const u64 *ev, u64 *a, int n, u64 m, const u64 *rpow, u64 ninv) {
    u64 *x = malloc(sizeof(u64) * n);
    for (int i = 0; i < n; i++) x[i] = ev[i] % m;
    cyclic_dft(x, n, m, rpow, -1);
    for (int i = 0; i < n; i++)                                       /* untwist, scale */
        a[i] = mulm(mulm(x[i], ninv, m), rpow[(2 * n - i) % (2 * n)], m);
    free(x);
}
/* exported for the pins */
void orc_eval_q(const orc_ctx *c, const u64 *a, u64 *ev, int slow) {
    if (slow) eval_odd_slow(a, ev, c->n, c->q, c->psi_pow); else eval_odd(a, ev, c->n, c->q, c->psi_pow);
}
void orc_interp_q(const orc_ctx *c, const u64 *ev, u64 *a, int slow) {
    if (slow) interp_odd_slow(ev, a, c->n, c->q, c->psi_pow, c->ninv_q);
    else interp_odd(ev, a, c->n, c->q, c->psi_pow, c->ninv_q);
}

/* ------------------------------------------------------------------ */
/* ring product in Z_q[X]/(X^n+1)                                      */
/* ------------------------------------------------------------------ */
void orc_polymul_schoolbook(const orc_ctx *c, const u64 *a, const u64 *b, u64 *out) {
    int n = c->n; u64 q = c->q;
    u64 *r = calloc(n, sizeof(u64));
    for (int i = 0; i < n; i++)
        for (int j = 0; j < n; j++) {
            u64 t = mulm(a[i], b[j], q);
            int k = i + j;
            if (k < n) r[k] = addm(r[k], t, q); else r[k - n] = subm(r[k - n], t, q);  /* X^n = -1 */
        }
    memcpy(out, r, sizeof(u64) * n); free(r);
}
/* product in Z_m[X]/(X^n+1) through evaluation at the odd powers of a 2n-th root mod m */
static void polymul_mod(int n, u64 m, const u64 *rpow, u64 ninv, const u64 *a, const u64 *b, u64 *out) {
    u64 *ea = malloc(sizeof(u64) * n), *eb = malloc(sizeof(u64) * n);
    eval_odd(a, ea, n, m, rpow);
    eval_odd(b, eb, n, m, rpow);
    for (int i = 0; i < n; i++) ea[i] = mulm(ea[i], eb[i], m);
    interp_odd(ea, out, n, m, rpow, ninv);
    free(ea); free(eb);
}
void orc_polymul(const orc_ctx *c, const u64 *a, const u64 *b, u64 *out) {
    polymul_mod(c->n, c->q, c->psi_pow, c->ninv_q, a, b, out);
}
/* the same product modulo the special prime (exported for the pins) */
void orc_polymul_special(const orc_ctx *c, const u64 *a, const u64 *b, u64 *out) {
    polymul_mod(c->n, c->P, c->psiP_pow, c->ninv_P, a, b, out);
}

/* ------------------------------------------------------------------ */
/* SIMD slot encoding mod p  (Sec. II-C(1): n slots per plaintext)      */
/*   slot s=(h,k), h in {0,1}, k in [0,n/2):  value = m(zeta^{+-3^k})    */
/* ------------------------------------------------------------------ */
void orc_decode(const orc_ctx *c, const u64 *poly_p, u64 *slots, int slow) {
    int n = c->n;
    u64 *ev = malloc(sizeof(u64) * n);
    if (slow) eval_odd_slow(poly_p, ev, n, c->p, c->zeta_pow); else eval_odd(poly_p, ev, n, c->p, c->zeta_pow);
    for (int s = 0; s < n; s++) slots[s] = ev[(c->slot_exp[s] - 1) / 2];
    free(ev);
}
void orc_encode(const orc_ctx *c, const u64 *slots, u64 *poly_p, int slow) {
    int n = c->n;
    u64 *ev = malloc(sizeof(u64) * n);
    for (int s = 0; s < n; s++) ev[(c->slot_exp[s] - 1) / 2] = slots[s] % c->p;
    if (slow) interp_odd_slow(ev, poly_p, n, c->p, c->zeta_pow, c->ninv_p);
    else interp_odd(ev, poly_p, n, c->p, c->zeta_pow, c->ninv_p);
    free(ev);
}
/* plaintext operand of ScMult: coefficients lifted to (-p/2, p/2] then mod q */
static void lift_centred(const orc_ctx *c, const u64 *poly_p, u64 *poly_q) {
    for (int i = 0; i < c->n; i++) {
        u64 v = poly_p[i];
        poly_q[i] = (v > c->p / 2) ? c->q - (c->p - v) : v;
    }
}
void orc_encode_weight(const orc_ctx *c, const u64 *slots, u64 *poly_q) {
    u64 *t = malloc(sizeof(u64) * c->n);
    orc_encode(c, slots, t, 0);
    lift_centred(c, t, poly_q);
    free(t);
}

/* ------------------------------------------------------------------ */
/* seeded samplers (this build's own recipe; both sides implement it)   */
/* ------------------------------------------------------------------ */
enum { STREAM_SK = 1, STREAM_KSK_A = 2, STREAM_KSK_E = 3, STREAM_CT_A = 4, STREAM_CT_E = 5, STREAM_MASK = 6,
       STREAM_KSK_AP = 7 };

static u64 mix64(u64 z) {   /* SplitMix64 output function */
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
u64 orc_mix64(u64 z) { return mix64(z); }
u64 orc_rand64(u64 seed, u64 stream, u64 idx, u64 attempt) {
    u64 h = mix64(seed + 0x9E3779B97F4A7C15ull);
    h = mix64(h + stream);
    h = mix64(h + idx);
    return mix64(h + attempt);
}
/* uniform in [0,m): top bitlen(m) bits, rejected while >= m */
u64 orc_uniform(u64 m, u64 seed, u64 stream, u64 idx) {
    int bits = bitlen(m);
    for (u64 t = 0;; t++) {
        u64 v = orc_rand64(seed, stream, idx, t) >> (64 - bits);
        if (v < m) return v;
    }
}
/* uniform on {-1,0,1}: top two bits, value 3 rejected */
int orc_ternary(u64 seed, u64 stream, u64 idx) {
    for (u64 t = 0;; t++) {
        u64 v = orc_rand64(seed, stream, idx, t) >> 62;
        if (v < 3) return (int)v - 1;
    }
}
/* discrete Gaussian, sigma = 3.2, support [-19,19]:
 * GAUSS_CDF[i] = floor(2^64 * P[X <= -19+i]); sample = -19 + #{i : u >= GAUSS_CDF[i]} */
static const u64 GAUSS_CDF[38] = {
    0xbd798c7acull, 0x53f5e234f7ull, 0x1e24b89625aull, 0x9adbc7900e1ull, 0x2d17ca1e3a82ull,
    0xbf05ff772ee2ull, 0x2e06843bbf95dull, 0xa19062dceb033ull, 0x204c0ded173b17ull,
    0x5e3163ffc656a8ull, 0xfab6a7e614dfaeull, 0x261b16e99bc14f8ull, 0x54c69348bbc9867ull,
    0xacd276539458231ull, 0x143796b3c337f00bull, 0x22d43df09de40e7aull, 0x37651d96aa4fb429ull,
    0x51a5da2b40f1bff1ull, 0x700ad4bf5a6e80e2ull, 0x8ff52b40a5917f1dull, 0xae5a25d4bf0e400eull,
    0xc89ae26955b04bd6ull, 0xdd2bc20f621bf185ull, 0xebc8694c3cc80ff4ull, 0xf532d89ac6ba7dceull,
    0xfab396cb74436798ull, 0xfd9e4e916643eb07ull, 0xff05495819eb2051ull, 0xffa1ce9c0039a957ull,
    0xffdfb3f212e8c4e8ull, 0xfff5e6f9d2314fccull, 0xfffd1f97bc4406a2ull, 0xffff40fa0088d11dull,
    0xffffd2e835e1c57dull, 0xfffff6524386ff1eull, 0xfffffe1db4769da5ull, 0xffffffac0a1dcb08ull,
    0xfffffff428673853ull };
const u64 *orc_gauss_cdf(void) { return GAUSS_CDF; }
int orc_gauss(u64 seed, u64 stream, u64 idx) {
    u64 u = orc_rand64(seed, stream, idx, 0);
    int x = -19;
    for (int i = 0; i < 38; i++) if (u >= GAUSS_CDF[i]) x++;
    return x;
}
static u64 signed_to_mod(int v, u64 q) { return v >= 0 ? (u64)v : q - (u64)(-v); }

/* ------------------------------------------------------------------ */
/* keys, encryption, decryption (client side; Sec. II-C(1))             */
/* ------------------------------------------------------------------ */
/* ternary secret as residues mod q */
void orc_keygen(const orc_ctx *c, u64 seed, u64 *s) {
    for (int i = 0; i < c->n; i++) s[i] = signed_to_mod(orc_ternary(seed, STREAM_SK, i), c->q);
}
/* symmetric-key encryption of a slot vector: ct = (c0, c1) = (-a s + e + delta*m, a) */
void orc_encrypt(const orc_ctx *c, const u64 *s, const u64 *slots, u64 seed, u64 *ct) {
    int n = c->n; u64 q = c->q;
    u64 *m = malloc(sizeof(u64) * n), *as = malloc(sizeof(u64) * n);
    u64 *c0 = ct, *c1 = ct + n;
    orc_encode(c, slots, m, 0);
    for (int i = 0; i < n; i++) c1[i] = orc_uniform(q, seed, STREAM_CT_A, i);
    orc_polymul(c, c1, s, as);
    for (int i = 0; i < n; i++) {
        u64 e = signed_to_mod(orc_gauss(seed, STREAM_CT_E, i), q);
        c0[i] = addm(subm(e, as[i], q), mulm(c->delta, m[i], q), q);
    }
    free(m); free(as);
}
/* v = c0 + c1 s; m = round(p v / q) mod p, all in integers */
static void decrypt_poly(const orc_ctx *c, const u64 *s, const u64 *ct, u64 *m, u64 *v_out) {
    int n = c->n; u64 q = c->q, p = c->p;
    u64 *v = malloc(sizeof(u64) * n);
    orc_polymul(c, ct + n, s, v);
    for (int i = 0; i < n; i++) {
        v[i] = addm(v[i], ct[i], q);
        u128 t = (u128)p * v[i] + q / 2;
        m[i] = (u64)(t / q) % p;
    }
    if (v_out) memcpy(v_out, v, sizeof(u64) * n);
    free(v);
}
void orc_decrypt(const orc_ctx *c, const u64 *s, const u64 *ct, u64 *slots) {
    u64 *m = malloc(sizeof(u64) * c->n);
    decrypt_poly(c, s, ct, m, NULL);
    orc_decode(c, m, slots, 0);
    free(m);
}
/* infinity norm of (c0 + c1 s - delta*m) centred, for m = encode(expected slots) */
u64 orc_noise(const orc_ctx *c, const u64 *s, const u64 *ct, const u64 *expected_slots) {
    int n = c->n; u64 q = c->q;
    u64 *m = malloc(sizeof(u64) * n), *v = malloc(sizeof(u64) * n), *junk = malloc(sizeof(u64) * n);
    orc_encode(c, expected_slots, m, 0);
    decrypt_poly(c, s, ct, junk, v);
    u64 worst = 0;
    for (int i = 0; i < n; i++) {
        u64 d = subm(v[i], mulm(c->delta, m[i], q), q);
        if (d > q / 2) d = q - d;
        if (d > worst) worst = d;
    }
    free(m); free(v); free(junk);
    return worst;
}

/* ------------------------------------------------------------------ */
/* Galois automorphisms and key switching  (Perm = DecPerm + HstPerm)   */
/* ------------------------------------------------------------------ */
/* rotation "left by step in both rows, rows swapped if swap": X -> X^g with
 * g = (+-) 3^step mod 2n */
int orc_galois_elt(const orc_ctx *c, int swap, int step) {
    int two_n = 2 * c->n, g = 1;
    step %= c->n / 2; if (step < 0) step += c->n / 2;
    for (int i = 0; i < step; i++) g = (int)(((long)g * 3) % two_n);
    return swap ? two_n - g : g;
}
/* a(X) -> a(X^g) in Z_q[X]/(X^n+1): coefficient i moves to i*g mod 2n, and
 * exponents >= n fold back with a sign change */
static void apply_galois_mod(int n, u64 m, const u64 *a, int g, u64 *out) {
    u64 *r = malloc(sizeof(u64) * n);
    for (int i = 0; i < n; i++) {
        int e = (int)(((long)i * g) % (2 * n));
        if (e < n) r[e] = a[i]; else r[e - n] = a[i] ? m - a[i] : 0;
    }
    memcpy(out, r, sizeof(u64) * n); free(r);
}
void orc_apply_galois(const orc_ctx *c, const u64 *a, int g, u64 *out) { apply_galois_mod(c->n, c->q, a, g, out); }
/* key-switching key for Galois element g: ndigits pairs (b_j, a_j),
 * b_j = -a_j s + e_j + B^j * s(X^g), B = 2^gadget_bits.  Layout ksk[j][0]=b_j, ksk[j][1]=a_j.
 *
 * With a special prime P the key lives modulo q*P and hides P * B^j * s(X^g): the two residues of a_j are
 * drawn independently (uniform mod q and mod P), the error is the same small integer on both sides, and
 *   b_j mod q = -a_{j,q} s + e_j + (P mod q) B^j s(X^g),     b_j mod P = -a_{j,P} s + e_j.
 * Layout ksk[j][0..3] = b_j mod q, a_j mod q, b_j mod P, a_j mod P. */
void orc_galois_key(const orc_ctx *c, const u64 *s, int g, u64 seed, u64 *ksk) {
    int n = c->n, kp = orc_key_polys(c); u64 q = c->q, P = c->P;
    u64 *sg = malloc(sizeof(u64) * n), *as = malloc(sizeof(u64) * n), *sP = malloc(sizeof(u64) * n);
    orc_apply_galois(c, s, g, sg);
    for (int i = 0; i < n; i++) sP[i] = s[i] == 0 ? 0 : (s[i] == 1 ? 1 : P - 1);   /* the ternary secret mod P */
    u64 Bj = P ? c->P_mod_q : 1;
    for (int j = 0; j < c->ndigits; j++) {
        u64 *b = ksk + (size_t)(kp * j) * n, *a = b + n;
        u64 base = ((u64)g << 32) + ((u64)j << 16);
        for (int i = 0; i < n; i++) a[i] = orc_uniform(q, seed, STREAM_KSK_A, base + i);
        orc_polymul(c, a, s, as);
        for (int i = 0; i < n; i++) {
            u64 e = signed_to_mod(orc_gauss(seed, STREAM_KSK_E, base + i), q);
            b[i] = addm(subm(e, as[i], q), mulm(Bj, sg[i], q), q);
        }
        if (P) {
            u64 *bP = a + n, *aP = bP + n;
            for (int i = 0; i < n; i++) aP[i] = orc_uniform(P, seed, STREAM_KSK_AP, base + i);
            orc_polymul_special(c, aP, sP, as);
            for (int i = 0; i < n; i++)
                bP[i] = subm(signed_to_mod(orc_gauss(seed, STREAM_KSK_E, base + i), P), as[i], P);
        }
        Bj = mulm(Bj, (1ull << c->gadget_bits) % q, q);
    }
    free(sg); free(as); free(sP);
}
/* DecPerm: unsigned base-B digits of the canonical coefficients of c1,
 * digits[j][i] = (c1[i] >> (j*w)) & (B-1).  Done once per ciphertext. */
void orc_decperm(const orc_ctx *c, const u64 *c1, u64 *digits) {
    u64 mask = (1ull << c->gadget_bits) - 1;
    for (int j = 0; j < c->ndigits; j++)
        for (int i = 0; i < c->n; i++)
            digits[(size_t)j * c->n + i] = (c1[i] >> (j * c->gadget_bits)) & mask;
}
/* HstPerm: out = ( c0(X^g) + sum_j d_j(X^g) b_j ,  sum_j d_j(X^g) a_j ).
 * The automorphism is applied to each digit polynomial AFTER decomposition
 * (a negated digit becomes q - d).
 *
 * With a special prime the two sums t are formed modulo q and modulo P (a negated digit is -d on both
 * sides), and each is divided by P exactly: with r = t mod P taken in [0,P),
 *   (t - r) / P  mod q  =  (t_q - (r mod q)) * P^-1  mod q,
 * i.e. the floor of t / P.  out = ( c0(X^g) + floor(t_b / P), floor(t_a / P) ). */
void orc_hstperm(const orc_ctx *c, const u64 *c0, const u64 *digits, int g, const u64 *ksk, u64 *out) {
    int n = c->n, kp = orc_key_polys(c); u64 q = c->q, P = c->P;
    u64 *o0 = malloc(sizeof(u64) * n), *o1 = calloc(n, sizeof(u64));
    u64 *dg = malloc(sizeof(u64) * n), *t = malloc(sizeof(u64) * n);
    u64 *tq = calloc(2 * (size_t)n, sizeof(u64)), *tP = calloc(2 * (size_t)n, sizeof(u64));
    orc_apply_galois(c, c0, g, o0);
    for (int j = 0; j < c->ndigits; j++) {
        const u64 *key = ksk + (size_t)(kp * j) * n;
        orc_apply_galois(c, digits + (size_t)j * n, g, dg);
        for (int h = 0; h < 2; h++) {
            orc_polymul(c, dg, key + (size_t)h * n, t);
            for (int i = 0; i < n; i++) tq[h * n + i] = addm(tq[h * n + i], t[i], q);
        }
        if (P) {
            apply_galois_mod(n, P, digits + (size_t)j * n, g, dg);
            for (int h = 0; h < 2; h++) {
                orc_polymul_special(c, dg, key + (size_t)(2 + h) * n, t);
                for (int i = 0; i < n; i++) tP[h * n + i] = addm(tP[h * n + i], t[i], P);
            }
        }
    }
    for (int i = 0; i < n; i++) {
        if (P) {
            o0[i] = addm(o0[i], mulm(subm(tq[i], tP[i] % q, q), c->Pinv_q, q), q);
            o1[i] = mulm(subm(tq[n + i], tP[n + i] % q, q), c->Pinv_q, q);
        } else {
            o0[i] = addm(o0[i], tq[i], q);
            o1[i] = tq[n + i];
        }
    }
    memcpy(out, o0, sizeof(u64) * n); memcpy(out + n, o1, sizeof(u64) * n);
    free(o0); free(o1); free(dg); free(t); free(tq); free(tP);
}
void orc_perm(const orc_ctx *c, const u64 *ct, int g, const u64 *ksk, u64 *out) {
    u64 *digits = malloc(sizeof(u64) * (size_t)c->ndigits * c->n);
    orc_decperm(c, ct + c->n, digits);
    orc_hstperm(c, ct, digits, g, ksk, out);
    free(digits);
}
/* Add and ScMult */
void orc_add(const orc_ctx *c, const u64 *x, const u64 *y, u64 *out) {
    for (int i = 0; i < 2 * c->n; i++) out[i] = addm(x[i], y[i], c->q);
}
void orc_scmult(const orc_ctx *c, const u64 *ct, const u64 *w_poly_q, u64 *out) {
    orc_polymul(c, ct, w_poly_q, out);
    orc_polymul(c, ct + c->n, w_poly_q, out + c->n);
}
/* plaintext subtraction used for share generation: c0 -= delta * encode(mask slots) */
void orc_sub_plain(const orc_ctx *c, const u64 *ct, const u64 *mask_slots, u64 *out) {
    int n = c->n; u64 q = c->q;
    u64 *m = malloc(sizeof(u64) * n);
    orc_encode(c, mask_slots, m, 0);
    for (int i = 0; i < n; i++) out[i] = subm(ct[i], mulm(c->delta, m[i], q), q);
    if (out != ct) memcpy(out + n, ct + n, sizeof(u64) * n);
    free(m);
}

/* operation counters, in the paper's vocabulary */
typedef struct { i64 perm, decperm_in, hstperm_in, scmult, add; } orc_counts;

/* ------------------------------------------------------------------ */
/* FC: row-encoding-share-RaS  (Sec. III-A(3))                          */
/* ------------------------------------------------------------------ */
static int pow2ceil(int v) { int r = 1; while (r < v) r <<= 1; return r; }

typedef struct { int n, half, no, ni, nop, nip, G, big; } fc_geom;   /* big: n_i fills the whole ciphertext */
static int fc_geometry(const orc_ctx *c, int n_o, int n_i, fc_geom *g) {
    g->n = c->n; g->half = c->n / 2; g->no = n_o; g->ni = n_i;
    g->nop = pow2ceil(n_o); g->nip = pow2ceil(n_i);
    if (g->nip > g->n || g->nop > g->n) return -1;
    g->big = g->nip == g->n;
    if (g->big) { if (g->nop > g->half) return -1; g->G = g->nop; }
    else { long prod = (long)g->nip * g->nop; g->G = prod >= g->n ? (int)(prod / g->n) : 1; }
    return 0;
}
int orc_fc_G(const orc_ctx *c, int n_o, int n_i) { fc_geom g; return fc_geometry(c, n_o, n_i, &g) ? -1 : g.G; }
/* which (padded) output row the partial sum in slot (h,k) belongs to; -1 if the
 * slot carries no weight (only when n_i*n_o < n: copies beyond the n_o-th) */
static int fc_row(const fc_geom *g, int h, int k) {
    if (g->big) return k % g->nop;
    int copy = h * (g->half / g->nip) + k / g->nip, j = k % g->nip;
    if ((long)g->nip * g->nop < g->n && copy >= g->nop) return -1;
    return (((j - copy * g->G) % g->nop) + g->nop) % g->nop;
}
/* which input entry sits in slot (h,k) of the packed input */
static int fc_col(const fc_geom *g, int h, int k) { return g->big ? h * g->half + k : k % g->nip; }

/* client side: n/n_i copies of x */
void orc_fc_pack_input(const orc_ctx *c, int n_o, int n_i, const u64 *x, u64 *slots) {
    fc_geom g; fc_geometry(c, n_o, n_i, &g);
    for (int h = 0; h < 2; h++)
        for (int k = 0; k < g.half; k++) {
            int col = fc_col(&g, h, k);
            slots[h * g.half + k] = col < n_i ? x[col] % c->p : 0;
        }
}
/* slot vector of the g-th encoded weight plaintext:
 * after rotating left by g, slot (h,k) must hold W[row(h,k)][col(h,k+g)] * x[col(h,k+g)],
 * so before rotation slot (h,k') holds W[row(h,k'-g)][col(h,k')] */
void orc_fc_weight_slots(const orc_ctx *c, const u64 *W, int n_o, int n_i, int gi, u64 *slots) {
    fc_geom g; fc_geometry(c, n_o, n_i, &g);
    for (int h = 0; h < 2; h++)
        for (int k = 0; k < g.half; k++) {
            int row = fc_row(&g, h, ((k - gi) % g.half + g.half) % g.half), col = fc_col(&g, h, k);
            slots[h * g.half + k] = (row >= 0 && row < n_o && col < n_i) ? W[(size_t)row * n_i + col] % c->p : 0;
        }
}
/* "encode-rowwise": the G plaintext polynomials (mod q, centred lift) */
void orc_fc_encode_rowwise(const orc_ctx *c, const u64 *W, int n_o, int n_i, u64 *wpoly) {
    fc_geom g; fc_geometry(c, n_o, n_i, &g);
    u64 *slots = malloc(sizeof(u64) * c->n);
    for (int gi = 0; gi < g.G; gi++) {
        orc_fc_weight_slots(c, W, n_o, n_i, gi, slots);
        orc_encode_weight(c, slots, wpoly + (size_t)gi * c->n);
    }
    free(slots);
}
/* plaintext RaS on a decrypted (or mask) slot vector: out[t] = sum of the slots of row t */
void orc_fc_unpack_share(const orc_ctx *c, int n_o, int n_i, const u64 *slots, u64 *out) {
    fc_geom g; fc_geometry(c, n_o, n_i, &g);
    for (int t = 0; t < n_o; t++) out[t] = 0;
    for (int h = 0; h < 2; h++)
        for (int k = 0; k < g.half; k++) {
            int row = fc_row(&g, h, k);
            if (row >= 0 && row < n_o) out[row] = addm(out[row], slots[h * g.half + k] % c->p, c->p);
        }
}
/* server's full-length random vector r' with unpack_share(r') = r: every slot is
 * drawn from the mask stream except the first slot of each real row, which
 * absorbs the difference */
void orc_fc_mask_slots(const orc_ctx *c, int n_o, int n_i, const u64 *r, u64 seed, int b, u64 *slots) {
    fc_geom g; fc_geometry(c, n_o, n_i, &g);
    int *first = malloc(sizeof(int) * n_o);
    u64 *sum = calloc(n_o, sizeof(u64));
    for (int t = 0; t < n_o; t++) first[t] = -1;
    for (int s = 0; s < c->n; s++) {
        int row = fc_row(&g, s / g.half, s % g.half);
        if (row >= 0 && row < n_o && first[row] < 0) { first[row] = s; continue; }
        slots[s] = orc_uniform(c->p, seed, STREAM_MASK, ((u64)b << 32) + (u64)s);
        if (row >= 0 && row < n_o) sum[row] = addm(sum[row], slots[s], c->p);
    }
    for (int t = 0; t < n_o; t++) slots[first[t]] = subm(r[t] % c->p, sum[t], c->p);
    free(first); free(sum);
}
/* he_fc for one input ciphertext:
 *   out = sum_g Perm_g( ScMult(ct, w_g) ) - r'      (Perm_0 = identity)
 * ksk holds the keys of rotations g = 1..G-1 in order (each ndigits * orc_key_polys * n words). */
void orc_he_fc(const orc_ctx *c, const u64 *wpoly, int G, const u64 *ct, const u64 *ksk,
               const u64 *mask_slots, u64 *out, orc_counts *cnt) {
    int n = c->n;
    size_t ksz = (size_t)c->ndigits * orc_key_polys(c) * n;
    u64 *u = malloc(sizeof(u64) * 2 * n), *v = malloc(sizeof(u64) * 2 * n), *acc = malloc(sizeof(u64) * 2 * n);
    for (int g = 0; g < G; g++) {
        orc_scmult(c, ct, wpoly + (size_t)g * n, u); if (cnt) cnt->scmult++;
        if (g == 0) { memcpy(acc, u, sizeof(u64) * 2 * n); continue; }
        orc_perm(c, u, orc_galois_elt(c, 0, g), ksk + (size_t)(g - 1) * ksz, v); if (cnt) cnt->perm++;
        orc_add(c, acc, v, acc); if (cnt) cnt->add++;
    }
    orc_sub_plain(c, acc, mask_slots, out);
    free(u); free(v); free(acc);
}

/* ------------------------------------------------------------------ */
/* Conv: kernel grouping, first-Add-second-Perm  (Sec. III-B(3))        */
/* ------------------------------------------------------------------ */
typedef struct { int n, half, co, ci, kh, kw, uh, uw, T, cn, hpos, nin, nout, ntap; } cv_geom;
static int cv_geometry(const orc_ctx *c, int co, int ci, int kh, int kw, int uh, int uw, cv_geom *g) {
    g->n = c->n; g->half = c->n / 2; g->co = co; g->ci = ci; g->kh = kh; g->kw = kw; g->uh = uh; g->uw = uw;
    g->T = pow2ceil(uh * uw);
    if (g->T > g->half || !(kh & 1) || !(kw & 1)) return -1;
    g->cn = c->n / g->T; g->hpos = g->cn / 2;
    g->nin = (ci + g->cn - 1) / g->cn; g->nout = (co + g->cn - 1) / g->cn; g->ntap = kh * kw;
    return 0;
}
int orc_conv_geometry(const orc_ctx *c, int co, int ci, int kh, int kw, int uh, int uw, int *out5) {
    cv_geom g; if (cv_geometry(c, co, ci, kh, kw, uh, uw, &g)) return -1;
    out5[0] = g.T; out5[1] = g.cn; out5[2] = g.nin; out5[3] = g.nout; out5[4] = g.ntap; return 0;
}
/* raster offset of tap t = (dy,dx), dy in [-kh/2,kh/2], dx likewise */
static int cv_tap_offset(const cv_geom *g, int tap) {
    int dy = tap / g->kw - g->kh / 2, dx = tap % g->kw - g->kw / 2;
    return dy * g->uw + dx;
}
/* client side: channel (I*cn + h*hpos + kappa) occupies slots (h, kappa*T + y*uw + x) of ciphertext I */
void orc_conv_pack_input(const orc_ctx *c, int co, int ci, int kh, int kw, int uh, int uw,
                         const u64 *in /* ci x uh x uw */, u64 *slots /* nin x n */) {
    cv_geom g; cv_geometry(c, co, ci, kh, kw, uh, uw, &g);
    memset(slots, 0, sizeof(u64) * (size_t)g.nin * g.n);
    for (int ch = 0; ch < ci; ch++) {
        int I = ch / g.cn, pos = ch % g.cn, h = pos / g.hpos, kap = pos % g.hpos;
        for (int y = 0; y < uh; y++)
            for (int x = 0; x < uw; x++)
                slots[(size_t)I * g.n + h * g.half + kap * g.T + y * uw + x] = in[((size_t)ch * uh + y) * uw + x] % c->p;
    }
}
/* slot vector of the plaintext that multiplies the tap-rotated input I for output
 * block O and kernel order (group element) gam = s*hpos + t:
 * at channel position pi' = (h,kappa): input channel I*cn + idx(pi'), output channel
 * O*cn + idx(pi' - g); zero where the tap falls outside the image. */
void orc_conv_weight_slots(const orc_ctx *c, const u64 *K /* co x ci x kh x kw */, int co, int ci, int kh, int kw,
                           int uh, int uw, int O, int gam, int I, int tap, u64 *slots) {
    cv_geom g; cv_geometry(c, co, ci, kh, kw, uh, uw, &g);
    int gs = gam / g.hpos, gt = gam % g.hpos;
    int dy = tap / kw - kh / 2, dx = tap % kw - kw / 2;
    memset(slots, 0, sizeof(u64) * g.n);
    for (int h = 0; h < 2; h++)
        for (int kap = 0; kap < g.hpos; kap++) {
            int in_ch = I * g.cn + h * g.hpos + kap;
            int oh = h ^ gs, okap = ((kap - gt) % g.hpos + g.hpos) % g.hpos;
            int out_ch = O * g.cn + oh * g.hpos + okap;
            if (in_ch >= ci || out_ch >= co) continue;
            for (int y = 0; y < uh; y++)
                for (int x = 0; x < uw; x++) {
                    if (y + dy < 0 || y + dy >= uh || x + dx < 0 || x + dx >= uw) continue;
                    slots[h * g.half + kap * g.T + y * uw + x] =
                        K[(((size_t)out_ch * ci + in_ch) * kh + (dy + kh / 2)) * kw + (dx + kw / 2)] % c->p;
                }
        }
}
/* Galois element that brings kernel order gam back to the output position:
 * out[(h,kappa)] = in[(h^s, kappa+t)], i.e. rows rotated left by t*T, swapped if s */
int orc_conv_group_galois(const orc_ctx *c, int co, int ci, int kh, int kw, int uh, int uw, int gam) {
    cv_geom g; cv_geometry(c, co, ci, kh, kw, uh, uw, &g);
    return orc_galois_elt(c, gam / g.hpos, (gam % g.hpos) * g.T);
}
int orc_conv_tap_galois(const orc_ctx *c, int co, int ci, int kh, int kw, int uh, int uw, int tap) {
    cv_geom g; cv_geometry(c, co, ci, kh, kw, uh, uw, &g);
    return orc_galois_elt(c, 0, cv_tap_offset(&g, tap));
}
/* mask for output ciphertext O: real outputs get r[co][y][x], every other slot a draw from the mask stream */
void orc_conv_mask_slots(const orc_ctx *c, int co, int ci, int kh, int kw, int uh, int uw,
                         const u64 *r /* co x uh x uw */, u64 seed, int b, int O, u64 *slots) {
    cv_geom g; cv_geometry(c, co, ci, kh, kw, uh, uw, &g);
    for (int s = 0; s < g.n; s++) {
        int h = s / g.half, k = s % g.half, kap = k / g.T, off = k % g.T;
        int ch = O * g.cn + h * g.hpos + kap;
        if (ch < co && off < uh * uw) slots[s] = r[(size_t)ch * uh * uw + off] % c->p;
        else slots[s] = orc_uniform(c->p, seed, STREAM_MASK, ((u64)b << 32) + ((u64)O << 16) + (u64)s);
    }
}
void orc_conv_unpack_share(const orc_ctx *c, int co, int ci, int kh, int kw, int uh, int uw,
                           int O, const u64 *slots, u64 *out /* co x uh x uw, block O filled */) {
    cv_geom g; cv_geometry(c, co, ci, kh, kw, uh, uw, &g);
    for (int pos = 0; pos < g.cn; pos++) {
        int ch = O * g.cn + pos, h = pos / g.hpos, kap = pos % g.hpos;
        if (ch >= co) continue;
        for (int off = 0; off < uh * uw; off++)
            out[(size_t)ch * uh * uw + off] = slots[h * g.half + kap * g.T + off] % c->p;
    }
}
/* he_conv for ONE output ciphertext O of one input (nin ciphertexts):
 *   1. per input ciphertext: one DecPerm, then one HstPerm per non-central tap;
 *   2. per kernel order gam: acc_gam = sum_{I,tap} ScMult(Xrot[I][tap], pt[O][gam][I][tap])   (Add first)
 *   3. out = sum_gam Perm_gam(acc_gam) - mask                                               (Perm second)
 * xrot, if non-NULL, supplies/receives the tap-rotated inputs (nin x ntap cts) so that
 * several output blocks of the same input can share step 1; *xrot_ready says whether it is filled.
 * tap_ksk: keys of the non-central taps in tap order; grp_ksk: keys of gam = 1..cn-1. */
void orc_he_conv_block(const orc_ctx *c, const u64 *K, int co, int ci, int kh, int kw, int uh, int uw,
                       int O, const u64 *cts /* nin x 2n */, const u64 *tap_ksk, const u64 *grp_ksk,
                       const u64 *mask_slots, u64 *xrot, int *xrot_ready, u64 *out, orc_counts *cnt) {
    cv_geom g; cv_geometry(c, co, ci, kh, kw, uh, uw, &g);
    int n = g.n, centre = (kh / 2) * kw + kw / 2;
    size_t ksz = (size_t)c->ndigits * orc_key_polys(c) * n, ctsz = 2 * (size_t)n;
    u64 *own = NULL;
    if (!xrot) { own = malloc(sizeof(u64) * ctsz * g.nin * g.ntap); xrot = own; }
    if (own || !*xrot_ready) {
        u64 *digits = malloc(sizeof(u64) * (size_t)c->ndigits * n);
        for (int I = 0; I < g.nin; I++) {
            const u64 *ct = cts + I * ctsz;
            if (g.ntap > 1) { orc_decperm(c, ct + n, digits); if (cnt) cnt->decperm_in++; }
            for (int tap = 0, kidx = 0; tap < g.ntap; tap++) {
                u64 *dst = xrot + ((size_t)I * g.ntap + tap) * ctsz;
                if (tap == centre) { memcpy(dst, ct, sizeof(u64) * ctsz); continue; }
                orc_hstperm(c, ct, digits, orc_galois_elt(c, 0, cv_tap_offset(&g, tap)), tap_ksk + kidx * ksz, dst);
                if (cnt) cnt->hstperm_in++;
                kidx++;
            }
        }
        free(digits);
        if (xrot_ready) *xrot_ready = 1;
    }
    u64 *slots = malloc(sizeof(u64) * n), *w = malloc(sizeof(u64) * n);
    u64 *u = malloc(sizeof(u64) * ctsz), *acc = malloc(sizeof(u64) * ctsz), *tot = malloc(sizeof(u64) * ctsz);
    for (int gam = 0; gam < g.cn; gam++) {
        int started = 0;
        for (int I = 0; I < g.nin; I++)
            for (int tap = 0; tap < g.ntap; tap++) {
                orc_conv_weight_slots(c, K, co, ci, kh, kw, uh, uw, O, gam, I, tap, slots);
                orc_encode_weight(c, slots, w);
                orc_scmult(c, xrot + ((size_t)I * g.ntap + tap) * ctsz, w, u); if (cnt) cnt->scmult++;
                if (!started) { memcpy(acc, u, sizeof(u64) * ctsz); started = 1; }
                else { orc_add(c, acc, u, acc); if (cnt) cnt->add++; }
            }
        if (gam == 0) { memcpy(tot, acc, sizeof(u64) * ctsz); continue; }
        orc_perm(c, acc, orc_galois_elt(c, gam / g.hpos, (gam % g.hpos) * g.T), grp_ksk + (size_t)(gam - 1) * ksz, u);
        if (cnt) cnt->perm++;
        orc_add(c, tot, u, tot); if (cnt) cnt->add++;
    }
    orc_sub_plain(c, tot, mask_slots, out);
    free(slots); free(w); free(u); free(acc); free(tot); free(own);
}

/* ------------------------------------------------------------------ */
/* The comparison schedules of the paper, on the same operations:       */
/* hybrid matrix-vector product (Sec. III-A(2)) and output-rotation     */
/* MIMO convolution (Sec. III-B(2)).                                    */
/* ------------------------------------------------------------------ */
/* Hybrid FC.  The paper gives the method on one cycle of n slots and leaves the packed layout to a figure; on
 * the 2 x n/2 torus it is read as follows (n_o, n_i padded to powers of two):
 *  n_i <= n/2: every half-row holds n/(2 n_i) copies of x.  Copy c owns R = max(1, n_i n_o / n) output rows
 *    c*R .. c*R+R-1 (no rows when n_i n_o < n and c >= n_o); slot (h,k) of copy c, j = k mod n_i, collects row
 *    c*R + (j mod R).  G = R input rotations: w_g[(h,k)] = W[row(h,k)][(j+g) mod n_i] multiplies x_pack rotated
 *    left by g.  After the sum over g slot (h,k) holds the partial product of its row over columns j .. j+R-1;
 *    the rotate-and-sum steps by n_i/2, n_i/4, .., R add the n_i/R partial sums of a row, and row c*R + j ends up
 *    in slot j < R of copy c.
 *  n_i = n: half h holds x[h*n/2 ..]; slot (h,k) collects row k mod n_o over the columns of its half, G = n_o
 *    input rotations, rotate-and-sum steps by n/4, .., n_o inside the rows and one row swap at the end; row t ends
 *    up in slot (0,t).
 * Counts: G ScMult, G-1 HstPerm of the input (one DecPerm), log2(n/n_o) Perm when n_i n_o >= n, as in Table
 * "Complexity comparison of three methods". */
typedef struct { int n, half, no, ni, nop, nip, G, R, big, steps; } hy_geom;
static int hy_geometry(const orc_ctx *c, int n_o, int n_i, hy_geom *g) {
    g->n = c->n; g->half = c->n / 2; g->no = n_o; g->ni = n_i;
    g->nop = pow2ceil(n_o); g->nip = pow2ceil(n_i);
    if (g->nip > g->n || g->nop > g->n) return -1;
    g->big = g->nip == g->n;
    if (g->big) {
        if (g->nop > g->half) return -1;
        g->G = g->R = g->nop; g->steps = ilog2(g->half / g->nop) + 1;
    } else {
        long prod = (long)g->nip * g->nop;
        g->R = prod >= g->n ? (int)(prod / g->n) : 1;
        g->G = g->R; g->steps = ilog2(g->nip / g->R);
    }
    return 0;
}
int orc_fc_hybrid_G(const orc_ctx *c, int n_o, int n_i) { hy_geom g; return hy_geometry(c, n_o, n_i, &g) ? -1 : g.G; }
/* the rotate-and-sum rotations in order; returns their number */
int orc_fc_hybrid_ras(const orc_ctx *c, int n_o, int n_i, int *swap, int *step) {
    hy_geom g; if (hy_geometry(c, n_o, n_i, &g)) return -1;
    int k = 0;
    for (int rho = (g.big ? g.half : g.nip) / 2; rho >= g.R; rho /= 2) { swap[k] = 0; step[k] = rho; k++; }
    if (g.big) { swap[k] = 1; step[k] = 0; k++; }
    return k;
}
static int hy_row(const hy_geom *g, int h, int k) {
    if (g->big) return k % g->nop;
    int copy = h * (g->half / g->nip) + k / g->nip, j = k % g->nip;
    if ((long)g->nip * g->nop < g->n && copy >= g->nop) return -1;
    return copy * g->R + j % g->R;
}
/* the slot that holds output row t after the rotate-and-sum steps */
static int hy_result_slot(const hy_geom *g, int t) {
    if (g->big) return t;
    int copy = t / g->R, per_row = g->half / g->nip;
    return (copy / per_row) * g->half + (copy % per_row) * g->nip + t % g->R;
}
void orc_fc_hybrid_weight_slots(const orc_ctx *c, const u64 *W, int n_o, int n_i, int gi, u64 *slots) {
    hy_geom g; hy_geometry(c, n_o, n_i, &g);
    for (int h = 0; h < 2; h++)
        for (int k = 0; k < g.half; k++) {
            int row = hy_row(&g, h, k);
            int col = g.big ? h * g.half + (k + gi) % g.half : (k % g.nip + gi) % g.nip;
            slots[h * g.half + k] = (row >= 0 && row < n_o && col < n_i) ? W[(size_t)row * n_i + col] % c->p : 0;
        }
}
void orc_fc_hybrid_encode(const orc_ctx *c, const u64 *W, int n_o, int n_i, u64 *wpoly) {
    hy_geom g; hy_geometry(c, n_o, n_i, &g);
    u64 *slots = malloc(sizeof(u64) * c->n);
    for (int gi = 0; gi < g.G; gi++) {
        orc_fc_hybrid_weight_slots(c, W, n_o, n_i, gi, slots);
        orc_encode_weight(c, slots, wpoly + (size_t)gi * c->n);
    }
    free(slots);
}
void orc_fc_hybrid_unpack(const orc_ctx *c, int n_o, int n_i, const u64 *slots, u64 *out) {
    hy_geom g; hy_geometry(c, n_o, n_i, &g);
    for (int t = 0; t < n_o; t++) out[t] = slots[hy_result_slot(&g, t)] % c->p;
}
/* the server's random vector: its share r at the result slots, a draw from the mask stream everywhere else */
void orc_fc_hybrid_mask_slots(const orc_ctx *c, int n_o, int n_i, const u64 *r, u64 seed, int b, u64 *slots) {
    hy_geom g; hy_geometry(c, n_o, n_i, &g);
    for (int s = 0; s < c->n; s++) slots[s] = orc_uniform(c->p, seed, STREAM_MASK, ((u64)b << 32) + (u64)s);
    for (int t = 0; t < n_o; t++) slots[hy_result_slot(&g, t)] = r[t] % c->p;
}
/* out = RaS( sum_g ScMult( HstPerm_g(ct), w_g ) ) - mask, every rotate-and-sum step a Perm and an Add on the
 * running ciphertext.  ksk_in: keys of the input rotations g = 1..G-1; ksk_ras: keys of orc_fc_hybrid_ras in order. */
void orc_he_fc_hybrid(const orc_ctx *c, const u64 *wpoly, int n_o, int n_i, const u64 *ct, const u64 *ksk_in,
                      const u64 *ksk_ras, const u64 *mask_slots, u64 *out, orc_counts *cnt) {
    hy_geom g; hy_geometry(c, n_o, n_i, &g);
    int n = c->n;
    size_t ksz = (size_t)c->ndigits * orc_key_polys(c) * n;
    u64 *digits = malloc(sizeof(u64) * (size_t)c->ndigits * n);
    u64 *xr = malloc(sizeof(u64) * 2 * n), *u = malloc(sizeof(u64) * 2 * n), *acc = malloc(sizeof(u64) * 2 * n);
    if (g.G > 1) { orc_decperm(c, ct + n, digits); if (cnt) cnt->decperm_in++; }
    for (int gi = 0; gi < g.G; gi++) {
        if (gi == 0) memcpy(xr, ct, sizeof(u64) * 2 * n);
        else { orc_hstperm(c, ct, digits, orc_galois_elt(c, 0, gi), ksk_in + (size_t)(gi - 1) * ksz, xr); if (cnt) cnt->hstperm_in++; }
        orc_scmult(c, xr, wpoly + (size_t)gi * n, u); if (cnt) cnt->scmult++;
        if (gi == 0) memcpy(acc, u, sizeof(u64) * 2 * n);
        else { orc_add(c, acc, u, acc); if (cnt) cnt->add++; }
    }
    int sw[32], st[32], steps = orc_fc_hybrid_ras(c, n_o, n_i, sw, st);
    for (int k = 0; k < steps; k++) {
        orc_perm(c, acc, orc_galois_elt(c, sw[k], st[k]), ksk_ras + (size_t)k * ksz, u); if (cnt) cnt->perm++;
        orc_add(c, acc, u, acc); if (cnt) cnt->add++;
    }
    orc_sub_plain(c, acc, mask_slots, out);
    free(digits); free(xr); free(u); free(acc);
}

/* Output-rotation MIMO convolution for ONE output ciphertext O (Sec. III-B(2)): the same encoded kernels, input
 * rotations and kernel orders as orc_he_conv_block, but every (O, I) block is finished on its own:
 *   block_I = sum_gam Perm_gam( sum_tap ScMult(Xrot[I][tap], pt[O][gam][I][tap]) ),   out = sum_I block_I - mask,
 * i.e. c_n - 1 Perm per block instead of per output ciphertext. */
void orc_he_conv_outrot_block(const orc_ctx *c, const u64 *K, int co, int ci, int kh, int kw, int uh, int uw,
                              int O, const u64 *cts /* nin x 2n */, const u64 *tap_ksk, const u64 *grp_ksk,
                              const u64 *mask_slots, u64 *xrot, int *xrot_ready, u64 *out, orc_counts *cnt) {
    cv_geom g; cv_geometry(c, co, ci, kh, kw, uh, uw, &g);
    int n = g.n, centre = (kh / 2) * kw + kw / 2;
    size_t ksz = (size_t)c->ndigits * orc_key_polys(c) * n, ctsz = 2 * (size_t)n;
    u64 *own = NULL;
    if (!xrot) { own = malloc(sizeof(u64) * ctsz * g.nin * g.ntap); xrot = own; }
    if (own || !*xrot_ready) {
        u64 *digits = malloc(sizeof(u64) * (size_t)c->ndigits * n);
        for (int I = 0; I < g.nin; I++) {
            const u64 *ct = cts + I * ctsz;
            if (g.ntap > 1) { orc_decperm(c, ct + n, digits); if (cnt) cnt->decperm_in++; }
            for (int tap = 0, kidx = 0; tap < g.ntap; tap++) {
                u64 *dst = xrot + ((size_t)I * g.ntap + tap) * ctsz;
                if (tap == centre) { memcpy(dst, ct, sizeof(u64) * ctsz); continue; }
                orc_hstperm(c, ct, digits, orc_galois_elt(c, 0, cv_tap_offset(&g, tap)), tap_ksk + kidx * ksz, dst);
                if (cnt) cnt->hstperm_in++;
                kidx++;
            }
        }
        free(digits);
        if (xrot_ready) *xrot_ready = 1;
    }
    u64 *slots = malloc(sizeof(u64) * n), *w = malloc(sizeof(u64) * n);
    u64 *u = malloc(sizeof(u64) * ctsz), *acc = malloc(sizeof(u64) * ctsz), *blk = malloc(sizeof(u64) * ctsz);
    u64 *tot = malloc(sizeof(u64) * ctsz);
    for (int I = 0; I < g.nin; I++) {
        for (int gam = 0; gam < g.cn; gam++) {
            for (int tap = 0; tap < g.ntap; tap++) {
                orc_conv_weight_slots(c, K, co, ci, kh, kw, uh, uw, O, gam, I, tap, slots);
                orc_encode_weight(c, slots, w);
                orc_scmult(c, xrot + ((size_t)I * g.ntap + tap) * ctsz, w, u); if (cnt) cnt->scmult++;
                if (tap == 0) memcpy(acc, u, sizeof(u64) * ctsz);
                else { orc_add(c, acc, u, acc); if (cnt) cnt->add++; }
            }
            if (gam == 0) { memcpy(blk, acc, sizeof(u64) * ctsz); continue; }
            orc_perm(c, acc, orc_galois_elt(c, gam / g.hpos, (gam % g.hpos) * g.T), grp_ksk + (size_t)(gam - 1) * ksz, u);
            if (cnt) cnt->perm++;
            orc_add(c, blk, u, blk); if (cnt) cnt->add++;
        }
        if (I == 0) memcpy(tot, blk, sizeof(u64) * ctsz);
        else { orc_add(c, tot, blk, tot); if (cnt) cnt->add++; }
    }
    orc_sub_plain(c, tot, mask_slots, out);
    free(slots); free(w); free(u); free(acc); free(blk); free(tot); free(own);
}

/* ------------------------------------------------------------------ */
/* batches: independent inputs, one OpenMP thread each                  */
/* ------------------------------------------------------------------ */
#ifdef _OPENMP
#include <omp.h>
int orc_max_threads(void) { return omp_get_max_threads(); }
#else
int orc_max_threads(void) { return 1; }
#endif
/* r: batch x n_o final server shares; b0: index of the first item (enters the mask stream) */
void orc_he_fc_batch(const orc_ctx *c, const u64 *wpoly, int n_o, int n_i, const u64 *cts, int batch, int b0,
                     const u64 *ksk, const u64 *r, u64 mask_seed, u64 *out, orc_counts *cnt) {
    int G = orc_fc_G(c, n_o, n_i), n = c->n;
    orc_counts *local = calloc(batch, sizeof *local);
    #pragma omp parallel for schedule(dynamic)
    for (int b = 0; b < batch; b++) {
        u64 *mask = malloc(sizeof(u64) * n);
        orc_fc_mask_slots(c, n_o, n_i, r + (size_t)b * n_o, mask_seed, b0 + b, mask);
        orc_he_fc(c, wpoly, G, cts + (size_t)b * 2 * n, ksk, mask, out + (size_t)b * 2 * n, &local[b]);
        free(mask);
    }
    if (cnt) for (int b = 0; b < batch; b++) {
        cnt->perm += local[b].perm; cnt->scmult += local[b].scmult; cnt->add += local[b].add;
    }
    free(local);
}
