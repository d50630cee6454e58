// Host half of the library: number theory, transform tables, seeded samplers,
// slot encoding, key generation, encryption / decryption and the offline
// encoders of the two layer types.  Device memory is touched only to upload
// tables, keys and encoded weights.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstring>
#include <new>
#include <thread>

#include "gala_internal.h"

namespace gala {

// ---------------------------------------------------------------------------
// number theory
// ---------------------------------------------------------------------------
static u64 mulmod_slow(u64 a, u64 b, u64 m) { return (u64)(((u128)a * b) % m); }
u64 pow_mod(u64 b, u64 e, u64 m) {
    u64 r = 1 % m;
    b %= m;
    for (; e; e >>= 1) {
        if (e & 1) r = mulmod_slow(r, b, m);
        b = mulmod_slow(b, b, m);
    }
    return r;
}
u64 inv_mod(u64 a, u64 m) { return pow_mod(a, m - 2, m); }
u64 shoup_companion(u64 w, u64 q) { return (u64)((((u128)w) << 64) / q); }
int bit_length(u64 v) {
    int l = 0;
    for (; v; v >>= 1) ++l;
    return l;
}
Modulus make_modulus(u64 q) {
    Modulus m;
    m.q = q;
    m.q2 = 2 * q;
    m.c64 = (u64)((((u128)1) << 64) % q);
    m.c64s = shoup_companion(m.c64, q);
    m.one_s = shoup_companion(1, q);
    return m;
}
bool is_prime_u64(u64 v) {
    if (v < 2) return false;
    static const u64 bases[] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    for (u64 b : bases)
        if (v % b == 0) return v == b;
    u64 d = v - 1;
    int r = 0;
    while (!(d & 1)) { d >>= 1; ++r; }
    for (u64 a : bases) {                 // deterministic for 64-bit inputs
        u64 x = pow_mod(a, d, v);
        if (x == 1 || x == v - 1) continue;
        bool composite = true;
        for (int i = 1; i < r && composite; ++i) {
            x = mulmod_slow(x, x, v);
            if (x == v - 1) composite = false;
        }
        if (composite) return false;
    }
    return true;
}
// a generator of the 2n-th roots of unity, found from the first x whose
// ((m-1)/2n)-th power has order exactly 2n
static u64 primitive_2n_root(u64 m, int n) {
    for (u64 x = 2; x < m; ++x) {
        u64 c = pow_mod(x, (m - 1) / (2 * (u64)n), m);
        if (pow_mod(c, (u64)n, m) == m - 1) return c;
    }
    return 0;
}
static u64 least_primitive_2n_root(u64 m, int n) {
    u64 c = primitive_2n_root(m, n), sq = mulmod_slow(c, c, m), cur = c, best = c;
    for (int e = 3; e < 2 * n; e += 2) {
        cur = mulmod_slow(cur, sq, m);
        best = std::min(best, cur);
    }
    return best;
}

// ---------------------------------------------------------------------------
// transform tables and the host transform
// ---------------------------------------------------------------------------
void NttHost::init(int n_, u64 q, u64 psi_) {
    n = n_;
    logn = bit_length((u64)n) - 1;
    mod = make_modulus(q);
    psi = psi_;
    u64 ipsi = inv_mod(psi, q);
    tw.assign(n, 0); tws.assign(n, 0); itw.assign(n, 0); itws.assign(n, 0);
    std::vector<u64> pw(n), ipw(n);
    pw[0] = ipw[0] = 1;
    for (int i = 1; i < n; ++i) {
        pw[i] = mulmod_slow(pw[i - 1], psi, q);
        ipw[i] = mulmod_slow(ipw[i - 1], ipsi, q);
    }
    for (int k = 0; k < n; ++k) {
        int r = brev(k, logn);
        tw[k] = pw[r];   tws[k] = shoup_companion(tw[k], q);
        itw[k] = ipw[r]; itws[k] = shoup_companion(itw[k], q);
    }
    ninv = inv_mod((u64)n, q);           ninvs = shoup_companion(ninv, q);
    itw1n = mulmod_slow(itw[1], ninv, q); itw1ns = shoup_companion(itw1n, q);
}
void NttHost::forward(u64 *a) const {
    const u64 q = mod.q, q2 = mod.q2;
    for (int m = 1, t = n >> 1; m < n; m <<= 1, t >>= 1)
        for (int i = 0; i < m; ++i) {
            const u64 w = tw[m + i], ws = tws[m + i];
            u64 *x = a + 2 * i * t, *y = x + t;
            for (int j = 0; j < t; ++j) butterfly_fwd(x[j], y[j], w, ws, q, q2);
        }
    for (int i = 0; i < n; ++i) a[i] = csub(csub(a[i], q2), q);
}
void NttHost::inverse(u64 *a) const {
    const u64 q = mod.q, q2 = mod.q2;
    int t = 1;
    for (int m = n >> 1; m > 1; m >>= 1, t <<= 1)
        for (int i = 0; i < m; ++i) {
            const u64 w = itw[m + i], ws = itws[m + i];
            u64 *x = a + 2 * i * t, *y = x + t;
            for (int j = 0; j < t; ++j) butterfly_inv(x[j], y[j], w, ws, q, q2);
        }
    // last stage (one block, t = n/2) with n^-1 folded in
    for (int j = 0; j < t; ++j) {
        u64 x = a[j], y = a[j + t];
        a[j] = mul_shoup(x + y, ninv, ninvs, q);
        a[j + t] = mul_shoup(x - y + q2, itw1n, itw1ns, q);
    }
}

// ---------------------------------------------------------------------------
// samplers
// ---------------------------------------------------------------------------
// floor(2^64 * P[X <= -19+i]) for the discrete Gaussian with sigma = 3.2 on [-19,19]
static const u64 kGaussCdf[38] = {
    0x0000000bd798c7acull, 0x00000053f5e234f7ull, 0x000001e24b89625aull, 0x000009adbc7900e1ull,
    0x00002d17ca1e3a82ull, 0x0000bf05ff772ee2ull, 0x0002e06843bbf95dull, 0x000a19062dceb033ull,
    0x00204c0ded173b17ull, 0x005e3163ffc656a8ull, 0x00fab6a7e614dfaeull, 0x0261b16e99bc14f8ull,
    0x054c69348bbc9867ull, 0x0acd276539458231ull, 0x143796b3c337f00bull, 0x22d43df09de40e7aull,
    0x37651d96aa4fb429ull, 0x51a5da2b40f1bff1ull, 0x700ad4bf5a6e80e2ull, 0x8ff52b40a5917f1dull,
    0xae5a25d4bf0e400eull, 0xc89ae26955b04bd6ull, 0xdd2bc20f621bf185ull, 0xebc8694c3cc80ff4ull,
    0xf532d89ac6ba7dceull, 0xfab396cb74436798ull, 0xfd9e4e916643eb07ull, 0xff05495819eb2051ull,
    0xffa1ce9c0039a957ull, 0xffdfb3f212e8c4e8ull, 0xfff5e6f9d2314fccull, 0xfffd1f97bc4406a2ull,
    0xffff40fa0088d11dull, 0xffffd2e835e1c57dull, 0xfffff6524386ff1eull, 0xfffffe1db4769da5ull,
    0xffffffac0a1dcb08ull, 0xfffffff428673853ull};
const u64 *gauss_cdf_table() { return kGaussCdf; }
}  // namespace gala
extern "C" uint64_t gala_mix64(uint64_t z) { return gala::mix64(z); }
extern "C" uint64_t gala_rand64(uint64_t seed, uint64_t stream, uint64_t idx, uint64_t attempt) {
    return gala::rand64(seed, stream, idx, attempt);
}
namespace gala {

static int draw_gauss(u64 seed, u64 stream, u64 idx) {
    const u64 u = rand64(seed, stream, idx, 0);
    // the table is increasing: binary search for the number of thresholds <= u
    int lo = 0, hi = 38;
    while (lo < hi) {
        int mid = (lo + hi) / 2;
        if (u >= kGaussCdf[mid]) lo = mid + 1; else hi = mid;
    }
    return lo - kGaussBound;
}
static int draw_ternary(u64 seed, u64 stream, u64 idx) {
    for (u64 t = 0;; ++t) {
        u64 v = rand64(seed, stream, idx, t) >> 62;
        if (v < 3) return (int)v - 1;
    }
}
static u64 lift_signed(int v, u64 q) { return v >= 0 ? (u64)v : q - (u64)(-v); }

// a(X) -> a(X^g) on coefficients
static void substitute_power(const u64 *a, int g, int n, u64 q, u64 *out) {
    for (int i = 0; i < n; ++i) {
        int e = (int)(((long)i * g) % (2 * n));
        if (e < n) out[e] = a[i];
        else out[e - n] = a[i] ? q - a[i] : 0;
    }
}
int galois_element(int n, int swap, int step) {
    long g = 1;
    for (int i = 0; i < step; ++i) g = g * 3 % (2 * n);
    return (int)(swap ? 2 * n - g : g);
}

// run f(i) for i in [0,count) on a few host threads
template <class F>
static void parallel_for(size_t count, F f) {
    unsigned nt = std::min<size_t>(std::max(1u, std::thread::hardware_concurrency()), 16);
    nt = (unsigned)std::min<size_t>(nt, count);
    if (nt <= 1) {
        for (size_t i = 0; i < count; ++i) f(i);
        return;
    }
    std::vector<std::thread> th;
    for (unsigned t = 0; t < nt; ++t)
        th.emplace_back([=]() { for (size_t i = t; i < count; i += nt) f(i); });
    for (auto &x : th) x.join();
}

static int pow2_ceil(int v) {
    int r = 1;
    while (r < v) r <<= 1;
    return r;
}

// slot vector -> weight plaintext in the evaluation domain mod q (centred lift)
static void encode_weight_hat(const gala_ctx *c, const u64 *slots, u64 *out) {
    const int n = c->n;
    std::vector<u64> a(n);
    for (int s = 0; s < n; ++s) a[c->slot_to_idx[s]] = slots[s] % c->p;
    c->ntt_p.inverse(a.data());
    for (int i = 0; i < n; ++i) out[i] = a[i] > c->p / 2 ? c->q - (c->p - a[i]) : a[i];
    c->ntt_q.forward(out);
}

template <class T>
static int upload(T **dst, const std::vector<T> &src) {
    if (src.empty()) { *dst = nullptr; return GALA_OK; }
    if (hipMalloc((void **)dst, src.size() * sizeof(T)) != hipSuccess) return GALA_ENOMEM;
    if (hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return GALA_EHIP;
    return GALA_OK;
}
static int upload_mask_layout(const gala_ctx *c, const MaskLayoutHost &h, MaskLayoutDev *d) {
    int rc;
    if ((rc = upload(&d->row_ptr, h.row_ptr))) return rc;
    if ((rc = upload(&d->row_slots, h.row_slots))) return rc;
    if ((rc = upload(&d->row_rindex, h.row_rindex))) return rc;
    if ((rc = upload(&d->nrows, h.nrows))) return rc;
    if ((rc = upload(&d->is_first, h.is_first))) return rc;
    // the same CSR seen from its entries, with the slot -> transform-position map applied
    const int n = c->n;
    std::vector<int> entry_row((size_t)h.nout * n, -1), entry_idx((size_t)h.nout * n, 0), first_idx((size_t)h.nout * n, 0);
    std::vector<int> slot_rowid((size_t)h.nout * n, -1);
    for (int O = 0; O < h.nout; ++O) {
        const int *rp = h.row_ptr.data() + (size_t)O * (n + 1), *rs = h.row_slots.data() + (size_t)O * n;
        for (int t = 0; t < h.nrows[O]; ++t) {
            if (rp[t + 1] <= rp[t]) continue;
            first_idx[(size_t)O * n + t] = c->slot_to_idx[rs[rp[t]]];
            for (int e = rp[t]; e < rp[t + 1]; ++e) slot_rowid[(size_t)O * n + rs[e]] = t;
            for (int e = rp[t] + 1; e < rp[t + 1]; ++e) {
                entry_row[(size_t)O * n + e] = t;
                entry_idx[(size_t)O * n + e] = c->slot_to_idx[rs[e]];
            }
        }
    }
    if ((rc = upload(&d->entry_row, entry_row))) return rc;
    if ((rc = upload(&d->entry_idx, entry_idx))) return rc;
    if ((rc = upload(&d->slot_rowid, slot_rowid))) return rc;
    return upload(&d->first_idx, first_idx);
}
static void free_mask_layout(MaskLayoutDev *d) {
    hipFree(d->row_ptr); hipFree(d->row_slots); hipFree(d->row_rindex); hipFree(d->nrows); hipFree(d->is_first);
    hipFree(d->entry_row); hipFree(d->entry_idx); hipFree(d->first_idx); hipFree(d->slot_rowid);
}

}  // namespace gala

using namespace gala;

// ===========================================================================
// context
// ===========================================================================
extern "C" int gala_ctx_create(const gala_params *par, gala_ctx **out) {
    if (!par || !out) return GALA_EARG;
    const int n = par->n;
    const u64 q = par->q, p = par->p;
    if (n < 8 || n > kMaxN || (n & (n - 1))) return GALA_EARG;
    if (q < (1ull << 40) || q >= (1ull << 61) || p >= (1ull << 31) || p >= q || p < 3) return GALA_EARG;
    if ((q - 1) % (2 * (u64)n) || (p - 1) % (2 * (u64)n)) return GALA_EARG;
    if (!is_prime_u64(q) || !is_prime_u64(p)) return GALA_EARG;
    if (par->gadget_bits < 1 || par->gadget_bits > 62) return GALA_EARG;
    int ndigits = (bit_length(q - 1) + par->gadget_bits - 1) / par->gadget_bits;
    if (ndigits > kMaxDigits) return GALA_EARG;
    const u64 P = par->special_prime;
    if (P && (P < (1ull << 40) || P >= (1ull << 61) || P == q || (P - 1) % (2 * (u64)n) || !is_prime_u64(P))) return GALA_EARG;

    gala_ctx *c = new (std::nothrow) gala_ctx;
    if (!c) return GALA_ENOMEM;
    c->n = n; c->logn = bit_length((u64)n) - 1;
    c->q = q; c->p = p;
    c->gadget_bits = par->gadget_bits; c->ndigits = ndigits;
    c->qbits = bit_length(q); c->pbits = bit_length(p);
    c->delta = q / p; c->delta_s = shoup_companion(c->delta, q);
    c->zeta = least_primitive_2n_root(p, n);
    c->ntt_q.init(n, q, primitive_2n_root(q, n));
    c->ntt_p.init(n, p, c->zeta);
    if (P) {
        c->special = P;
        c->ntt_P.init(n, P, primitive_2n_root(P, n));
        c->Pq = P % q; c->Pq_s = shoup_companion(c->Pq, q);
        c->Pinv = inv_mod(c->Pq, q); c->Pinv_s = shoup_companion(c->Pinv, q);
    }
    // slot (h,k) is the value at zeta^(+-3^k); the transform puts the value at
    // zeta^(2 r + 1) at index brev(r)
    c->slot_to_idx.resize(n);
    long e = 1;
    for (int k = 0; k < n / 2; ++k) {
        c->slot_to_idx[k] = brev((int)((e - 1) / 2), c->logn);
        c->slot_to_idx[n / 2 + k] = brev((int)((2 * n - e - 1) / 2), c->logn);
        e = e * 3 % (2 * n);
    }
    // device tables; a host without a HIP device still gets a context for the
    // client-side calls (keygen, encode, encrypt, decrypt), every device entry
    // point then fails with GALA_EHIP
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) {
        (void)hipGetLastError();
        c->has_device = false;
        *out = c;
        return GALA_OK;
    }
    if (hipGetDevice(&c->device) != hipSuccess) { delete c; return GALA_EHIP; }
    std::vector<u64> host(8 * (size_t)n);
    const NttHost *hs[2] = {&c->ntt_q, &c->ntt_p};
    for (int k = 0; k < 2; ++k) {
        u64 *base = host.data() + (size_t)k * 4 * n;
        std::copy(hs[k]->tw.begin(), hs[k]->tw.end(), base);
        std::copy(hs[k]->tws.begin(), hs[k]->tws.end(), base + n);
        std::copy(hs[k]->itw.begin(), hs[k]->itw.end(), base + 2 * n);
        std::copy(hs[k]->itws.begin(), hs[k]->itws.end(), base + 3 * n);
    }
    // pass-major twiddle blocks for the n = 2048 kernel: block T (1 <= T < 512) holds the pairs
    // tw[T], tw[2T], tw[2T+1], tw[4T..4T+3] and one unused pair; forward table then inverse table
    std::vector<u64> pairs, pairs_p, pairs_P, hostP;
    if (n == 2048) {
        auto build = [&](const NttHost &h, std::vector<u64> &out) {
            // ... followed, for each direction, by the same pairs level by level with the constant's number before
            // the block's: level c (blocks c .. 2c-1, c = 1, 4, 8, 32, 64, 256) is [e][j] = block (c + j), pair e, so
            // that a wavefront's load of constant e reads neighbouring pairs (2555 pairs per direction)
            static const int kLevels[6] = {1, 4, 8, 32, 64, 256};
            const size_t blocks_words = 2 * 2 * 8 * (size_t)512, level_pairs = 7 * (1 + 4 + 8 + 32 + 64 + 256);
            out.assign(blocks_words + 2 * 2 * level_pairs, 0);
            for (int inv = 0; inv < 2; ++inv) {
                const std::vector<u64> &w = inv ? h.itw : h.tw, &ws = inv ? h.itws : h.tws;
                u64 *base = out.data() + (size_t)inv * 2 * 8 * 512;
                for (int T = 1; T < 512; ++T) {
                    const int idx[7] = {T, 2 * T, 2 * T + 1, 4 * T, 4 * T + 1, 4 * T + 2, 4 * T + 3};
                    for (int e = 0; e < 7; ++e) {
                        base[2 * (8 * T + e)] = w[idx[e]];
                        base[2 * (8 * T + e) + 1] = ws[idx[e]];
                    }
                }
                u64 *lev = out.data() + blocks_words + (size_t)inv * 2 * level_pairs;
                for (int L = 0; L < 6; ++L) {
                    const int cnt = kLevels[L];
                    for (int e = 0; e < 7; ++e)
                        for (int j = 0; j < cnt; ++j) {
                            lev[2 * ((size_t)e * cnt + j)] = base[2 * (8 * (cnt + j) + e)];
                            lev[2 * ((size_t)e * cnt + j) + 1] = base[2 * (8 * (cnt + j) + e) + 1];
                        }
                    lev += 2 * 7 * (size_t)cnt;
                }
            }
        };
        build(c->ntt_q, pairs);
        build(c->ntt_p, pairs_p);
        if (P) build(c->ntt_P, pairs_P);
    }
    if (P) {
        hostP.resize(4 * (size_t)n);
        std::copy(c->ntt_P.tw.begin(), c->ntt_P.tw.end(), hostP.begin());
        std::copy(c->ntt_P.tws.begin(), c->ntt_P.tws.end(), hostP.begin() + n);
        std::copy(c->ntt_P.itw.begin(), c->ntt_P.itw.end(), hostP.begin() + 2 * n);
        std::copy(c->ntt_P.itws.begin(), c->ntt_P.itws.end(), hostP.begin() + 3 * n);
    }
    if (upload(&c->d_tables, host) || upload(&c->d_slot_to_idx, c->slot_to_idx) ||
        upload(&c->d_tw2, pairs) || upload(&c->d_tw2p, pairs_p) || upload(&c->d_tablesP, hostP) ||
        upload(&c->d_tw2P, pairs_P)) {
        gala_ctx_destroy(c);
        return GALA_EHIP;
    }
    if (P) {
        const u64 *base = c->d_tablesP;
        c->dev_P.tw = base; c->dev_P.tws = base + n; c->dev_P.itw = base + 2 * n; c->dev_P.itws = base + 3 * n;
        c->dev_P.ninv = c->ntt_P.ninv; c->dev_P.ninvs = c->ntt_P.ninvs;
        c->dev_P.itw1n = c->ntt_P.itw1n; c->dev_P.itw1ns = c->ntt_P.itw1ns;
        c->dev_P.mod = c->ntt_P.mod;
    }
    NttDev *dv[2] = {&c->dev_q, &c->dev_p};
    for (int k = 0; k < 2; ++k) {
        const u64 *base = c->d_tables + (size_t)k * 4 * n;
        dv[k]->tw = base; dv[k]->tws = base + n; dv[k]->itw = base + 2 * n; dv[k]->itws = base + 3 * n;
        dv[k]->ninv = hs[k]->ninv; dv[k]->ninvs = hs[k]->ninvs;
        dv[k]->itw1n = hs[k]->itw1n; dv[k]->itw1ns = hs[k]->itw1ns;
        dv[k]->mod = hs[k]->mod;
    }
    // address of the fixed scratch array of gala_he_fc_static on this device (resolved once per device)
    if (static_scratch_init() != GALA_OK) {
        gala_ctx_destroy(c);
        return GALA_EHIP;
    }
    c->has_device = true;
    *out = c;
    return GALA_OK;
}
extern "C" void gala_ctx_destroy(gala_ctx *c) {
    if (!c) return;
    if (c->has_device) {
        for (void *e : c->prof_events) (void)hipEventDestroy((hipEvent_t)e);
        hipFree(c->d_tables);
        hipFree(c->d_slot_to_idx);
        hipFree(c->d_tw2);
        hipFree(c->d_tw2p);
        hipFree(c->d_tablesP);
        hipFree(c->d_tw2P);
    }
    delete c;
}
extern "C" int gala_ctx_ndigits(const gala_ctx *c) { return c ? c->ndigits : GALA_EARG; }
extern "C" uint64_t gala_ctx_delta(const gala_ctx *c) { return c ? c->delta : 0; }
extern "C" const uint64_t *gala_gauss_cdf(void) { return gauss_cdf_table(); }

// ===========================================================================
// keys
// ===========================================================================
extern "C" int gala_keygen(const gala_ctx *c, uint64_t seed, gala_sk **out) {
    if (!c || !out) return GALA_EARG;
    gala_sk *sk = new (std::nothrow) gala_sk;
    if (!sk) return GALA_ENOMEM;
    sk->s.resize(c->n);
    for (int i = 0; i < c->n; ++i) sk->s[i] = lift_signed(draw_ternary(seed, kStreamSk, (u64)i), c->q);
    sk->s_hat = sk->s;
    c->ntt_q.forward(sk->s_hat.data());
    if (c->has_device && upload(&sk->d_s_hat, sk->s_hat)) {
        gala_sk_destroy(sk);
        return GALA_EHIP;
    }
    *out = sk;
    return GALA_OK;
}
extern "C" void gala_sk_destroy(gala_sk *sk) {
    if (!sk) return;
    if (sk->d_s_hat) hipFree(sk->d_s_hat);
    delete sk;
}
extern "C" int gala_sk_export(const gala_ctx *c, const gala_sk *sk, uint64_t *s_host) {
    if (!c || !sk || !s_host) return GALA_EARG;
    std::memcpy(s_host, sk->s.data(), sizeof(u64) * c->n);
    return GALA_OK;
}

extern "C" int gala_galois_keygen(gala_ctx *c, const gala_sk *sk, const gala_rot *rots, int nrots, uint64_t seed,
                                  gala_gk **out) {
    if (!c || !sk || !out || nrots < 0 || (nrots && !rots)) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    const int n = c->n, L = c->ndigits;
    gala_gk *gk = new (std::nothrow) gala_gk;
    if (!gk) return GALA_ENOMEM;
    gk->ctx = c; gk->n = n; gk->ndigits = L; gk->polys = c->key_polys();
    for (int i = 0; i < nrots; ++i) {
        if (rots[i].step < 0 || rots[i].step >= n / 2 || (rots[i].swap & ~1)) { delete gk; return GALA_EARG; }
        int g = galois_element(n, rots[i].swap, rots[i].step);
        if (g == 1 || gk->index_of.count(g)) continue;
        gk->index_of[g] = (int)gk->elements.size();
        gk->elements.push_back(g);
    }
    const size_t nkeys = gk->elements.size(), kw = gk->key_words();
    {
        std::vector<int> iota(nkeys), one(1, 1), zeros(std::max<size_t>(nkeys, 1), 0);
        for (size_t k = 0; k < nkeys; ++k) iota[k] = (int)k;
        if (upload(&gk->d_elements, gk->elements) || upload(&gk->d_iota, iota) || upload(&gk->d_one, one) ||
            upload(&gk->d_zeros, zeros)) {
            gala_gk_destroy(gk);
            return GALA_EHIP;
        }
    }
    *out = gk;
    if (!nkeys) return GALA_OK;
    // Coefficient-domain samples per digit: [1] <- a_j, [0] <- e_j + B^j s(X^g) modulo q.  With a special prime P
    // the hidden value is P B^j s(X^g) (zero modulo P) and two more polynomials follow: [2] <- e_j, [3] <- a_j
    // modulo P, the residues of a_j drawn independently.
    const u64 q = c->q, P = c->special;
    const int polys = gk->polys;
    std::vector<u64> host, sP_hat;
    try { host.resize(nkeys * kw); } catch (...) { gala_gk_destroy(gk); *out = nullptr; return GALA_ENOMEM; }
    parallel_for(nkeys, [&](size_t k) {
        const int g = gk->elements[k];
        std::vector<u64> sg(n);
        substitute_power(sk->s.data(), g, n, q, sg.data());
        u64 Bj = P ? c->Pq : 1;
        const u64 B = (1ull << c->gadget_bits) % q;
        for (int j = 0; j < L; ++j) {
            u64 *t = host.data() + k * kw + (size_t)(polys * j) * n, *a = t + n;
            const u64 base = ((u64)g << 32) + ((u64)j << 16);
            for (int i = 0; i < n; ++i) {
                a[i] = draw_uniform(q, c->qbits, seed, kStreamKskA, base + i);
                const int e = draw_gauss(seed, kStreamKskE, base + i);
                t[i] = add_mod(lift_signed(e, q), mulmod_slow(Bj, sg[i], q), q);
                if (P) {
                    t[2 * n + i] = lift_signed(e, P);
                    t[3 * n + i] = draw_uniform(P, bit_length(P), seed, kStreamKskAP, base + i);
                }
            }
            Bj = mulmod_slow(Bj, B, q);
        }
    });
    if (P) {   // the ternary secret modulo P, evaluation domain
        sP_hat.resize(n);
        for (int i = 0; i < n; ++i) sP_hat[i] = sk->s[i] == 0 ? 0 : (sk->s[i] == 1 ? 1 : P - 1);
        c->ntt_P.forward(sP_hat.data());
    }
    u64 *d_s = nullptr, *d_sP = nullptr;
    int rc = GALA_OK;
    if (hipMalloc((void **)&gk->d_keys, nkeys * kw * sizeof(u64)) != hipSuccess ||
        hipMalloc((void **)&d_s, n * sizeof(u64)) != hipSuccess || (P && hipMalloc((void **)&d_sP, n * sizeof(u64)) != hipSuccess))
        rc = GALA_ENOMEM;
    if (!rc && (hipMemcpy(gk->d_keys, host.data(), nkeys * kw * sizeof(u64), hipMemcpyHostToDevice) != hipSuccess ||
                hipMemcpy(d_s, sk->s_hat.data(), n * sizeof(u64), hipMemcpyHostToDevice) != hipSuccess ||
                (P && hipMemcpy(d_sP, sP_hat.data(), n * sizeof(u64), hipMemcpyHostToDevice) != hipSuccess)))
        rc = GALA_EHIP;
    // to the evaluation domain, then b_hat = t_hat - a_hat * s_hat in place
    if (!P) {
        if (!rc && launch_ntt(c, nullptr, gk->d_keys, gk->d_keys, nkeys * L * 2, 0)) rc = GALA_EHIP;
        if (!rc && launch_key_finish(c, nullptr, gk->d_keys, d_s, nkeys * L, c->dev_q.mod)) rc = GALA_EHIP;
    } else {
        for (size_t d = 0; d < nkeys * L && !rc; ++d) {   // per digit: one pair modulo q, one modulo P
            u64 *pq = gk->d_keys + d * 4 * n, *pP = pq + 2 * n;
            if (launch_ntt_mod(c, nullptr, pq, pq, 2, 0, c->dev_q) || launch_key_finish(c, nullptr, pq, d_s, 1, c->dev_q.mod) ||
                launch_ntt_mod(c, nullptr, pP, pP, 2, 0, c->dev_P) || launch_key_finish(c, nullptr, pP, d_sP, 1, c->dev_P.mod))
                rc = GALA_EHIP;
        }
    }
    if (!rc && uses_fast_perm(c)) {
        if (hipMalloc((void **)&gk->d_keys2, 2 * nkeys * kw * sizeof(u64)) != hipSuccess) rc = GALA_ENOMEM;
        if (!rc && launch_pair_pack(c, nullptr, gk->d_keys, gk->d_keys2, nkeys * kw, polys)) rc = GALA_EHIP;
    }
    if (!rc && hipDeviceSynchronize() != hipSuccess) rc = GALA_EHIP;
    hipFree(d_s);
    hipFree(d_sP);
    if (rc) { gala_gk_destroy(gk); *out = nullptr; }
    return rc;
}
extern "C" void gala_gk_destroy(gala_gk *gk) {
    if (!gk) return;
    hipFree(gk->d_keys); hipFree(gk->d_keys2); hipFree(gk->d_elements); hipFree(gk->d_iota); hipFree(gk->d_one); hipFree(gk->d_zeros);
    delete gk;
}
extern "C" int gala_gk_export(gala_ctx *c, const gala_gk *gk, gala_rot rot, uint64_t *ksk_host) {
    if (!c || !gk || !ksk_host || rot.step < 0 || rot.step >= c->n / 2) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    auto it = gk->index_of.find(galois_element(c->n, rot.swap, rot.step));
    if (it == gk->index_of.end()) return GALA_ENOKEY;
    const size_t kw = gk->key_words();
    u64 *tmp = nullptr;
    if (hipMalloc((void **)&tmp, kw * sizeof(u64)) != hipSuccess) return GALA_ENOMEM;
    int rc = GALA_OK;
    if (gk->polys == 2) {
        if (launch_ntt(c, nullptr, gk->d_keys + it->second * kw, tmp, (size_t)gk->ndigits * 2, 1)) rc = GALA_EHIP;
    } else {
        for (int j = 0; j < gk->ndigits && !rc; ++j) {
            const u64 *src = gk->d_keys + it->second * kw + (size_t)j * 4 * c->n;
            u64 *dst = tmp + (size_t)j * 4 * c->n;
            if (launch_ntt_mod(c, nullptr, src, dst, 2, 1, c->dev_q) ||
                launch_ntt_mod(c, nullptr, src + 2 * c->n, dst + 2 * c->n, 2, 1, c->dev_P))
                rc = GALA_EHIP;
        }
    }
    if (!rc && hipMemcpy(ksk_host, tmp, kw * sizeof(u64), hipMemcpyDeviceToHost) != hipSuccess) rc = GALA_EHIP;
    hipFree(tmp);
    return rc;
}

// ===========================================================================
// encoding, encryption, decryption (host)
// ===========================================================================
extern "C" int gala_encode(const gala_ctx *c, const uint64_t *slots, uint64_t *poly_p) {
    if (!c || !slots || !poly_p) return GALA_EARG;
    std::vector<u64> a(c->n);
    for (int s = 0; s < c->n; ++s) a[c->slot_to_idx[s]] = slots[s] % c->p;
    c->ntt_p.inverse(a.data());
    std::memcpy(poly_p, a.data(), sizeof(u64) * c->n);
    return GALA_OK;
}
extern "C" int gala_decode(const gala_ctx *c, const uint64_t *poly_p, uint64_t *slots) {
    if (!c || !slots || !poly_p) return GALA_EARG;
    std::vector<u64> a(c->n);
    for (int i = 0; i < c->n; ++i) a[i] = poly_p[i] % c->p;
    c->ntt_p.forward(a.data());
    for (int s = 0; s < c->n; ++s) slots[s] = a[c->slot_to_idx[s]];
    return GALA_OK;
}
extern "C" int gala_encrypt(const gala_ctx *c, const gala_sk *sk, const uint64_t *slots, uint64_t seed,
                            uint64_t *ct) {
    if (!c || !sk || !slots || !ct) return GALA_EARG;
    const int n = c->n;
    const u64 q = c->q;
    std::vector<u64> m(n), as(n);
    gala_encode(c, slots, m.data());
    u64 *c0 = ct, *c1 = ct + n;
    for (int i = 0; i < n; ++i) as[i] = c1[i] = draw_uniform(q, c->qbits, seed, kStreamCtA, (u64)i);
    c->ntt_q.forward(as.data());
    for (int i = 0; i < n; ++i) as[i] = mul_mod(as[i], sk->s_hat[i], c->ntt_q.mod);
    c->ntt_q.inverse(as.data());
    for (int i = 0; i < n; ++i) {
        u64 e = lift_signed(draw_gauss(seed, kStreamCtE, (u64)i), q);
        u64 dm = mul_shoup(m[i], c->delta, c->delta_s, q);
        c0[i] = add_mod(sub_mod(e, as[i], q), dm, q);
    }
    return GALA_OK;
}
extern "C" int gala_decrypt(const gala_ctx *c, const gala_sk *sk, const uint64_t *ct, uint64_t *slots) {
    if (!c || !sk || !slots || !ct) return GALA_EARG;
    const int n = c->n;
    const u64 q = c->q, p = c->p;
    std::vector<u64> v(ct + n, ct + 2 * n), m(n);
    c->ntt_q.forward(v.data());
    for (int i = 0; i < n; ++i) v[i] = mul_mod(v[i], sk->s_hat[i], c->ntt_q.mod);
    c->ntt_q.inverse(v.data());
    for (int i = 0; i < n; ++i) {
        u64 ph = add_mod(v[i], ct[i] % q, q);
        m[i] = (u64)((((u128)p * ph) + q / 2) / q) % p;
    }
    return gala_decode(c, m.data(), slots);
}

// ===========================================================================
// he_fc plan: row-wise weight encoding (Sec. III-A(3))
// ===========================================================================
namespace {
// row of W whose partial sum sits in slot (h,k) after all rotations; -1 if none
int fc_slot_row(const gala_fc_plan *pl, int h, int k) {
    const int n = pl->ctx->n, half = n / 2;
    if (pl->big) return k % pl->nop;
    const int copy = h * (half / pl->nip) + k / pl->nip, j = k % pl->nip;
    if ((long)pl->nip * pl->nop < n && copy >= pl->nop) return -1;
    int r = (j - copy * pl->G) % pl->nop;
    return r < 0 ? r + pl->nop : r;
}
int fc_slot_col(const gala_fc_plan *pl, int h, int k) {
    return pl->big ? h * (pl->ctx->n / 2) + k : k % pl->nip;
}
}  // namespace

namespace {
// Encoded weights of an FC plan, built on the device: W and the slot -> row table go up once, one kernel writes the G
// slot vectors and the plaintext encoder takes them to the evaluation domain (centred lift, as ScMult expects).
// *d_w receives G x n words.
int encode_fc_weights_on_device(const gala_ctx *c, const uint64_t *W, int n_o, int n_i, int nip, bool big, bool rotate_output,
                                const std::vector<int> &slot_row_padded, int G, u64 **d_w) {
    const int n = c->n;
    u64 *d_W = nullptr, *d_slots = nullptr;
    int *d_row = nullptr;
    int rc = GALA_OK;
    const size_t words = (size_t)n_o * n_i;
    if (hipMalloc((void **)&d_W, words * sizeof(u64)) != hipSuccess ||
        hipMalloc((void **)&d_slots, (size_t)G * n * sizeof(u64)) != hipSuccess ||
        hipMalloc((void **)d_w, (size_t)G * n * sizeof(u64)) != hipSuccess)
        rc = GALA_ENOMEM;
    if (!rc) rc = upload(&d_row, slot_row_padded);
    if (!rc && hipMemcpy(d_W, W, words * sizeof(u64), hipMemcpyHostToDevice) != hipSuccess) rc = GALA_EHIP;
    const FcGeom geo{n, n_o, n_i, nip, big ? 1 : 0, rotate_output ? 1 : 0, c->p};
    if (!rc && (launch_fc_weight_slots(c, nullptr, d_W, geo, d_row, G, d_slots) ||
                launch_encode_plain(c, nullptr, d_slots, G, 0, *d_w) || hipDeviceSynchronize() != hipSuccess))
        rc = GALA_EHIP;
    hipFree(d_W); hipFree(d_slots); hipFree(d_row);
    return rc;
}
}  // namespace

extern "C" int gala_fc_plan_create(gala_ctx *c, const uint64_t *W, int n_o, int n_i, gala_fc_plan **out) {
    if (!c || !W || !out || n_o < 1 || n_i < 1) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    const int n = c->n, half = n / 2;
    gala_fc_plan *pl = new (std::nothrow) gala_fc_plan;
    if (!pl) return GALA_ENOMEM;
    pl->ctx = c; pl->n_o = n_o; pl->n_i = n_i;
    pl->nop = pow2_ceil(n_o); pl->nip = pow2_ceil(n_i);
    if (pl->nip > n || pl->nop > n) { delete pl; return GALA_ESHAPE; }
    pl->big = pl->nip == n;
    if (pl->big) {
        if (pl->nop > half) { delete pl; return GALA_ESHAPE; }
        pl->G = pl->nop;
    } else {
        long prod = (long)pl->nip * pl->nop;
        pl->G = prod >= n ? (int)(prod / n) : 1;
    }
    const int G = pl->G;
    pl->slot_row.resize(n);
    for (int s = 0; s < n; ++s) {
        int row = fc_slot_row(pl, s / half, s % half);
        pl->slot_row[s] = row < n_o ? row : -1;
    }
    pl->gal.resize(G);
    for (int g = 0; g < G; ++g) pl->gal[g] = galois_element(n, 0, g);
    // encoded weights: before the left rotation by g, slot (h,k) holds W[row(h,k-g)][col(h,k)]
    std::vector<int> row_padded(n);
    for (int s = 0; s < n; ++s) row_padded[s] = fc_slot_row(pl, s / half, s % half);
    const size_t wsize = (size_t)G * n;
    {
        const int erc = encode_fc_weights_on_device(c, W, n_o, n_i, pl->nip, pl->big, true, row_padded, G, &pl->d_w);
        if (erc) { gala_fc_plan_destroy(pl); return erc; }
    }
    // mask layout: one output ciphertext, rows = real outputs
    MaskLayoutHost &mh = pl->mask_h;
    mh.nout = 1;
    mh.nrows = {n_o};
    mh.row_ptr.assign(n + 1, 0);
    mh.row_slots.assign(n, 0);
    mh.row_rindex.assign(n, 0);
    mh.is_first.assign(n, 0);
    std::vector<std::vector<int>> members(n_o);
    for (int s = 0; s < n; ++s)
        if (pl->slot_row[s] >= 0) members[pl->slot_row[s]].push_back(s);
    int pos = 0;
    for (int t = 0; t < n_o; ++t) {
        mh.row_ptr[t] = pos;
        mh.row_rindex[t] = t;
        for (int s : members[t]) mh.row_slots[pos++] = s;
        if (!members[t].empty()) mh.is_first[members[t][0]] = 1;
    }
    for (int t = n_o; t <= n; ++t) mh.row_ptr[t] = pos;
    std::vector<int> key_idx(G, -1);
    int rc = GALA_OK;
    if (!rc && uses_fast_perm(c)) {
        // pairs in natural order, then once more in the order the Perm kernel's threads own them
        if (hipMalloc((void **)&pl->d_w2, 4 * wsize * sizeof(u64)) != hipSuccess) rc = GALA_ENOMEM;
        if (!rc && (launch_pair_pack(c, nullptr, pl->d_w, pl->d_w2, wsize, 2) ||
                    launch_owner_order_2048(nullptr, pl->d_w2, pl->d_w2 + 2 * wsize, (size_t)G) ||
                    hipDeviceSynchronize() != hipSuccess))
            rc = GALA_EHIP;
    }
    if (!rc) rc = upload(&pl->d_gal, pl->gal);
    if (!rc) rc = upload(&pl->d_key_idx, key_idx);
    if (!rc) rc = upload_mask_layout(c, mh, &pl->mask_d);
    if (rc) { gala_fc_plan_destroy(pl); return rc; }
    *out = pl;
    return GALA_OK;
}
extern "C" void gala_fc_plan_destroy(gala_fc_plan *pl) {
    if (!pl) return;
    hipFree(pl->d_w); hipFree(pl->d_w2); hipFree(pl->d_gal); hipFree(pl->d_key_idx);
    free_mask_layout(&pl->mask_d);
    delete pl;
}
extern "C" int gala_fc_plan_G(const gala_fc_plan *pl) { return pl ? pl->G : GALA_EARG; }
extern "C" int gala_fc_plan_rotations(const gala_fc_plan *pl, gala_rot *rots, int *nrots) {
    if (!pl || !nrots) return GALA_EARG;
    *nrots = pl->G - 1;
    if (rots)
        for (int g = 1; g < pl->G; ++g) rots[g - 1] = gala_rot{0, g};
    return GALA_OK;
}
extern "C" int gala_fc_plan_bind(gala_fc_plan *pl, const gala_gk *gk) {
    if (!pl || !gk || gk->ctx != pl->ctx) return GALA_EARG;
    std::vector<int> idx(pl->G, -1);
    for (int g = 1; g < pl->G; ++g) {
        auto it = gk->index_of.find(pl->gal[g]);
        if (it == gk->index_of.end()) return GALA_ENOKEY;
        idx[g] = it->second;
    }
    if (hipMemcpy(pl->d_key_idx, idx.data(), sizeof(int) * pl->G, hipMemcpyHostToDevice) != hipSuccess) return GALA_EHIP;
    pl->bound = gk;
    return GALA_OK;
}
extern "C" int gala_fc_pack_input(const gala_fc_plan *pl, const uint64_t *x, uint64_t *slots) {
    if (!pl || !x || !slots) return GALA_EARG;
    const int half = pl->ctx->n / 2;
    for (int h = 0; h < 2; ++h)
        for (int k = 0; k < half; ++k) {
            int col = fc_slot_col(pl, h, k);
            slots[h * half + k] = col < pl->n_i ? x[col] % pl->ctx->p : 0;
        }
    return GALA_OK;
}
extern "C" int gala_fc_unpack_share(const gala_fc_plan *pl, const uint64_t *slots, uint64_t *out) {
    if (!pl || !out || !slots) return GALA_EARG;
    const u64 p = pl->ctx->p;
    for (int t = 0; t < pl->n_o; ++t) out[t] = 0;
    for (int s = 0; s < pl->ctx->n; ++s)
        if (pl->slot_row[s] >= 0) out[pl->slot_row[s]] = add_mod(out[pl->slot_row[s]], slots[s] % p, p);
    return GALA_OK;
}

// ===========================================================================
// hybrid FC plan (Sec. III-A(2)): the comparison schedule, on the same operations
// ===========================================================================
// Layout on the 2 x n/2 slot torus.  n_i <= n/2: every half-row holds n/(2 n_i) copies of x; copy c owns the
// R = max(1, n_i n_o / n) output rows c*R .. c*R+R-1 and slot j of the copy collects row c*R + (j mod R); the G = R
// diagonal vectors w_g[(h,k)] = W[row(h,k)][(j+g) mod n_i] multiply the input rotated left by g, and rotate-and-sum
// steps by n_i/2, .., R finish row c*R + j in slot j < R of copy c.  n_i = n: half h holds x[h*n/2 ..], slot (h,k)
// collects row k mod n_o over the columns of its half (G = n_o), steps by n/4, .., n_o and one row swap.
namespace {
int hy_slot_row(const gala_fc_hybrid_plan *pl, int h, int k) {
    const int n = pl->ctx->n, half = n / 2;
    if (pl->big) return k % pl->nop;
    const int copy = h * (half / pl->nip) + k / pl->nip, j = k % pl->nip;
    if ((long)pl->nip * pl->nop < n && copy >= pl->nop) return -1;
    return copy * pl->R + j % pl->R;
}
}  // namespace
extern "C" int gala_fc_hybrid_plan_create(gala_ctx *c, const uint64_t *W, int n_o, int n_i, gala_fc_hybrid_plan **out) {
    if (!c || !W || !out || n_o < 1 || n_i < 1) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    const int n = c->n, half = n / 2;
    gala_fc_hybrid_plan *pl = new (std::nothrow) gala_fc_hybrid_plan;
    if (!pl) return GALA_ENOMEM;
    pl->ctx = c; pl->n_o = n_o; pl->n_i = n_i;
    pl->nop = pow2_ceil(n_o); pl->nip = pow2_ceil(n_i);
    if (pl->nip > n || pl->nop > n) { delete pl; return GALA_ESHAPE; }
    pl->big = pl->nip == n;
    if (pl->big) {
        if (pl->nop > half) { delete pl; return GALA_ESHAPE; }
        pl->R = pl->nop;
    } else {
        const long prod = (long)pl->nip * pl->nop;
        pl->R = prod >= n ? (int)(prod / n) : 1;
    }
    const int G = pl->G = pl->R;
    pl->in_gal.resize(G);
    for (int g = 0; g < G; ++g) pl->in_gal[g] = galois_element(n, 0, g);
    for (int rho = (pl->big ? half : pl->nip) / 2; rho >= pl->R; rho /= 2) pl->ras_gal.push_back(galois_element(n, 0, rho));
    if (pl->big) pl->ras_gal.push_back(galois_element(n, 1, 0));
    pl->result_slot.resize(n_o);
    for (int t = 0; t < n_o; ++t) {
        if (pl->big) { pl->result_slot[t] = t; continue; }
        const int copy = t / pl->R, per_row = half / pl->nip;
        pl->result_slot[t] = (copy / per_row) * half + (copy % per_row) * pl->nip + t % pl->R;
    }
    std::vector<int> row_padded(n);
    for (int s = 0; s < n; ++s) row_padded[s] = hy_slot_row(pl, s / half, s % half);
    {
        const int erc = encode_fc_weights_on_device(c, W, n_o, n_i, pl->nip, pl->big, false, row_padded, G, &pl->d_w);
        if (erc) { gala_fc_hybrid_plan_destroy(pl); return erc; }
    }
    // mask layout: every real output is a row of one slot (its result slot); all other slots are drawn
    MaskLayoutHost &mh = pl->mask_h;
    mh.nout = 1;
    mh.nrows = {n_o};
    mh.row_ptr.assign(n + 1, 0);
    mh.row_slots.assign(n, 0);
    mh.row_rindex.assign(n, 0);
    mh.is_first.assign(n, 0);
    for (int t = 0; t < n_o; ++t) {
        mh.row_ptr[t] = t;
        mh.row_slots[t] = pl->result_slot[t];
        mh.row_rindex[t] = t;
        mh.is_first[pl->result_slot[t]] = 1;
    }
    for (int t = n_o; t <= n; ++t) mh.row_ptr[t] = n_o;
    const int steps = (int)pl->ras_gal.size();
    std::vector<int> zeros(G, 0), in_key(G, -1), ras_gal(2 * std::max(steps, 1), 1), ras_key(2 * std::max(steps, 1), -1);
    for (int k = 0; k < steps; ++k) ras_gal[2 * k + 1] = pl->ras_gal[k];
    int rc = upload(&pl->d_in_ct, zeros);
    if (!rc) rc = upload(&pl->d_in_gal, pl->in_gal);
    if (!rc) rc = upload(&pl->d_in_key, in_key);
    if (!rc) rc = upload(&pl->d_ras_gal, ras_gal);
    if (!rc) rc = upload(&pl->d_ras_key, ras_key);
    if (!rc) rc = upload_mask_layout(c, mh, &pl->mask_d);
    if (rc) { gala_fc_hybrid_plan_destroy(pl); return rc; }
    *out = pl;
    return GALA_OK;
}
extern "C" void gala_fc_hybrid_plan_destroy(gala_fc_hybrid_plan *pl) {
    if (!pl) return;
    hipFree(pl->d_w); hipFree(pl->d_in_ct); hipFree(pl->d_in_gal); hipFree(pl->d_in_key);
    hipFree(pl->d_ras_gal); hipFree(pl->d_ras_key);
    free_mask_layout(&pl->mask_d);
    delete pl;
}
extern "C" int gala_fc_hybrid_plan_G(const gala_fc_hybrid_plan *pl) { return pl ? pl->G : GALA_EARG; }
extern "C" int gala_fc_hybrid_plan_steps(const gala_fc_hybrid_plan *pl) { return pl ? (int)pl->ras_gal.size() : GALA_EARG; }
extern "C" int gala_fc_hybrid_pack_input(const gala_fc_hybrid_plan *pl, const uint64_t *x, uint64_t *slots) {
    if (!pl || !x || !slots) return GALA_EARG;
    const int half = pl->ctx->n / 2;
    for (int h = 0; h < 2; ++h)
        for (int k = 0; k < half; ++k) {
            const int col = pl->big ? h * half + k : k % pl->nip;
            slots[h * half + k] = col < pl->n_i ? x[col] % pl->ctx->p : 0;
        }
    return GALA_OK;
}
extern "C" int gala_fc_hybrid_unpack(const gala_fc_hybrid_plan *pl, const uint64_t *slots, uint64_t *out) {
    if (!pl || !slots || !out) return GALA_EARG;
    for (int t = 0; t < pl->n_o; ++t) out[t] = slots[pl->result_slot[t]] % pl->ctx->p;
    return GALA_OK;
}

// ===========================================================================
// he_conv plan: kernel grouping (Sec. III-B(3))
// ===========================================================================
extern "C" int gala_conv_plan_create(gala_ctx *c, const uint64_t *K, int c_o, int c_i, int k_h, int k_w, int u_h,
                                     int u_w, gala_conv_plan **out) {
    if (!c || !K || !out || c_o < 1 || c_i < 1 || k_h < 1 || k_w < 1 || u_h < 1 || u_w < 1) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    const int n = c->n, half = n / 2;
    if (!(k_h & 1) || !(k_w & 1)) return GALA_ESHAPE;
    if ((long)u_h * u_w > half) return GALA_ESHAPE;
    gala_conv_plan *pl = new (std::nothrow) gala_conv_plan;
    if (!pl) return GALA_ENOMEM;
    pl->ctx = c; pl->c_o = c_o; pl->c_i = c_i; pl->k_h = k_h; pl->k_w = k_w; pl->u_h = u_h; pl->u_w = u_w;
    pl->T = pow2_ceil(u_h * u_w);
    pl->cn = n / pl->T; pl->hpos = pl->cn / 2;
    pl->nin = (c_i + pl->cn - 1) / pl->cn; pl->nout = (c_o + pl->cn - 1) / pl->cn;
    pl->ntap = k_h * k_w; pl->centre = (k_h / 2) * k_w + k_w / 2;
    const int T = pl->T, cn = pl->cn, hpos = pl->hpos, nin = pl->nin, nout = pl->nout, ntap = pl->ntap;
    // taps: the input shifted so that pixel (y+dy, x+dx) lands on (y,x): left rotation by dy*u_w+dx
    pl->tap_gal.resize(ntap);
    for (int tap = 0; tap < ntap; ++tap) {
        int off = (tap / k_w - k_h / 2) * u_w + (tap % k_w - k_w / 2);
        pl->tap_gal[tap] = galois_element(n, 0, ((off % half) + half) % half);
    }
    // kernel orders: group element (s,t) moves channel position (h,kappa) <- (h^s, kappa+t)
    pl->grp_gal.resize(cn);
    for (int gam = 0; gam < cn; ++gam) pl->grp_gal[gam] = galois_element(n, gam / hpos, (gam % hpos) * T);

    // Terms: an (input ciphertext, tap) pair takes part when some kernel value it carries is non-zero mod p and the
    // tap reaches inside the image; every (input channel, output channel) pair sits in exactly one kernel order, so
    // this is the set of pairs with a non-zero encoded kernel.  An all-zero layer keeps one term.
    for (int tap = 0; tap < ntap; ++tap)
        for (int I = 0; I < nin; ++I) {
            const int dy = tap / k_w - k_h / 2, dx = tap % k_w - k_w / 2;
            bool active = false;
            if (std::abs(dy) < u_h && std::abs(dx) < u_w)
                for (int in_ch = I * cn; in_ch < std::min(c_i, (I + 1) * cn) && !active; ++in_ch)
                    for (int out_ch = 0; out_ch < c_o && !active; ++out_ch)
                        active = K[((size_t)out_ch * c_i + in_ch) * ntap + tap] % c->p != 0;
            if (active) { pl->term_ct.push_back(I); pl->term_tap.push_back(tap); }
        }
    if (pl->term_ct.empty()) { pl->term_ct.push_back(0); pl->term_tap.push_back(pl->centre); }
    const int nterm = pl->nterm = (int)pl->term_ct.size();
    const size_t npoly = (size_t)nout * cn * nterm;
    // "encode" on the device: the slot vectors of a few thousand kernels at a time are written from K by one
    // kernel and taken to the evaluation domain by the plaintext encoder (centred lift, as ScMult expects)
    {
        const ConvGeom geo{c_o, c_i, k_h, k_w, u_h, u_w, T, cn, hpos, nterm, n, c->p};
        const size_t chunk = std::min<size_t>(npoly, 4096);
        u64 *d_K = nullptr, *d_slots = nullptr;
        int *d_tct = nullptr, *d_ttap = nullptr;
        int rc = GALA_OK;
        const size_t kwords = (size_t)c_o * c_i * k_h * k_w;
        if (hipMalloc((void **)&d_K, kwords * sizeof(u64)) != hipSuccess ||
            hipMalloc((void **)&d_slots, chunk * n * sizeof(u64)) != hipSuccess ||
            hipMalloc((void **)&pl->d_w, npoly * n * sizeof(u64)) != hipSuccess)
            rc = GALA_ENOMEM;
        if (!rc) rc = upload(&d_tct, pl->term_ct);
        if (!rc) rc = upload(&d_ttap, pl->term_tap);
        if (!rc && hipMemcpy(d_K, K, kwords * sizeof(u64), hipMemcpyHostToDevice) != hipSuccess) rc = GALA_EHIP;
        for (size_t first = 0; !rc && first < npoly; first += chunk) {
            const size_t cnt = std::min(chunk, npoly - first);
            if (launch_conv_weight_slots(c, nullptr, d_K, geo, d_tct, d_ttap, first, cnt, d_slots) ||
                launch_encode_plain(c, nullptr, d_slots, (int)cnt, 0, pl->d_w + first * n))
                rc = GALA_EHIP;
        }
        if (!rc && hipDeviceSynchronize() != hipSuccess) rc = GALA_EHIP;
        hipFree(d_K); hipFree(d_slots); hipFree(d_tct); hipFree(d_ttap);
        if (rc) { gala_conv_plan_destroy(pl); return rc; }
    }
    // mask layout: every real output is a row of its own
    MaskLayoutHost &mh = pl->mask_h;
    mh.nout = nout;
    mh.nrows.assign(nout, 0);
    mh.row_ptr.assign((size_t)nout * (n + 1), 0);
    mh.row_slots.assign((size_t)nout * n, 0);
    mh.row_rindex.assign((size_t)nout * n, 0);
    mh.is_first.assign((size_t)nout * n, 0);
    for (int O = 0; O < nout; ++O) {
        int rows = 0;
        for (int s = 0; s < n; ++s) {
            const int h = s / half, k = s % half, ch = O * cn + h * hpos + k / T, off = k % T;
            if (ch >= c_o || off >= u_h * u_w) continue;
            mh.row_ptr[(size_t)O * (n + 1) + rows] = rows;
            mh.row_slots[(size_t)O * n + rows] = s;
            mh.row_rindex[(size_t)O * n + rows] = ch * u_h * u_w + off;
            mh.is_first[(size_t)O * n + s] = 1;
            ++rows;
        }
        for (int t = rows; t <= n; ++t) mh.row_ptr[(size_t)O * (n + 1) + t] = rows;
        mh.nrows[O] = rows;
    }
    std::vector<int> term_key(nterm, -1), grp_key(cn, -1), term_gal(nterm);
    std::vector<char> ct_rotates(nin, 0);
    for (int e = 0; e < nterm; ++e) {
        term_gal[e] = pl->tap_gal[pl->term_tap[e]];
        if (term_gal[e] != 1) { ++pl->nrot_terms; ct_rotates[pl->term_ct[e]] = 1; }
    }
    for (char f : ct_rotates) pl->nrot_cts += f;
    int rc = upload(&pl->d_term_ct, pl->term_ct);
    if (!rc) rc = upload(&pl->d_term_gal, term_gal);
    if (!rc) rc = upload(&pl->d_term_key, term_key);
    if (!rc) rc = upload(&pl->d_grp_gal, pl->grp_gal);
    if (!rc) rc = upload(&pl->d_grp_key, grp_key);
    {
        std::vector<int> or_gal((size_t)cn * nin), or_key((size_t)cn * nin, -1), seg(nin + 1, 0);
        for (int gam = 0; gam < cn; ++gam)
            for (int I = 0; I < nin; ++I) or_gal[(size_t)gam * nin + I] = pl->grp_gal[gam];
        std::vector<int> seg_terms(nterm), fill(nin, 0);
        for (int e = 0; e < nterm; ++e) ++seg[pl->term_ct[e] + 1];
        for (int I = 0; I < nin; ++I) seg[I + 1] += seg[I];
        for (int e = 0; e < nterm; ++e) seg_terms[seg[pl->term_ct[e]] + fill[pl->term_ct[e]]++] = e;
        if (!rc) rc = upload(&pl->d_or_gal, or_gal);
        if (!rc) rc = upload(&pl->d_or_key, or_key);
        if (!rc) rc = upload(&pl->d_seg_ptr, seg);
        if (!rc) rc = upload(&pl->d_seg_terms, seg_terms);
    }
    if (!rc) rc = upload_mask_layout(c, mh, &pl->mask_d);
    if (rc) { gala_conv_plan_destroy(pl); return rc; }
    *out = pl;
    return GALA_OK;
}
extern "C" int gala_conv_plan_prepare_batched(gala_conv_plan *pl) {
    if (!pl) return GALA_EARG;
    if (pl->d_wl) return GALA_OK;
    const gala_ctx *c = pl->ctx;
    // the matrix-core product keeps exact sums of 192 products in 128 bits, which needs q < 2^60
    if (c->n < 16 || c->q >= (1ull << 60)) return GALA_ESHAPE;
    const int groups = pl->nout * pl->cn, nterm = pl->nterm;
    int mt, nt, kb;
    conv_mfma_geometry(groups, groups, nterm, &mt, &nt, &kb);
    if (hipMalloc((void **)&pl->d_wl, conv_mfma_image_bytes(c->n, mt, kb)) != hipSuccess) return GALA_ENOMEM;
    if (launch_limb_pack(c, nullptr, pl->d_w, 0, groups, nterm, pl->d_wl) || hipDeviceSynchronize() != hipSuccess) {
        hipFree(pl->d_wl);
        pl->d_wl = nullptr;
        return GALA_EHIP;
    }
    return GALA_OK;
}
extern "C" void gala_conv_plan_destroy(gala_conv_plan *pl) {
    if (!pl) return;
    hipFree(pl->d_w); hipFree(pl->d_wl); hipFree(pl->d_term_ct); hipFree(pl->d_term_gal); hipFree(pl->d_term_key);
    hipFree(pl->d_grp_gal); hipFree(pl->d_grp_key);
    hipFree(pl->d_or_gal); hipFree(pl->d_or_key); hipFree(pl->d_seg_ptr); hipFree(pl->d_seg_terms);
    free_mask_layout(&pl->mask_d);
    delete pl;
}
extern "C" int gala_conv_plan_geometry(const gala_conv_plan *pl, int32_t *g) {
    if (!pl || !g) return GALA_EARG;
    g[0] = pl->T; g[1] = pl->cn; g[2] = pl->nin; g[3] = pl->nout; g[4] = pl->ntap; g[5] = pl->nterm;
    return GALA_OK;
}
namespace {
// rotation (swap, step) of a Galois element produced by galois_element()
gala_rot rot_of(const gala_ctx *c, int g) {
    const int n = c->n;
    gala_rot r{0, 0};
    if (g == 1) return r;
    long e = 1;
    for (int step = 0; step < n / 2; ++step) {
        if (e == g) { r.step = step; return r; }
        if (2 * n - e == g) { r.swap = 1; r.step = step; return r; }
        e = e * 3 % (2 * n);
    }
    return r;
}
}  // namespace
extern "C" int gala_conv_plan_rotations(const gala_conv_plan *pl, gala_rot *rots, int *nrots) {
    if (!pl || !nrots) return GALA_EARG;
    std::vector<int> els;
    for (int t : pl->term_tap) {
        const int g = pl->tap_gal[t];
        if (g != 1 && std::find(els.begin(), els.end(), g) == els.end()) els.push_back(g);
    }
    for (int g : pl->grp_gal) if (g != 1 && std::find(els.begin(), els.end(), g) == els.end()) els.push_back(g);
    *nrots = (int)els.size();
    if (rots)
        for (size_t i = 0; i < els.size(); ++i) rots[i] = rot_of(pl->ctx, els[i]);
    return GALA_OK;
}
extern "C" int gala_conv_plan_bind(gala_conv_plan *pl, const gala_gk *gk) {
    if (!pl || !gk || gk->ctx != pl->ctx) return GALA_EARG;
    std::vector<int> tk(pl->nterm, -1), gkey(pl->cn, -1);
    for (int e = 0; e < pl->nterm; ++e) {
        const int g = pl->tap_gal[pl->term_tap[e]];
        if (g == 1) continue;
        auto it = gk->index_of.find(g);
        if (it == gk->index_of.end()) return GALA_ENOKEY;
        tk[e] = it->second;
    }
    for (int g = 0; g < pl->cn; ++g) {
        if (pl->grp_gal[g] == 1) continue;
        auto it = gk->index_of.find(pl->grp_gal[g]);
        if (it == gk->index_of.end()) return GALA_ENOKEY;
        gkey[g] = it->second;
    }
    std::vector<int> okey((size_t)pl->cn * pl->nin);
    for (int g = 0; g < pl->cn; ++g)
        for (int I = 0; I < pl->nin; ++I) okey[(size_t)g * pl->nin + I] = gkey[g];
    if (hipMemcpy(pl->d_term_key, tk.data(), sizeof(int) * pl->nterm, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(pl->d_grp_key, gkey.data(), sizeof(int) * pl->cn, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(pl->d_or_key, okey.data(), sizeof(int) * okey.size(), hipMemcpyHostToDevice) != hipSuccess)
        return GALA_EHIP;
    pl->bound = gk;
    return GALA_OK;
}
// rotations of a hybrid FC plan: the input rotations by 1..G-1, then the rotate-and-sum rotations (duplicates left out)
extern "C" int gala_fc_hybrid_plan_rotations(const gala_fc_hybrid_plan *pl, gala_rot *rots, int *nrots) {
    if (!pl || !nrots) return GALA_EARG;
    std::vector<int> els;
    for (int g : pl->in_gal) if (g != 1 && std::find(els.begin(), els.end(), g) == els.end()) els.push_back(g);
    for (int g : pl->ras_gal) if (g != 1 && std::find(els.begin(), els.end(), g) == els.end()) els.push_back(g);
    *nrots = (int)els.size();
    if (rots)
        for (size_t i = 0; i < els.size(); ++i) rots[i] = rot_of(pl->ctx, els[i]);
    return GALA_OK;
}
extern "C" int gala_fc_hybrid_plan_bind(gala_fc_hybrid_plan *pl, const gala_gk *gk) {
    if (!pl || !gk || gk->ctx != pl->ctx) return GALA_EARG;
    const int steps = (int)pl->ras_gal.size();
    std::vector<int> in_key(pl->G, -1), ras_key(2 * std::max(steps, 1), -1);
    for (int g = 1; g < pl->G; ++g) {
        auto it = gk->index_of.find(pl->in_gal[g]);
        if (it == gk->index_of.end()) return GALA_ENOKEY;
        in_key[g] = it->second;
    }
    for (int k = 0; k < steps; ++k) {
        auto it = gk->index_of.find(pl->ras_gal[k]);
        if (it == gk->index_of.end()) return GALA_ENOKEY;
        ras_key[2 * k + 1] = it->second;
    }
    if (hipMemcpy(pl->d_in_key, in_key.data(), sizeof(int) * in_key.size(), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(pl->d_ras_key, ras_key.data(), sizeof(int) * ras_key.size(), hipMemcpyHostToDevice) != hipSuccess)
        return GALA_EHIP;
    pl->bound = gk;
    return GALA_OK;
}
extern "C" int gala_conv_pack_input(const gala_conv_plan *pl, const uint64_t *x, uint64_t *slots) {
    if (!pl || !x || !slots) return GALA_EARG;
    const int n = pl->ctx->n, half = n / 2, px = pl->u_h * pl->u_w;
    std::fill(slots, slots + (size_t)pl->nin * n, 0);
    for (int ch = 0; ch < pl->c_i; ++ch) {
        const int I = ch / pl->cn, pos = ch % pl->cn, h = pos / pl->hpos, kap = pos % pl->hpos;
        for (int off = 0; off < px; ++off)
            slots[(size_t)I * n + h * half + kap * pl->T + off] = x[(size_t)ch * px + off] % pl->ctx->p;
    }
    return GALA_OK;
}
extern "C" int gala_conv_unpack_share(const gala_conv_plan *pl, int O, const uint64_t *slots, uint64_t *out) {
    if (!pl || !out || !slots || O < 0 || O >= pl->nout) return GALA_EARG;
    const int half = pl->ctx->n / 2, px = pl->u_h * pl->u_w;
    for (int pos = 0; pos < pl->cn; ++pos) {
        const int ch = O * pl->cn + pos, h = pos / pl->hpos, kap = pos % pl->hpos;
        if (ch >= pl->c_o) continue;
        for (int off = 0; off < px; ++off) out[(size_t)ch * px + off] = slots[h * half + kap * pl->T + off] % pl->ctx->p;
    }
    return GALA_OK;
}

// ===========================================================================
// spatial tiling and stride (host)
// ===========================================================================
extern "C" int gala_conv_tiling_plan(const gala_ctx *c, int in_h, int in_w, int k_h, int k_w, int stride,
                                     gala_conv_tiling *t) {
    if (!c || !t || in_h < 1 || in_w < 1 || k_h < 1 || k_w < 1 || stride < 1) return GALA_EARG;
    if (!(k_h & 1) || !(k_w & 1)) return GALA_ESHAPE;
    const int half = c->n / 2;
    int side = 1;
    while ((long)(2 * side) * (2 * side) <= half) side *= 2;       // largest power of two with side^2 <= n/2
    t->in_h = in_h; t->in_w = in_w; t->k_h = k_h; t->k_w = k_w; t->stride = stride;
    if ((long)in_h * in_w <= half) {                                // the whole image is one tile
        t->tile_h = in_h; t->tile_w = in_w;
    } else {
        t->tile_w = in_w <= side ? in_w : side;
        t->tile_h = std::min(in_h, half / t->tile_w);
    }
    t->halo_x = t->tile_w == in_w ? 0 : k_w / 2;
    t->halo_y = t->tile_h == in_h ? 0 : k_h / 2;
    t->step_x = t->tile_w - 2 * t->halo_x;
    t->step_y = t->tile_h - 2 * t->halo_y;
    if (t->step_x < 1 || t->step_y < 1) return GALA_ESHAPE;
    t->tiles_x = (in_w + t->step_x - 1) / t->step_x;
    t->tiles_y = (in_h + t->step_y - 1) / t->step_y;
    t->out_h = (in_h + stride - 1) / stride;
    t->out_w = (in_w + stride - 1) / stride;
    return GALA_OK;
}
namespace {
// image coordinates of the tile's local (0,0)
inline void tile_origin(const gala_conv_tiling *t, int tile, int *oy, int *ox) {
    *oy = (tile / t->tiles_x) * t->step_y - t->halo_y;
    *ox = (tile % t->tiles_x) * t->step_x - t->halo_x;
}
// whether local (ty,tx) is an output this tile keeps, and where it goes
inline bool tile_keeps(const gala_conv_tiling *t, int oy, int ox, int ty, int tx, int *yo, int *xo) {
    if (ty < t->halo_y || ty >= t->halo_y + t->step_y || tx < t->halo_x || tx >= t->halo_x + t->step_x) return false;
    const int y = oy + ty, x = ox + tx;
    if (y < 0 || y >= t->in_h || x < 0 || x >= t->in_w || y % t->stride || x % t->stride) return false;
    *yo = y / t->stride; *xo = x / t->stride;
    return true;
}
}  // namespace
extern "C" int gala_conv_tile_extract(const gala_conv_tiling *t, int ch, const uint64_t *image, int tile,
                                      uint64_t *out) {
    if (!t || !image || !out || ch < 1 || tile < 0 || tile >= t->tiles_x * t->tiles_y) return GALA_EARG;
    int oy, ox;
    tile_origin(t, tile, &oy, &ox);
    for (int c = 0; c < ch; ++c)
        for (int ty = 0; ty < t->tile_h; ++ty)
            for (int tx = 0; tx < t->tile_w; ++tx) {
                const int y = oy + ty, x = ox + tx;
                const bool in = y >= 0 && y < t->in_h && x >= 0 && x < t->in_w;
                out[((size_t)c * t->tile_h + ty) * t->tile_w + tx] = in ? image[((size_t)c * t->in_h + y) * t->in_w + x] : 0;
            }
    return GALA_OK;
}
extern "C" int gala_conv_tile_mask(const gala_conv_tiling *t, int ch, const uint64_t *r, int tile, uint64_t *out) {
    if (!t || !r || !out || ch < 1 || tile < 0 || tile >= t->tiles_x * t->tiles_y) return GALA_EARG;
    int oy, ox, yo, xo;
    tile_origin(t, tile, &oy, &ox);
    for (int c = 0; c < ch; ++c)
        for (int ty = 0; ty < t->tile_h; ++ty)
            for (int tx = 0; tx < t->tile_w; ++tx)
                out[((size_t)c * t->tile_h + ty) * t->tile_w + tx] =
                    tile_keeps(t, oy, ox, ty, tx, &yo, &xo) ? r[((size_t)c * t->out_h + yo) * t->out_w + xo] : 0;
    return GALA_OK;
}
extern "C" int gala_conv_tile_scatter(const gala_conv_tiling *t, int ch, const uint64_t *vals, int tile,
                                      uint64_t *out) {
    if (!t || !vals || !out || ch < 1 || tile < 0 || tile >= t->tiles_x * t->tiles_y) return GALA_EARG;
    int oy, ox, yo, xo;
    tile_origin(t, tile, &oy, &ox);
    for (int c = 0; c < ch; ++c)
        for (int ty = 0; ty < t->tile_h; ++ty)
            for (int tx = 0; tx < t->tile_w; ++tx)
                if (tile_keeps(t, oy, ox, ty, tx, &yo, &xo))
                    out[((size_t)c * t->out_h + yo) * t->out_w + xo] = vals[((size_t)c * t->tile_h + ty) * t->tile_w + tx];
    return GALA_OK;
}

// ===========================================================================
// stride as a polyphase split (host)
// ===========================================================================
namespace {
inline int floor_div(int a, int b) { return a >= 0 ? a / b : -((-a + b - 1) / b); }
// phases read by taps d in [-half, half]: residues of d modulo s, ascending
int phases_of(int half, int s, int32_t *list) {
    int cnt = 0;
    for (int a = 0; a < s; ++a)
        for (int d = -half; d <= half; ++d)
            if (((d % s) + s) % s == a) { list[cnt++] = a; break; }
    return cnt;
}
}  // namespace
extern "C" int gala_conv_polyphase_plan(int c_i, int in_h, int in_w, int k_h, int k_w, int stride,
                                        gala_conv_polyphase *pp) {
    if (!pp || c_i < 1 || in_h < 1 || in_w < 1 || k_h < 1 || k_w < 1 || stride < 1 || stride > 8) return GALA_EARG;
    if (!(k_h & 1) || !(k_w & 1)) return GALA_ESHAPE;
    std::memset(pp, 0, sizeof *pp);
    pp->c_i = c_i; pp->in_h = in_h; pp->in_w = in_w; pp->k_h = k_h; pp->k_w = k_w; pp->stride = stride;
    pp->phases_y = phases_of(k_h / 2, stride, pp->phase_y);
    pp->phases_x = phases_of(k_w / 2, stride, pp->phase_x);
    pp->c_i_poly = c_i * pp->phases_y * pp->phases_x;
    // tap d = s*m + a with m = floor(d/s): the most negative m sets the (symmetric) window
    pp->k_h_poly = 2 * -floor_div(-(k_h / 2), stride) + 1;
    pp->k_w_poly = 2 * -floor_div(-(k_w / 2), stride) + 1;
    pp->out_h = (in_h + stride - 1) / stride;
    pp->out_w = (in_w + stride - 1) / stride;
    return GALA_OK;
}
extern "C" int gala_conv_polyphase_kernel(const gala_conv_polyphase *pp, int c_o, const uint64_t *K, uint64_t *Kp) {
    if (!pp || !K || !Kp || c_o < 1) return GALA_EARG;
    const int s = pp->stride, kh = pp->k_h, kw = pp->k_w, khp = pp->k_h_poly, kwp = pp->k_w_poly, ci = pp->c_i;
    std::fill(Kp, Kp + (size_t)c_o * pp->c_i_poly * khp * kwp, 0);
    for (int o = 0; o < c_o; ++o)
        for (int ch = 0; ch < ci; ++ch)
            for (int ty = 0; ty < kh; ++ty)
                for (int tx = 0; tx < kw; ++tx) {
                    const int dy = ty - kh / 2, dx = tx - kw / 2;
                    const int m = floor_div(dy, s), l = floor_div(dx, s), a = dy - m * s, b = dx - l * s;
                    const int ia = (int)(std::find(pp->phase_y, pp->phase_y + pp->phases_y, a) - pp->phase_y);
                    const int ib = (int)(std::find(pp->phase_x, pp->phase_x + pp->phases_x, b) - pp->phase_x);
                    const int chp = (ia * pp->phases_x + ib) * ci + ch;
                    Kp[(((size_t)o * pp->c_i_poly + chp) * khp + (m + khp / 2)) * kwp + (l + kwp / 2)] =
                        K[(((size_t)o * ci + ch) * kh + ty) * kw + tx];
                }
    return GALA_OK;
}
extern "C" int gala_conv_polyphase_input(const gala_conv_polyphase *pp, const uint64_t *x, uint64_t *xp) {
    if (!pp || !x || !xp) return GALA_EARG;
    const int s = pp->stride, ci = pp->c_i, oh = pp->out_h, ow = pp->out_w;
    for (int ia = 0; ia < pp->phases_y; ++ia)
        for (int ib = 0; ib < pp->phases_x; ++ib)
            for (int ch = 0; ch < ci; ++ch) {
                uint64_t *dst = xp + (size_t)((ia * pp->phases_x + ib) * ci + ch) * oh * ow;
                const uint64_t *src = x + (size_t)ch * pp->in_h * pp->in_w;
                for (int Y = 0; Y < oh; ++Y)
                    for (int X = 0; X < ow; ++X) {
                        const int y = s * Y + pp->phase_y[ia], xx = s * X + pp->phase_x[ib];
                        dst[(size_t)Y * ow + X] = (y < pp->in_h && xx < pp->in_w) ? src[(size_t)y * pp->in_w + xx] : 0;
                    }
            }
    return GALA_OK;
}
