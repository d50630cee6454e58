/*
 * gala.h -- C ABI of the MI355X-native GALA linear-layer library.
 *
 * GALA (arXiv 2105.01827) evaluates the linear layers of a neural network on
 * packed-BFV ciphertexts held by a server: plaintext-weight x ciphertext
 * matrix-vector products with row-wise weight encoding fused with share
 * generation (Sec. III-A(3)) and convolutions with kernel grouping
 * (Sec. III-B(3)), as sequences of the homomorphic operations Add, ScMult and
 * Perm of Sec. II-C(1).
 *
 * Conventions
 *  - Every function returns 0 on success or a negative gala_status; nothing
 *    throws or aborts across this boundary.
 *  - "host" pointers are ordinary CPU memory.  "device" pointers are HIP device
 *    memory on the device that was current when the context was created; they
 *    stay owned by the caller.  Handles (gala_ctx, gala_sk, gala_gk, plans) are
 *    created and destroyed by the library and own whatever device memory they
 *    need (allocated at creation time, never inside he_fc / he_conv / rotate).
 *  - A residue is a uint64_t in [0,q).  The INTERCHANGE form of a ciphertext is
 *    2n residues: the coefficients of c0 then of c1, natural order.  The
 *    INTERNAL device form is also 2n uint64_t per ciphertext but is private
 *    (evaluation domain, permuted order); convert with gala_ct_import/export.
 *  - A slot vector is n values mod p, laid out as two rows of n/2: slot
 *    (h,k) = index h*n/2 + k holds the plaintext polynomial's value at
 *    zeta^(+-3^k), zeta the smallest primitive 2n-th root of unity mod p.
 *  - Streams are hipStream_t passed as void* (NULL = the default stream).
 *    Device work is enqueued on that stream and not waited for.
 */
#ifndef GALA_H
#define GALA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GALA_OK = 0,
    GALA_EARG = -1,      /* null pointer, bad size, bad parameter set          */
    GALA_ESHAPE = -2,    /* layer shape not supported by one ciphertext block  */
    GALA_ENOKEY = -3,    /* a needed Galois key is missing / plan not bound    */
    GALA_ENOMEM = -4,    /* host or device allocation failed, workspace small  */
    GALA_EHIP = -5       /* a HIP call failed                                   */
} gala_status;

/* BFV parameters of Sec. II-C(1) / Sec. IV: n slots (power of two, 8..8192; n = 2048, the paper's ring, has kernels
 * of its own, every other ring runs on kernels written for any n),
 * ciphertext prime q (2^40 <= q < 2^61, q = 1 mod 2n), plaintext prime p
 * (p = 1 mod 2n, p < 2^31, p < q), key-switching digit width gadget_bits
 * (digits = ceil(bitlen(q-1)/gadget_bits) <= 32).  The error distribution is the
 * discrete Gaussian with sigma = 3.2 cut at +-19; the secret is ternary. */
typedef struct {
    int32_t n;
    int32_t gadget_bits;
    uint64_t q;
    uint64_t p;
    /* 0, or a second prime P (P = 1 mod 2n, P != q, 2^40 <= P < 2^61) used only inside key switching:
     * Galois keys then live modulo q*P and hide P * B^j * s(X^g), and every key switch ends with the exact
     * division  floor(t / P)  of its two sums.  A rotation then adds a few units of noise instead of about
     * sqrt(digits * n) * B * sigma, which is what the input rotations of Sec. III-B need to precede ScMult at
     * a 20-bit p.  Costs about twice the transforms per Perm; ciphertexts stay modulo q. */
    uint64_t special_prime;
} gala_params;

/* One slot rotation: both rows rotate left by step (0 <= step < n/2); the two
 * rows are exchanged when swap = 1.  It is the Galois map X -> X^((-1)^swap 3^step). */
typedef struct {
    int32_t swap;
    int32_t step;
} gala_rot;

/* Homomorphic operations executed by one call, in the paper's vocabulary.  A
 * full Perm is one DecPerm plus one HstPerm on a ciphertext of its own;
 * decperm_in / hstperm_in count the hoisted rotations of the convolution's
 * input ciphertexts (Sec. III-B).  The numbers are computed on the host from the
 * dimensions of the launches the call enqueued (items, sums, terms of the plan:
 * the work of every workgroup is fixed by them); nothing is counted on the device.
 * Terms of a convolution whose encoded kernels are all zero are not launched and
 * not counted. */
typedef struct {
    int64_t perm, decperm_in, hstperm_in, scmult, add;
} gala_opcount;

typedef struct gala_ctx gala_ctx;
typedef struct gala_sk gala_sk;
typedef struct gala_gk gala_gk;
typedef struct gala_fc_plan gala_fc_plan;
typedef struct gala_conv_plan gala_conv_plan;

/* ---- context ------------------------------------------------------------ */
/* Validates the parameters, finds the roots of unity and uploads the transform
 * tables to the current HIP device. */
int gala_ctx_create(const gala_params *params, gala_ctx **out);
void gala_ctx_destroy(gala_ctx *ctx);
/* Number of key-switching digits and delta = floor(q/p) of the context. */
int gala_ctx_ndigits(const gala_ctx *ctx);
uint64_t gala_ctx_delta(const gala_ctx *ctx);
/* The 38 thresholds floor(2^64 * P[X <= -19+i]) of the error sampler (host). */
const uint64_t *gala_gauss_cdf(void);

/* The counter-based generator behind every seeded draw of the library (secret and key-switching keys, encryption
 * randomness and noise, the expansion of the masks of gala_he_fc / gala_he_conv from mask_seed): gala_mix64 is the
 * output function of SplitMix64, and
 *   gala_rand64(seed, stream, idx, attempt) = mix64(mix64(mix64(mix64(seed + 0x9E3779B97F4A7C15) + stream) + idx) + attempt).
 * It exists so that seeded runs can be reproduced bit for bit; it is NOT a cryptographic source.  The slots of a
 * mask that are drawn from it are part of the server's secret share (Sec. II-C(2), Sec. III-A(3)): a deployment has
 * to replace these draws by a cryptographic generator keyed with a secret seed. */
uint64_t gala_mix64(uint64_t z);
uint64_t gala_rand64(uint64_t seed, uint64_t stream, uint64_t idx, uint64_t attempt);

/* Measurement aid.  After gala_profile_enable(ctx, capacity) the next `capacity`
 * launches of the rotate-and-accumulate kernel (the Perm kernel inside
 * gala_rotate, gala_he_fc and gala_he_conv) are bracketed by HIP events on the
 * call's stream; gala_profile_collect waits for them, writes the elapsed
 * milliseconds of each launch (host array) and re-arms the events.
 * capacity = 0 switches it off.  Creates / destroys HIP events, so call it
 * outside timed regions. */
int gala_profile_enable(gala_ctx *ctx, int capacity);
/* Which kernel the events bracket: 0 = rotate-and-accumulate (default), 1 = the convolution's
 * multiply-accumulate kernel inside gala_he_conv, 2 = the input rotations of gala_he_conv (DecPerm of the
 * input ciphertexts and HstPerm of every term, one or two launches). */
int gala_profile_select(gala_ctx *ctx, int which);
int gala_profile_collect(gala_ctx *ctx, float *ms, int capacity, int *count);

/* ---- keys (client side, host; Sec. II-C(1)) ------------------------------- */
/* Ternary secret drawn from the seeded generator. */
int gala_keygen(const gala_ctx *ctx, uint64_t seed, gala_sk **out);
void gala_sk_destroy(gala_sk *sk);
/* Copies the secret as n residues mod q (1, 0, q-1) to host memory. */
int gala_sk_export(const gala_ctx *ctx, const gala_sk *sk, uint64_t *s_host);
/* Key-switching keys for the given rotations (duplicates and the identity are
 * ignored), sampled on the host from `seed` and kept on the device. */
int gala_galois_keygen(gala_ctx *ctx, const gala_sk *sk, const gala_rot *rots, int nrots, uint64_t seed,
                       gala_gk **out);
void gala_gk_destroy(gala_gk *gk);
/* Interchange form of one key: ndigits x (b_j, a_j) polynomials, coefficient
 * domain, to host memory (ndigits*2*n words); with a special prime ndigits x
 * (b_j mod q, a_j mod q, b_j mod P, a_j mod P), ndigits*4*n words.  Returns
 * GALA_ENOKEY if absent.  Synchronises the device. */
int gala_gk_export(gala_ctx *ctx, const gala_gk *gk, gala_rot rot, uint64_t *ksk_host);

/* ---- plaintext encoding, encryption, decryption (host) -------------------- */
int gala_encode(const gala_ctx *ctx, const uint64_t *slots /* n */, uint64_t *poly_p /* n, mod p */);
int gala_decode(const gala_ctx *ctx, const uint64_t *poly_p, uint64_t *slots);
/* Symmetric-key encryption ct = (-a s + e + delta*m, a) of a slot vector, in
 * interchange form (2n words, host). */
int gala_encrypt(const gala_ctx *ctx, const gala_sk *sk, const uint64_t *slots, uint64_t seed, uint64_t *ct_host);
/* slots = decode(round(p (c0 + c1 s) / q) mod p); ct in interchange form (host). */
int gala_decrypt(const gala_ctx *ctx, const gala_sk *sk, const uint64_t *ct_host, uint64_t *slots);

/* ---- interchange <-> internal form (device, asynchronous) ----------------- */
/* count ciphertexts of 2n words each; src and dst are device pointers and may
 * be the same buffer. */
int gala_ct_import(const gala_ctx *ctx, void *stream, const uint64_t *ct_coeff_dev, int count, uint64_t *ct_dev);
int gala_ct_export(const gala_ctx *ctx, void *stream, const uint64_t *ct_dev, int count, uint64_t *ct_coeff_dev);

/* ---- the client's steps on the device (batched, asynchronous) --------------- */
/* The same functions as gala_encrypt / gala_decrypt (Sec. II-C(1)) for `count` slot vectors at once, with the
 * ciphertexts in the INTERNAL device form, so that no import / export is needed around he_fc / he_conv.
 * slots_dev: count x n values (reduced mod p on the way in); seeds_dev: count generator seeds, one per
 * ciphertext; ct_dev: count x 2n words.  Bit for bit what gala_encrypt followed by gala_ct_import gives, and
 * what gala_ct_export followed by gala_decrypt gives.  All pointers are device pointers owned by the caller;
 * the secret key's device copy belongs to the key handle.  GALA_EHIP without a device. */
int gala_encrypt_batch(const gala_ctx *ctx, void *stream, const gala_sk *sk, const uint64_t *slots_dev,
                       const uint64_t *seeds_dev, int count, uint64_t *ct_dev);
int gala_decrypt_batch(const gala_ctx *ctx, void *stream, const gala_sk *sk, const uint64_t *ct_dev, int count,
                       uint64_t *slots_dev);

/* The plaintext half of share generation for a batch, on the device (Sec. III-A(3): the slots of one output are
 * added up after decryption, by the client and by the server on its mask alike; the outputs of a convolution are
 * single slots, Sec. III-B).  slots_dev: decrypted slot vectors, count x n for he_fc, count x (output ciphertexts
 * of the plan) x n for he_conv; out_dev: count x n_o, resp. count x c_o x u_h x u_w values mod p.  The same
 * values as gala_fc_unpack_share / gala_conv_unpack_share on every item.  Device pointers, caller-owned. */
int gala_fc_unpack_share_batch(const gala_fc_plan *plan, void *stream, const uint64_t *slots_dev, int count,
                               uint64_t *out_dev);
int gala_conv_unpack_share_batch(const gala_conv_plan *plan, void *stream, const uint64_t *slots_dev, int count,
                                 uint64_t *out_dev);

/* ---- Add, ScMult and plaintext operands on their own (Sec. II-C(1)) --------- */
/* The layers fuse these operations into their kernels; the stand-alone forms are for composing layers the
 * plans do not cover (for example a matrix wider than n, split into blocks whose outputs are added, Sec. III-A).
 * All buffers are device memory in the internal form and may alias where noted; work is enqueued on `stream`.
 *
 * gala_encode_plain: count slot vectors (count x n values, reduced mod p) -> count plaintext polynomials of n
 * words in the evaluation domain.  mode 0: coefficients lifted to (-p/2, p/2] -- the operand of ScMult (the same
 * encoding the plans use for weights).  mode 1: coefficients in [0,p) times delta -- the operand of
 * gala_add_plain / gala_sub_plain, i.e. what encryption adds to c0. */
int gala_encode_plain(const gala_ctx *ctx, void *stream, const uint64_t *slots_dev, int count, int mode,
                      uint64_t *plain_dev);
/* out[i] = a[i] + b[i] slot-wise (both polynomials mod q); out may be a or b. */
int gala_add(const gala_ctx *ctx, void *stream, const uint64_t *a, const uint64_t *b, int count, uint64_t *out);
/* out[i] = ct[i] (.) plain[i * plain_stride]: both polynomials times a mode-0 plaintext; plain_stride is n for
 * one plaintext per ciphertext or 0 to use the same one for all; out may be ct. */
int gala_scmult(const gala_ctx *ctx, void *stream, const uint64_t *ct, const uint64_t *plain, size_t plain_stride,
                int count, uint64_t *out);
/* out[i] = ct[i] -/+ plain[i * plain_stride] with a mode-1 plaintext (only c0 changes); out may be ct.  The
 * subtraction is the share generation of Sec. III-A(3) on its own. */
int gala_sub_plain(const gala_ctx *ctx, void *stream, const uint64_t *ct, const uint64_t *plain, size_t plain_stride,
                   int count, uint64_t *out);
int gala_add_plain(const gala_ctx *ctx, void *stream, const uint64_t *ct, const uint64_t *plain, size_t plain_stride,
                   int count, uint64_t *out);

/* ---- Perm: one slot rotation per ciphertext (Sec. II-C(1)) ----------------- */
/* ct_out[i] = Perm_rot(ct_in[i]) for i < count, internal form, device.  A Perm
 * is a DecPerm (inverse transform of c1, base-2^gadget_bits digits, forward
 * transforms) followed by a HstPerm (automorphism of c0 and of every digit,
 * inner product with the key).  ct_out must not overlap ct_in. */
int gala_rotate(const gala_ctx *ctx, void *stream, const gala_gk *gk, const uint64_t *ct_in, int count,
                gala_rot rot, uint64_t *ct_out);

/* Hoisted rotations (Sec. III-B(1): the k_w k_h - 1 rotations of one input ciphertext; Sec. II-C(1): a Perm is a
 * DecPerm followed by a HstPerm): ct_out[i][k] = Perm_k(ct_in[i]) for every key k of gk, in the order of
 * gala_galois_keygen's list (distinct rotations, the identity left out; gala_gk_count of them), with ONE DecPerm
 * per input shared by all its HstPerm.  Internal form, device; ct_out holds count * gala_gk_count ciphertexts and
 * must not overlap ct_in.  workspace: device scratch of gala_rotate_hoisted_workspace(ctx, count) bytes for the
 * decompositions, caller-owned.  Errors: GALA_EARG, GALA_ENOMEM (workspace too small), GALA_EHIP. */
int gala_gk_count(const gala_gk *gk);
size_t gala_rotate_hoisted_workspace(const gala_ctx *ctx, int count);
int gala_rotate_hoisted(const gala_ctx *ctx, void *stream, const gala_gk *gk, const uint64_t *ct_in, int count,
                        uint64_t *ct_out, void *workspace, size_t workspace_bytes);

/* ---- he_fc: row-encoding-share-RaS matrix-vector product (Sec. III-A(3)) --- */
/* "encode-rowwise" (offline): W is n_o x n_i row-major on the host, entries
 * mod p.  n_o and n_i are padded to powers of two; supported in one block:
 * n_i <= n/2 with n_o <= n, or n/2 < n_i <= n with n_o <= n/2.  The plan
 * holds G = max(1, n_i n_o / n) encoded weight plaintexts on the device. */
int gala_fc_plan_create(gala_ctx *ctx, const uint64_t *W, int n_o, int n_i, gala_fc_plan **out);
void gala_fc_plan_destroy(gala_fc_plan *plan);
/* G of the plan (ScMult count per input); the plan needs rotations by 1..G-1. */
int gala_fc_plan_G(const gala_fc_plan *plan);
/* Writes the G-1 rotations the plan needs (rots may be NULL to query *nrots). */
int gala_fc_plan_rotations(const gala_fc_plan *plan, gala_rot *rots, int *nrots);
/* Resolves the plan's rotations against a key set (offline; GALA_ENOKEY if one is missing, GALA_EARG if the keys
 * were generated for another context).  The plan keeps a pointer to the key set: the key set must outlive every
 * call that uses the plan, and is destroyed by the caller after the plan (or after binding another key set).
 * Binding copies a small index table to the device with a blocking copy: do not bind while calls that use the
 * plan are still in flight on other streams.  The same holds for gala_conv_plan_bind and
 * gala_fc_hybrid_plan_bind. */
int gala_fc_plan_bind(gala_fc_plan *plan, const gala_gk *gk);
/* Client side: slot vector holding n/n_i copies of x (host). */
int gala_fc_pack_input(const gala_fc_plan *plan, const uint64_t *x /* n_i */, uint64_t *slots /* n */);
/* The plaintext rotate-and-sum both parties apply to their share (host):
 * out[t] = sum of the slots that hold partial sums of output t, mod p. */
int gala_fc_unpack_share(const gala_fc_plan *plan, const uint64_t *slots /* n */, uint64_t *out /* n_o */);
/* Bytes of device workspace gala_he_fc needs for a batch. */
size_t gala_he_fc_workspace(const gala_fc_plan *plan, int batch);
/* ct_out[b] = sum_g Perm_g(ScMult(ct_in[b], w_g)) - r'_b for b < batch, where r'_b
 * is the full-length random vector whose plaintext rotate-and-sum is r[b]
 * (every slot but the first of each output's group is drawn from the generator
 * keyed by mask_seed and b).  ct_in/ct_out: batch x 2n, internal form, device;
 * r: batch x n_o values mod p, device.  counts (host, may be NULL) receives the
 * operations executed.  Asynchronous on `stream`. */
int gala_he_fc(const gala_ctx *ctx, void *stream, const gala_fc_plan *plan, const uint64_t *ct_in, int batch,
               const uint64_t *r, uint64_t mask_seed, uint64_t *ct_out, void *workspace, size_t workspace_bytes,
               gala_opcount *counts);

/* gala_he_fc for callers that cannot allocate device memory or bring a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same computation and the same results as gala_he_fc,
 * with the partial ciphertexts in a fixed array of gala_he_fc_static_capacity() bytes (32 MiB) that is part of the
 * library's device code; each GPU the library runs on holds its copy until the process ends.  The call allocates
 * nothing and only enqueues kernels on `stream`.  Returns GALA_ENOMEM when gala_he_fc_workspace(plan, batch)
 * exceeds the capacity (nothing is launched), GALA_EARG when the current device is not the context's.  All calls
 * on one GPU share the array: calls that overlap in time on one GPU (different streams or threads) race; calls
 * on one stream are ordered and safe.  Nothing needs clearing between calls: a call reads only what it wrote. */
size_t gala_he_fc_static_capacity(void);
int gala_he_fc_static(const gala_ctx *ctx, void *stream, const gala_fc_plan *plan, const uint64_t *ct_in, int batch,
                      const uint64_t *r, uint64_t mask_seed, uint64_t *ct_out, gala_opcount *counts);

/* ---- he_conv: kernel-grouping convolution (Sec. III-B(3)) ------------------ */
/* K is c_o x c_i x k_h x k_w row-major on the host, entries mod p; the image
 * is u_h x u_w per channel; stride 1, zero "same" padding, odd k_h and k_w.
 * c_n = n / T channels share a ciphertext, T the power of two >= u_h*u_w
 * (T <= n/2); channel counts are padded to multiples of c_n. */
int gala_conv_plan_create(gala_ctx *ctx, const uint64_t *K, int c_o, int c_i, int k_h, int k_w, int u_h, int u_w,
                          gala_conv_plan **out);
void gala_conv_plan_destroy(gala_conv_plan *plan);
/* Optional, offline: also keeps the encoded kernels as base-256 digit planes so that gala_he_conv
 * runs its ScMult/Add step (a dense per-coefficient matrix product, Sec. III-B) on the matrix cores
 * whenever a call brings at least 2 inputs.  Costs about 1.3x the plan's device memory again;
 * results are bit-identical either way for sums of any length (the running sums are reduced mod q every 192
 * terms).  Needs n >= 16 and q < 2^60; otherwise GALA_ESHAPE, and gala_he_conv keeps using the vector ALU. */
int gala_conv_plan_prepare_batched(gala_conv_plan *plan);
/* geometry[0..5] = T, c_n, input ciphertexts per image, output ciphertexts, taps, terms: the (input ciphertext,
   tap) pairs whose encoded kernels are not all zero; only these are rotated and multiplied. */
int gala_conv_plan_geometry(const gala_conv_plan *plan, int32_t *geometry);
int gala_conv_plan_rotations(const gala_conv_plan *plan, gala_rot *rots, int *nrots);
int gala_conv_plan_bind(gala_conv_plan *plan, const gala_gk *gk);
/* Client side: x is c_i x u_h x u_w; slots receives (input ciphertexts) x n values. */
int gala_conv_pack_input(const gala_conv_plan *plan, const uint64_t *x, uint64_t *slots);
/* Gathers the real outputs of output ciphertext O from its decrypted slots into out (c_o x u_h x u_w). */
int gala_conv_unpack_share(const gala_conv_plan *plan, int O, const uint64_t *slots, uint64_t *out);
size_t gala_he_conv_workspace(const gala_conv_plan *plan, int batch);
/* For each input b: one DecPerm per input ciphertext and one HstPerm per
 * non-central tap; per output block and kernel order the ScMults are added
 * first, then each sum is rotated once and added (first-Add-second-Perm); the
 * mask r[b] (c_o x u_h x u_w, device) is subtracted, pad slots masked from the
 * generator.  ct_in: batch x n_in x 2n; ct_out: batch x n_out x 2n; internal form. */
int gala_he_conv(const gala_ctx *ctx, void *stream, const gala_conv_plan *plan, const uint64_t *ct_in, int batch,
                 const uint64_t *r, uint64_t mask_seed, uint64_t *ct_out, void *workspace, size_t workspace_bytes,
                 gala_opcount *counts);

/* ---- the paper's comparison schedules on the same operations ------------------------------------------------
 * The two schedules GALA is measured against in Sec. IV-A, built from the same kernels so that the ratio of the
 * schedules can be measured on one device.  Results decrypt to the same W x and the same convolution.
 *
 * Hybrid matrix-vector product (Sec. III-A(2)): the input ciphertext is rotated by 1..G-1 (HstPerm with one common
 * DecPerm), each rotation is multiplied by one diagonal vector of W (ScMult) and the products are added; then
 * log2(n / n_o) rotate-and-sum steps, each a Perm and an Add on the running ciphertext, leave output t in one slot;
 * the mask (r[t] at that slot, a generator draw in every other slot) is subtracted.  G = max(1, n_i n_o / n).
 * Shapes as for gala_fc_plan_create; the input is packed as for he_fc (gala_fc_hybrid_pack_input gives the same
 * slot vector as gala_fc_pack_input); gala_fc_hybrid_unpack reads the n_o result slots of a decrypted vector.
 * gala_fc_hybrid_plan_rotations lists the input rotations and the rotate-and-sum rotations (GALA_ENOKEY from
 * bind if one is missing).  Because the input is rotated before ScMult, results decrypt only when the rotation
 * noise times the weights stays below delta / 2 (Sec. III-C): for G > 1 at a 20-bit p this needs special-prime keys. */
typedef struct gala_fc_hybrid_plan gala_fc_hybrid_plan;
int gala_fc_hybrid_plan_create(gala_ctx *ctx, const uint64_t *W, int n_o, int n_i, gala_fc_hybrid_plan **out);
void gala_fc_hybrid_plan_destroy(gala_fc_hybrid_plan *plan);
int gala_fc_hybrid_plan_G(const gala_fc_hybrid_plan *plan);
int gala_fc_hybrid_plan_steps(const gala_fc_hybrid_plan *plan);      /* rotate-and-sum steps = Perms per input */
int gala_fc_hybrid_plan_rotations(const gala_fc_hybrid_plan *plan, gala_rot *rots, int *nrots);
int gala_fc_hybrid_plan_bind(gala_fc_hybrid_plan *plan, const gala_gk *gk);
int gala_fc_hybrid_pack_input(const gala_fc_hybrid_plan *plan, const uint64_t *x /* n_i */, uint64_t *slots /* n */);
int gala_fc_hybrid_unpack(const gala_fc_hybrid_plan *plan, const uint64_t *slots /* n */, uint64_t *out /* n_o */);
size_t gala_he_fc_hybrid_workspace(const gala_fc_hybrid_plan *plan, int batch);
/* Arguments as gala_he_fc.  The rotate-and-sum steps of one input depend on each other, so a call runs them as
 * log2(n / n_o) launches of `batch` workgroups each. */
int gala_he_fc_hybrid(const gala_ctx *ctx, void *stream, const gala_fc_hybrid_plan *plan, const uint64_t *ct_in, int batch,
                      const uint64_t *r, uint64_t mask_seed, uint64_t *ct_out, void *workspace, size_t workspace_bytes,
                      gala_opcount *counts);
/* Output-rotation MIMO convolution (Sec. III-B(2)) on a gala_conv_plan: the same packing, encoded kernels, input
 * rotations, keys and mask as gala_he_conv, but the products of every input ciphertext are summed on their own and
 * every (output ciphertext, input ciphertext, kernel order) sum is rotated before the additions, i.e.
 * c_i c_o (c_n - 1) / c_n^2 Perms instead of c_o (c_n - 1) / c_n.  Arguments as gala_he_conv (the multiply-accumulate
 * runs on the vector ALU). */
size_t gala_he_conv_outrot_workspace(const gala_conv_plan *plan, int batch);
int gala_he_conv_outrot(const gala_ctx *ctx, void *stream, const gala_conv_plan *plan, const uint64_t *ct_in, int batch,
                        const uint64_t *r, uint64_t mask_seed, uint64_t *ct_out, void *workspace, size_t workspace_bytes,
                        gala_opcount *counts);

/* ---- spatial tiling and stride for images larger than half a ciphertext (host) ---- */
/* The paper assumes u_w*u_h fits a ciphertext (Sec. III-B(1), footnote) and never mentions stride.
 * Here an in_h x in_w image is cut into overlapping tile_h x tile_w tiles (tile_h*tile_w <= n/2) whose
 * halo of k-1 rows/columns supplies the neighbours; every tile is an independent input of the same
 * convolution plan (u_h = tile_h, u_w = tile_w), i.e. the tiles form the batch of gala_he_conv.  Only
 * the interior of a tile is a valid output.  A stride-s convolution is evaluated at stride 1 and the
 * outputs at multiples of s are kept (out_h = ceil(in_h/s)), the rest is masked and dropped. */
typedef struct {
    int32_t in_h, in_w, k_h, k_w, stride;
    int32_t tile_h, tile_w;      /* u_h, u_w of the plan to create                          */
    int32_t tiles_y, tiles_x;    /* number of tiles; the batch is tiles_y*tiles_x per image */
    int32_t step_y, step_x;      /* interior size = distance between tile origins           */
    int32_t halo_y, halo_x;      /* rows / columns of halo on each side (0 if not tiled)    */
    int32_t out_h, out_w;
} gala_conv_tiling;
int gala_conv_tiling_plan(const gala_ctx *ctx, int in_h, int in_w, int k_h, int k_w, int stride,
                          gala_conv_tiling *out);
/* tile_out (ch x tile_h x tile_w) = the tile's window of image (ch x in_h x in_w), zeros outside it. */
int gala_conv_tile_extract(const gala_conv_tiling *t, int ch, const uint64_t *image, int tile, uint64_t *tile_out);
/* r_tile (ch x tile_h x tile_w) = the layer-level mask r (ch x out_h x out_w) at the outputs this tile
 * keeps, 0 at the positions that are dropped. */
int gala_conv_tile_mask(const gala_conv_tiling *t, int ch, const uint64_t *r, int tile, uint64_t *r_tile);
/* Writes the outputs this tile keeps from tile_vals (ch x tile_h x tile_w) into out (ch x out_h x out_w). */
int gala_conv_tile_scatter(const gala_conv_tiling *t, int ch, const uint64_t *tile_vals, int tile, uint64_t *out);

/* ---- stride as a polyphase split (host) ----
 * The paper never mentions stride.  A stride-s "same" convolution, out[Y][X] = sum K[dy][dx] * x[sY+dy][sX+dx]
 * over |dy| <= k_h/2, |dx| <= k_w/2, equals a stride-1 convolution (Sec. III-B) over the phase images
 * x_(a,b)[Y][X] = x[sY+a][sX+b] taken as input channels, with the kernel of phase (a,b) holding K[sm+a][sl+b] at
 * tap (m,l).  Only phases that some tap reads are kept (a 1x1 kernel reads phase (0,0) alone), in phase-major
 * channel order: channel = (ia*phases_x + ib)*c_i + ch, where ia, ib index phase_y[], phase_x[].  The rearranged
 * kernel is mostly zero taps, which convolution plans leave out; the layer's output comes out at its final size,
 * nothing is computed and dropped.  1 <= stride <= 8. */
typedef struct {
    int32_t c_i, in_h, in_w, k_h, k_w, stride;
    int32_t phases_y, phases_x;          /* number of row / column phases kept                     */
    int32_t phase_y[8], phase_x[8];      /* their residues a, b in [0, stride), ascending          */
    int32_t c_i_poly;                    /* c_i * phases_y * phases_x input channels of the plan   */
    int32_t k_h_poly, k_w_poly;          /* odd sizes of the stride-1 kernel                       */
    int32_t out_h, out_w;                /* ceil(in/stride): size of every phase image and of the output */
} gala_conv_polyphase;
int gala_conv_polyphase_plan(int c_i, int in_h, int in_w, int k_h, int k_w, int stride, gala_conv_polyphase *out);
/* K (c_o x c_i x k_h x k_w) -> K_poly (c_o x c_i_poly x k_h_poly x k_w_poly), values copied unchanged. */
int gala_conv_polyphase_kernel(const gala_conv_polyphase *pp, int c_o, const uint64_t *K, uint64_t *K_poly);
/* x (c_i x in_h x in_w) -> x_poly (c_i_poly x out_h x out_w), zero where a phase runs past the image. */
int gala_conv_polyphase_input(const gala_conv_polyphase *pp, const uint64_t *x, uint64_t *x_poly);

#ifdef __cplusplus
}
#endif
#endif /* GALA_H */
