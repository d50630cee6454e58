// Internal data structures of the library (host side) and the launch interface
// of the HIP kernels.  Nothing here is visible through the C ABI.
#pragma once
#include <cstddef>
#include <map>
#include <vector>

#include "../../include/gala.h"
#include "modarith.h"

namespace gala {

constexpr int kMaxDigits = 32;
constexpr int kMaxN = 8192;   // rings above 2048 run on the any-n kernels (512 or 1024 threads per polynomial)
constexpr int kGaussBound = 19;

// Cumulative table of the discrete Gaussian (passed to kernels by value) and the draw from it: one 64-bit word
// of the counter-based generator compared with the 38 thresholds.
struct GaussCdf {
    u64 t[2 * kGaussBound];   // floor(2^64 * P[X <= -bound + i])
};
GALA_HD int draw_gauss_cdf(const GaussCdf &cdf, u64 seed, u64 stream, u64 idx) {
    const u64 u = rand64(seed, stream, idx, 0);
    int x = -kGaussBound;
    for (int i = 0; i < 2 * kGaussBound; ++i) x += u >= cdf.t[i] ? 1 : 0;
    return x;
}

// Entries g0 .. g1-1 of a rotate-and-accumulate sum that chunk `chunk` of `nchunks` takes.  The first entry is the
// rotation by zero in he_fc and he_conv (a ScMult and no key switch): it rides with chunk 0, and the G-1 entries
// after it are spread evenly, so that no workgroup is launched for the cheap entry alone.
GALA_HD void chunk_range(int chunk, int nchunks, int G, int &g0, int &g1) {
    g0 = chunk ? 1 + (int)((long)chunk * (G - 1) / nchunks) : 0;
    g1 = 1 + (int)((long)(chunk + 1) * (G - 1) / nchunks);
}

// ---------------------------------------------------------------------------
// Negacyclic number-theoretic transform tables for one modulus.
// Forward: natural-order coefficients -> values a(psi^(2*brev(i)+1)) at index i.
// tw[m+i] = psi^brev(m+i) for the stage with m blocks; itw holds the inverses.
// The inverse folds n^-1 into its last stage (ninv, itw1n = itw[1]*ninv).
// ---------------------------------------------------------------------------
struct NttHost {
    int n = 0, logn = 0;
    Modulus mod{};
    u64 psi = 0;
    std::vector<u64> tw, tws, itw, itws;
    u64 ninv = 0, ninvs = 0, itw1n = 0, itw1ns = 0;

    void init(int n, u64 q, u64 psi);
    void forward(u64 *a) const;   // in place, canonical in -> canonical out
    void inverse(u64 *a) const;
};

// Device view of the same tables (pointers into one device allocation).
struct NttDev {
    const u64 *tw, *tws, *itw, *itws;
    u64 ninv, ninvs, itw1n, itw1ns;
    Modulus mod;
};

u64 pow_mod(u64 b, u64 e, u64 m);
u64 inv_mod(u64 a, u64 m);
u64 shoup_companion(u64 w, u64 q);
Modulus make_modulus(u64 q);
bool is_prime_u64(u64 v);
int bit_length(u64 v);
inline int brev(int v, int bits) {
    int r = 0;
    for (int b = 0; b < bits; ++b) r |= ((v >> b) & 1) << (bits - 1 - b);
    return r;
}

}  // namespace gala

// ---------------------------------------------------------------------------
// Handles
// ---------------------------------------------------------------------------
struct gala_ctx {
    int n = 0, logn = 0, gadget_bits = 0, ndigits = 0, pbits = 0, qbits = 0;
    gala::u64 q = 0, p = 0, delta = 0, delta_s = 0, zeta = 0;
    gala::NttHost ntt_q, ntt_p;
    // special prime of key switching (0: keys modulo q only)
    gala::u64 special = 0, Pq = 0, Pq_s = 0, Pinv = 0, Pinv_s = 0;   // P mod q and P^-1 mod q with companions
    gala::NttHost ntt_P;
    std::vector<int> slot_to_idx;      // slot s -> index of its value in the mod-p transform
    int device = 0;
    bool has_device = false;           // tables uploaded; false on a host without a HIP device
    gala::u64 *d_tables = nullptr;     // 8*n words: tw,tws,itw,itws for q then for p
    int *d_slot_to_idx = nullptr;
    gala::u64 *d_tw2 = nullptr;        // n = 2048 only: pass-major (w, companion) twiddle blocks, forward then inverse
    gala::u64 *d_tw2p = nullptr;       // the same for the plaintext modulus
    gala::u64 *d_tablesP = nullptr;    // 4*n words: tw,tws,itw,itws for the special prime
    gala::u64 *d_tw2P = nullptr;       // pass-major blocks for the special prime (n = 2048)
    gala::NttDev dev_q{}, dev_p{}, dev_P{};
    int key_polys() const { return special ? 4 : 2; }
    // measurement aid: event pairs recorded around rotate-and-accumulate launches
    mutable std::vector<void *> prof_events;   // 2*capacity hipEvent_t
    mutable int prof_used = 0;
    mutable int prof_which = 0;                // 0: rotate-and-accumulate launches, 1: convolution multiply-accumulate
};

struct gala_sk {
    std::vector<gala::u64> s;          // coefficients mod q (0, 1, q-1)
    std::vector<gala::u64> s_hat;      // forward transform of s
    gala::u64 *d_s_hat = nullptr;      // device copy of s_hat (null on a host without a device)
};

struct gala_gk {
    const gala_ctx *ctx = nullptr;     // the context the keys were generated for (plans of another context refuse them)
    int n = 0, ndigits = 0, polys = 2; // polynomials per digit: (b, a) mod q, then (b, a) mod P with a special prime
    std::map<int, int> index_of;       // Galois element -> key index
    std::vector<int> elements;
    gala::u64 *d_keys = nullptr;       // nkeys x ndigits x polys x n, evaluation domain (b then a)
    gala::u64 *d_keys2 = nullptr;      // same keys as (value, companion) pairs for the n = 2048 kernel, or null
    int *d_elements = nullptr;         // nkeys Galois elements, device
    int *d_iota = nullptr;             // 0,1,2,... (key index of element k is k), device
    int *d_one = nullptr;              // the single value 1 (Galois element of the identity), device
    int *d_zeros = nullptr;            // nkeys zeros (every hoisted rotation reads input ciphertext 0 of its item), device
    size_t key_words() const { return (size_t)ndigits * polys * n; }
};

// Device description of how the server's mask is laid out in one output
// ciphertext: which slots are drawn from the generator and which absorb r.
struct MaskLayoutHost {
    int nout = 0;                      // output ciphertexts
    std::vector<int> row_ptr;          // nout x (n+1): CSR over the "rows" (outputs) of each ciphertext
    std::vector<int> row_slots;        // nout x n: slots of each row, first slot first
    std::vector<int> row_rindex;       // nout x n: index into r of each row
    std::vector<int> nrows;            // nout
    std::vector<unsigned char> is_first;  // nout x n: slot is the first of a real row (not drawn)
};
struct MaskLayoutDev {
    int *row_ptr = nullptr, *row_slots = nullptr, *row_rindex = nullptr, *nrows = nullptr;
    unsigned char *is_first = nullptr;
    // per entry e of the CSR (nout x n): its row, or -1 for the first entry of a row, and the position of its slot
    // in the mod-p transform's input; per row (nout x n): that position for the row's first slot
    int *entry_row = nullptr, *entry_idx = nullptr, *first_idx = nullptr;
    int *slot_rowid = nullptr;         // nout x n: the row a slot belongs to, -1 for slots outside every row
};

struct gala_fc_plan {
    gala_ctx *ctx = nullptr;
    int n_o = 0, n_i = 0, nop = 0, nip = 0, G = 0;
    bool big = false;
    std::vector<int> slot_row;         // padded row of each slot, -1 if it carries no weight
    std::vector<int> gal;              // Galois element of rotation g (gal[0] = 1)
    gala::u64 *d_w = nullptr;          // G x n encoded weights, evaluation domain
    gala::u64 *d_w2 = nullptr;         // the same as (value, companion) pairs for the n = 2048 kernel, or null: G polynomials in
                                       // natural order, then the same G in the threads' ownership order
    int *d_gal = nullptr;              // G Galois elements
    int *d_key_idx = nullptr;          // G key indices (valid once bound)
    const gala_gk *bound = nullptr;
    MaskLayoutHost mask_h;
    MaskLayoutDev mask_d;
};

// The hybrid matrix-vector product of Sec. III-A(2) (comparison schedule): G diagonal vectors that multiply the
// input rotated by 0..G-1, then rotate-and-sum steps on the running ciphertext.
struct gala_fc_hybrid_plan {
    gala_ctx *ctx = nullptr;
    int n_o = 0, n_i = 0, nop = 0, nip = 0, G = 0, R = 0;
    bool big = false;
    std::vector<int> in_gal;           // Galois elements of the input rotations g = 0..G-1 (in_gal[0] = 1)
    std::vector<int> ras_gal;          // Galois elements of the rotate-and-sum steps, in order
    std::vector<int> result_slot;      // slot that holds output t after the last step
    gala::u64 *d_w = nullptr;          // G x n diagonal vectors, evaluation domain
    int *d_in_ct = nullptr, *d_in_gal = nullptr, *d_in_key = nullptr;   // G each: the term list of the input rotations
    int *d_ras_gal = nullptr, *d_ras_key = nullptr;   // per step the pair (1, gal) / (-1, key index): 2 ints each
    const gala_gk *bound = nullptr;
    MaskLayoutHost mask_h;
    MaskLayoutDev mask_d;
};

struct gala_conv_plan {
    gala_ctx *ctx = nullptr;
    int c_o = 0, c_i = 0, k_h = 0, k_w = 0, u_h = 0, u_w = 0;
    int T = 0, cn = 0, hpos = 0, nin = 0, nout = 0, ntap = 0, centre = 0;
    std::vector<int> tap_gal, grp_gal; // Galois elements of taps (ntap) and kernel orders (cn)
    // Terms of the multiply-accumulate: the (input ciphertext, tap) pairs whose encoded kernels are not all zero,
    // in (tap, input) order: consecutive terms share their tap, i.e. their rotation and key, which the kernel that
    // rotates the inputs sixteen terms at a time loads once.  A dense kernel has nin*ntap of them.
    int nterm = 0, nrot_terms = 0, nrot_cts = 0;   // terms; those that rotate; input ciphertexts with a rotating term
    std::vector<int> term_ct, term_tap;
    int *d_term_ct = nullptr, *d_term_gal = nullptr, *d_term_key = nullptr;   // nterm each (key valid once bound)
    gala::u64 *d_w = nullptr;          // nout x cn x nterm x n encoded kernels, evaluation domain
    gala::u64 *d_wl = nullptr;         // the same as balanced base-256 digit planes for the matrix-core path, or null
    int *d_grp_gal = nullptr, *d_grp_key = nullptr;   // cn
    // output-rotation schedule (Sec. III-B(2)): entry gam * nin + I of an output ciphertext's sum is the block of input
    // ciphertext I in kernel order gam; seg_ptr[I] .. seg_ptr[I+1]-1 are the terms of input ciphertext I
    int *d_or_gal = nullptr, *d_or_key = nullptr;     // cn * nin
    int *d_seg_ptr = nullptr, *d_seg_terms = nullptr;  // nin + 1 offsets into the nterm term numbers grouped by input ciphertext
    const gala_gk *bound = nullptr;
    MaskLayoutHost mask_h;
    MaskLayoutDev mask_d;
};

// ---------------------------------------------------------------------------
// Kernel launchers (defined in gala_kernels.hip).  All return a hipError_t cast to int.
// ---------------------------------------------------------------------------
namespace gala {

// resolves, once per device, the device address of the fixed scratch array behind gala_he_fc_static (gala_api.cpp)
int static_scratch_init();

// batched transform of `count` polynomials of n words: inverse=0 forward.
int launch_ntt(const gala_ctx *ctx, void *stream, const u64 *src, u64 *dst, size_t count, int inverse);
// the same with the tables of another modulus of the context (dev_q, dev_p or dev_P)
int launch_ntt_mod(const gala_ctx *ctx, void *stream, const u64 *src, u64 *dst, size_t count, int inverse, const NttDev &T);

// Batched client steps on internal-form ciphertexts (one workgroup per ciphertext).
int launch_encrypt(const gala_ctx *ctx, void *stream, const u64 *s_hat, const u64 *slots, const u64 *seeds, int count,
                   u64 *ct_out);
int launch_decrypt(const gala_ctx *ctx, void *stream, const u64 *s_hat, const u64 *ct_in, int count, u64 *slots);
const u64 *gauss_cdf_table();
// the same two steps with the radix-8 transforms of the n = 2048 kernels
int launch_encrypt_2048(const gala_ctx *ctx, void *stream, const u64 *s_hat, const u64 *slots, const u64 *seeds, int count,
                        u64 *ct_out);
int launch_decrypt_2048(const gala_ctx *ctx, void *stream, const u64 *s_hat, const u64 *ct_in, int count, u64 *slots);

// Stand-alone Add / ScMult / plaintext operations on internal-form buffers (op: 0 add ct, 1 scmult, 2 sub plain, 3 add plain).
int launch_encode_plain(const gala_ctx *ctx, void *stream, const u64 *slots, int count, int mode, u64 *plain);
int launch_ct_op(const gala_ctx *ctx, void *stream, int op, const u64 *a, const u64 *b, size_t b_stride, int count, u64 *out);
// "encode" of a convolution plan on the device (Sec. III-B(3), kernel grouping): slot vectors of the encoded kernels
// `first` .. `first + count - 1` in (O, gamma, term) order, from the kernel tensor K (c_o x c_i x k_h x k_w, device)
struct ConvGeom {
    int c_o, c_i, k_h, k_w, u_h, u_w, T, cn, hpos, nterm, n;
    u64 p;
};
int launch_conv_weight_slots(const gala_ctx *ctx, void *stream, const u64 *K, const ConvGeom &g, const int *term_ct,
                             const int *term_tap, size_t first, size_t count, u64 *slots);
// "encode" of an FC plan on the device: slot vectors of the encoded weights g = 0..count-1 from W (n_o x n_i, device)
// and the plan's slot -> padded row table (n ints, device; -1: the slot carries no weight).  rotate_output: GALA's
// row-wise encoding (the product is rotated by g afterwards); otherwise the hybrid method's diagonals (the input is
// rotated by g before the product).
struct FcGeom {
    int n, n_o, n_i, nip, big, rotate_output;
    u64 p;
};
int launch_fc_weight_slots(const gala_ctx *ctx, void *stream, const u64 *W, const FcGeom &g, const int *slot_row, int count,
                           u64 *slots);
// out[b][rindex of row t] = sum of the row's slots mod p, for `count` items of nout slot vectors each
int launch_unpack_share(const gala_ctx *ctx, void *stream, const u64 *slots, int count, int nout, const MaskLayoutDev &layout,
                        size_t out_stride, u64 *out);

// key generation helper on `npairs` consecutive (t_hat, a_hat) pairs of n-word evaluation-domain
// polynomials: t_hat <- t_hat - a_hat * s_hat in place (s_hat shared by all pairs).
int launch_key_finish(const gala_ctx *ctx, void *stream, u64 *pairs, const u64 *s_hat, size_t npairs, const Modulus &mod);
// dst[i] = (src[i], floor(src[i] * 2^64 / q)) for i < count: constants with the precomputed quotient
// that the n = 2048 kernel multiplies by.
// With a special prime the polynomials alternate (b, a) mod q, (b, a) mod P: `polys` = 4 selects the modulus
// by polynomial index, `polys` = 2 uses q throughout.
int launch_pair_pack(const gala_ctx *ctx, void *stream, const u64 *src, u64 *dst, size_t count, int polys);
// dst[poly][512*(t/64) + 64*k + t%64] = src[poly][8*t + k] on 16-byte pairs of n = 2048 polynomials: the order in which
// the threads of the Perm kernel read the 8 consecutive coefficients they own - one coalesced load per k, the eight of
// a wavefront within 8 KiB
int launch_owner_order_2048(void *stream, const u64 *src_pairs, u64 *dst_pairs, size_t npolys);
// whether launch_perm_accumulate will use the n = 2048 kernel for this context
bool uses_fast_perm(const gala_ctx *ctx);

// One job of the rotate-and-accumulate kernel.  For item in [0,items), chunk in [0,nchunks):
//   partial[item][chunk] = sum over g in the chunk of Perm_{gal[g]}( in[item][g] (.) w[g] )
// where in[item][g] = ct_in + item*in_item_stride + g*in_g_stride (2n words each) and w[g] = w + g*n
// (w == nullptr: no ScMult).  gal[g] == 1 means no rotation.  key_idx[g] selects the key.
struct PermJob {
    const u64 *ct_in;
    size_t in_item_stride, in_g_stride;
    const u64 *w;
    const int *gal, *key_idx;
    const u64 *keys;
    const u64 *w2, *keys2;   // (value, companion) pair images of w and keys (n = 2048 kernel only)
    const int *in_g_index;   // optional: rotation g reads input number in_g_index[g] instead of g
    // n = 2048 kernel only, in8_S != 0: the inputs are the matrix-core product's sums in blocks of eight coefficients,
    // word (i/8)*in8_S + i%8 of a polynomial, c1 eight words after c0; item = b*in8_nout + O starts at
    // ct_in + O*in8_o_stride + 16*b and rotation g in_g_stride words further.
    size_t in8_S, in8_o_stride;
    int in8_nout;
    int G, items, nchunks;
    int slots;               // partial ciphertexts reserved per item (>= nchunks)
    u64 *partial;            // items x slots x 2n
};
int launch_perm_accumulate(const gala_ctx *ctx, void *stream, const PermJob &job);
// the n = 2048, q < 2^60 specialisation (gala_perm2048.hip); launch_perm_accumulate dispatches to it
int launch_perm_accumulate_2048(const gala_ctx *ctx, void *stream, const PermJob &job);

// out[item] = sum_chunk partial[item][chunk] - mask(item) ; mask built from r and the generator.
struct FinalizeJob {
    const u64 *partial;
    int items, nchunks;
    int slots;               // partial ciphertexts reserved per item (>= nchunks)
    int nout;                // output ciphertexts per batch element (item = b*nout + O)
    const u64 *r;            // batch x r_stride values mod p (nullptr: no mask)
    size_t r_stride;
    u64 mask_seed;
    MaskLayoutDev mask;
    u64 *ct_out;             // items x 2n
};
int launch_finalize(const gala_ctx *ctx, void *stream, const FinalizeJob &job);
// Rotate-and-accumulate followed by share generation.  With the n = 2048 kernel the mask of every
// item is built by extra workgroups of the same launch (as one more partial ciphertext, slot
// `nchunks`, so job.slots must be >= nchunks + 1) and a light kernel adds the partials up;
// otherwise this is launch_perm_accumulate + launch_finalize.
int launch_perm_finalize(const gala_ctx *ctx, void *stream, const PermJob &job, const FinalizeJob &fin);
int launch_perm_accumulate_2048_masked(const gala_ctx *ctx, void *stream, const PermJob &job, const FinalizeJob &fin);

// DecPerm of `count` ciphertexts: digits[c][j] = forward(digit_j(inverse(c1))), j < ndigits.
int launch_decperm(const gala_ctx *ctx, void *stream, const u64 *ct_in, size_t count, u64 *digits);
// The convolution's rotated inputs, one per (batch element, term): the description of the terms of a plan.
struct TermList {
    int nin, nterm;               // input ciphertexts per batch element, terms
    const int *ct, *gal, *key;    // per term: input ciphertext, Galois element of its tap, key index (device)
};
// HstPerm for the convolution's input rotations:
//   xrot[b][e] = HstPerm_{gal[e]}(ct_in[b*nin + ct[e]], its digits) ; a term with Galois element 1 is a copy.
int launch_hstperm_taps(const gala_ctx *ctx, void *stream, const u64 *ct_in, const u64 *digits, int batch,
                        const TermList &terms, const u64 *keys, u64 *xrot);
// acc[b][O][gam] = sum_{I,tap} w[O][gam][I][tap] (.) xrot[b][I][tap]   (both polynomials)
// seg_ptr (device, nseg + 1 ints) and seg_terms (device, term numbers) give nseg groups of terms sums of their own:
//   acc[b][O][gam][s] = sum over the terms seg_terms[seg_ptr[s] .. seg_ptr[s+1]-1]; nullptr: one sum over all terms
int launch_conv_mac(const gala_ctx *ctx, void *stream, const u64 *w, const u64 *xrot, int batch, int nout, int cn,
                    int nterm, u64 *acc, const int *seg_ptr = nullptr, const int *seg_terms = nullptr, int nseg = 1);

// Matrix-core path of the convolution's multiply-accumulate (gala_conv_mfma.hip): digit-plane images of the
// encoded kernels (built once per plan) and of the rotated inputs (built per call), then one MFMA kernel.
void conv_mfma_geometry(int groups, int cols, int nterm, int *mtiles, int *ntiles, int *kblocks);
size_t conv_mfma_image_bytes(int n, int tiles, int kblocks);
int launch_limb_pack(const gala_ctx *ctx, void *stream, const u64 *src, int mode, int rows, int nterm, u64 *dst);
bool uses_fast_hoist(const gala_ctx *ctx);
int launch_hoist_taps_2048(const gala_ctx *ctx, void *stream, const u64 *ct_in, int batch, const TermList &terms,
                           bool any_rotation, const u64 *keys2, u64 *digits, u64 *xrot);
size_t conv_mfma_tmp_bytes(int n, int mtiles, int ntiles);
// blocks_of_eight: tmp[(i/8)][row][column][i%8] instead of tmp[i][row][column] (what PermJob::in8_S describes)
int launch_conv_mfma(const gala_ctx *ctx, void *stream, const u64 *wl, const u64 *xl, int batch, int groups,
                     int nterm, u64 *tmp, bool blocks_of_eight = false);
int launch_conv_untranspose(const gala_ctx *ctx, void *stream, const u64 *tmp, int batch, int groups, u64 *acc);
int launch_hstperm_pack_2048(const gala_ctx *ctx, void *stream, const u64 *ct_in, u64 *digits, int batch,
                             const TermList &terms, bool any_rotation, const u64 *keys2, u64 *xl);

}  // namespace gala
