// Device-side entry points of the C ABI: argument checks, workspace carving and
// the kernel sequences of Perm, he_fc and he_conv.  No allocation happens here.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <mutex>

#include "gala_internal.h"

using namespace gala;

namespace gala {
int galois_element(int n, int swap, int step);
}

namespace {

// Workgroups the rotate-and-accumulate launch aims for.  Short sums (G < 32: a convolution's kernel orders) get
// what the chip holds at once (256 CUs, three workgroups each at this kernel's register count): every further
// chunk costs a partial ciphertext and a mask round.  Long sums (an FC layer's G rotations) are cut finer, into
// 1280 to 2560 workgroups: chunks of equal length matter more there than a single round (63 rotations in 12 chunks
// leave a third of the workgroups with 6 instead of 5), and a chunk count that is a multiple of eight lets the
// XCD-aware mapping keep every chunk's keys in one L2.  Measured on he_fc 128x1024 and 1000x2048 at batch 64:
// 32 chunks are 4 % and 6 % faster than 12.
// The G rotations of one item are split into this many chunks, each summed by one workgroup.
int choose_chunks(const gala_ctx *ctx, int items, int G) {
    items = std::max(items, 1);
    // With a special prime the kernel holds two workgroups per CU, not three, and a rotation is twice the work:
    // one round of 512 workgroups was the fastest cut for short and long sums alike (he_fc 128x1024: 0.43 ms
    // against 0.48 ms with 2048 workgroups and 0.58 ms with 768).
    if (G < 32 || ctx->special) {
        const int c = ((ctx->special ? 512 : 768) + items - 1) / items;
        return std::max(1, std::min(c, G - 1));     // G-1 entries cost a key switch (chunk_range)
    }
    // a power of two (it divides the padded G, and from 8 on it keeps the XCD mapping): 1280 to 2560 workgroups,
    // halved while a workgroup would be left with a single term and a round of the chip is still filled
    int c = 1;
    while (2 * c * items <= 2560) c *= 2;
    c = std::min(c, G);
    while (c > 1 && G / c < 2 && items * (c / 2) >= 768) c /= 2;
    return std::max(1, c);
}
size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace

// ---------------------------------------------------------------------------
// measurement aid: HIP events around every rotate-and-accumulate launch
// ---------------------------------------------------------------------------
extern "C" int gala_profile_enable(gala_ctx *c, int capacity) {
    if (!c || capacity < 0) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    for (void *e : c->prof_events) (void)hipEventDestroy((hipEvent_t)e);
    c->prof_events.clear();
    c->prof_used = 0;
    for (int i = 0; i < 2 * capacity; ++i) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return GALA_EHIP;
        c->prof_events.push_back((void *)e);
    }
    return GALA_OK;
}
extern "C" int gala_profile_select(gala_ctx *c, int which) {
    if (!c || which < 0 || which > 2) return GALA_EARG;
    c->prof_which = which;
    return GALA_OK;
}
extern "C" int gala_profile_collect(gala_ctx *c, float *ms, int capacity, int *count) {
    if (!c || !ms || !count) return GALA_EARG;
    const int n = std::min(capacity, c->prof_used);
    for (int i = 0; i < n; ++i) {
        hipEvent_t a = (hipEvent_t)c->prof_events[2 * i], b = (hipEvent_t)c->prof_events[2 * i + 1];
        if (hipEventSynchronize(b) != hipSuccess || hipEventElapsedTime(&ms[i], a, b) != hipSuccess) return GALA_EHIP;
    }
    *count = n;
    c->prof_used = 0;
    return GALA_OK;
}

extern "C" int gala_ct_import(const gala_ctx *c, void *stream, const uint64_t *src, int count, uint64_t *dst) {
    if (!c || !src || !dst || count < 0) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    return launch_ntt(c, stream, src, dst, (size_t)count * 2, 0) ? GALA_EHIP : GALA_OK;
}
extern "C" int gala_ct_export(const gala_ctx *c, void *stream, const uint64_t *src, int count, uint64_t *dst) {
    if (!c || !src || !dst || count < 0) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    return launch_ntt(c, stream, src, dst, (size_t)count * 2, 1) ? GALA_EHIP : GALA_OK;
}

extern "C" int gala_encrypt_batch(const gala_ctx *c, void *stream, const gala_sk *sk, const uint64_t *slots,
                                  const uint64_t *seeds, int count, uint64_t *ct) {
    if (!c || !sk || !slots || !seeds || !ct || count < 0) return GALA_EARG;
    if (!c->has_device || !sk->d_s_hat) return GALA_EHIP;
    return launch_encrypt(c, stream, sk->d_s_hat, slots, seeds, count, ct) ? GALA_EHIP : GALA_OK;
}
extern "C" int gala_decrypt_batch(const gala_ctx *c, void *stream, const gala_sk *sk, const uint64_t *ct, int count,
                                  uint64_t *slots) {
    if (!c || !sk || !slots || !ct || count < 0) return GALA_EARG;
    if (!c->has_device || !sk->d_s_hat) return GALA_EHIP;
    return launch_decrypt(c, stream, sk->d_s_hat, ct, count, slots) ? GALA_EHIP : GALA_OK;
}

extern "C" int gala_fc_unpack_share_batch(const gala_fc_plan *pl, void *stream, const uint64_t *slots, int count,
                                          uint64_t *out) {
    if (!pl || !slots || !out || count < 0) return GALA_EARG;
    if (!pl->ctx->has_device) return GALA_EHIP;
    return launch_unpack_share(pl->ctx, stream, slots, count, 1, pl->mask_d, (size_t)pl->n_o, out) ? GALA_EHIP : GALA_OK;
}
extern "C" int gala_conv_unpack_share_batch(const gala_conv_plan *pl, void *stream, const uint64_t *slots, int count,
                                            uint64_t *out) {
    if (!pl || !slots || !out || count < 0) return GALA_EARG;
    if (!pl->ctx->has_device) return GALA_EHIP;
    return launch_unpack_share(pl->ctx, stream, slots, count, pl->nout, pl->mask_d, (size_t)pl->c_o * pl->u_h * pl->u_w, out)
               ? GALA_EHIP
               : GALA_OK;
}

extern "C" int gala_encode_plain(const gala_ctx *c, void *stream, const uint64_t *slots, int count, int mode,
                                 uint64_t *plain) {
    if (!c || !slots || !plain || count < 0 || (mode != 0 && mode != 1)) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    return launch_encode_plain(c, stream, slots, count, mode, plain) ? GALA_EHIP : GALA_OK;
}
extern "C" int gala_add(const gala_ctx *c, void *stream, const uint64_t *a, const uint64_t *b, int count, uint64_t *out) {
    if (!c || !a || !b || !out || count < 0) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    return launch_ct_op(c, stream, 0, a, b, 2 * (size_t)c->n, count, out) ? GALA_EHIP : GALA_OK;
}
namespace {
int plain_op(const gala_ctx *c, void *stream, int op, const uint64_t *ct, const uint64_t *plain, size_t stride, int count,
             uint64_t *out) {
    if (!c || !ct || !plain || !out || count < 0 || (stride != 0 && stride != (size_t)c->n)) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    return launch_ct_op(c, stream, op, ct, plain, stride, count, out) ? GALA_EHIP : GALA_OK;
}
}  // namespace
extern "C" int gala_scmult(const gala_ctx *c, void *stream, const uint64_t *ct, const uint64_t *plain, size_t stride,
                           int count, uint64_t *out) {
    return plain_op(c, stream, 1, ct, plain, stride, count, out);
}
extern "C" int gala_sub_plain(const gala_ctx *c, void *stream, const uint64_t *ct, const uint64_t *plain, size_t stride,
                              int count, uint64_t *out) {
    return plain_op(c, stream, 2, ct, plain, stride, count, out);
}
extern "C" int gala_add_plain(const gala_ctx *c, void *stream, const uint64_t *ct, const uint64_t *plain, size_t stride,
                              int count, uint64_t *out) {
    return plain_op(c, stream, 3, ct, plain, stride, count, out);
}

extern "C" int gala_rotate(const gala_ctx *c, void *stream, const gala_gk *gk, const uint64_t *ct_in, int count,
                           gala_rot rot, uint64_t *ct_out) {
    if (!c || !gk || !ct_in || !ct_out || count < 0 || rot.step < 0 || rot.step >= c->n / 2 || (rot.swap & ~1))
        return GALA_EARG;
    if (ct_in == ct_out) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    const int g = galois_element(c->n, rot.swap, rot.step);
    PermJob job{};
    job.ct_in = ct_in;
    job.in_item_stride = 2 * (size_t)c->n;
    job.in_g_stride = 0;
    job.w = nullptr;
    job.G = 1; job.items = count; job.nchunks = 1; job.slots = 1;
    job.partial = ct_out;
    job.keys = gk->d_keys;
    job.keys2 = gk->d_keys2;
    if (g == 1) {
        job.gal = gk->d_one; job.key_idx = gk->d_one;
    } else {
        auto it = gk->index_of.find(g);
        if (it == gk->index_of.end()) return GALA_ENOKEY;
        job.gal = gk->d_elements + it->second;
        job.key_idx = gk->d_iota + it->second;
    }
    return launch_perm_accumulate(c, stream, job) ? GALA_EHIP : GALA_OK;
}

namespace {
// xrot[b][e] = HstPerm_e(ct of term e of item b) for every term, one DecPerm per input ciphertext that rotates
// (Sec. III-B(1): the rotations of one input share its decomposition).  digits: scratch for the decompositions.
int hoist_terms(const gala_ctx *c, void *stream, const u64 *ct_in, int batch, const TermList &terms, bool rotates,
                const u64 *keys, const u64 *keys2, u64 *digits, u64 *xrot) {
    const int n = c->n;
    const bool fast = uses_fast_hoist(c) && (!rotates || keys2);
    if (fast) return launch_hoist_taps_2048(c, stream, ct_in, batch, terms, rotates, keys2, digits, xrot);
    if (c->special) {
        // every term as a Perm of its own: one workgroup per (item, term)
        PermJob taps{};
        taps.ct_in = ct_in;
        taps.in_item_stride = (size_t)terms.nin * 2 * n;
        taps.in_g_stride = 2 * (size_t)n;
        taps.in_g_index = terms.ct;
        taps.w = nullptr;
        taps.gal = terms.gal; taps.key_idx = terms.key;
        taps.keys = keys; taps.keys2 = keys2;
        taps.G = terms.nterm; taps.items = batch; taps.nchunks = terms.nterm; taps.slots = terms.nterm;
        taps.partial = xrot;
        const int which = c->prof_which;     // these launches are not the ones the events are for
        c->prof_which = -1;
        const int rc = launch_perm_accumulate(c, stream, taps);
        c->prof_which = which;
        return rc;
    }
    if (rotates && launch_decperm(c, stream, ct_in, (size_t)batch * terms.nin, digits)) return 1;
    return launch_hstperm_taps(c, stream, ct_in, digits, batch, terms, keys, xrot);
}
size_t hoist_digit_bytes(const gala_ctx *c, size_t ncts) {
    return align_up(ncts * c->ndigits * c->n * sizeof(u64) * (c->special ? 2 : 1));
}
}  // namespace

extern "C" int gala_gk_count(const gala_gk *gk) { return gk ? (int)gk->elements.size() : GALA_EARG; }
extern "C" size_t gala_rotate_hoisted_workspace(const gala_ctx *c, int count) {
    return (!c || count <= 0) ? 0 : hoist_digit_bytes(c, (size_t)count);
}
extern "C" int gala_rotate_hoisted(const gala_ctx *c, void *stream, const gala_gk *gk, const uint64_t *ct_in, int count,
                                   uint64_t *ct_out, void *workspace, size_t workspace_bytes) {
    if (!c || !gk || !ct_in || !ct_out || count < 0 || ct_in == ct_out) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    const int nkeys = (int)gk->elements.size();
    if (!count || !nkeys) return GALA_OK;
    if (!workspace || workspace_bytes < hoist_digit_bytes(c, (size_t)count)) return GALA_ENOMEM;
    const TermList terms{1, nkeys, gk->d_zeros, gk->d_elements, gk->d_iota};
    return hoist_terms(c, stream, ct_in, count, terms, true, gk->d_keys, gk->d_keys2, (u64 *)workspace, ct_out) ? GALA_EHIP
                                                                                                                : GALA_OK;
}

// ---------------------------------------------------------------------------
// he_fc
// ---------------------------------------------------------------------------
extern "C" size_t gala_he_fc_workspace(const gala_fc_plan *pl, int batch) {
    if (!pl || batch <= 0) return 0;
    const int chunks = choose_chunks(pl->ctx, batch, pl->G);
    return align_up((size_t)batch * (chunks + 1) * 2 * pl->ctx->n * sizeof(u64));
}
extern "C" int gala_he_fc(const gala_ctx *c, void *stream, const gala_fc_plan *pl, const uint64_t *ct_in, int batch,
                          const uint64_t *r, uint64_t mask_seed, uint64_t *ct_out, void *workspace,
                          size_t workspace_bytes, gala_opcount *counts) {
    if (!c || !pl || pl->ctx != c || !ct_in || !ct_out || !r || batch <= 0) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    if (pl->G > 1 && !pl->bound) return GALA_ENOKEY;
    if (!workspace || workspace_bytes < gala_he_fc_workspace(pl, batch)) return GALA_ENOMEM;
    const int n = c->n, chunks = choose_chunks(pl->ctx, batch, pl->G);
    PermJob job{};
    job.ct_in = ct_in;
    job.in_item_stride = 2 * (size_t)n;
    job.in_g_stride = 0;                 // every rotation starts from the same input ciphertext
    job.w = pl->d_w;
    job.gal = pl->d_gal; job.key_idx = pl->d_key_idx;
    job.keys = pl->bound ? pl->bound->d_keys : nullptr;
    job.keys2 = pl->bound ? pl->bound->d_keys2 : nullptr;
    job.w2 = pl->d_w2;
    job.G = pl->G; job.items = batch; job.nchunks = chunks; job.slots = chunks + 1;
    job.partial = (u64 *)workspace;
    FinalizeJob fin{};
    fin.partial = job.partial;
    fin.items = batch; fin.nchunks = chunks; fin.slots = chunks + 1; fin.nout = 1;
    fin.r = r; fin.r_stride = (size_t)pl->n_o;
    fin.mask_seed = mask_seed;
    fin.mask = pl->mask_d;
    fin.ct_out = ct_out;
    if (launch_perm_finalize(c, stream, job, fin)) return GALA_EHIP;
    if (counts) {
        counts->perm = (int64_t)batch * (pl->G - 1);
        counts->scmult = (int64_t)batch * pl->G;
        counts->add = (int64_t)batch * (pl->G - 1);
        counts->decperm_in = counts->hstperm_in = 0;
    }
    return GALA_OK;
}

// ---------------------------------------------------------------------------
// he_fc for callers that cannot allocate: the partial ciphertexts live in a fixed array of the code object
// ---------------------------------------------------------------------------
namespace {
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
// In host code `scratch` is only a handle for hipGetSymbolAddress.  Every device has its own copy of the array at
// its own address, resolved once per device and kept here; host code passes these pointers, never the name.
constexpr int kMaxDevices = 64;
void *scratch_ptr[kMaxDevices];
std::mutex scratch_mu;
}  // namespace

namespace gala {
// Resolves the device address of the fixed scratch array on the current device (called by gala_ctx_create).
int static_scratch_init() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GALA_EHIP;
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (scratch_ptr[dev]) return GALA_OK;
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return GALA_EHIP;
    scratch_ptr[dev] = ptr;
    return GALA_OK;
}
}  // namespace gala

extern "C" size_t gala_he_fc_static_capacity(void) { return kStaticScratchBytes; }
extern "C" int gala_he_fc_static(const gala_ctx *c, void *stream, const gala_fc_plan *pl, const uint64_t *ct_in, int batch,
                                 const uint64_t *r, uint64_t mask_seed, uint64_t *ct_out, gala_opcount *counts) {
    if (!c || !pl || pl->ctx != c || batch <= 0) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    const size_t need = gala_he_fc_workspace(pl, batch);
    if (need > kStaticScratchBytes) return GALA_ENOMEM;      // batch x (chunks + 1) partial ciphertexts do not fit
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return GALA_EHIP;
    if (dev != c->device || dev < 0 || dev >= kMaxDevices) return GALA_EARG;
    void *ptr;
    {
        std::lock_guard<std::mutex> lock(scratch_mu);
        ptr = scratch_ptr[dev];
    }
    if (!ptr) return GALA_EHIP;                               // gala_ctx_create resolves it; no device, no address
    // Every word of the partial ciphertexts that the summing kernel reads has been written by this call's
    // rotate-and-accumulate and mask workgroups, so nothing left by an earlier call needs clearing.
    return gala_he_fc(c, stream, pl, ct_in, batch, r, mask_seed, ct_out, ptr, kStaticScratchBytes, counts);
}

// ---------------------------------------------------------------------------
// he_conv
// ---------------------------------------------------------------------------
namespace {
struct ConvWorkspace {
    size_t digits, xrot, acc, partial, xl, tmp, total;
    int chunks;
    bool mfma;      // the multiply-accumulate of this call runs on the matrix cores
};
ConvWorkspace conv_workspace(const gala_conv_plan *pl, int batch) {
    const gala_ctx *c = pl->ctx;
    const size_t n = c->n, w = sizeof(u64);
    ConvWorkspace ws{};
    ws.chunks = choose_chunks(c, batch * pl->nout, pl->cn);
    ws.mfma = pl->d_wl && batch >= 2;    // from two inputs on (4 of a workgroup's 32 columns) the matrix cores win
    // the one-prime n = 2048 path writes the rotated inputs straight into the product's column image and the Perm
    // kernel reads the product in place: neither the rotated inputs nor the per-ciphertext sums are materialised
    const bool rotates = pl->nrot_terms > 0;
    const bool direct = ws.mfma && !c->special && uses_fast_hoist(c) && (!rotates || (pl->bound && pl->bound->d_keys2));
    ws.digits = 0;
    ws.xrot = ws.digits + hoist_digit_bytes(c, (size_t)batch * pl->nin);
    const bool in8 = ws.mfma && uses_fast_perm(c);
    ws.acc = ws.xrot + (direct ? 0 : align_up((size_t)batch * pl->nterm * 2 * n * w));
    ws.partial = ws.acc + (in8 ? 0 : align_up((size_t)batch * pl->nout * pl->cn * 2 * n * w));
    ws.xl = ws.partial + align_up((size_t)batch * pl->nout * (ws.chunks + 1) * 2 * n * w);
    size_t xl_bytes = 0, tmp_bytes = 0;
    if (ws.mfma) {
        int mt, nt, kb;
        conv_mfma_geometry(pl->nout * pl->cn, 2 * batch, pl->nterm, &mt, &nt, &kb);
        xl_bytes = conv_mfma_image_bytes(c->n, nt, kb);
        tmp_bytes = conv_mfma_tmp_bytes(c->n, mt, nt);
    }
    ws.tmp = ws.xl + align_up(xl_bytes);
    ws.total = ws.tmp + align_up(tmp_bytes);
    return ws;
}
}  // namespace

extern "C" size_t gala_he_conv_workspace(const gala_conv_plan *pl, int batch) {
    if (!pl || batch <= 0) return 0;
    return conv_workspace(pl, batch).total;
}
extern "C" int gala_he_conv(const gala_ctx *c, void *stream, const gala_conv_plan *pl, const uint64_t *ct_in,
                            int batch, const uint64_t *r, uint64_t mask_seed, uint64_t *ct_out, void *workspace,
                            size_t workspace_bytes, gala_opcount *counts) {
    if (!c || !pl || pl->ctx != c || !ct_in || !ct_out || !r || batch <= 0) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    if ((pl->nrot_terms > 0 || pl->cn > 1) && !pl->bound) return GALA_ENOKEY;
    const ConvWorkspace ws = conv_workspace(pl, batch);
    if (!workspace || workspace_bytes < ws.total) return GALA_ENOMEM;
    char *base = (char *)workspace;
    u64 *digits = (u64 *)(base + ws.digits), *xrot = (u64 *)(base + ws.xrot), *acc = (u64 *)(base + ws.acc),
        *partial = (u64 *)(base + ws.partial);
    const int n = c->n;
    const u64 *keys = pl->bound ? pl->bound->d_keys : nullptr;
    // 1. input rotations: one DecPerm per input ciphertext, one HstPerm per term off the central tap
    // 2. ScMult and Add first: one sum per (output block, kernel order)
    const bool rotates = pl->nrot_terms > 0;
    const bool fast_hoist = uses_fast_hoist(c) && (!rotates || (pl->bound && pl->bound->d_keys2));
    const u64 *keys2 = pl->bound ? pl->bound->d_keys2 : nullptr;
    const int nterm = pl->nterm, groups = pl->nout * pl->cn;
    const TermList terms{pl->nin, nterm, pl->d_term_ct, pl->d_term_gal, pl->d_term_key};
    // measurement aid: events around the multiply-accumulate (selection 1) or around the input rotations (2)
    const bool armed = (size_t)(2 * c->prof_used + 1) < c->prof_events.size();
    auto mark_as = [&](int which, int end) {
        if (!armed || c->prof_which != which) return;
        (void)hipEventRecord((hipEvent_t)c->prof_events[2 * c->prof_used + end], (hipStream_t)stream);
        if (end) ++c->prof_used;
    };
    auto mark = [&](int end) { mark_as(1, end); };
    // The n = 2048 Perm kernels read the product's sums in their own blocks of eight coefficients: no transposition
    // pass in between.  With one-prime keys the rotated inputs also go straight into the product's column image.
    const bool direct = ws.mfma && fast_hoist && !c->special;
    const bool in8 = ws.mfma && uses_fast_perm(c);      // both n = 2048 Perm kernels read the blocks of eight
    const u64 *perm_in = acc;
    if (direct) {
        // the rotated inputs go straight into the column image of the matrix-core product
        u64 *xl = (u64 *)(base + ws.xl), *tmp = (u64 *)(base + ws.tmp);
        mark_as(2, 0);
        if (launch_hstperm_pack_2048(c, stream, ct_in, digits, batch, terms, rotates, keys2, xl))
            return GALA_EHIP;
        mark_as(2, 1);
        mark(0);
        if (launch_conv_mfma(c, stream, pl->d_wl, xl, batch, groups, nterm, tmp, in8)) return GALA_EHIP;
        mark(1);
        if (in8) perm_in = tmp;
        else if (launch_conv_untranspose(c, stream, tmp, batch, groups, acc)) return GALA_EHIP;
    } else {
        mark_as(2, 0);
        if (hoist_terms(c, stream, ct_in, batch, terms, rotates, keys, keys2, digits, xrot)) return GALA_EHIP;
        mark_as(2, 1);
        if (ws.mfma) {
            u64 *xl = (u64 *)(base + ws.xl), *tmp = (u64 *)(base + ws.tmp);
            if (launch_limb_pack(c, stream, xrot, 1, 2 * batch, nterm, xl)) return GALA_EHIP;
            mark(0);
            if (launch_conv_mfma(c, stream, pl->d_wl, xl, batch, groups, nterm, tmp, in8)) return GALA_EHIP;
            mark(1);
            if (in8) perm_in = tmp;
            else if (launch_conv_untranspose(c, stream, tmp, batch, groups, acc)) return GALA_EHIP;
        } else {
            mark(0);
            if (launch_conv_mac(c, stream, pl->d_w, xrot, batch, pl->nout, pl->cn, nterm, acc)) return GALA_EHIP;
            mark(1);
        }
    }
    // 3. Perm second: rotate each kernel order into place and add, then subtract the mask
    PermJob job{};
    job.ct_in = perm_in;
    job.in_item_stride = (size_t)pl->cn * 2 * n;
    job.in_g_stride = 2 * (size_t)n;
    if (in8) {
        int mt, nt, kb;
        conv_mfma_geometry(groups, 2 * batch, nterm, &mt, &nt, &kb);
        const size_t rowsP = (size_t)mt * 16, colsP = (size_t)nt * 16;
        job.in8_S = rowsP * colsP * 8;                       // the next eight coefficients
        job.in_g_stride = colsP * 8;                         // the next row of the product
        job.in8_o_stride = (size_t)pl->cn * colsP * 8;       // the rows of the next output ciphertext
        job.in8_nout = pl->nout;
    }
    job.w = nullptr;
    job.gal = pl->d_grp_gal; job.key_idx = pl->d_grp_key;
    job.keys = keys;
    job.keys2 = pl->bound ? pl->bound->d_keys2 : nullptr;
    job.G = pl->cn; job.items = batch * pl->nout; job.nchunks = ws.chunks; job.slots = ws.chunks + 1;
    job.partial = partial;
    FinalizeJob fin{};
    fin.partial = partial;
    fin.items = job.items; fin.nchunks = ws.chunks; fin.slots = ws.chunks + 1; fin.nout = pl->nout;
    fin.r = r; fin.r_stride = (size_t)pl->c_o * pl->u_h * pl->u_w;
    fin.mask_seed = mask_seed;
    fin.mask = pl->mask_d;
    fin.ct_out = ct_out;
    if (launch_perm_finalize(c, stream, job, fin)) return GALA_EHIP;
    if (counts) {
        const int64_t nt = nterm;
        counts->decperm_in = (int64_t)batch * pl->nrot_cts;
        counts->hstperm_in = (int64_t)batch * pl->nrot_terms;
        counts->scmult = (int64_t)batch * pl->nout * pl->cn * nt;
        counts->perm = (int64_t)batch * pl->nout * (pl->cn - 1);
        counts->add = (int64_t)batch * pl->nout * (pl->cn * (nt - 1) + (pl->cn - 1));
    }
    return GALA_OK;
}

// ---------------------------------------------------------------------------
// The paper's comparison schedules on the same kernels (Sec. III-A(2), Sec. III-B(2))
// ---------------------------------------------------------------------------
namespace {
struct HybridWorkspace {
    size_t digits, xrot, s0, s1, total;
};
HybridWorkspace hybrid_workspace(const gala_fc_hybrid_plan *pl, int batch) {
    const gala_ctx *c = pl->ctx;
    const size_t ct = 2 * (size_t)c->n * sizeof(u64);
    HybridWorkspace ws{};
    ws.digits = 0;
    ws.xrot = ws.digits + (pl->G > 1 ? hoist_digit_bytes(c, (size_t)batch) : 0);
    ws.s0 = ws.xrot + (pl->G > 1 ? align_up((size_t)batch * pl->G * ct) : 0);
    ws.s1 = ws.s0 + align_up((size_t)batch * 2 * ct);      // two partial ciphertexts per item in the last step
    ws.total = ws.s1 + align_up((size_t)batch * 2 * ct);
    return ws;
}
}  // namespace

extern "C" size_t gala_he_fc_hybrid_workspace(const gala_fc_hybrid_plan *pl, int batch) {
    return (!pl || batch <= 0) ? 0 : hybrid_workspace(pl, batch).total;
}
// out = RaS( sum_g ScMult(HstPerm_g(ct), w_g) ) - mask: the input rotations share one DecPerm (gala_rotate_hoisted's
// kernels), the products are summed by the convolution's multiply-accumulate with a single row, and every
// rotate-and-sum step is one launch of the rotate-and-accumulate kernel over the pair (identity, rotation) of the
// running ciphertext; the last step also builds and subtracts the mask.
extern "C" int gala_he_fc_hybrid(const gala_ctx *c, void *stream, const gala_fc_hybrid_plan *pl, const uint64_t *ct_in,
                                 int batch, const uint64_t *r, uint64_t mask_seed, uint64_t *ct_out, void *workspace,
                                 size_t workspace_bytes, gala_opcount *counts) {
    if (!c || !pl || pl->ctx != c || !ct_in || !ct_out || !r || batch <= 0) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    const int steps = (int)pl->ras_gal.size(), G = pl->G, n = c->n;
    if ((G > 1 || steps > 0) && !pl->bound) return GALA_ENOKEY;
    const HybridWorkspace ws = hybrid_workspace(pl, batch);
    if (!workspace || workspace_bytes < ws.total) return GALA_ENOMEM;
    char *base = (char *)workspace;
    u64 *digits = (u64 *)(base + ws.digits), *xrot = (u64 *)(base + ws.xrot);
    u64 *buf[2] = {(u64 *)(base + ws.s0), (u64 *)(base + ws.s1)};
    const u64 *keys = pl->bound ? pl->bound->d_keys : nullptr, *keys2 = pl->bound ? pl->bound->d_keys2 : nullptr;
    const int which = c->prof_which;     // the measurement aid brackets the rotate-and-sum launches only
    const u64 *mac_in = ct_in;
    if (G > 1) {
        const TermList terms{1, G, pl->d_in_ct, pl->d_in_gal, pl->d_in_key};
        c->prof_which = -1;
        const int rc = hoist_terms(c, stream, ct_in, batch, terms, true, keys, keys2, digits, xrot);
        c->prof_which = which;
        if (rc) return GALA_EHIP;
        mac_in = xrot;
    }
    if (launch_conv_mac(c, stream, pl->d_w, mac_in, batch, 1, 1, G, buf[0])) return GALA_EHIP;
    int cur = 0;
    for (int k = 0; k < std::max(steps, 1); ++k) {
        const bool last = k + 1 >= steps;
        PermJob job{};
        job.ct_in = buf[cur];
        job.in_item_stride = 2 * (size_t)n;
        job.in_g_stride = 0;                       // both entries read the running ciphertext
        job.w = nullptr;
        job.gal = pl->d_ras_gal + 2 * k; job.key_idx = pl->d_ras_key + 2 * k;
        job.keys = keys; job.keys2 = keys2;
        job.G = steps ? 2 : 1; job.items = batch; job.nchunks = 1;
        job.slots = last ? 2 : 1;
        job.partial = buf[cur ^ 1];
        if (!last) {
            if (launch_perm_accumulate(c, stream, job)) return GALA_EHIP;
        } else {
            FinalizeJob fin{};
            fin.partial = job.partial;
            fin.items = batch; fin.nchunks = 1; fin.slots = 2; fin.nout = 1;
            fin.r = r; fin.r_stride = (size_t)pl->n_o;
            fin.mask_seed = mask_seed;
            fin.mask = pl->mask_d;
            fin.ct_out = ct_out;
            if (launch_perm_finalize(c, stream, job, fin)) return GALA_EHIP;
        }
        cur ^= 1;
    }
    if (counts) {
        counts->perm = (int64_t)batch * steps;
        counts->decperm_in = G > 1 ? batch : 0;
        counts->hstperm_in = (int64_t)batch * (G - 1);
        counts->scmult = (int64_t)batch * G;
        counts->add = (int64_t)batch * (G - 1 + steps);
    }
    return GALA_OK;
}

namespace {
struct OutrotWorkspace {
    size_t digits, xrot, acc, partial, total;
    int chunks;
};
OutrotWorkspace outrot_workspace(const gala_conv_plan *pl, int batch) {
    const gala_ctx *c = pl->ctx;
    const size_t ct = 2 * (size_t)c->n * sizeof(u64);
    OutrotWorkspace ws{};
    ws.chunks = choose_chunks(c, batch * pl->nout, pl->cn * pl->nin);
    ws.digits = 0;
    ws.xrot = ws.digits + hoist_digit_bytes(c, (size_t)batch * pl->nin);
    ws.acc = ws.xrot + align_up((size_t)batch * pl->nterm * ct);
    ws.partial = ws.acc + align_up((size_t)batch * pl->nout * pl->cn * pl->nin * ct);
    ws.total = ws.partial + align_up((size_t)batch * pl->nout * (ws.chunks + 1) * ct);
    return ws;
}
}  // namespace

extern "C" size_t gala_he_conv_outrot_workspace(const gala_conv_plan *pl, int batch) {
    return (!pl || batch <= 0) ? 0 : outrot_workspace(pl, batch).total;
}
// The same plan, keys, input rotations and encoded kernels as gala_he_conv; the products are summed per input
// ciphertext (segments of the term list) and every (output ciphertext, input ciphertext, kernel order) sum is rotated
// on its own before the additions: nin times the Perms of gala_he_conv.
extern "C" int gala_he_conv_outrot(const gala_ctx *c, void *stream, const gala_conv_plan *pl, const uint64_t *ct_in,
                                   int batch, const uint64_t *r, uint64_t mask_seed, uint64_t *ct_out, void *workspace,
                                   size_t workspace_bytes, gala_opcount *counts) {
    if (!c || !pl || pl->ctx != c || !ct_in || !ct_out || !r || batch <= 0) return GALA_EARG;
    if (!c->has_device) return GALA_EHIP;
    if ((pl->nrot_terms > 0 || pl->cn > 1) && !pl->bound) return GALA_ENOKEY;
    const OutrotWorkspace ws = outrot_workspace(pl, batch);
    if (!workspace || workspace_bytes < ws.total) return GALA_ENOMEM;
    char *base = (char *)workspace;
    u64 *digits = (u64 *)(base + ws.digits), *xrot = (u64 *)(base + ws.xrot), *acc = (u64 *)(base + ws.acc),
        *partial = (u64 *)(base + ws.partial);
    const int n = c->n, nin = pl->nin;
    const u64 *keys = pl->bound ? pl->bound->d_keys : nullptr, *keys2 = pl->bound ? pl->bound->d_keys2 : nullptr;
    const TermList terms{nin, pl->nterm, pl->d_term_ct, pl->d_term_gal, pl->d_term_key};
    const int which = c->prof_which;
    c->prof_which = -1;
    const int rc = hoist_terms(c, stream, ct_in, batch, terms, pl->nrot_terms > 0, keys, keys2, digits, xrot);
    c->prof_which = which;
    if (rc) return GALA_EHIP;
    if (launch_conv_mac(c, stream, pl->d_w, xrot, batch, pl->nout, pl->cn, pl->nterm, acc, pl->d_seg_ptr, pl->d_seg_terms, nin))
        return GALA_EHIP;
    PermJob job{};
    job.ct_in = acc;
    job.in_item_stride = (size_t)pl->cn * nin * 2 * n;
    job.in_g_stride = 2 * (size_t)n;
    job.w = nullptr;
    job.gal = pl->d_or_gal; job.key_idx = pl->d_or_key;
    job.keys = keys; job.keys2 = keys2;
    job.G = pl->cn * nin; job.items = batch * pl->nout; job.nchunks = ws.chunks; job.slots = ws.chunks + 1;
    job.partial = partial;
    FinalizeJob fin{};
    fin.partial = partial;
    fin.items = job.items; fin.nchunks = ws.chunks; fin.slots = ws.chunks + 1; fin.nout = pl->nout;
    fin.r = r; fin.r_stride = (size_t)pl->c_o * pl->u_h * pl->u_w;
    fin.mask_seed = mask_seed;
    fin.mask = pl->mask_d;
    fin.ct_out = ct_out;
    if (launch_perm_finalize(c, stream, job, fin)) return GALA_EHIP;
    if (counts) {
        const int64_t nt = pl->nterm;
        counts->decperm_in = (int64_t)batch * pl->nrot_cts;
        counts->hstperm_in = (int64_t)batch * pl->nrot_terms;
        counts->scmult = (int64_t)batch * pl->nout * pl->cn * nt;
        counts->perm = (int64_t)batch * pl->nout * nin * (pl->cn - 1);
        counts->add = (int64_t)batch * pl->nout * (pl->cn * (nt - nin) + nin * (pl->cn - 1) + (nin - 1));
    }
    return GALA_OK;
}
