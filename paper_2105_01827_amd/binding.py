"""Thin ctypes binding of the C ABI declared in ``include/gala.h``.

Argument marshalling only: every step of the layers runs inside
``libgala_hip.so``.  PyTorch is used by callers for device memory and streams;
this module takes any object with ``data_ptr()`` (or a raw integer address) for
device pointers and numpy ``uint64`` arrays for host pointers.  The library
must be present: there is no fallback path.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgala_hip.so")

GALA_OK, GALA_EARG, GALA_ESHAPE, GALA_ENOKEY, GALA_ENOMEM, GALA_EHIP = 0, -1, -2, -3, -4, -5
_NAMES = {GALA_EARG: "GALA_EARG (bad argument)", GALA_ESHAPE: "GALA_ESHAPE (shape not supported)",
          GALA_ENOKEY: "GALA_ENOKEY (Galois key missing or plan not bound)",
          GALA_ENOMEM: "GALA_ENOMEM (allocation failed or workspace too small)",
          GALA_EHIP: "GALA_EHIP (HIP call failed or no device)"}


class GalaError(RuntimeError):
    def __init__(self, code, where):
        super().__init__(f"{where}: {_NAMES.get(code, code)}")
        self.code = code


class Params(C.Structure):
    _fields_ = [("n", C.c_int32), ("gadget_bits", C.c_int32), ("q", C.c_uint64), ("p", C.c_uint64),
                ("special_prime", C.c_uint64)]


class Rot(C.Structure):
    _fields_ = [("swap", C.c_int32), ("step", C.c_int32)]


class ConvTiling(C.Structure):
    _fields_ = [(k, C.c_int32) for k in ("in_h", "in_w", "k_h", "k_w", "stride", "tile_h", "tile_w", "tiles_y",
                                         "tiles_x", "step_y", "step_x", "halo_y", "halo_x", "out_h", "out_w")]

    @property
    def tiles(self):
        return self.tiles_y * self.tiles_x


class ConvPolyphase(C.Structure):
    _fields_ = ([(k, C.c_int32) for k in ("c_i", "in_h", "in_w", "k_h", "k_w", "stride", "phases_y", "phases_x")] +
                [("phase_y", C.c_int32 * 8), ("phase_x", C.c_int32 * 8)] +
                [(k, C.c_int32) for k in ("c_i_poly", "k_h_poly", "k_w_poly", "out_h", "out_w")])


class OpCount(C.Structure):
    _fields_ = [("perm", C.c_int64), ("decperm_in", C.c_int64), ("hstperm_in", C.c_int64),
                ("scmult", C.c_int64), ("add", C.c_int64)]

    def as_dict(self):
        return {k: int(getattr(self, k)) for k, _ in self._fields_}


_VP, _U64P, _I = C.c_void_p, C.c_void_p, C.c_int
# name -> (restype, argtypes); the list mirrors include/gala.h one to one
SIGNATURES = {
    "gala_ctx_create": (_I, [C.POINTER(Params), C.POINTER(_VP)]),
    "gala_ctx_destroy": (None, [_VP]),
    "gala_ctx_ndigits": (_I, [_VP]),
    "gala_ctx_delta": (C.c_uint64, [_VP]),
    "gala_gauss_cdf": (C.POINTER(C.c_uint64), []),
    "gala_mix64": (C.c_uint64, [C.c_uint64]),
    "gala_rand64": (C.c_uint64, [C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint64]),
    "gala_profile_enable": (_I, [_VP, _I]),
    "gala_profile_select": (_I, [_VP, _I]),
    "gala_profile_collect": (_I, [_VP, C.POINTER(C.c_float), _I, C.POINTER(_I)]),
    "gala_keygen": (_I, [_VP, C.c_uint64, C.POINTER(_VP)]),
    "gala_sk_destroy": (None, [_VP]),
    "gala_sk_export": (_I, [_VP, _VP, _U64P]),
    "gala_galois_keygen": (_I, [_VP, _VP, C.POINTER(Rot), _I, C.c_uint64, C.POINTER(_VP)]),
    "gala_gk_destroy": (None, [_VP]),
    "gala_gk_export": (_I, [_VP, _VP, Rot, _U64P]),
    "gala_encode": (_I, [_VP, _U64P, _U64P]),
    "gala_decode": (_I, [_VP, _U64P, _U64P]),
    "gala_encrypt": (_I, [_VP, _VP, _U64P, C.c_uint64, _U64P]),
    "gala_decrypt": (_I, [_VP, _VP, _U64P, _U64P]),
    "gala_ct_import": (_I, [_VP, _VP, _U64P, _I, _U64P]),
    "gala_ct_export": (_I, [_VP, _VP, _U64P, _I, _U64P]),
    "gala_encrypt_batch": (_I, [_VP, _VP, _VP, _U64P, _U64P, _I, _U64P]),
    "gala_decrypt_batch": (_I, [_VP, _VP, _VP, _U64P, _I, _U64P]),
    "gala_fc_unpack_share_batch": (_I, [_VP, _VP, _U64P, _I, _U64P]),
    "gala_conv_unpack_share_batch": (_I, [_VP, _VP, _U64P, _I, _U64P]),
    "gala_encode_plain": (_I, [_VP, _VP, _U64P, _I, _I, _U64P]),
    "gala_add": (_I, [_VP, _VP, _U64P, _U64P, _I, _U64P]),
    "gala_scmult": (_I, [_VP, _VP, _U64P, _U64P, C.c_size_t, _I, _U64P]),
    "gala_sub_plain": (_I, [_VP, _VP, _U64P, _U64P, C.c_size_t, _I, _U64P]),
    "gala_add_plain": (_I, [_VP, _VP, _U64P, _U64P, C.c_size_t, _I, _U64P]),
    "gala_rotate": (_I, [_VP, _VP, _VP, _U64P, _I, Rot, _U64P]),
    "gala_gk_count": (_I, [_VP]),
    "gala_rotate_hoisted_workspace": (C.c_size_t, [_VP, _I]),
    "gala_rotate_hoisted": (_I, [_VP, _VP, _VP, _U64P, _I, _U64P, _VP, C.c_size_t]),
    "gala_fc_plan_create": (_I, [_VP, _U64P, _I, _I, C.POINTER(_VP)]),
    "gala_fc_plan_destroy": (None, [_VP]),
    "gala_fc_plan_G": (_I, [_VP]),
    "gala_fc_plan_rotations": (_I, [_VP, C.POINTER(Rot), C.POINTER(_I)]),
    "gala_fc_plan_bind": (_I, [_VP, _VP]),
    "gala_fc_pack_input": (_I, [_VP, _U64P, _U64P]),
    "gala_fc_unpack_share": (_I, [_VP, _U64P, _U64P]),
    "gala_he_fc_workspace": (C.c_size_t, [_VP, _I]),
    "gala_he_fc": (_I, [_VP, _VP, _VP, _U64P, _I, _U64P, C.c_uint64, _U64P, _VP, C.c_size_t, C.POINTER(OpCount)]),
    "gala_he_fc_static_capacity": (C.c_size_t, []),
    "gala_he_fc_static": (_I, [_VP, _VP, _VP, _U64P, _I, _U64P, C.c_uint64, _U64P, C.POINTER(OpCount)]),
    "gala_conv_plan_create": (_I, [_VP, _U64P, _I, _I, _I, _I, _I, _I, C.POINTER(_VP)]),
    "gala_conv_plan_destroy": (None, [_VP]),
    "gala_conv_plan_prepare_batched": (_I, [_VP]),
    "gala_conv_plan_geometry": (_I, [_VP, C.POINTER(C.c_int32)]),
    "gala_conv_plan_rotations": (_I, [_VP, C.POINTER(Rot), C.POINTER(_I)]),
    "gala_conv_plan_bind": (_I, [_VP, _VP]),
    "gala_conv_pack_input": (_I, [_VP, _U64P, _U64P]),
    "gala_conv_unpack_share": (_I, [_VP, _I, _U64P, _U64P]),
    "gala_he_conv_workspace": (C.c_size_t, [_VP, _I]),
    "gala_he_conv": (_I, [_VP, _VP, _VP, _U64P, _I, _U64P, C.c_uint64, _U64P, _VP, C.c_size_t, C.POINTER(OpCount)]),
    "gala_fc_hybrid_plan_create": (_I, [_VP, _U64P, _I, _I, C.POINTER(_VP)]),
    "gala_fc_hybrid_plan_destroy": (None, [_VP]),
    "gala_fc_hybrid_plan_G": (_I, [_VP]),
    "gala_fc_hybrid_plan_steps": (_I, [_VP]),
    "gala_fc_hybrid_plan_rotations": (_I, [_VP, C.POINTER(Rot), C.POINTER(_I)]),
    "gala_fc_hybrid_plan_bind": (_I, [_VP, _VP]),
    "gala_fc_hybrid_pack_input": (_I, [_VP, _U64P, _U64P]),
    "gala_fc_hybrid_unpack": (_I, [_VP, _U64P, _U64P]),
    "gala_he_fc_hybrid_workspace": (C.c_size_t, [_VP, _I]),
    "gala_he_fc_hybrid": (_I, [_VP, _VP, _VP, _U64P, _I, _U64P, C.c_uint64, _U64P, _VP, C.c_size_t, C.POINTER(OpCount)]),
    "gala_he_conv_outrot_workspace": (C.c_size_t, [_VP, _I]),
    "gala_he_conv_outrot": (_I, [_VP, _VP, _VP, _U64P, _I, _U64P, C.c_uint64, _U64P, _VP, C.c_size_t, C.POINTER(OpCount)]),
    "gala_conv_tiling_plan": (_I, [_VP, _I, _I, _I, _I, _I, C.POINTER(ConvTiling)]),
    "gala_conv_tile_extract": (_I, [C.POINTER(ConvTiling), _I, _U64P, _I, _U64P]),
    "gala_conv_tile_mask": (_I, [C.POINTER(ConvTiling), _I, _U64P, _I, _U64P]),
    "gala_conv_tile_scatter": (_I, [C.POINTER(ConvTiling), _I, _U64P, _I, _U64P]),
    "gala_conv_polyphase_plan": (_I, [_I, _I, _I, _I, _I, _I, C.POINTER(ConvPolyphase)]),
    "gala_conv_polyphase_kernel": (_I, [C.POINTER(ConvPolyphase), _I, _U64P, _U64P]),
    "gala_conv_polyphase_input": (_I, [C.POINTER(ConvPolyphase), _U64P, _U64P]),
}

_lib = None


def load():
    """Load libgala_hip.so (built by ``paper_2105_01827_amd.build``); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2105_01827_amd.build` "
                              "(there is no CPU fallback for the HIP path)")
        # PyTorch ships a HIP runtime of its own; when a process uses both, that copy has to be the one that
        # is loaded first, or torch finds no device afterwards.  Callers pass torch tensors, so import it here.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            f = getattr(lib, name)
            f.restype, f.argtypes = res, args
        _lib = lib
    return _lib


def _check(code, where):
    if code != GALA_OK:
        raise GalaError(code, where)


def _host(a):
    a = np.ascontiguousarray(np.asarray(a, dtype=np.uint64))
    return a, a.ctypes.data_as(C.c_void_p)


def _dev(t):
    """Address of a device buffer: a torch tensor (uint64/int64 storage) or an int."""
    return C.c_void_p(t if isinstance(t, int) else t.data_ptr())


def _stream(s):
    if s is None:
        return None
    return C.c_void_p(s if isinstance(s, int) else s.cuda_stream)


def _rots(rots):
    arr = (Rot * max(1, len(rots)))()
    for i, (swap, step) in enumerate(rots):
        arr[i].swap, arr[i].step = int(swap), int(step)
    return arr


class Context:
    """gala_ctx: one BFV parameter set; device tables live on the current HIP device."""

    def __init__(self, n, q, p, gadget_bits, special=0):
        self.lib = load()
        self.n, self.q, self.p, self.gadget_bits, self.special = n, q, p, gadget_bits, special
        par = Params(n, gadget_bits, q, p, special)
        h = C.c_void_p()
        _check(self.lib.gala_ctx_create(C.byref(par), C.byref(h)), "gala_ctx_create")
        self.h = h
        self.ndigits = self.lib.gala_ctx_ndigits(h)
        self.delta = int(self.lib.gala_ctx_delta(h))
        self.ksk_words = self.ndigits * (4 if special else 2) * n

    def close(self):
        if getattr(self, "h", None):
            self.lib.gala_ctx_destroy(self.h)
            self.h = None

    __del__ = close

    def gauss_cdf(self):
        ptr = self.lib.gala_gauss_cdf()
        return [int(ptr[i]) for i in range(38)]

    def profile_enable(self, capacity):
        _check(self.lib.gala_profile_enable(self.h, capacity), "gala_profile_enable")

    def profile_select(self, which):
        _check(self.lib.gala_profile_select(self.h, which), "gala_profile_select")

    def profile_collect(self, capacity):
        ms = (C.c_float * max(1, capacity))(); n = C.c_int()
        _check(self.lib.gala_profile_collect(self.h, ms, capacity, C.byref(n)), "gala_profile_collect")
        return [float(ms[i]) for i in range(n.value)]

    # ---- client side (host)
    def keygen(self, seed):
        return SecretKey(self, seed)

    def encode(self, slots):
        s, sp = _host(slots); out = np.empty(self.n, np.uint64)
        _check(self.lib.gala_encode(self.h, sp, out.ctypes.data_as(C.c_void_p)), "gala_encode"); return out

    def decode(self, poly_p):
        a, ap = _host(poly_p); out = np.empty(self.n, np.uint64)
        _check(self.lib.gala_decode(self.h, ap, out.ctypes.data_as(C.c_void_p)), "gala_decode"); return out

    def encrypt(self, sk, slots, seed):
        s, sp = _host(slots); ct = np.empty(2 * self.n, np.uint64)
        _check(self.lib.gala_encrypt(self.h, sk.h, sp, seed, ct.ctypes.data_as(C.c_void_p)), "gala_encrypt"); return ct

    def decrypt(self, sk, ct):
        c, cp = _host(ct); out = np.empty(self.n, np.uint64)
        _check(self.lib.gala_decrypt(self.h, sk.h, cp, out.ctypes.data_as(C.c_void_p)), "gala_decrypt"); return out

    def galois_keygen(self, sk, rots, seed):
        return GaloisKeys(self, sk, rots, seed)

    # ---- device side
    def ct_import(self, src_dev, count, dst_dev, stream=None):
        _check(self.lib.gala_ct_import(self.h, _stream(stream), _dev(src_dev), count, _dev(dst_dev)), "gala_ct_import")

    def ct_export(self, src_dev, count, dst_dev, stream=None):
        _check(self.lib.gala_ct_export(self.h, _stream(stream), _dev(src_dev), count, _dev(dst_dev)), "gala_ct_export")

    def encrypt_batch(self, sk, slots_dev, seeds_dev, count, ct_dev, stream=None):
        _check(self.lib.gala_encrypt_batch(self.h, _stream(stream), sk.h, _dev(slots_dev), _dev(seeds_dev), count,
                                           _dev(ct_dev)), "gala_encrypt_batch")

    def decrypt_batch(self, sk, ct_dev, count, slots_dev, stream=None):
        _check(self.lib.gala_decrypt_batch(self.h, _stream(stream), sk.h, _dev(ct_dev), count, _dev(slots_dev)),
               "gala_decrypt_batch")

    def encode_plain(self, slots_dev, count, mode, plain_dev, stream=None):
        _check(self.lib.gala_encode_plain(self.h, _stream(stream), _dev(slots_dev), count, mode, _dev(plain_dev)),
               "gala_encode_plain")

    def add(self, a, b, count, out, stream=None):
        _check(self.lib.gala_add(self.h, _stream(stream), _dev(a), _dev(b), count, _dev(out)), "gala_add")

    def scmult(self, ct, plain, count, out, shared=False, stream=None):
        _check(self.lib.gala_scmult(self.h, _stream(stream), _dev(ct), _dev(plain), 0 if shared else self.n, count,
                                    _dev(out)), "gala_scmult")

    def sub_plain(self, ct, plain, count, out, shared=False, stream=None):
        _check(self.lib.gala_sub_plain(self.h, _stream(stream), _dev(ct), _dev(plain), 0 if shared else self.n, count,
                                       _dev(out)), "gala_sub_plain")

    def add_plain(self, ct, plain, count, out, shared=False, stream=None):
        _check(self.lib.gala_add_plain(self.h, _stream(stream), _dev(ct), _dev(plain), 0 if shared else self.n, count,
                                       _dev(out)), "gala_add_plain")

    def rotate(self, gk, ct_in, count, rot, ct_out, stream=None):
        _check(self.lib.gala_rotate(self.h, _stream(stream), gk.h, _dev(ct_in), count, Rot(*rot), _dev(ct_out)),
               "gala_rotate")

    def rotate_hoisted_workspace(self, count):
        return int(self.lib.gala_rotate_hoisted_workspace(self.h, count))

    def rotate_hoisted(self, gk, ct_in, count, ct_out, workspace, workspace_bytes, stream=None):
        _check(self.lib.gala_rotate_hoisted(self.h, _stream(stream), gk.h, _dev(ct_in), count, _dev(ct_out),
                                            _dev(workspace), workspace_bytes), "gala_rotate_hoisted")

    def fc_plan(self, W):
        return FcPlan(self, W)

    # ---- spatial tiling / stride helpers (host)
    def conv_tiling(self, in_h, in_w, k_h, k_w, stride):
        t = ConvTiling()
        _check(self.lib.gala_conv_tiling_plan(self.h, in_h, in_w, k_h, k_w, stride, C.byref(t)), "gala_conv_tiling_plan")
        return t

    def tile_extract(self, t, image, tile):
        a, ap = _host(image); ch = a.shape[0]; out = np.empty((ch, t.tile_h, t.tile_w), np.uint64)
        _check(self.lib.gala_conv_tile_extract(C.byref(t), ch, ap, tile, out.ctypes.data_as(C.c_void_p)),
               "gala_conv_tile_extract")
        return out

    def tile_mask(self, t, r, tile):
        a, ap = _host(r); ch = a.shape[0]; out = np.empty((ch, t.tile_h, t.tile_w), np.uint64)
        _check(self.lib.gala_conv_tile_mask(C.byref(t), ch, ap, tile, out.ctypes.data_as(C.c_void_p)),
               "gala_conv_tile_mask")
        return out

    def tile_scatter(self, t, vals, tile, out):
        a, ap = _host(vals); ch = a.shape[0]
        assert out.dtype == np.uint64 and out.flags["C_CONTIGUOUS"] and out.shape == (ch, t.out_h, t.out_w)
        _check(self.lib.gala_conv_tile_scatter(C.byref(t), ch, ap, tile, out.ctypes.data_as(C.c_void_p)),
               "gala_conv_tile_scatter")

    # ---- stride as a polyphase split (host)
    def conv_polyphase(self, c_i, in_h, in_w, k_h, k_w, stride):
        pp = ConvPolyphase()
        _check(self.lib.gala_conv_polyphase_plan(c_i, in_h, in_w, k_h, k_w, stride, C.byref(pp)),
               "gala_conv_polyphase_plan")
        return pp

    def polyphase_kernel(self, pp, K):
        a, ap = _host(K); c_o = a.shape[0]
        assert a.shape[1:] == (pp.c_i, pp.k_h, pp.k_w)
        out = np.empty((c_o, pp.c_i_poly, pp.k_h_poly, pp.k_w_poly), np.uint64)
        _check(self.lib.gala_conv_polyphase_kernel(C.byref(pp), c_o, ap, out.ctypes.data_as(C.c_void_p)),
               "gala_conv_polyphase_kernel")
        return out

    def polyphase_input(self, pp, x):
        a, ap = _host(x)
        assert a.shape == (pp.c_i, pp.in_h, pp.in_w)
        out = np.empty((pp.c_i_poly, pp.out_h, pp.out_w), np.uint64)
        _check(self.lib.gala_conv_polyphase_input(C.byref(pp), ap, out.ctypes.data_as(C.c_void_p)),
               "gala_conv_polyphase_input")
        return out

    def conv_plan(self, K, u_h, u_w):
        return ConvPlan(self, K, u_h, u_w)

    def fc_hybrid_plan(self, W):
        return FcHybridPlan(self, W)


class SecretKey:
    def __init__(self, ctx, seed):
        self.ctx = ctx
        h = C.c_void_p()
        _check(ctx.lib.gala_keygen(ctx.h, seed, C.byref(h)), "gala_keygen")
        self.h = h

    def export(self):
        out = np.empty(self.ctx.n, np.uint64)
        _check(self.ctx.lib.gala_sk_export(self.ctx.h, self.h, out.ctypes.data_as(C.c_void_p)), "gala_sk_export")
        return out

    def __del__(self):
        if getattr(self, "h", None):
            self.ctx.lib.gala_sk_destroy(self.h)
            self.h = None


class GaloisKeys:
    def __init__(self, ctx, sk, rots, seed):
        self.ctx = ctx
        h = C.c_void_p()
        _check(ctx.lib.gala_galois_keygen(ctx.h, sk.h, _rots(rots), len(rots), seed, C.byref(h)), "gala_galois_keygen")
        self.h = h

    @property
    def count(self):
        return int(self.ctx.lib.gala_gk_count(self.h))

    def export(self, rot):
        out = np.empty(self.ctx.ksk_words, np.uint64)
        _check(self.ctx.lib.gala_gk_export(self.ctx.h, self.h, Rot(*rot), out.ctypes.data_as(C.c_void_p)),
               "gala_gk_export")
        return out

    def __del__(self):
        if getattr(self, "h", None):
            self.ctx.lib.gala_gk_destroy(self.h)
            self.h = None


class FcPlan:
    """gala_fc_plan: the row-wise encoded weights of one FC layer."""

    def __init__(self, ctx, W):
        self.ctx = ctx
        W, wp = _host(W)
        self.n_o, self.n_i = W.shape
        h = C.c_void_p()
        _check(ctx.lib.gala_fc_plan_create(ctx.h, wp, self.n_o, self.n_i, C.byref(h)), "gala_fc_plan_create")
        self.h = h
        self.G = ctx.lib.gala_fc_plan_G(h)

    def rotations(self):
        n = C.c_int()
        _check(self.ctx.lib.gala_fc_plan_rotations(self.h, None, C.byref(n)), "gala_fc_plan_rotations")
        arr = (Rot * max(1, n.value))()
        _check(self.ctx.lib.gala_fc_plan_rotations(self.h, arr, C.byref(n)), "gala_fc_plan_rotations")
        return [(arr[i].swap, arr[i].step) for i in range(n.value)]

    def bind(self, gk):
        _check(self.ctx.lib.gala_fc_plan_bind(self.h, gk.h), "gala_fc_plan_bind")
        self._gk = gk

    def pack_input(self, x):
        x, xp = _host(x); out = np.empty(self.ctx.n, np.uint64)
        _check(self.ctx.lib.gala_fc_pack_input(self.h, xp, out.ctypes.data_as(C.c_void_p)), "gala_fc_pack_input")
        return out

    def unpack_share(self, slots):
        s, sp = _host(slots); out = np.empty(self.n_o, np.uint64)
        _check(self.ctx.lib.gala_fc_unpack_share(self.h, sp, out.ctypes.data_as(C.c_void_p)), "gala_fc_unpack_share")
        return out

    def unpack_share_batch(self, slots_dev, count, out_dev, stream=None):
        _check(self.ctx.lib.gala_fc_unpack_share_batch(self.h, _stream(stream), _dev(slots_dev), count, _dev(out_dev)),
               "gala_fc_unpack_share_batch")

    def workspace_bytes(self, batch):
        return int(self.ctx.lib.gala_he_fc_workspace(self.h, batch))

    def he_fc(self, ct_in, batch, r, mask_seed, ct_out, workspace, workspace_bytes, stream=None):
        cnt = OpCount()
        _check(self.ctx.lib.gala_he_fc(self.ctx.h, _stream(stream), self.h, _dev(ct_in), batch, _dev(r), mask_seed,
                                       _dev(ct_out), _dev(workspace), workspace_bytes, C.byref(cnt)), "gala_he_fc")
        return cnt.as_dict()

    def he_fc_static(self, ct_in, batch, r, mask_seed, ct_out, stream=None):
        cnt = OpCount()
        _check(self.ctx.lib.gala_he_fc_static(self.ctx.h, _stream(stream), self.h, _dev(ct_in), batch, _dev(r), mask_seed,
                                              _dev(ct_out), C.byref(cnt)), "gala_he_fc_static")
        return cnt.as_dict()

    def __del__(self):
        if getattr(self, "h", None):
            self.ctx.lib.gala_fc_plan_destroy(self.h)
            self.h = None


class FcHybridPlan:
    """gala_fc_hybrid_plan: the hybrid matrix-vector product of Sec. III-A(2), the paper's comparison schedule."""

    def __init__(self, ctx, W):
        self.ctx = ctx
        W, wp = _host(W)
        self.n_o, self.n_i = W.shape
        h = C.c_void_p()
        _check(ctx.lib.gala_fc_hybrid_plan_create(ctx.h, wp, self.n_o, self.n_i, C.byref(h)), "gala_fc_hybrid_plan_create")
        self.h = h
        self.G = ctx.lib.gala_fc_hybrid_plan_G(h)
        self.steps = ctx.lib.gala_fc_hybrid_plan_steps(h)

    def rotations(self):
        n = C.c_int()
        _check(self.ctx.lib.gala_fc_hybrid_plan_rotations(self.h, None, C.byref(n)), "gala_fc_hybrid_plan_rotations")
        arr = (Rot * max(1, n.value))()
        _check(self.ctx.lib.gala_fc_hybrid_plan_rotations(self.h, arr, C.byref(n)), "gala_fc_hybrid_plan_rotations")
        return [(arr[i].swap, arr[i].step) for i in range(n.value)]

    def bind(self, gk):
        _check(self.ctx.lib.gala_fc_hybrid_plan_bind(self.h, gk.h), "gala_fc_hybrid_plan_bind")
        self._gk = gk

    def pack_input(self, x):
        x, xp = _host(x); out = np.empty(self.ctx.n, np.uint64)
        _check(self.ctx.lib.gala_fc_hybrid_pack_input(self.h, xp, out.ctypes.data_as(C.c_void_p)), "gala_fc_hybrid_pack_input")
        return out

    def unpack(self, slots):
        s, sp = _host(slots); out = np.empty(self.n_o, np.uint64)
        _check(self.ctx.lib.gala_fc_hybrid_unpack(self.h, sp, out.ctypes.data_as(C.c_void_p)), "gala_fc_hybrid_unpack")
        return out

    def workspace_bytes(self, batch):
        return int(self.ctx.lib.gala_he_fc_hybrid_workspace(self.h, batch))

    def he_fc_hybrid(self, ct_in, batch, r, mask_seed, ct_out, workspace, workspace_bytes, stream=None):
        cnt = OpCount()
        _check(self.ctx.lib.gala_he_fc_hybrid(self.ctx.h, _stream(stream), self.h, _dev(ct_in), batch, _dev(r), mask_seed,
                                              _dev(ct_out), _dev(workspace), workspace_bytes, C.byref(cnt)),
               "gala_he_fc_hybrid")
        return cnt.as_dict()

    def __del__(self):
        if getattr(self, "h", None):
            self.ctx.lib.gala_fc_hybrid_plan_destroy(self.h)
            self.h = None


class ConvPlan:
    """gala_conv_plan: the kernel-grouping encoding of one convolution layer."""

    def __init__(self, ctx, K, u_h, u_w):
        self.ctx = ctx
        K, kp = _host(K)
        self.c_o, self.c_i, self.k_h, self.k_w = K.shape
        self.u_h, self.u_w = u_h, u_w
        h = C.c_void_p()
        _check(ctx.lib.gala_conv_plan_create(ctx.h, kp, self.c_o, self.c_i, self.k_h, self.k_w, u_h, u_w, C.byref(h)),
               "gala_conv_plan_create")
        self.h = h
        g = (C.c_int32 * 6)()
        _check(ctx.lib.gala_conv_plan_geometry(h, g), "gala_conv_plan_geometry")
        self.T, self.cn, self.nin, self.nout, self.ntap, self.nterm = (int(v) for v in g)

    def rotations(self):
        n = C.c_int()
        _check(self.ctx.lib.gala_conv_plan_rotations(self.h, None, C.byref(n)), "gala_conv_plan_rotations")
        arr = (Rot * max(1, n.value))()
        _check(self.ctx.lib.gala_conv_plan_rotations(self.h, arr, C.byref(n)), "gala_conv_plan_rotations")
        return [(arr[i].swap, arr[i].step) for i in range(n.value)]

    def bind(self, gk):
        _check(self.ctx.lib.gala_conv_plan_bind(self.h, gk.h), "gala_conv_plan_bind")
        self._gk = gk

    def prepare_batched(self):
        _check(self.ctx.lib.gala_conv_plan_prepare_batched(self.h), "gala_conv_plan_prepare_batched")

    def pack_input(self, x):
        x, xp = _host(x); out = np.empty((self.nin, self.ctx.n), np.uint64)
        _check(self.ctx.lib.gala_conv_pack_input(self.h, xp, out.ctypes.data_as(C.c_void_p)), "gala_conv_pack_input")
        return out

    def unpack_share(self, O, slots, out):
        s, sp = _host(slots)
        assert out.dtype == np.uint64 and out.flags["C_CONTIGUOUS"]
        _check(self.ctx.lib.gala_conv_unpack_share(self.h, O, sp, out.ctypes.data_as(C.c_void_p)),
               "gala_conv_unpack_share")

    def unpack_share_batch(self, slots_dev, count, out_dev, stream=None):
        _check(self.ctx.lib.gala_conv_unpack_share_batch(self.h, _stream(stream), _dev(slots_dev), count, _dev(out_dev)),
               "gala_conv_unpack_share_batch")

    def workspace_bytes(self, batch):
        return int(self.ctx.lib.gala_he_conv_workspace(self.h, batch))

    def outrot_workspace_bytes(self, batch):
        return int(self.ctx.lib.gala_he_conv_outrot_workspace(self.h, batch))

    def he_conv_outrot(self, ct_in, batch, r, mask_seed, ct_out, workspace, workspace_bytes, stream=None):
        cnt = OpCount()
        _check(self.ctx.lib.gala_he_conv_outrot(self.ctx.h, _stream(stream), self.h, _dev(ct_in), batch, _dev(r), mask_seed,
                                                _dev(ct_out), _dev(workspace), workspace_bytes, C.byref(cnt)),
               "gala_he_conv_outrot")
        return cnt.as_dict()

    def he_conv(self, ct_in, batch, r, mask_seed, ct_out, workspace, workspace_bytes, stream=None):
        cnt = OpCount()
        _check(self.ctx.lib.gala_he_conv(self.ctx.h, _stream(stream), self.h, _dev(ct_in), batch, _dev(r), mask_seed,
                                         _dev(ct_out), _dev(workspace), workspace_bytes, C.byref(cnt)), "gala_he_conv")
        return cnt.as_dict()

    def __del__(self):
        if getattr(self, "h", None):
            self.ctx.lib.gala_conv_plan_destroy(self.h)
            self.h = None
