"""ctypes wrapper around ``gala_oracle.c`` -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this module.  It marshals numpy ``uint64`` arrays into
the C oracle and holds no arithmetic of its own.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gala_oracle.c")
_LIB = os.path.join(_HERE, "libgala_oracle.so")


def build(force=False):
    """Compile the C oracle with gcc (plain -O2, OpenMP over batch items only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


class Counts(C.Structure):
    _fields_ = [("perm", C.c_int64), ("decperm_in", C.c_int64), ("hstperm_in", C.c_int64),
                ("scmult", C.c_int64), ("add", C.c_int64)]

    def as_dict(self):
        return {k: int(getattr(self, k)) for k, _ in self._fields_}


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_ctx_new.restype = C.c_void_p
        _lib.orc_ctx_new.argtypes = [C.c_int, C.c_uint64, C.c_uint64, C.c_int]
        for name in ("orc_delta", "orc_zeta", "orc_psi", "orc_rand64", "orc_mix64", "orc_uniform", "orc_noise"):
            getattr(_lib, name).restype = C.c_uint64
        _lib.orc_gauss_cdf.restype = C.POINTER(C.c_uint64)
    return _lib


def _p(a):
    assert a.dtype == np.uint64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.c_void_p)


def _u64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.uint64))


class Oracle:
    """One parameter set (n, q, p, gadget_bits); `special` > 0 turns on special-prime key switching."""

    def __init__(self, n, q, p, gadget_bits, special=0):
        self.L = lib()
        self.n, self.q, self.p, self.gadget_bits = n, q, p, gadget_bits
        self.h = C.c_void_p(self.L.orc_ctx_new(n, C.c_uint64(q), C.c_uint64(p), gadget_bits))
        if not self.h:
            raise ValueError("oracle: unsupported parameters")
        self.special = int(special)
        if special and self.L.orc_ctx_set_special(self.h, C.c_uint64(special)) != 0:
            raise ValueError("oracle: unsupported special prime")
        self.ndigits = self.L.orc_ndigits(self.h)
        self.delta = int(self.L.orc_delta(self.h))
        self.zeta = int(self.L.orc_zeta(self.h))
        self.psi = int(self.L.orc_psi(self.h))
        self.ksk_words = self.ndigits * self.L.orc_key_polys(self.h) * n

    def __del__(self):
        try:
            self.L.orc_ctx_free(self.h)
        except Exception:
            pass

    # ---- transforms and ring product
    def eval_q(self, a, slow=False):
        a = _u64(a); out = np.empty(self.n, np.uint64)
        self.L.orc_eval_q(self.h, _p(a), _p(out), int(slow)); return out

    def interp_q(self, ev, slow=False):
        ev = _u64(ev); out = np.empty(self.n, np.uint64)
        self.L.orc_interp_q(self.h, _p(ev), _p(out), int(slow)); return out

    def polymul(self, a, b, schoolbook=False):
        a, b = _u64(a), _u64(b); out = np.empty(self.n, np.uint64)
        f = self.L.orc_polymul_schoolbook if schoolbook else self.L.orc_polymul
        f(self.h, _p(a), _p(b), _p(out)); return out

    def polymul_special(self, a, b):
        a, b = _u64(a), _u64(b); out = np.empty(self.n, np.uint64)
        self.L.orc_polymul_special(self.h, _p(a), _p(b), _p(out)); return out

    # ---- slot encoding
    def encode(self, slots, slow=False):
        s = _u64(slots); out = np.empty(self.n, np.uint64)
        self.L.orc_encode(self.h, _p(s), _p(out), int(slow)); return out

    def decode(self, poly_p, slow=False):
        a = _u64(poly_p); out = np.empty(self.n, np.uint64)
        self.L.orc_decode(self.h, _p(a), _p(out), int(slow)); return out

    def encode_weight(self, slots):
        s = _u64(slots); out = np.empty(self.n, np.uint64)
        self.L.orc_encode_weight(self.h, _p(s), _p(out)); return out

    # ---- samplers
    def mix64(self, z):
        return int(self.L.orc_mix64(C.c_uint64(z)))

    def rand64(self, seed, stream, idx, attempt=0):
        return int(self.L.orc_rand64(C.c_uint64(seed), C.c_uint64(stream), C.c_uint64(idx), C.c_uint64(attempt)))

    def uniform(self, m, seed, stream, idx):
        return int(self.L.orc_uniform(C.c_uint64(m), C.c_uint64(seed), C.c_uint64(stream), C.c_uint64(idx)))

    def ternary(self, seed, stream, idx):
        return int(self.L.orc_ternary(C.c_uint64(seed), C.c_uint64(stream), C.c_uint64(idx)))

    def gauss(self, seed, stream, idx):
        return int(self.L.orc_gauss(C.c_uint64(seed), C.c_uint64(stream), C.c_uint64(idx)))

    def gauss_cdf(self):
        ptr = self.L.orc_gauss_cdf()
        return [int(ptr[i]) for i in range(38)]

    # ---- scheme
    def keygen(self, seed):
        s = np.empty(self.n, np.uint64); self.L.orc_keygen(self.h, C.c_uint64(seed), _p(s)); return s

    def encrypt(self, sk, slots, seed):
        slots = _u64(slots); ct = np.empty(2 * self.n, np.uint64)
        self.L.orc_encrypt(self.h, _p(sk), _p(slots), C.c_uint64(seed), _p(ct)); return ct

    def decrypt(self, sk, ct):
        ct = _u64(ct); out = np.empty(self.n, np.uint64)
        self.L.orc_decrypt(self.h, _p(sk), _p(ct), _p(out)); return out

    def noise(self, sk, ct, expected_slots):
        ct, e = _u64(ct), _u64(expected_slots)
        return int(self.L.orc_noise(self.h, _p(sk), _p(ct), _p(e)))

    def galois_elt(self, swap, step):
        return int(self.L.orc_galois_elt(self.h, int(swap), int(step)))

    def apply_galois(self, a, g):
        a = _u64(a); out = np.empty(self.n, np.uint64)
        self.L.orc_apply_galois(self.h, _p(a), int(g), _p(out)); return out

    def galois_key(self, sk, g, seed):
        k = np.empty(self.ksk_words, np.uint64)
        self.L.orc_galois_key(self.h, _p(sk), int(g), C.c_uint64(seed), _p(k)); return k

    def decperm(self, c1):
        c1 = _u64(c1); d = np.empty(self.ndigits * self.n, np.uint64)
        self.L.orc_decperm(self.h, _p(c1), _p(d)); return d

    def hstperm(self, c0, digits, g, ksk):
        c0, digits, ksk = _u64(c0), _u64(digits), _u64(ksk); out = np.empty(2 * self.n, np.uint64)
        self.L.orc_hstperm(self.h, _p(c0), _p(digits), int(g), _p(ksk), _p(out)); return out

    def perm(self, ct, g, ksk):
        ct, ksk = _u64(ct), _u64(ksk); out = np.empty(2 * self.n, np.uint64)
        self.L.orc_perm(self.h, _p(ct), int(g), _p(ksk), _p(out)); return out

    def add(self, x, y):
        x, y = _u64(x), _u64(y); out = np.empty(2 * self.n, np.uint64)
        self.L.orc_add(self.h, _p(x), _p(y), _p(out)); return out

    def scmult(self, ct, w_poly_q):
        ct, w = _u64(ct), _u64(w_poly_q); out = np.empty(2 * self.n, np.uint64)
        self.L.orc_scmult(self.h, _p(ct), _p(w), _p(out)); return out

    def sub_plain(self, ct, mask_slots):
        ct, m = _u64(ct), _u64(mask_slots); out = np.empty(2 * self.n, np.uint64)
        self.L.orc_sub_plain(self.h, _p(ct), _p(m), _p(out)); return out

    # ---- FC (row-encoding-share-RaS)
    def fc_G(self, n_o, n_i):
        return int(self.L.orc_fc_G(self.h, n_o, n_i))

    def fc_pack_input(self, n_o, n_i, x):
        x = _u64(x); out = np.empty(self.n, np.uint64)
        self.L.orc_fc_pack_input(self.h, n_o, n_i, _p(x), _p(out)); return out

    def fc_weight_slots(self, W, g):
        W = _u64(W); n_o, n_i = W.shape; out = np.empty(self.n, np.uint64)
        self.L.orc_fc_weight_slots(self.h, _p(W), n_o, n_i, int(g), _p(out)); return out

    def fc_encode_rowwise(self, W):
        W = _u64(W); n_o, n_i = W.shape
        out = np.empty((self.fc_G(n_o, n_i), self.n), np.uint64)
        self.L.orc_fc_encode_rowwise(self.h, _p(W), n_o, n_i, _p(out)); return out

    def fc_unpack_share(self, n_o, n_i, slots):
        s = _u64(slots); out = np.empty(n_o, np.uint64)
        self.L.orc_fc_unpack_share(self.h, n_o, n_i, _p(s), _p(out)); return out

    def fc_mask_slots(self, n_o, n_i, r, seed, b):
        r = _u64(r); out = np.empty(self.n, np.uint64)
        self.L.orc_fc_mask_slots(self.h, n_o, n_i, _p(r), C.c_uint64(seed), int(b), _p(out)); return out

    def fc_keys(self, sk, n_o, n_i, seed):
        """Galois keys of rotations g = 1..G-1 (left by g, both rows), concatenated."""
        G = self.fc_G(n_o, n_i)
        if G <= 1:
            return np.zeros(0, np.uint64)
        return np.concatenate([self.galois_key(sk, self.galois_elt(0, g), seed) for g in range(1, G)])

    def he_fc(self, wpoly, ct, ksk, mask_slots):
        wpoly, ct, ksk, m = _u64(wpoly), _u64(ct), _u64(ksk), _u64(mask_slots)
        out = np.empty(2 * self.n, np.uint64); cnt = Counts()
        self.L.orc_he_fc(self.h, _p(wpoly), wpoly.shape[0], _p(ct), _p(ksk), _p(m), _p(out), C.byref(cnt))
        return out, cnt.as_dict()

    def he_fc_batch(self, wpoly, n_o, n_i, cts, ksk, r, mask_seed, b0=0):
        wpoly, cts, ksk, r = _u64(wpoly), _u64(cts), _u64(ksk), _u64(r)
        batch = cts.shape[0]; out = np.empty((batch, 2 * self.n), np.uint64); cnt = Counts()
        self.L.orc_he_fc_batch(self.h, _p(wpoly), n_o, n_i, _p(cts), batch, int(b0), _p(ksk), _p(r),
                               C.c_uint64(mask_seed), _p(out), C.byref(cnt))
        return out, cnt.as_dict()

    # ---- comparison schedules (Sec. III-A(2) hybrid FC, Sec. III-B(2) output-rotation convolution)
    def fc_hybrid_G(self, n_o, n_i):
        return int(self.L.orc_fc_hybrid_G(self.h, n_o, n_i))

    def fc_hybrid_ras(self, n_o, n_i):
        """The rotate-and-sum rotations (swap, step) in order."""
        sw, st = (C.c_int * 32)(), (C.c_int * 32)()
        k = self.L.orc_fc_hybrid_ras(self.h, n_o, n_i, sw, st)
        if k < 0:
            raise ValueError("oracle: FC shape not supported")
        return [(sw[i], st[i]) for i in range(k)]

    def fc_hybrid_weight_slots(self, W, g):
        W = _u64(W); out = np.empty(self.n, np.uint64)
        self.L.orc_fc_hybrid_weight_slots(self.h, _p(W), W.shape[0], W.shape[1], g, _p(out)); return out

    def fc_hybrid_encode(self, W):
        W = _u64(W); G = self.fc_hybrid_G(*W.shape); out = np.empty((G, self.n), np.uint64)
        self.L.orc_fc_hybrid_encode(self.h, _p(W), W.shape[0], W.shape[1], _p(out)); return out

    def fc_hybrid_unpack(self, n_o, n_i, slots):
        s = _u64(slots); out = np.empty(n_o, np.uint64)
        self.L.orc_fc_hybrid_unpack(self.h, n_o, n_i, _p(s), _p(out)); return out

    def fc_hybrid_mask_slots(self, n_o, n_i, r, seed, b):
        r = _u64(r); out = np.empty(self.n, np.uint64)
        self.L.orc_fc_hybrid_mask_slots(self.h, n_o, n_i, _p(r), C.c_uint64(seed), int(b), _p(out)); return out

    def fc_hybrid_keys(self, sk, n_o, n_i, seed):
        """(keys of the input rotations g = 1..G-1, keys of the rotate-and-sum rotations), each concatenated."""
        G = self.fc_hybrid_G(n_o, n_i)
        cat = lambda l: np.concatenate(l) if l else np.zeros(0, np.uint64)
        return (cat([self.galois_key(sk, self.galois_elt(0, g), seed) for g in range(1, G)]),
                cat([self.galois_key(sk, self.galois_elt(s, t), seed) for s, t in self.fc_hybrid_ras(n_o, n_i)]))

    def he_fc_hybrid(self, wpoly, n_o, n_i, ct, ksk_in, ksk_ras, mask_slots):
        wpoly, ct, ki, kr, m = _u64(wpoly), _u64(ct), _u64(ksk_in), _u64(ksk_ras), _u64(mask_slots)
        out = np.empty(2 * self.n, np.uint64); cnt = Counts()
        self.L.orc_he_fc_hybrid(self.h, _p(wpoly), n_o, n_i, _p(ct), _p(ki), _p(kr), _p(m), _p(out), C.byref(cnt))
        return out, cnt.as_dict()

    def he_conv_outrot_block(self, shape, K, O, cts, tap_ksk, grp_ksk, mask_slots, xrot=None, ready=None):
        """One output ciphertext O by the output-rotation schedule; arguments as he_conv_block."""
        co, ci, kh, kw, uh, uw = shape
        K, cts, tk, gk, m = _u64(K), _u64(cts), _u64(tap_ksk), _u64(grp_ksk), _u64(mask_slots)
        out = np.empty(2 * self.n, np.uint64); cnt = Counts()
        self.L.orc_he_conv_outrot_block(self.h, _p(K), co, ci, kh, kw, uh, uw, int(O), _p(cts), _p(tk), _p(gk), _p(m),
                                        _p(xrot) if xrot is not None else None,
                                        C.byref(ready) if ready is not None else None, _p(out), C.byref(cnt))
        return out, cnt.as_dict()

    def max_threads(self):
        return int(self.L.orc_max_threads())

    # ---- Conv (kernel grouping)
    def conv_geometry(self, co, ci, kh, kw, uh, uw):
        out = (C.c_int * 5)()
        if self.L.orc_conv_geometry(self.h, co, ci, kh, kw, uh, uw, out):
            raise ValueError("oracle: conv shape not supported")
        return dict(T=out[0], cn=out[1], nin=out[2], nout=out[3], ntap=out[4])

    def conv_pack_input(self, shape, x):
        co, ci, kh, kw, uh, uw = shape
        x = _u64(x); g = self.conv_geometry(*shape); out = np.empty((g["nin"], self.n), np.uint64)
        self.L.orc_conv_pack_input(self.h, co, ci, kh, kw, uh, uw, _p(x), _p(out)); return out

    def conv_weight_slots(self, shape, K, O, gam, I, tap):
        co, ci, kh, kw, uh, uw = shape
        K = _u64(K); out = np.empty(self.n, np.uint64)
        self.L.orc_conv_weight_slots(self.h, _p(K), co, ci, kh, kw, uh, uw, O, gam, I, tap, _p(out)); return out

    def conv_group_galois(self, shape, gam):
        return int(self.L.orc_conv_group_galois(self.h, *shape, int(gam)))

    def conv_tap_galois(self, shape, tap):
        return int(self.L.orc_conv_tap_galois(self.h, *shape, int(tap)))

    def conv_keys(self, sk, shape, seed):
        """(tap keys in tap order without the centre, group keys gam = 1..cn-1)."""
        co, ci, kh, kw, uh, uw = shape
        g = self.conv_geometry(*shape)
        centre = (kh // 2) * kw + kw // 2
        taps = [self.galois_key(sk, self.conv_tap_galois(shape, t), seed) for t in range(g["ntap"]) if t != centre]
        grps = [self.galois_key(sk, self.conv_group_galois(shape, gam), seed) for gam in range(1, g["cn"])]
        cat = lambda l: np.concatenate(l) if l else np.zeros(0, np.uint64)
        return cat(taps), cat(grps)

    def conv_mask_slots(self, shape, r, seed, b, O):
        co, ci, kh, kw, uh, uw = shape
        r = _u64(r); out = np.empty(self.n, np.uint64)
        self.L.orc_conv_mask_slots(self.h, co, ci, kh, kw, uh, uw, _p(r), C.c_uint64(seed), int(b), int(O), _p(out))
        return out

    def conv_unpack_share(self, shape, O, slots, out):
        co, ci, kh, kw, uh, uw = shape
        s = _u64(slots)
        self.L.orc_conv_unpack_share(self.h, co, ci, kh, kw, uh, uw, int(O), _p(s), _p(out))

    def he_conv_block(self, shape, K, O, cts, tap_ksk, grp_ksk, mask_slots, xrot=None, ready=None):
        """One output ciphertext O.  ``xrot``/``ready`` (a uint64 array of nin*ntap cts and a
        ctypes c_int) let several blocks of the same input share the input rotations."""
        co, ci, kh, kw, uh, uw = shape
        K, cts, tk, gk, m = _u64(K), _u64(cts), _u64(tap_ksk), _u64(grp_ksk), _u64(mask_slots)
        out = np.empty(2 * self.n, np.uint64); cnt = Counts()
        self.L.orc_he_conv_block(self.h, _p(K), co, ci, kh, kw, uh, uw, int(O), _p(cts), _p(tk), _p(gk), _p(m),
                                 _p(xrot) if xrot is not None else None,
                                 C.byref(ready) if ready is not None else None, _p(out), C.byref(cnt))
        return out, cnt.as_dict()


# ---------------------------------------------------------------------------
# Stride.  The paper's convolution (Sec. III-B) is stride 1; a strided layer is defined here by the usual
# "same"-padded sum and reduced to the stride-1 form by splitting the image into its phases.
# ---------------------------------------------------------------------------
def strided_conv_plain(K, x, p, stride):
    """out[o][Y][X] = sum_{c,dy,dx} K[o][c][dy+kh//2][dx+kw//2] * x[c][stride*Y+dy][stride*X+dx] mod p, x zero
    outside the image; the definition written out with Python integers (small cases only)."""
    co, ci, kh, kw = K.shape
    _, H, W = x.shape
    oh, ow = -(-H // stride), -(-W // stride)
    out = np.zeros((co, oh, ow), np.uint64)
    for o in range(co):
        for Y in range(oh):
            for X in range(ow):
                acc = 0
                for c in range(ci):
                    for dy in range(-(kh // 2), kh // 2 + 1):
                        for dx in range(-(kw // 2), kw // 2 + 1):
                            y, xx = stride * Y + dy, stride * X + dx
                            if 0 <= y < H and 0 <= xx < W:
                                acc += int(K[o, c, dy + kh // 2, dx + kw // 2]) * int(x[c, y, xx])
                out[o, Y, X] = acc % p
    return out


def polyphase_split(K, x, stride):
    """(K_poly, x_poly): the stride-1 convolution of x_poly with K_poly equals the stride-`stride` convolution of
    x with K.  Phase (a, b) of the image, x[:, a::s, b::s], becomes a block of c_i input channels (phase-major,
    only phases that a tap reads); tap (dy, dx) = (s*m + a, s*l + b) of K becomes tap (m, l) of that block."""
    K, x = np.asarray(K, np.uint64), np.asarray(x, np.uint64)
    co, ci, kh, kw = K.shape
    _, H, W = x.shape
    s = stride

    def axis(k):
        taps = range(-(k // 2), k // 2 + 1)
        return sorted({d % s for d in taps}), 2 * max(abs(d // s) for d in taps) + 1     # // floors

    ry, khp = axis(kh)
    rx, kwp = axis(kw)
    oh, ow = -(-H // s), -(-W // s)
    Kp = np.zeros((co, len(ry) * len(rx) * ci, khp, kwp), np.uint64)
    xp = np.zeros((len(ry) * len(rx) * ci, oh, ow), np.uint64)
    for ia, a in enumerate(ry):
        for ib, b in enumerate(rx):
            base = (ia * len(rx) + ib) * ci
            sub = x[:, a::s, b::s]
            xp[base:base + ci, :sub.shape[1], :sub.shape[2]] = sub
            for dy in range(-(kh // 2), kh // 2 + 1):
                for dx in range(-(kw // 2), kw // 2 + 1):
                    if dy % s == a and dx % s == b:
                        Kp[:, base:base + ci, dy // s + khp // 2, dx // s + kwp // 2] = K[:, :, dy + kh // 2, dx + kw // 2]
    return Kp, xp
