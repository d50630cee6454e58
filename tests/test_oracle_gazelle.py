"""Pins for the oracle's comparison schedules: the hybrid matrix-vector product (Sec. III-A(2)) and the
output-rotation MIMO convolution (Sec. III-B(2)), i.e. the GAZELLE columns of the paper's tables."""
import os

import numpy as np
import pytest

from oracle.oracle import Oracle
from paper_2105_01827_amd import workloads as wl
from tests.helpers import rotate_slots, small_params
from tests.test_oracle_conv import plain_conv
from tests.test_oracle_fc import plain_matvec

GOLD = os.path.join(os.path.dirname(__file__), "golden", "gazelle_counts.txt")


def gold_lines(prefix):
    return [l.split() for l in open(GOLD) if l.startswith(prefix + " ") or l.startswith(prefix + ":")]


def ilog2(v):
    return v.bit_length() - 1


def test_hybrid_toy_example_of_the_paper():
    """Rows A, B of a 4x4 matrix on n = 8 slots: the first copy of x owns rows A and B and its four slots carry
    exactly the two diagonal vectors the paper prints for its 2x4 example; the second copy repeats the pattern with
    rows C and D."""
    par = small_params(8, p_limit=1 << 12)
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    ident = {f"{r}{c + 1}": 10 * (ri + 1) + c + 1 for ri, r in enumerate("ABCD") for c in range(4)}
    W = np.array([[ident[f"{r}{c + 1}"] for c in range(4)] for r in "ABCD"], dtype=np.uint64)
    assert o.fc_hybrid_G(4, 4) == 2
    for g, key in ((0, "hybrid_w0:"), (1, "hybrid_w1:")):
        names = [l for l in open(GOLD) if l.startswith(key)][0].split()[1:]
        slots = [int(v) for v in o.fc_hybrid_weight_slots(W, g)]
        assert slots[:4] == [ident[t] for t in names]
        assert slots[4:] == [ident[t.replace("A", "C").replace("B", "D")] for t in names]
    # the input is rotated by g before the product, and one rotate-and-sum step by 2 finishes the rows
    assert o.fc_hybrid_ras(4, 4) == [(0, 2)]
    x = np.array([3, 5, 7, 9], dtype=np.uint64)
    xs = o.fc_pack_input(4, 4, x)
    s = sum(o.fc_hybrid_weight_slots(W, g) * rotate_slots(xs, g) for g in range(2))
    s = s + rotate_slots(s, 2)
    assert np.array_equal(o.fc_hybrid_unpack(4, 4, s % np.uint64(par.p)), plain_matvec(W, x, par.p))


SHAPES = [(16, 128), (128, 1024), (1000, 2048), (2, 2048), (1, 2048), (2, 1024), (16, 512), (16, 64), (10, 100),
          (512, 1000), (256, 4), (1024, 8)]


@pytest.mark.parametrize("n_o,n_i", SHAPES)
def test_hybrid_layout_computes_the_product_on_plain_slot_vectors(n_o, n_i):
    """The layout alone, no encryption: products of the diagonal vectors with the rotated packed input, summed,
    then the rotate-and-sum steps as slot rotations, give W x at the result slots (n = 2048, exact integers)."""
    n = 2048
    par = wl.DEFAULT
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    rng = np.random.default_rng(n_o * 4099 + n_i)
    W = rng.integers(0, par.p, size=(n_o, n_i), dtype=np.uint64)
    x = rng.integers(0, par.p, size=n_i, dtype=np.uint64)
    xs = o.fc_pack_input(n_o, n_i, x).astype(object)
    G = o.fc_hybrid_G(n_o, n_i)
    s = np.zeros(n, dtype=object)
    for g in range(G):
        s = s + o.fc_hybrid_weight_slots(W, g).astype(object) * rotate_slots(xs, g)
    ras = o.fc_hybrid_ras(n_o, n_i)
    for swap, step in ras:
        s = s + rotate_slots(s, step, bool(swap))
    got = o.fc_hybrid_unpack(n_o, n_i, np.array([int(v) % par.p for v in s], dtype=np.uint64))
    assert np.array_equal(got, plain_matvec(W, x, par.p))
    nop, nip = 1 << (n_o - 1).bit_length(), 1 << (n_i - 1).bit_length()
    if nop * nip >= n:      # Table "Complexity comparison of three methods", GAZELLE row
        assert G == nop * nip // n and len(ras) == ilog2(n // nop)


def run_hybrid(o, par, W, x, r, sk, b=0, seed=5):
    n_o, n_i = W.shape
    ct = o.encrypt(sk, o.fc_pack_input(n_o, n_i, x), seed=77)
    k_in, k_ras = o.fc_hybrid_keys(sk, n_o, n_i, seed=1)
    mask = o.fc_hybrid_mask_slots(n_o, n_i, r, seed, b)
    out, cnt = o.he_fc_hybrid(o.fc_hybrid_encode(W), n_o, n_i, ct, k_in, k_ras, mask)
    dec = o.decrypt(sk, out)
    return o.fc_hybrid_unpack(n_o, n_i, dec), cnt, o.noise(sk, out, dec), mask, dec


@pytest.mark.parametrize("n,n_o,n_i", [(64, 4, 16), (64, 8, 32), (64, 16, 64), (64, 3, 20), (64, 1, 64), (64, 32, 2),
                                       (256, 2, 256), (256, 64, 128), (1024, 8, 512)])
def test_he_fc_hybrid_identity_and_counts_small_rings(n, n_o, n_i):
    # The input is rotated BEFORE ScMult here, so the rotation noise is multiplied by the weights (Sec. III-C):
    # with one-prime keys this only decrypts for a small plaintext modulus and narrow digits, as for convolutions.
    par = small_params(n, p_limit=1 << 14, gadget_bits=4)
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    W, x, r = wl.fc_inputs(wl.FcShape("t", n_o, n_i, 1), p=par.p, seed=n_o + n_i)
    sk = o.keygen(3)
    share, cnt, worst, mask, dec = run_hybrid(o, par, W, x[0], r[0], sk)
    assert np.array_equal((share + r[0]) % np.uint64(par.p), plain_matvec(W, x[0], par.p))
    assert worst < o.delta // 4
    G, steps = o.fc_hybrid_G(n_o, n_i), len(o.fc_hybrid_ras(n_o, n_i))
    assert cnt == dict(perm=steps, decperm_in=1 if G > 1 else 0, hstperm_in=G - 1, scmult=G, add=G - 1 + steps)
    # every slot that is not a result is hidden by a draw of the mask stream: the decrypted vector minus the mask
    # differs from it only through the layer's partial sums, and the mask itself carries r at the result slots
    assert np.array_equal(o.fc_hybrid_unpack(n_o, n_i, mask), r[0] % np.uint64(par.p))


def test_he_fc_hybrid_counts_of_the_papers_table():
    """Table "Computation complexity of matrix-vector multiplication", GAZELLE column, executed at n = 2048."""
    par = wl.DEFAULT
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    sk = o.keygen(3)
    for _, dims, perm, hst, scm, add in gold_lines("fc"):
        n_o, n_i = (int(v) for v in dims.split("x"))
        W, x, r = wl.fc_inputs(wl.FcShape("t", n_o, n_i, 1), seed=n_o)
        share, cnt, worst, _, _ = run_hybrid(o, par, W, x[0], r[0], sk)
        assert (cnt["perm"], cnt["hstperm_in"], cnt["scmult"], cnt["add"]) == (int(perm), int(hst), int(scm), int(add))
        assert np.array_equal((share + r[0]) % np.uint64(par.p), (W @ x[0]) % np.uint64(par.p))
        assert worst < o.delta // 4


def outrot_closed_form(co, ci, kh, kw, cn):
    """Table "Complexity comparison of convolution", GAZELLE row (plus the common DecPerms of the inputs)."""
    k2 = kh * kw
    return dict(perm=ci * co * (cn - 1) // (cn * cn), decperm_in=(ci // cn if k2 > 1 else 0),
                hstperm_in=ci * (k2 - 1) // cn, scmult=ci * co * k2 // cn, add=co * (ci * k2 - 1) // cn)


def run_outrot(o, par, shape, K, x, r, sk, mask_seed=3, b=0):
    import ctypes
    geo = o.conv_geometry(*shape)
    slots = o.conv_pack_input(shape, x)
    cts = np.stack([o.encrypt(sk, slots[i], seed=100 + i) for i in range(geo["nin"])])
    tk, gk = o.conv_keys(sk, shape, seed=8)
    xrot, ready = np.empty(geo["nin"] * geo["ntap"] * 2 * par.n, np.uint64), ctypes.c_int(0)
    share = np.zeros(r.shape, np.uint64)
    total = dict(perm=0, decperm_in=0, hstperm_in=0, scmult=0, add=0)
    worst = 0
    for O in range(geo["nout"]):
        out, cnt = o.he_conv_outrot_block(shape, K, O, cts, tk, gk, o.conv_mask_slots(shape, r, mask_seed, b, O), xrot, ready)
        dec = o.decrypt(sk, out)
        worst = max(worst, o.noise(sk, out, dec))
        o.conv_unpack_share(shape, O, dec, share)
        for k in total:
            total[k] += cnt[k]
    return share, total, worst, geo


@pytest.mark.parametrize("n,p_limit,gb,shape", [
    (16, 1 << 7, 4, (4, 4, 3, 3, 2, 2)),
    (64, 1 << 9, 4, (8, 16, 3, 3, 2, 4)),
    (64, 1 << 9, 4, (5, 3, 3, 1, 3, 2)),
    (64, 1 << 9, 4, (4, 12, 1, 1, 4, 4)),
    (128, 1 << 9, 4, (6, 6, 5, 5, 4, 4)),
])
def test_he_conv_outrot_identity_and_counts_small_rings(n, p_limit, gb, shape):
    par = small_params(n, p_limit=p_limit, gadget_bits=gb)
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    co, ci, kh, kw, uh, uw = shape
    K, x, r = wl.conv_inputs(wl.ConvShape("t", co, ci, kh, kw, uh, uw, 1), p=par.p, seed=n + co)
    sk = o.keygen(4)
    share, cnt, worst, geo = run_outrot(o, par, shape, K, x[0], r[0], sk)
    assert np.array_equal((share + r[0]) % np.uint64(par.p), plain_conv(K, x[0], par.p))
    assert worst < o.delta // 4
    cn = geo["cn"]
    assert cnt == outrot_closed_form(geo["nout"] * cn, geo["nin"] * cn, kh, kw, cn)


def test_outrot_counts_of_the_papers_table():
    """Table "Computation complexity of convolution", GAZELLE column: the closed form on every printed row, and the
    3x3@128 row executed on a small ring with the same channel structure (c_n = 8)."""
    for _, inp, ker, dec, hst, scm, add in gold_lines("conv"):
        ci, co, k = int(inp.split("@")[1]), int(ker.split("@")[1]), int(ker[0])
        want = outrot_closed_form(co, ci, k, k, 8)
        assert (want["decperm_in"] + want["perm"], want["hstperm_in"] + want["perm"], want["scmult"], want["add"]) == \
               (int(dec), int(hst), int(scm), int(add))
    _, inp, ker, hst, scm = gold_lines("conv_hstperm_scmult")[0]
    want = outrot_closed_form(int(ker.split("@")[1]), int(inp.split("@")[1]), 1, 1, 8)
    assert (want["hstperm_in"] + want["perm"], want["scmult"]) == (int(hst), int(scm))
    par = small_params(64, p_limit=1 << 9, gadget_bits=6)
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    shape = (128, 128, 3, 3, 2, 4)
    K, x, r = wl.conv_inputs(wl.ConvShape("t", *shape, 1), p=par.p, seed=1)
    sk = o.keygen(1)
    share, cnt, worst, geo = run_outrot(o, par, shape, K, x[0], r[0], sk)
    assert geo["cn"] == 8
    assert (cnt["decperm_in"] + cnt["perm"], cnt["hstperm_in"] + cnt["perm"], cnt["scmult"], cnt["add"]) == (1808, 1920, 18432, 18416)
    assert np.array_equal((share + r[0]) % np.uint64(par.p), plain_conv(K, x[0], par.p))
