"""GPU parity with special-prime key switching (keys modulo q*P, exact division by P): the HIP library against
the CPU oracle, bit for bit, through the C ABI, and the functional identity of a 3x3 convolution at the
parameters of Sec. IV, which only decrypts in this mode."""
import dataclasses

import numpy as np
import pytest

from paper_2105_01827_amd import binding, workloads as wl
from tests.helpers import rotate_slots, small_params
from tests.test_gpu_parity import _punch_holes, both, conv_case, fc_case, harness, plain_conv, plain_matvec

pytestmark = pytest.mark.gpu


def with_special(par):
    P = wl.find_prime_below(1 << 60, 2 * par.n)
    if P == par.q:
        P = wl.find_prime_below(P, 2 * par.n)
    return dataclasses.replace(par, special=P)


def params(n, **kw):
    return with_special(small_params(n, **kw)) if n != 2048 or kw else wl.DEFAULT_SPECIAL


@pytest.mark.parametrize("n,gb", [(64, 20), (64, 7), (2048, 20)])
def test_galois_keys_match_the_oracle(n, gb):
    par = params(n, gadget_bits=gb) if n != 2048 else params(n)
    ctx, o = both(par)
    sk, osk = ctx.keygen(3), o.keygen(3)
    rots = [(0, 1), (1, 0), (1, n // 2 - 1)]
    gk = ctx.galois_keygen(sk, rots, seed=42)
    for swap, step in rots:
        want = o.galois_key(osk, o.galois_elt(swap, step), 42)
        assert want.size == o.ndigits * 4 * n
        assert np.array_equal(gk.export((swap, step)), want), (swap, step)


@pytest.mark.parametrize("n,gb,rots", [
    (8, 20, [(0, 1), (0, 3), (1, 0), (1, 2)]),
    (64, 20, [(0, 1), (0, 31), (1, 17)]),
    (64, 7, [(0, 3), (1, 5)]),                          # 9 digits
    (64, 60, [(0, 9)]),                                 # a single digit
    (1024, 30, [(0, 511), (1, 1)]),
    (2048, 20, [(0, 1), (0, 1023), (1, 512)]),
])
def test_rotate_matches_oracle_perm(n, gb, rots):
    H = harness()
    par = params(n, gadget_bits=gb) if (n, gb) != (2048, 20) else params(n)
    ctx, o = both(par)
    sk, osk = ctx.keygen(3), o.keygen(3)
    rng = np.random.default_rng(5)
    count = 3
    slots = rng.integers(0, par.p, size=(count, n), dtype=np.uint64)
    cts = np.stack([ctx.encrypt(sk, slots[i], seed=10 + i) for i in range(count)])
    gk = ctx.galois_keygen(sk, rots, seed=42)
    d_in = H.import_cts(ctx, cts)
    for swap, step in rots:
        d_out = H.dev_empty(count * 2 * n)
        ctx.rotate(gk, d_in, count, (swap, step), d_out)
        got = H.export_cts(ctx, d_out, count)
        g = o.galois_elt(swap, step)
        ksk = o.galois_key(osk, g, 42)
        for i in range(count):
            assert np.array_equal(got[i], o.perm(cts[i], g, ksk)), (swap, step, i)
            assert np.array_equal(ctx.decrypt(sk, got[i]), rotate_slots(slots[i], step, bool(swap)))
            assert o.noise(osk, got[i], rotate_slots(slots[i], step, bool(swap))) <= 20 + n
    d_out = H.dev_empty(count * 2 * n)
    ctx.rotate(gk, d_in, count, (0, 0), d_out)
    assert np.array_equal(H.export_cts(ctx, d_out, count), cts)


@pytest.mark.parametrize("n,n_o,n_i,batch", [(64, 4, 16, 3), (64, 16, 64, 2), (64, 3, 20, 1), (256, 64, 128, 5)])
def test_he_fc_small_rings(n, n_o, n_i, batch):
    par = params(n, gadget_bits=20)
    ctx, o, plan, sk, W, x, r, got = fc_case(par, n_o, n_i, batch, list(range(batch)), seed=n_o + n_i)
    for b in range(batch):
        share = plan.unpack_share(ctx.decrypt(sk, got[b]))
        assert np.array_equal((share + r[b]) % np.uint64(par.p), plain_matvec(W, x[b], par.p))


def test_he_fc_128x1024_full_parameters():
    par = params(2048)
    ctx, o, plan, sk, W, x, r, got = fc_case(par, 128, 1024, 4, [0, 3], seed=2)
    for b in range(4):
        share = plan.unpack_share(ctx.decrypt(sk, got[b]))
        assert np.array_equal((share + r[b]) % np.uint64(par.p), plain_matvec(W, x[b], par.p))


@pytest.mark.parametrize("n,p_limit,gb,shape,batch,mc", [
    (16, 1 << 7, 4, (4, 4, 3, 3, 2, 2), 2, False),
    (64, 1 << 9, 20, (8, 8, 3, 3, 2, 4), 3, False),
    (64, 1 << 9, 30, (4, 12, 1, 1, 4, 4), 2, False),
    (128, 1 << 9, 20, (6, 6, 5, 5, 4, 4), 9, True),
])
def test_he_conv_small_rings(n, p_limit, gb, shape, batch, mc):
    par = params(n, p_limit=p_limit, gadget_bits=gb)
    ctx0, o0 = both(par)
    nout = o0.conv_geometry(*shape)["nout"]
    outs = [(b, O) for b in range(min(batch, 3)) for O in range(nout)]
    ctx, o, plan, sk, K, x, r, got, cnt = conv_case(par, shape, batch, outs, seed=n, matrix_cores=mc)
    for b in range(batch):     # with the special prime the identity holds even at large gadget bases
        share = np.zeros(r[b].shape, np.uint64)
        for O in range(plan.nout):
            plan.unpack_share(O, ctx.decrypt(sk, got[b, O]), share)
        assert np.array_equal((share + r[b]) % np.uint64(par.p), plain_conv(K, x[b], par.p))


@pytest.mark.parametrize("n,p_limit,gb,shape,batch", [
    (64, 1 << 9, 20, (8, 16, 3, 3, 2, 4), 3),            # any-n kernels: every term a Perm of its own
    (2048, None, 20, (8, 32, 3, 3, 16, 16), 2),          # n = 2048 kernels
])
def test_he_conv_skips_zero_terms(n, p_limit, gb, shape, batch):
    par = params(n, p_limit=p_limit, gadget_bits=gb) if p_limit else params(2048)
    ctx, o, plan, sk, K, x, r, got, cnt = conv_case(par, shape, batch, [(0, 0), (batch - 1, 0)], seed=5,
                                                    edit_kernel=_punch_holes)
    assert plan.nterm == 6 * (plan.nin // 2) + plan.nin // 2
    for b in range(batch):
        share = np.zeros(r[b].shape, np.uint64)
        for O in range(plan.nout):
            plan.unpack_share(O, ctx.decrypt(sk, got[b, O]), share)
        assert np.array_equal((share + r[b]) % np.uint64(par.p), plain_conv(K, x[b], par.p))


def test_he_conv_3x3_decrypts_at_the_papers_parameters():
    """n = 2048, p ~ 2^20, 60-bit q, 20-bit digits: 16x16x32 input, 32 kernels of 3x3, batch 8 on the matrix cores.
    Bit-exact against the oracle on sampled outputs and the plain convolution is recovered for every input."""
    par = params(2048)
    shape = (32, 32, 3, 3, 16, 16)
    ctx, o, plan, sk, K, x, r, got, cnt = conv_case(par, shape, 8, [(0, 0), (5, 3)], seed=11, matrix_cores=True)
    assert plan.cn == 8 and plan.nout == 4
    assert cnt["hstperm_in"] == 8 * 4 * 8 and cnt["perm"] == 8 * 4 * 7
    for b in range(8):
        share = np.zeros(r[b].shape, np.uint64)
        for O in range(plan.nout):
            plan.unpack_share(O, ctx.decrypt(sk, got[b, O]), share)
        assert np.array_equal((share + r[b]) % np.uint64(par.p), plain_conv(K, x[b], par.p))


def test_he_conv_config4_decrypts_at_full_size():
    """16x16x128 input, 128 kernels of 3x3, batch 16, n = 2048, p ~ 2^20: the convolution of the fourth benchmark
    configuration.  One output ciphertext is recomputed by the oracle; the plain convolution is recovered for two
    of the inputs from all their output ciphertexts."""
    par = params(2048)
    s = wl.CONV_16x16_128_3x3
    ctx, o, plan, sk, K, x, r, got, cnt = conv_case(par, s.tuple, s.batch, [(3, 7)], seed=0, matrix_cores=True)
    assert cnt == dict(perm=1792, decperm_in=256, hstperm_in=2048, scmult=294912, add=294656)
    for b in (0, 15):
        share = np.zeros(r[b].shape, np.uint64)
        for O in range(plan.nout):
            plan.unpack_share(O, ctx.decrypt(sk, got[b, O]), share)
        assert np.array_equal((share + r[b]) % np.uint64(par.p), plain_conv(K, x[b], par.p))


def fast_plain_conv(K, x, p):
    """The same "same"-padded convolution as plain_conv in uint64 (products below 2^40, at most 2^11 of them)."""
    co, ci, kh, kw = K.shape
    _, uh, uw = x.shape
    out = np.zeros((co, uh, uw), np.uint64)
    for dy in range(kh):
        for dx in range(kw):
            oy, ox = dy - kh // 2, dx - kw // 2
            ys = slice(max(0, -oy), min(uh, uh - oy)); xs = slice(max(0, -ox), min(uw, uw - ox))
            src = x[:, ys.start + oy:ys.stop + oy, xs.start + ox:xs.stop + ox]
            out[:, ys, xs] += np.einsum("oc,cyx->oyx", K[:, :, dy, dx], src)
    return out % np.uint64(p)


@pytest.mark.parametrize("c,hw", [(128, 28), (512, 7)])
def test_resnet_3x3_layers_decrypt_at_full_size(c, hw):
    """3x3 layers of the ResNet-18-shaped list on one input (c_n = 2 with 576 terms; c_n = 32 with 144 terms): the
    streaming multiply-accumulate and the special-prime rotations together; every output decrypts to the plain
    convolution and one ciphertext is recomputed by the oracle."""
    par = params(2048)
    shape = (c, c, 3, 3, hw, hw)
    ctx, o, plan, sk, K, x, r, got, cnt = conv_case(par, shape, 1, [(0, plan_o) for plan_o in (1,)], seed=c)
    small = np.random.default_rng(1).integers(0, 50, size=(4, 3, 3, 3), dtype=np.uint64)
    img = np.random.default_rng(2).integers(0, 50, size=(3, 5, 5), dtype=np.uint64)
    assert np.array_equal(fast_plain_conv(small, img, par.p), plain_conv(small, img, par.p))
    share = np.zeros(r[0].shape, np.uint64)
    for O in range(plan.nout):
        plan.unpack_share(O, ctx.decrypt(sk, got[0, O]), share)
    assert np.array_equal((share + r[0]) % np.uint64(par.p), fast_plain_conv(K, x[0], par.p))


@pytest.mark.parametrize("gb", [60, 20, 15, 9])
def test_n2048_special_prime_kernels_with_other_digit_counts(gb):
    """Every other full-size special-prime test uses two digits of 30 bits: one, three, four and seven digits here,
    through Perm, hoisted rotations, he_fc and he_conv on both multiply-accumulate paths, against the oracle."""
    H = harness()
    par = dataclasses.replace(wl.DEFAULT_SPECIAL, gadget_bits=gb)
    ctx, o = both(par)
    n = par.n
    sk, osk = ctx.keygen(3), o.keygen(3)
    rng = np.random.default_rng(gb)
    slots = rng.integers(0, par.p, size=(2, n), dtype=np.uint64)
    cts = np.stack([ctx.encrypt(sk, slots[i], seed=10 + i) for i in range(2)])
    rots = [(0, 5), (1, 77)]
    gk = ctx.galois_keygen(sk, rots, seed=42)
    d_in = H.import_cts(ctx, cts)
    for swap, step in rots:
        d_out = H.dev_empty(2 * 2 * n)
        ctx.rotate(gk, d_in, 2, (swap, step), d_out)
        got = H.export_cts(ctx, d_out, 2)
        g = o.galois_elt(swap, step)
        for i in range(2):
            assert np.array_equal(got[i], o.perm(cts[i], g, o.galois_key(osk, g, 42))), (swap, step, i)
            assert np.array_equal(ctx.decrypt(sk, got[i]), rotate_slots(slots[i], step, bool(swap)))
    fc_case(par, 64, 512, 2, [0, 1], seed=gb)
    shape = (10, 12, 3, 3, 16, 16)
    conv_case(par, shape, 1, [(0, 0), (0, 1)], seed=gb)
    ctx2, o2, plan, sk2, K, x, r, got, cnt = conv_case(par, shape, 3, [(0, 1), (2, 0)], seed=gb, matrix_cores=True)
    for b in range(3):     # with the special prime the 3x3 layer decrypts at p ~ 2^20
        share = np.zeros((10, 16, 16), np.uint64)
        for O in range(plan.nout):
            plan.unpack_share(O, ctx2.decrypt(sk2, got[b, O]), share)
        assert np.array_equal((share + r[b]) % np.uint64(par.p), plain_conv(K, x[b], par.p))
