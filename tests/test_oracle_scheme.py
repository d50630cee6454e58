"""Pins for the oracle's encryption, Add / ScMult / Perm (Sec. II-C(1)) and key switching."""
import numpy as np
import pytest

from oracle.oracle import Oracle
from paper_2105_01827_amd import workloads as wl
from tests.helpers import centred, negacyclic_mul, rotate_slots, small_params

RNG = np.random.default_rng(99)


def make(n, **kw):
    par = small_params(n, **kw) if n != 2048 or kw else wl.DEFAULT
    return par, Oracle(par.n, par.q, par.p, par.gadget_bits)


@pytest.mark.parametrize("n", [8, 64, 2048])
def test_encrypt_decrypt_roundtrip_and_fresh_noise(n):
    par, o = make(n)
    sk = o.keygen(5)
    assert set(int(v) for v in sk) <= {0, 1, par.q - 1}
    v = RNG.integers(0, par.p, n, dtype=np.uint64)
    ct = o.encrypt(sk, v, seed=11)
    assert np.array_equal(o.decrypt(sk, ct), v)
    assert o.noise(sk, ct, v) <= 19                      # the Gaussian is cut at 6 sigma
    # c0 + c1*s - delta*m is exactly the sampled error polynomial
    phase = (negacyclic_mul(ct[n:], sk, n, par.q).astype(object) + ct[:n].astype(object)) % par.q
    m = o.encode(v)
    err = [centred((int(ph) - o.delta * int(mm)) % par.q, par.q) for ph, mm in zip(phase, m)]
    assert err == [o.gauss(11, 5, i) for i in range(n)]
    assert [int(a) for a in ct[n:]] == [o.uniform(par.q, 11, 4, i) for i in range(n)]


@pytest.mark.parametrize("n", [16, 2048])
def test_add_and_scmult_act_slotwise(n):
    par, o = make(n)
    sk = o.keygen(1)
    p = np.uint64(par.p)
    a, b, w = (RNG.integers(0, par.p, n, dtype=np.uint64) for _ in range(3))
    ca, cb = o.encrypt(sk, a, 1), o.encrypt(sk, b, 2)
    assert np.array_equal(o.decrypt(sk, o.add(ca, cb)), (a + b) % p)
    prod = o.scmult(ca, o.encode_weight(w))
    assert np.array_equal(o.decrypt(sk, prod), (a * w) % p)
    # multiplicative noise growth stays far below delta/2 for one ScMult (Sec. III-C)
    assert o.noise(sk, prod, (a * w) % p) < o.delta // 2 ** 8
    masked = o.sub_plain(prod, b)
    assert np.array_equal(o.decrypt(sk, masked), (a * w + p - b) % p)


def test_decomposition_recomposes_and_is_bounded():
    par, o = make(2048)
    c1 = RNG.integers(0, par.q, par.n, dtype=np.uint64)
    d = o.decperm(c1).reshape(3, par.n)
    assert d.max() < 2 ** 20
    assert np.array_equal(d[0] + (d[1] << np.uint64(20)) + (d[2] << np.uint64(40)), c1)


@pytest.mark.parametrize("n,steps", [(8, "all"), (64, "all"), (2048, [1, 5, 63, 512, 1023])])
def test_perm_rotates_the_slots(n, steps):
    par, o = make(n)
    sk = o.keygen(3)
    v = RNG.integers(0, par.p, n, dtype=np.uint64)
    ct = o.encrypt(sk, v, 4)
    cases = [(s, r) for s in (0, 1) for r in (range(n // 2) if steps == "all" else steps) if (s, r) != (0, 0)]
    if steps != "all":
        cases.append((1, 0))
    worst = 0
    for swap, step in cases:
        g = o.galois_elt(swap, step)
        ksk = o.galois_key(sk, g, seed=77)
        out = o.perm(ct, g, ksk)
        want = rotate_slots(v, step, bool(swap))
        assert np.array_equal(o.decrypt(sk, out), want), (swap, step)
        worst = max(worst, o.noise(sk, out, want))
        # hoisted form is the same function
        assert np.array_equal(o.hstperm(ct[:n], o.decperm(ct[n:]), g, ksk), out)
    # additive rotation noise: about sqrt(3n) * B/sqrt(3) * sigma, far below delta/2 ~ 2^39
    assert worst < 2 ** 33


def test_galois_key_encrypts_gadget_multiples_of_rotated_secret():
    par, o = make(64)
    sk = o.keygen(9)
    g = o.galois_elt(1, 5)
    ksk = o.galois_key(sk, g, seed=21).reshape(o.ndigits, 2, par.n)
    sg = o.apply_galois(sk, g)
    for j in range(o.ndigits):
        phase = (negacyclic_mul(ksk[j, 1], sk, par.n, par.q).astype(object) + ksk[j, 0].astype(object)) % par.q
        want = (pow(2, 20 * j, par.q) * sg.astype(object)) % par.q
        err = [centred((int(a) - int(b)) % par.q, par.q) for a, b in zip(phase, want)]
        assert max(abs(e) for e in err) <= 19
        assert err == [o.gauss(21, 3, (g << 32) + (j << 16) + i) for i in range(par.n)]


def test_apply_galois_is_substitution():
    par, o = make(16)
    a = RNG.integers(0, par.q, 16, dtype=np.uint64)
    for g in (3, 9, 31, 27):
        out = [0] * 16
        for i, c in enumerate(int(x) for x in a):
            e = i * g % 32
            if e < 16:
                out[e] = (out[e] + c) % par.q
            else:
                out[e - 16] = (out[e - 16] - c) % par.q
        assert [int(x) for x in o.apply_galois(a, g)] == out


def test_many_digit_gadget_also_rotates():
    par, o = make(64, gadget_bits=2)
    assert o.ndigits == 30
    sk = o.keygen(3)
    v = RNG.integers(0, par.p, 64, dtype=np.uint64)
    ct = o.encrypt(sk, v, 4)
    g = o.galois_elt(0, 7)
    out = o.perm(ct, g, o.galois_key(sk, g, 5))
    assert np.array_equal(o.decrypt(sk, out), rotate_slots(v, 7))
    assert o.noise(sk, out, rotate_slots(v, 7)) < 2 ** 14
