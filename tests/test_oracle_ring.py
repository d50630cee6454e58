"""Pins for the oracle's parameters, transforms, ring product and slot encoding.

Each check compares the oracle with something that is not the oracle: Python
big-integer arithmetic, numpy's convolution, closed forms or brute force.
"""
from decimal import Decimal, getcontext

import numpy as np
import pytest

from oracle.oracle import Oracle
from paper_2105_01827_amd import workloads as wl
from tests.helpers import negacyclic_mul, poly_eval, rotate_slots, small_params

RNG = np.random.default_rng(1234)


def rand_poly(n, m):
    return RNG.integers(0, m, size=n, dtype=np.uint64)


# ---------------------------------------------------------------- parameters
def test_default_parameters_are_what_they_claim():
    n, p, q = wl.N, wl.P, wl.Q
    assert wl._is_prime(p) and wl._is_prime(q)
    assert p < 2 ** 20 and p % (2 * n) == 1
    assert not any(wl._is_prime(c) for c in range(p + 2 * n, 2 ** 20, 2 * n))      # largest such p
    assert q.bit_length() == 60 and q % (2 * n * p) == 1
    assert not any(wl._is_prime(c) for c in range(q + 2 * n * p, 2 ** 60, 2 * n * p))
    assert (q - 1) // p * p == q - 1


@pytest.mark.parametrize("n", [4, 8, 64, 2048])
def test_roots_are_primitive_and_zeta_is_the_smallest(n):
    par = small_params(n) if n != 2048 else wl.DEFAULT
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    assert pow(o.psi, n, par.q) == par.q - 1
    assert pow(o.zeta, n, par.p) == par.p - 1
    assert all(pow(x, n, par.p) != par.p - 1 for x in range(2, o.zeta))


def test_digit_count_and_delta():
    o = Oracle(wl.N, wl.Q, wl.P, 20)
    assert o.ndigits == 3 and o.delta * wl.P == wl.Q - 1
    assert Oracle(wl.N, wl.Q, wl.P, 2).ndigits == 30
    assert Oracle(wl.N, wl.Q, wl.P, 16).ndigits == 4


# ---------------------------------------------------------------- transforms
@pytest.mark.parametrize("n", [4, 8, 16, 64])
def test_eval_matches_horner_and_slow_definition(n):
    par = small_params(n)
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    a = rand_poly(n, par.q)
    fast, slow = o.eval_q(a), o.eval_q(a, slow=True)
    assert np.array_equal(fast, slow)
    for k in range(n):
        assert int(fast[k]) == poly_eval(a, pow(o.psi, 2 * k + 1, par.q), par.q)
    assert np.array_equal(o.interp_q(fast), a)
    assert np.array_equal(o.interp_q(fast, slow=True), a)


def test_eval_full_size_matches_slow_definition():
    o = Oracle(wl.N, wl.Q, wl.P, 20)
    a = rand_poly(wl.N, wl.Q)
    fast = o.eval_q(a)
    assert np.array_equal(fast, o.eval_q(a, slow=True))
    for k in (0, 1, 1023, 2047):
        assert int(fast[k]) == poly_eval(a, pow(o.psi, 2 * k + 1, wl.Q), wl.Q)
    assert np.array_equal(o.interp_q(fast), a)


@pytest.mark.parametrize("n", [4, 8, 16, 32, 64])
def test_polymul_is_schoolbook_negacyclic(n):
    par = small_params(n)
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    for _ in range(3):
        a, b = rand_poly(n, par.q), rand_poly(n, par.q)
        ref = negacyclic_mul(a, b, n, par.q)
        assert np.array_equal(o.polymul(a, b), ref)
        assert np.array_equal(o.polymul(a, b, schoolbook=True), ref)


def test_polymul_full_size():
    o = Oracle(wl.N, wl.Q, wl.P, 20)
    a, b = rand_poly(wl.N, wl.Q), rand_poly(wl.N, wl.Q)
    assert np.array_equal(o.polymul(a, b), negacyclic_mul(a, b, wl.N, wl.Q))
    # X * X^(n-1) = X^n = -1
    x1 = np.zeros(wl.N, np.uint64); x1[1] = 1
    xl = np.zeros(wl.N, np.uint64); xl[wl.N - 1] = 1
    minus_one = np.zeros(wl.N, np.uint64); minus_one[0] = wl.Q - 1
    assert np.array_equal(o.polymul(x1, xl), minus_one)


# ---------------------------------------------------------------- slot encoding
@pytest.mark.parametrize("n", [4, 8, 32, 2048])
def test_encode_decode_roundtrip_and_slot_definition(n):
    par = small_params(n) if n != 2048 else wl.DEFAULT
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    v = rand_poly(n, par.p)
    m = o.encode(v)
    assert np.array_equal(o.decode(m), v)
    if n <= 32:
        assert np.array_equal(o.encode(v, slow=True), m)
        assert np.array_equal(o.decode(m, slow=True), v)
    # slot (h,k) is the value of the plaintext polynomial at zeta^(+-3^k)
    for s in ([0, 1, n // 2 - 1, n // 2, n - 1] if n > 8 else range(n)):
        h, k = divmod(s, n // 2)
        e = pow(3, k, 2 * n)
        e = 2 * n - e if h else e
        assert int(v[s]) == poly_eval(m, pow(o.zeta, e, par.p), par.p)


@pytest.mark.parametrize("n", [8, 64])
def test_simd_property_and_automorphisms_on_plaintexts(n):
    par = small_params(n)
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    a, b = rand_poly(n, par.p), rand_poly(n, par.p)
    prod = negacyclic_mul(o.encode(a), o.encode(b), n, par.p)
    assert np.array_equal(o.decode(prod), (a * b) % np.uint64(par.p))          # slot-wise product
    total = (o.encode(a) + o.encode(b)) % np.uint64(par.p)
    assert np.array_equal(o.decode(total), (a + b) % np.uint64(par.p))          # slot-wise sum

    def substitute(m, g):      # m(X) -> m(X^g) mod (X^n+1, p) with Python ints
        out = [0] * n
        for i, c in enumerate(int(x) for x in m):
            e = i * g % (2 * n)
            if e < n:
                out[e] = (out[e] + c) % par.p
            else:
                out[e - n] = (out[e - n] - c) % par.p
        return np.array(out, dtype=np.uint64)

    for step in (1, 3, n // 2 - 1):
        g = o.galois_elt(0, step)
        assert g == pow(3, step, 2 * n)
        assert np.array_equal(o.decode(substitute(o.encode(a), g)), rotate_slots(a, step))
    g = o.galois_elt(1, 0)
    assert g == 2 * n - 1
    assert np.array_equal(o.decode(substitute(o.encode(a), g)), rotate_slots(a, 0, swap=True))
    g = o.galois_elt(1, 2)
    assert np.array_equal(o.decode(substitute(o.encode(a), g)), rotate_slots(a, 2, swap=True))


def test_weight_lift_is_centred():
    par = small_params(16)
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    v = rand_poly(16, par.p)
    m, w = o.encode(v), o.encode_weight(v)
    for c, l in zip(m, w):
        c, l = int(c), int(l)
        assert l == (c if c <= par.p // 2 else par.q - (par.p - c))


# ---------------------------------------------------------------- samplers
def test_gaussian_table_is_the_sigma_3_2_cdf():
    getcontext().prec = 80
    sigma = Decimal("3.2")
    rho = [(-(Decimal(x) ** 2) / (2 * sigma * sigma)).exp() for x in range(-19, 20)]
    z, acc, ref = sum(rho), Decimal(0), []
    for i in range(38):
        acc += rho[i]
        ref.append(int((acc / z * Decimal(2) ** 64).to_integral_value(rounding="ROUND_FLOOR")))
    o = Oracle(8, small_params(8).q, small_params(8).p, 20)
    assert o.gauss_cdf() == ref


def test_sampler_statistics_and_ranges():
    o = Oracle(8, small_params(8).q, small_params(8).p, 20)
    N = 60000
    g = np.array([o.gauss(7, 5, i) for i in range(N)])
    assert abs(g.mean()) < 0.06 and abs(g.var() - 3.2 ** 2) < 0.3 and np.abs(g).max() <= 19
    t = np.array([o.ternary(7, 1, i) for i in range(N)])
    for v in (-1, 0, 1):
        assert abs((t == v).mean() - 1 / 3) < 0.01
    u = np.array([o.uniform(wl.P, 7, 6, i) for i in range(N)])
    assert u.max() < wl.P and abs(u.mean() / wl.P - 0.5) < 0.01
    uq = [o.uniform(wl.Q, 7, 4, i) for i in range(2000)]
    assert max(uq) < wl.Q and min(uq) >= 0 and len(set(uq)) == 2000
    # streams and seeds are independent inputs of the generator
    assert o.rand64(1, 2, 3) != o.rand64(1, 3, 2) and o.rand64(1, 2, 3) != o.rand64(2, 2, 3)
    assert o.rand64(1, 2, 3, 0) != o.rand64(1, 2, 3, 1)


def _splitmix64_stream(seed, count):
    """SplitMix64 as published (Steele, Lea, Flood 2014; the reference C version by Vigna): the state advances by the
    golden-ratio constant, the output is the state through two xor-shift-multiply rounds and a final xor-shift."""
    mask, out, state = (1 << 64) - 1, [], seed
    for _ in range(count):
        state = (state + 0x9E3779B97F4A7C15) & mask
        z = state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
        out.append(z ^ (z >> 31))
    return out


# first outputs of SplitMix64 seeded with 0, as published with the reference implementation
SPLITMIX64_SEED0 = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_generator_is_splitmix64_output_function_composed_four_times():
    """The samplers' bit recipe is this build's own, but its core is a published function with published outputs:
    mix64 of the oracle against SplitMix64's test vector for seed 0, and rand64 against the stated composition."""
    assert _splitmix64_stream(0, 3) == SPLITMIX64_SEED0
    o = Oracle(8, small_params(8).q, small_params(8).p, 20)
    phi, mask = 0x9E3779B97F4A7C15, (1 << 64) - 1
    assert o.mix64(phi) == SPLITMIX64_SEED0[0]
    assert o.mix64((2 * phi) & mask) == SPLITMIX64_SEED0[1] and o.mix64((3 * phi) & mask) == SPLITMIX64_SEED0[2]

    def mix(z):      # one output of the published generator whose state was z - phi
        return _splitmix64_stream((z - phi) & mask, 1)[0]

    for seed, stream, idx, attempt in [(0, 0, 0, 0), (1, 2, 3, 0), (17, 6, (5 << 32) + (3 << 16) + 9, 2), (mask, mask, mask, mask)]:
        want = mix((mix((mix((mix((seed + phi) & mask) + stream) & mask) + idx) & mask) + attempt) & mask)
        assert o.rand64(seed, stream, idx, attempt) == want
