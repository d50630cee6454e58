"""CPU-side checks of the HIP library: it loads, exports the whole C ABI, and its
host-side (client) functions agree bit for bit with the oracle.  No GPU needed."""
import os
import re

import numpy as np
import pytest

from oracle.oracle import Oracle
from paper_2105_01827_amd import binding, workloads as wl
from tests.helpers import small_params

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
RNG = np.random.default_rng(7)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "gala.h")).read()
    declared = set(re.findall(r"\b(gala_[A-Za-z0-9_]+)\s*\(", header))
    lib = binding.load()
    assert declared == set(binding.SIGNATURES), declared ^ set(binding.SIGNATURES)
    for name in declared:
        assert hasattr(lib, name), name


def test_bad_parameters_are_rejected():
    lib = binding.load()
    for n, q, p, gb in [(100, wl.Q, wl.P, 20), (4096, wl.Q, wl.P, 20), (16384, wl.find_prime_below(1 << 60, 32768 * 65537), 65537, 20), (2048, wl.Q + 2, wl.P, 20),
                        (2048, wl.Q, wl.P + 4096, 20), (2048, wl.Q, wl.P, 0), (2048, wl.Q, wl.P, 1),
                        (2048, 12289, 12289, 4)]:
        with pytest.raises(binding.GalaError) as e:
            binding.Context(n, q, p, gb)
        assert e.value.code == binding.GALA_EARG
    assert lib.gala_ctx_create(None, None) == binding.GALA_EARG


@pytest.mark.parametrize("n", [8, 64, 2048])
def test_client_side_functions_match_the_oracle_bit_for_bit(n):
    par = small_params(n) if n != 2048 else wl.DEFAULT
    ctx = binding.Context(par.n, par.q, par.p, par.gadget_bits)
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    assert ctx.ndigits == o.ndigits and ctx.delta == o.delta
    assert ctx.gauss_cdf() == o.gauss_cdf()
    sk = ctx.keygen(5)
    osk = o.keygen(5)
    assert np.array_equal(sk.export(), osk)
    v = RNG.integers(0, par.p, n, dtype=np.uint64)
    assert np.array_equal(ctx.encode(v), o.encode(v))
    assert np.array_equal(ctx.decode(ctx.encode(v)), v)
    assert np.array_equal(ctx.decode(v), o.decode(v))
    ct = ctx.encrypt(sk, v, seed=123)
    assert np.array_equal(ct, o.encrypt(osk, v, seed=123))
    assert np.array_equal(ctx.decrypt(sk, ct), v)
    # decrypting an oracle-made ciphertext after homomorphic work
    w = RNG.integers(0, par.p, n, dtype=np.uint64)
    prod = o.scmult(ct, o.encode_weight(w))
    assert np.array_equal(ctx.decrypt(sk, prod), o.decrypt(osk, prod))
    assert np.array_equal(ctx.decrypt(sk, prod), v * w % np.uint64(par.p))


def test_device_entry_points_reject_null_arguments_and_missing_devices():
    """Argument checks come before any device work, so they can be exercised here; without a GPU every device
    entry point answers GALA_EHIP instead of falling back to host code."""
    import ctypes as C
    import torch
    lib = binding.load()
    par = wl.DEFAULT
    ctx = binding.Context(par.n, par.q, par.p, par.gadget_bits)
    null = C.c_void_p(None)
    one = C.c_void_p(8)          # a non-null placeholder that is never dereferenced on these paths
    assert lib.gala_gk_count(null) == binding.GALA_EARG
    assert lib.gala_rotate_hoisted(ctx.h, null, null, one, 1, one, one, 64) == binding.GALA_EARG
    assert lib.gala_rotate_hoisted_workspace(null, 4) == 0 and lib.gala_rotate_hoisted_workspace(ctx.h, 0) == 0
    assert lib.gala_rotate_hoisted_workspace(ctx.h, 3) >= 3 * 3 * par.n * 8
    assert lib.gala_fc_unpack_share_batch(null, null, one, 1, one) == binding.GALA_EARG
    assert lib.gala_conv_unpack_share_batch(null, null, one, 1, one) == binding.GALA_EARG
    assert lib.gala_encrypt_batch(ctx.h, null, null, one, one, 1, one) == binding.GALA_EARG
    assert lib.gala_add(ctx.h, null, null, one, 1, one) == binding.GALA_EARG
    if not torch.cuda.is_available():
        sk = ctx.keygen(1)
        with pytest.raises(binding.GalaError) as e:
            ctx.galois_keygen(sk, [(0, 1)], seed=1)
        assert e.value.code == binding.GALA_EHIP
        with pytest.raises(binding.GalaError) as e:
            ctx.fc_plan(np.ones((4, 8), np.uint64))
        assert e.value.code == binding.GALA_EHIP
        with pytest.raises(binding.GalaError) as e:
            ctx.conv_plan(np.ones((2, 2, 3, 3), np.uint64), 4, 4)
        assert e.value.code == binding.GALA_EHIP
        assert lib.gala_add(ctx.h, null, one, one, 1, one) == binding.GALA_EHIP


def test_library_generator_is_splitmix64_and_equals_the_oracles():
    """The library's own copy of the seeded generator: the published SplitMix64 outputs for seed 0, and the same
    words as the oracle's generator on a spread of (seed, stream, index, attempt)."""
    lib = binding.load()
    phi, mask = 0x9E3779B97F4A7C15, (1 << 64) - 1
    assert [lib.gala_mix64((k * phi) & mask) for k in (1, 2, 3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    par = small_params(8)
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    rng = np.random.default_rng(11)
    for _ in range(200):
        seed, stream, idx, attempt = (int(v) for v in rng.integers(0, 1 << 63, size=4, dtype=np.uint64))
        stream %= 8
        assert lib.gala_rand64(seed, stream, idx, attempt) == o.rand64(seed, stream, idx, attempt)
