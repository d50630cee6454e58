"""Rings above the paper's n = 2048 (n = 4096 and 8192, one 60-bit prime) on the any-n kernels: the same parity as
everywhere else, the library against the oracle bit for bit through the C ABI."""
import dataclasses

import numpy as np
import pytest

from oracle.oracle import Oracle
from paper_2105_01827_amd import binding, workloads as wl
from tests.helpers import rotate_slots, small_params
from tests.test_gpu_parity import conv_case, fc_case, plain_conv, plain_matvec

pytestmark = pytest.mark.gpu


def both(par):
    return (binding.Context(par.n, par.q, par.p, par.gadget_bits, par.special),
            Oracle(par.n, par.q, par.p, par.gadget_bits, special=par.special))


@pytest.mark.parametrize("n", [4096, 8192])
def test_transforms_keys_and_client_steps(n):
    import torch
    from paper_2105_01827_amd import devmem as D
    par = small_params(n)
    ctx, o = both(par)
    rng = np.random.default_rng(n)
    cts = rng.integers(0, par.q, size=(3, 2 * n), dtype=np.uint64)
    dev = D.import_cts(ctx, cts)
    assert np.array_equal(D.export_cts(ctx, dev, 3), cts)
    sk, osk = ctx.keygen(3), o.keygen(3)
    assert np.array_equal(sk.export(), osk)
    rots = [(0, 1), (1, n // 2 - 1)]
    gk = ctx.galois_keygen(sk, rots, seed=42)
    for swap, step in rots:
        assert np.array_equal(gk.export((swap, step)), o.galois_key(osk, o.galois_elt(swap, step), 42))
    # the client's two steps on the device against the oracle's
    slots = rng.integers(0, par.p, size=(4, n), dtype=np.uint64)
    d_ct = D.dev_empty(4 * 2 * n)
    ctx.encrypt_batch(sk, D.to_dev(slots), D.to_dev(np.arange(4, dtype=np.uint64) + 7), 4, d_ct)
    got = D.export_cts(ctx, d_ct, 4)
    for b in range(4):
        assert np.array_equal(got[b], o.encrypt(osk, slots[b], 7 + b))
    d_slots = D.dev_empty(4 * n)
    ctx.decrypt_batch(sk, d_ct, 4, d_slots)
    torch.cuda.synchronize()
    assert np.array_equal(D.to_host(d_slots).reshape(4, n), slots)


@pytest.mark.parametrize("n,gb,special", [(4096, 20, False), (8192, 20, False), (8192, 30, True)])
def test_rotate_matches_oracle_perm(n, gb, special):
    from paper_2105_01827_amd import devmem as D
    par = small_params(n, gadget_bits=gb)
    if special:
        P = wl.find_prime_below(1 << 60, 2 * n)
        par = dataclasses.replace(par, special=P if P != par.q else wl.find_prime_below(P, 2 * n))
    ctx, o = both(par)
    sk, osk = ctx.keygen(3), o.keygen(3)
    rng = np.random.default_rng(5)
    slots = rng.integers(0, par.p, size=(2, n), dtype=np.uint64)
    cts = np.stack([ctx.encrypt(sk, slots[i], seed=10 + i) for i in range(2)])
    rots = [(0, 1), (0, n // 2 - 1), (1, 0), (1, 1000)]
    gk = ctx.galois_keygen(sk, rots, seed=42)
    d_in = D.import_cts(ctx, cts)
    for swap, step in rots:
        d_out = D.dev_empty(2 * 2 * n)
        ctx.rotate(gk, d_in, 2, (swap, step), d_out)
        got = D.export_cts(ctx, d_out, 2)
        g = o.galois_elt(swap, step)
        ksk = o.galois_key(osk, g, 42)
        for i in range(2):
            assert np.array_equal(got[i], o.perm(cts[i], g, ksk)), (swap, step, i)
            assert np.array_equal(ctx.decrypt(sk, got[i]), rotate_slots(slots[i], step, bool(swap)))


@pytest.mark.parametrize("n,n_o,n_i,batch", [(4096, 8, 2048, 2), (4096, 100, 4096, 1), (8192, 16, 2048, 3)])
def test_he_fc(n, n_o, n_i, batch):
    par = small_params(n)
    ctx, o, plan, sk, W, x, r, got = fc_case(par, n_o, n_i, batch, list(range(batch)), seed=n_o)
    for b in range(batch):
        share = plan.unpack_share(ctx.decrypt(sk, got[b]))
        assert np.array_equal((share + r[b]) % np.uint64(par.p), plain_matvec(W, x[b], par.p))


@pytest.mark.parametrize("n,shape,batch,mc", [
    (4096, (16, 32, 3, 3, 16, 16), 1, False),      # c_n = 16: two input ciphertexts, one output
    (4096, (32, 16, 3, 3, 16, 16), 3, True),       # matrix-core multiply-accumulate
    (8192, (8, 8, 1, 1, 32, 32), 2, False),        # c_n = 8
])
def test_he_conv(n, shape, batch, mc):
    par = small_params(n, p_limit=1 << 17, gadget_bits=4)       # small p: 3x3 results decrypt
    co, ci, kh, kw, uh, uw = shape
    nout = Oracle(par.n, par.q, par.p, par.gadget_bits).conv_geometry(*shape)["nout"]
    picks = [(b, O) for b in range(batch) for O in range(nout)]
    ctx, o, plan, sk, K, x, r, got, cnt = conv_case(par, shape, batch, picks, seed=n, matrix_cores=mc)
    for b in range(batch):
        share = np.zeros((co, uh, uw), np.uint64)
        for O in range(plan.nout):
            plan.unpack_share(O, ctx.decrypt(sk, got[b, O]), share)
        assert np.array_equal((share + r[b]) % np.uint64(par.p), plain_conv(K, x[b], par.p))
