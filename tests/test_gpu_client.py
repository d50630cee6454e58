"""GPU parity of the batched client steps (encryption and decryption on the device, internal ciphertext form)
against the CPU oracle's encrypt / decrypt (Sec. II-C(1)), bit for bit, through the C ABI."""
import numpy as np
import pytest

from paper_2105_01827_amd import workloads as wl
from tests.helpers import small_params
from tests.test_gpu_parity import both, fc_case, harness, plain_matvec

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,count", [(8, 3), (64, 5), (512, 4), (2048, 7)])
def test_encrypt_batch_matches_oracle_encrypt(n, count):
    H = harness()
    par = small_params(n) if n != 2048 else wl.DEFAULT
    ctx, o = both(par)
    sk, osk = ctx.keygen(9), o.keygen(9)
    rng = np.random.default_rng(n)
    slots = rng.integers(0, par.p, size=(count, n), dtype=np.uint64)
    slots[0, :3] += np.uint64(par.p)                    # values are reduced mod p on the way in
    seeds = np.array([11 + 1000 * i for i in range(count)], dtype=np.uint64)
    d_ct = H.dev_empty(count * 2 * n)
    ctx.encrypt_batch(sk, H.to_dev(slots), H.to_dev(seeds), count, d_ct)
    got = H.export_cts(ctx, d_ct, count)
    for i in range(count):
        assert np.array_equal(got[i], o.encrypt(osk, slots[i] % np.uint64(par.p), int(seeds[i]))), i
        assert np.array_equal(got[i], ctx.encrypt(sk, slots[i] % np.uint64(par.p), int(seeds[i])))
    ctx.encrypt_batch(sk, H.to_dev(slots), H.to_dev(seeds), 0, d_ct)          # an empty batch is a no-op


@pytest.mark.parametrize("n,count", [(8, 3), (64, 5), (512, 4), (2048, 7)])
def test_decrypt_batch_matches_oracle_decrypt(n, count):
    H = harness()
    par = small_params(n) if n != 2048 else wl.DEFAULT
    ctx, o = both(par)
    sk, osk = ctx.keygen(4), o.keygen(4)
    rng = np.random.default_rng(n + 1)
    slots = rng.integers(0, par.p, size=(count, n), dtype=np.uint64)
    cts = np.stack([o.encrypt(osk, slots[i], seed=5 + i) for i in range(count)])
    # make the rounding matter: also decrypt arbitrary ring elements (results are whatever the formula gives)
    junk = rng.integers(0, par.q, size=(2, 2 * n), dtype=np.uint64)
    allc = np.concatenate([cts, junk])
    d_slots = H.dev_empty((count + 2) * n)
    ctx.decrypt_batch(sk, H.import_cts(ctx, allc), count + 2, d_slots)
    got = H.to_host(d_slots).reshape(count + 2, n)
    for i in range(count):
        assert np.array_equal(got[i], slots[i])
    for i in range(count + 2):
        assert np.array_equal(got[i], o.decrypt(osk, allc[i])), i


def test_client_and_server_on_the_device_end_to_end():
    """encrypt_batch -> he_fc -> decrypt_batch without leaving the device; the shares add up to W x."""
    import torch
    H = harness()
    par = wl.DEFAULT
    ctx, o = both(par)
    shape = wl.FcShape("t", 128, 1024, 6)
    W, x, r = wl.fc_inputs(shape, seed=3)
    sk = ctx.keygen(0)
    plan = ctx.fc_plan(W)
    plan.bind(ctx.galois_keygen(sk, plan.rotations(), seed=1))
    slots = np.stack([plan.pack_input(x[b]) for b in range(shape.batch)])
    seeds = np.arange(shape.batch, dtype=np.uint64)
    d_in, d_out = H.dev_empty(shape.batch * 2 * par.n), H.dev_empty(shape.batch * 2 * par.n)
    ctx.encrypt_batch(sk, H.to_dev(slots), H.to_dev(seeds), shape.batch, d_in)
    wsb = plan.workspace_bytes(shape.batch)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    plan.he_fc(d_in, shape.batch, H.to_dev(r), 17, d_out, ws, wsb)
    d_slots = H.dev_empty(shape.batch * par.n)
    ctx.decrypt_batch(sk, d_out, shape.batch, d_slots)
    dec = H.to_host(d_slots).reshape(shape.batch, par.n)
    for b in range(shape.batch):
        share = plan.unpack_share(dec[b])
        assert np.array_equal((share + r[b]) % np.uint64(par.p), plain_matvec(W, x[b], par.p))


@pytest.mark.parametrize("n,n_o,n_i", [(64, 4, 16), (64, 16, 8), (512, 10, 100), (2048, 16, 128), (2048, 128, 1024),
                                       (2048, 1000, 2048)])
def test_fc_unpack_share_batch_matches_oracle(n, n_o, n_i):
    """The plaintext sum of every output's slots (Sec. III-A(3)) on the device, against the oracle's and the
    library's host function, on arbitrary slot vectors (values above p are reduced on the way in)."""
    H = harness()
    par = small_params(n) if n != 2048 else wl.DEFAULT
    ctx, o = both(par)
    rng = np.random.default_rng(n_o * n_i)
    W = rng.integers(0, par.p, size=(n_o, n_i), dtype=np.uint64)
    plan = ctx.fc_plan(W)
    count = 3
    slots = rng.integers(0, 2 * par.p, size=(count, n), dtype=np.uint64)
    d_out = H.dev_empty(count * n_o)
    plan.unpack_share_batch(H.to_dev(slots), count, d_out)
    got = H.to_host(d_out).reshape(count, n_o)
    for i in range(count):
        assert np.array_equal(got[i], o.fc_unpack_share(n_o, n_i, slots[i] % np.uint64(par.p))), i
        assert np.array_equal(got[i], plan.unpack_share(slots[i]))
    plan.unpack_share_batch(H.to_dev(slots), 0, d_out)


@pytest.mark.parametrize("n,shape", [(64, (5, 3, 3, 1, 3, 2)), (256, (20, 4, 3, 3, 4, 4)), (2048, (70, 4, 3, 3, 24, 24)),
                                     (2048, (128, 8, 1, 1, 7, 7))])
def test_conv_unpack_share_batch_matches_oracle(n, shape):
    H = harness()
    par = small_params(n) if n != 2048 else wl.DEFAULT
    ctx, o = both(par)
    co, ci, kh, kw, uh, uw = shape
    rng = np.random.default_rng(co + n)
    K = rng.integers(0, par.p, size=(co, ci, kh, kw), dtype=np.uint64)
    plan = ctx.conv_plan(K, uh, uw)
    count = 2
    slots = rng.integers(0, 2 * par.p, size=(count, plan.nout, n), dtype=np.uint64)
    d_out = H.dev_empty(count * co * uh * uw)
    plan.unpack_share_batch(H.to_dev(slots), count, d_out)
    got = H.to_host(d_out).reshape(count, co, uh, uw)
    for i in range(count):
        want = np.zeros((co, uh, uw), np.uint64)
        mine = np.zeros((co, uh, uw), np.uint64)
        for O in range(plan.nout):
            o.conv_unpack_share(shape, O, slots[i, O] % np.uint64(par.p), want)
            plan.unpack_share(O, slots[i, O], mine)
        assert np.array_equal(got[i], want) and np.array_equal(mine, want), i


@pytest.mark.parametrize("qbits,p", [(60, 12289), (50, 1032193), (44, 65537), (59, 40961)])
def test_client_steps_on_the_n2048_kernels_with_other_moduli(qbits, p):
    """encrypt_2048 / decrypt_2048 at other ciphertext and plaintext moduli (uniform draws of other bit lengths, the
    transform mod p, the rounding of decryption) against the oracle, junk ciphertexts included."""
    H = harness()
    n, count = 2048, 3
    par = wl.Params(n=n, q=wl.find_prime_below(1 << qbits, 2 * n * p), p=p, gadget_bits=20)
    ctx, o = both(par)
    sk, osk = ctx.keygen(9), o.keygen(9)
    rng = np.random.default_rng(qbits)
    slots = rng.integers(0, par.p, size=(count, n), dtype=np.uint64)
    seeds = np.array([7 + 100 * i for i in range(count)], dtype=np.uint64)
    d_ct = H.dev_empty(count * 2 * n)
    ctx.encrypt_batch(sk, H.to_dev(slots), H.to_dev(seeds), count, d_ct)
    got = H.export_cts(ctx, d_ct, count)
    for i in range(count):
        assert np.array_equal(got[i], o.encrypt(osk, slots[i], int(seeds[i]))), i
    junk = rng.integers(0, par.q, size=(2, 2 * n), dtype=np.uint64)
    allc = np.concatenate([got, junk])
    d_slots = H.dev_empty((count + 2) * n)
    ctx.decrypt_batch(sk, H.import_cts(ctx, allc), count + 2, d_slots)
    dec = H.to_host(d_slots).reshape(count + 2, n)
    for i in range(count):
        assert np.array_equal(dec[i], slots[i])
    for i in range(count + 2):
        assert np.array_equal(dec[i], o.decrypt(osk, allc[i])), i
