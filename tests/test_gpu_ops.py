"""GPU parity of the stand-alone homomorphic operations Add, ScMult and plaintext add / subtract (Sec. II-C(1))
against the oracle, and a matrix wider than n composed from two blocks with them (Sec. III-A: larger matrices
are split into blocks that are processed independently)."""
import numpy as np
import pytest

from paper_2105_01827_amd import workloads as wl
from tests.helpers import small_params
from tests.test_gpu_parity import both, harness, plain_matvec

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,count", [(8, 2), (64, 5), (2048, 3)])
def test_add_scmult_and_plain_operations_match_the_oracle(n, count):
    H = harness()
    par = small_params(n) if n != 2048 else wl.DEFAULT
    ctx, o = both(par)
    sk, osk = ctx.keygen(2), o.keygen(2)
    rng = np.random.default_rng(n)
    p = np.uint64(par.p)
    va, vb, vw = (rng.integers(0, par.p, size=(count, n), dtype=np.uint64) for _ in range(3))
    ca = np.stack([o.encrypt(osk, va[i], seed=i) for i in range(count)])
    cb = np.stack([o.encrypt(osk, vb[i], seed=100 + i) for i in range(count)])
    d_a, d_b = H.import_cts(ctx, ca), H.import_cts(ctx, cb)
    d_out = H.dev_empty(count * 2 * n)
    # Add
    ctx.add(d_a, d_b, count, d_out)
    got = H.export_cts(ctx, d_out, count)
    for i in range(count):
        assert np.array_equal(got[i], o.add(ca[i], cb[i]))
        assert np.array_equal(ctx.decrypt(sk, got[i]), (va[i] + vb[i]) % p)
    # ScMult with one plaintext per ciphertext, then with a shared one, in place
    d_w = H.dev_empty(count * n)
    ctx.encode_plain(H.to_dev(vw), count, 0, d_w)
    ctx.scmult(d_a, d_w, count, d_out)
    got = H.export_cts(ctx, d_out, count)
    for i in range(count):
        assert np.array_equal(got[i], o.scmult(ca[i], o.encode_weight(vw[i])))
        assert np.array_equal(ctx.decrypt(sk, got[i]), (va[i] * vw[i]) % p)
    ctx.scmult(d_b, d_w, count, d_b, shared=True)
    got = H.export_cts(ctx, d_b, count)
    for i in range(count):
        assert np.array_equal(got[i], o.scmult(cb[i], o.encode_weight(vw[0])))
    # plaintext subtraction (share generation on its own) and addition
    d_m = H.dev_empty(count * n)
    ctx.encode_plain(H.to_dev(vb), count, 1, d_m)
    ctx.sub_plain(d_a, d_m, count, d_out)
    got = H.export_cts(ctx, d_out, count)
    for i in range(count):
        assert np.array_equal(got[i], o.sub_plain(ca[i], vb[i]))
        assert np.array_equal(ctx.decrypt(sk, got[i]), (va[i] + p - vb[i]) % p)
    ctx.add_plain(d_out, d_m, count, d_out)
    assert np.array_equal(H.export_cts(ctx, d_out, count), ca)


def test_matrix_wider_than_n_from_two_blocks():
    """W is 8 x 128 on a ring with n = 64 slots: two 8 x 64 blocks, one he_fc each (the mask on the first only),
    outputs added.  Bit-exact against the same composition of oracle calls, and the shares add up to W x."""
    import torch
    H = harness()
    par = small_params(64)
    ctx, o = both(par)
    sk, osk = ctx.keygen(0), o.keygen(0)
    rng = np.random.default_rng(5)
    n_o, half, batch = 8, 64, 3
    W = rng.integers(0, par.p, size=(n_o, 2 * half), dtype=np.uint64)
    x = rng.integers(0, par.p, size=(batch, 2 * half), dtype=np.uint64)
    r = rng.integers(0, par.p, size=(batch, n_o), dtype=np.uint64)
    zero = np.zeros_like(r)
    outs, wants = [], []
    for blk in range(2):
        Wb, xb = np.ascontiguousarray(W[:, blk * half:(blk + 1) * half]), x[:, blk * half:(blk + 1) * half]
        plan = ctx.fc_plan(Wb)
        gk = ctx.galois_keygen(sk, plan.rotations(), seed=1)
        plan.bind(gk)
        cts = np.stack([ctx.encrypt(sk, plan.pack_input(xb[b]), seed=10 * blk + b) for b in range(batch)])
        rb = r if blk == 0 else zero
        got, _ = H.gpu_he_fc(ctx, plan, cts, rb, mask_seed=7 + blk)
        outs.append(got)
        wpoly, ksk = o.fc_encode_rowwise(Wb), o.fc_keys(osk, n_o, half, seed=1)
        wants.append(np.stack([o.he_fc(wpoly, cts[b], ksk, o.fc_mask_slots(n_o, half, rb[b], 7 + blk, b))[0]
                               for b in range(batch)]))
        keep = plan
    d_sum = H.dev_empty(batch * 2 * par.n)
    ctx.add(H.import_cts(ctx, outs[0]), H.import_cts(ctx, outs[1]), batch, d_sum)
    total = H.export_cts(ctx, d_sum, batch)
    for b in range(batch):
        assert np.array_equal(total[b], o.add(wants[0][b], wants[1][b]))
        share = keep.unpack_share(ctx.decrypt(sk, total[b]))
        assert np.array_equal((share + r[b]) % np.uint64(par.p), plain_matvec(W, x[b], par.p))
