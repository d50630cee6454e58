"""Pins for the oracle's row-encoding-share-RaS matrix-vector product (Sec. III-A(3))."""
import os

import numpy as np
import pytest

from oracle.oracle import Oracle
from paper_2105_01827_amd import workloads as wl
from tests.helpers import rotate_slots, small_params

GOLD = os.path.join(os.path.dirname(__file__), "golden", "fc_toy_2x4.txt")


def golden():
    out = {}
    for line in open(GOLD):
        if line.startswith("#") or ":" not in line:
            continue
        k, v = line.split(":", 1)
        out[k.strip()] = v.split()
    return out


def plain_matvec(W, x, p):
    return np.array([sum(int(a) * int(b) for a, b in zip(row, x)) % p for row in W], dtype=np.uint64)


def test_toy_example_of_the_paper():
    """n = n_i = 4, n_o = 2: the encoded vectors and the slot contents the prose describes."""
    gold = golden()
    par = small_params(4, p_limit=1 << 12)
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    ident = {f"{r}{c + 1}": 10 * (ri + 1) + c + 1 for ri, r in enumerate("AB") for c in range(4)}   # A1=11.. B4=24
    W = np.array([[ident[f"{r}{c + 1}"] for c in range(4)] for r in "AB"], dtype=np.uint64)
    assert o.fc_G(2, 4) == 2
    assert [int(v) for v in o.fc_weight_slots(W, 0)] == [ident[t] for t in gold["w0"]]
    assert [int(v) for v in o.fc_weight_slots(W, 1)] == [ident[t] for t in gold["w1"]]
    x = np.array([3, 5, 7, 9], dtype=np.uint64)
    xs = o.fc_pack_input(2, 4, x)
    assert np.array_equal(xs, x)                                    # no copies when n_i = n
    u0 = o.fc_weight_slots(W, 0) * xs
    u1 = o.fc_weight_slots(W, 1) * xs
    assert int(u0[0]) == ident["A1"] * 3 and int(u1[0]) == ident["B1"] * 3
    total = u0 + rotate_slots(u1, 1)
    # slot j is a partial sum of output j mod 2, and the two halves complete it
    assert np.array_equal(o.fc_unpack_share(2, 4, total % np.uint64(par.p)), plain_matvec(W, x, par.p))


SHAPES = [(16, 128), (128, 1024), (1000, 2048), (1024, 2048), (2, 2048), (1, 2048), (2, 1024),
          (16, 512), (16, 64), (10, 100), (512, 1000), (256, 4), (1024, 8)]


@pytest.mark.parametrize("n_o,n_i", SHAPES)
def test_every_weight_is_used_exactly_once_and_meets_its_input(n_o, n_i):
    """Brute force over all (g, slot): ids of W cover the matrix once, each next to its own column."""
    n = 2048
    big_p = wl.find_prime_below(1 << 30, 2 * n)           # ids up to n_o*n_i need more than 20 bits
    o = Oracle(n, wl.find_prime_below(1 << 60, 2 * n), big_p, 20)
    W = (np.arange(n_o * n_i, dtype=np.uint64) + 1).reshape(n_o, n_i)
    x_ids = np.arange(n_i, dtype=np.uint64) + 1
    xs = o.fc_pack_input(n_o, n_i, x_ids)
    G = o.fc_G(n_o, n_i)
    nop, nip = 1 << (n_o - 1).bit_length(), 1 << (n_i - 1).bit_length()
    assert G == max(1, nop * nip // n) if nip < n else G == nop
    seen = np.zeros(n_o * n_i + 1, dtype=np.int64)
    rows_at_slot = np.full(n, -1, dtype=np.int64)
    for g in range(G):
        w = o.fc_weight_slots(W, g)
        ids = w[w > 0].astype(np.int64)
        np.add.at(seen, ids, 1)
        cols = (ids - 1) % n_i
        assert np.array_equal(xs[w > 0].astype(np.int64) - 1, cols)          # weight sits on its own input entry
        # after the left rotation by g the product must land on a slot of its own row
        rot = rotate_slots(w, g).astype(np.int64)
        rows = np.where(rot > 0, (rot - 1) // n_i, -1)
        fresh = (rows_at_slot < 0) & (rows >= 0)
        rows_at_slot[fresh] = rows[fresh]
        assert np.all((rows < 0) | (rows == rows_at_slot))
    assert np.all(seen[1:] == 1)
    # unpack_share adds exactly the slots of each row
    ones = np.ones(n, dtype=np.uint64)
    counts = o.fc_unpack_share(n_o, n_i, ones)
    for t in range(0, n_o, max(1, n_o // 7)):
        seen_slots = int(np.sum(rows_at_slot == t))
        assert seen_slots <= int(counts[t])
        if (nop, nip) == (n_o, n_i):                 # no zero padding: every slot of the row carries a weight
            assert seen_slots == int(counts[t]) == min(n, nop * nip) // nop


@pytest.mark.parametrize("n,n_o,n_i,batch", [(64, 4, 16, 2), (64, 8, 32, 1), (64, 16, 64, 1), (64, 3, 20, 1),
                                             (256, 2, 256, 1), (2048, 16, 128, 1), (2048, 2, 2048, 1)])
def test_he_fc_identity_counts_and_mask(n, n_o, n_i, batch):
    par = small_params(n) if n != 2048 else wl.DEFAULT
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    W, x, r = wl.fc_inputs(wl.FcShape("t", n_o, n_i, batch), p=par.p, seed=n_o)
    sk = o.keygen(0)
    wpoly = o.fc_encode_rowwise(W)
    ksk = o.fc_keys(sk, n_o, n_i, seed=1)
    G = o.fc_G(n_o, n_i)
    for b in range(batch):
        ct = o.encrypt(sk, o.fc_pack_input(n_o, n_i, x[b]), seed=b)
        mask = o.fc_mask_slots(n_o, n_i, r[b], seed=17, b=b)
        assert np.array_equal(o.fc_unpack_share(n_o, n_i, mask), r[b])           # server's share after plaintext RaS
        out, cnt = o.he_fc(wpoly, ct, ksk, mask)
        share = o.fc_unpack_share(n_o, n_i, o.decrypt(sk, out))                  # client's share
        assert np.array_equal((share + r[b]) % np.uint64(par.p), plain_matvec(W, x[b], par.p))
        assert cnt == dict(perm=G - 1, decperm_in=0, hstperm_in=0, scmult=G, add=G - 1)   # Table "complexity"
    # batch entry point gives the same ciphertexts
    cts = np.stack([o.encrypt(sk, o.fc_pack_input(n_o, n_i, x[b]), seed=b) for b in range(batch)])
    outs, cnt = o.he_fc_batch(wpoly, n_o, n_i, cts, ksk, r, mask_seed=17)
    assert np.array_equal(outs[batch - 1], out) and cnt["perm"] == batch * (G - 1)


def test_paper_instance_counts():
    gold = golden()
    o = Oracle(wl.N, wl.Q, wl.P, 20)
    for key, (n_o, n_i) in {"counts_2x2048": (2, 2048), "counts_1x2048": (1, 2048),
                            "counts_2x1024": (2, 1024), "counts_16x128": (16, 128)}.items():
        want = dict(kv.split("=") for kv in gold[key])
        G = o.fc_G(n_o, n_i)
        assert (G - 1, G, G - 1) == (int(want["perm"]), int(want["scmult"]), int(want["add"]))


def test_config2_one_input_full_size_decrypts_with_margin():
    """128x1024 at n = 2048: 64 ScMult, 63 Perm; the result decrypts and the noise has margin."""
    par = wl.DEFAULT
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    W, x, r = wl.fc_inputs(wl.FcShape("t", 128, 1024, 1))
    sk = o.keygen(0)
    wpoly, ksk = o.fc_encode_rowwise(W), o.fc_keys(sk, 128, 1024, seed=1)
    ct = o.encrypt(sk, o.fc_pack_input(128, 1024, x[0]), seed=0)
    mask = o.fc_mask_slots(128, 1024, r[0], seed=5, b=0)
    out, cnt = o.he_fc(wpoly, ct, ksk, mask)
    dec = o.decrypt(sk, out)
    assert np.array_equal((o.fc_unpack_share(128, 1024, dec) + r[0]) % np.uint64(par.p), plain_matvec(W, x[0], par.p))
    assert cnt == dict(perm=63, decperm_in=0, hstperm_in=0, scmult=64, add=63)
    assert o.noise(sk, out, dec) < o.delta // 2 ** 4
