"""GPU tests of whole layers: spatial tiling + stride on top of he_conv, and the ResNet-18-shaped list."""
import ctypes

import numpy as np
import pytest

from oracle.oracle import Oracle
from paper_2105_01827_amd import binding, workloads as wl
from tests.helpers import small_params
from tests.test_gpu_parity import plain_conv

pytestmark = pytest.mark.gpu


def strided_conv(K, x, p, stride):
    return plain_conv(K, x, p)[:, ::stride, ::stride]


def oracle_block(o, shape, K, cts_b, r_tile, mask_seed, b, O, osk, key_seed=8):
    tk, gkk = o.conv_keys(osk, shape, seed=key_seed)
    mask = o.conv_mask_slots(shape, r_tile, mask_seed, b, O)
    want, _ = o.he_conv_block(shape, K, O, cts_b, tk, gkk, mask)
    return want


@pytest.mark.parametrize("n,p_limit,gb,c_o,c_i,k,stride,H,W", [
    (64, 1 << 9, 4, 4, 4, 3, 1, 12, 12),      # tiled in both directions
    (64, 1 << 9, 4, 4, 2, 3, 2, 12, 12),      # tiled and strided
    (64, 1 << 9, 4, 6, 4, 1, 2, 9, 5),        # 1x1 stride 2, one tile covers the width
    (256, 1 << 13, 4, 4, 4, 5, 1, 30, 17),
    (256, 1 << 13, 4, 8, 4, 3, 2, 10, 10),    # single tile, stride 2
])
def test_tiled_strided_layer_matches_plain_convolution(n, p_limit, gb, c_o, c_i, k, stride, H, W):
    from tests import gpu_harness as Hn
    par = small_params(n, p_limit=p_limit, gadget_bits=gb)
    ctx = binding.Context(par.n, par.q, par.p, par.gadget_bits)
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    rng = np.random.default_rng(n + H)
    K = rng.integers(0, par.p, size=(c_o, c_i, k, k), dtype=np.uint64)
    image = rng.integers(0, par.p, size=(c_i, H, W), dtype=np.uint64)
    sk, osk = ctx.keygen(0), o.keygen(0)
    t = ctx.conv_tiling(H, W, k, k, stride)
    r = rng.integers(0, par.p, size=(c_o, t.out_h, t.out_w), dtype=np.uint64)
    t, plan, x_tiles, r_tiles, cts, got, cnt = Hn.gpu_conv_layer(ctx, sk, K, image, r, stride, mask_seed=5)
    share = Hn.stitch_layer_share(ctx, sk, t, plan, got, c_o)
    assert np.array_equal((share + r) % np.uint64(par.p), strided_conv(K, image, par.p, stride))
    # ciphertext parity on one tile / output block
    shape = (c_o, c_i, k, k, t.tile_h, t.tile_w)
    b, O = t.tiles - 1, plan.nout - 1
    assert np.array_equal(o.conv_pack_input(shape, x_tiles[b]), plan.pack_input(x_tiles[b]))
    assert np.array_equal(got[b, O], oracle_block(o, shape, K, cts[b], r_tiles[b], 5, b, O, osk))


def test_resnet18_shaped_layer_list():
    """Config 5: every linear layer of an ImageNet-shaped ResNet-18, one input, random weights mod p.
    Each layer runs in full on the GPU; the oracle recomputes one output ciphertext per layer (a sampled
    tile and output block) and the ciphertexts must agree exactly.  1x1 layers and the FC also decrypt
    (Sec. III-C noise budget) and are checked against the plain strided convolution / matrix product."""
    from tests import gpu_harness as Hn
    par = wl.DEFAULT
    ctx = binding.Context(par.n, par.q, par.p, par.gadget_bits)
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    sk, osk = ctx.keygen(0), o.keygen(0)
    layers, fc = wl.resnet18_layers()
    total = dict(perm=0, decperm_in=0, hstperm_in=0, scmult=0, add=0)
    for li, L in enumerate(layers):
        rng = np.random.default_rng(1000 + li)
        K = rng.integers(0, par.p, size=(L.c_o, L.c_i, L.k, L.k), dtype=np.uint64)
        image = rng.integers(0, par.p, size=(L.c_i, L.in_hw, L.in_hw), dtype=np.uint64)
        t = ctx.conv_tiling(L.in_hw, L.in_hw, L.k, L.k, L.stride)
        r = rng.integers(0, par.p, size=(L.c_o, t.out_h, t.out_w), dtype=np.uint64)
        print(f"layer {L.name}: tiles {t.tiles} of {t.tile_h}x{t.tile_w}", flush=True)
        t, plan, x_tiles, r_tiles, cts, got, cnt = Hn.gpu_conv_layer(ctx, sk, K, image, r, L.stride, mask_seed=li)
        for key in total:
            total[key] += cnt[key]
        # closed forms of Table "Complexity comparison of convolution" per tile
        cn, nin, nout, k2 = plan.cn, plan.nin, plan.nout, L.k * L.k
        assert cnt["perm"] == t.tiles * nout * (cn - 1) and cnt["scmult"] == t.tiles * nout * cn * nin * k2
        assert cnt["hstperm_in"] == t.tiles * nin * (k2 - 1)
        shape = (L.c_o, L.c_i, L.k, L.k, t.tile_h, t.tile_w)
        b, O = (li * 7) % t.tiles, (li * 5) % nout
        want = oracle_block(o, shape, K, cts[b], r_tiles[b], li, b, O, osk)
        assert np.array_equal(got[b, O], want), f"{L.name}: ciphertext mismatch at tile {b}, block {O}"
        if L.k == 1:
            share = Hn.stitch_layer_share(ctx, sk, t, plan, got, L.c_o)
            assert np.array_equal((share + r) % np.uint64(par.p), strided_conv(K, image, par.p, L.stride)), L.name
        del plan
    # the final FC 512 -> 1000
    W, x, r = wl.fc_inputs(fc, seed=77)
    plan = ctx.fc_plan(W)
    gk = ctx.galois_keygen(sk, plan.rotations(), seed=1)
    plan.bind(gk)
    ct = ctx.encrypt(sk, plan.pack_input(x[0]), seed=0)[None, :]
    got, cnt = Hn.gpu_he_fc(ctx, plan, ct, r, mask_seed=99)
    assert plan.G == 256 and cnt["perm"] == 255
    want, _ = o.he_fc(o.fc_encode_rowwise(W), ct[0], o.fc_keys(osk, fc.n_o, fc.n_i, seed=1),
                      o.fc_mask_slots(fc.n_o, fc.n_i, r[0], 99, 0))
    assert np.array_equal(got[0], want)
    share = plan.unpack_share(ctx.decrypt(sk, got[0]))
    assert np.array_equal((share + r[0]) % np.uint64(par.p), (W @ x[0]) % np.uint64(par.p))
    print("ResNet-18 conv op totals:", total, flush=True)
