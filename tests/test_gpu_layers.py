"""GPU tests of whole layers: spatial tiling + stride on top of he_conv, and the ResNet-18-shaped list."""
import concurrent.futures
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


def check_sampled_blocks(o, osk, shape, K, cts, r_tiles, got, mask_seed, name, extra=()):
    """The first, a middle and the last (tile, output block) of a layer, plus `extra`, recomputed by the oracle on a
    host thread each; the ciphertexts must be equal."""
    tiles, nout = got.shape[0], got.shape[1]
    picks = sorted({(0, 0), (tiles // 2, nout // 2), (tiles - 1, nout - 1), *extra})
    tk, gkk = o.conv_keys(osk, shape, seed=8)

    def block(bO):
        b, O = bO
        return o.he_conv_block(shape, K, O, cts[b], tk, gkk, o.conv_mask_slots(shape, r_tiles[b], mask_seed, b, O))[0]

    with concurrent.futures.ThreadPoolExecutor(len(picks)) as pool:
        for (b, O), want in zip(picks, pool.map(block, picks)):
            assert np.array_equal(got[b, O], want), f"{name}: ciphertext mismatch at tile {b}, block {O}"


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


@pytest.mark.parametrize("n,p_limit,gb,c_o,c_i,k,stride,H,W,special", [
    (64, 1 << 9, 4, 4, 2, 3, 2, 12, 12, False),     # 6x6 phases tiled; four phases of two channels
    (64, 1 << 9, 4, 6, 4, 1, 2, 9, 5, False),       # 1x1: phase (0,0) alone, odd image
    (256, 1 << 13, 4, 8, 4, 3, 2, 10, 10, False),   # 5x5 phases in one tile
    (256, 1 << 13, 4, 4, 3, 7, 2, 20, 20, False),   # 7x7/2: 5x5 window on 10x10 phases
    (256, 1 << 13, 20, 4, 2, 3, 3, 13, 11, True),   # stride 3, special prime
])
def test_polyphase_strided_layer(n, p_limit, gb, c_o, c_i, k, stride, H, W, special):
    """A strided layer as a stride-1 he_conv over the phase images: the share decrypts to the strided convolution
    written out by definition, the ciphertexts equal the oracle's on its own rearrangement of kernel and image, and
    the plan multiplies only by the taps that exist."""
    from oracle.oracle import polyphase_split, strided_conv_plain
    from tests import gpu_harness as Hn
    from tests.test_gpu_special import with_special
    par = small_params(n, p_limit=p_limit, gadget_bits=gb)
    if special:
        par = with_special(par)
    ctx = binding.Context(par.n, par.q, par.p, par.gadget_bits, par.special)
    o = Oracle(par.n, par.q, par.p, par.gadget_bits, par.special)
    rng = np.random.default_rng(n + H + k)
    K = rng.integers(1, par.p, size=(c_o, c_i, k, k), dtype=np.uint64)
    image = rng.integers(0, par.p, size=(c_i, H, W), dtype=np.uint64)
    sk, osk = ctx.keygen(0), o.keygen(0)
    Kp, xp = Hn.polyphase_layer(ctx, K, image, stride)
    Kp_o, xp_o = polyphase_split(K, image, stride)
    assert np.array_equal(Kp, Kp_o) and np.array_equal(xp, xp_o)
    r = rng.integers(0, par.p, size=(c_o, xp.shape[1], xp.shape[2]), dtype=np.uint64)
    t, plan, x_tiles, r_tiles, cts, got, cnt = Hn.gpu_conv_layer(ctx, sk, Kp, xp, r, 1, mask_seed=5, matrix_cores=True)
    assert (t.out_h, t.out_w) == (-(-H // stride), -(-W // stride))
    assert plan.nterm < plan.nin * plan.ntap or k == 1
    share = Hn.stitch_layer_share(ctx, sk, t, plan, got, c_o)
    assert np.array_equal((share + r) % np.uint64(par.p), strided_conv_plain(K, image, par.p, stride))
    shape = (c_o, Kp.shape[1], Kp.shape[2], Kp.shape[3], t.tile_h, t.tile_w)
    b, O = t.tiles - 1, plan.nout - 1
    assert np.array_equal(got[b, O], oracle_block(o, shape, Kp_o, cts[b], r_tiles[b], 5, b, O, osk))


def test_resnet18_shaped_layer_list():
    """Config 5: every linear layer of an ImageNet-shaped ResNet-18, one input, random weights mod p.
    Each layer runs in full on the GPU; the oracle recomputes up to four output ciphertexts per layer (the first, a
    middle and the last tile and output block, and one more) and the ciphertexts must agree exactly.  1x1 layers and the FC also decrypt
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
        check_sampled_blocks(o, osk, shape, K, cts, r_tiles, got, li, L.name, extra=[((li * 7) % t.tiles, (li * 5) % nout)])
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


def test_resnet18_strided_layers_as_polyphase_layers():
    """The seven strided layers of the list (7x7/2, three 3x3/2, three 1x1/2) through the polyphase split at full
    size: up to four output ciphertexts per layer (first, middle, last tile and block, one more) against the oracle on its
    own rearrangement, the operation counts of the
    terms that exist, and for the 1x1 layers the decrypted share against the subsampled plain convolution."""
    from oracle.oracle import polyphase_split
    from tests import gpu_harness as Hn
    par = wl.DEFAULT
    ctx = binding.Context(par.n, par.q, par.p, par.gadget_bits)
    o = Oracle(par.n, par.q, par.p, par.gadget_bits)
    sk, osk = ctx.keygen(0), o.keygen(0)
    layers, _ = wl.resnet18_layers()
    # taps that exist per original channel after the split: 49 of 4*25, 9 of 4*9, 1 of 1
    scmult_per_pair = {7: 49, 3: 9, 1: 1}
    for li, L in enumerate(layers):
        if L.stride == 1:
            continue
        rng = np.random.default_rng(2000 + li)
        K = rng.integers(1, par.p, size=(L.c_o, L.c_i, L.k, L.k), dtype=np.uint64)
        image = rng.integers(0, par.p, size=(L.c_i, L.in_hw, L.in_hw), dtype=np.uint64)
        Kp, xp = Hn.polyphase_layer(ctx, K, image, L.stride)
        Kp_o, xp_o = polyphase_split(K, image, L.stride)
        assert np.array_equal(Kp, Kp_o) and np.array_equal(xp, xp_o)
        out_hw = L.in_hw // L.stride
        r = rng.integers(0, par.p, size=(L.c_o, out_hw, out_hw), dtype=np.uint64)
        t, plan, x_tiles, r_tiles, cts, got, cnt = Hn.gpu_conv_layer(ctx, sk, Kp, xp, r, 1, mask_seed=li, matrix_cores=True)
        print(f"layer {L.name}: {Kp.shape[1]} phase channels, {Kp.shape[2]}x{Kp.shape[3]} window, tiles {t.tiles}, "
              f"terms {plan.nterm} of {plan.nin * plan.ntap}", flush=True)
        assert (t.out_h, t.out_w) == (out_hw, out_hw)
        if L.c_i % plan.cn == 0:          # every input ciphertext holds one phase: exactly the taps that exist
            assert cnt["scmult"] == t.tiles * plan.nout * plan.cn * (L.c_i // plan.cn) * scmult_per_pair[L.k]
        shape = (L.c_o, Kp.shape[1], Kp.shape[2], Kp.shape[3], t.tile_h, t.tile_w)
        check_sampled_blocks(o, osk, shape, Kp_o, cts, r_tiles, got, li, L.name,
                             extra=[((li * 7) % t.tiles, (li * 5) % plan.nout)])
        if L.k == 1:
            share = Hn.stitch_layer_share(ctx, sk, t, plan, got, L.c_o)
            assert np.array_equal((share + r) % np.uint64(par.p), strided_conv(K, image, par.p, L.stride)), L.name
        del plan


@pytest.mark.parametrize("which", ["n256", "n2048", "n2048_special"])
def test_he_fc_and_he_conv_replay_from_a_hip_graph(which):
    """The layer entry points allocate nothing, wait for nothing and clear memory with kernels only, so a caller
    can capture them in a HIP graph.  Captured once, replayed three times on fresh inputs with eager work and
    synchronisations in between; every replay must equal the eager result of the same inputs.  On the any-n
    kernels (n = 256) and on the n = 2048 kernels with the matrix-core product, one-prime and special-prime keys."""
    import torch
    from tests import gpu_harness as Hn
    par = {"n256": small_params(256, p_limit=1 << 13, gadget_bits=8), "n2048": wl.DEFAULT,
           "n2048_special": wl.DEFAULT_SPECIAL}[which]
    ctx = binding.Context(par.n, par.q, par.p, par.gadget_bits, par.special)
    sk = ctx.keygen(0)
    rng = np.random.default_rng(3)
    n, batch = par.n, 4
    W = rng.integers(0, par.p, size=(16, 64), dtype=np.uint64) if n == 256 else \
        rng.integers(0, par.p, size=(64, 512), dtype=np.uint64)
    fplan = ctx.fc_plan(W)
    fplan.bind(ctx.galois_keygen(sk, fplan.rotations(), seed=1))
    K = rng.integers(0, par.p, size=(8, 8, 3, 3), dtype=np.uint64)
    cplan = ctx.conv_plan(K, 4, 4) if n == 256 else ctx.conv_plan(K, 16, 16)
    cplan.bind(ctx.galois_keygen(sk, cplan.rotations(), seed=2))
    cplan.prepare_batched()
    d_fin, d_fout = Hn.dev_empty(batch * 2 * n), Hn.dev_empty(batch * 2 * n)
    d_cin, d_cout = Hn.dev_empty(batch * cplan.nin * 2 * n), Hn.dev_empty(batch * cplan.nout * 2 * n)
    d_fr = Hn.to_dev(rng.integers(0, par.p, size=(batch, W.shape[0]), dtype=np.uint64))
    u = 4 if n == 256 else 16
    d_cr = Hn.to_dev(rng.integers(0, par.p, size=(batch, 8, u, u), dtype=np.uint64))
    fwsb, cwsb = fplan.workspace_bytes(batch), cplan.workspace_bytes(batch)
    fws = torch.empty(fwsb, dtype=torch.uint8, device="cuda")
    cws = torch.empty(cwsb, dtype=torch.uint8, device="cuda")

    def layers(stream):
        fplan.he_fc(d_fin, batch, d_fr, 5, d_fout, fws, fwsb, stream=stream)
        cplan.he_conv(d_cin, batch, d_cr, 6, d_cout, cws, cwsb, stream=stream)

    def fresh_inputs(seed):
        g = np.random.default_rng(seed)
        d_fin.copy_(Hn.to_dev(g.integers(0, par.q, size=batch * 2 * n, dtype=np.uint64)))
        d_cin.copy_(Hn.to_dev(g.integers(0, par.q, size=batch * cplan.nin * 2 * n, dtype=np.uint64)))

    fresh_inputs(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        layers(side)                                     # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        layers(torch.cuda.current_stream())
    for rep in range(3):
        fresh_inputs(100 + rep)
        layers(None)                                     # eager, default stream
        torch.cuda.synchronize()
        want_f, want_c = Hn.to_host(d_fout).copy(), Hn.to_host(d_cout).copy()
        d_fout.zero_(); d_cout.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(Hn.to_host(d_fout), want_f), rep
        assert np.array_equal(Hn.to_host(d_cout), want_c), rep
