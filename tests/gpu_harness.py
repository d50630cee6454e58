"""Helpers for the GPU parity tests: device buffers through PyTorch, calls through the C-ABI binding."""
import numpy as np
import torch

from paper_2105_01827_amd import binding  # noqa: F401
from paper_2105_01827_amd.devmem import dev_empty, export_cts, import_cts, to_dev, to_host  # noqa: F401


def gpu_he_fc(ctx, plan, cts_coeff, r, mask_seed):
    """Whole he_fc through the library; returns interchange-form outputs (batch, 2n) and the op counts."""
    batch = cts_coeff.shape[0]
    d_in = import_cts(ctx, cts_coeff)
    d_out = dev_empty(batch * 2 * ctx.n)
    d_r = to_dev(r)
    ws_bytes = plan.workspace_bytes(batch)
    ws = torch.empty(max(ws_bytes, 8), dtype=torch.uint8, device="cuda")
    cnt = plan.he_fc(d_in, batch, d_r, mask_seed, d_out, ws, ws_bytes)
    return export_cts(ctx, d_out, batch), cnt


def gpu_he_conv(ctx, plan, cts_coeff, r, mask_seed):
    """cts_coeff: (batch, nin, 2n); r: (batch, c_o, u_h, u_w).  Returns (batch, nout, 2n) and counts."""
    batch = cts_coeff.shape[0]
    d_in = import_cts(ctx, cts_coeff.reshape(-1, 2 * ctx.n))
    d_out = dev_empty(batch * plan.nout * 2 * ctx.n)
    d_r = to_dev(r)
    ws_bytes = plan.workspace_bytes(batch)
    ws = torch.empty(max(ws_bytes, 8), dtype=torch.uint8, device="cuda")
    cnt = plan.he_conv(d_in, batch, d_r, mask_seed, d_out, ws, ws_bytes)
    return export_cts(ctx, d_out, batch * plan.nout).reshape(batch, plan.nout, 2 * ctx.n), cnt


def polyphase_layer(ctx, K, image, stride):
    """(K_poly, image_poly) of the library: the stride-1 layer that computes the strided one."""
    c_o, c_i, k_h, k_w = K.shape
    pp = ctx.conv_polyphase(c_i, image.shape[1], image.shape[2], k_h, k_w, stride)
    return ctx.polyphase_kernel(pp, K), ctx.polyphase_input(pp, image)


def gpu_conv_layer(ctx, sk, K, image, r_layer, stride, mask_seed, key_seed=8, enc_seed=0, matrix_cores=False):
    """A whole convolution layer on one image (c_i x H x W) through the library: spatial tiling, stride,
    he_conv over the tiles.  Returns (tiling, plan, tile inputs, tile masks, input cts, output cts, counts)."""
    c_o, c_i, k_h, k_w = K.shape
    _, H, W = image.shape
    t = ctx.conv_tiling(H, W, k_h, k_w, stride)
    plan = ctx.conv_plan(K, t.tile_h, t.tile_w)
    gk = ctx.galois_keygen(sk, plan.rotations(), seed=key_seed)
    plan.bind(gk)
    tiles = t.tiles
    if matrix_cores and tiles >= 2:
        plan.prepare_batched()
    x_tiles = np.stack([ctx.tile_extract(t, image, b) for b in range(tiles)])
    r_tiles = np.stack([ctx.tile_mask(t, r_layer, b) for b in range(tiles)])
    slots = np.stack([plan.pack_input(x_tiles[b]) for b in range(tiles)])          # (tiles, nin, n)
    cts = np.stack([[ctx.encrypt(sk, slots[b, I], seed=enc_seed + 1000 * b + I) for I in range(plan.nin)]
                    for b in range(tiles)])
    got, cnt = gpu_he_conv(ctx, plan, cts, r_tiles, mask_seed)
    return t, plan, x_tiles, r_tiles, cts, got, cnt


def stitch_layer_share(ctx, sk, t, plan, got, c_o):
    """Client side: decrypt every tile's outputs, unpack, keep the outputs each tile is responsible for."""
    share = np.zeros((c_o, t.out_h, t.out_w), np.uint64)
    for b in range(t.tiles):
        tile_vals = np.zeros((c_o, t.tile_h, t.tile_w), np.uint64)
        for O in range(plan.nout):
            plan.unpack_share(O, ctx.decrypt(sk, got[b, O]), tile_vals)
        ctx.tile_scatter(t, tile_vals, b, share)
    return share
