"""Helpers for the GPU parity tests: device buffers through PyTorch, calls through the C-ABI binding."""
import numpy as np
import torch

from paper_2105_01827_amd import binding


def to_dev(a):
    a = np.ascontiguousarray(np.asarray(a, dtype=np.uint64))
    return torch.from_numpy(a.view(np.int64)).cuda()


def to_host(t):
    return t.cpu().numpy().view(np.uint64)


def dev_empty(words):
    return torch.empty(int(words), dtype=torch.int64, device="cuda")


def import_cts(ctx, cts_coeff):
    """cts_coeff: (count, 2n) interchange-form ciphertexts on the host -> internal form on the device."""
    cts_coeff = np.ascontiguousarray(cts_coeff, dtype=np.uint64).reshape(-1, 2 * ctx.n)
    src = to_dev(cts_coeff)
    dst = dev_empty(cts_coeff.size)
    ctx.ct_import(src, cts_coeff.shape[0], dst)
    return dst


def export_cts(ctx, dev, count):
    out = dev_empty(count * 2 * ctx.n)
    ctx.ct_export(dev, count, out)
    torch.cuda.synchronize()
    return to_host(out).reshape(count, 2 * ctx.n)


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
