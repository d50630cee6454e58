"""Device buffers for callers of the binding: PyTorch supplies the memory, the library does the work.

Words are uint64 on the host and int64 tensors on the device (PyTorch has no unsigned 64-bit arithmetic; the
library only takes the pointer)."""
import numpy as np
import torch


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
    """Internal-form ciphertexts on the device -> (count, 2n) interchange form on the host (waits for the device)."""
    out = dev_empty(count * 2 * ctx.n)
    ctx.ct_export(dev, count, out)
    torch.cuda.synchronize()
    return to_host(out).reshape(count, 2 * ctx.n)
