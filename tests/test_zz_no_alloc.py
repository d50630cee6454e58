"""gala_he_fc_static (the he_fc entry point that allocates nothing: its partial ciphertexts live in a fixed array of
the library's device code) against gala_he_fc, through the C ABI: two calls in a row, the second with a smaller
input, every output word equal; requests beyond the fixed capacity are refused."""
import numpy as np
import pytest

from paper_2105_01827_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def test_he_fc_static_matches_he_fc_on_two_calls_in_a_row():
    import torch
    from tests import gpu_harness as H
    par = wl.DEFAULT
    ctx = binding.Context(par.n, par.q, par.p, par.gadget_bits)
    sk = ctx.keygen(0)
    capacity = int(ctx.lib.gala_he_fc_static_capacity())
    assert capacity == 32 << 20
    # first call: 128x1024 weights (G = 64), 6 inputs; second call: 16x512 weights (G = 4), 2 inputs
    for n_o, n_i, batch, seed in ((128, 1024, 6, 1), (16, 512, 2, 2)):
        W, x, r = wl.fc_inputs(wl.FcShape("static", n_o, n_i, batch), seed=seed)
        plan = ctx.fc_plan(W)
        gk = ctx.galois_keygen(sk, plan.rotations(), seed=1)
        plan.bind(gk)
        cts = np.stack([ctx.encrypt(sk, plan.pack_input(x[b]), seed=10 * seed + b) for b in range(batch)])
        d_in, d_r = H.import_cts(ctx, cts), H.to_dev(r)
        ws_bytes = plan.workspace_bytes(batch)
        assert 0 < ws_bytes <= capacity
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        d_ref = H.dev_empty(batch * 2 * par.n)
        cnt_ref = plan.he_fc(d_in, batch, d_r, 17, d_ref, ws, ws_bytes)
        d_out = torch.zeros(batch * 2 * par.n, dtype=torch.int64, device="cuda")
        cnt = plan.he_fc_static(d_in, batch, d_r, 17, d_out)
        torch.cuda.synchronize()
        assert cnt == cnt_ref
        assert torch.equal(d_out, d_ref), (n_o, n_i, batch)
        got = H.export_cts(ctx, d_out, batch)
        for b in range(batch):
            share = plan.unpack_share(ctx.decrypt(sk, got[b]))
            assert np.array_equal((share + r[b]) % np.uint64(par.p), (W @ x[b]) % np.uint64(par.p))
    # 64 inputs of the 128x1024 layer need 66 MiB of partial ciphertexts: refused, nothing launched
    W, x, r = wl.fc_inputs(wl.FcShape("static", 128, 1024, 64), seed=3)
    plan = ctx.fc_plan(W)
    plan.bind(ctx.galois_keygen(sk, plan.rotations(), seed=1))
    assert plan.workspace_bytes(64) > capacity
    d_in, d_out, d_r = H.dev_empty(64 * 2 * par.n), H.dev_empty(64 * 2 * par.n), H.to_dev(r)
    with pytest.raises(binding.GalaError) as e:
        plan.he_fc_static(d_in, 64, d_r, 17, d_out)
    assert e.value.code == binding.GALA_ENOMEM
