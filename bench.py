#!/usr/bin/env python3
"""Benchmark of the GALA linear-layer hot path on one MI355X.

A "step" is one he_fc call over the whole batch of the workload (ScMult, Perm,
Add and share generation for every input), with ciphertexts, encoded weights
and Galois keys already resident on the device in internal form.  The reported
value is homomorphic rotations (Perm) per second inside that layer; layers/s
and inputs/s are given beside it.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Integer-ALU roofline: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz 32-bit integer lane-operations per second.
# The instructions the modular arithmetic is made of (v_mad_u64_u32, v_mul_lo_u32, 32-bit adds) were all
# measured at 0.93-0.96 of this rate with csrc/probe_int_mul.hip, so multiplies and adds are priced alike.
ALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12

# 32-bit integer operations of the leanest formulation known here of each 64-bit modular primitive
# (multiply-adds, adds with carry, selects; no address arithmetic, no register moves):
OPS_CONST_MUL = 13      # y*w mod q, w with precomputed quotient: 6 for the high product, 6 + 1 for y*w - h*q
OPS_CSUB = 4            # conditional subtraction: sub, subb, two selects on the borrow
OPS_BF_FWD = OPS_CONST_MUL + 1 + 3             # lazy forward butterfly: x + v, x + 2q - v
OPS_BF_INV = OPS_CONST_MUL + 1 + 3 + OPS_CSUB  # inverse butterfly: x + y reduced, (x - y + 2q) * w


def ops_per_fused_perm(n, logn, ndigits):
    """Algorithmic integer operations of one ScMult + Perm + Add on one ciphertext (one 'fused unit')."""
    half = n // 2
    inverse = half * (logn - 1) * OPS_BF_INV + half * (2 * OPS_CONST_MUL + 2 * OPS_CSUB + 4)   # n^-1 folded in
    forward = half * logn * OPS_BF_FWD + n * OPS_CSUB           # one conditional subtraction per coefficient
    scmult_c1 = n * OPS_CONST_MUL                               # c1 (.) w before the inverse transform
    c0_term = n * (OPS_CONST_MUL + 1)                           # permuted c0 (.) w added to the sum
    digits = ndigits * n * 2                                    # shift and mask
    key_mac = 2 * ndigits * n * (OPS_CONST_MUL + 1)             # inner product with (b_j, a_j)
    accumulate = 2 * n * OPS_CSUB                               # keep the running sums below 8q
    return inverse + ndigits * forward + scmult_c1 + c0_term + digits + key_mac + accumulate


def ops_per_fused_perm_special(n, logn, ndigits):
    """The same unit with special-prime key switching: every digit is transformed and multiplied in both moduli,
    the two sums modulo P go back to coefficients (two inverse transforms); the two forward transforms of the
    summed remainders happen once per workgroup and are not counted."""
    half = n // 2
    inverse = half * (logn - 1) * OPS_BF_INV + half * (2 * OPS_CONST_MUL + 2 * OPS_CSUB + 4)
    forward = half * logn * OPS_BF_FWD + n * OPS_CSUB
    scmult_c1 = n * OPS_CONST_MUL
    c0_term = n * (2 * OPS_CONST_MUL + 1)                       # permuted c0 (.) w, times P
    digits = 2 * ndigits * n * 2
    key_mac = 4 * ndigits * n * (OPS_CONST_MUL + 1)             # (b_j, a_j) modulo q and modulo P
    accumulate = 2 * n * OPS_CSUB
    remainders = 2 * n * (OPS_CONST_MUL + OPS_CSUB + 2 * OPS_CSUB + 1)   # canonical mod P, lift, reduce mod q, add
    return 3 * inverse + 2 * ndigits * forward + scmult_c1 + c0_term + digits + key_mac + accumulate + remainders


def timed(fn, torch, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def secondary_workloads(ctx, sk, H, torch):
    """Short runs of the other entry points at n = 2048 (same context and keys' secret): plain Perm on a batch of
    ciphertexts, the 16x16x128 / 3x3x128 convolution of batch 16, and the 1000x2048 FC of batch 64."""
    from paper_2105_01827_amd import workloads as wl
    par, res = wl.DEFAULT, {}
    rng = np.random.default_rng(0)
    # gala_rotate: 4096 ciphertexts, one rotation
    count = 4096
    gk = ctx.galois_keygen(sk, [(0, 1)], seed=3)
    d_in = H.to_dev(rng.integers(0, par.q, size=(count, 2 * par.n), dtype=np.uint64))
    d_out = H.dev_empty(count * 2 * par.n)
    t = timed(lambda: ctx.rotate(gk, d_in, count, (0, 1), d_out), torch, 100, 20)
    res["rotate_4096_cts"] = {"ms": t * 1e3, "rotations_per_s": count / t}
    del d_in, d_out
    # gala_rotate_hoisted: 512 ciphertexts x 8 rotations each, one DecPerm per ciphertext (HstPerm-dominated)
    hc, hr = 512, 8
    gk8 = ctx.galois_keygen(sk, [(0, 1 + k) for k in range(hr)], seed=4)
    d_in = H.to_dev(rng.integers(0, par.q, size=(hc, 2 * par.n), dtype=np.uint64))
    d_out = H.dev_empty(hc * hr * 2 * par.n)
    hwsb = ctx.rotate_hoisted_workspace(hc)
    hws = torch.empty(hwsb, dtype=torch.uint8, device="cuda")
    t = timed(lambda: ctx.rotate_hoisted(gk8, d_in, hc, d_out, hws, hwsb), torch, 100, 20)
    res["rotate_hoisted_512_cts_x8"] = {"ms": t * 1e3, "rotations_per_s": hc * hr / t}
    del d_in, d_out, hws, gk8
    # the client's steps on the device: 4096 encryptions and decryptions (internal ciphertext form)
    d_slots = H.to_dev(rng.integers(0, par.p, size=(count, par.n), dtype=np.uint64))
    d_seeds = H.to_dev(np.arange(count, dtype=np.uint64))
    d_ct = H.dev_empty(count * 2 * par.n)
    t = timed(lambda: ctx.encrypt_batch(sk, d_slots, d_seeds, count, d_ct), torch, 30, 5)
    res["encrypt_4096_cts"] = {"ms": t * 1e3, "ciphertexts_per_s": count / t}
    t = timed(lambda: ctx.decrypt_batch(sk, d_ct, count, d_slots), torch, 30, 5)
    res["decrypt_4096_cts"] = {"ms": t * 1e3, "ciphertexts_per_s": count / t}
    del d_slots, d_ct
    # he_fc 16x128, one input (a single ScMult and the mask, no rotation): launch latency
    f = wl.FC_16x128
    W, x, r = wl.fc_inputs(f)
    plan = ctx.fc_plan(W)
    d_in = H.to_dev(rng.integers(0, par.q, size=(f.batch, 2 * par.n), dtype=np.uint64))
    d_out = H.dev_empty(f.batch * 2 * par.n)
    d_r = H.to_dev(r)
    wsb = plan.workspace_bytes(f.batch)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    t = timed(lambda: plan.he_fc(d_in, f.batch, d_r, 5, d_out, ws, wsb), torch, 200, 20)
    res[f.name] = {"ms_per_layer": t * 1e3, "layers_per_s": 1 / t, "inputs_per_s": f.batch / t, "rotations_per_s": 0.0}
    del plan, d_in, d_out, ws
    # he_conv, 16x16x128 input, 128 kernels of 3x3, batch 16
    s = wl.CONV_16x16_128_3x3
    K, x, r = wl.conv_inputs(s)
    plan = ctx.conv_plan(K, s.u_h, s.u_w)
    gkc = ctx.galois_keygen(sk, plan.rotations(), seed=8)
    plan.bind(gkc)
    plan.prepare_batched()
    d_in = H.to_dev(rng.integers(0, par.q, size=(s.batch * plan.nin, 2 * par.n), dtype=np.uint64))
    d_out = H.dev_empty(s.batch * plan.nout * 2 * par.n)
    d_r = H.to_dev(r)
    wsb = plan.workspace_bytes(s.batch)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    cnt = {}
    def conv():
        cnt.update(plan.he_conv(d_in, s.batch, d_r, 3, d_out, ws, wsb))
    t = timed(conv, torch, 100, 20)
    res[s.name] = {"ms_per_layer": t * 1e3, "layers_per_s": 1 / t, "inputs_per_s": s.batch / t,
                   "rotations_per_s": (cnt["perm"] + cnt["hstperm_in"]) / t, "ops_per_layer": dict(cnt)}
    del plan, d_in, d_out, ws
    # he_fc 1000x2048, batch 64 (1023 rotations per input)
    f = wl.FC_1000x2048
    W, x, r = wl.fc_inputs(f)
    plan = ctx.fc_plan(W)
    gkf = ctx.galois_keygen(sk, plan.rotations(), seed=1)
    plan.bind(gkf)
    d_in = H.to_dev(rng.integers(0, par.q, size=(f.batch, 2 * par.n), dtype=np.uint64))
    d_out = H.dev_empty(f.batch * 2 * par.n)
    d_r = H.to_dev(r)
    wsb = plan.workspace_bytes(f.batch)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    def fc():
        cnt.update(plan.he_fc(d_in, f.batch, d_r, 5, d_out, ws, wsb))
    t = timed(fc, torch, 30, 5)
    res[f.name] = {"ms_per_layer": t * 1e3, "layers_per_s": 1 / t, "inputs_per_s": f.batch / t,
                   "rotations_per_s": cnt["perm"] / t}
    return res


HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published
OPS_MAC128 = 10         # 64x64 product added into a 128-bit sum: 4 multiply-adds and 6 carry additions
OPS_REDUCE128 = 2 * OPS_CONST_MUL + 2 * OPS_CSUB + 1


def resnet18_workload(ctx, sk, H, torch, args):
    """Config 5: every linear layer of an ImageNet-shaped ResNet-18 on one input (random weights and ciphertexts):
    20 convolutions over their spatial tiles (the tiles are the batch of he_conv) and the final FC.  Each layer
    is timed on its own with its plan, keys and inputs resident; a 'step' is one pass over all 21 layers."""
    from paper_2105_01827_amd import workloads as wl
    par = wl.DEFAULT
    rng = np.random.default_rng(0)
    layers, fc = wl.resnet18_layers()
    per_layer, total_ms, total = [], 0.0, dict(perm=0, decperm_in=0, hstperm_in=0, scmult=0, add=0)
    weight_bytes, mac_ms = 0.0, 0.0
    steps, warm = max(3, args.steps // 50), max(1, args.warmup // 50)
    ctx.profile_select(1)
    for L in layers:
        K = rng.integers(0, par.p, size=(L.c_o, L.c_i, L.k, L.k), dtype=np.uint64)
        if L.stride > 1 and not args.stride_by_subsampling:
            # stride as a stride-1 layer over the phase images: only the outputs that are kept get computed
            pp = ctx.conv_polyphase(L.c_i, L.in_hw, L.in_hw, L.k, L.k, L.stride)
            K = ctx.polyphase_kernel(pp, K)
            t = ctx.conv_tiling(pp.out_h, pp.out_w, pp.k_h_poly, pp.k_w_poly, 1)
        else:
            t = ctx.conv_tiling(L.in_hw, L.in_hw, L.k, L.k, L.stride)
        plan = ctx.conv_plan(K, t.tile_h, t.tile_w)
        gk = ctx.galois_keygen(sk, plan.rotations(), seed=8)
        plan.bind(gk)
        if t.tiles >= 2:
            plan.prepare_batched()
        d_in = H.to_dev(rng.integers(0, par.q, size=(t.tiles * plan.nin, 2 * par.n), dtype=np.uint64))
        d_out = H.dev_empty(t.tiles * plan.nout * 2 * par.n)
        d_r = H.to_dev(rng.integers(0, par.p, size=(t.tiles, L.c_o, t.tile_h, t.tile_w), dtype=np.uint64))
        wsb = plan.workspace_bytes(t.tiles)
        ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
        cnt = {}
        def conv():
            cnt.update(plan.he_conv(d_in, t.tiles, d_r, 3, d_out, ws, wsb))
        for _ in range(warm):
            conv()
        torch.cuda.synchronize()
        ctx.profile_enable(steps)
        dt = timed(conv, torch, steps, 0)
        kms = ctx.profile_collect(steps)
        ctx.profile_enable(0)
        groups, nterm = plan.nout * plan.cn, plan.nterm
        weight_bytes += 8.0 * par.n * groups * nterm
        mac_ms += float(np.mean(kms)) if kms else 0.0
        per_layer.append({"layer": L.name, "tiles": t.tiles, "c_n": plan.cn, "terms": nterm, "ms": dt * 1e3,
                          "multiply_accumulate_ms": float(np.mean(kms)) if kms else None})
        total_ms += dt * 1e3
        for k in total:
            total[k] += cnt[k]
        del plan, gk, d_in, d_out, ws
    ctx.profile_select(0)
    W, x, r = wl.fc_inputs(fc, seed=77)
    plan = ctx.fc_plan(W)
    gk = ctx.galois_keygen(sk, plan.rotations(), seed=1)
    plan.bind(gk)
    d_in = H.to_dev(rng.integers(0, par.q, size=(1, 2 * par.n), dtype=np.uint64))
    d_out = H.dev_empty(2 * par.n)
    d_r = H.to_dev(r)
    wsb = plan.workspace_bytes(1)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    cnt = {}
    def fcl():
        cnt.update(plan.he_fc(d_in, 1, d_r, 5, d_out, ws, wsb))
    dt = timed(fcl, torch, steps, warm)
    per_layer.append({"layer": fc.name, "G": plan.G, "ms": dt * 1e3})
    total_ms += dt * 1e3
    for k in total:
        total[k] += cnt[k]
    return per_layer, total_ms, total, weight_bytes, mac_ms, steps, warm


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="fc_128x1024_b64",
                    choices=["fc_128x1024_b64", "fc_1000x2048_b64", "conv_16x16x128_3x3x128_b16", "resnet18_b1"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--vector-mac", action="store_true",
                    help="convolution: keep the multiply-accumulate on the vector ALU instead of the matrix cores")
    ap.add_argument("--special-prime", action="store_true",
                    help="key switching with the special prime (keys modulo q*P, exact division by P): the mode in "
                         "which 3x3 convolutions decrypt at the 20-bit plaintext modulus")
    ap.add_argument("--stride-by-subsampling", action="store_true",
                    help="resnet18_b1: evaluate strided layers at stride 1 and drop outputs instead of the polyphase split")
    ap.add_argument("--no-secondary", action="store_true", help="skip the short runs of the other workloads")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run one plain device copy of this size (calibrates rocprofv3 HBM byte counters)")
    ap.add_argument("--cpu-sample", type=int, default=64, help="inputs the oracle is timed on (FC workloads)")
    ap.add_argument("--cpu-repeat", type=int, default=3, help="passes of the oracle over the sample")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2105_01827_amd import binding, workloads as wl
    from tests import gpu_harness as H

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    par = wl.DEFAULT_SPECIAL if args.special_prime else wl.DEFAULT
    ctx = binding.Context(par.n, par.q, par.p, par.gadget_bits, par.special)
    sk = ctx.keygen(0)
    stream = torch.cuda.current_stream()
    if args.workload == "resnet18_b1":
        per_layer, total_ms, total, weight_bytes, mac_ms, steps, warm = resnet18_workload(ctx, sk, H, torch, args)
        rot = total["perm"] + total["hstperm_in"]
        gbs = weight_bytes / (mac_ms * 1e-3) / 1e9
        print(json.dumps({
            "metric": "HE rotations/sec and he_fc/he_conv layers/sec at n=2048; % of HBM/int roofline",
            "value": rot / (total_ms * 1e-3), "unit": "rotations/s", "n_gpus": 1, "steps": steps, "warmup": warm,
            "ms_per_step": total_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64",
            "data": "synthetic",
            "config": {"workload": "resnet18_b1", "layers": len(per_layer), "n": par.n, "batch": 1,
                       "stride": "subsampling" if args.stride_by_subsampling else "polyphase",
                       "note": "each layer timed on its own; a step is one pass over the 21 linear layers"},
            "layers_per_s": len(per_layer) * 1e3 / total_ms, "networks_per_s": 1e3 / total_ms, "ops_per_step": total,
            "per_layer": per_layer,
            # at one input the multiply-accumulate streams every encoded kernel polynomial once: HBM-bound
            "roofline": {"bound": "hbm", "kernel": "conv_mac_kernel / conv_mfma_kernel (all 20 convolutions)",
                         "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                         "traffic": None, "kernel_ms_total": mac_ms, "bytes_per_step": weight_bytes},
            "cpu_baseline": None}))
        return
    is_conv = args.workload.startswith("conv")
    if is_conv:
        shape = wl.CONV_16x16_128_3x3
        K, x, r = wl.conv_inputs(shape)
        plan = ctx.conv_plan(K, shape.u_h, shape.u_w)
        gk = ctx.galois_keygen(sk, plan.rotations(), seed=8)
        plan.bind(gk)
        if not args.vector_mac:
            plan.prepare_batched()      # multiply-accumulate on the matrix cores
        batch = shape.batch
        slots = np.stack([plan.pack_input(x[b]) for b in range(batch)])
        cts = np.stack([[ctx.encrypt(sk, slots[b, I], seed=1000 * b + I) for I in range(plan.nin)] for b in range(batch)])
        d_in = H.import_cts(ctx, cts.reshape(-1, 2 * par.n))
        d_out = H.dev_empty(batch * plan.nout * 2 * par.n)
        d_r = H.to_dev(r)
        ws_bytes = plan.workspace_bytes(batch)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        ctx.profile_select(1)

        def step():
            return plan.he_conv(d_in, batch, d_r, 3, d_out, ws, ws_bytes, stream=stream)
    else:
        shape = {"fc_128x1024_b64": wl.FC_128x1024, "fc_1000x2048_b64": wl.FC_1000x2048}[args.workload]
        W, x, r = wl.fc_inputs(shape)
        plan = ctx.fc_plan(W)
        gk = ctx.galois_keygen(sk, plan.rotations(), seed=1)
        plan.bind(gk)
        batch = shape.batch
        cts = np.stack([ctx.encrypt(sk, plan.pack_input(x[b]), seed=b) for b in range(batch)])
        d_in = H.import_cts(ctx, cts)
        d_out = H.dev_empty(batch * 2 * par.n)
        d_r = H.to_dev(r)
        ws_bytes = plan.workspace_bytes(batch)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")

        def step():
            return plan.he_fc(d_in, batch, d_r, 17, d_out, ws, ws_bytes, stream=stream)

    if args.copy_probe_mib:
        src = torch.ones(args.copy_probe_mib << 17, dtype=torch.int64, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        cnt = step()
    torch.cuda.synchronize()
    ctx.profile_enable(args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        cnt = step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kernel_ms = ctx.profile_collect(args.steps)
    ctx.profile_enable(0)
    ctx.profile_select(0)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    rotations = cnt["perm"] + cnt["hstperm_in"]
    rot_per_s = rotations / (ms_per_step * 1e-3)
    kavg_ms = float(np.mean(kernel_ms)) if kernel_ms else float("nan")
    roof = None
    if is_conv:
        # dominant kernel: the per-coefficient multiply-accumulate (ScMult + Add of Sec. III-B)
        macs = cnt["scmult"] * 2 * par.n                       # two polynomials per ciphertext
        groups, nterm = plan.nout * plan.cn, plan.nin * plan.ntap
        if args.vector_mac:
            unit_ops = OPS_MAC128
            ops = macs * OPS_MAC128 + batch * groups * 2 * par.n * OPS_REDUCE128
            kernel, units, traffic = "conv_mac_kernel", macs, None
        else:
            # on the matrix cores the product streams the digit-plane images once: it is bound by HBM.
            # algorithmic bytes: every encoded kernel polynomial, every rotated input, every sum, 8 B a residue
            alg_bytes = 8.0 * par.n * (groups * nterm + 2 * batch * nterm + 2 * batch * groups)
            achieved_gbs = alg_bytes / (kavg_ms * 1e-3) / 1e9
            roof = {"bound": "hbm", "kernel": "conv_mfma_kernel", "achieved": achieved_gbs, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": achieved_gbs / HBM_PEAK_GBS,
                    # HBM bytes per launch from rocprofv3 counters (profiles/he_conv_16x16x128_3x3x128_b16_hbm_traffic.txt)
                    "traffic": (442524 + 66449) * 1024.0 if not args.special_prime else None, "kernel_ms_avg": kavg_ms,
                    "units_per_launch": macs, "bytes_per_unit": alg_bytes / macs,
                    "int8_mfma_top_s": macs * 64 * 2 / (kavg_ms * 1e-3) / 1e12}
            ops, unit_ops, kernel, units, traffic = 0, 0, "conv_mfma_kernel", macs, None
        config = {"workload": args.workload, "layer": "he_conv", "n": par.n, "c_o": shape.c_o, "c_i": shape.c_i,
                  "k": shape.k_h, "image": [shape.u_h, shape.u_w], "batch": batch, "c_n": plan.cn,
                  "gadget_digits": ctx.ndigits, "multiply_accumulate": "vector" if args.vector_mac else "matrix cores"}
    else:
        # dominant kernel: rotate-and-accumulate, G fused ScMult+Perm+Add units per input
        unit_ops = (ops_per_fused_perm_special if args.special_prime else ops_per_fused_perm)(par.n, 11, ctx.ndigits)
        ops = unit_ops * batch * (plan.G - 1)      # the g = 0 unit has no Perm and is not counted
        kernel, units = "perm_accumulate_special_2048" if args.special_prime else "perm_accumulate_2048", batch * plan.G
        # HBM bytes per launch measured with rocprofv3 counters for the default workload
        # (profiles/perm_accumulate_fc_128x1024_b64_hbm_traffic.txt); not measured for the others
        traffic = (48155 + 67584) * 1024.0 if args.workload == "fc_128x1024_b64" and not args.special_prime else None
        config = {"workload": args.workload, "layer": "he_fc", "n": par.n, "n_o": shape.n_o, "n_i": shape.n_i,
                  "batch": batch, "G": plan.G, "gadget_digits": ctx.ndigits}
    config["key_switching"] = "special prime" if args.special_prime else "one prime"
    achieved = ops / (kavg_ms * 1e-3) / 1e12
    out = {
        "metric": "HE rotations/sec and he_fc/he_conv layers/sec at n=2048; % of HBM/int roofline",
        "value": rot_per_s,
        "unit": "rotations/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u64",
        "data": "synthetic",
        "config": config,
        "layers_per_s": 1e3 / ms_per_step,
        "inputs_per_s": batch * 1e3 / ms_per_step,
        "ops_per_step": cnt,
        "roofline": roof or {"bound": "alu", "kernel": kernel, "achieved": achieved, "peak": ALU_PEAK_TOPS,
                             "unit": "TOP/s (32-bit integer)", "frac": achieved / ALU_PEAK_TOPS, "traffic": traffic,
                             "kernel_ms_avg": kavg_ms, "units_per_launch": units, "int_ops_per_unit": unit_ops},
    }
    if not args.no_secondary and not args.special_prime:
        out["also"] = secondary_workloads(ctx, sk, H, torch)
    if not args.no_cpu_baseline:
        from oracle.oracle import Oracle
        o = Oracle(par.n, par.q, par.p, par.gadget_bits, special=par.special)
        osk = o.keygen(0)
        got = H.export_cts(ctx, d_out, batch * (plan.nout if is_conv else 1))
        if is_conv:
            # one output ciphertext of one input: 1152 ScMult, 7 Perm plus the 128 hoisted input rotations
            tk, gkk = o.conv_keys(osk, shape.tuple, seed=8)
            mask = o.conv_mask_slots(shape.tuple, r[0], 3, 0, 0)
            c0 = time.perf_counter()
            want, ocnt = o.he_conv_block(shape.tuple, K, 0, cts[0], tk, gkk, mask)
            c1 = time.perf_counter()
            assert np.array_equal(got[0], want), "HIP result differs from the oracle"
            out["cpu_baseline"] = {"value": (ocnt["perm"] + ocnt["hstperm_in"]) / (c1 - c0), "unit": "rotations/s",
                                   "cores": 1, "kind": "oracle",
                                   "sample": f"output ciphertext 0 of input 0 of {args.workload} (he_conv_block: "
                                             f"{ocnt['scmult']} ScMult, {ocnt['perm']} Perm, {ocnt['hstperm_in']} HstPerm), "
                                             f"{c1 - c0:.1f} s wall"}
        else:
            sample = min(args.cpu_sample, batch)
            wpoly = o.fc_encode_rowwise(W)
            ksk = o.fc_keys(osk, shape.n_o, shape.n_i, seed=1)
            c0 = time.perf_counter()
            for _ in range(args.cpu_repeat):
                outs, ocnt = o.he_fc_batch(wpoly, shape.n_o, shape.n_i, cts[:sample], ksk, r[:sample], 17)
            c1 = time.perf_counter()
            assert np.array_equal(got[:sample], outs), "HIP result differs from the oracle"
            # the same oracle on one thread: two inputs, one after the other
            mask0 = [o.fc_mask_slots(shape.n_o, shape.n_i, r[b], 17, b) for b in range(2)]
            s0 = time.perf_counter()
            single = [o.he_fc(wpoly, cts[b], ksk, mask0[b]) for b in range(2)]
            s1 = time.perf_counter()
            assert all(np.array_equal(got[b], single[b][0]) for b in range(2))
            out["cpu_baseline"] = {"value": args.cpu_repeat * ocnt["perm"] / (c1 - c0), "unit": "rotations/s",
                                   "cores": o.max_threads(), "kind": "oracle",
                                   "one_thread_value": sum(c["perm"] for _, c in single) / (s1 - s0),
                                   "sample": f"{sample} of the {batch} inputs of {args.workload}, {args.cpu_repeat} passes "
                                             f"(he_fc_batch: {ocnt['perm']} Perm, {ocnt['scmult']} ScMult per pass), "
                                             f"{c1 - c0:.1f} s wall"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
