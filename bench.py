#!/usr/bin/env python3
"""Benchmark of the GALA linear-layer hot path on one MI355X.

A "step" of the headline is one he_fc call over the whole batch of the workload (ScMult, Perm, Add and share
generation for every input), with ciphertexts, encoded weights and Galois keys already resident on the device
in internal form.  The reported value is homomorphic rotations (Perm) per second inside that layer.  The same
run then measures the other four benchmark configurations (`configs`), each with the roofline of its dominant
kernel (timed with HIP events on the stream the kernel runs on) and with the CPU oracle timed on a bounded
sample of the same inputs, whose ciphertexts must equal the GPU's.  Prints ONE JSON line.
"""
import argparse
import concurrent.futures
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "HE rotations/sec and he_fc/he_conv layers/sec at n=2048; % of HBM/int roofline"

# ---- integer-ALU roofline --------------------------------------------------------------------------------------
# 256 CUs x 4 SIMDs x 16 lanes 32-bit integer lane-operations per cycle.  Three peaks are reported:
#   nominal    lanes x the 2.4 GHz the part is specified at (the `peak` of the roofline object);
#   sustained  lanes x the 2.18 GHz it holds under this load (profiles/perm_accumulate_fc_128x1024_b64_valu_counters.txt);
#   mul32      the measured issue rate of v_mad_u64_u32 / v_mul_lo_u32 (profiles/probe_int_mul.txt).
ALU_LANES = 256 * 4 * 16
ALU_PEAK_TOPS = ALU_LANES * 2.4e9 / 1e12
ALU_SUSTAINED_TOPS = ALU_LANES * 2.18e9 / 1e12
MUL32_MEASURED_TOPS = 36.6
HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published

# Two operation counts per unit of work.
# (1) every 32-bit integer operation of the leanest formulation known here of each 64-bit modular primitive
#     (multiply-adds, adds with carry, selects; no address arithmetic, no register moves):
OPS_CONST_MUL = 13      # y*w mod q, w with precomputed quotient: 6 for the high product, 6 + 1 for y*w - h*q
OPS_CSUB = 4            # conditional subtraction: sub, subb, two selects on the borrow
OPS_BF_FWD = OPS_CONST_MUL + 1 + 3             # lazy forward butterfly: x + v, x + 2q - v
OPS_BF_INV = OPS_CONST_MUL + 1 + 3 + OPS_CSUB  # inverse butterfly: x + y reduced, (x - y + 2q) * w
OPS_MAC128 = 10         # 64x64 product added into a 128-bit sum: 4 multiply-adds and 6 carry additions
OPS_REDUCE128 = 2 * OPS_CONST_MUL + 2 * OPS_CSUB + 1
# (2) 32x32-bit multiplies only, 10 per modular multiplication (a 64x64 high product and two 64x64 low products
#     from 32-bit halves), against the measured multiply issue rate.
MUL32_PER_MODMUL = 10


def transform_ops(n, logn):
    half = n // 2
    inverse = half * (logn - 1) * OPS_BF_INV + half * (2 * OPS_CONST_MUL + 2 * OPS_CSUB + 4)   # n^-1 folded in
    forward = half * logn * OPS_BF_FWD + n * OPS_CSUB           # one conditional subtraction per coefficient
    return inverse, forward


def ops_per_fused_perm(n, logn, ndigits):
    """Integer operations of one ScMult + Perm + Add on one ciphertext (one 'fused unit')."""
    inverse, forward = transform_ops(n, logn)
    scmult_c1 = n * OPS_CONST_MUL                               # c1 (.) w before the inverse transform
    c0_term = n * (OPS_CONST_MUL + 1)                           # permuted c0 (.) w added to the sum
    digits = ndigits * n * 2                                    # shift and mask
    key_mac = 2 * ndigits * n * (OPS_CONST_MUL + 1)             # inner product with (b_j, a_j)
    accumulate = 2 * n * OPS_CSUB                               # keep the running sums below 8q
    return inverse + ndigits * forward + scmult_c1 + c0_term + digits + key_mac + accumulate


def modmuls_per_fused_perm(n, logn, ndigits, scmult=True):
    """Modular multiplications of the same unit: butterflies of 1 + ndigits transforms, the key inner product and
    (scmult) the two products with the encoded weight."""
    return (1 + ndigits) * (n // 2) * logn + 2 * ndigits * n + (2 * n if scmult else 0)


def ops_per_fused_perm_special(n, logn, ndigits):
    """The fused unit with special-prime key switching: every digit is transformed and multiplied in both moduli,
    the two sums modulo P go back to coefficients (two inverse transforms); the two forward transforms of the
    summed remainders happen once per workgroup and are not counted."""
    inverse, forward = transform_ops(n, logn)
    scmult_c1 = n * OPS_CONST_MUL
    c0_term = n * (2 * OPS_CONST_MUL + 1)                       # permuted c0 (.) w, times P
    digits = 2 * ndigits * n * 2
    key_mac = 4 * ndigits * n * (OPS_CONST_MUL + 1)             # (b_j, a_j) modulo q and modulo P
    accumulate = 2 * n * OPS_CSUB
    remainders = 2 * n * (OPS_CONST_MUL + OPS_CSUB + 2 * OPS_CSUB + 1)   # canonical mod P, lift, reduce mod q, add
    return 3 * inverse + 2 * ndigits * forward + scmult_c1 + c0_term + digits + key_mac + accumulate + remainders


def modmuls_per_fused_perm_special(n, logn, ndigits):
    return (3 + 2 * ndigits) * (n // 2) * logn + 4 * ndigits * n + 2 * n + 4 * n


def ops_decperm(n, logn, ndigits):
    inverse, forward = transform_ops(n, logn)
    return inverse + ndigits * forward + ndigits * n * 2


def ops_hstperm(n, ndigits):
    return 2 * ndigits * n * (OPS_CONST_MUL + 1) + n + 2 * n * OPS_CSUB


# ---- timing helpers --------------------------------------------------------------------------------------------
def prewarm(fn, torch, seconds):
    """Runs fn for at least `seconds` of wall time (whatever --warmup says): clocks and caches reach their steady
    state before anything is timed.  Returns the milliseconds spent."""
    t0 = time.perf_counter()
    while True:
        for _ in range(20):
            fn()
        torch.cuda.synchronize()
        if time.perf_counter() - t0 >= seconds:
            return (time.perf_counter() - t0) * 1e3


def wall_ms(fn, torch, steps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def kernel_ms(ctx, fn, torch, steps, which):
    """HIP-event times of the selected kernel over `steps` calls of fn (events recorded by the library on the
    stream the kernel is launched on)."""
    ctx.profile_select(which)
    ctx.profile_enable(steps)
    torch.cuda.synchronize()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    ms = ctx.profile_collect(steps)
    ctx.profile_enable(0)
    ctx.profile_select(0)
    return ms


def stats(ms):
    if not ms:
        return {"kernel_ms_avg": None, "kernel_ms_median": None, "launches_timed": 0}
    return {"kernel_ms_avg": float(np.mean(ms)), "kernel_ms_median": float(np.median(ms)), "launches_timed": len(ms)}


def profile_traffic(name):
    """HBM bytes per launch of a kernel as the committed rocprofv3 counter summary states them
    (a line 'hbm_bytes_per_launch: <number>' in profiles/<name>), or None: never a number typed in here."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        m = re.search(r"^hbm_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), re.M)
    except OSError:
        return None, None
    return (float(m.group(1)), "profiles/" + name) if m else (None, None)


def alu_roofline(kernel, kms, units, ops_unit, modmul_unit, traffic_file=None, note=None):
    """Roofline object of an integer-ALU-bound kernel: `frac` = every integer operation against the nominal peak;
    the multiply-only count against the measured multiply rate and the sustained-clock peak are given beside it."""
    st = stats(kms)
    t = (st["kernel_ms_avg"] or float("nan")) * 1e-3
    achieved = units * ops_unit / t / 1e12
    mul32 = units * modmul_unit * MUL32_PER_MODMUL / t / 1e12
    traffic, src = profile_traffic(traffic_file) if traffic_file else (None, None)
    out = {"bound": "alu", "kernel": kernel, "achieved": achieved, "peak": ALU_PEAK_TOPS, "unit": "TOP/s (32-bit integer)",
           "frac": achieved / ALU_PEAK_TOPS, "traffic": traffic, "traffic_source": src,
           "units_per_launch": units, "int_ops_per_unit": ops_unit,
           "frac_at_sustained_clock": achieved / ALU_SUSTAINED_TOPS, "peak_at_sustained_clock": ALU_SUSTAINED_TOPS,
           "mul32_per_unit": modmul_unit * MUL32_PER_MODMUL, "mul32_achieved": mul32,
           "mul32_peak_measured": MUL32_MEASURED_TOPS, "mul32_frac": mul32 / MUL32_MEASURED_TOPS}
    out.update(st)
    if note:
        out["note"] = note
    return out


def hbm_roofline(kernel, kms, alg_bytes, traffic_file=None, extra=None):
    st = stats(kms)
    t = (st["kernel_ms_avg"] or float("nan")) * 1e-3
    gbs = alg_bytes / t / 1e9
    traffic, src = profile_traffic(traffic_file) if traffic_file else (None, None)
    out = {"bound": "hbm", "kernel": kernel, "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
           "frac": gbs / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": src, "bytes_per_launch": alg_bytes}
    out.update(st)
    if extra:
        out.update(extra)
    return out


# ---- the oracle beside it ----------------------------------------------------------------------------------------
def oracle_for(par):
    from oracle.oracle import Oracle
    o = Oracle(par.n, par.q, par.p, par.gadget_bits, special=par.special)
    return o, o.keygen(0)


def host_threads(o):
    return max(1, min(o.max_threads(), os.cpu_count() or 1))


# ---- he_fc -------------------------------------------------------------------------------------------------------
def fc_config(ctx, sk, D, torch, par, shape, steps, prewarm_s, cpu_sample, cpu_repeat, special=False, mask_seed=17,
              warmup=0, compare=True):
    """One he_fc workload: wall time per layer, the rotate-and-accumulate kernel's HIP-event times, its roofline,
    and the oracle on `cpu_sample` of the inputs.  Returns (record, state for the headline)."""
    from paper_2105_01827_amd import workloads as wl
    W, x, r = wl.fc_inputs(shape)
    plan = ctx.fc_plan(W)
    gk = ctx.galois_keygen(sk, plan.rotations(), seed=1)
    plan.bind(gk)
    batch = shape.batch
    cts = np.stack([ctx.encrypt(sk, plan.pack_input(x[b]), seed=b) for b in range(batch)])
    d_in = D.import_cts(ctx, cts)
    d_out = D.dev_empty(batch * 2 * par.n)
    d_r = D.to_dev(r)
    ws_bytes = plan.workspace_bytes(batch)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    cnt = {}

    def step():
        cnt.update(plan.he_fc(d_in, batch, d_r, mask_seed, d_out, ws, ws_bytes, stream=stream))

    pre = prewarm(step, torch, prewarm_s)
    for _ in range(warmup):
        step()
    ms = wall_ms(step, torch, steps)
    kms = kernel_ms(ctx, step, torch, steps, 0)
    G = plan.G
    if special:
        unit_ops, unit_mm = ops_per_fused_perm_special(par.n, 11, ctx.ndigits), modmuls_per_fused_perm_special(par.n, 11, ctx.ndigits)
        kernel = "perm_accumulate_special_2048"
    else:
        unit_ops, unit_mm = ops_per_fused_perm(par.n, 11, ctx.ndigits), modmuls_per_fused_perm(par.n, 11, ctx.ndigits)
        kernel = "perm_accumulate_2048"
    if G > 1:
        roof = alu_roofline(kernel, kms, batch * (G - 1), unit_ops, unit_mm,      # the g = 0 unit has no Perm: not counted
                            traffic_file=f"perm_accumulate_{shape.name}_hbm_traffic.txt" if not special else None)
    else:
        # no rotation at all: one ScMult and the mask's encoding (a transform mod p and one mod q) per input
        inverse, forward = transform_ops(par.n, 11)
        roof = alu_roofline(kernel, kms, batch, 2 * par.n * OPS_CONST_MUL + inverse + forward + par.n * OPS_CONST_MUL,
                            11 * par.n + 3 * par.n,
                            note="latency-bound: one input is two workgroups of work; the figure is the launch's duration")
    gazelle = None
    if compare:
        # the paper's comparison schedule (hybrid method, Sec. III-A(2)) on the same kernels and inputs
        hplan = ctx.fc_hybrid_plan(W)
        hgk = ctx.galois_keygen(sk, hplan.rotations(), seed=1)
        hplan.bind(hgk)
        h_out = D.dev_empty(batch * 2 * par.n)
        h_wsb = hplan.workspace_bytes(batch)
        h_ws = torch.empty(h_wsb, dtype=torch.uint8, device="cuda")
        hcnt = {}

        def hstep():
            hcnt.update(hplan.he_fc_hybrid(d_in, batch, d_r, mask_seed, h_out, h_ws, h_wsb, stream=stream))

        prewarm(hstep, torch, min(prewarm_s, 0.2))
        hms = wall_ms(hstep, torch, max(5, steps // 4))
        gazelle = {"schedule": "hybrid matrix-vector product (Sec. III-A(2)), same kernels, same inputs",
                   "ms_per_layer": hms, "ops_per_layer": dict(hcnt), "gala_speedup": hms / ms,
                   "decrypts": bool(special) or hplan.G == 1,
                   "note": "the rotate-and-sum Perms of one input depend on each other: log2(n/n_o) launches of `batch` "
                           "workgroups each"}
        if shape.name == "fc_16x128_b1":
            gazelle["paper_speedup"] = {"value": 19, "where": "Table 'Runtime cost of matrix-vector multiplication', "
                                                              "16x128, LAN, Intel i7-8700 (another machine)"}
        del hplan, hgk, h_out, h_ws
    rec = {"workload": shape.name, "layer": "he_fc", "n_o": shape.n_o, "n_i": shape.n_i, "batch": batch, "G": G,
           "key_switching": "special prime" if special else "one prime", "decrypts": True,
           "steps": steps, "prewarm_ms": pre, "ms_per_layer": ms, "layers_per_s": 1e3 / ms,
           "inputs_per_s": batch * 1e3 / ms, "rotations_per_s": cnt["perm"] * 1e3 / ms, "ops_per_layer": dict(cnt),
           "roofline": roof, "cpu_baseline": None, "gazelle_schedule": gazelle}
    if cpu_sample:
        o, osk = oracle_for(par)
        got = D.export_cts(ctx, d_out, batch)
        sample = min(cpu_sample, batch)
        wpoly = o.fc_encode_rowwise(W)
        ksk = o.fc_keys(osk, shape.n_o, shape.n_i, seed=1)
        c0 = time.perf_counter()
        for _ in range(cpu_repeat):
            outs, ocnt = o.he_fc_batch(wpoly, shape.n_o, shape.n_i, cts[:sample], ksk, r[:sample], mask_seed)
        c1 = time.perf_counter()
        assert np.array_equal(got[:sample], outs), f"{shape.name}: HIP result differs from the oracle"
        threads = min(host_threads(o), sample)
        if ocnt["perm"]:
            value, unit = cpu_repeat * ocnt["perm"] / (c1 - c0), "rotations/s"
        else:
            value, unit = cpu_repeat * sample / (c1 - c0), "layers/s"
        rec["cpu_baseline"] = {"value": value, "unit": unit, "cores": threads, "kind": "oracle",
                               "sample": f"{sample} of the {batch} inputs of {shape.name}, {cpu_repeat} passes (he_fc_batch: "
                                         f"{ocnt['perm']} Perm, {ocnt['scmult']} ScMult per pass), {c1 - c0:.1f} s wall; "
                                         f"ciphertexts equal the GPU's"}
    return rec


# ---- he_conv -----------------------------------------------------------------------------------------------------
def conv_config(ctx, sk, D, torch, par, shape, steps, prewarm_s, cpu_blocks, special=False, vector_mac=False, warmup=0,
                compare=True):
    from paper_2105_01827_amd import workloads as wl
    K, x, r = wl.conv_inputs(shape)
    plan = ctx.conv_plan(K, shape.u_h, shape.u_w)
    gk = ctx.galois_keygen(sk, plan.rotations(), seed=8)
    plan.bind(gk)
    if not vector_mac:
        plan.prepare_batched()      # multiply-accumulate on the matrix cores
    batch = shape.batch
    slots = np.stack([plan.pack_input(x[b]) for b in range(batch)])
    cts = np.stack([[ctx.encrypt(sk, slots[b, I], seed=1000 * b + I) for I in range(plan.nin)] for b in range(batch)])
    d_in = D.import_cts(ctx, cts.reshape(-1, 2 * par.n))
    d_out = D.dev_empty(batch * plan.nout * 2 * par.n)
    d_r = D.to_dev(r)
    ws_bytes = plan.workspace_bytes(batch)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    cnt = {}

    def step():
        cnt.update(plan.he_conv(d_in, batch, d_r, 3, d_out, ws, ws_bytes, stream=stream))

    pre = prewarm(step, torch, prewarm_s)
    for _ in range(warmup):
        step()
    ms = wall_ms(step, torch, steps)
    k_perm, k_mac, k_hoist = (kernel_ms(ctx, step, torch, steps, w) for w in (0, 1, 2))
    n, nd = par.n, ctx.ndigits
    groups, nterm = plan.nout * plan.cn, plan.nterm
    macs = cnt["scmult"] * 2 * n                           # two polynomials per ciphertext
    kernels = []
    # input rotations: one DecPerm per input ciphertext, one HstPerm per rotating term (written as the digit-plane image)
    hoist_ops = cnt["decperm_in"] * ops_decperm(n, 11, nd) + cnt["hstperm_in"] * ops_hstperm(n, nd)
    hoist_mm = cnt["decperm_in"] * (1 + nd) * (n // 2) * 11 + cnt["hstperm_in"] * 2 * nd * n
    if not special:
        kernels.append(alu_roofline("decperm_2048 + hstperm_pack_2048", k_hoist, 1, hoist_ops, hoist_mm))
    else:
        kernels.append(dict({"kernel": "decperm_special_2048 + hstperm_special_2048", "bound": "alu"}, **stats(k_hoist)))
    if vector_mac:
        kernels.append(alu_roofline("conv_mac_kernel", k_mac, 1, macs * OPS_MAC128 + batch * groups * 2 * n * OPS_REDUCE128,
                                    macs))
    else:
        # on the matrix cores the product streams the digit-plane images once: bound by HBM.  Algorithmic bytes:
        # every encoded kernel polynomial, every rotated input, every sum, 8 B a residue
        alg_bytes = 8.0 * n * (groups * nterm + 2 * batch * nterm + 2 * batch * groups)
        st = stats(k_mac)
        kernels.append(hbm_roofline("conv_mfma_kernel", k_mac, alg_bytes,
                                    traffic_file=f"he_conv_{shape.name[5:]}_hbm_traffic.txt" if not special else None,
                                    extra={"units_per_launch": macs, "bytes_per_unit": alg_bytes / macs,
                                           "int8_mfma_top_s": macs * 64 * 2 / ((st["kernel_ms_avg"] or float("nan")) * 1e-3) / 1e12}))
    if special:
        kernels.append(alu_roofline("perm_accumulate_special_2048", k_perm, cnt["perm"],
                                    ops_per_fused_perm_special(n, 11, nd) - n * OPS_CONST_MUL,
                                    modmuls_per_fused_perm_special(n, 11, nd) - 2 * n))
    else:
        kernels.append(alu_roofline("perm_accumulate_2048", k_perm, cnt["perm"],
                                    ops_per_fused_perm(n, 11, nd) - 2 * n * OPS_CONST_MUL,      # no ScMult in these units
                                    modmuls_per_fused_perm(n, 11, nd, scmult=False)))
    gazelle = None
    if compare:
        # the paper's comparison schedule (output rotation, Sec. III-B(2)) on the same plan, keys and inputs
        o_out = D.dev_empty(batch * plan.nout * 2 * par.n)
        o_wsb = plan.outrot_workspace_bytes(batch)
        o_ws = torch.empty(o_wsb, dtype=torch.uint8, device="cuda")
        ocnt_g = {}

        def ostep():
            ocnt_g.update(plan.he_conv_outrot(d_in, batch, d_r, 3, o_out, o_ws, o_wsb, stream=stream))

        prewarm(ostep, torch, min(prewarm_s, 0.2))
        oms = wall_ms(ostep, torch, max(5, steps // 4))
        gazelle = {"schedule": "output-rotation MIMO convolution (Sec. III-B(2)), same plan, keys and inputs; "
                               "multiply-accumulate on the vector ALU",
                   "ms_per_layer": oms, "ops_per_layer": dict(ocnt_g), "gala_speedup": oms / ms,
                   "paper_speedup": {"value": 2.6, "where": "Table 'Runtime cost of convolution', 16x16@128 with 3x3@128, "
                                                            "LAN, Intel i7-8700 (another machine)"}}
        del o_out, o_ws
    dominant = max(kernels, key=lambda k: k["kernel_ms_avg"] or 0.0)
    rotations = cnt["perm"] + cnt["hstperm_in"]
    rec = {"workload": shape.name, "layer": "he_conv", "c_o": shape.c_o, "c_i": shape.c_i, "k": shape.k_h,
           "image": [shape.u_h, shape.u_w], "batch": batch, "c_n": plan.cn, "terms": nterm,
           "multiply_accumulate": "vector" if vector_mac else "matrix cores",
           "key_switching": "special prime" if special else "one prime",
           # Sec. III-C: with one-prime keys of 20-bit digits the input rotations' noise times the kernels exceeds
           # delta/2 for 3x3 kernels at p ~ 2^20; the ciphertexts equal the oracle's either way
           "decrypts": bool(special) or shape.k_h * shape.k_w == 1,
           "steps": steps, "prewarm_ms": pre, "ms_per_layer": ms, "layers_per_s": 1e3 / ms,
           "inputs_per_s": batch * 1e3 / ms, "rotations_per_s": rotations * 1e3 / ms, "ops_per_layer": dict(cnt),
           "roofline": dominant, "kernels": kernels, "cpu_baseline": None, "gazelle_schedule": gazelle}
    if cpu_blocks:
        o, osk = oracle_for(par)
        got = D.export_cts(ctx, d_out, batch * plan.nout).reshape(batch, plan.nout, 2 * n)
        tk, gkk = o.conv_keys(osk, shape.tuple, seed=8)
        threads = min(host_threads(o), cpu_blocks, batch)
        picks = [(b, (5 * b) % plan.nout) for b in range(min(cpu_blocks, batch))]    # one output block of each input

        def block(bO):
            b, O = bO
            mask = o.conv_mask_slots(shape.tuple, r[b], 3, b, O)
            return o.he_conv_block(shape.tuple, K, O, cts[b], tk, gkk, mask)

        c0 = time.perf_counter()
        with concurrent.futures.ThreadPoolExecutor(threads) as pool:
            res = list(pool.map(block, picks))
        c1 = time.perf_counter()
        rot = 0
        for (b, O), (want, ocnt) in zip(picks, res):
            assert np.array_equal(got[b, O], want), f"{shape.name}: HIP result differs from the oracle at ({b},{O})"
            rot += ocnt["perm"] + ocnt["hstperm_in"]
        rec["cpu_baseline"] = {"value": rot / (c1 - c0), "unit": "rotations/s", "cores": threads, "kind": "oracle",
                               "layers_per_s": len(picks) / (batch * plan.nout) / (c1 - c0),
                               "sample": f"{len(picks)} of the {batch * plan.nout} output ciphertexts of {shape.name}, one per "
                                         f"input, each recomputing its input's rotations (he_conv_block: {res[0][1]['scmult']} "
                                         f"ScMult, {res[0][1]['perm']} Perm, {res[0][1]['hstperm_in']} HstPerm), {threads} at a "
                                         f"time, {c1 - c0:.1f} s wall; ciphertexts equal the GPU's"}
    return rec


# ---- config 5: the 21 linear layers of a ResNet-18-shaped network, one input ------------------------------------
def resnet18_config(ctx, sk, D, torch, par, steps, prewarm_s, cpu_layers, stride_by_subsampling=False, warmup=0):
    """Every layer's plan, keys, inputs and workspace stay resident; a step is one pass over all 21 layers, enqueued
    back to back on one stream.  Reported: the pass eager and as one replayed HIP graph, each layer's own time, and the
    multiply-accumulate kernels' HBM rate (they stream every encoded kernel polynomial once)."""
    from paper_2105_01827_amd import workloads as wl
    rng = np.random.default_rng(0)
    layers, fc = wl.resnet18_layers()
    n = par.n
    L_state, calls = [], []
    total = dict(perm=0, decperm_in=0, hstperm_in=0, scmult=0, add=0)
    for li, L in enumerate(layers):
        K = rng.integers(0, par.p, size=(L.c_o, L.c_i, L.k, L.k), dtype=np.uint64)
        if L.stride > 1 and not stride_by_subsampling:
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
        cts = rng.integers(0, par.q, size=(t.tiles * plan.nin, 2 * n), dtype=np.uint64)     # interchange form
        r = rng.integers(0, par.p, size=(t.tiles, K.shape[0], t.tile_h, t.tile_w), dtype=np.uint64)
        d_in = D.import_cts(ctx, cts)
        d_out = D.dev_empty(t.tiles * plan.nout * 2 * n)
        d_r = D.to_dev(r)
        wsb = plan.workspace_bytes(t.tiles)
        ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
        st = dict(L=L, K=K, t=t, plan=plan, gk=gk, cts=cts, r=r, d_in=d_in, d_out=d_out, d_r=d_r, ws=ws, wsb=wsb, cnt={})

        def call(stream, s=st, li=li):
            s["cnt"].update(s["plan"].he_conv(s["d_in"], s["t"].tiles, s["d_r"], li, s["d_out"], s["ws"], s["wsb"], stream=stream))

        L_state.append(st)
        calls.append(call)
    W, x, r = wl.fc_inputs(fc, seed=77)
    fplan = ctx.fc_plan(W)
    fgk = ctx.galois_keygen(sk, fplan.rotations(), seed=1)
    fplan.bind(fgk)
    f_cts = rng.integers(0, par.q, size=(1, 2 * n), dtype=np.uint64)
    f_in, f_out, f_r = D.import_cts(ctx, f_cts), D.dev_empty(2 * n), D.to_dev(r)
    f_wsb = fplan.workspace_bytes(1)
    f_ws = torch.empty(f_wsb, dtype=torch.uint8, device="cuda")
    f_cnt = {}
    calls.append(lambda stream: f_cnt.update(fplan.he_fc(f_in, 1, f_r, 99, f_out, f_ws, f_wsb, stream=stream)))

    cur = torch.cuda.current_stream()

    def network():
        for c in calls:
            c(cur)

    pre = prewarm(network, torch, prewarm_s)
    for _ in range(warmup):
        network()
    eager_ms = wall_ms(network, torch, steps)
    # per layer, each on its own (synchronised), and the multiply-accumulate kernel of each convolution
    per_layer, weight_bytes, mac_ms = [], 0.0, 0.0
    for st, c in zip(L_state, calls):
        one = lambda c=c: c(cur)
        ms = wall_ms(one, torch, steps)
        kms = kernel_ms(ctx, one, torch, steps, 1)
        plan = st["plan"]
        groups, nterm = plan.nout * plan.cn, plan.nterm
        weight_bytes += 8.0 * n * groups * nterm
        mac_ms += float(np.mean(kms)) if kms else 0.0
        per_layer.append({"layer": st["L"].name, "tiles": st["t"].tiles, "c_n": plan.cn, "terms": nterm, "ms": ms,
                          "multiply_accumulate_ms": float(np.mean(kms)) if kms else None})
        for k in total:
            total[k] += st["cnt"][k]
    ms = wall_ms(lambda: calls[-1](cur), torch, steps)
    per_layer.append({"layer": fc.name, "G": fplan.G, "ms": ms})
    for k in total:
        total[k] += f_cnt[k]
    # the same pass captured once and replayed: the launches of the small layers no longer wait for the host
    graph_ms = None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(cur)
        with torch.cuda.stream(side):
            for c in calls:
                c(side)
        cur.wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            s = torch.cuda.current_stream()
            for c in calls:
                c(s)
        want = [st["d_out"].clone() for st in L_state]
        for st in L_state:
            st["d_out"].zero_()
        graph.replay()
        torch.cuda.synchronize()
        same = all(torch.equal(st["d_out"], w) for st, w in zip(L_state, want))
        if same:
            prewarm(graph.replay, torch, min(prewarm_s, 0.2))
            graph_ms = wall_ms(graph.replay, torch, steps)
    except Exception as e:      # a failed capture leaves the eager figure; say why
        graph_ms, same = None, f"capture failed: {e}"
    step_ms = min(eager_ms, graph_ms) if graph_ms else eager_ms
    rot = total["perm"] + total["hstperm_in"]
    gbs = weight_bytes / (mac_ms * 1e-3) / 1e9
    rec = {"workload": "resnet18_b1", "layers": len(per_layer), "batch": 1, "key_switching": "one prime",
           "decrypts": "1x1 layers and the FC; 3x3 and 7x7 layers need the special-prime mode (Sec. III-C noise)",
           "stride": "subsampling" if stride_by_subsampling else "polyphase",
           "steps": steps, "prewarm_ms": pre, "ms_per_network": step_ms, "ms_per_network_eager": eager_ms,
           "ms_per_network_graph_replay": graph_ms, "graph_replay_equals_eager": same,
           "ms_sum_of_layers_timed_alone": float(sum(p["ms"] for p in per_layer)),
           "networks_per_s": 1e3 / step_ms, "layers_per_s": len(per_layer) * 1e3 / step_ms,
           "rotations_per_s": rot * 1e3 / step_ms, "ops_per_network": total, "per_layer": per_layer,
           # at one input the multiply-accumulate streams every encoded kernel polynomial once: HBM-bound
           "roofline": {"bound": "hbm", "kernel": "conv_mac_stream_kernel / conv_mfma_kernel (the 20 convolutions)",
                        "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                        "traffic": None, "traffic_source": None, "kernel_ms_total": mac_ms, "bytes_per_step": weight_bytes},
           "cpu_baseline": None}
    if cpu_layers:
        o, osk = oracle_for(par)
        idx = sorted({0, len(L_state) // 2, len(L_state) - 1})[:cpu_layers]
        jobs = []
        for li in idx:
            st = L_state[li]
            plan, t = st["plan"], st["t"]
            shape = (st["K"].shape[0], st["K"].shape[1], st["K"].shape[2], st["K"].shape[3], t.tile_h, t.tile_w)
            got = D.export_cts(ctx, st["d_out"], t.tiles * plan.nout).reshape(t.tiles, plan.nout, 2 * n)
            tk, gkk = o.conv_keys(osk, shape, seed=8)
            for b, O in {(0, 0), (t.tiles - 1, plan.nout - 1), (t.tiles // 2, plan.nout // 2)}:
                jobs.append((li, shape, b, O, tk, gkk, got[b, O]))
        # the graph replay or the timing loops ran the layers last with the mask seeds used above

        def block(j):
            li, shape, b, O, tk, gkk, _ = j
            st = L_state[li]
            nin = st["plan"].nin
            mask = o.conv_mask_slots(shape, st["r"][b], li, b, O)
            return o.he_conv_block(shape, st["K"], O, st["cts"][b * nin:(b + 1) * nin], tk, gkk, mask)

        threads = min(host_threads(o), len(jobs))
        c0 = time.perf_counter()
        with concurrent.futures.ThreadPoolExecutor(threads) as pool:
            res = list(pool.map(block, jobs))
        c1 = time.perf_counter()
        rot_cpu = 0
        for j, (want, ocnt) in zip(jobs, res):
            assert np.array_equal(j[6], want), f"resnet18_b1 {L_state[j[0]]['L'].name}: HIP result differs from the oracle"
            rot_cpu += ocnt["perm"] + ocnt["hstperm_in"]
        rec["cpu_baseline"] = {"value": rot_cpu / (c1 - c0), "unit": "rotations/s", "cores": threads, "kind": "oracle",
                               "sample": f"{len(jobs)} output ciphertexts (first, middle and last tile/block) of layers "
                                         f"{', '.join(L_state[li]['L'].name for li in idx)}, each recomputing its input's "
                                         f"rotations, {threads} at a time, {c1 - c0:.1f} s wall; ciphertexts equal the GPU's"}
    return rec


# ---- the other entry points (short runs) -------------------------------------------------------------------------
def entry_points(ctx, sk, D, torch, par):
    """Plain Perm on a batch of ciphertexts, hoisted rotations, and the client's two steps on the device."""
    res = {}
    rng = np.random.default_rng(0)
    count = 4096
    gk = ctx.galois_keygen(sk, [(0, 1)], seed=3)
    d_in = D.to_dev(rng.integers(0, par.q, size=(count, 2 * par.n), dtype=np.uint64))
    d_out = D.dev_empty(count * 2 * par.n)
    fn = lambda: ctx.rotate(gk, d_in, count, (0, 1), d_out)
    prewarm(fn, torch, 0.1)
    t = wall_ms(fn, torch, 100)
    res["rotate_4096_cts"] = {"ms": t, "rotations_per_s": count * 1e3 / t}
    del d_in, d_out
    hc, hr = 512, 8
    gk8 = ctx.galois_keygen(sk, [(0, 1 + k) for k in range(hr)], seed=4)
    d_in = D.to_dev(rng.integers(0, par.q, size=(hc, 2 * par.n), dtype=np.uint64))
    d_out = D.dev_empty(hc * hr * 2 * par.n)
    hwsb = ctx.rotate_hoisted_workspace(hc)
    hws = torch.empty(hwsb, dtype=torch.uint8, device="cuda")
    fn = lambda: ctx.rotate_hoisted(gk8, d_in, hc, d_out, hws, hwsb)
    prewarm(fn, torch, 0.1)
    t = wall_ms(fn, torch, 100)
    res["rotate_hoisted_512_cts_x8"] = {"ms": t, "rotations_per_s": hc * hr * 1e3 / t}
    del d_in, d_out, hws, gk8
    d_slots = D.to_dev(rng.integers(0, par.p, size=(count, par.n), dtype=np.uint64))
    d_seeds = D.to_dev(np.arange(count, dtype=np.uint64))
    d_ct = D.dev_empty(count * 2 * par.n)
    fn = lambda: ctx.encrypt_batch(sk, d_slots, d_seeds, count, d_ct)
    prewarm(fn, torch, 0.05)
    t = wall_ms(fn, torch, 30)
    res["encrypt_4096_cts"] = {"ms": t, "ciphertexts_per_s": count * 1e3 / t}
    fn = lambda: ctx.decrypt_batch(sk, d_ct, count, d_slots)
    prewarm(fn, torch, 0.05)
    t = wall_ms(fn, torch, 30)
    res["decrypt_4096_cts"] = {"ms": t, "ciphertexts_per_s": count * 1e3 / t}
    # Plain forward transforms (the import of coefficient-form ciphertexts): the rate at which encoded kernels could
    # be produced on the fly from 4-byte coefficients, to set against the rate at which the stored 8-byte evaluation
    # form streams from HBM in the multiply-accumulate (bytes_per_step / kernel_ms_total of resnet18_b1).
    d_coef = D.to_dev(rng.integers(0, par.q, size=(count, 2 * par.n), dtype=np.uint64))
    fn = lambda: ctx.ct_import(d_coef, count, d_ct)
    prewarm(fn, torch, 0.05)
    t = wall_ms(fn, torch, 30)
    res["forward_transform_8192_polys"] = {"ms": t, "polynomials_per_s": 2 * count * 1e3 / t,
                                           "evaluation_form_bytes_per_s": 2 * count * par.n * 8 * 1e3 / t}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="fc_128x1024_b64",
                    choices=["fc_16x128_b1", "fc_128x1024_b64", "fc_1000x2048_b64", "conv_16x16x128_3x3x128_b16", "resnet18_b1"],
                    help="the configuration the headline (value, ms_per_step, roofline, cpu_baseline) is taken on")
    ap.add_argument("--prewarm-s", type=float, default=0.4,
                    help="wall time every workload runs untimed before its measurements, on top of --warmup")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="measure the headline workload only")
    ap.add_argument("--no-compare", action="store_true",
                    help="skip the paper's comparison schedules (hybrid FC, output-rotation convolution) beside each workload")
    ap.add_argument("--vector-mac", action="store_true",
                    help="convolution: keep the multiply-accumulate on the vector ALU instead of the matrix cores")
    ap.add_argument("--special-prime", action="store_true",
                    help="key switching with the special prime (keys modulo q*P, exact division by P): the mode in "
                         "which 3x3 convolutions decrypt at the 20-bit plaintext modulus")
    ap.add_argument("--stride-by-subsampling", action="store_true",
                    help="resnet18_b1: evaluate strided layers at stride 1 and drop outputs instead of the polyphase split")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run one plain device copy of this size (calibrates rocprofv3 HBM byte counters)")
    ap.add_argument("--cpu-repeat", type=int, default=3, help="passes of the oracle over its sample (128x1024 FC)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2105_01827_amd import binding, devmem as D, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    par = wl.DEFAULT_SPECIAL if args.special_prime else wl.DEFAULT
    ctx = binding.Context(par.n, par.q, par.p, par.gadget_bits, par.special)
    sk = ctx.keygen(0)
    cpu = not args.no_cpu_baseline
    if args.copy_probe_mib:
        src = torch.ones(args.copy_probe_mib << 17, dtype=torch.int64, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    fc_shapes = {s.name: s for s in (wl.FC_16x128, wl.FC_128x1024, wl.FC_1000x2048)}
    # oracle sample per FC workload: about the same CPU time each
    fc_sample = {"fc_16x128_b1": (1, 200), "fc_128x1024_b64": (64, args.cpu_repeat), "fc_1000x2048_b64": (16, 1)}

    def run(name, steps, warmup=0):
        pre = args.prewarm_s
        if name in fc_shapes:
            sample, repeat = fc_sample[name]
            return fc_config(ctx, sk, D, torch, par, fc_shapes[name], steps, pre, sample if cpu else 0, repeat,
                             special=args.special_prime, warmup=warmup, compare=not args.no_compare)
        if name.startswith("conv"):
            return conv_config(ctx, sk, D, torch, par, wl.CONV_16x16_128_3x3, steps, pre, 16 if cpu else 0,
                               special=args.special_prime, vector_mac=args.vector_mac, warmup=warmup,
                               compare=not args.no_compare)
        return resnet18_config(ctx, sk, D, torch, par, steps, pre, 3 if cpu else 0, args.stride_by_subsampling,
                               warmup=warmup)

    # the headline: a time-based pre-warm, then --warmup untimed steps, then exactly --steps timed steps
    head_steps = max(1, args.steps if args.workload != "resnet18_b1" else max(3, args.steps // 50))
    head_warm = args.warmup if args.workload != "resnet18_b1" else max(1, args.warmup // 50)
    head = run(args.workload, head_steps, warmup=head_warm)
    if args.workload == "resnet18_b1":
        ms_per_step = head["ms_per_network"]
    else:
        ms_per_step = head["ms_per_layer"]
    cfg = {"workload": args.workload, "n": par.n, "gadget_digits": ctx.ndigits,
           "key_switching": head["key_switching"], "decrypts": head["decrypts"]}
    for k in ("layer", "n_o", "n_i", "batch", "G", "c_o", "c_i", "k", "image", "c_n", "terms", "multiply_accumulate", "layers", "stride"):
        if k in head:
            cfg[k] = head[k]
    out = {"metric": METRIC, "value": head["rotations_per_s"] if head["rotations_per_s"] else head["layers_per_s"],
           "unit": "rotations/s" if head["rotations_per_s"] else "layers/s", "n_gpus": 1, "steps": head_steps,
           "warmup": head_warm, "prewarm_ms": head["prewarm_ms"], "ms_per_step": ms_per_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
           "config": cfg, "layers_per_s": head["layers_per_s"],
           "ops_per_step": head.get("ops_per_layer") or head.get("ops_per_network"),
           "roofline": head["roofline"], "cpu_baseline": head["cpu_baseline"]}
    for k in ("inputs_per_s", "gazelle_schedule", "kernels", "per_layer", "ms_per_network_eager", "ms_per_network_graph_replay",
              "graph_replay_equals_eager", "ms_sum_of_layers_timed_alone", "networks_per_s"):
        if k in head:
            out[k] = head[k]
    if not args.no_configs:
        # the other benchmark configurations, each with its own roofline and oracle timing
        others = {}
        for name, steps in (("fc_16x128_b1", 200), ("fc_128x1024_b64", 200), ("fc_1000x2048_b64", 30),
                            ("conv_16x16x128_3x3x128_b16", 100), ("resnet18_b1", 5)):
            if name != args.workload:
                others[name] = run(name, steps)
        out["configs"] = others
        if not args.special_prime:
            # config 4 in the mode whose outputs decrypt (keys modulo q*P): a context of its own
            sp = wl.DEFAULT_SPECIAL
            ctx_s = binding.Context(sp.n, sp.q, sp.p, sp.gadget_bits, sp.special)
            others["conv_16x16x128_3x3x128_b16_special_prime"] = conv_config(
                ctx_s, ctx_s.keygen(0), D, torch, sp, wl.CONV_16x16_128_3x3, 50, args.prewarm_s, 0, special=True, compare=False)
            out["also"] = entry_points(ctx, sk, D, torch, par)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
