"""Benchmark of the hot path: one step = slz_pbs_batch + slz_keyswitch_batch(_prepared) over one batch of ciphertexts.

Prints ONE JSON line.  Headline workload: configuration 5 of the baseline, the largest single-GPU batch of the
128-bit-shaped parameter set (16 384 LWE ciphertexts, 64 lookup tables, n=742, k=1, N=2048, PBS base 2^23 x 1 level,
keyswitch base 2^3 x 5 levels); the object "per_config" of the same line carries a short run of every other parameter
set (configurations 1 to 4) with its own rates, roofline fractions and oracle check.  --config N times that
configuration alone.  Inputs are seeded
and synthetic and already resident in HBM when the timed region starts.  Key and ciphertext material for
the timed run is uniform random u64 words (what TFHE keys and ciphertexts look like; the kernels have no
data-dependent control flow); LUT polynomials come from slz_lut_encode.  The cpu_baseline leg runs the
CPU oracle on a bounded sample of the same inputs and also checks that the GPU's outputs for that sample
are bit-identical.
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

PEAK_ALU_TINSTR = 256 * 4 * 16 * 2.4e9 / 1e12      # 256 CUs x 4 SIMD16 x 2.4 GHz: FP64/INT32 lane-instructions per second


def alu_model_ops_per_pbs(p) -> float:
    """Algorithmic VALU lane-instructions of one PBS, from this op table:
    8 per butterfly (6 modular multiply + add + sub), 7 per pointwise multiply-accumulate, 3 per inverse
    post-scaling beyond the butterflies' share (6-instruction modular multiply per coefficient), 12 per
    decomposed coefficient (rotate, subtract, round, digit, convert) and 20 per CRT-lifted coefficient."""
    logN = p.N.bit_length() - 1
    R, C = (p.k + 1) * p.pbs_level, p.k + 1
    per_prime = (R + C) * (p.N // 2) * logN * 8 + R * C * p.N * 7 + C * p.N * 6
    per_cmux = 2 * per_prime + C * p.N * (12 + 4 * (p.pbs_level - 1)) + C * p.N * 20
    return float(p.n) * per_cmux


def bench_matmul_rns(args):
    """One step = one Matmul^RNS (the paper's Algorithm "Matmul^RNS") of an encrypted 8 x 28 by an encrypted 28 x 8 matrix
    (the paper's batch of 8 and the first dense layer of its 28-8-2 network) over the moduli {7, 11, 13}: 7 104 table
    lookups in three dependent rounds plus the leveled sums.  --gadget matmul_highres: the same product by
    MatmulHighRes^RNS over the 5-bit moduli {29, 31, 30}.  Key and ciphertext material is uniform random words."""
    import torch
    import synth
    import paper_2504_17785_amd as slz

    if args.gadget_params == "cfg3":
        p, max_batch = synth.CONFIGS[3], 256
    else:
        p = synth.Params(name="gadget_toy", n=4, k=1, N=2048, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8,
                         msg_bits=8, sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1, seed=0x6AD6E7)
        max_batch = 8192
    highres = args.gadget == "matmul_highres"
    a, b, c, m = 8, 28, 8, ((29, 31, 30) if highres else (7, 11, 13))
    k = len(m)
    if highres:     # residues, two bit chunks of X', four lookups per product, blocks of 7
        nblk = (b + 6) // 7
        lookups = k * (a * b + b * c) + 2 * k * a * b + 4 * k * a * b * c + k * a * c * nblk
        sub = k * (b + b) + 2 * k * b + 4 * k * b + k * nblk        # lookups behind one output entry
        rounds = 6 + nblk
    else:
        nblk = (b + 14) // 15
        lookups = k * (a * b + b * c) + k * a * b * c + k * a * c * nblk
        sub = k * (b + b) + k * b + k * nblk
        rounds = 2 + nblk
    torch.cuda.set_device(0)
    ctx = slz.Context(p, max_batch)
    R, C = (p.k + 1) * p.pbs_level, p.k + 1
    bsk = synth.raw_words(p, "raw_bsk", p.n * R * C * p.N).reshape(p.n, p.k + 1, p.pbs_level, C, p.N)
    ksk = synth.raw_words(p, "raw_ksk", p.k * p.N * p.ks_level * (p.n + 1)).reshape(p.k * p.N, p.ks_level, p.n + 1)
    x_cts = synth.raw_words(p, "raw_ct", a * b * (p.n + 1)).reshape(a, b, p.n + 1)
    w_cts = synth.raw_words(p, "raw_ct", b * c * (p.n + 1), a * b * (p.n + 1)).reshape(b, c, p.n + 1)
    d_std = slz.to_device_u64(bsk)
    d_bskp = ctx.bsk_prepare(d_std)
    del d_std
    d_ksk, d_x, d_w = slz.to_device_u64(ksk), slz.to_device_u64(x_cts), slz.to_device_u64(w_cts)
    d_luts = slz.to_device_u64((slz.matmul_highres_luts if highres else slz.matmul_rns_luts)(p, m, a, b, c))
    d_y = torch.empty((k, a, c, p.n + 1), dtype=torch.int64, device="cuda")
    for _ in range(args.warmup):
        ctx.matmul_rns(d_x, d_w, m, d_luts, d_bskp, d_ksk, out=d_y, highres=highres)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ctx.matmul_rns(d_x, d_w, m, d_luts, d_bskp, d_ksk, out=d_y, highres=highres)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    achieved = lookups * alu_model_ops_per_pbs(p) / (ms * 1e-3) / 1e12
    result = {
        "metric": "%s_lookups_per_s" % args.gadget, "value": lookups / (ms * 1e-3), "unit": "PBS+KS/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": "%s %dx%d by %dx%d over moduli %s at %s: %d lookups in %d dependent rounds" % (
            args.gadget, a, b, b, c, list(m), p.name, lookups, rounds), "path": ctx.path},
        "roofline": {"bound": "alu", "kernel": "blind rotation inside the lookups (whole gadget timed)", "achieved": achieved,
                     "peak": PEAK_ALU_TINSTR, "unit": "Tinstr/s", "frac": achieved / PEAK_ALU_TINSTR, "traffic": None},
    }
    if not args.no_cpu_baseline and args.gadget_params == "toy":
        # the oracle follows one output entry (row 0 of X, column 0 of W: every step of the algorithm, 1/64 of the work)
        import oracle
        from oracle import gadgets
        t1 = time.perf_counter()
        want = (gadgets.matmul_highres_encrypted if highres else gadgets.matmul_rns_encrypted)(p, x_cts[:1], w_cts[:, :1], m, bsk, ksk)
        t2 = time.perf_counter()
        got = slz.to_host_u64(d_y)[:, :1, :1]
        result["cpu_baseline"] = {"value": sub / (t2 - t1), "unit": "PBS+KS/s", "cores": min(oracle.num_threads(), k * b),
                                  "kind": "oracle", "sample": "output entry (0, 0) of the product: %d of the %d lookups" % (sub, lookups),
                                  "gpu_bit_exact_on_sample": bool(np.array_equal(got, want))}
    else:
        result["cpu_baseline"] = None       # one lookup at the 8-bit parameter set is 9e12 multiply-adds in the oracle
    print(json.dumps(result))


def bench_sign_rns(args):
    """One step = Sign_(-1,0,1)^RNS (RNS-to-MRNS conversion, top-digit lookup, final lookup) of --batch numbers (default 64:
    the 8 x 8 outputs of the product above) given as residues modulo {13, 15, 14}: 5 lookups per number in 4 dependent
    rounds.  Key and ciphertext material is uniform random words."""
    import torch
    import synth
    import paper_2504_17785_amd as slz

    if args.gadget_params == "cfg3":
        p, max_batch = synth.CONFIGS[3], 256
    else:
        p = synth.Params(name="gadget_toy", n=4, k=1, N=2048, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8,
                         msg_bits=8, sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1, seed=0x6AD6E7)
        max_batch = 8192
    m = (13, 15, 14)
    k = len(m)
    count = args.batch or 64
    shift = args.gadget == "shift2msbs"      # Shift2MSBs^+- to Gamma = 8 signed bits (gamma = 7, w = 4) instead of the sign alone
    conv = count * k * (k - 1) // 2
    if shift:
        # sign, |x|, then Shift2MSBs^+: conversion, bit positions, maximum tree (one lookup per pair), codes, shifts; sign back
        lookups = (conv + 2 * count) + k * count + (conv + k * count + (k * count - 1) + k + k * count) + count
        tree = (k * count - 1).bit_length()
        rounds = (k - 1 + 2) + 1 + (k - 1 + 1 + tree + 1 + 1) + 1
    else:
        lookups = conv + 2 * count
        rounds = k + 1
    torch.cuda.set_device(0)
    ctx = slz.Context(p, max_batch)
    R, C = (p.k + 1) * p.pbs_level, p.k + 1
    bsk = synth.raw_words(p, "raw_bsk", p.n * R * C * p.N).reshape(p.n, p.k + 1, p.pbs_level, C, p.N)
    ksk = synth.raw_words(p, "raw_ksk", p.k * p.N * p.ks_level * (p.n + 1)).reshape(p.k * p.N, p.ks_level, p.n + 1)
    x_cts = synth.raw_words(p, "raw_ct", k * count * (p.n + 1)).reshape(k, count, p.n + 1)
    d_std = slz.to_device_u64(bsk)
    d_bskp = ctx.bsk_prepare(d_std)
    del d_std
    d_ksk, d_x = slz.to_device_u64(ksk), slz.to_device_u64(x_cts)
    d_luts = slz.to_device_u64(slz.shift2msbs_luts(p, m, 4, 7) if shift else slz.rns_luts(p, m, -1, 0, 1))
    d_s = torch.empty((count, p.n + 1), dtype=torch.int64, device="cuda")

    def run():
        if shift:
            return ctx.shift2msbs(d_x, m, 4, 7, d_luts, d_bskp, d_ksk, signed=True)
        return ctx.sign_rns(d_x, m, d_luts, d_bskp, d_ksk, out=d_s), None

    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        d_s, d_shift = run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    achieved = lookups * alu_model_ops_per_pbs(p) / (ms * 1e-3) / 1e12
    result = {
        "metric": "%s_lookups_per_s" % args.gadget, "value": lookups / (ms * 1e-3), "unit": "PBS+KS/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": "%s of %d numbers over moduli %s at %s: %d lookups in %d dependent rounds" % (
            args.gadget, count, list(m), p.name, lookups, rounds), "path": ctx.path},
        "roofline": {"bound": "alu", "kernel": "blind rotation inside the lookups (whole gadget timed)", "achieved": achieved,
                     "peak": PEAK_ALU_TINSTR, "unit": "Tinstr/s", "frac": achieved / PEAK_ALU_TINSTR, "traffic": None},
    }
    if not args.no_cpu_baseline and args.gadget_params == "toy":
        import oracle
        from oracle import gadgets
        if shift:       # the maximum couples all numbers: the oracle follows the whole tensor
            t1 = time.perf_counter()
            want, want_shift = gadgets.shift2msbs_pm_encrypted(p, x_cts, m, 4, 8, bsk, ksk)
            t2 = time.perf_counter()
            result["cpu_baseline"] = {"value": lookups / (t2 - t1), "unit": "PBS+KS/s", "cores": oracle.num_threads(), "kind": "oracle",
                                      "sample": "the whole tensor of %d numbers" % count,
                                      "gpu_bit_exact_on_sample": bool(np.array_equal(slz.to_host_u64(d_s), want)
                                                                      and np.array_equal(slz.to_host_u64(d_shift), want_shift))}
        else:
            sub = min(count, 16)
            t1 = time.perf_counter()
            want = gadgets.sign_rns_encrypted(p, x_cts[:, :sub], m, -1, 0, 1, bsk, ksk)
            t2 = time.perf_counter()
            result["cpu_baseline"] = {"value": sub * (k * (k - 1) // 2 + 2) / (t2 - t1), "unit": "PBS+KS/s",
                                      "cores": min(oracle.num_threads(), (k - 1) * sub), "kind": "oracle",
                                      "sample": "the first %d of the %d numbers" % (sub, count),
                                      "gpu_bit_exact_on_sample": bool(np.array_equal(slz.to_host_u64(d_s)[:sub], want))}
    else:
        result["cpu_baseline"] = None       # one lookup at the 8-bit parameter set is 9e12 multiply-adds in the oracle
    print(json.dumps(result))


def bench_loss(args):
    """--gadget loss_deriv: one step = IntCELossDeriv of a batch of 8 samples with 3 classes (Gamma = 7, kappa = 2, the largest
    level whose packed lookup fits 8 bits): 5 lookups per entry in 5 dependent rounds.  --gadget weight_update: one step = the
    clipped update of the 28 x 8 + 8 x 2 = 240 weights of the paper's largest network (alpha = 6), one lookup per weight.
    --gadget-params wide: the paper's own kappa = 4 and alpha = 8 on an 11-bit message space (N = 65536).
    Key and ciphertext material is uniform random words."""
    import torch
    import synth
    import paper_2504_17785_amd as slz

    if args.gadget_params == "cfg3":
        p, max_batch = synth.CONFIGS[3], 256
    elif args.gadget_params == "wide":
        # the shape of a parameter set for 11-bit lookups (the paper's kappa = 4 and alpha = 8): configuration 3 with twice
        # the polynomial size, the largest the large-N path takes
        p, max_batch = synth.CONFIGS[3].with_(name="wide_n1024_N65536", N=65536, msg_bits=11), 128
    else:
        p = synth.Params(name="gadget_toy", n=4, k=1, N=2048, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8,
                         msg_bits=8, sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1, seed=0x6AD6E7)
        max_batch = 8192
    loss = args.gadget == "loss_deriv"
    wide = args.gadget_params == "wide"
    a, b, Gamma, kappa, alpha = 8, 3, 7, (4 if wide else 2), (8 if wide else 6)
    count = a * b if loss else (args.batch or 240)
    lookups, rounds = (5 * count, 5) if loss else (count, 1)
    torch.cuda.set_device(0)
    ctx = slz.Context(p, max_batch)
    R, C = (p.k + 1) * p.pbs_level, p.k + 1
    bsk = synth.raw_words(p, "raw_bsk", p.n * R * C * p.N).reshape(p.n, p.k + 1, p.pbs_level, C, p.N)
    ksk = synth.raw_words(p, "raw_ksk", p.k * p.N * p.ks_level * (p.n + 1)).reshape(p.k * p.N, p.ks_level, p.n + 1)
    cts = synth.raw_words(p, "raw_ct", 2 * count * (p.n + 1)).reshape(2, count, p.n + 1)
    d_std = slz.to_device_u64(bsk)
    d_bskp = ctx.bsk_prepare(d_std)
    del d_std
    d_ksk = slz.to_device_u64(ksk)
    if loss:
        d_x, d_y = slz.to_device_u64(cts[0].reshape(a, b, p.n + 1)), slz.to_device_u64(cts[1].reshape(a, b, p.n + 1))
        d_luts = slz.to_device_u64(slz.loss_luts(p, b, Gamma, kappa))
        run = lambda: ctx.int_ce_loss_deriv(d_x, d_y, Gamma, kappa, d_luts, d_bskp, d_ksk)
    else:
        d_x, d_y = slz.to_device_u64(cts[0]), slz.to_device_u64(cts[1])
        d_luts = slz.to_device_u64(slz.weight_update_luts(p, alpha))
        run = lambda: ctx.weight_update(d_x, d_y, alpha, d_luts, d_bskp, d_ksk)
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        d_out = run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    achieved = lookups * alu_model_ops_per_pbs(p) / (ms * 1e-3) / 1e12
    what = ("IntCELossDeriv of %d x %d logits (Gamma %d, kappa %d)" % (a, b, Gamma, kappa)) if loss else \
        ("clipped update of %d weights (alpha %d)" % (count, alpha))
    result = {
        "metric": "%s_lookups_per_s" % args.gadget, "value": lookups / (ms * 1e-3), "unit": "PBS+KS/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": "%s at %s: %d lookups in %d dependent rounds" % (what, p.name, lookups, rounds), "path": ctx.path},
        "roofline": {"bound": "alu", "kernel": "blind rotation inside the lookups (whole gadget timed)", "achieved": achieved,
                     "peak": PEAK_ALU_TINSTR, "unit": "Tinstr/s", "frac": achieved / PEAK_ALU_TINSTR, "traffic": None},
    }
    if not args.no_cpu_baseline and args.gadget_params == "toy":
        import oracle
        from oracle import loss as oloss
        t1 = time.perf_counter()
        if loss:        # the row sums couple the classes: the oracle follows the first two samples
            sub = 2
            want = oloss.int_ce_loss_deriv_encrypted(p, cts[0].reshape(a, b, -1)[:sub], cts[1].reshape(a, b, -1)[:sub], Gamma, kappa, bsk, ksk)
            done, same = 5 * sub * b, np.array_equal(slz.to_host_u64(d_out)[:sub], want)
        else:
            sub = min(count, 32)
            want = oloss.weight_update_encrypted(p, cts[0][:sub], cts[1][:sub], alpha, bsk, ksk)
            done, same = sub, np.array_equal(slz.to_host_u64(d_out)[:sub], want)
        t2 = time.perf_counter()
        result["cpu_baseline"] = {"value": done / (t2 - t1), "unit": "PBS+KS/s", "cores": min(oracle.num_threads(), done // (5 if loss else 1)),
                                  "kind": "oracle", "sample": "the first %d %s" % (sub, "samples" if loss else "weights"),
                                  "gpu_bit_exact_on_sample": bool(same)}
    else:
        result["cpu_baseline"] = None       # one lookup at the 8-bit parameter set is 9e12 multiply-adds in the oracle
    print(json.dumps(result))


# ---- the PBS + keyswitch step of one configuration ---------------------------------------------------------------------

PATH_SOURCES = {       # sources of the dominant kernel of each path (for the check that a stored traffic figure is current)
    "fused_n2048": ("slz_fused.hip", "slz_wave_ntt.h", "slz_modarith.h"),
    "fused_n512": ("slz_fused_n512.hip", "slz_wave_ntt.h", "slz_modarith.h"),
    "three_pass_large_n": ("slz_bign.hip", "slz_wave_ntt.h", "slz_modarith.h"),
}


def kernel_source_hash(path: str):
    import hashlib
    files = PATH_SOURCES.get(path)
    if not files:
        return None
    h = hashlib.sha256()
    for f in files:
        with open(os.path.join(ROOT, "paper_2504_17785_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def stored_traffic(path: str, workload: str):
    """HBM bytes per launch of the dominant kernel from the rocprofv3 FETCH_SIZE / WRITE_SIZE passes recorded in
    profiles/hbm_traffic.txt (already scaled by the copy-kernel calibration).  None when no pass was recorded for this
    path and workload, or when the kernel's sources have changed since (the line carries their hash)."""
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.txt")) as fh:
            for line in fh:
                f = line.split()
                if len(f) >= 6 and not line.startswith("#") and f[0] == path and f[1] == workload:
                    return float(f[2]) + float(f[3]) if f[5] == kernel_source_hash(path) else None
    except OSError:
        pass
    return None


def host_info():
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count()
    return {"nproc": os.cpu_count(), "usable_cpus": usable, "cpu_model": model}


class Workload:
    """Keys, tables and ciphertexts of one configuration, resident in HBM, and the launch of one step."""

    def __init__(self, cfg, args, batch=0):
        import torch
        import synth
        import paper_2504_17785_amd as slz
        self.slz, self.synth, self.torch, self.cfg = slz, synth, torch, cfg
        p = synth.CONFIGS[cfg]
        if args.override:       # another shape with the configuration's tables and message space, e.g. N=4096,pbs_base_log=22,n=256
            kw = {k.strip(): int(v) for k, v in (item.split("=") for item in args.override.split(","))}
            p = p.with_(name="%s+%s" % (p.name, args.override), **kw)
        self.p = p
        self.batch = batch = batch or p.batch
        self.ctx = ctx = slz.Context(p, batch)
        if args.generic:
            ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
        if args.no_pacing:
            ctx.set_option(slz.SLZ_OPT_FUSED_PACING, 0)
        if args.large_n_lanes:
            ctx.set_option(slz.SLZ_OPT_LARGE_N_LANES, args.large_n_lanes)
        if args.large_n_block:
            ctx.set_option(slz.SLZ_OPT_LARGE_N_BLOCK, args.large_n_block)
        R, C = (p.k + 1) * p.pbs_level, p.k + 1
        self.bsk = synth.raw_words(p, "raw_bsk", p.n * R * C * p.N).reshape(p.n, p.k + 1, p.pbs_level, C, p.N)
        self.ksk = synth.raw_words(p, "raw_ksk", p.k * p.N * p.ks_level * (p.n + 1)).reshape(p.k * p.N, p.ks_level, p.n + 1)
        cts = synth.raw_words(p, "raw_ct", batch * (p.n + 1)).reshape(batch, p.n + 1)
        self.luts = slz.lut_encode(p, synth.config_tables(cfg))
        self.lut_idx = synth.config_lut_idx(cfg, batch)
        d_bsk_std = slz.to_device_u64(self.bsk)
        self.d_bskp = ctx.bsk_prepare(d_bsk_std)
        torch.cuda.synchronize()
        del d_bsk_std
        self.d_ksk = slz.to_device_u64(self.ksk)
        # the keyswitching key in the matrix-core contraction's operand form (one-off, untimed, like the bootstrapping key);
        # parameter sets or modes without that contraction keep the standard key
        self.d_kskp = None
        if p.ks_base_log <= 8 and (p.k * p.N) % 32 == 0 and not args.generic and not args.ksk_standard:
            self.d_kskp = ctx.ksk_prepare(self.d_ksk)
        self.d_cts = slz.to_device_u64(cts)
        self.d_luts = slz.to_device_u64(self.luts)
        self.d_idx = torch.from_numpy(self.lut_idx.astype(np.int32)).cuda()
        self.d_big = torch.empty((batch, p.k * p.N + 1), dtype=torch.int64, device="cuda")
        self.d_small = torch.empty((batch, p.n + 1), dtype=torch.int64, device="cuda")
        # configuration 4 adds the leveled linear part in front: per modulus, 32 x 784 ciphertexts times a clear 784 x 128 matrix
        self.lin = None
        if cfg == 4 and batch == p.batch and not args.override:
            G, J, O = synth.CFG4_BATCH, synth.CFG4_IN, synth.CFG4_OUT
            _, ws = synth.cfg4_clear_inputs()
            lin_cts = [slz.to_device_u64(synth.raw_words(p, "lin_mask", G * J * (p.n + 1), r * G * J * (p.n + 1)).reshape(G, J, p.n + 1))
                       for r in range(3)]
            lin_w = [torch.from_numpy(ws[r]).cuda() for r in range(3)]
            self.lin = (lin_cts, lin_w, self.d_cts.view(3, G, O, p.n + 1))
        torch.cuda.synchronize()

    def lincomb(self):
        if self.lin is not None:
            for r in range(3):
                self.ctx.lwe_lincomb_batch(self.lin[0][r], self.lin[1][r], out=self.lin[2][r])

    def keyswitch(self):
        if self.d_kskp is not None:
            self.ctx.keyswitch_batch_prepared(self.d_big, self.d_kskp, out=self.d_small)
        else:
            self.ctx.keyswitch_batch(self.d_big, self.d_ksk, out=self.d_small)

    def step(self):
        self.lincomb()
        self.ctx.pbs_batch(self.d_cts, self.d_luts, self.d_idx, self.d_bskp, out=self.d_big)
        self.keyswitch()

    def run(self, steps, warmup):
        """W untimed steps, then exactly K timed ones; per-call HIP events on the launch stream give the kernel split."""
        torch = self.torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
        t0 = time.perf_counter()
        for k in range(steps):
            ev[k][0].record()
            self.lincomb()
            ev[k][1].record()
            self.ctx.pbs_batch(self.d_cts, self.d_luts, self.d_idx, self.d_bskp, out=self.d_big)
            ev[k][2].record()
            self.keyswitch()
            ev[k][3].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return {"ms_per_step": wall * 1e3 / steps,
                "pbs_ms": float(np.mean([e[1].elapsed_time(e[2]) for e in ev])),
                "ks_ms": float(np.mean([e[2].elapsed_time(e[3]) for e in ev])),
                "lin_ms": float(np.mean([e[0].elapsed_time(e[1]) for e in ev])) if self.lin is not None else None}

    def report(self, t, generic=False):
        """Rates and roofline fractions of one timed run (`t` from run())."""
        p, batch, synth = self.p, self.batch, self.synth
        achieved = alu_model_ops_per_pbs(p) * batch / (t["pbs_ms"] * 1e-3) / 1e12
        prepared_bytes = self.ctx.bsk_prepared_bytes()
        r = {"workload": "%s: batch %d, n=%d, k=%d, N=%d, PBS 2^%d x %d, KS 2^%d x %d" % (
                 p.name, batch, p.n, p.k, p.N, p.pbs_base_log, p.pbs_level, p.ks_base_log, p.ks_level),
             "path": self.ctx.path,
             "pbs_plus_keyswitch_per_s": batch / (t["ms_per_step"] * 1e-3),
             "pbs_per_s": batch / (t["pbs_ms"] * 1e-3), "keyswitch_per_s": batch / (t["ks_ms"] * 1e-3),
             "ms_per_step": t["ms_per_step"], "pbs_ms": t["pbs_ms"], "keyswitch_ms": t["ks_ms"], "lincomb_ms": t["lin_ms"],
             "keyswitch_key": "prepared" if self.d_kskp is not None else "standard",
             "bsk_prepared_bytes": prepared_bytes,
             "bsk_stream_GBps_min": prepared_bytes / (t["pbs_ms"] * 1e-3) / 1e9,
             "roofline": {"bound": "alu", "kernel": "blind rotation (slz_pbs_batch)", "achieved": achieved,
                          "peak": PEAK_ALU_TINSTR, "unit": "Tinstr/s", "frac": achieved / PEAK_ALU_TINSTR,
                          "traffic": stored_traffic(self.ctx.path, "%s_batch%d" % (p.name, batch))}}
        # the same launch against the memory roofline, from the measured traffic past the L2s (large N: the accumulators and the
        # intermediates of the three passes move through memory every step, and this bound is as close as the arithmetic one)
        traffic = r["roofline"]["traffic"]
        if traffic is not None:
            gbps = traffic / (t["pbs_ms"] * 1e-3) / 1e9
            r["memory_roofline"] = {"bound": "hbm", "achieved": gbps, "peak": 8000.0, "unit": "GB/s", "frac": gbps / 8000.0,
                                    "note": "measured bytes past the L2s (not algorithmic bytes) / launch time"}
        # secondary kernels against their own bounds (whole entry point, helper kernels and launch gaps included)
        kN = p.k * p.N
        if p.ks_base_log <= 8 and kN % 32 == 0 and not generic and batch >= 16:
            ks_ops = 2.0 * batch * kN * p.ks_level * (p.n + 1) * 8          # int8 multiply-adds over the eight byte planes, x2
            ks_pops = ks_ops / (t["ks_ms"] * 1e-3) / 1e15
            r["keyswitch_roofline"] = {"bound": "mfma", "dtype": "int8", "achieved": ks_pops, "peak": 5.0, "unit": "POP/s",
                                       "frac": ks_pops / 5.0}
        else:       # a handful of ciphertexts: the key streams from HBM once
            ks_bytes = float(kN) * p.ks_level * (p.n + 1) * 8 + batch * (kN + 1 + p.n + 1) * 8.0
            r["keyswitch_roofline"] = {"bound": "hbm", "achieved": ks_bytes / (t["ks_ms"] * 1e-3) / 1e9, "peak": 8000.0, "unit": "GB/s",
                                       "frac": ks_bytes / (t["ks_ms"] * 1e-3) / 8e12}
        if t["lin_ms"] is not None:
            G, J, O = synth.CFG4_BATCH, synth.CFG4_IN, synth.CFG4_OUT
            lin_bytes = 3.0 * G * (J + O) * (p.n + 1) * 8             # ciphertext words in, sums out (weights are negligible)
            r["lincomb_roofline"] = {"bound": "hbm", "achieved": lin_bytes / (t["lin_ms"] * 1e-3) / 1e9, "peak": 8000.0,
                                     "unit": "GB/s", "frac": lin_bytes / (t["lin_ms"] * 1e-3) / 8e12}
        return r

    def oracle_sample(self, seconds=20.0):
        """The CPU oracle on a bounded sample of the same inputs (timed: the baseline), and the GPU's outputs for that
        sample compared with it bit for bit.  Outputs of the last step() must still be in d_big / d_small."""
        import oracle
        slz, p, batch = self.slz, self.p, self.batch
        threads = oracle.num_threads()
        macs_per_pbs = p.n * (p.k + 1) ** 2 * p.pbs_level * float(p.N) ** 2
        info = host_info()
        if macs_per_pbs > 1e12:
            return self._oracle_induction(oracle, threads, info)
        budget_macs = 0.9e9 * seconds * threads                    # about 0.9 GMAC/s per core, schoolbook
        sample = int(max(1, min(batch, threads * max(1, int(budget_macs / threads / macs_per_pbs)))))
        idx = np.linspace(0, batch - 1, sample).astype(np.int64)
        cts_h = slz.to_host_u64(self.d_cts)     # configuration 4: the PBS inputs are the GPU's own linear combinations
        t1 = time.perf_counter()
        o_big = oracle.pbs_batch(p, cts_h[idx], self.luts, self.lut_idx[idx], self.bsk)
        t2 = time.perf_counter()
        o_small = oracle.keyswitch_batch(p, o_big, self.ksk)
        t3 = time.perf_counter()
        g_big = slz.to_host_u64(self.d_big)[idx]
        g_small = slz.to_host_u64(self.d_small)[idx]
        used = min(threads, sample)
        return {"value": sample / (t3 - t1), "unit": "PBS+KS/s", "cores": used, "kind": "oracle",
                "sample": "%d of the %d ciphertexts (evenly spaced), full PBS + keyswitch each" % (sample, batch),
                "omp_threads": threads, **info,
                "pbs_s_per_ct_per_core": (t2 - t1) * used / sample,
                "keyswitch_s_per_ct_per_core": (t3 - t2) * used / sample,
                "gpu_bit_exact_on_sample": bool(np.array_equal(g_big, o_big) and np.array_equal(g_small, o_small))}

    def _oracle_induction(self, oracle, threads, info):
        """Parameter sets where one oracle bootstrapping is hours of schoolbook products: the oracle applies ONE CMux step
        (the last one) to the GPU's accumulators after n - 1 steps, which must give the GPU's accumulators after n steps
        word for word; the keyswitch of the sampled outputs is compared in full.  Rate: timed CMux steps x n."""
        import concurrent.futures
        slz, p, batch, torch = self.slz, self.p, self.batch, self.torch
        sample = min(batch, threads)
        idx = np.linspace(0, batch - 1, sample).astype(np.int64)
        i = p.n - 1
        before = slz.to_host_u64(self.ctx.blind_rotate_batch(self.d_cts, self.d_luts, self.d_idx, self.d_bskp, i))[idx]
        after = slz.to_host_u64(self.ctx.blind_rotate_batch(self.d_cts, self.d_luts, self.d_idx, self.d_bskp, i + 1))[idx]
        cts_h = slz.to_host_u64(self.d_cts)
        rot = [oracle.modswitch(int(cts_h[c, i]), p.N) for c in idx]
        t1 = time.perf_counter()
        with concurrent.futures.ThreadPoolExecutor(sample) as ex:       # the C oracle runs outside the interpreter lock
            stepped = list(ex.map(lambda q: oracle.cmux(p, before[q], self.bsk[i], rot[q]), range(sample)))
        t2 = time.perf_counter()
        g_big = slz.to_host_u64(self.d_big)[idx]
        same = all(np.array_equal(stepped[q], after[q]) for q in range(sample))
        same = same and np.array_equal(g_big, np.stack([oracle.sample_extract(p, a) for a in after]))
        t3 = time.perf_counter()
        o_small = oracle.keyswitch_batch(p, g_big, self.ksk)
        t4 = time.perf_counter()
        same = same and np.array_equal(slz.to_host_u64(self.d_small)[idx], o_small)
        pbs_s = (t2 - t1) * p.n                                      # `sample` bootstrappings at this rate, in parallel
        return {"value": sample / (pbs_s + (t4 - t3)), "unit": "PBS+KS/s", "cores": sample, "kind": "oracle",
                "sample": "the last of the %d CMux steps on %d of the %d ciphertexts (the oracle continues from the GPU's "
                          "accumulators after %d steps; rate = timed step x %d), full keyswitch of those outputs" % (
                              p.n, sample, batch, i, p.n),
                "omp_threads": threads, **info,
                "pbs_s_per_ct_per_core": pbs_s, "keyswitch_s_per_ct_per_core": (t4 - t3) * min(threads, sample) / sample,
                "gpu_bit_exact_on_sample": bool(same)}


PER_CONFIG_RUNS = {1: (50, 5), 2: (5, 2), 3: (2, 1), 4: (3, 1)}     # (steps, warm-ups) of the other parameter sets in the default run


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=0,
                    help="time this configuration only (default: configuration 5 as the headline plus a per_config object "
                         "with configurations 1 to 4)")
    ap.add_argument("--batch", type=int, default=0, help="override the configuration's batch size")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="default run: skip configurations 1 to 4")
    ap.add_argument("--generic", action="store_true", help="force the generic multi-kernel path")
    ap.add_argument("--override", default="", help="comma-separated parameter overrides of the configuration, e.g. N=4096,pbs_base_log=22,n=256")
    ap.add_argument("--no-pacing", action="store_true", help="fused N = 2048 kernel: let the workgroups run free between ciphertexts")
    ap.add_argument("--large-n-block", type=int, default=0, help="large-N path: block size of the row pass, 1024 or 2048")
    ap.add_argument("--large-n-lanes", type=int, default=0, help="large-N path: 1 = one chunk at a time, 2 = two half chunks on two streams")
    ap.add_argument("--ksk-standard", action="store_true",
                    help="keyswitch with the standard key (slz_keyswitch_batch) instead of the prepared one")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain device copy of 256 MiB (a known-size kernel to scale FETCH_SIZE/WRITE_SIZE by)")
    ap.add_argument("--gadget", choices=["matmul_rns", "matmul_highres", "sign_rns", "shift2msbs", "loss_deriv", "weight_update"], default=None,
                    help="time a gadget built on the lookup primitive instead of the PBS + keyswitch step")
    ap.add_argument("--gadget-params", choices=["cfg3", "toy", "wide"], default="cfg3",
                    help="the 8-bit parameter set of configuration 3, the toy set the oracle can follow, or (loss_deriv and "
                         "weight_update only) an 11-bit set of twice configuration 3's polynomial size")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only (this build has no multi-GPU path); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.gadget in ("matmul_rns", "matmul_highres"):
        return bench_matmul_rns(args)
    if args.gadget in ("sign_rns", "shift2msbs"):
        return bench_sign_rns(args)
    if args.gadget in ("loss_deriv", "weight_update"):
        return bench_loss(args)

    import torch
    torch.cuda.set_device(0)
    headline = args.config or 5
    wl = Workload(headline, args, args.batch)
    if args.calib_copy:
        src = torch.ones(256 * 1024 * 1024 // 8, dtype=torch.int64, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    t = wl.run(args.steps, args.warmup)
    rep = wl.report(t, args.generic)
    result = {
        "metric": "pbs_plus_keyswitch_per_s", "value": rep["pbs_plus_keyswitch_per_s"], "unit": "PBS+KS/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": t["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64", "data": "synthetic",
        "config": {"workload": rep["workload"], "path": rep["path"]},
    }
    for key in ("pbs_per_s", "keyswitch_per_s", "pbs_ms", "keyswitch_ms", "lincomb_ms", "bsk_prepared_bytes", "bsk_stream_GBps_min",
                "roofline", "memory_roofline", "keyswitch_roofline", "lincomb_roofline"):
        if key in rep:
            result[key] = rep[key]
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = wl.oracle_sample(30.0)
    del wl
    torch.cuda.empty_cache()

    # ---- the other parameter sets, each with its own short run and its own oracle sample -------------------------------
    if not args.config and not args.no_per_config and not args.batch and not args.override:
        per = {}
        for cfg, (steps, warmup) in PER_CONFIG_RUNS.items():
            w = Workload(cfg, args)
            tt = w.run(steps, warmup)
            e = w.report(tt, args.generic)
            e["steps"], e["warmup"] = steps, warmup
            if not args.no_cpu_baseline:
                e["cpu_baseline"] = w.oracle_sample(6.0)
                e["gpu_bit_exact_on_sample"] = e["cpu_baseline"]["gpu_bit_exact_on_sample"]
            per["cfg%d" % cfg] = e
            del w
            torch.cuda.empty_cache()
        result["per_config"] = per
    print(json.dumps(result))


if __name__ == "__main__":
    main()
