#!/usr/bin/env python3
"""Benchmark of the layer-wise quantization solve on one MI355X.

A step is one pass of the whole hot path over one synthetic layer:
Hessian accumulation -> damped Cholesky factor of the inverse -> blocked
column quantization -> layer error, with all inputs resident in HBM.
Prints ONE JSON line: metric / value / unit (columns quantized per second for the whole step),
ms_per_step and the per-call times, the Hessian rate, a "roofline" object for the dominant
kernel and a "cpu_baseline" object (the oracle timed on a sample of the same layer).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C3 --layer 1] [--no-cpu-baseline]

Default workload: the 4096 x 11008 down projection of the MLP pair (the widest single layer of
the 7B shape, the one the metric's columns/s is quoted on).  --config C2 / C4 / C1 and --layer
select the other layers; --config C5 times the seven linears of a decoder block back to back in
one timed region.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_F64_TFLOPS = 78.6      # MI355X float64 (vector and matrix)
HBM_GBPS = 8000.0

# HBM bytes per launch of the dominant kernel (Hessian main kernel).  NOT measured by this run:
# copied from two separate rocprofv3 --pmc runs of this file (FETCH_SIZE, then WRITE_SIZE), each
# scaled by what the same counter reads for a plain 1 GiB device copy (--copy-calibration):
# FETCH_SIZE reads 524288 per GiB read (factor 2 KiB per count), WRITE_SIZE 1048576 per GiB written
# (1 KiB per count).  The profile file that holds the run is named beside the number; None for
# workloads that were not profiled.
MEASURED_TRAFFIC_BYTES = {
    "C2:attn_proj": (3.483e6 * 2048 + 5.222e5 * 1024, "profiles/hessian_C2_hbm_traffic.txt"),
    "C3:down_proj": (3.565e7 * 2048 + 1.050e6 * 1024, "profiles/hessian_C3_down_hbm_traffic.txt"),
}


def log(msg):
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def host_cpu_info():
    """(logical CPUs the OS shows, CPUs this process may run on, physical cores from /proc/cpuinfo or None)."""
    logical = os.cpu_count() or 1
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = logical
    physical = None
    try:
        cores = set()
        phys = core = None
        for line in open("/proc/cpuinfo"):
            if line.startswith("physical id"):
                phys = line.split(":")[1].strip()
            elif line.startswith("core id"):
                core = line.split(":")[1].strip()
            elif not line.strip():
                if phys is not None and core is not None:
                    cores.add((phys, core))
                phys = core = None
        physical = len(cores) or None
    except OSError:
        pass
    return logical, usable, physical


def cpu_baseline(cfg, spec, seed, full_factor=True):
    """The oracle, as it stands, on a bounded sample of the same layer: the Hessian over a prefix of
    the tokens, the factor of the layer's full n x n matrix (or, with full_factor False, of its leading
    4096 x 4096 block, scaled by the cube of the size ratio), the solve and the error on the first rows.
    Each stage is timed on its own; the stage times are scaled linearly in tokens / rows to the full
    layer and added.  Reported in the metric's unit, columns per second for the whole step."""
    import numpy as np
    from threadpoolctl import threadpool_info

    import ptq_workloads as wl
    from oracle import ptq_oracle as orc

    t_s = min(spec.t, 16384)
    rows_s = min(spec.m, 256)
    Ws = wl.gen_weight(spec, seed)
    X64 = wl.to_f64(wl.gen_activations(spec, seed, 0, t_s))
    W64 = wl.to_f64(Ws)[:rows_s]
    t0 = time.perf_counter()
    H = orc.hessian(X64)
    t1 = time.perf_counter()
    log(f"cpu baseline: oracle Hessian over {t_s} tokens {t1 - t0:.1f} s")
    nf = spec.n if (full_factor or spec.n <= 4096) else 4096
    Hd, dead = orc.damp(H[:nf, :nf], cfg.damps[0])
    Uf = orc.inverse_cholesky_upper(Hd)
    t2 = time.perf_counter()
    log(f"cpu baseline: oracle factor of {nf} x {nf} {t2 - t1:.1f} s")
    factor_s = (t2 - t1) * (spec.n / nf) ** 3
    if nf == spec.n:
        U = Uf
    else:  # the solve needs some upper factor of the right size: the sampled one, extended by the identity
        U = np.eye(spec.n)
        U[:nf, :nf] = Uf
        dead = np.zeros(spec.n, dtype=bool)
    out = orc.quantize_layer(W64, U, cfg.bits, cfg.group, dead=dead)
    t3 = time.perf_counter()
    log(f"cpu baseline: oracle solve of {rows_s} rows {t3 - t2:.1f} s")
    orc.layer_error(W64, out["Wq"], H)
    t4 = time.perf_counter()
    est = (t1 - t0) * spec.t / t_s + factor_s + (t3 - t2) * spec.m / rows_s + (t4 - t3) * spec.m / rows_s
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    logical, usable, physical = host_cpu_info()
    return {
        "value": spec.n / est, "unit": "columns/s", "cores": int(min(threads, usable)), "kind": "oracle",
        "sample": (f"{t_s} of {spec.t} tokens for H, "
                   + (f"the full {spec.n}x{spec.n} factor" if nf == spec.n else
                      f"the factor of the leading {nf}x{nf} block scaled by ({spec.n}/{nf})^3")
                   + f", {rows_s} of {spec.m} rows for solve and error; stage times scaled linearly in tokens / rows "
                     f"to the full layer and added (measured: H {t1 - t0:.2f}s, factor {t2 - t1:.2f}s, "
                     f"solve {t3 - t2:.2f}s, error {t4 - t3:.2f}s)"),
        "est_seconds_full_layer": est,
        "measured_seconds": {"hessian": t1 - t0, "factor": t2 - t1, "solve": t3 - t2, "layer_error": t4 - t3},
        "blas_threads": int(threads), "host_logical_cpus": logical, "host_usable_cpus": usable,
        "host_physical_cores": physical,
    }


def single_block_us_per_column(ptq, bits, group, reps=30):
    """Time per column of the column walk where the call holds nothing else: 16 rows (one workgroup)
    and a layer that is a single block, so that there is no lazy update; a 256-column call minus a
    128-column call removes the launch.  It contains the walk, the in-block pushes and the block's
    set-up and outputs, so it is an upper estimate of the walk's share.  Microseconds per column."""
    import torch

    from paper_2601_19675_amd import binding
    gen = torch.Generator(device="cuda").manual_seed(7)
    times = {}
    for n in (128, 256):
        W = torch.randn((16, n), device="cuda", generator=gen) * 0.02
        U = torch.triu(torch.randn((n, n), dtype=torch.float64, device="cuda", generator=gen) * 0.01, 1)
        U += torch.eye(n, dtype=torch.float64, device="cuda")
        g = min(group, n)
        codes = torch.empty((16, n), dtype=torch.uint8, device="cuda")
        scales = torch.empty((16, n // g), dtype=torch.float32, device="cuda")
        zeros = torch.empty((16, n // g), dtype=torch.uint8, device="cuda")
        ws = torch.empty(max(256, ptq.ptq_workspace_bytes(binding.OP_QUANTIZE, 16, n, 0, n)), dtype=torch.uint8, device="cuda")
        runs = []
        for k in range(reps + 3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            ptq.ptq_quantize_layer(W, U, None, bits, g, n, codes, scales, zeros, None, None, ws)
            e1.record()
            torch.cuda.synchronize()
            if k >= 3:
                runs.append(e0.elapsed_time(e1))
        times[n] = sorted(runs)[len(runs) // 2]
    return 1e3 * (times[256] - times[128]) / 128.0


def lopro_timings(ptq, W, H, m, n, ws, b_I=256, b_H=256, reps=10):
    """LoPRo's pre-conditioning kernels on the benchmark layer: all memory-bound; GB/s are algorithmic
    bytes (each operand read once, each result written once) over the event-bracketed call."""
    import torch
    perm = torch.empty(n, dtype=torch.int32, device="cuda")
    Rr = torch.empty((m, n), dtype=torch.float64, device="cuda")
    back = torch.empty_like(Rr)
    Hr = torch.empty((n, n), dtype=torch.float64, device="cuda")
    esz = W.element_size()

    def timed(f):
        for _ in range(2):
            f()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    calls = {
        "column_order": (lambda: ptq.ptq_lopro_column_order(W, H, perm, True, None, ws), m * n * esz),
        "rotate_weight": (lambda: ptq.ptq_lopro_rotate_weight(W, perm, b_I, b_H, Rr), m * n * (esz + 8)),
        "rotate_hessian": (lambda: ptq.ptq_lopro_rotate_hessian(H, perm, b_I, b_H, Hr, ws), n * n * (4 + 8)),
        "unrotate_weight": (lambda: ptq.ptq_lopro_unrotate_weight(Rr, perm, b_I, b_H, back), m * n * 16),
    }
    out = {"b_I": b_I, "b_H": b_H}
    for name, (f, nbytes) in calls.items():
        ms = timed(f)
        out[name] = {"ms": ms, "algorithmic_GBps": nbytes / ms / 1e6, "frac_of_hbm_peak": nbytes / ms / 1e6 / HBM_GBPS}
    out["total_ms"] = sum(v["ms"] for v in out.values() if isinstance(v, dict))
    return out


def r1svd_timings(ptq, W, X, m, n, t, rank=16, it=8, reps=5):
    """The low-rank step that precedes the solve in LoPRo: per-channel activation magnitude over all of X
    (memory-bound, one read of X), the scale, and the scaled rank-one sketching loop in the paper's setting
    (rank 16, 8 power iterations: 16 x 9 applications of "u = A v, z = A^T u" to the float32 matrix)."""
    import torch
    from paper_2601_19675_amd import binding
    dev = "cuda"
    asum = torch.zeros(n, dtype=torch.float64, device=dev)
    s = torch.empty(n, dtype=torch.float64, device=dev)
    g = torch.Generator(device=dev)
    g.manual_seed(19675)
    S = torch.randn((rank, n), generator=g, device=dev, dtype=torch.float32)
    U = torch.empty((rank, m), dtype=torch.uint8, device=dev)
    V = torch.empty((rank, n), dtype=torch.uint8, device=dev)
    sg = torch.empty(rank, dtype=torch.float16, device=dev)
    R = torch.empty((m, n), dtype=torch.float32, device=dev)
    ws = torch.empty(max(ptq.ptq_workspace_bytes(binding.OP_ACTIVATION_ABS_SUM, 0, n),
                         ptq.ptq_workspace_bytes(binding.OP_SCALED_R1SVD, m, n)), dtype=torch.uint8, device=dev)

    def timed(f):
        f()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def magnitude():
        asum.zero_()
        ptq.ptq_activation_abs_sum(asum, X, ws)
        ptq.ptq_activation_scale(asum, t, s)

    a_ms = timed(magnitude)
    r_ms = timed(lambda: ptq.ptq_scaled_r1svd(W, s, S, it, U, V, sg, R, ws))
    apps = rank * (it + 1)
    xbytes = float(t) * n * X.element_size()

    # the same loop on the two MLP projection shapes of the 7B model this layer comes from (random bfloat16
    # weights, log-normal scale): too large for the tile form, kept on the chip as bfloat16 instead
    mlp = {}
    for (mm, nn) in ((11008, 4096), (4096, 11008)):
        W2 = (torch.randn((mm, nn), generator=g, device=dev, dtype=torch.float32) * 0.02).to(torch.bfloat16)
        s2 = torch.exp(torch.randn(nn, generator=g, device=dev, dtype=torch.float32)).double()
        S2 = torch.randn((rank, nn), generator=g, device=dev, dtype=torch.float32)
        U2 = torch.empty((rank, mm), dtype=torch.uint8, device=dev)
        V2 = torch.empty((rank, nn), dtype=torch.uint8, device=dev)
        R2 = torch.empty((mm, nn), dtype=torch.float32, device=dev)
        ws2 = torch.empty(ptq.ptq_workspace_bytes(binding.OP_SCALED_R1SVD, mm, nn), dtype=torch.uint8, device=dev)
        ms2 = timed(lambda: ptq.ptq_scaled_r1svd(W2, s2, S2, it, U2, V2, sg, R2, ws2))
        mlp[f"{mm}x{nn}"] = {"ms": ms2, "us_per_application": 1e3 * ms2 / apps,
                             "equivalent_GBps_of_unfused_gemvs": rank * (2 * it + 2) * 4.0 * mm * nn / ms2 / 1e6}
        del W2, R2, ws2
    ptq.ptq_scaled_r1svd(W, s, S, it, U, V, sg, R, ws)   # sg again holds this layer's sigma
    return {
        "rank": rank, "iterations": it,
        "activation_scale": {"ms": a_ms, "algorithmic_GBps": xbytes / a_ms / 1e6,
                             "frac_of_hbm_peak": xbytes / a_ms / 1e6 / HBM_GBPS},
        "sketch": {"ms": r_ms, "applications": apps, "us_per_application": 1e3 * r_ms / apps,
                   "matrix_bytes_f32": 4.0 * m * n,
                   # what a pass-per-product implementation would stream: (2 it + 2) reads of A per rank
                   "equivalent_GBps_of_unfused_gemvs": rank * (2 * it + 2) * 4.0 * m * n / r_ms / 1e6},
        "sketch_mlp_shapes": mlp,
        "sigma_first": [float(x) for x in sg[:4].float().cpu()],
        "total_ms": a_ms + r_ms,
    }


def vq_timings(ptq, wl, L, reps=5):
    """The vector-quantized form of the solve on the benchmark layer with the factor of the step just run, in the
    paper's two settings (4-D vectors with 256 entries = 2 bits per weight, 2-D vectors with 64 entries = 3 bits);
    the codebook is drawn at random from the layer's own weights.  Float64 throughout: the lazy update is the
    scalar solve's, so the same m n^2 flop count applies."""
    import torch
    out = {}
    W64 = L.W.double().cpu().numpy()
    for K, d in ((256, 4), (64, 2)):
        C = torch.from_numpy(wl.gen_codebook(W64, K, d, L.spec, L.cfg.seed)).cuda()
        idx = torch.empty((L.m, L.n // d), dtype=torch.uint8, device="cuda")
        f = lambda: ptq.ptq_quantize_layer_vq(L.W, L.U, L.dead, C, L.cfg.block, idx, L.Wq, L.err2, L.ws)
        f()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            f()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        ptq.ptq_layer_error(L.W, L.Wq, L.H, L.out, L.ws)
        torch.cuda.synchronize()
        out[f"{K}_entries_x_{d}"] = {"ms": ms, "columns_per_s": L.n / (ms * 1e-3),
                                      "tflops_f64": float(L.m) * L.n * L.n / (ms * 1e-3) / 1e12,
                                      "rel_layer_error": float(L.out[0])}
    return out


def mfma_control(ptq, L):
    """What the matrix cores sustain on this chip, beside the Hessian kernel: (1) a register-only MFMA loop
    (nothing else issued: no loads, no LDS) in bfloat16 and float64, with benign operands and with random
    operand bits, each for tens of milliseconds, with the shader clock read inside the kernel (cycle counter
    over the constant-rate counter); (2) the Hessian kernel itself on the benchmark layer's activations and
    on small-integer activations of the same shape (fewer bits toggling in the multipliers)."""
    import ctypes
    import torch
    from paper_2601_19675_amd import build as b
    lib = ctypes.CDLL(b.PROBE_LIB)
    for fn in (lib.ptq_probe_mfma, lib.ptq_probe_mfma_vgpr):
        fn.restype = ctypes.c_double
        fn.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                       ctypes.c_void_p]
    blocks = 2048
    outb = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    clk = torch.zeros(2, dtype=torch.int64, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    res = {"register_only_loops": []}
    # (accumulators in AGPRs is how the bf16 Hessian kernel is compiled, in VGPRs how the float64 kernels are)
    for kind, name, iters, peak, probe in (
            (0, "bf16 32x32x16, accumulators in AGPRs", 9000, PEAK_BF16_TFLOPS, lib.ptq_probe_mfma),
            (1, "f64 16x16x4, accumulators in AGPRs", 36000, PEAK_F64_TFLOPS, lib.ptq_probe_mfma),
            (1, "f64 16x16x4, accumulators in VGPRs", 36000, PEAK_F64_TFLOPS, lib.ptq_probe_mfma_vgpr)):
        for rnd in (0, 1):
            probe(kind, rnd, 200, blocks, outb.data_ptr(), clk.data_ptr(), st)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            flops = probe(kind, rnd, iters, blocks, outb.data_ptr(), clk.data_ptr(), st)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            c = clk.cpu().tolist()
            res["register_only_loops"].append({
                "mfma": name, "operands": "random bits" if rnd else "benign", "ms": ms,
                "tflops": flops / ms / 1e9, "frac_of_peak": flops / ms / 1e9 / peak,
                "shader_clock_ghz": c[1] / (c[0] / 100e6) / 1e9 if c[0] else None})
    # the Hessian kernel: real activations, then small integers in the same buffer
    def hess_ms(X, reps=3):
        ptq.ptq_hessian_accumulate(L.H, X, L.ws)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            ptq.ptq_hessian_accumulate(L.H, X, L.ws)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    syrk = float(L.t) * L.n * (L.n + 1)
    real_ms = hess_ms(L.X)
    gen = torch.Generator(device="cuda").manual_seed(3)
    for lo in range(0, L.t, 32768):
        hi = min(L.t, lo + 32768)
        L.X[lo:hi] = torch.randint(-2, 3, (hi - lo, L.n), device="cuda", generator=gen, dtype=torch.int8).to(L.X.dtype)
    small_ms = hess_ms(L.X)
    res["hessian_kernel"] = {
        "shape": f"X {L.t}x{L.n}",
        "real_activations": {"ms": real_ms, "tflops_syrk": syrk / real_ms / 1e9, "frac_of_peak": syrk / real_ms / 1e9 / PEAK_BF16_TFLOPS},
        "small_integer_activations": {"ms": small_ms, "tflops_syrk": syrk / small_ms / 1e9,
                                      "frac_of_peak": syrk / small_ms / 1e9 / PEAK_BF16_TFLOPS}}
    return res


def forward_timings(ptq, codes, scales, zeros, m, n, bits, group, rank=16, reps=20):
    """The stored layer applied to 1, 4, 16 and 64 tokens in the rotated-input form (packed codes of the step just
    run, a random permutation, random rank-16 e4m3 factors): bound by the packed codes streaming from memory."""
    import torch
    from paper_2601_19675_amd import binding
    dev = "cuda"
    g = torch.Generator(device=dev)
    g.manual_seed(7)
    packed = torch.empty((n // 32, m, bits), dtype=torch.int32, device=dev)
    st = torch.empty((n // group, m), dtype=torch.float32, device=dev)
    zt = torch.empty((n // group, m), dtype=torch.uint8, device=dev)
    ptq.ptq_pack_codes(codes, bits, packed, scales, zeros, group, st, zt)
    perm = torch.randperm(n, generator=g, device=dev).to(torch.int32)
    U = torch.randint(0x20, 0x38, (rank, m), generator=g, device=dev, dtype=torch.uint8)
    V = torch.randint(0x20, 0x38, (rank, n), generator=g, device=dev, dtype=torch.uint8)
    sg = torch.rand(rank, generator=g, device=dev).to(torch.float16)
    s = torch.ones(n, dtype=torch.float64, device=dev)
    out = {"bits": bits, "group": group, "rank": rank, "packed_bytes": packed.numel() * 4}
    nbytes = packed.numel() * 4 + scales.numel() * 4 + zeros.numel() + rank * (m + n)
    for tokens in (1, 4, 16, 64):
        X = torch.randn((tokens, n), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
        O = torch.empty((tokens, m), dtype=torch.float32, device=dev)
        ws = torch.empty(ptq.ptq_workspace_bytes(binding.OP_LINEAR_FORWARD, m, n, tokens, rank), dtype=torch.uint8,
                         device=dev)
        f = lambda: ptq.ptq_lopro_linear_forward(X, packed, bits, st, zt, group, perm, 256, 256, U, V, sg, s, O, ws)
        for _ in range(3):
            f()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            f()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        out[f"tokens_{tokens}"] = {"ms_per_call": ms, "algorithmic_GBps": nbytes / ms / 1e6,
                                   "frac_of_hbm_peak": nbytes / ms / 1e6 / HBM_GBPS}
    return out


class LayerRun:
    """Device buffers of one layer and one pass of the whole path over them."""

    def __init__(self, ptq, wl, cfg, spec, device_x=False):
        import torch
        self.ptq, self.cfg, self.spec = ptq, cfg, spec
        m, n, t = spec.m, spec.n, spec.t
        self.m, self.n, self.t = m, n, t
        self.damp = cfg.damps[0]
        dev = "cuda"
        self.W = wl.to_device(wl.gen_weight(spec, cfg.seed))
        self.X = torch.empty((t, n), dtype=torch.bfloat16 if spec.dtype == "bf16" else torch.float32, device=dev)
        step_t = 32768
        if device_x:
            gen = torch.Generator(device=dev).manual_seed(cfg.seed + spec.layer_id)
            if spec.x_kind == "student_t":
                ch_scale = torch.ones(n, device=dev)
            else:
                ch_scale = torch.exp(spec.x_sigma * torch.randn(n, device=dev, generator=gen))
            for lo in range(0, t, step_t):
                z = torch.randn((min(t, lo + step_t) - lo, n), device=dev, generator=gen)
                if spec.x_kind == "student_t":
                    chi = sum(torch.randn(z.shape, device=dev, generator=gen).square_() for _ in range(3)) / 3.0
                    z = z / chi.sqrt_()
                self.X[lo:lo + step_t] = (z * ch_scale).to(self.X.dtype)
            del z
        else:
            for lo in range(0, t, step_t):          # generate on the host in slabs, upload
                self.X[lo:lo + step_t] = wl.to_device(wl.gen_activations(spec, cfg.seed, lo, min(t, lo + step_t)))
        self.H = torch.zeros((n, n), dtype=torch.float64, device=dev)
        self.U = torch.empty((n, n), dtype=torch.float64, device=dev)
        self.dead = torch.empty((n,), dtype=torch.uint8, device=dev)
        self.info = torch.empty((2,), dtype=torch.int32, device=dev)
        self.codes = torch.empty((m, n), dtype=torch.uint8, device=dev)
        self.scales = torch.empty((m, n // cfg.group), dtype=torch.float32, device=dev)
        self.zeros = torch.empty((m, n // cfg.group), dtype=torch.uint8, device=dev)
        self.Wq = torch.empty((m, n), dtype=torch.float64, device=dev)
        self.err2 = torch.empty((m,), dtype=torch.float64, device=dev)
        self.out = torch.zeros(3, dtype=torch.float64, device=dev)
        self.ws_bytes = max(ptq.ptq_workspace_bytes(op, m, n, t, cfg.block) for op in range(6))
        self.ws = None

    def step(self, ev=None):
        ptq, cfg = self.ptq, self.cfg
        self.H.zero_()
        if ev: ev[0].record()
        ptq.ptq_hessian_accumulate(self.H, self.X, self.ws)
        if ev: ev[1].record()
        ptq.ptq_damped_cholesky_inv(self.H, self.damp, self.U, self.dead, self.info, self.ws)
        if ev: ev[2].record()
        ptq.ptq_quantize_layer(self.W, self.U, self.dead, cfg.bits, cfg.group, cfg.block, self.codes, self.scales,
                               self.zeros, self.Wq, self.err2, self.ws)
        if ev: ev[3].record()
        ptq.ptq_layer_error(self.W, self.Wq, self.H, self.out, self.ws)
        if ev: ev[4].record()

    def label(self, name):
        s, c = self.spec, self.cfg
        return (f"{name}:{s.name} W {s.m}x{s.n} {s.dtype}, X {s.t}x{s.n} {s.dtype}, "
                f"{c.bits}-bit asym group {c.group} block {c.block} damp {self.damp}")


def calls_alone(L, reps):
    """Each of the four calls of a step on its own, `reps` launches back to back (state left by the last
    step): what the call costs when the chip has not just run another one.  The factor's chain of small
    launches follows the shader clock, which is still low right after the Hessian kernel, so inside a step
    it is slower than alone."""
    import torch
    ptq, cfg = L.ptq, L.cfg
    calls = {
        "hessian": lambda: ptq.ptq_hessian_accumulate(L.H, L.X, L.ws),
        "factor": lambda: ptq.ptq_damped_cholesky_inv(L.H, L.damp, L.U, L.dead, L.info, L.ws),
        "quantize": lambda: ptq.ptq_quantize_layer(L.W, L.U, L.dead, cfg.bits, cfg.group, cfg.block, L.codes, L.scales,
                                                   L.zeros, L.Wq, L.err2, L.ws),
        "layer_error": lambda: ptq.ptq_layer_error(L.W, L.Wq, L.H, L.out, L.ws),
    }
    out = {}
    for name, fn in calls.items():
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[name] = e0.elapsed_time(e1) / reps
    return out


def time_layers(layers, steps, warmup):
    """W untimed passes, then exactly `steps` timed passes over all the layers, one after the other on
    the current stream; returns (ms per pass by the host clock around synchronised ends, per-layer
    per-call event times in ms averaged over the passes)."""
    import torch
    n_ev = 5
    events = [[[torch.cuda.Event(enable_timing=True) for _ in range(n_ev)] for _ in layers] for _ in range(steps)]
    for _ in range(warmup):
        for L in layers:
            L.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        for i, L in enumerate(layers):
            L.step(events[k][i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    for L in layers:
        assert L.info.cpu().tolist() == [0, 0], "factorization failed"
    phases = [[sum(events[k][i][j].elapsed_time(events[k][i][j + 1]) for k in range(steps)) / steps
               for j in range(n_ev - 1)] for i in range(len(layers))]
    return 1e3 * elapsed / steps, phases


def time_block_two_streams(layers, ws_hessian, steps, warmup):
    """The block's layers with the Hessian calls on a stream of their own (both streams at the default
    priority): layer k+1's Hessian runs beside factor, solve and layer error of layer k, whose chain of
    small launches leaves most of the chip idle.  A layer's factor waits for its Hessian; a pass starts
    only when the previous pass has ended (a block is timed as a unit, no overlap from block to block).
    `ws_hessian`: a workspace of the Hessian calls' own, the other calls keep the layers' shared one.
    Returns ms per pass by the host clock around synchronised ends."""
    import torch
    s_h, s_r = torch.cuda.Stream(), torch.cuda.Stream()
    ready = [torch.cuda.Event() for _ in layers]
    block_done = torch.cuda.Event()

    def one_pass():
        s_h.wait_event(block_done)
        for L, ev in zip(layers, ready):
            with torch.cuda.stream(s_h):
                L.H.zero_()
                L.ptq.ptq_hessian_accumulate(L.H, L.X, ws_hessian)
                ev.record(s_h)
            with torch.cuda.stream(s_r):
                s_r.wait_event(ev)
                L.ptq.ptq_damped_cholesky_inv(L.H, L.damp, L.U, L.dead, L.info, L.ws)
                L.ptq.ptq_quantize_layer(L.W, L.U, L.dead, L.cfg.bits, L.cfg.group, L.cfg.block, L.codes, L.scales,
                                         L.zeros, L.Wq, L.err2, L.ws)
                L.ptq.ptq_layer_error(L.W, L.Wq, L.H, L.out, L.ws)
        block_done.record(s_r)

    torch.cuda.synchronize()
    block_done.record(s_r)
    for _ in range(warmup):
        one_pass()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        one_pass()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    for L in layers:
        assert L.info.cpu().tolist() == [0, 0], "factorization failed"
    return 1e3 * elapsed / steps


def layer_numbers(L, phase):
    """Rates of one layer's four calls from their event-bracketed times."""
    m, n, t, cfg, spec = L.m, L.n, L.t, L.cfg, L.spec
    h_ms, f_ms, q_ms, e_ms = phase
    syrk_flops = float(t) * n * (n + 1)           # algorithmic: upper triangle incl. diagonal
    h_tflops = syrk_flops / (h_ms * 1e-3) / 1e12
    f_flops = 2.0 / 3.0 * float(n) ** 3
    q_flops = float(m) * n * n
    # piece products per term: layers of at least 65536 entries run with two bfloat16 pieces per operand (3 products
    # for tr(D H D^T) + 2 for tr(W H W^T) when W is stored in bfloat16, else 3 + 3), smaller ones with three (6 + 3, 6 + 6)
    two = m * n >= 65536
    pieces = ((5.0 if two else 9.0) if spec.dtype == "bf16" else (6.0 if two else 12.0))
    e_exec = pieces * m * n * (n + 128.0)         # piece products the kernel executes on the bf16 MFMA
    e_alg = 2.0 * m * n * (n + 128.0)             # the two traces of the method itself
    peak_f64 = PEAK_F64_TFLOPS
    return {
        "phases_ms": {"hessian": h_ms, "factor": f_ms, "quantize": q_ms, "layer_error": e_ms},
        "hessian_tflops_syrk": h_tflops,
        "hessian_tflops_full_square": 2.0 * t * n * n / (h_ms * 1e-3) / 1e12,
        "hessian_pct_mfma_peak": 100.0 * h_tflops / PEAK_BF16_TFLOPS,
        "solve_columns_per_s": n / ((f_ms + q_ms) * 1e-3),
        "quantize_columns_per_s": n / (q_ms * 1e-3),
        "quantize_tflops_f64": q_flops / (q_ms * 1e-3) / 1e12,
        # W in, codes + Wq out, the upper triangle of U, the grids: what the column walk has to move
        "quantize_algorithmic_gbps": (float(m) * n * (L.W.element_size() + 1 + 8) + 4.0 * n * n
                                      + 5.0 * m * n / cfg.group) / (q_ms * 1e-3) / 1e9,
        "syrk_flops": syrk_flops,
        # the other three calls against the peak of the unit that bounds them: algorithmic flops of the call over
        # its event-bracketed time; for the layer error both the method's own two traces and the bf16 piece
        # products the kernel executes to form them at float32 precision
        "rooflines_other_calls": [
            {"call": "ptq_damped_cholesky_inv", "bound": "mfma", "dtype": "f64",
             "achieved": f_flops / (f_ms * 1e-3) / 1e12, "peak": peak_f64, "unit": "TFLOP/s",
             "frac": f_flops / (f_ms * 1e-3) / 1e12 / peak_f64},
            {"call": "ptq_quantize_layer", "bound": "mfma", "dtype": "f64",
             "achieved": q_flops / (q_ms * 1e-3) / 1e12, "peak": peak_f64, "unit": "TFLOP/s",
             "frac": q_flops / (q_ms * 1e-3) / 1e12 / peak_f64},
            {"call": "ptq_layer_error", "bound": "mfma", "dtype": "bf16",
             "achieved": e_alg / (e_ms * 1e-3) / 1e12, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
             "frac": e_alg / (e_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
             "flops_counted": "algorithmic: the two traces, 2 m n (n + 128)",
             "executed_piece_products_tflops": e_exec / (e_ms * 1e-3) / 1e12,
             "executed_frac": e_exec / (e_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
        ],
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="C3", help="C1..C4: one layer of that configuration (see --layer); "
                    "C5: the seven linears of a decoder block as one timed region")
    ap.add_argument("--layer", type=int, default=None,
                    help="index of the layer inside the configuration (default: the last one, which for C3 is the "
                         "4096 x 11008 down projection)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-factor-sample", action="store_true",
                    help="time the oracle's factor on the leading 4096 x 4096 block and scale by the cube of the size "
                         "ratio instead of factoring the layer's full matrix (n = 11008: about a minute and a half)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short extra timing of the 4096 x 4096 attention projection (C2) that the default "
                         "run reports under \"other_workloads\"")
    ap.add_argument("--lopro", action="store_true",
                    help="also time LoPRo's pre-conditioning of the same layer (column order, rotation of W and H, "
                         "way back; b_I = b_H = 256) and report it under \"lopro\"; the step itself is unchanged")
    ap.add_argument("--r1svd", action="store_true",
                    help="also time the low-rank step on the same layer (activation scale from X, then the scaled "
                         "rank-one sketch with rank 16 and 8 iterations) and report it under \"r1svd\"")
    ap.add_argument("--forward", action="store_true",
                    help="also time the stored layer applied to 1 and 4 tokens (packed codes, rotated input, "
                         "rank-16 low-rank part) and report it under \"forward\"")
    ap.add_argument("--calls-alone", action="store_true",
                    help="also time each of the four calls alone, back to back (phases_alone_ms)")
    ap.add_argument("--two-streams", action="store_true",
                    help="with --config C5: time the block again with the Hessian calls on a second stream (layer k+1's "
                         "Hessian beside factor, solve and error of layer k) and report that time, the one-stream time "
                         "beside it; measured 1.3 %% faster to 0.5 %% slower from box to box, hence not the default")
    ap.add_argument("--mfma-control", action="store_true",
                    help="also run the controls behind the Hessian roofline: register-only MFMA loops (bfloat16 and "
                         "float64, benign and random operand bits, shader clock read in the kernel) and the Hessian "
                         "kernel on small-integer activations; reported under \"mfma_control\" (overwrites X: runs last)")
    ap.add_argument("--vq", action="store_true",
                    help="also time the vector-quantized form of the solve (256 entries x 4 and 64 entries x 2) on the "
                         "same layer and factor and report it under \"vq\"")
    ap.add_argument("--device-x", action="store_true",
                    help="draw the activations on the GPU (same distribution family, torch generator) instead of "
                         "the seeded host generator")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run plain 1 GiB device copies and exit (reference reading for the "
                         "FETCH_SIZE / WRITE_SIZE counters under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (the path has no multi-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2601_19675_amd as ptq
    import ptq_workloads as wl

    if not os.path.exists(ptq.lib_path()):
        from paper_2601_19675_amd import build
        build.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 1 << 30, "copy_bytes_written": 1 << 30, "copies": 3}))
        return

    cfg = wl.CONFIGS[args.config]
    block_mode = args.config == "C5" and args.layer is None
    specs = list(cfg.layers) if block_mode else [cfg.layers[args.layer if args.layer is not None else -1]]
    layers = []
    for spec in specs:
        log(f"generating inputs of {spec.name} {spec.m}x{spec.n}, X {spec.t}x{spec.n}")
        layers.append(LayerRun(ptq, wl, cfg, spec, args.device_x))
    ws = torch.empty(max(L.ws_bytes for L in layers), dtype=torch.uint8, device="cuda")
    for L in layers:
        L.ws = ws
    log("timing")
    ms, phases = time_layers(layers, args.steps, args.warmup)
    ms_one_stream = None
    if block_mode and args.two_streams:
        # the same passes again with the Hessian calls on a second stream; the per-call times above are from
        # the one-stream passes, where calls do not overlap
        one_stream_out = [float(Li.out[0]) for Li in layers]
        ws_h = torch.empty(max(ptq.ptq_workspace_bytes(0, Li.m, Li.n, Li.t, cfg.block) for Li in layers),
                           dtype=torch.uint8, device="cuda")
        ms_one_stream, ms = ms, time_block_two_streams(layers, ws_h, args.steps, args.warmup)
        assert [float(Li.out[0]) for Li in layers] == one_stream_out, "the two-stream pass changed a result"
        del ws_h
    total_cols = sum(L.n for L in layers)
    # the layer whose Hessian call is the longest carries the roofline object (a block: the down projection)
    dom = max(range(len(layers)), key=lambda i: phases[i][0])
    L, spec = layers[dom], layers[dom].spec
    m, n, t = L.m, L.n, L.t
    nums = layer_numbers(L, phases[dom])
    h_ms, f_ms, q_ms, e_ms = phases[dom]
    traffic = MEASURED_TRAFFIC_BYTES.get(f"{args.config}:{spec.name}", (None, None))

    result = {
        "metric": "layer-solve columns quantized/sec + Hessian TFLOP/s (% MFMA peak), 1 GPU",
        "value": total_cols / (ms * 1e-3), "unit": "columns/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16,f32,f64" if spec.dtype == "bf16" else "f32,f64",
        "data": "synthetic (device-drawn activations)" if args.device_x else "synthetic",
        "config": {"workload": (f"C5: decoder block, 7 linears back to back ({total_cols} columns; each layer its own "
                                f"X {t} tokens), {cfg.bits}-bit asym group {cfg.group} block {cfg.block} damp {L.damp}"
                                if block_mode else L.label(args.config))},
    }
    for k in ("phases_ms", "hessian_tflops_syrk", "hessian_tflops_full_square", "hessian_pct_mfma_peak",
              "solve_columns_per_s", "quantize_columns_per_s", "quantize_tflops_f64", "quantize_algorithmic_gbps"):
        result[k] = nums[k]
    result["rel_layer_error"] = float(L.out[0])
    result["roofline"] = {
        "kernel": "ptq_hessian_accumulate (Hessian MFMA kernel + partial-tile reduction)"
                  + (f" of {spec.name} {m}x{n}" if block_mode else ""),
        "bound": "mfma", "achieved": nums["hessian_tflops_syrk"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
        "frac": nums["hessian_tflops_syrk"] / PEAK_BF16_TFLOPS,
        "traffic": traffic[0], "traffic_source": traffic[1],
        "algorithmic_flops_per_launch": nums["syrk_flops"], "algorithmic_bytes_per_launch": 2.0 * t * n,
    }
    result["rooflines_other_calls"] = nums["rooflines_other_calls"]
    if block_mode:
        result["streams"] = 1 if ms_one_stream is None else 2
        if ms_one_stream is not None:
            result["ms_per_step_one_stream"] = ms_one_stream
        result["layers"] = [dict(name=Li.spec.name, m=Li.m, n=Li.n, rel_layer_error=float(Li.out[0]),
                                 **{k: v for k, v in layer_numbers(Li, ph).items()
                                    if k in ("phases_ms", "hessian_pct_mfma_peak", "solve_columns_per_s")})
                            for Li, ph in zip(layers, phases)]
    # the solve against its floors (bytes at the HBM rate, flops at the float64 peak), and what its
    # serial part costs: n columns at the per-column time of a call that is nothing but the walk
    q_bytes = float(m) * n * (L.W.element_size() + 1 + 8) + 4.0 * n * n + 5.0 * m * n / cfg.group
    t_col_us = single_block_us_per_column(ptq, cfg.bits, cfg.group)
    floors = {"hbm_ms": q_bytes / (HBM_GBPS * 1e9) * 1e3, "f64_ms": float(m) * n * n / (PEAK_F64_TFLOPS * 1e12) * 1e3}
    result["quantize_floors"] = dict(floors, frac_of_largest_floor=max(floors.values()) / q_ms,
                                     single_block_us_per_column=t_col_us, walk_ms_upper_estimate=n * t_col_us * 1e-3)
    if args.calls_alone:
        result["phases_alone_ms"] = calls_alone(L, max(3, args.steps))
    if args.lopro:
        result["lopro"] = lopro_timings(ptq, L.W, L.H, m, n, ws)
    if args.r1svd:
        result["r1svd"] = r1svd_timings(ptq, L.W, L.X, m, n, t)
    if args.forward:
        result["forward"] = forward_timings(ptq, L.codes, L.scales, L.zeros, m, n, cfg.bits, cfg.group)
    if args.vq:
        result["vq"] = vq_timings(ptq, wl, L)
    if args.mfma_control:
        result["mfma_control"] = mfma_control(ptq, L)
    main_is_headline = (args.config == "C3" and not block_mode and spec.name == "down_proj")
    del layers, L, ws
    torch.cuda.empty_cache()
    if main_is_headline and not args.no_other_workloads:
        # the 4096 x 4096 attention projection (second configuration), a few passes, for comparison across runs
        cfg2 = wl.CONFIGS["C2"]
        log("generating inputs of C2 attn_proj for the extra timing")
        L2 = LayerRun(ptq, wl, cfg2, cfg2.layers[0], args.device_x)
        L2.ws = torch.empty(L2.ws_bytes, dtype=torch.uint8, device="cuda")
        ms2, ph2 = time_layers([L2], max(3, args.steps // 2), 2)
        n2 = layer_numbers(L2, ph2[0])
        result["other_workloads"] = {L2.label("C2"): {
            "ms_per_step": ms2, "columns_per_s": L2.n / (ms2 * 1e-3), "phases_ms": n2["phases_ms"],
            "hessian_pct_mfma_peak": n2["hessian_pct_mfma_peak"], "solve_columns_per_s": n2["solve_columns_per_s"],
            "quantize_tflops_f64": n2["quantize_tflops_f64"]}}
        del L2
        torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        log("cpu baseline (oracle on the host cores)")
        result["cpu_baseline"] = cpu_baseline(cfg, spec, cfg.seed, full_factor=not args.cpu_baseline_factor_sample)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
