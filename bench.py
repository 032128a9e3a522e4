#!/usr/bin/env python3
"""Benchmark of the layer-wise quantization solve on one MI355X.

A step is one pass of the whole hot path over one synthetic layer:
Hessian accumulation -> damped Cholesky factor of the inverse -> blocked
column quantization -> layer error, with all inputs resident in HBM.
Prints ONE JSON line: metric / value / unit (columns quantized per second for the whole step),
ms_per_step and the per-call times, the Hessian rate, a "roofline" object for the dominant
kernel and a "cpu_baseline" object (the oracle timed on a sample of the same layer).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C2] [--no-cpu-baseline]
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

# HBM bytes per launch of the dominant kernel (Hessian main kernel), from two rocprofv3 --pmc
# runs of this file (FETCH_SIZE, then WRITE_SIZE), each scaled by what the same counter reads
# for a plain 1 GiB device copy (--copy-calibration): FETCH_SIZE reads 524288 per GiB read
# (factor 2 KiB per count), WRITE_SIZE 1048576 per GiB written (1 KiB per count).
# See profiles/hessian_C2_hbm_traffic.txt.  None for workloads that were not profiled.
MEASURED_TRAFFIC_BYTES = {
    "C2:attn_proj": 3.655e6 * 2048 + 5.222e5 * 1024,
}


def cpu_baseline(cfg, spec, seed):
    """The oracle, as it stands, on a bounded sample of the same layer; scaled to columns/s."""
    import numpy as np
    from threadpoolctl import threadpool_info

    import ptq_workloads as wl
    from oracle import ptq_oracle as orc

    t_s = min(spec.t, 4096)
    rows_s = min(spec.m, 64)
    Ws = wl.gen_weight(spec, seed)
    X64 = wl.to_f64(wl.gen_activations(spec, seed, 0, t_s))
    W64 = wl.to_f64(Ws)[:rows_s]
    t0 = time.perf_counter()
    H = orc.hessian(X64)
    t1 = time.perf_counter()
    Hd, dead = orc.damp(H, cfg.damps[0])
    U = orc.inverse_cholesky_upper(Hd)
    t2 = time.perf_counter()
    out = orc.quantize_layer(W64, U, cfg.bits, cfg.group, dead=dead)
    t3 = time.perf_counter()
    orc.layer_error(W64, out["Wq"], H)
    t4 = time.perf_counter()
    est = ((t1 - t0) * spec.t / t_s + (t2 - t1) + (t3 - t2) * spec.m / rows_s + (t4 - t3) * spec.m / rows_s)
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    return {
        "value": spec.n / est, "unit": "columns/s", "cores": int(threads), "kind": "oracle",
        "sample": (f"{t_s} of {spec.t} tokens for H, full {spec.n}x{spec.n} factor, {rows_s} of {spec.m} rows "
                   f"for solve and error; times scaled linearly to the full layer "
                   f"(H {t1 - t0:.2f}s, factor {t2 - t1:.2f}s, solve {t3 - t2:.2f}s, error {t4 - t3:.2f}s measured)"),
        "est_seconds_full_layer": est,
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="C2")
    ap.add_argument("--layer", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--lopro", action="store_true",
                    help="also time LoPRo's pre-conditioning of the same layer (column order, rotation of W and H, "
                         "way back; b_I = b_H = 256) and report it under \"lopro\"; the step itself is unchanged")
    ap.add_argument("--r1svd", action="store_true",
                    help="also time the low-rank step on the same layer (activation scale from X, then the scaled "
                         "rank-one sketch with rank 16 and 8 iterations) and report it under \"r1svd\"")
    ap.add_argument("--forward", action="store_true",
                    help="also time the stored layer applied to 1 and 4 tokens (packed codes, rotated input, "
                         "rank-16 low-rank part) and report it under \"forward\"")
    ap.add_argument("--device-x", action="store_true",
                    help="draw the activations on the GPU (same distribution family, torch generator) instead of "
                         "the seeded host generator: for timing the widest layers, whose host generation takes minutes")
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

    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from parity import to_device

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
    spec = cfg.layers[args.layer]
    m, n, t = spec.m, spec.n, spec.t
    damp = cfg.damps[0]
    W = to_device(wl.gen_weight(spec, cfg.seed))
    X = torch.empty((t, n), dtype=torch.bfloat16 if spec.dtype == "bf16" else torch.float32, device="cuda")
    step_t = 32768
    if args.device_x:
        gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
        if spec.x_kind == "student_t":
            ch_scale = torch.ones(n, device="cuda")
        else:
            ch_scale = torch.exp(spec.x_sigma * torch.randn(n, device="cuda", generator=gen))
        for lo in range(0, t, step_t):
            z = torch.randn((min(t, lo + step_t) - lo, n), device="cuda", generator=gen)
            if spec.x_kind == "student_t":
                chi = sum(torch.randn_like(z).square_() for _ in range(3)) / 3.0
                z = z / chi.sqrt_()
            X[lo:lo + step_t] = (z * ch_scale).to(X.dtype)
        del z
    else:
        for lo in range(0, t, step_t):          # generate on the host in slabs, upload
            X[lo:lo + step_t] = to_device(wl.gen_activations(spec, cfg.seed, lo, min(t, lo + step_t)))

    dev = "cuda"
    H = torch.zeros((n, n), dtype=torch.float64, device=dev)
    U = torch.empty((n, n), dtype=torch.float64, device=dev)
    dead = torch.empty((n,), dtype=torch.uint8, device=dev)
    info = torch.empty((2,), dtype=torch.int32, device=dev)
    codes = torch.empty((m, n), dtype=torch.uint8, device=dev)
    scales = torch.empty((m, n // cfg.group), dtype=torch.float32, device=dev)
    zeros = torch.empty((m, n // cfg.group), dtype=torch.uint8, device=dev)
    Wq = torch.empty((m, n), dtype=torch.float64, device=dev)
    err2 = torch.empty((m,), dtype=torch.float64, device=dev)
    out = torch.zeros(3, dtype=torch.float64, device=dev)
    ws_bytes = max(ptq.ptq_workspace_bytes(op, m, n, t, cfg.block) for op in range(6))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    n_ev = 5
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(n_ev)] for _ in range(args.steps)]

    def step(ev=None):
        H.zero_()
        if ev: ev[0].record()
        ptq.ptq_hessian_accumulate(H, X, ws)
        if ev: ev[1].record()
        ptq.ptq_damped_cholesky_inv(H, damp, U, dead, info, ws)
        if ev: ev[2].record()
        ptq.ptq_quantize_layer(W, U, dead, cfg.bits, cfg.group, cfg.block, codes, scales, zeros, Wq, err2, ws)
        if ev: ev[3].record()
        ptq.ptq_layer_error(W, Wq, H, out, ws)
        if ev: ev[4].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert info.cpu().tolist() == [0, 0], "factorization failed"

    ms = 1e3 * elapsed / args.steps
    phase = [sum(events[k][i].elapsed_time(events[k][i + 1]) for k in range(args.steps)) / args.steps
             for i in range(n_ev - 1)]
    h_ms, f_ms, q_ms, e_ms = phase
    syrk_flops = float(t) * n * (n + 1)           # algorithmic: upper triangle incl. diagonal
    h_tflops = syrk_flops / (h_ms * 1e-3) / 1e12
    rel = float(out[0])

    result = {
        "metric": "layer-solve columns quantized/sec + Hessian TFLOP/s (% MFMA peak), 1 GPU",
        "value": n / (ms * 1e-3), "unit": "columns/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16,f32,f64" if spec.dtype == "bf16" else "f32,f64", "data": "synthetic (device-drawn activations)" if args.device_x else "synthetic",
        "config": {"workload": f"{args.config}:{spec.name} W {m}x{n} {spec.dtype}, X {t}x{n} {spec.dtype}, "
                               f"{cfg.bits}-bit asym group {cfg.group} block {cfg.block} damp {damp}"},
        "phases_ms": {"hessian": h_ms, "factor": f_ms, "quantize": q_ms, "layer_error": e_ms},
        "hessian_tflops_syrk": h_tflops,
        "hessian_tflops_full_square": 2.0 * t * n * n / (h_ms * 1e-3) / 1e12,
        "hessian_pct_mfma_peak": 100.0 * h_tflops / PEAK_BF16_TFLOPS,
        "solve_columns_per_s": n / ((f_ms + q_ms) * 1e-3),
        "quantize_columns_per_s": n / (q_ms * 1e-3),
        "quantize_tflops_f64": float(m) * n * n / (q_ms * 1e-3) / 1e12,
        # W in, codes + Wq out, the upper triangle of U, the grids: what the column walk has to move
        "quantize_algorithmic_gbps": (float(m) * n * (W.element_size() + 1 + 8) + 4.0 * n * n
                                      + 5.0 * m * n / cfg.group) / (q_ms * 1e-3) / 1e9,
        "rel_layer_error": rel,
        "roofline": {
            "kernel": "ptq_hessian_accumulate (Hessian MFMA kernel + partial-tile reduction)",
            "bound": "mfma", "achieved": h_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": h_tflops / PEAK_BF16_TFLOPS,
            "traffic": MEASURED_TRAFFIC_BYTES.get(f"{args.config}:{spec.name}"),
            "algorithmic_flops_per_launch": syrk_flops, "algorithmic_bytes_per_launch": 2.0 * t * n,
        },
    }
    # the other three calls against the peak of the unit that bounds them (algorithmic flops of the call
    # over its event-bracketed time; the layer error counts the piece products it executes on the bf16 MFMA)
    f_flops = 2.0 / 3.0 * float(n) ** 3
    q_flops = float(m) * n * n
    pieces = 9.0 if spec.dtype == "bf16" else 12.0
    e_flops = pieces * m * n * (n + 128.0)
    result["rooflines_other_calls"] = [
        {"call": "ptq_damped_cholesky_inv", "bound": "mfma", "dtype": "f64", "achieved": f_flops / (f_ms * 1e-3) / 1e12,
         "peak": PEAK_F64_TFLOPS, "unit": "TFLOP/s", "frac": f_flops / (f_ms * 1e-3) / 1e12 / PEAK_F64_TFLOPS},
        {"call": "ptq_quantize_layer", "bound": "mfma", "dtype": "f64", "achieved": q_flops / (q_ms * 1e-3) / 1e12,
         "peak": PEAK_F64_TFLOPS, "unit": "TFLOP/s", "frac": q_flops / (q_ms * 1e-3) / 1e12 / PEAK_F64_TFLOPS},
        {"call": "ptq_layer_error", "bound": "mfma", "dtype": "bf16", "achieved": e_flops / (e_ms * 1e-3) / 1e12,
         "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": e_flops / (e_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
    ]
    # the solve against its floors (bytes at the HBM rate, flops at the float64 peak), and what its
    # serial part costs: n columns at the per-column time of a call that is nothing but the walk
    q_bytes = float(m) * n * (W.element_size() + 1 + 8) + 4.0 * n * n + 5.0 * m * n / cfg.group
    t_col_us = single_block_us_per_column(ptq, cfg.bits, cfg.group)
    floors = {"hbm_ms": q_bytes / (HBM_GBPS * 1e9) * 1e3, "f64_ms": float(m) * n * n / (PEAK_F64_TFLOPS * 1e12) * 1e3}
    result["quantize_floors"] = dict(floors, frac_of_largest_floor=max(floors.values()) / q_ms,
                                     single_block_us_per_column=t_col_us, walk_ms_upper_estimate=n * t_col_us * 1e-3)
    if args.lopro:
        result["lopro"] = lopro_timings(ptq, W, H, m, n, ws)
    if args.r1svd:
        result["r1svd"] = r1svd_timings(ptq, W, X, m, n, t)
    if args.forward:
        result["forward"] = forward_timings(ptq, codes, scales, zeros, m, n, cfg.bits, cfg.group)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, spec, cfg.seed)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
