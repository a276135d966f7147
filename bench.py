#!/usr/bin/env python3
"""Benchmark of the APB layer forward pass on one MI355X.

One "step" = the whole per-batch hot path on inputs already resident in HBM:
apb_quantize_acts (quantize + bit-plane packing) followed by apb_forward (binary product on the
matrix cores, then CSR part + epilogue).  apb_compress is per-layer offline work and is not timed.

Prints ONE JSON line.  `value` is (2*N*K*M + 2*nnz*M) / step time, in GOPS, for the workload
named in config.workload; `roofline` describes the kernel that dominates the step and
`roofline_forward` the two forward kernels together; `cpu_baseline` is the CPU oracle timed on a bounded
column sample of the same workload on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0                  # MI355X HBM3E, published
MFMA_FP4_PEAK_TFLOPS = 10100.0         # dense FP4 MFMA, published
FP64_VECTOR_PEAK_TFLOPS = 78.6         # 256 CUs x 64 lanes x 2.4 GHz x 2 (fused multiply-add)
VALU_LANE_OPS_PER_S = 256 * 64 * 2.4e9 # 39.3e12 32-bit vector lane-ops/s: the bit-op roof of a popcount formulation

# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# calibrated against a plain copy of known size (profiles/traffic_C2_pmc.txt says how).
MEASURED_TRAFFIC_BYTES = {("C2", "k_quantize_pack"): 321.5e6, ("C2", "one_kernel_step"): 335.9e6}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C2", help="name in paper_2306_08960_amd.synth.CONFIGS")
    ap.add_argument("--all", action="store_true", help="also time every other benchmark layer (reported in 'others')")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="before the steps, copy X into a buffer of the same size three times: a plain copy kernel of "
                         "known size, against which FETCH_SIZE / WRITE_SIZE of a rocprofv3 --pmc run are scaled")
    ap.add_argument("--sweep", action="store_true",
                    help="square-matrix sweep of the three bitwise products (1/1, 1/2, 2/2; Sec. V protocol): one JSON "
                         "line with the time of the product alone at each size")
    ap.add_argument("--routine", default="apb", choices=["apb", "gemm_2_2", "chain", "conv_chain"],
                    help="apb: the APB layer forward (the headline metric); gemm_2_2: the 2-bit x 2-bit "
                         "product of Sec. IV on the same shapes (weights packed offline)")
    return ap.parse_args()


def time_in_step(quant, fwd, iters, ms_step_plain):
    """Per-launch times of the two entry points INSIDE the step loop (quantize, forward, quantize, ...),
    from HIP events recorded on the stream the kernels run on.  Timed alone in a tight loop the quantize
    kernel looks faster than it is in a pipeline, because part of X then survives in the memory-side
    cache from one launch to the next.  Every event record costs the stream a couple of microseconds;
    that cost (the slowdown of this instrumented pass against the plain timed pass, per record) is
    taken off each interval, so the two figures add up to the plain step time less the launch gap."""
    import torch
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(iters)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b_, c in ev:
        a.record()
        quant()
        b_.record()
        fwd()
        c.record()
    torch.cuda.synchronize()
    ms_step_events = (time.perf_counter() - t0) * 1e3 / iters
    per_record = max(0.0, (ms_step_events - ms_step_plain) / 3.0)
    tq = sum(a.elapsed_time(b_) for a, b_, c in ev) / iters - per_record
    tf = sum(b_.elapsed_time(c) for a, b_, c in ev) / iters - per_record
    return tq, tf, per_record          # ms


def run_workload(name, steps, warmup, calibration_copy=False):
    import torch
    from paper_2306_08960_amd import binding as b
    from paper_2306_08960_amd import synth

    cfg = synth.CONFIGS[name]
    W, delta, X, step = synth.make_layer(cfg)
    N, K, M, bits = cfg.N, cfg.K, cfg.M, cfg.bits
    Wd = torch.from_numpy(W).cuda()
    Xd = torch.from_numpy(X).cuda()
    layer = b.apb_compress(Wd, float(delta))
    nnz = layer.info()["nnz"]
    packed = b.alloc_packed(K, M, bits)
    Y = torch.empty((N, M), dtype=torch.float32, device="cuda")
    s = float(step)
    if calibration_copy:
        Xc = torch.empty_like(Xd)
        for _ in range(3):
            Xc.copy_(Xd)                     # reads and writes 4*K*M bytes
        torch.cuda.synchronize()
        del Xc

    def quant():
        b.apb_quantize_acts(Xd, bits, s, packed=packed)

    def fwd():
        b.apb_forward(layer, packed, M, bits, s, Y=Y)

    def two_calls():
        quant()
        fwd()

    def one_call():                          # the step: quantize + forward through the single entry point
        b.apb_quantize_forward(layer, Xd, bits, s, packed=packed, Y=Y)

    def timed(fn):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    one_kernel = b.apb_quantize_forward_is_one_kernel(layer, M, bits)
    ms_two = timed(two_calls)
    ms_quant, ms_fwd, ms_event_record = time_in_step(quant, fwd, steps, ms_two)
    ms_step = timed(one_call)
    # the single call between events on its stream (same treatment of the record cost as in time_in_step)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, c in ev:
        a.record()
        one_call()
        c.record()
    torch.cuda.synchronize()
    per_record = max(0.0, ((time.perf_counter() - t0) * 1e3 / steps - ms_step) / 2.0)
    ms_one = sum(a.elapsed_time(c) for a, c in ev) / steps - per_record

    ops = 2.0 * N * K * M + 2.0 * nnz * M
    Kw, Mp = (K + 31) // 32, 64 * ((M + 63) // 64)
    # quantize: reads X once, writes the bit-planes and the column sums
    quant_bytes = 4.0 * K * M + 4.0 * bits * Kw * Mp + 4.0 * Mp
    roof_quant = {"kernel": "k_quantize_pack", "bound": "hbm", "achieved": quant_bytes / (ms_quant * 1e-3) / 1e9,
                  "peak": HBM_PEAK_GBS, "unit": "GB/s", "traffic": MEASURED_TRAFFIC_BYTES.get((name, "k_quantize_pack")),
                  "algorithmic_bytes": quant_bytes, "ms": ms_quant}
    roof_quant["frac"] = roof_quant["achieved"] / roof_quant["peak"]
    # forward = one kernel (binary tile on the matrix cores + residual part + epilogue).  Its floor is the
    # largest of: the bytes it has to move
    # (sign words, bit-planes, residual entries, Y), the FP4 matrix-core time of the binary product and
    # the float64 vector time of the residual multiply-adds.
    fwd_bytes = 4.0 * N * Kw + 4.0 * bits * Kw * Mp + 4.0 * Mp + 12.0 * nnz + 4.0 * N * M
    t_hbm = fwd_bytes / (HBM_PEAK_GBS * 1e9)
    t_mfma = 2.0 * N * K * M / (MFMA_FP4_PEAK_TFLOPS * 1e12)
    t_f64 = 2.0 * nnz * M / (FP64_VECTOR_PEAK_TFLOPS * 1e12)
    t_fwd = ms_fwd * 1e-3
    if t_hbm >= max(t_mfma, t_f64):
        roof_fwd = {"bound": "hbm", "achieved": fwd_bytes / t_fwd / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    elif t_mfma >= t_f64:
        roof_fwd = {"bound": "mfma", "achieved": 2.0 * N * K * M / t_fwd / 1e12, "peak": MFMA_FP4_PEAK_TFLOPS,
                    "unit": "TFLOP/s"}
    else:
        roof_fwd = {"bound": "alu", "achieved": 2.0 * nnz * M / t_fwd / 1e12, "peak": FP64_VECTOR_PEAK_TFLOPS,
                    "unit": "TFLOP/s"}
    roof_fwd = {"kernel": "k_sparse_epilogue or k_forward_ksplit (the forward kernel)"} | roof_fwd
    roof_fwd |= {"frac": roof_fwd["achieved"] / roof_fwd["peak"], "traffic": None, "ms": ms_fwd,
                 "floor_us": {"hbm": t_hbm * 1e6, "mfma_fp4": t_mfma * 1e6, "fp64_vector": t_f64 * 1e6}}
    # The roof the benchmark spec names for the forward: the vector-ALU bit-op rate of the popcount
    # formulation (per weight word, plane and column one logic op + one accumulating popcount; per residual
    # and column one multiply-add).  The binary part runs on the matrix cores here, so this is a yardstick,
    # not a bound: the fraction may exceed 1.
    t_valu = (2.0 * bits * N * Kw * M + float(nnz) * M) / VALU_LANE_OPS_PER_S
    roof_valu = {"bound": "alu", "what": "VALU bit-op roof of the popcount formulation", "roof_us": t_valu * 1e6,
                 "achieved": ops / t_fwd / 1e12, "peak": ops / t_valu / 1e12, "unit": "TOP/s", "frac": t_valu / t_fwd}
    # Layers of at most 128 rows run the step as ONE kernel (quantize into LDS + forward): it reads X and the
    # layer and writes Y, nothing else, so its floor is those bytes at the HBM peak.
    one_bytes = 4.0 * K * M + 4.0 * N * M + 4.0 * N * Kw + 12.0 * nnz
    roof_one = {"kernel": "k_sparse_epilogue<.., float input> (quantize + forward in one kernel)", "bound": "hbm",
                "achieved": one_bytes / (ms_one * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "traffic": MEASURED_TRAFFIC_BYTES.get((name, "one_kernel_step")),
                "algorithmic_bytes": one_bytes, "ms": ms_one}
    roof_one["frac"] = roof_one["achieved"] / roof_one["peak"]
    roof_two = roof_quant if ms_quant >= ms_fwd else roof_fwd
    res = {
        "workload": name, "N": N, "K": K, "M": M, "act_bits": bits, "nnz": int(nnz),
        "ms_per_step": ms_step, "gops_step": ops / (ms_step * 1e-3) / 1e9, "one_kernel_step": bool(one_kernel),
        "ms_per_step_two_calls": ms_two,
        "ms_quantize": ms_quant, "ms_forward": ms_fwd, "ms_event_record_removed": ms_event_record,
        "gops_forward": ops / (ms_fwd * 1e-3) / 1e9,
        "roofline": roof_one if one_kernel else roof_two, "roofline_forward": roof_fwd,
        "roofline_forward_valu_bitop": roof_valu,
        "roofline_quantize": roof_quant,
    }
    layer.free()
    del Wd, Xd, packed, Y
    torch.cuda.empty_cache()
    return res, (cfg, W, delta, X, step)


def run_gemm_2_2(name, steps, warmup):
    """Step = apb_quantize_acts (2 bits) + apb_gemm_2_2 on the workload's W and X; weights packed once."""
    import torch
    from paper_2306_08960_amd import binding as b
    from paper_2306_08960_amd import synth

    cfg = synth.CONFIGS[name]
    W, _, X, step = synth.make_layer(cfg)
    N, K, M = cfg.N, cfg.K, cfg.M
    step_w = float(np.std(W))
    w2 = b.apb_w2_pack(torch.from_numpy(W).cuda(), step_w)
    Xd = torch.from_numpy(X).cuda()
    packed = b.alloc_packed(K, M, 2)
    Y = torch.empty((N, M), dtype=torch.float32, device="cuda")
    s = float(step)

    def quant():
        b.apb_quantize_acts(Xd, 2, s, packed=packed)

    def gemm():
        b.apb_gemm_2_2(w2, packed, M, s, Y=Y)

    for _ in range(warmup):
        quant()
        gemm()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        quant()
        gemm()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / steps
    ms_quant, ms_gemm, ms_event_record = time_in_step(quant, gemm, steps, ms_step)
    ops = 2.0 * N * K * M
    Kw, Mp = (K + 31) // 32, 64 * ((M + 63) // 64)
    gemm_bytes = 8.0 * N * Kw + 8.0 * Kw * Mp + 4.0 * Mp + 4.0 * N * M
    t_hbm, t_mfma = gemm_bytes / (HBM_PEAK_GBS * 1e9), ops / (MFMA_FP4_PEAK_TFLOPS * 1e12)
    t = ms_gemm * 1e-3
    if t_hbm >= t_mfma:
        roof = {"kernel": "k_binary_mfma<2,2,...>", "bound": "hbm", "achieved": gemm_bytes / t / 1e9,
                "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    else:
        roof = {"kernel": "k_binary_mfma<2,2,...>", "bound": "mfma", "achieved": ops / t / 1e12,
                "peak": MFMA_FP4_PEAK_TFLOPS, "unit": "TFLOP/s"}
    roof |= {"frac": roof["achieved"] / roof["peak"], "traffic": None, "ms": ms_gemm,
             "floor_us": {"hbm": t_hbm * 1e6, "mfma_fp4": t_mfma * 1e6}}
    w2.free()
    res = {"workload": name, "N": N, "K": K, "M": M, "ms_per_step": ms_step, "ms_quantize": ms_quant, "ms_gemm": ms_gemm,
           "ms_event_record_removed": ms_event_record, "gops_step": ops / (ms_step * 1e-3) / 1e9,
           "gops_gemm": ops / t / 1e9, "roofline_gemm": roof}
    del Xd, packed, Y
    torch.cuda.empty_cache()
    return res, (cfg, W, step_w, X, step)


def run_chain(name, steps, warmup):
    """A layer in the middle of a network: its input arrives packed (written by the layer before) and its
    output leaves packed for the layer after.  Step = apb_forward_requant alone; beside it the two-call route
    to the same buffer, apb_forward (float Y to HBM) + apb_quantize_acts (Y read back)."""
    import torch
    from paper_2306_08960_amd import binding as b
    from paper_2306_08960_amd import synth

    cfg = synth.CONFIGS[name]
    W, delta, X, step = synth.make_layer(cfg)
    N, K, M, bits = cfg.N, cfg.K, cfg.M, cfg.bits
    layer = b.apb_compress(torch.from_numpy(W).cuda(), float(delta))
    nnz = layer.info()["nnz"]
    packed = b.apb_quantize_acts(torch.from_numpy(X).cuda(), bits, float(step))
    s = float(step)
    bits_out = bits
    step_out = float(0.03 * np.sqrt(K)) if bits_out == 2 else 1.0       # spreads Y over the four levels
    out_a = b.alloc_packed(N, M, bits_out)
    out_b = b.alloc_packed(N, M, bits_out)
    Y = torch.empty((N, M), dtype=torch.float32, device="cuda")

    def chained():
        b.apb_forward_requant(layer, packed, M, bits, s, bits_out, step_out, packed_out=out_a)

    def two_calls():
        b.apb_forward(layer, packed, M, bits, s, Y=Y)
        b.apb_quantize_acts(Y, bits_out, step_out, packed=out_b)

    def timed(fn):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    ms_chain, ms_two = timed(chained), timed(two_calls)
    # the chained call alone between HIP events on its stream, the cost of the records taken off as in time_in_step
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, c in ev:
        a.record()
        chained()
        c.record()
    torch.cuda.synchronize()
    per_record = max(0.0, ((time.perf_counter() - t0) * 1e3 / steps - ms_chain) / 2.0)
    ms_call = sum(a.elapsed_time(c) for a, c in ev) / steps - per_record
    same = bool(torch.equal(out_a, out_b))
    differing = int((out_a != out_b).sum().item())
    ops = 2.0 * N * K * M + 2.0 * nnz * M
    Kw, Mp, Nw = (K + 31) // 32, 64 * ((M + 63) // 64), (N + 31) // 32
    out_bytes = 4.0 * (bits_out * Nw + 1) * Mp
    # sign words, bit-planes, residual entries in; the packed output is stored once (layers of at most 128 rows)
    # or zero-filled, then read-modify-written
    fwd_bytes = 4.0 * N * Kw + 4.0 * bits * Kw * Mp + 4.0 * Mp + 12.0 * nnz + (1.0 if N <= 128 else 3.0) * out_bytes
    t_hbm = fwd_bytes / (HBM_PEAK_GBS * 1e9)
    t_mfma = 2.0 * N * K * M / (MFMA_FP4_PEAK_TFLOPS * 1e12)
    t_f64 = 2.0 * nnz * M / (FP64_VECTOR_PEAK_TFLOPS * 1e12)
    t = ms_call * 1e-3
    if t_hbm >= max(t_mfma, t_f64):
        roof = {"bound": "hbm", "achieved": fwd_bytes / t / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    elif t_mfma >= t_f64:
        roof = {"bound": "mfma", "achieved": 2.0 * N * K * M / t / 1e12, "peak": MFMA_FP4_PEAK_TFLOPS, "unit": "TFLOP/s"}
    else:
        roof = {"bound": "alu", "achieved": 2.0 * nnz * M / t / 1e12, "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s"}
    roof = {"kernel": "forward kernel with the packed-output epilogue (+ zero fill)"} | roof
    roof |= {"frac": roof["achieved"] / roof["peak"], "traffic": None, "ms": ms_call,
             "floor_us": {"hbm": t_hbm * 1e6, "mfma_fp4": t_mfma * 1e6, "fp64_vector": t_f64 * 1e6}}
    res = {"workload": name, "N": N, "K": K, "M": M, "act_bits": bits, "nnz": int(nnz), "ms_per_step": ms_chain,
           "gops_step": ops / (ms_chain * 1e-3) / 1e9, "ms_forward_plus_quantize": ms_two, "gops_forward_plus_quantize": ops / (ms_two * 1e-3) / 1e9,
           "same_packed_output": same, "words_differing": differing, "roofline": roof, "bits_out": bits_out, "step_out": step_out}
    layer.free()
    return res, (cfg, W, delta, X, step, bits_out, step_out)


# (batch, height, width) of the feature maps behind the benchmark's convolution layers (M = B*H*W, K = 9*C)
CONV_GEOMETRY = {"C2": (128, 32, 32), "C4": (64, 28, 28), "C5b": (256, 7, 7)} | {
    f"C3_r{r}_b{b_}": (128, 8, 8) for r in ("05", "20", "50") for b_ in (1, 2)}


def run_conv_chain(name, steps, warmup):
    """A 3x3 convolution layer in the middle of a network: packed feature map in, packed feature map out
    (apb_forward_conv3x3_requant; implicit im2col, no float activations in memory).  Beside it: the same
    layer as the benchmark's headline step runs it (apb_quantize_acts on the explicit float im2col matrix +
    apb_forward), and the convolution with a float output."""
    import torch
    from paper_2306_08960_amd import binding as b
    from paper_2306_08960_amd import synth

    cfg = synth.CONFIGS[name]
    B, H, W_ = CONV_GEOMETRY[name]
    Wt, delta = synth.make_weights(cfg)
    N, K, M, bits = cfg.N, cfg.K, cfg.M, cfg.bits
    C = K // 9
    assert M == B * H * W_ and K == 9 * C
    layer = b.apb_compress(torch.from_numpy(Wt).cuda(), float(delta))
    nnz = layer.info()["nnz"]
    g = torch.Generator(device="cuda").manual_seed(synth.BASE_SEED + cfg.index)
    Xmap = torch.randn((C, M), generator=g, device="cuda", dtype=torch.float32)
    if bits == 2:
        Xmap.clamp_(min=0)
    s = float(cfg.step)
    fmap = b.apb_quantize_acts(Xmap, bits, s)
    bits_out = bits
    step_out = float(0.03 * np.sqrt(K)) if bits_out == 2 else 1.0
    fmap_out = b.alloc_packed(N, M, bits_out)
    Y = torch.empty((N, M), dtype=torch.float32, device="cuda")
    # the explicit route's input: the float im2col matrix [K, M]
    pad = torch.full((C, B, H + 2, W_ + 2), 0.0 if bits == 2 else -1.0, device="cuda")
    pad[:, :, 1:H + 1, 1:W_ + 1] = Xmap.view(C, B, H, W_)
    X = torch.cat([pad[:, :, ky:ky + H, kx:kx + W_].reshape(C, M) for ky in range(3) for kx in range(3)], dim=0)
    del pad
    packed = b.alloc_packed(K, M, bits)

    def chained():
        b.apb_forward_conv3x3_requant(layer, fmap, B, H, W_, bits, s, bits_out, step_out, fmap_out=fmap_out)

    def conv_float():
        b.apb_forward_conv3x3(layer, fmap, B, H, W_, bits, s, Y=Y)

    def explicit():
        b.apb_quantize_acts(X, bits, s, packed=packed)
        b.apb_forward(layer, packed, M, bits, s, Y=Y)

    def timed(fn):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    ms_chain, ms_float, ms_explicit = timed(chained), timed(conv_float), timed(explicit)
    Y_conv = Y.clone()
    conv_float()
    same = bool(torch.equal(Y, Y_conv))                      # explicit and implicit routes, bit for bit
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, c in ev:
        a.record()
        chained()
        c.record()
    torch.cuda.synchronize()
    per_record = max(0.0, ((time.perf_counter() - t0) * 1e3 / steps - ms_chain) / 2.0)
    ms_call = sum(a.elapsed_time(c) for a, c in ev) / steps - per_record
    ops = 2.0 * N * K * M + 2.0 * nnz * M
    Kw, Mp, Cw, Nw = (K + 31) // 32, 64 * ((M + 63) // 64), C // 32, (N + 31) // 32
    out_bytes = 4.0 * (bits_out * Nw + 1) * Mp
    # sign words, the packed map (read once from HBM; its nine shifted views hit in cache), residual entries;
    # the packed output is stored once (layers of at most 128 rows) or zero-filled, then read-modify-written
    fwd_bytes = 4.0 * N * Kw + 4.0 * (bits * Cw + 1) * Mp + 12.0 * nnz + (1.0 if N <= 128 else 3.0) * out_bytes
    t_hbm = fwd_bytes / (HBM_PEAK_GBS * 1e9)
    t_mfma = 2.0 * N * K * M / (MFMA_FP4_PEAK_TFLOPS * 1e12)
    t_f64 = 2.0 * nnz * M / (FP64_VECTOR_PEAK_TFLOPS * 1e12)
    t = ms_call * 1e-3
    if t_hbm >= max(t_mfma, t_f64):
        roof = {"bound": "hbm", "achieved": fwd_bytes / t / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    elif t_mfma >= t_f64:
        roof = {"bound": "mfma", "achieved": 2.0 * N * K * M / t / 1e12, "peak": MFMA_FP4_PEAK_TFLOPS, "unit": "TFLOP/s"}
    else:
        roof = {"bound": "alu", "achieved": 2.0 * nnz * M / t / 1e12, "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s"}
    roof = {"kernel": "forward kernel, implicit im2col + packed-output epilogue (+ zero fill)"} | roof
    roof |= {"frac": roof["achieved"] / roof["peak"], "traffic": None, "ms": ms_call,
             "floor_us": {"hbm": t_hbm * 1e6, "mfma_fp4": t_mfma * 1e6, "fp64_vector": t_f64 * 1e6}}
    t_valu = (2.0 * bits * N * Kw * M + float(nnz) * M) / VALU_LANE_OPS_PER_S
    res = {"workload": name, "N": N, "C": C, "B": B, "H": H, "W": W_, "act_bits": bits, "nnz": int(nnz),
           "ms_per_step": ms_chain, "gops_step": ops / (ms_chain * 1e-3) / 1e9,
           "ms_conv_float_output": ms_float, "ms_explicit_im2col_quantize_plus_forward": ms_explicit,
           "implicit_equals_explicit_bitwise": same, "roofline": roof, "bits_out": bits_out, "step_out": step_out,
           "frac_of_valu_bitop_roof": t_valu / t}
    layer.free()
    return res, cfg


def cpu_baseline_conv_chain(cfg, B, H, W_, bits_out, step_out):
    """The CPU oracle of the chained convolution (im2col of the quantized map, forward, re-quantize, pack) on
    the first images of the batch."""
    from oracle import apb_oracle as o
    from oracle import capi
    from paper_2306_08960_amd import synth
    cores = max(1, min(len(os.sched_getaffinity(0)), capi.max_threads()))
    Wt, delta = synth.make_weights(cfg)
    L = o.compress(Wt, delta)
    nnz = int(L["row_ptr"][-1])
    C = cfg.K // 9
    per_col = 2.0 * cfg.N * cfg.K + 2.0 * nnz
    images = int(max(1, min(B, 60e9 * cores ** 0.5 / per_col / (H * W_))))
    m = images * H * W_
    Xmap = np.random.default_rng(cfg.index).standard_normal((C, m)).astype(np.float32)
    if cfg.bits == 2:
        np.maximum(Xmap, 0, out=Xmap)
    c_map = o.quantize(Xmap, cfg.bits, np.float32(cfg.step))
    passes, dt = 0, 0.0
    while passes == 0 or (dt < 1.0 and passes < 20):
        t0 = time.perf_counter()
        patches = o.im2col_codes(c_map, images, H, W_, cfg.bits)
        F = capi.forward(L, o.pack_acts(patches, cfg.bits), patches, cfg.bits, np.float32(cfg.step), threads=cores)
        o.requant(L["alpha"], np.float32(cfg.step), F["D"], F["R"], bits_out, np.float32(step_out))
        dt += time.perf_counter() - t0
        passes += 1
    return {"value": per_col * m * passes / dt / 1e9, "unit": "GOPS", "cores": cores, "kind": "oracle",
            "sample": f"first {images} of {B} images of {cfg.name}, {passes} passes (im2col of the codes + pack + forward + "
                      f"requantize + pack), {dt:.2f} s"}


def cpu_baseline_chain(cfg, W, delta, X, step, bits_out, step_out):
    """The CPU oracle of the chained step (forward from packed codes, re-quantize, pack) on the first columns."""
    from oracle import apb_oracle as o
    from oracle import capi
    cores = max(1, min(len(os.sched_getaffinity(0)), capi.max_threads()))
    L = o.compress(W, delta)
    nnz = int(L["row_ptr"][-1])
    per_col = 2.0 * cfg.N * cfg.K + 2.0 * nnz
    m = int(max(64, min(cfg.M, 60e9 * cores ** 0.5 / per_col)))
    c = o.quantize(np.ascontiguousarray(X[:, :m]), cfg.bits, step)
    packed = o.pack_acts(c, cfg.bits)
    passes, dt = 0, 0.0
    while passes == 0 or (dt < 1.0 and passes < 20):
        t0 = time.perf_counter()
        F = capi.forward(L, packed, c, cfg.bits, step, threads=cores)
        o.requant(L["alpha"], step, F["D"], F["R"], bits_out, np.float32(step_out))
        dt += time.perf_counter() - t0
        passes += 1
    return {"value": per_col * m * passes / dt / 1e9, "unit": "GOPS", "cores": cores, "kind": "oracle",
            "sample": f"first {m} of {cfg.M} columns of {cfg.name}, {passes} passes (forward+requantize+pack), {dt:.2f} s"}


def run_square_sweep(sizes=(512, 1024, 2048, 4096, 8192), iters=30):
    """The paper's efficiency protocol (square matrices, the product alone, operands already packed) for
    its three bitwise routines: 1/1 and 1/2 are a binary layer without residuals (integer part D through
    apb_forward_int), 2/2 is apb_gemm_2_2_int.  Seeded normal weights, ReLU-normal activations."""
    import torch
    from paper_2306_08960_amd import binding as b
    rows = []
    for n in sizes:
        g = torch.Generator(device="cuda").manual_seed(230608960 + n)
        W = torch.randn((n, n), generator=g, device="cuda") * 0.05
        X = torch.relu(torch.randn((n, n), generator=g, device="cuda"))
        layer = b.apb_compress(W, float("inf"), alpha=0.05)
        w2 = b.apb_w2_pack(W, 0.05)
        p1 = b.apb_quantize_acts(X - 0.5, 1, 1.0)
        p2 = b.apb_quantize_acts(X, 2, 0.75)
        D = torch.empty((n, n), dtype=torch.int32, device="cuda")

        def timed(fn):
            for _ in range(3):
                fn()
            a, c = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            a.record()
            for _ in range(iters):
                fn()
            c.record()
            c.synchronize()
            return a.elapsed_time(c) / iters

        t11 = timed(lambda: b.apb_forward_int(layer, p1, n, 1, D=D))
        t12 = timed(lambda: b.apb_forward_int(layer, p2, n, 2, D=D))
        t22 = timed(lambda: b.apb_gemm_2_2_int(w2, p2, n, D=D))
        ops = 2.0 * n ** 3
        rows.append({"n": n, "ms_1_1": t11, "ms_1_2": t12, "ms_2_2": t22,
                     "tops_1_1": ops / t11 / 1e9, "tops_1_2": ops / t12 / 1e9, "tops_2_2": ops / t22 / 1e9,
                     "cost_1_2_over_1_1": t12 / t11, "cost_2_2_over_1_1": t22 / t11})
        layer.free()
        w2.free()
        del W, X, p1, p2, D
        torch.cuda.empty_cache()
    return rows


def cpu_baseline_2_2(cfg, W, step_w, X, step):
    """The CPU oracle of the 2/2 routine (quantize both operands, integer product, scaling) on the
    first columns of the workload; the product is a float64 library matmul on all host cores."""
    from oracle import apb_oracle as o
    cores = max(1, len(os.sched_getaffinity(0)))
    m = int(max(64, min(cfg.M, 20e9 * cores ** 0.5 / (2.0 * cfg.N * cfg.K))))
    Xs = np.ascontiguousarray(X[:, :m])
    t0 = time.perf_counter()
    o.gemm_2_2(o.quantize_weights_2bit(W, step_w), o.quantize(Xs, 2, step), step_w, step)
    dt = time.perf_counter() - t0
    return {"value": 2.0 * cfg.N * cfg.K * m / dt / 1e9, "unit": "GOPS", "cores": cores, "kind": "oracle",
            "sample": f"first {m} of {cfg.M} columns of {cfg.name}, one pass (quantize both operands + product), {dt:.2f} s"}


def cpu_baseline(cfg, W, delta, X, step):
    """The CPU oracle (quantize, pack, popcount integer part, CSR part, epilogue) on the first
    columns of the same workload, all host cores this process may use."""
    from oracle import apb_oracle as o
    from oracle import capi
    cores = max(1, min(len(os.sched_getaffinity(0)), capi.max_threads()))
    L = o.compress(W, delta)
    nnz = int(L["row_ptr"][-1])
    per_col = 2.0 * cfg.N * cfg.K + 2.0 * nnz
    target_ops = 60e9 * cores ** 0.5                 # sized for roughly 10-30 s of CPU work
    m = int(max(64, min(cfg.M, target_ops / per_col)))
    Xs = np.ascontiguousarray(X[:, :m])
    passes, dt = 0, 0.0
    while passes == 0 or (dt < 1.0 and passes < 20):    # about 10-30 core-seconds in all
        t0 = time.perf_counter()
        c = o.quantize(Xs, cfg.bits, step)
        packed = o.pack_acts(c, cfg.bits)
        capi.forward(L, packed, c, cfg.bits, step, threads=cores)
        dt += time.perf_counter() - t0
        passes += 1
    return {"value": per_col * m * passes / dt / 1e9, "unit": "GOPS", "cores": cores, "kind": "oracle",
            "sample": f"first {m} of {cfg.M} columns of {cfg.name}, {passes} passes (quantize+pack+forward), {dt:.2f} s"}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the layer shards over the columns of X with no "
              "exchange between GPUs, so one GPU shows the whole path). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2306_08960_amd import binding as b
    from paper_2306_08960_amd import synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    b.load()
    if args.workload not in synth.CONFIGS:
        print(f"bench.py: unknown workload {args.workload}; choose from {sorted(synth.CONFIGS)}", file=sys.stderr)
        sys.exit(2)

    if args.sweep:
        print(json.dumps({"metric": "square-matrix sweep of the bitwise products (integer part alone, operands packed)",
                          "unit": "TOPS (2*n^3 / time)", "n_gpus": 1, "data": "synthetic",
                          "note": "1/1 and 1/2: apb_forward_int on a layer without residuals; 2/2: apb_gemm_2_2_int; "
                                  "the paper predicts cost ratios 2 and 8 on a popcount machine",
                          "sweep": run_square_sweep()}))
        return
    if args.routine == "gemm_2_2":
        res, inputs = run_gemm_2_2(args.workload, args.steps, args.warmup)
        cfg = inputs[0]
        quant_bytes = 4.0 * cfg.K * cfg.M + 8.0 * ((cfg.K + 31) // 32) * 64 * ((cfg.M + 63) // 64) + 4.0 * 64 * ((cfg.M + 63) // 64)
        roof_q = {"kernel": "k_quantize_pack", "bound": "hbm", "achieved": quant_bytes / (res["ms_quantize"] * 1e-3) / 1e9,
                  "peak": HBM_PEAK_GBS, "unit": "GB/s", "traffic": None, "ms": res["ms_quantize"]}
        roof_q["frac"] = roof_q["achieved"] / roof_q["peak"]
        out = {
            "metric": "2/2 GEMM (2-bit weights x 2-bit activations, Sec. IV) GOPS", "value": res["gops_step"],
            "unit": "GOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "fp4 (exact 2-bit codes) on MFMA, f32 out", "data": "synthetic",
            "config": {"workload": f"{cfg.name}: {cfg.note}", "N": cfg.N, "K": cfg.K, "M": cfg.M,
                       "step": "apb_quantize_acts (2 bits) + apb_gemm_2_2, inputs resident in HBM, weights packed offline"},
            "ms_quantize": res["ms_quantize"], "ms_gemm": res["ms_gemm"], "gops_gemm_only": res["gops_gemm"],
            "ms_event_record_removed": res["ms_event_record_removed"],
            "roofline": roof_q if res["ms_quantize"] >= res["ms_gemm"] else res["roofline_gemm"],
            "roofline_gemm": res["roofline_gemm"], "roofline_quantize": roof_q,
        }
        if not args.no_cpu_baseline:
            out["cpu_baseline"] = cpu_baseline_2_2(*inputs)
        print(json.dumps(out))
        return

    if args.routine == "conv_chain":
        if args.workload not in CONV_GEOMETRY:
            print(f"bench.py: {args.workload} is not a convolution layer; choose from {sorted(CONV_GEOMETRY)}", file=sys.stderr)
            sys.exit(2)
        res, cfg = run_conv_chain(args.workload, args.steps, args.warmup)
        cpu = None if args.no_cpu_baseline else cpu_baseline_conv_chain(cfg, res["B"], res["H"], res["W"], res["bits_out"],
                                                                         res["step_out"])
        print(json.dumps({
            "metric": "APB 3x3 conv layer GOPS, chained (packed feature map in, packed feature map out)",
            "value": res["gops_step"], "unit": "GOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "fp4 (exact 0/1 and 2-bit codes) on MFMA + f64 accumulate, packed codes in/out", "data": "synthetic",
            "config": {"workload": f"{cfg.name}: {cfg.note}", "N": res["N"], "C": res["C"], "B": res["B"], "H": res["H"],
                       "W": res["W"], "act_bits": cfg.bits, "outlier_rate": cfg.rho, "nnz": res["nnz"],
                       "bits_out": res["bits_out"], "step_out": res["step_out"],
                       "step": "apb_forward_conv3x3_requant, packed input map resident in HBM"},
            "ms_conv_float_output": res["ms_conv_float_output"],
            "ms_explicit_im2col_quantize_plus_forward": res["ms_explicit_im2col_quantize_plus_forward"],
            "implicit_equals_explicit_bitwise": res["implicit_equals_explicit_bitwise"],
            "frac_of_valu_bitop_roof": res["frac_of_valu_bitop_roof"], "roofline": res["roofline"]}
            | ({} if cpu is None else {"cpu_baseline": cpu})))
        return
    if args.routine == "chain":
        res, inputs = run_chain(args.workload, args.steps, args.warmup)
        cfg = inputs[0]
        out = {
            "metric": "APB layer forward GOPS, chained (packed activations in, packed activations out)",
            "value": res["gops_step"], "unit": "GOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "fp4 (exact 0/1 and 2-bit codes) on MFMA + f64 accumulate, packed codes in/out", "data": "synthetic",
            "config": {"workload": f"{cfg.name}: {cfg.note}", "N": cfg.N, "K": cfg.K, "M": cfg.M, "act_bits": cfg.bits,
                       "outlier_rate": cfg.rho, "nnz": res["nnz"], "bits_out": res["bits_out"], "step_out": res["step_out"],
                       "step": "apb_forward_requant, packed input resident in HBM"},
            "ms_forward_plus_quantize": res["ms_forward_plus_quantize"],
            "gops_forward_plus_quantize": res["gops_forward_plus_quantize"],
            "same_packed_output_as_two_calls": res["same_packed_output"], "words_differing": res["words_differing"],
            "roofline": res["roofline"],
        }
        if not args.no_cpu_baseline:
            out["cpu_baseline"] = cpu_baseline_chain(*inputs)
        print(json.dumps(out))
        return

    res, inputs = run_workload(args.workload, args.steps, args.warmup, args.calibration_copy)
    cfg = inputs[0]
    out = {
        "metric": "APB layer forward GOPS (binary+sparse) and % of MI355X roofline",
        "value": res["gops_step"], "unit": "GOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp4 (exact 0/1 and 2-bit codes) on MFMA + f64 accumulate (f32 in/out)", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.note}", "N": cfg.N, "K": cfg.K, "M": cfg.M,
                   "act_bits": cfg.bits, "outlier_rate": cfg.rho, "nnz": res["nnz"],
                   "step": "apb_quantize_forward (= apb_quantize_acts + apb_forward; one kernel for layers of at most "
                           "128 rows), inputs resident in HBM", "one_kernel_step": res["one_kernel_step"]},
        "ms_per_step_two_calls": res["ms_per_step_two_calls"],
        "ms_quantize": res["ms_quantize"], "ms_forward": res["ms_forward"],
        "ms_event_record_removed": res["ms_event_record_removed"],
        "gops_forward_only": res["gops_forward"],
        "roofline": res["roofline"], "roofline_forward": res["roofline_forward"],
        "roofline_forward_valu_bitop": res["roofline_forward_valu_bitop"],
        "roofline_quantize": res["roofline_quantize"],
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(*inputs)
    del inputs
    if args.all:
        others = []
        for name in synth.CONFIGS:
            if name == args.workload:
                continue
            r, _ = run_workload(name, max(20, args.steps // 4), max(5, args.warmup // 4))
            others.append({k: r[k] for k in ("workload", "N", "K", "M", "act_bits", "nnz", "ms_per_step", "gops_step",
                                             "one_kernel_step", "ms_per_step_two_calls",
                                             "ms_quantize", "ms_forward", "gops_forward")}
                          | {"forward_frac_of_valu_bitop_roof": r["roofline_forward_valu_bitop"]["frac"],
                             "forward_bound": r["roofline_forward"]["bound"],
                             "forward_frac_of_roof": r["roofline_forward"]["frac"],
                             "quantize_frac_of_hbm_roof": r["roofline_quantize"]["frac"]})
        out["others"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
