#!/usr/bin/env python3
"""Benchmark of the APB layer forward pass on one MI355X.

One "step" = the whole per-batch hot path on inputs already resident in HBM: quantize + bit-plane
packing of the activations, then the forward (binary product on the matrix cores, residual part,
epilogue), through the one entry point apb_quantize_forward.  apb_compress is per-layer offline work
and is not timed.

Prints ONE JSON line.  `value` is (2*N*K*M + 2*nnz*M) / step time, in GOPS, for the workload named
in config.workload (default: C5b, the largest layer of the benchmark); `roofline` describes the kernel
that dominates that step; `others` holds the same measurements for every other benchmark layer;
`cpu_baseline` is the CPU oracle timed on a bounded column sample of the headline workload on this
box's host cores.

How times are taken.  `ms_per_step` is the wall clock over the timed steps (launches from Python,
synchronised on both sides).  Kernel-level figures (`ms_forward`, `ms_quantize`, `ms_step_graph`, every
`roofline.ms`) are replays of a captured HIP graph that holds several launches, between two HIP events
recorded on the stream the graph replays on: no host launch gaps, nothing subtracted, nothing
estimated.  `roofline.traffic` is read from profiles/traffic_<workload>_pmc.txt when that file has a
figure for the kernel, else null.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0                  # MI355X HBM3E, published
MFMA_FP4_PEAK_TFLOPS = 10100.0         # dense FP4 MFMA, published
FP64_VECTOR_PEAK_TFLOPS = 78.6         # 256 CUs x 64 lanes x 2.4 GHz x 2 (fused multiply-add)
VALU_LANE_OPS_PER_S = 256 * 64 * 2.4e9 # 39.3e12 32-bit vector lane-ops/s: the bit-op roof of a popcount formulation

HEADLINE = "C5b"
NO_GRAPH = False                       # --no-graph


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=HEADLINE, help="name in paper_2306_08960_amd.synth.CONFIGS")
    ap.add_argument("--no-others", action="store_true", help="time the headline workload only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true",
                    help="time kernels with a short loop of plain launches between two events instead of graph replays "
                         "(few dispatches: for rocprofv3 --pmc runs, which serialise every dispatch)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="before the steps, copy X into a buffer of the same size three times: a plain copy kernel of "
                         "known size, against which FETCH_SIZE / WRITE_SIZE of a rocprofv3 --pmc run are scaled")
    ap.add_argument("--sweep", action="store_true",
                    help="square-matrix sweep of the three bitwise products (1/1, 1/2, 2/2; Sec. V protocol): one JSON "
                         "line with the time of the product alone at each size")
    ap.add_argument("--routine", default="apb",
                    choices=["apb", "gemm_2_2", "chain", "conv_chain", "popcount_vs_mfma", "peaks", "resnet18",
                             "rho_sweep", "train"],
                    help="apb: the APB layer forward (the headline metric); gemm_2_2: the 2-bit x 2-bit product of "
                         "Sec. IV on the same shapes; chain / conv_chain: a layer inside a network (packed in, packed "
                         "out); popcount_vs_mfma: the binary part in its two formulations on the same inputs; peaks: "
                         "register-only instruction-rate probes; resnet18: the 3x3 layers of an ImageNet ResNet-18 as "
                         "im2col products (Sec. V-B protocol); rho_sweep: forward time against the outlier rate "
                         "(Sec. V-C crossover); train: the training-side kernels (Sec. III Eqs. 3-9)")
    return ap.parse_args()


def graph_ms(fn, reps=None, target_ms=30.0):
    """Milliseconds per call of fn(): `reps` calls recorded into one HIP graph, which is then replayed between
    two HIP events on the current stream.  Launches inside a graph follow one another without host gaps, so
    a kernel of a few microseconds is timed as the GPU runs it; nothing is subtracted from the interval."""
    import torch
    for _ in range(3):
        fn()                                   # first launches load code objects and set launch attributes
    torch.cuda.synchronize()
    a, c = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(5):
        fn()
    c.record()
    c.synchronize()
    rough = max(a.elapsed_time(c) / 5, 1e-3)   # upper estimate (host gaps included), only to size the graph
    if NO_GRAPH:
        return rough
    if reps is None:
        reps = int(min(50, max(4, 2.0 / rough)))
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(reps):
            fn()
    g.replay()
    torch.cuda.synchronize()
    replays = int(min(200, max(3, target_ms / (rough * reps))))
    a.record()
    for _ in range(replays):
        g.replay()
    c.record()
    c.synchronize()
    ms = a.elapsed_time(c) / (replays * reps)
    del g
    return ms


def wall_ms(fn, steps, warmup):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def measured_traffic(workload, kernel_key):
    """Bytes per launch from profiles/traffic_<workload>_pmc.txt: a line `traffic_bytes <kernel_key> <number>`
    written from calibrated rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs.  None when there is no such line."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}_pmc.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        m = re.match(r"\s*traffic_bytes\s+(\S+)\s+([0-9.eE+]+)", line)
        if m and m.group(1) == kernel_key:
            return float(m.group(2))
    return None


def forward_floors(N, K, M, bits, nnz):
    """Seconds the forward kernel cannot go below: the bytes it must move (sign words, bit-planes, residual
    entries, Y) at the HBM peak, the binary product at the FP4 matrix-core peak, the residual multiply-adds
    at the float64 vector peak; and the yardstick the benchmark spec names, the vector-ALU bit-op time of
    the popcount formulation (per weight word, plane and column one logic op + one accumulating popcount,
    per residual and column one multiply-add)."""
    Kw, Mp = (K + 31) // 32, 64 * ((M + 63) // 64)
    fwd_bytes = 4.0 * N * Kw + 4.0 * bits * Kw * Mp + 4.0 * Mp + 12.0 * nnz + 4.0 * N * M
    return {"hbm": fwd_bytes / (HBM_PEAK_GBS * 1e9), "mfma_fp4": 2.0 * N * K * M / (MFMA_FP4_PEAK_TFLOPS * 1e12),
            "fp64_vector": 2.0 * nnz * M / (FP64_VECTOR_PEAK_TFLOPS * 1e12),
            "valu_bitop_yardstick": (2.0 * bits * N * Kw * M + float(nnz) * M) / VALU_LANE_OPS_PER_S}, fwd_bytes


def forward_roofline(N, K, M, bits, nnz, ms, kernel, traffic=None):
    fl, fwd_bytes = forward_floors(N, K, M, bits, nnz)
    t = ms * 1e-3
    if fl["hbm"] >= max(fl["mfma_fp4"], fl["fp64_vector"]):
        roof = {"bound": "hbm", "achieved": fwd_bytes / t / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    elif fl["mfma_fp4"] >= fl["fp64_vector"]:
        roof = {"bound": "mfma", "achieved": 2.0 * N * K * M / t / 1e12, "peak": MFMA_FP4_PEAK_TFLOPS, "unit": "TFLOP/s"}
    else:
        roof = {"bound": "alu", "achieved": 2.0 * nnz * M / t / 1e12, "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s"}
    roof = {"kernel": kernel} | roof
    roof |= {"frac": roof["achieved"] / roof["peak"], "traffic": traffic, "ms": ms,
             "floor_us": {k: v * 1e6 for k, v in fl.items() if k != "valu_bitop_yardstick"},
             "valu_bitop_yardstick_us": fl["valu_bitop_yardstick"] * 1e6,
             "frac_of_valu_bitop_yardstick": fl["valu_bitop_yardstick"] / t}
    return roof


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

    def one_call():                          # the step: quantize + forward through the single entry point
        b.apb_quantize_forward(layer, Xd, bits, s, packed=packed, Y=Y)

    one_kernel = b.apb_quantize_forward_is_one_kernel(layer, M, bits)
    ms_step = wall_ms(one_call, steps, warmup)
    ms_step_graph = graph_ms(one_call)
    quant()
    ms_fwd = graph_ms(fwd)
    ms_quant = graph_ms(quant)
    # The forward kernel as it runs INSIDE a step, right after the quantize kernel has streamed X through the caches
    # (launched alone back to back it finds the planes and the layer in its L2): HIP events on the launch stream
    # around the forward launch of every timed step of the two-call route; the interval includes the dispatch gap
    # between the two kernels, nothing is subtracted.
    ms_fwd_in_step = ms_quant_in_step = None
    if not one_kernel:
        for _ in range(warmup):
            quant()
            fwd()
        ev = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(3)) for _ in range(steps)]
        torch.cuda.synchronize()
        for e0, e1, e2 in ev:
            e0.record()
            quant()
            e1.record()
            fwd()
            e2.record()
        torch.cuda.synchronize()
        ms_quant_in_step = sum(e0.elapsed_time(e1) for e0, e1, _ in ev) / steps
        ms_fwd_in_step = sum(e1.elapsed_time(e2) for _, e1, e2 in ev) / steps

    ops = 2.0 * N * K * M + 2.0 * nnz * M
    Kw, Mp = (K + 31) // 32, 64 * ((M + 63) // 64)
    # quantize: reads X once, writes the bit-planes and the column sums
    quant_bytes = 4.0 * K * M + 4.0 * bits * Kw * Mp + 4.0 * Mp
    roof_quant = {"kernel": "k_quantize_pack", "bound": "hbm", "achieved": quant_bytes / (ms_quant * 1e-3) / 1e9,
                  "peak": HBM_PEAK_GBS, "unit": "GB/s", "traffic": measured_traffic(name, "k_quantize_pack"),
                  "algorithmic_bytes": quant_bytes, "ms": ms_quant,
                  "note": "launched alone back to back: where X is smaller than the 256 MB memory-side cache part of "
                          "it survives between launches; ms_quantize_in_step is the figure inside the step"}
    roof_quant["frac"] = roof_quant["achieved"] / roof_quant["peak"]
    roof_fwd = forward_roofline(N, K, M, bits, nnz, ms_fwd, b.apb_forward_kernel_name(layer, M, bits),
                                measured_traffic(name, "forward"))
    # Layers of at most 128 rows run the step as ONE kernel (quantize into LDS + forward): it reads X and the
    # layer and writes Y, nothing else, so its floor is those bytes at the HBM peak.
    one_bytes = 4.0 * K * M + 4.0 * N * M + 4.0 * N * Kw + 12.0 * nnz
    roof_one = {"kernel": b.apb_forward_kernel_name(layer, M, bits).replace("false>", "true>") +
                          " (float input: quantize + forward in one kernel)", "bound": "hbm",
                "achieved": one_bytes / (ms_step_graph * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "traffic": measured_traffic(name, "one_kernel_step"),
                "algorithmic_bytes": one_bytes, "ms": ms_step_graph}
    roof_one["frac"] = roof_one["achieved"] / roof_one["peak"]
    if one_kernel:
        dominant = roof_one
    else:                                    # the longer of the two kernels of the step, as timed inside the step
        roof_fwd_in_step = forward_roofline(N, K, M, bits, nnz, ms_fwd_in_step, b.apb_forward_kernel_name(layer, M, bits),
                                            measured_traffic(name, "forward")) | {
            "timed": "HIP events around the forward launch inside each timed step (after the quantize kernel)"}
        dominant = roof_fwd_in_step if ms_fwd_in_step >= ms_quant_in_step else roof_quant | {
            "ms": ms_quant_in_step, "achieved": quant_bytes / (ms_quant_in_step * 1e-3) / 1e9,
            "frac": quant_bytes / (ms_quant_in_step * 1e-3) / 1e9 / HBM_PEAK_GBS}
    res = {
        "workload": name, "N": N, "K": K, "M": M, "act_bits": bits, "nnz": int(nnz),
        "ms_per_step": ms_step, "gops_step": ops / (ms_step * 1e-3) / 1e9, "one_kernel_step": bool(one_kernel),
        "ms_step_graph": ms_step_graph, "gops_step_graph": ops / (ms_step_graph * 1e-3) / 1e9,
        "ms_quantize": ms_quant, "ms_quantize_in_step": ms_quant_in_step, "ms_forward": ms_fwd,
        "ms_forward_in_step": ms_fwd_in_step,
        "gops_forward": ops / (ms_fwd * 1e-3) / 1e9,
        "roofline": dominant, "roofline_forward": roof_fwd, "roofline_quantize": roof_quant,
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

    def both():
        quant()
        gemm()

    ms_step = wall_ms(both, steps, warmup)
    ms_quant, ms_gemm = graph_ms(quant), graph_ms(gemm)
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
           "gops_step": ops / (ms_step * 1e-3) / 1e9,
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

    ms_chain, ms_two = wall_ms(chained, steps, warmup), wall_ms(two_calls, steps, warmup)
    ms_call = graph_ms(chained)              # the chained call alone, graph replay between HIP events
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

    # the step is called with a workspace of apb_acts_bytes(K, M, bits): layers with many residuals per row write
    # the packed patch matrix there and multiply it as a plain matrix, the others gather inside the kernel
    workspace = b.alloc_packed(K, M, bits)
    takes_patch_route = b.apb_forward_kernel_name(layer, M, bits).startswith("k_forward_rows")

    def chained():
        b.apb_forward_conv3x3_requant(layer, fmap, B, H, W_, bits, s, bits_out, step_out, fmap_out=fmap_out,
                                      workspace=workspace)

    def chained_gather():
        b.apb_forward_conv3x3_requant(layer, fmap, B, H, W_, bits, s, bits_out, step_out, fmap_out=fmap_out)

    def conv_float():
        b.apb_forward_conv3x3(layer, fmap, B, H, W_, bits, s, Y=Y, workspace=workspace)

    def explicit():
        b.apb_quantize_acts(X, bits, s, packed=packed)
        b.apb_forward(layer, packed, M, bits, s, Y=Y)

    ms_chain, ms_float, ms_explicit = (wall_ms(f, steps, warmup) for f in (chained, conv_float, explicit))
    Y_conv = Y.clone()
    conv_float()
    same = bool(torch.equal(Y, Y_conv))                      # explicit and implicit routes, bit for bit
    ms_call = graph_ms(chained)
    ms_call_gather = graph_ms(chained_gather) if takes_patch_route else ms_call
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
    roof = {"kernel": ("packed patch matrix + rows-in-lanes forward kernel with the packed-output epilogue (+ zero fill)"
                       if takes_patch_route else
                       "forward kernel, implicit im2col + packed-output epilogue (+ zero fill)")} | roof
    roof |= {"frac": roof["achieved"] / roof["peak"], "traffic": None, "ms": ms_call,
             "floor_us": {"hbm": t_hbm * 1e6, "mfma_fp4": t_mfma * 1e6, "fp64_vector": t_f64 * 1e6}}
    t_valu = (2.0 * bits * N * Kw * M + float(nnz) * M) / VALU_LANE_OPS_PER_S
    res = {"workload": name, "N": N, "C": C, "B": B, "H": H, "W": W_, "act_bits": bits, "nnz": int(nnz),
           "ms_per_step": ms_chain, "gops_step": ops / (ms_chain * 1e-3) / 1e9,
           "packed_patch_route": takes_patch_route, "ms_step_graph": ms_call, "ms_step_graph_gather_in_kernel": ms_call_gather,
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


def run_square_sweep(sizes=(512, 1024, 2048, 4096, 8192)):
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

        timed = graph_ms                       # (launches back to back in a replayed graph: no host gaps at small n)

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


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg, W, delta, X, step):
    """The CPU oracle as it stands, timed on this machine's host cores on the first columns of the workload:
    the packed forward of the C oracle (popcount integer part over packed words, CSR part, float64 epilogue --
    the activations are quantized and packed beforehand, outside the timed region, as they are resident
    and packed for the GPU's forward kernel too) single-threaded and on all cores this process may use, and the
    numpy quantize + pack step on its own.  The plain dense definition (brute force) is timed on C1."""
    from oracle import apb_oracle as o
    from oracle import capi
    from paper_2306_08960_amd import synth
    cores = max(1, min(len(os.sched_getaffinity(0)), capi.max_threads()))
    L = o.compress(W, delta)
    nnz = int(L["row_ptr"][-1])
    per_col = 2.0 * cfg.N * cfg.K + 2.0 * nnz
    m = int(max(64, min(cfg.M, 12e9 / per_col)))        # a few seconds single-threaded
    Xs = np.ascontiguousarray(X[:, :m])
    t0 = time.perf_counter()
    c = o.quantize(Xs, cfg.bits, step)
    packed = o.pack_acts(c, cfg.bits)
    dt_pack = time.perf_counter() - t0

    def leg(threads, budget_s, max_passes):
        passes, dt = 0, 0.0
        while passes == 0 or (dt < budget_s and passes < max_passes):
            t0 = time.perf_counter()
            capi.forward(L, packed, c, cfg.bits, step, threads=threads)
            dt += time.perf_counter() - t0
            passes += 1
        return per_col * m * passes / dt / 1e9, passes, dt

    g1, p1, d1 = leg(1, 0.0, 1)                          # one repetition
    gN, pN, dN = leg(cores, 3.0, 20)                     # at least three where they are short
    # the plain definition on C1 (dense float64 product with the reconstructed weights)
    c1 = synth.CONFIGS["C1"]
    W1, delta1, X1, step1 = synth.make_layer(c1)
    a1 = o.default_alpha(W1, delta1)
    t0 = time.perf_counter()
    reps = 20
    for _ in range(reps):
        o.brute_force(W1, delta1, a1, X1, c1.bits, step1)
    dt_bf = (time.perf_counter() - t0) / reps
    return {"value": gN, "unit": "GOPS", "cores": cores, "kind": "oracle", "cpu_model": cpu_model(),
            "sample": f"first {m} of {cfg.M} columns of {cfg.name}: packed forward of the C oracle (integer part, CSR "
                      f"part, epilogue), {pN} passes on {cores} threads in {dN:.2f} s",
            "single_thread": {"value": g1, "unit": "GOPS", "cores": 1,
                              "sample": f"same columns, {p1} pass in {d1:.2f} s"},
            "quantize_and_pack_numpy": {"seconds": dt_pack, "sample": f"same columns, once, outside the timed forward"},
            "brute_force_C1": {"value": 2.0 * c1.N * c1.K * c1.M / dt_bf / 1e9, "unit": "GOPS", "ms": dt_bf * 1e3,
                               "sample": f"C1 ({c1.N}x{c1.K}, M={c1.M}): dense float64 product with the "
                                         f"reconstructed weights, mean of {reps} passes (numpy matmul, library threads)"}}


def main():
    global NO_GRAPH
    args = parse_args()
    NO_GRAPH = args.no_graph
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
                       "step": "apb_forward_conv3x3_requant with a workspace, packed input map resident in HBM",
                       "packed_patch_route": res["packed_patch_route"]},
            "ms_step_graph": res["ms_step_graph"], "ms_step_graph_gather_in_kernel": res["ms_step_graph_gather_in_kernel"],
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

    if args.routine != "apb":
        EXTRA_ROUTINES[args.routine](args)
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
        "ms_step_graph": res["ms_step_graph"], "gops_step_graph": res["gops_step_graph"],
        "ms_quantize": res["ms_quantize"], "ms_quantize_in_step": res["ms_quantize_in_step"],
        "ms_forward": res["ms_forward"], "ms_forward_in_step": res["ms_forward_in_step"], "gops_forward_only": res["gops_forward"],
        "roofline": res["roofline"], "roofline_forward": res["roofline_forward"],
        "roofline_quantize": res["roofline_quantize"],
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(*inputs)
    del inputs
    if not args.no_others:
        others = []
        for name in synth.CONFIGS:
            if name == args.workload:
                continue
            r, _ = run_workload(name, max(20, args.steps // 4), max(5, args.warmup // 4))
            rf = r["roofline_forward"]
            others.append({k: r[k] for k in ("workload", "N", "K", "M", "act_bits", "nnz", "ms_per_step", "gops_step",
                                             "one_kernel_step", "ms_step_graph", "gops_step_graph", "ms_quantize",
                                             "ms_quantize_in_step", "ms_forward", "ms_forward_in_step", "gops_forward")}
                          | {"roofline": {k: r["roofline"][k] for k in ("kernel", "bound", "achieved", "peak", "unit",
                                                                        "frac", "traffic", "ms")},
                             "roofline_forward": {k: rf[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic",
                                                                     "ms", "floor_us", "frac_of_valu_bitop_yardstick")},
                             "quantize_frac_of_hbm_roof": r["roofline_quantize"]["frac"]})
        out["others"] = others
    print(json.dumps(out))


def routine_popcount_vs_mfma(args):
    """The binary part in its two formulations on the same packed inputs: the paper's and/xor + popcount on the
    vector ALU (apb_forward_int_popcount) against the FP4 matrix-core kernel (apb_forward_int), and the whole
    forward built on each (apb_forward_popcount, apb_forward).  The two integer results must be equal."""
    import torch
    from paper_2306_08960_amd import binding as b
    from paper_2306_08960_amd import synth
    rows = []
    for name in ("C2", "C3_r20_b1", "C3_r20_b2", "C4", "C5a", "C5b"):
        cfg = synth.CONFIGS[name]
        W, delta, X, step = synth.make_layer(cfg)
        N, K, M, bits = cfg.N, cfg.K, cfg.M, cfg.bits
        layer = b.apb_compress(torch.from_numpy(W).cuda(), float(delta))
        nnz = layer.info()["nnz"]
        packed = b.apb_quantize_acts(torch.from_numpy(X).cuda(), bits, float(step))
        D1 = torch.empty((N, M), dtype=torch.int32, device="cuda")
        D2 = torch.empty((N, M), dtype=torch.int32, device="cuda")
        Y = torch.empty((N, M), dtype=torch.float32, device="cuda")
        t_pop = graph_ms(lambda: b.apb_forward_int_popcount(layer, packed, M, bits, D=D1))
        t_mfma = graph_ms(lambda: b.apb_forward_int(layer, packed, M, bits, D=D2))
        t_fpop = graph_ms(lambda: b.apb_forward_popcount(layer, packed, M, bits, float(step), Y=Y))
        t_fwd = graph_ms(lambda: b.apb_forward(layer, packed, M, bits, float(step), Y=Y))
        Kw = (K + 31) // 32
        t_valu_roof = 2.0 * bits * N * Kw * M / VALU_LANE_OPS_PER_S
        rows.append({"workload": name, "N": N, "K": K, "M": M, "act_bits": bits, "nnz": int(nnz),
                     "integer_results_equal": bool(torch.equal(D1, D2)),
                     "us_int_popcount": t_pop * 1e3, "us_int_matrix_cores": t_mfma * 1e3,
                     "us_forward_popcount": t_fpop * 1e3, "us_forward": t_fwd * 1e3,
                     "popcount_frac_of_its_valu_bitop_roof": t_valu_roof / (t_pop * 1e-3),
                     "matrix_cores_frac_of_fp4_peak": 2.0 * N * K * M / (t_mfma * 1e-3) / (MFMA_FP4_PEAK_TFLOPS * 1e12)})
        layer.free()
        del packed, D1, D2, Y
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "binary part of the APB forward: popcount on the vector ALU vs FP4 matrix cores",
                      "unit": "us per launch (graph replay between HIP events)", "n_gpus": 1, "data": "synthetic",
                      "rows": rows}))


def routine_peaks(args):
    """What the chip sustains for the instruction mixes of the forward kernels, register-only loops."""
    import torch
    from paper_2306_08960_amd import binding as b
    out = torch.empty(b.apb_probe_out_bytes() // 8, dtype=torch.float64, device="cuda")
    published = {"mfma_fp4": (MFMA_FP4_PEAK_TFLOPS * 1e12, "flop/s (2 per multiply-add), dense FP4"),
                 "mfma_i8": (5.0e15, "op/s (2 per multiply-add), dense int8"),
                 "and_bcnt": (VALU_LANE_OPS_PER_S, "32-bit vector lane-ops/s (256 CUs x 64 lanes x 2.4 GHz)"),
                 "fma_f64": (VALU_LANE_OPS_PER_S, "float64 multiply-add lane-ops/s (78.6 TFLOP/s / 2)"),
                 "lds_u8": (256 * 32 * 2.4e9, "LDS lane-reads/s at 32 banks per compute unit and cycle"),
                 "lds_b128": (256 * 128 * 2.4e9, "LDS bytes/s read 16 bytes per lane, against 128 bytes per compute unit and cycle"),
                 "mfma_fp4_lds": (MFMA_FP4_PEAK_TFLOPS * 1e12, "flop/s, one operand of every matrix instruction read from LDS"),
                 "mfma_fp4_lds_barrier": (MFMA_FP4_PEAK_TFLOPS * 1e12,
                                          "flop/s, ... plus an LDS write and a workgroup barrier per four matrix instructions"),
                 "mfma_fp4_lds_barrier_valu": (MFMA_FP4_PEAK_TFLOPS * 1e12,
                                               "flop/s, ... plus 32 vector instructions per four matrix instructions")}
    rows = []
    for name, kind in b.PROBES.items():
        iters = 2048
        work = b.apb_probe_rate(kind, iters, out)
        torch.cuda.synchronize()
        a, c = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(5):
            b.apb_probe_rate(kind, iters, out)
        c.record()
        c.synchronize()
        rate = work / (a.elapsed_time(c) / 5 * 1e-3)
        rows.append({"probe": name, "measured_per_s": rate, "published_or_derived_per_s": published[name][0],
                     "unit": published[name][1], "frac": rate / published[name][0],
                     "ms_per_launch": a.elapsed_time(c) / 5})
    print(json.dumps({"metric": "register-only instruction-rate probes", "n_gpus": 1, "rows": rows}))


# The 3x3 convolutions of an ImageNet ResNet-18 as im2col products: (name, N = C_out, C_in, output H = W, stride).
RESNET18_3X3 = [("layer1.x (64->64 @56)", 64, 64, 56, 1), ("layer2.0.conv1 (64->128 @28, stride 2)", 128, 64, 28, 2),
                ("layer2.x (128->128 @28)", 128, 128, 28, 1), ("layer3.0.conv1 (128->256 @14, stride 2)", 256, 128, 14, 2),
                ("layer3.x (256->256 @14)", 256, 256, 14, 1), ("layer4.0.conv1 (256->512 @7, stride 2)", 512, 256, 7, 2),
                ("layer4.x (512->512 @7)", 512, 512, 7, 1)]


def routine_resnet18(args):
    """Sec. V-B protocol on the shapes Sec. V-C evaluates: every 3x3 layer of an ImageNet ResNet-18 as the
    im2col product N x K x M (K = 9 C_in, M = batch * H_out * W_out; the first 7x7 layer, the 1x1 downsampling
    layers and the classifier are left out as in the paper): the three bitwise products alone (operands
    packed) and the APB layer forward (2-bit activations, 2 % of the weights outside the interval)."""
    import torch
    from paper_2306_08960_amd import binding as b
    from paper_2306_08960_amd import synth
    batch = 64
    rows = []
    for idx, (lname, N, Cin, Hout, stride) in enumerate(RESNET18_3X3):
        K, M = 9 * Cin, batch * Hout * Hout
        W, delta, X, step = synth.random_case(1800 + idx, N, K, M, 2, rho=0.02)
        Wd, Xd = torch.from_numpy(W).cuda(), torch.from_numpy(X).cuda()
        apb = b.apb_compress(Wd, float(delta))
        binl = b.apb_compress(Wd, float("inf"), alpha=0.05)
        w2 = b.apb_w2_pack(Wd, 0.05)
        nnz = apb.info()["nnz"]
        p1 = b.apb_quantize_acts(Xd - 0.5, 1, 1.0)
        p2 = b.apb_quantize_acts(Xd, 2, float(step))
        D = torch.empty((N, M), dtype=torch.int32, device="cuda")
        Y = torch.empty((N, M), dtype=torch.float32, device="cuda")
        t11 = graph_ms(lambda: b.apb_forward_int(binl, p1, M, 1, D=D))
        t12 = graph_ms(lambda: b.apb_forward_int(binl, p2, M, 2, D=D))
        t22 = graph_ms(lambda: b.apb_gemm_2_2_int(w2, p2, M, D=D))
        tf = graph_ms(lambda: b.apb_forward(apb, p2, M, 2, float(step), Y=Y))
        tq = graph_ms(lambda: b.apb_quantize_acts(Xd, 2, float(step), packed=p2))
        ops = 2.0 * N * K * M
        roof = forward_roofline(N, K, M, 2, nnz, tf, "the forward kernel")
        rows.append({"layer": lname, "N": N, "K": K, "M": M, "nnz": int(nnz), "us_1_1": t11 * 1e3, "us_1_2": t12 * 1e3,
                     "us_2_2": t22 * 1e3, "us_apb_forward": tf * 1e3, "us_quantize": tq * 1e3,
                     "tops_1_1": ops / t11 / 1e9, "tops_1_2": ops / t12 / 1e9, "tops_2_2": ops / t22 / 1e9,
                     "tops_apb_forward": (ops + 2.0 * nnz * M) / tf / 1e9,
                     "cost_1_2_over_1_1": t12 / t11, "cost_2_2_over_1_1": t22 / t11, "cost_apb_over_1_2": tf / t12,
                     "apb_forward_bound": roof["bound"], "apb_forward_frac_of_roof": roof["frac"],
                     "apb_forward_frac_of_valu_bitop_yardstick": roof["frac_of_valu_bitop_yardstick"]})
        for h in (apb, binl, w2):
            h.free()
        del Wd, Xd, p1, p2, D, Y
        torch.cuda.empty_cache()
    total = {k: sum(r[k] for r in rows) for k in ("us_1_1", "us_1_2", "us_2_2", "us_apb_forward")}
    print(json.dumps({"metric": "3x3 layers of ResNet-18 (ImageNet shapes) as im2col products: bitwise products and APB forward",
                      "unit": "us per launch (graph replay between HIP events); TOPS = 2*N*K*M (+ 2*nnz*M) / time",
                      "n_gpus": 1, "data": "synthetic", "batch": batch,
                      "note": "one row per distinct shape (layer1/2/3/4.x occur 4/3/3/3 times in the network)",
                      "rows": rows, "sum_over_shapes_us": total}))


def routine_rho_sweep(args):
    """Sec. V-C crossover: the forward of the C3 layer (256 x 2304, M = 8192) against the fraction rho of
    weights kept outside the binarization interval, for 1-bit and 2-bit activations.  The time of the residual
    part is forward(rho) - forward(0); it equals the binary part's at the rate `crossover_rho` (interpolated)."""
    import torch
    from dataclasses import replace
    from paper_2306_08960_amd import binding as b
    from paper_2306_08960_amd import synth
    rates = (0.0, 0.005, 0.01, 0.02, 0.03, 0.04, 0.05, 0.06, 0.08)
    out = {}
    for bits in (1, 2):
        base = synth.CONFIGS[f"C3_r20_b{bits}"]
        W, _ = synth.make_weights(base)
        X = synth.make_acts(base)
        Wd = torch.from_numpy(W).cuda()
        packed = b.apb_quantize_acts(torch.from_numpy(X).cuda(), bits, float(base.step))
        Y = torch.empty((base.N, base.M), dtype=torch.float32, device="cuda")
        rows = []
        for rho in rates:
            delta = float("inf") if rho == 0.0 else float(synth._delta_for_rate(W, rho))
            layer = b.apb_compress(Wd, delta)
            nnz = layer.info()["nnz"]
            t = graph_ms(lambda: b.apb_forward(layer, packed, base.M, bits, float(base.step), Y=Y))
            rows.append({"rho": rho, "nnz": int(nnz), "us_forward": t * 1e3})
            layer.free()
        t0 = rows[0]["us_forward"]
        cross = None
        for r0, r1 in zip(rows, rows[1:]):
            s0, s1 = r0["us_forward"] - t0, r1["us_forward"] - t0
            r0["us_residual_part"], r1["us_residual_part"] = s0, s1
            if cross is None and s0 < t0 <= s1:
                cross = r0["rho"] + (r1["rho"] - r0["rho"]) * (t0 - s0) / (s1 - s0)
        out[f"act_bits_{bits}"] = {"us_binary_part": t0, "rows": rows, "crossover_rho": cross,
                                   "crossover_sparsity_percent": None if cross is None else 100.0 * (1.0 - cross)}
    print(json.dumps({"metric": "APB forward time against the outlier rate (C3 shape, N=256 K=2304 M=8192)",
                      "unit": "us per launch (graph replay between HIP events)", "n_gpus": 1, "data": "synthetic",
                      "sweep": out}))


def routine_train(args):
    """The training-side operators (Sec. III Eqs. 3-9) on the latent weights of a layer the size of C5a's
    (4096 x 4096) and of a whole ResNet-18's worth of 3x3 weights (11 M): HBM-bound, one pass each."""
    import torch
    from paper_2306_08960_amd import binding as b
    rows = []
    for label, n in (("C5a latent weights 4096x4096", 4096 * 4096), ("64 Mi weights", 1 << 26), ("256 Mi weights", 1 << 28)):
        g = torch.Generator(device="cuda").manual_seed(230608960)
        W = torch.randn(n, generator=g, device="cuda") * 0.05
        G = torch.randn(n, generator=g, device="cuda")
        out, gw = torch.empty_like(W), torch.empty_like(W)
        sums = torch.empty(2, dtype=torch.float64, device="cuda")
        cnt = torch.empty(1, dtype=torch.int64, device="cuda")
        ws = torch.empty(b.apb_train_workspace_bytes() // 8, dtype=torch.float64, device="cuda")
        tf = graph_ms(lambda: b.apb_train_forward(W, 0.04, 0.06, out=out))
        tb = graph_ms(lambda: b.apb_train_backward(W, G, 0.04, 0.06, grad_w=gw, sums=sums, count=cnt, workspace=ws))
        tb2 = graph_ms(lambda: b.apb_train_backward(W, G, 0.04, 0.06, want_grad_w=False, sums=sums, count=cnt, workspace=ws))
        rows.append({"what": label, "n": n,
                     "forward": {"ms": tf, "algorithmic_bytes": 8.0 * n, "GBps": 8.0 * n / tf / 1e6, "frac_of_hbm_peak": 8.0 * n / tf / 1e6 / HBM_PEAK_GBS},
                     "backward": {"ms": tb, "algorithmic_bytes": 12.0 * n, "GBps": 12.0 * n / tb / 1e6, "frac_of_hbm_peak": 12.0 * n / tb / 1e6 / HBM_PEAK_GBS},
                     "backward_reductions_only": {"ms": tb2, "algorithmic_bytes": 8.0 * n, "GBps": 8.0 * n / tb2 / 1e6, "frac_of_hbm_peak": 8.0 * n / tb2 / 1e6 / HBM_PEAK_GBS}})
        del W, G, out, gw
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "APB training-side operators (Eq. 3 forward; straight-through gradient + dL/dalpha, dL/ddelta)",
                      "unit": "ms per call (graph replay between HIP events); GB/s of algorithmic bytes against 8 TB/s",
                      "n_gpus": 1, "data": "synthetic", "rows": rows}))


EXTRA_ROUTINES = {"popcount_vs_mfma": routine_popcount_vs_mfma, "peaks": routine_peaks, "resnet18": routine_resnet18,
                  "rho_sweep": routine_rho_sweep, "train": routine_train}


if __name__ == "__main__":
    main()
