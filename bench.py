#!/usr/bin/env python3
"""Benchmark of the MX hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--quick] [--all-configs] [--no-cpu-baseline]

One step = one pass of the whole hot path over seeded synthetic tensors that are
already resident in HBM:
  * 12 casts of an 8192 x 8192 bf16 activation tensor (Student-t(3), 0.1 % of the
    entries x100, 0.01 % exact zeros): six element formats x {blocks along the
    last axis, blocks along axis 0}, round-to-nearest-even;
  * one dequantize (MXFP8 E4M3 -> bf16) of the same tensor;
  * the transformer projection GEMM 8192 x 4096 x 4096, MXFP8 E4M3 x E4M3, bf16
    output, once from pre-quantized operands (mx_gemm) and once with the bf16
    activations cast on load (mx_gemm_qa).
Sources and destinations rotate over three / two copies so that no call finds its
input in the 256 MB Infinity Cache.  K steps are timed as a whole (ms_per_step).
Each call's own average duration is then measured the same way: K launches of
that call back to back on the stream it runs on, between two events, with the same
buffer rotation.  The headline value is the cast throughput (algorithmic bytes of
the 12 casts divided by their summed average durations); GEMM TFLOP/s are reported
beside it.

Also in the default run, per call and with the same protocol:
  "ceilings"       what the cast's access pattern reaches on this machine with no arithmetic
                   (mx_stream_pattern: pure read, pure write, copy, 2 and 4 bytes read per byte
                   written), and each cast as a fraction of the ceiling of its read : write ratio;
  "other_configs"  the other full-size workloads: the 4096 x 11008 projection of config 3, the
                   mixed-format inference GEMM of config 4 with its two casts, the MXFP6 training
                   triple of config 5 (six casts, three GEMMs, the dual-axis casts), and config 1
                   in microseconds -- every GEMM with its fraction of the matrix peak, every cast
                   with its fraction of the HBM peak;
  "gemm_clock"     the shader clock during the headline GEMM and the clocks one K step takes, from
                   counters read inside the kernel (mx_gemm_probe), on the real operands and on zeros;
  "mfma_instruction_ceiling"  what the GEMM's matrix instruction sustains from registers alone on
                   the headline GEMM's MX-quantized operand values (mx_mfma_stream_probe), per element width
                   and on zeros: the power-limited ceiling of the instruction on such operand values;
  "gemm_zero_operands"  the headline GEMM launch on all-zero operands: what the same kernel
                   does when operand switching activity does not hold the clock down;
  "vendor_reference_8192x4096x4096"  context only: the vendor library's FP8 GEMM (one scale per tensor) and
                   its MX block-scaled FP8 GEMM through torch._scaled_mm, same shape, same box;
  "gemm_max_rel_err"    (with the CPU baseline leg) max |dC| / sum |a||b| of sampled entries
                   against the double-precision reference, per GEMM workload.
--quick leaves out "other_configs"; --all-configs adds decoding shapes, MXINT8, the added
rounding modes and the GEMM-epilogue cast.

Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2310_10537_amd import binding as mx  # noqa: E402
from paper_2310_10537_amd import inputs  # noqa: E402

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {8: 5000.0, 6: 10100.0, 4: 10100.0}
ROWS = COLS = 8192
GM, GK, GN = 8192, 4096, 4096
NCOPY = 3
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "bench_hot_path_hbm_traffic.txt")
FORMAT_INDEX = {"fp8_e4m3": 0, "fp8_e5m2": 1, "fp6_e3m2": 2, "fp6_e2m3": 3, "fp4_e2m1": 4, "int8": 5}


def measured_traffic():
    """HBM bytes per launch (read + write) of this file's headline kernels, from the committed hardware
    counter summary (FETCH_SIZE / WRITE_SIZE scaled by a copy of known size; the file names its
    commands).  One kernel serves several workloads, so the summary has a row per kernel and grid
    size; for each label the row of its kernel nearest to the label's algorithmic bytes is taken.
    label -> bytes; empty when the summary is missing or a kernel is not in it."""
    rows = []
    try:
        lines = open(TRAFFIC_SUMMARY).read().splitlines()
    except OSError:
        return {}
    for ln in lines:
        f = ln.split()
        if len(f) < 7 or not f[0].isdigit():
            continue
        try:
            rows.append((" ".join(f[6:]), (float(f[3]) + float(f[4])) * 2 ** 20))
        except ValueError:
            continue
    n_elem = ROWS * COLS
    want = {"dequantize_fp8_e4m3_bf16": ("dequant_flat_kernel<0, 1>", n_elem * (1.0 + 1.0 / 32.0 + 2.0)),
            "gemm_fp8_e4m3": ("gemm_tile16_kernel<0, 0, 1, false", (GM + GN) * GK * (1.0 + 1.0 / 32.0) + GM * GN * 2.0)}
    for fmt in range(6):
        for kname, axis in (("cast_row_bf16_kernel<%d, 0," % fmt, 1), ("cast_col_bf16_kernel<%d, 0," % fmt, 0)):
            want[f"cast_{mx.FORMAT_NAMES[fmt]}_axis{axis}"] = (kname, cast_bytes(fmt, n_elem))
    out = {}
    for label, (kname, algo) in want.items():
        cand = [b for k, b in rows if k.startswith(kname)]
        if cand:
            best = min(cand, key=lambda b: abs(b - algo))
            if 0.5 * algo <= best <= 4.0 * algo:      # a row of another workload is no measurement of this one
                out[label] = int(best)
    return out


def clock_probe(A, fmtA, B, fmtB, K, C, mfma_clocks_per_step, n=6):
    """Shader clock under the tiled GEMM's load and clocks per K step, from the kernel's own counters
    (mx_gemm_probe: per work-group, shader clocks and 100 MHz ticks from start to the end of the K loop).
    n launches back to back so that the clock has settled; the last one is read."""
    for _ in range(n):
        clk, ticks = mx.mx_gemm_probe(A[0], A[1], fmtA, B[0], B[1], fmtB, K, C)
    torch.cuda.synchronize()
    clk, ticks = clk.double(), ticks.double()
    steps = K // 128
    per_step = float(clk.mean()) / steps
    return {"shader_GHz": round(float(clk.sum() / ticks.sum()) * 0.1, 3), "clocks_per_k_step": round(per_step, 0),
            "mfma_clocks_per_k_step": mfma_clocks_per_step,
            "k_loop_us_per_tile": round(float(ticks.mean()) / 100.0, 2)}


def instruction_ceiling(a_bf16):
    """What the GEMM kernels' matrix instruction sustains on this machine from registers alone
    (mx_mfma_stream_probe: four waves per compute unit, no memory access in the loop), with the A
    registers holding MX-quantized activations of the headline GEMM and the B registers MX-quantized
    weights drawn like its weights, per element width, and on zeros: the chip's power limit holds the
    clock down as operand switching activity rises, so this, not the nominal peak, is what a kernel
    that fed the instruction perfectly would reach on such operand values."""
    out = {}
    a = a_bf16[:256].contiguous()
    w = torch.from_numpy(inputs.gaussian_f32((256, GK), seed=103, std=0.02)).cuda()
    for name, fmt, iters, zero in (("fp8_e4m3", mx.FP8_E4M3, 2000, False), ("fp6_e3m2", mx.FP6_E3M2, 4000, False),
                                   ("fp4_e2m1", mx.FP4_E2M1, 4000, False), ("fp8_e4m3_zero_operands", mx.FP8_E4M3, 2000, True)):
        codes = torch.cat([mx.mx_quantize(t, 1, fmt)[0].reshape(-1)[:32768] for t in (a, w)]).contiguous()
        if zero:
            codes.zero_()
        res = []
        ms = time_call(lambda: res.append(mx.mx_mfma_stream_probe(fmt, codes, iters)), 5)
        clk, ticks = res[-1]
        flop = mx.MX_MFMA_STREAM_WGS * 4 * 16.0 * iters * 131072
        tf = flop / ms / 1e9
        out[name] = {"TFLOPs": round(tf, 1), "frac_mfma_peak": round(tf / MFMA_PEAK_TFLOPS[mx.FORMAT_BITS[fmt]], 4),
                     "shader_GHz": round(float(clk.double().sum() / ticks.double().sum()) * 0.1, 3)}
    return out


def vendor_reference(n):
    """Context, not a target and no part of the product: the vendor library's FP8 GEMMs (through
    torch._scaled_mm) on the same box and shape as the headline GEMM, on N(0,1) x N(0,1) operands --
    with one scale per tensor (no MX blocks) and with E8M0 scales per 32 elements (the MX product) --
    and this library's mx_gemm on the same operand bytes with unit scales, since the operands'
    switching activity sets the clock.  None where this torch build does not offer the call."""
    out = {}
    M, N, K = GM, GN, GK
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    a = torch.randn((M, K), device="cuda", generator=g).to(torch.float8_e4m3fn)
    b = torch.randn((N, K), device="cuda", generator=g).to(torch.float8_e4m3fn)
    one = torch.tensor(1.0, device="cuda")
    flop = 2.0 * M * N * K
    try:
        ms = time_call(lambda: torch._scaled_mm(a, b.t(), scale_a=one, scale_b=one, out_dtype=torch.bfloat16), n)
        out["fp8_one_scale_per_tensor_TFLOPs"] = round(flop / ms / 1e9, 1)
    except Exception:                      # noqa: BLE001  (an unsupported call is reported as absent)
        out["fp8_one_scale_per_tensor_TFLOPs"] = None
    # this library's MX GEMM on the very same operand bytes (every scale byte 127: X = 1)
    s_a = torch.full((M, K // 32), 127, dtype=torch.uint8, device="cuda")
    s_b = torch.full((N, K // 32), 127, dtype=torch.uint8, device="cuda")
    c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    ms = time_call(lambda: mx.mx_gemm(a.view(torch.uint8), s_a, mx.FP8_E4M3, b.view(torch.uint8), s_b, mx.FP8_E4M3, K, out=c), n)
    out["this_library_same_operands_TFLOPs"] = round(flop / ms / 1e9, 1)
    try:
        sa = torch.full((M, K // 32), 127, dtype=torch.uint8, device="cuda").view(torch.float8_e8m0fnu)
        sb = torch.full((N, K // 32), 127, dtype=torch.uint8, device="cuda").view(torch.float8_e8m0fnu)
        ms = time_call(lambda: torch._scaled_mm(a, b.t(), scale_a=sa, scale_b=sb, out_dtype=torch.bfloat16), n)
        out["mxfp8_block_scaled_TFLOPs"] = round(flop / ms / 1e9, 1)
    except Exception:                      # noqa: BLE001
        out["mxfp8_block_scaled_TFLOPs"] = None
    return out


def cast_bytes(fmt, n_elem):
    """Algorithmic bytes of one cast: bf16 source + packed elements + scale bytes."""
    return n_elem * (2.0 + mx.FORMAT_BITS[fmt] / 8.0 + 1.0 / 32.0)


def to_dev_bf16(bits):
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()


class Timed:
    """Average duration per label: run(label, fn, n) launches fn n times between
    two events on the current stream."""

    def __init__(self, n):
        self.n = n
        self.recs = []

    def run(self, label, fn):
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(self.n):
            fn()
        b.record()
        self.recs.append((label, a, b))

    def totals(self):
        """label -> [summed ms, launches]"""
        out = {}
        for label, a, b in self.recs:
            t = out.setdefault(label, [0.0, 0])
            t[0] += a.elapsed_time(b)
            t[1] += self.n
        return out


def sample_entries(M, N, n, seed):
    rng = np.random.default_rng(seed)
    return rng.integers(0, M, n), rng.integers(0, N, n)


def cpu_leg(x_bits, samples):
    """The CPU reference as it stands: (1) timed on the host cores on one pass of the cast
    workload -- all 12 casts (6 formats x 2 axes) of the whole tensor, a few seconds on 16
    threads; (2) the sampled GEMM entries of every workload in double precision, against which
    the GPU's Float32-output results are compared (max |dC| / sum |a||b|)."""
    import oracle
    oracle.lib()
    x = np.ascontiguousarray(x_bits)
    t0 = time.perf_counter()
    nbytes = 0.0
    for fmt in range(6):
        oracle.quantize(x, 1, fmt, 0)
        oracle.quantize(x, 0, fmt, 0)
        nbytes += 2 * cast_bytes(fmt, x.size)
    dt = time.perf_counter() - t0
    base = {"value": round(nbytes / dt / 1e9, 3), "unit": "GB/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "one pass of the cast workload: 12 casts (6 formats x 2 axes, RNE) of the whole "
                      "8192x8192 bf16 tensor; %.1f s of wall time" % dt}
    rel = {}
    for label, (ea, sa, fa, eb, sb, fb, K, mi, ni, got) in samples.items():
        ref, cabs = oracle.gemm_entries(ea, sa, fa, eb, sb, fb, K, mi, ni)
        rel[label] = float("%.3g" % float((np.abs(got.astype(np.float64) - ref) / cabs).max()))
    return base, rel


def time_call(fn, n):
    """Average duration in ms of n back-to-back launches of fn (after 2 warm-up launches)."""
    fn()
    fn()
    a = torch.cuda.Event(enable_timing=True)
    b = torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(n):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / n


def accuracy_sample(samples, label, A, fa, B, fb, K, seed, n=512):
    """Float32-output mx_gemm on the operands (device MX tensors), n sampled entries kept with the host
    copies of the rows and columns they need, for the CPU leg."""
    M, N = A[1].shape[0], B[1].shape[0]
    mi, ni = sample_entries(M, N, n, seed)
    C32 = mx.mx_gemm(A[0], A[1], fa, B[0], B[1], fb, K, dtype=torch.float32)
    got = C32[torch.from_numpy(mi).cuda(), torch.from_numpy(ni).cuda()].cpu().numpy()
    del C32
    um, inv_m = np.unique(mi, return_inverse=True)
    un, inv_n = np.unique(ni, return_inverse=True)
    tm, tn = torch.from_numpy(um).cuda(), torch.from_numpy(un).cuda()
    samples[label] = (A[0][tm].cpu().numpy(), A[1][tm].cpu().numpy(), fa, B[0][tn].cpu().numpy(), B[1][tn].cpu().numpy(), fb, K,
                      inv_m, inv_n, got)


def other_configs(n, samples, extras):
    """Configs 1, 3 (wide projection), 4 and 5 at full size; returns a dict of per-call results."""
    out = {}

    def gemm_entry(label, M, N, K, ms, bits):
        tf = 2.0 * M * N * K / ms / 1e9
        out[label] = {"avg_ms": round(ms, 5), "TFLOPs": round(tf, 1), "frac_mfma_peak": round(tf / MFMA_PEAK_TFLOPS[bits], 4)}

    def cast_entry(label, n_elem, src_bytes, fmt, ms):
        b = n_elem * (src_bytes + mx.FORMAT_BITS[fmt] / 8.0 + 1.0 / 32.0)
        out[label] = {"avg_ms": round(ms, 5), "GBps": round(b / ms / 1e6, 1), "frac_hbm_peak": round(b / ms / 1e6 / HBM_PEAK_GBS, 4)}

    # config 1: 1024 x 1024 fp32 round trip and a 256^3 GEMM -- cache-resident and launch-latency-bound,
    # reported in microseconds; not an HBM measurement
    x1 = torch.from_numpy(inputs.gaussian_f32((1024, 1024), seed=0)).cuda()
    q1 = mx.mx_quantize(x1, 1, mx.FP8_E4M3)
    y1 = torch.empty_like(x1)
    out["cfg1_quantize_1024x1024_f32_e4m3_us"] = round(1e3 * time_call(lambda: mx.mx_quantize(x1, 1, mx.FP8_E4M3, mx.ROUND_RNE, q1[0], q1[1]), n), 2)
    out["cfg1_dequantize_1024x1024_e4m3_f32_us"] = round(1e3 * time_call(lambda: mx.mx_dequantize(q1[0], q1[1], mx.FP8_E4M3, 1024, 1024, 1, out=y1), n), 2)
    ga1 = mx.mx_quantize(torch.from_numpy(inputs.gaussian_f32((256, 256), seed=1)).cuda(), 1, mx.FP8_E4M3)
    gb1 = mx.mx_quantize(torch.from_numpy(inputs.gaussian_f32((256, 256), seed=2)).cuda(), 1, mx.FP8_E4M3)
    c1 = torch.empty((256, 256), dtype=torch.float32, device="cuda")
    out["cfg1_gemm_256x256x256_e4m3_us"] = round(1e3 * time_call(lambda: mx.mx_gemm(ga1[0], ga1[1], mx.FP8_E4M3, gb1[0], gb1[1], mx.FP8_E4M3, 256, out=c1), n), 2)
    accuracy_sample(samples, "cfg1_256x256x256_e4m3", ga1, 0, gb1, 0, 256, seed=21)

    # fp32 sources and destinations at the size of config 2 (config 1's types, HBM-sized)
    xf = torch.from_numpy(inputs.gaussian_f32((ROWS, COLS), seed=11)).cuda()
    qf = mx.mx_quantize(xf, 1, mx.FP8_E4M3)
    cast_entry("cast_8192x8192_f32_e4m3_axis1", ROWS * COLS, 4, mx.FP8_E4M3,
               time_call(lambda: mx.mx_quantize(xf, 1, mx.FP8_E4M3, mx.ROUND_RNE, qf[0], qf[1]), n))
    ms = time_call(lambda: mx.mx_dequantize(qf[0], qf[1], mx.FP8_E4M3, ROWS, COLS, 1, out=xf), n)
    b = ROWS * COLS * (1.0 + 1.0 / 32.0 + 4.0)
    out["dequantize_8192x8192_e4m3_f32"] = {"avg_ms": round(ms, 5), "GBps": round(b / ms / 1e6, 1), "frac_hbm_peak": round(b / ms / 1e6 / HBM_PEAK_GBS, 4)}
    del xf, qf

    # config 3, second projection: 8192 x 11008 x 4096, E4M3, A cast on load
    M, K, N = 8192, 4096, 11008
    a = to_dev_bf16(inputs.gaussian_bf16((M, K), seed=2))
    w = torch.from_numpy(inputs.gaussian_f32((K, N), seed=112, std=0.02)).cuda()
    Be, Bs = mx.mx_quantize(w, 0, mx.FP8_E4M3)
    Ae, As = mx.mx_quantize(a, 1, mx.FP8_E4M3)
    C = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    gemm_entry("cfg3_gemm_8192x11008x4096_e4m3", M, N, K,
               time_call(lambda: mx.mx_gemm(Ae, As, mx.FP8_E4M3, Be, Bs, mx.FP8_E4M3, K, out=C), n), 8)
    gemm_entry("cfg3_gemm_qa_8192x11008x4096_e4m3", M, N, K,
               time_call(lambda: mx.mx_gemm_qa(a, mx.FP8_E4M3, mx.ROUND_RNE, Be, Bs, mx.FP8_E4M3, out=C), n), 8)
    del C
    accuracy_sample(samples, "cfg3_8192x11008x4096_e4m3", (Ae, As), 0, (Be, Bs), 0, K, seed=23)
    del a, w, Be, Bs, Ae, As

    if extras:
        # config 3, first projection with C delivered as MXFP8 (cast in the GEMM epilogue) against GEMM + cast of C
        M, K, N = 8192, 4096, 4096
        a = to_dev_bf16(inputs.gaussian_bf16((M, K), seed=2))
        w = torch.from_numpy(inputs.gaussian_f32((K, N), seed=102, std=0.02)).cuda()
        Be, Bs = mx.mx_quantize(w, 0, mx.FP8_E4M3)
        Ae, As = mx.mx_quantize(a, 1, mx.FP8_E4M3)
        C = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        qc = mx.mx_quantize(C, 1, mx.FP8_E4M3)
        gemm_entry("cfg3_gemm_q_8192x4096x4096_e4m3_to_e4m3", M, N, K,
                   time_call(lambda: mx.mx_gemm_q(Ae, As, mx.FP8_E4M3, Be, Bs, mx.FP8_E4M3, K, mx.FP8_E4M3, mx.ROUND_RNE, out=qc), n), 8)
        ms_g = time_call(lambda: mx.mx_gemm(Ae, As, mx.FP8_E4M3, Be, Bs, mx.FP8_E4M3, K, out=C), n)
        ms_c = time_call(lambda: mx.mx_quantize(C, 1, mx.FP8_E4M3, mx.ROUND_RNE, qc[0], qc[1]), n)
        out["cfg3_gemm_then_cast_of_C_ms"] = round(ms_g + ms_c, 5)
        # the added rounding modes on the activation tensor of that shape (generic integer kernels)
        for label, call in (("toward_zero", lambda: mx.mx_quantize(a, 1, mx.FP8_E4M3, mx.ROUND_TOWARD_ZERO, Ae, As)),
                            ("stochastic", lambda: mx.mx_quantize_sr(a, 1, mx.FP8_E4M3, 1234, Ae, As))):
            cast_entry("cast_8192x4096_bf16_e4m3_axis1_" + label, M * K, 2, mx.FP8_E4M3, time_call(call, n))
        del a, w, Be, Bs, Ae, As, C, qc

        # decoding shapes: few rows of A against the wide projection's E4M3 weights (one pass over 45 MB)
        N, K = 11008, 4096
        w = torch.from_numpy(inputs.gaussian_f32((K, N), seed=112, std=0.02)).cuda()
        for fmt, name in ((mx.FP8_E4M3, "e4m3"), (mx.INT8, "int8")):
            Be, Bs = mx.mx_quantize(w, 0, fmt)
            for M in (1, 16, 128):
                a = to_dev_bf16(inputs.gaussian_bf16((M, K), seed=5))
                Ae, As = mx.mx_quantize(a, 1, fmt)
                C = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
                ms = time_call(lambda: mx.mx_gemm(Ae, As, fmt, Be, Bs, fmt, K, out=C), n)
                out[f"decode_gemm_{M}x{N}x{K}_{name}"] = {"avg_us": round(1e3 * ms, 2), "weights_GBps": round(N * K * (1 + 1 / 32) / ms / 1e6, 1)}
        del w, Be, Bs

        # MXINT8 on the projection shape of config 3 (each element split into two E2M3 halves, tiled kernel at depth 4K)
        M, K, N = 8192, 4096, 4096
        a = to_dev_bf16(inputs.gaussian_bf16((M, K), seed=2))
        w = torch.from_numpy(inputs.gaussian_f32((K, N), seed=102, std=0.02)).cuda()
        ga = mx.mx_quantize(a, 1, mx.INT8)
        gb = mx.mx_quantize(w, 0, mx.INT8)
        C = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        ms = time_call(lambda: mx.mx_gemm(ga[0], ga[1], mx.INT8, gb[0], gb[1], mx.INT8, K, out=C), max(2, n // 3))
        out["int8_gemm_8192x4096x4096"] = {"avg_ms": round(ms, 5), "TOPs": round(2.0 * M * N * K / ms / 1e9, 1)}
        del a, w, ga, gb, C

    # config 4: E3M2 activations [4096, 8192] x E2M1 weights (logical 8192 x 28672)
    M, K, N = 4096, 8192, 28672
    act = to_dev_bf16(inputs.student_t_bf16((M, K), seed=3))
    w = torch.from_numpy(inputs.gaussian_f32((K, N), seed=103, std=0.02)).cuda()
    ga = mx.mx_quantize(act, 1, mx.FP6_E3M2)
    gb = mx.mx_quantize(w, 0, mx.FP4_E2M1)
    cast_entry("cfg4_cast_act_e3m2_axis1", M * K, 2, mx.FP6_E3M2,
               time_call(lambda: mx.mx_quantize(act, 1, mx.FP6_E3M2, mx.ROUND_RNE, ga[0], ga[1]), n))
    cast_entry("cfg4_cast_w_f32_e2m1_axis0", K * N, 4, mx.FP4_E2M1,
               time_call(lambda: mx.mx_quantize(w, 0, mx.FP4_E2M1, mx.ROUND_RNE, gb[0], gb[1]), n))
    del w
    C = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    gemm_entry("cfg4_gemm_4096x28672x8192_e3m2_e2m1", M, N, K,
               time_call(lambda: mx.mx_gemm(ga[0], ga[1], mx.FP6_E3M2, gb[0], gb[1], mx.FP4_E2M1, K, out=C), n), 6)
    out["cfg4_gemm_4096x28672x8192_e3m2_e2m1"]["clock"] = clock_probe(ga, mx.FP6_E3M2, gb, mx.FP4_E2M1, K, C, 1024, n=3)
    del C
    accuracy_sample(samples, "cfg4_4096x28672x8192_e3m2_e2m1", ga, 2, gb, 4, K, seed=24)
    del act, ga, gb

    # config 5: E3M2 training triple, half-away rounding; T tokens, hidden H, ffn F
    T, H, F = 16384, 2048, 8192
    fmt, rnd = mx.FP6_E3M2, mx.ROUND_HALF_AWAY
    X = to_dev_bf16(inputs.gaussian_bf16((T, H), seed=4))
    W = to_dev_bf16(inputs.gaussian_bf16((H, F), seed=104, std=0.02))
    dY = to_dev_bf16(inputs.gaussian_bf16((T, F), seed=204))
    q = {}
    for name, t, axis in (("X_axis1", X, 1), ("W_axis0", W, 0), ("dY_axis1", dY, 1), ("W_axis1", W, 1),
                          ("X_axis0", X, 0), ("dY_axis0", dY, 0)):
        q[name] = mx.mx_quantize(t, axis, fmt, rnd)
        e, s = q[name]
        cast_entry("cfg5_cast_" + name, t.numel(), 2, fmt, time_call(lambda: mx.mx_quantize(t, axis, fmt, rnd, e, s), n))
    total = sum(out[k]["avg_ms"] for k in out if k.startswith("cfg5_cast_"))
    # the same six MX tensors from three one-pass dual-axis casts
    dual_total = 0.0
    for name, t in (("X", X), ("W", W), ("dY", dY)):
        o1, o0 = q[name + "_axis1"], q[name + "_axis0"]
        ms = time_call(lambda: mx.mx_quantize_dual(t, fmt, rnd, o1, o0), n)
        b = t.numel() * (2.0 + 2.0 * (mx.FORMAT_BITS[fmt] / 8.0 + 1.0 / 32.0))
        out["cfg5_dualcast_" + name] = {"avg_ms": round(ms, 5), "GBps": round(b / ms / 1e6, 1), "frac_hbm_peak": round(b / ms / 1e6 / HBM_PEAK_GBS, 4)}
        dual_total += ms
    for name, A, B, (M, N, K) in (("fwd", q["X_axis1"], q["W_axis0"], (T, F, H)), ("dgrad", q["dY_axis1"], q["W_axis1"], (T, H, F)),
                                  ("wgrad", q["X_axis0"], q["dY_axis0"], (H, F, T))):
        C = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        ms = time_call(lambda: mx.mx_gemm(A[0], A[1], fmt, B[0], B[1], fmt, K, out=C), n)
        gemm_entry(f"cfg5_gemm_{name}_{M}x{N}x{K}_e3m2", M, N, K, ms, 6)
        out[f"cfg5_gemm_{name}_{M}x{N}x{K}_e3m2"]["clock"] = clock_probe(A, fmt, B, fmt, K, C, 1024, n=3)
        total += ms
        del C
        accuracy_sample(samples, f"cfg5_{name}_{M}x{N}x{K}_e3m2", A, fmt, B, fmt, K, seed=25, n=256)
    casts_ms = sum(out[k]["avg_ms"] for k in out if k.startswith("cfg5_cast_"))
    out["cfg5_triple_total_ms"] = round(total, 5)
    out["cfg5_triple_total_ms_with_dual_casts"] = round(total - casts_ms + dual_total, 5)
    return out


def ceilings(xs, n):
    """What the row cast's access pattern reaches with no arithmetic: GB/s of bytes moved."""
    src_b = ROWS * COLS * 2
    dst = [torch.empty(src_b, dtype=torch.uint8, device="cuda") for _ in range(2)]
    rot = [0]

    def run(rpw, write, dst_bytes):
        def f():
            rot[0] += 1
            mx.mx_stream_pattern(xs[rot[0] % NCOPY] if rpw else None, dst[rot[0] % 2], dst_bytes, rpw, write)
        ms = time_call(f, n)
        return round((rpw * dst_bytes + (dst_bytes if write else 0)) / ms / 1e6, 1)
    out = {"read_GBps": run(1, False, src_b), "write_GBps": run(0, True, src_b), "copy_GBps": run(1, True, src_b),
           "read2_write1_GBps": run(2, True, src_b // 2), "read4_write1_GBps": run(4, True, src_b // 4)}
    del dst
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--quick", action="store_true", help="leave out the other full-size configs")
    ap.add_argument("--all-configs", action="store_true", help="also time decoding shapes, MXINT8, the added rounding modes, the GEMM-epilogue cast")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (no collectives exist in the MX hot path); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    mx.lib()  # fail loudly if the HIP library is missing
    TRAFFIC = measured_traffic()

    # ---- synthetic inputs, resident in HBM before the timed region --------------
    x_bits = inputs.student_t_bf16((ROWS, COLS), seed=1)
    xs = [to_dev_bf16(x_bits) for _ in range(NCOPY)]
    a_bits = inputs.gaussian_bf16((GM, GK), seed=2)
    As = [to_dev_bf16(a_bits) for _ in range(NCOPY)]
    w = torch.from_numpy(inputs.gaussian_f32((GK, GN), seed=102, std=0.02)).cuda()
    Be, Bs = mx.mx_quantize(w, 0, mx.FP8_E4M3)               # weights pre-quantized once: [N][K]
    del w
    Aq = [mx.mx_quantize(a, 1, mx.FP8_E4M3) for a in As]
    Cs = [torch.empty((GM, GN), dtype=torch.bfloat16, device="cuda") for _ in range(NCOPY)]
    outs = {}
    for fmt in range(6):
        for axis in (1, 0):
            outs[(fmt, axis)] = [(torch.empty((ROWS, COLS * mx.FORMAT_BITS[fmt] // 8), dtype=torch.uint8, device="cuda"),
                                  torch.empty((ROWS, COLS // 32), dtype=torch.uint8, device="cuda")) for _ in range(2)]
    deq_out = [torch.empty((ROWS, COLS), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    deq_in = [mx.mx_quantize(x, 1, mx.FP8_E4M3) for x in xs]   # three copies: the 66 MiB input would fit the Infinity Cache
    torch.cuda.synchronize()

    rot = [0]

    def nxt():
        rot[0] += 1
        return rot[0]

    def cast_call(fmt, axis):
        def f():
            i = nxt()
            e, s = outs[(fmt, axis)][i % 2]
            mx.mx_quantize(xs[i % NCOPY], axis, fmt, mx.ROUND_RNE, e, s)
        return f

    def deq_call():
        i = nxt()
        mx.mx_dequantize(deq_in[i % NCOPY][0], deq_in[i % NCOPY][1], mx.FP8_E4M3, ROWS, COLS, 1, out=deq_out[i % 2])

    def gemm_call():
        i = nxt()
        mx.mx_gemm(Aq[i % NCOPY][0], Aq[i % NCOPY][1], mx.FP8_E4M3, Be, Bs, mx.FP8_E4M3, GK, out=Cs[i % NCOPY])

    def gemm_qa_call():
        i = nxt()
        mx.mx_gemm_qa(As[i % NCOPY], mx.FP8_E4M3, mx.ROUND_RNE, Be, Bs, mx.FP8_E4M3, out=Cs[i % NCOPY])

    calls = [(f"cast_{mx.FORMAT_NAMES[fmt]}_axis{axis}", cast_call(fmt, axis)) for fmt in range(6) for axis in (1, 0)]
    calls += [("dequantize_fp8_e4m3_bf16", deq_call), ("gemm_fp8_e4m3", gemm_call), ("gemm_qa_fp8_e4m3", gemm_qa_call)]

    def step(_timer=None):
        for _label, fn in calls:
            fn()

    for _ in range(args.warmup):
        step()
    # One plain 128 MiB -> 128 MiB device copy outside the timed region: the kernel of known
    # traffic against which hardware byte counters of a profiled run are scaled.
    deq_out[0].copy_(xs[0])
    torch.cuda.synchronize()

    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3

    # per-call average durations over the same number of launches
    timer = Timed(args.steps)
    for label, fn in calls:
        timer.run(label, fn)
    torch.cuda.synchronize()
    tot = timer.totals()

    ceil = ceilings(xs, args.steps)
    # the headline GEMM launch on all-zero operands (codes 0, scale bytes 127): same kernel, same grid
    zA = [(torch.zeros_like(Aq[0][0]), torch.full_like(Aq[0][1], 127)) for _ in range(NCOPY)]
    zB = (torch.zeros_like(Be), torch.full_like(Bs, 127))

    def gemm_zero_call():
        i = nxt()
        mx.mx_gemm(zA[i % NCOPY][0], zA[i % NCOPY][1], mx.FP8_E4M3, zB[0], zB[1], mx.FP8_E4M3, GK, out=Cs[i % NCOPY])
    zero_ms = time_call(gemm_zero_call, args.steps)
    gemm_clock = {"real_operands": clock_probe(Aq[0], mx.FP8_E4M3, (Be, Bs), mx.FP8_E4M3, GK, Cs[0], 2048),
                  "zero_operands": clock_probe(zA[0], mx.FP8_E4M3, zB, mx.FP8_E4M3, GK, Cs[0], 2048)}
    del zA, zB

    n_elem = ROWS * COLS
    cast_ms = 0.0
    cast_b = 0.0
    per_kernel = {}
    for fmt in range(6):
        for axis in (1, 0):
            label = f"cast_{mx.FORMAT_NAMES[fmt]}_axis{axis}"
            ms, n = tot[label]
            avg = ms / n
            cast_ms += avg
            cast_b += cast_bytes(fmt, n_elem)
            gbps = cast_bytes(fmt, n_elem) / avg / 1e6
            pattern = ceil["read4_write1_GBps"] if mx.FORMAT_BITS[fmt] == 4 else ceil["read2_write1_GBps"]
            per_kernel[label] = {"avg_ms": round(avg, 5), "GBps": round(gbps, 1), "frac_hbm_peak": round(gbps / HBM_PEAK_GBS, 4),
                                 "frac_pattern_ceiling": round(gbps / pattern, 4)}
    flop = 2.0 * GM * GN * GK
    for label in ("gemm_fp8_e4m3", "gemm_qa_fp8_e4m3"):
        ms, n = tot[label]
        per_kernel[label] = {"avg_ms": round(ms / n, 5), "TFLOPs": round(flop / (ms / n) / 1e9, 1),
                             "frac_mfma_peak": round(flop / (ms / n) / 1e9 / MFMA_PEAK_TFLOPS[8], 4)}
    ms, n = tot["dequantize_fp8_e4m3_bf16"]
    deq_b = n_elem * (1.0 + 1.0 / 32.0 + 2.0)
    per_kernel["dequantize_fp8_e4m3_bf16"] = {"avg_ms": round(ms / n, 5), "GBps": round(deq_b / (ms / n) / 1e6, 1),
                                              "frac_hbm_peak": round(deq_b / (ms / n) / 1e6 / HBM_PEAK_GBS, 4)}

    # Dominant kernel of the step by time: reported against its roofline.  The two GEMM calls
    # run the same tiled kernel (mx_gemm_qa adds a cast launch in front of it), so its duration
    # is taken from the plain mx_gemm call.  The slowest cast is reported beside it, since the
    # headline value is the cast throughput.
    def cast_roof(label):
        fmt = [i for i in range(6) if label.startswith("cast_" + mx.FORMAT_NAMES[i])][0]
        ach = cast_bytes(fmt, n_elem) / (tot[label][0] / tot[label][1]) / 1e6
        return {"kernel": label, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": TRAFFIC.get(label)}

    dom = max(tot, key=lambda k: tot[k][0])
    slowest_cast = max((k for k in tot if k.startswith("cast_")), key=lambda k: tot[k][0])
    if dom.startswith("cast_"):
        roof = cast_roof(dom)
    elif dom.startswith("gemm"):
        dms = tot["gemm_fp8_e4m3"][0] / tot["gemm_fp8_e4m3"][1]
        ach = flop / dms / 1e9
        roof = {"kernel": "gemm_fp8_e4m3", "bound": "mfma", "achieved": round(ach, 1), "peak": MFMA_PEAK_TFLOPS[8],
                "unit": "TFLOP/s", "frac": round(ach / MFMA_PEAK_TFLOPS[8], 4),
                "traffic": TRAFFIC.get("gemm_fp8_e4m3")}
    else:
        dms = tot[dom][0] / tot[dom][1]
        ach = deq_b / dms / 1e6
        roof = {"kernel": dom, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": TRAFFIC.get(dom)}

    samples = {}
    accuracy_sample(samples, "cfg3_8192x4096x4096_e4m3", Aq[0], 0, (Be, Bs), 0, GK, seed=22)

    value = cast_b / cast_ms / 1e6   # GB/s over the 12 casts
    line = {
        "metric": "MX cast GB/s (% HBM peak) + MX GEMM TFLOPS (% scaled-MFMA peak)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_ms / args.steps, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1]: mx_quantize of 8192x8192 bf16 Student-t(3) activations into 6 MX formats x 2 axes"
                               " (+ dequantize, + configs[2] 8192x4096x4096 MXFP8 GEMM plain and quantize-on-load)"},
        "cast_frac_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "gemm_tflops": per_kernel["gemm_fp8_e4m3"]["TFLOPs"],
        "gemm_qa_tflops": per_kernel["gemm_qa_fp8_e4m3"]["TFLOPs"],
        "roofline": roof,
        "roofline_slowest_cast": cast_roof(slowest_cast),
        "ceilings": ceil,
        "gemm_zero_operands": {"avg_ms": round(zero_ms, 5), "TFLOPs": round(flop / zero_ms / 1e9, 1),
                               "frac_mfma_peak": round(flop / zero_ms / 1e9 / MFMA_PEAK_TFLOPS[8], 4)},
        "gemm_clock": gemm_clock,
        "mfma_instruction_ceiling": instruction_ceiling(As[0]),
        "kernels": per_kernel,
    }
    del xs, As, Aq, Cs, outs, deq_out, deq_in, Be, Bs
    torch.cuda.empty_cache()
    if not args.quick:
        line["other_configs"] = other_configs(args.steps, samples, args.all_configs)
        line["vendor_reference_8192x4096x4096"] = vendor_reference(args.steps)
    if not args.no_cpu_baseline:
        line["cpu_baseline"], line["gemm_max_rel_err"] = cpu_leg(x_bits, samples)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
