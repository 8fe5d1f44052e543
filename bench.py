#!/usr/bin/env python3
"""Benchmark of the MXFP4 OAS+MBS hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input resident in HBM:
    quantize A and W (OAS + MBS-S, one launch)  ->  C = A.W^T with the MBS correction (bf16 out)
on the Llama-3-70B FFN shape (A 8192x8192, W 28672x8192), the largest single-GPU configuration.  Prints ONE
JSON line.

`value` is 2*M*N*K divided by the wall time of a whole step (quantizers included), at the sustained rate: the
device is first brought out of its idle clocks by an untimed run of the same step.  The roofline object is for
the dominant kernel, the MBS GEMM, timed with HIP events on the launch stream inside the timed region; its
`secondary` object carries the bound that actually binds that kernel, vector-instruction issue.  `extras` holds
the other configurations (Llama-3-8B FFN up-projection, decode, mixture-of-experts grouped GEMM, square shapes)
and the side measurements.  The CPU oracle is timed on a bounded sample as a reported baseline.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

WORKLOADS = {
    "llama3-70b-ffn": dict(
        M=8192, N=28672, K=8192, gen="llama70b_ffn", buffers=(2, 2, 2),
        desc="llama3-70b-ffn: A 8192x8192 bf16 Student-t(3) + 0.5% outlier channels x50, W 28672x8192 bf16 N(0,0.015^2)"),
    "llama3-8b-ffn-up": dict(
        M=4096, N=14336, K=4096, gen="llama8b_ffn_up", buffers=(8, 5, 3),
        desc="llama3-8b-ffn-up: A 4096x4096 bf16 Student-t(4) + 1% outlier channels x20, W 14336x4096 bf16 N(0,0.02^2)"),
}
HEADLINE = "llama3-70b-ffn"
PROFILE_TRAFFIC = os.path.join(ROOT, "profiles", "bench_llama70b_ffn_hbm_traffic.txt")
# vector instructions per 32x32 output fragment and macro block in the MBS kernel's inner loop (what the
# correction itself needs; the loop's address and table work comes on top), and matrix instructions per fragment
MBS_VALU_PER_FRAGMENT = 16    # one multiply-add per output: acc += P * S
MBS_MFMA_PER_FRAGMENT = 2.5   # two products, and half of the instruction that forms S = sigma_A (x) sigma_B for two fragments


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=100)
    p.add_argument("--warmup", type=int, default=20)
    p.add_argument("--prewarm-ms", type=float, default=150.0,
                   help="untimed run of the step before the warm-up steps, so that the device has left its idle "
                        "clocks (it takes some tens of milliseconds from a cold start); 0 disables it")
    p.add_argument("--workload", choices=sorted(WORKLOADS), default=HEADLINE)
    p.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    p.add_argument("--no-extras", action="store_true", help="skip the other configurations and side measurements")
    return p.parse_args()


class Work:
    """One configuration's tensors on the device, inputs and outputs rotated over distinct buffers so that the
    bf16 inputs are read from HBM, not from the 256 MB Infinity Cache."""

    def __init__(self, torch, np, synth, name):
        cfg = WORKLOADS[name]
        self.name, self.desc = name, cfg["desc"]
        self.M, self.N, self.K = cfg["M"], cfg["N"], cfg["K"]
        self.a_bits, self.w_bits = getattr(synth, cfg["gen"])()
        dev = torch.device("cuda:0")
        na, nw, nc = cfg["buffers"]

        def to_dev(bits):
            return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)

        M, N, K = self.M, self.N, self.K
        self.xa = [to_dev(self.a_bits) for _ in range(na)]
        self.xw = [to_dev(self.w_bits) for _ in range(nw)]
        self.qa = [tuple(torch.empty(s, dtype=torch.uint8, device=dev) for s in ((M, K // 2), (M, K // 32), (M, K // 128)))
                   for _ in self.xa]
        self.qw = [tuple(torch.empty(s, dtype=torch.uint8, device=dev) for s in ((N, K // 2), (N, K // 32), (N, K // 128)))
                   for _ in self.xw]
        self.cs = [torch.empty((M, N), dtype=torch.bfloat16, device=dev) for _ in range(nc)]
        self.flops = 2.0 * M * N * K

    def step(self, mx, i, ev=None):
        # ev: 3 events bracketing the quantizer launch and the GEMM launch
        a, w, c = i % len(self.xa), i % len(self.xw), i % len(self.cs)
        if ev:
            ev[0].record()
        mx.mx_quantize_mbs_pair(self.xa[a], self.xw[w], "oas", self.qa[a], self.qw[w])     # both GEMM operands, one launch
        if ev:
            ev[1].record()
        mx.mx_gemm_mbs(*self.qa[a], *self.qw[w], "bf16", out=self.cs[c])
        if ev:
            ev[2].record()


def run_steps(mx, torch, work, steps, warmup, prewarm_ms):
    """Whole steps: untimed pre-warm, warm-up, then `steps` timed steps bracketed by synchronisation.  The
    events sit on torch's current stream, which is the stream the binding launches on."""
    prewarm_steps = 0
    t_pre = time.perf_counter()
    while (time.perf_counter() - t_pre) * 1e3 < prewarm_ms:
        for i in range(5):
            work.step(mx, prewarm_steps + i)
        torch.cuda.synchronize()
        prewarm_steps += 5
    for i in range(warmup):
        work.step(mx, i)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        work.step(mx, warmup + i, events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    def avg(j):
        return sum(e[j].elapsed_time(e[j + 1]) for e in events) / len(events)

    return {"ms_per_step": (t1 - t0) * 1e3 / steps, "ms_quantize": avg(0), "ms_gemm": avg(1), "prewarm_steps": prewarm_steps}


def step_report(metrics, work, t):
    bpe = metrics.QUANT_BYTES_PER_ELT_MBS
    q_gbps = (work.M + work.N) * work.K * bpe / (t["ms_quantize"] * 1e-3) / 1e9
    return {
        "step_tflops": round(work.flops / (t["ms_per_step"] * 1e-3) / 1e12, 2),
        "ms_per_step": round(t["ms_per_step"], 4),
        "gemm_mbs_tflops_in_step": round(work.flops / (t["ms_gemm"] * 1e-3) / 1e12, 2),
        "gemm_mbs_frac_of_peak": round(work.flops / (t["ms_gemm"] * 1e-3) / 1e12 / metrics.MFMA_FP4_PEAK_TFLOPS, 4),
        "quantize_gbps_in_step": round(q_gbps, 1),
        "quantize_frac_of_peak": round(q_gbps / metrics.HBM_PEAK_GBPS, 4),
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported. "
              "`value` is one MI355X's throughput." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2603_08713_amd as mx
    from paper_2603_08713_amd import metrics, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    mx.load_library()
    torch.cuda.set_device(0)

    work = Work(torch, np, synth, args.workload)
    M, N, K = work.M, work.N, work.K
    t = run_steps(mx, torch, work, args.steps, args.warmup, args.prewarm_ms)
    value = work.flops / (t["ms_per_step"] * 1e-3) / 1e12
    gemm_tflops = work.flops / (t["ms_gemm"] * 1e-3) / 1e12
    bpe = metrics.QUANT_BYTES_PER_ELT_MBS
    q_gbps = (M + N) * K * bpe / (t["ms_quantize"] * 1e-3) / 1e9
    ceiling = metrics.valu_issue_ceiling_tflops(MBS_VALU_PER_FRAGMENT, MBS_MFMA_PER_FRAGMENT)
    traffic = metrics.read_profile_value(PROFILE_TRAFFIC, "gemm_mbs_traffic_bytes_per_launch") if args.workload == HEADLINE else None

    out = {
        "metric": "OAS+MBS MXFP4 GEMM TFLOP/s (whole step: quantize A and W, MBS GEMM)",
        "value": round(value, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(t["ms_per_step"], 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "mxfp4 (E2M1 x E8M0/32, fp32 accumulate, bf16 out)",
        "data": "synthetic",
        "config": {"workload": work.desc, "M": M, "N": N, "K": K, "rule": "oas", "mbs": "static/128",
                   "buffers": "inputs rotated over %d A / %d W / %d C buffers" % (len(work.xa), len(work.xw), len(work.cs)),
                   "prewarm_steps": t["prewarm_steps"]},
        "roofline": {
            "kernel": mx.gemm_plan(M, N, K, True, True) + " (mx_gemm_mbs)",
            "bound": "mfma",
            "achieved": round(gemm_tflops, 2),
            "peak": metrics.MFMA_FP4_PEAK_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(gemm_tflops / metrics.MFMA_FP4_PEAK_TFLOPS, 4),
            "traffic": None if traffic is None else int(traffic),
            "traffic_source": "profiles/%s (rocprofv3 FETCH_SIZE and WRITE_SIZE runs of this command; not read in this run)"
                              % os.path.basename(PROFILE_TRAFFIC),
            "algorithmic_bytes": metrics.gemm_operand_bytes(M, N, K, mbs=True) + M * N * 2,
            "avg_launch_ms": round(t["ms_gemm"], 4),
            "secondary": {
                "bound": "valu-issue",
                "model": "per 32x32 fragment and macro block: %d vector instructions x %.1f clocks + %.1f matrix instructions x %d "
                         "clocks of the SIMD's issue port, %d SIMDs at %.1f GHz"
                         % (MBS_VALU_PER_FRAGMENT, metrics.VALU_ISSUE_CLOCKS, MBS_MFMA_PER_FRAGMENT, metrics.MFMA_ISSUE_CLOCKS,
                            metrics.SIMDS, metrics.CLOCK_GHZ),
                "ceiling": round(ceiling, 1), "unit": "TFLOP/s", "achieved_over_ceiling": round(gemm_tflops / ceiling, 4),
            },
        },
        "quantize": {
            "bound": "hbm", "bytes_per_element": bpe, "peak": metrics.HBM_PEAK_GBPS, "unit": "GB/s",
            "kernel": "quantize_kernel<mbs> on A and W in one launch (mx_quantize_mbs_pair)",
            "ms": round(t["ms_quantize"], 4), "achieved": round(q_gbps, 1), "frac": round(q_gbps / metrics.HBM_PEAK_GBPS, 4),
        },
    }

    if not args.no_extras:
        ex = out["extras"] = {}
        ex["gemm_forms"] = gemm_forms(mx, torch, metrics, work, args)
        ex["qsnr_db_gpu"] = qsnr_ladder_gpu(mx, torch, work.xa[0][:QSNR_ROWS])
        ex["qsnr_db_gpu_weights"] = qsnr_weights_gpu(mx, torch, work.xw[0][:QSNR_ROWS])
        ex["qsnr_ab_db_gpu"] = qsnr_ab_gpu(mx, torch, work.xa[0], work.xw[0])
        ex.update(yardsticks(torch, work, args))
        head_bits = (work.a_bits, work.w_bits)
        del work
        torch.cuda.empty_cache()
        other = "llama3-8b-ffn-up" if args.workload == HEADLINE else HEADLINE
        w2 = Work(torch, np, synth, other)
        t2 = run_steps(mx, torch, w2, min(3 * args.steps, 300) if other != HEADLINE else args.steps, args.warmup, args.prewarm_ms)
        ex[other] = dict(step_report(metrics, w2, t2), workload=w2.desc, gemm_forms=gemm_forms(mx, torch, metrics, w2, args))
        small = w2 if other != HEADLINE else None
        if small is not None:
            ex["quantizers_on_8b_W"] = quantizer_extras(mx, torch, metrics, small, args)
            ex["mxfp8_e4m3"] = mxfp8_extras(mx, torch, small, args)
            ex["mxfp6_e2m3"] = mxfp8_extras(mx, torch, small, args, elem="e2m3")
            ex["mxfp8_e4m3"]["decode"] = elem_decode_extras(mx, torch, synth, np, "e4m3")
            ex["mxfp6_e2m3"]["decode"] = elem_decode_extras(mx, torch, synth, np, "e2m3")
        del w2, small
        torch.cuda.empty_cache()
        ex["moe_grouped"] = moe_extras(mx, torch, synth, np, metrics, args)
        ex["decode_m16_k4096"] = decode_extras(mx, torch, synth, np)
        ex["square_shapes"] = square_shapes(mx, torch, synth, np, metrics)
    else:
        head_bits = (work.a_bits, work.w_bits)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(np, synth, head_bits[0], head_bits[1], M, N, K, args.no_extras)
    print(json.dumps(out))


QSNR_ROWS = 256  # rows of the activation tensor the QSNR ladder is computed on, by both paths
# Sec. 3.1's metric on the rungs of Sec. 4: plain MXFP4 = the OCP rule; +MBS = static words over the no-overflow
# ("floor") rule, since MBS-S maps the window's absmax to 6 without overflow; the same over the OCP rule is
# listed beside it
QSNR_LADDER = (("mxfp4", "ocp", False), ("+oas", "oas", False), ("+mbs", "floor", True), ("+mbs(ocp rule)", "ocp", True),
               ("+oas+mbs", "oas", True))


def qsnr_ladder_gpu(mx, torch, x):
    """QSNR (dB) of quantize -> dequantize through the HIP kernels for plain MXFP4, +OAS, +MBS, +OAS+MBS
    (Sec. 3.1's metric: 10 log10(sum x^2 / sum (x - xq)^2)); the sums are taken in fp64 with torch."""
    res = {}
    ref = x.to(torch.float64)
    for name, rule, mbs in QSNR_LADDER:
        q = mx.mx_quantize_mbs(x, rule) if mbs else mx.mx_quantize(x, rule)
        back = mx.mx_dequantize(q[0], q[1], q[2] if mbs else None, "f32").to(torch.float64)
        res[name] = round(float(10.0 * torch.log10((ref * ref).sum() / ((ref - back) ** 2).sum())), 3)
    res["sample"] = "first %d rows of A" % QSNR_ROWS
    return res


QSNR_AB_ROWS, QSNR_AB_COLS = 64, 2048   # output sample of QSNR(AB): rows of A x rows of W
QSNR_AB_LADDER = (("mxfp4", "ocp", "none"), ("+oas", "oas", "none"), ("+oas+mbs-s", "oas", "static"),
                  ("+oas+mbs-h", "oas", "hybrid"))


def qsnr_ab_gpu(mx, torch, xa, xw):
    """QSNR (dB) of the product (Eq. 2: reference = the bf16 tensors multiplied in fp64, here with torch) for
    plain MXFP4, +OAS, +OAS+MBS-S and MBS-Hybrid (searched words for W, static for A), every operand quantized
    and multiplied by the HIP kernels (fp32 output)."""
    a, w = xa[:QSNR_AB_ROWS], xw[:QSNR_AB_COLS]
    ref = a.to(torch.float64) @ w.to(torch.float64).T
    res = {}
    for name, rule, mbs in QSNR_AB_LADDER:
        if mbs == "none":
            qa, qw = mx.mx_quantize(a, rule), mx.mx_quantize(w, rule)
            c = mx.mx_gemm(qa[0], qa[1], qw[0], qw[1], "f32")
        else:
            qa = mx.mx_quantize_mbs(a, rule)
            qw = mx.mx_quantize_mbs(w, rule) if mbs == "static" else mx.mx_quantize_mbs_dynamic(w, rule)
            c = mx.mx_gemm_mbs(*qa, *qw, "f32")
        res[name] = round(float(10.0 * torch.log10((ref * ref).sum() / ((ref - c.to(torch.float64)) ** 2).sum())), 3)
    res["sample"] = "first %d rows of A x first %d rows of W" % (QSNR_AB_ROWS, QSNR_AB_COLS)
    return res


def qsnr_weights_gpu(mx, torch, x):
    """QSNR (dB) of the weight tensor with OAS alone, with the static MBS word and with the searched one
    (MBS-Dynamic, the weight half of the paper's MBS-Hybrid, Sec. 4.3.3 and 4.4), through the HIP kernels."""
    res = {}
    ref = x.to(torch.float64)
    for name, q in (("+oas", mx.mx_quantize(x, "oas") + (None,)), ("+oas+mbs-s", mx.mx_quantize_mbs(x, "oas")),
                    ("+oas+mbs-d", mx.mx_quantize_mbs_dynamic(x, "oas")),
                    ("+oas+mbs-d(table)", mx.mx_quantize_mbs_dynamic_lut(x, mx.mx_mbs_lut_build(), "oas"))):
        back = mx.mx_dequantize(q[0], q[1], q[2], "f32").to(torch.float64)
        res[name] = round(float(10.0 * torch.log10((ref * ref).sum() / ((ref - back) ** 2).sum())), 3)
    res["sample"] = "first %d rows of W" % QSNR_ROWS
    return res


def time_loop(torch, fn, iters, warm=20):
    for i in range(warm):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(iters):
        fn(warm + i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def gemm_forms(mx, torch, metrics, work, args):
    """The GEMM kernels of one configuration launched back to back on operands quantized beforehand: plain MXFP4
    (Tab. 4's baseline), MBS words on both operands, and the one-sided kernels (words on A only / on B only: a
    deployment that applies MBS to one operand pays one multiply-add per output and macro block instead of two
    operations).  Overhead = 1 - TFLOPS_MBS / TFLOPS_plain, the convention of Tab. 4."""
    n = max(5, min(args.steps, 60))
    cs, qa, qw = work.cs, work.qa, work.qw
    for i in range(len(qa)):   # (the step loop left these filled; a side measurement may have rewritten them)
        mx.mx_quantize_mbs_pair(work.xa[i % len(work.xa)], work.xw[i % len(work.xw)], "oas", qa[i], qw[i % len(qw)])
    pa = mx.mx_quantize(work.xa[0], "ocp")
    pw = mx.mx_quantize(work.xw[0], "ocp")
    M, N, K = work.M, work.N, work.K

    def rate(fn):
        return work.flops / (time_loop(torch, fn, n, warm=max(10, n // 3)) * 1e-3) / 1e12

    plain = rate(lambda i: mx.mx_gemm(pa[0], pa[1], pw[0], pw[1], "bf16", out=cs[i % len(cs)]))
    both = rate(lambda i: mx.mx_gemm_mbs(*qa[i % len(qa)], *qw[i % len(qw)], "bf16", out=cs[i % len(cs)]))
    a_only = rate(lambda i: mx.mx_gemm_mbs(*qa[i % len(qa)], qw[0][0], qw[0][1], None, "bf16", out=cs[i % len(cs)]))
    b_only = rate(lambda i: mx.mx_gemm_mbs(qa[0][0], qa[0][1], None, *qw[i % len(qw)], "bf16", out=cs[i % len(cs)]))
    peak = metrics.MFMA_FP4_PEAK_TFLOPS
    return {
        "plain_tflops": round(plain, 1), "plain_frac_of_peak": round(plain / peak, 4),
        "plain_kernel": mx.gemm_plan(M, N, K, False, False),
        "mbs_tflops": round(both, 1), "mbs_frac_of_peak": round(both / peak, 4),
        "mbs_overhead": round(metrics.overhead_fraction(plain, both), 4),
        "mbs_a_only_tflops": round(a_only, 1), "mbs_a_only_overhead": round(metrics.overhead_fraction(plain, a_only), 4),
        "mbs_b_only_tflops": round(b_only, 1), "mbs_b_only_overhead": round(metrics.overhead_fraction(plain, b_only), 4),
        "paper_context": "Tab. 4 (NVIDIA B200, CUTLASS 4.3.0): 6.2 % average overhead on square shapes (other hardware)",
    }


def bench_library():
    """The benchmark's own helper library (yardstick kernels; not part of the product library)."""
    from paper_2603_08713_amd import build as mxbuild

    if not os.path.exists(mxbuild.BENCH_LIB):
        return None
    L = ctypes.CDLL(mxbuild.BENCH_LIB)
    L.mxb_mfma_rate.restype = ctypes.c_int
    L.mxb_mfma_rate.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
    return L


def yardsticks(torch, work, args):
    """What the device sustains with nothing else going on: the matrix cores out of registers (the published peak
    assumes 2.4 GHz, which random operand bits do not reach under this power limit) and a plain device copy."""
    res = {}
    L = bench_library()
    if L is not None:
        rates = {}
        for name, rnd in (("constant_operands", 0), ("random_operands", 1)):
            v = ctypes.c_double(0.0)
            if L.mxb_mfma_rate(rnd, 20000, ctypes.byref(v)) == 0:
                rates[name] = round(v.value, 1)
        res["mfma_issue_only_tflops"] = rates
    n = max(5, min(args.steps, 50))
    src, dst = work.xw[0], work.xw[1]
    ms_copy = time_loop(torch, lambda i: dst.copy_(src), n, warm=5)
    res["copy_gbps"] = round(2 * src.numel() * 2 / (ms_copy * 1e-3) / 1e9, 1)
    return res


def quantizer_extras(mx, torch, metrics, work, args):
    """Quantizer and dequantizer rates (algorithmic bytes) on the 14336x4096 weight tensor, outside the step."""
    n = max(5, min(args.steps, 100))
    xa, xw, qa, qw = work.xa, work.xw, work.qa, work.qw
    res = {}
    pw = mx.mx_quantize(xw[0], "ocp")
    ms_q = time_loop(torch, lambda i: mx.mx_quantize(xw[i % len(xw)], "ocp", pw[0], pw[1]), n)
    res["quantize_plain_W_gbps"] = round(xw[0].numel() * metrics.QUANT_BYTES_PER_ELT_PLAIN / (ms_q * 1e-3) / 1e9, 1)
    ms_pair = time_loop(torch, lambda i: mx.mx_quantize_mbs_pair(xa[i % len(xa)], xw[i % len(xw)], "oas", qa[i % len(qa)], qw[i % len(qw)]), n)
    res["quantize_pair_alone_gbps"] = round((xa[0].numel() + xw[0].numel()) * metrics.QUANT_BYTES_PER_ELT_MBS / (ms_pair * 1e-3) / 1e9, 1)
    # MBS-Dynamic (offline weight quantization: 17 evaluations of the window instead of one)
    ms_s = time_loop(torch, lambda i: mx.mx_quantize_mbs(xw[i % len(xw)], "oas", *qw[i % len(qw)]), n)
    ms_dyn = time_loop(torch, lambda i: mx.mx_quantize_mbs_dynamic(xw[i % len(xw)], "oas", 0, 16, 16, *qw[i % len(qw)]), n)
    res["quantize_dynamic_W"] = {"ms": round(ms_dyn, 4), "static_ms": round(ms_s, 4), "slowdown_vs_static": round(ms_dyn / ms_s, 2),
                                 "gbps": round(xw[0].numel() * metrics.QUANT_BYTES_PER_ELT_MBS / (ms_dyn * 1e-3) / 1e9, 1),
                                 "candidates": "static word + 16 equally spaced",
                                 "paper_context": "paper reports its MBS-D kernel 2.5-3x slower than MBS-S (NVIDIA B200)"}
    lut = mx.mx_mbs_lut_build()
    ms_lut = time_loop(torch, lambda i: mx.mx_quantize_mbs_dynamic_lut(xw[i % len(xw)], lut, "oas", True, *qw[i % len(qw)]), n)
    res["quantize_dynamic_table_W"] = {"ms": round(ms_lut, 4), "slowdown_vs_static": round(ms_lut / ms_s, 2),
                                       "gbps": round(xw[0].numel() * metrics.QUANT_BYTES_PER_ELT_MBS / (ms_lut * 1e-3) / 1e9, 1),
                                       "candidates": "words 16 j priced by the 2 x 64 x 16 fp16 table of Eq. 5; static word kept if not worse"}
    # the timing loop above rewrote qw with searched words: put the static ones back for what follows
    for i in range(len(qw)):
        mx.mx_quantize_mbs(xw[i % len(xw)], "oas", *qw[i])
    deq = torch.empty((xw[0].shape[0], xw[0].shape[1]), dtype=torch.bfloat16, device=xw[0].device)
    ms_d = time_loop(torch, lambda i: mx.mx_dequantize(*qw[i % len(qw)], "bf16", out=deq), n)
    res["dequantize_W_gbps"] = round(xw[0].numel() * metrics.QUANT_BYTES_PER_ELT_MBS / (ms_d * 1e-3) / 1e9, 1)
    return res


def mxfp8_extras(mx, torch, work, args, elem="e4m3"):
    """The same step in MXFP8 (E4M3 elements) or MXFP6 (E2M3, packed codes), OAS and MBS restated on the element
    format's own constants: both quantizers, then the MBS GEMM; and QSNR(AB) of the plain OCP rule against
    OAS + MBS-S on the product sample."""
    n = max(5, min(args.steps, 60))
    xa, xw, cs, flops = work.xa, work.xw, work.cs, work.flops
    six = elem in ("e2m3", "e3m2")
    qa = [mx.mx_quantize_elem(x, elem, "oas") for x in xa]
    qw = [mx.mx_quantize_elem(x, elem, "oas") for x in xw]

    def step(i):
        a, w = qa[i % len(qa)], qw[i % len(qw)]
        mx.mx_quantize_elem(xa[i % len(xa)], elem, "oas", True, *a)
        mx.mx_quantize_elem(xw[i % len(xw)], elem, "oas", True, *w)
        mx.mx_gemm_mbs_elem(elem, a[0], a[1], a[2], elem, w[0], w[1], w[2], "bf16", out=cs[i % len(cs)])

    ms_step = time_loop(torch, step, n)
    ms_mbs = time_loop(torch, lambda i: mx.mx_gemm_mbs_elem(elem, *qa[i % len(qa)], elem, *qw[i % len(qw)], "bf16", out=cs[i % len(cs)]), n)
    ms_plain = time_loop(torch, lambda i: mx.mx_gemm_mbs_elem(elem, qa[0][0], qa[0][1], None, elem, qw[0][0], qw[0][1], None, "bf16",
                                                              out=cs[i % len(cs)]), n)
    ms_qw = time_loop(torch, lambda i: mx.mx_quantize_elem(xw[i % len(xw)], elem, "oas", True, *qw[i % len(qw)]), n)
    bytes_per_elt = 2 + (0.75 if six else 1) + 1 / 32 + 1 / 128
    deq = torch.empty(tuple(xw[0].shape), dtype=torch.bfloat16, device=xw[0].device)
    ms_d = time_loop(torch, lambda i: mx.mx_dequantize_elem(elem, *qw[i % len(qw)], "bf16", out=deq), n)
    res = {"shape": work.name, "step_tflops": round(flops / (ms_step * 1e-3) / 1e12, 1), "ms_per_step": round(ms_step, 4),
           "dequantize_W_gbps": round(xw[0].numel() * bytes_per_elt / (ms_d * 1e-3) / 1e9, 1),
           "gemm_mbs_tflops": round(flops / (ms_mbs * 1e-3) / 1e12, 1), "gemm_plain_tflops": round(flops / (ms_plain * 1e-3) / 1e12, 1),
           "quantize_W_gbps": round(xw[0].numel() * bytes_per_elt / (ms_qw * 1e-3) / 1e9, 1),
           "peak_context": ("published dense FP6 peak 10.1 PFLOP/s" if six else "published dense FP8 peak 5.0 PFLOP/s") + "; the paper has no figure for this format"}
    a, w = xa[0][:QSNR_AB_ROWS], xw[0][:QSNR_AB_COLS]
    ref = a.to(torch.float64) @ w.to(torch.float64).T
    q = {}
    fam = "MXFP6" if six else "MXFP8"
    for name, rule, mbs in ((fam + "-OCP", "ocp", False), (fam + "-OAS", "oas", False), (fam + "-OAS+MBS-S", "oas", True)):
        ta, tw = mx.mx_quantize_elem(a, elem, rule, mbs), mx.mx_quantize_elem(w, elem, rule, mbs)
        c = mx.mx_gemm_mbs_elem(elem, *ta, elem, *tw, "f32")
        q[name] = round(float(10.0 * torch.log10((ref * ref).sum() / ((ref - c.to(torch.float64)) ** 2).sum())), 3)
    res["qsnr_ab_db_gpu"] = q
    # MBS-Dynamic on these formats (exact search over 16 candidates), the weights of this shape
    ms_dyn = time_loop(torch, lambda i: mx.mx_quantize_elem_mbs_dynamic(xw[i % len(xw)], elem, "oas", 0, 16, 16, *qw[i % len(qw)]), max(3, n // 4))
    res["quantize_dynamic_W_ms"] = round(ms_dyn, 4)
    res["quantize_static_W_ms"] = round(ms_qw, 4)
    for i in range(len(qw)):  # (the timed search left its words in qw: back to the static ones)
        mx.mx_quantize_elem(xw[i], elem, "oas", True, *qw[i])
    return res


def elem_decode_extras(mx, torch, synth, np, elem):
    """Decode in MXFP8 / MXFP6: 16 activation rows against a 4096 x 4096 and a 14336 x 4096 weight through the few-row
    kernel (quantized activations given), replayed from a HIP graph over enough copies of the weights to exceed the
    Infinity Cache.  Bound: the weight bytes streamed once."""
    res = {}
    bpe = (0.75 if elem in ("e2m3", "e3m2") else 1.0) + 1 / 32 + 1 / 128
    for n, copies in ((4096, 20), (14336, 6)):
        a_bits, w_bits = synth.decode_skinny(n, 4096)
        xa = torch.from_numpy(a_bits.view(np.int16)).view(torch.bfloat16).cuda()
        w0 = mx.mx_quantize_elem(torch.from_numpy(w_bits.view(np.int16)).view(torch.bfloat16).cuda(), elem, "oas")
        ws = [tuple(t.clone() for t in w0) for _ in range(copies)]
        aq = mx.mx_quantize_elem(xa, elem, "oas")
        c = torch.empty((16, n), dtype=torch.bfloat16, device="cuda")
        mx.mx_gemm_mbs_elem(elem, *aq, elem, *ws[0], "bf16", out=c)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(copies):
                mx.mx_gemm_mbs_elem(elem, *aq, elem, *ws[i], "bf16", out=c)
        us = time_loop(torch, lambda i: graph.replay(), 20, warm=5) * 1e3 / copies
        res["N=%d" % n] = {"gemm_us": round(us, 2), "weight_gbps": round(n * 4096 * bpe / us / 1e3, 1)}
        del ws
    res["bound"] = "hbm (weights streamed once: %.3f B per weight element)" % bpe
    return res


def moe_extras(mx, torch, synth, np, metrics, args):
    """The mixture-of-experts configuration: 8192 tokens x 2880 routed to 4 of 32 experts (Zipf load), rows
    gathered into expert order, every expert's 2880x2880 weight quantized with OAS + MBS-S; one step = quantize
    the 32768 gathered rows + the grouped MBS GEMM.  TFLOP/s on sum_e 2 M_e N K; K = 2880 ends in half a macro block."""
    x_bits, w_bits, offsets, token_of_row = synth.moe()
    G, dim = 32, 2880
    dev = torch.device("cuda:0")
    xa = torch.from_numpy(x_bits[token_of_row].view(np.int16)).view(torch.bfloat16).to(dev)
    xw = torch.from_numpy(w_bits.view(np.int16)).view(torch.bfloat16).to(dev)
    b = mx.mx_quantize_mbs(xw, "oas")
    a = mx.mx_quantize_mbs(xa, "oas")
    off = torch.from_numpy(np.asarray(offsets, dtype=np.int64)).to(dev)
    c = torch.empty((xa.shape[0], dim), dtype=torch.bfloat16, device=dev)
    n = max(5, min(args.steps, 60))
    rows = int(offsets[-1])
    flops = 2.0 * rows * dim * dim
    ms_g = time_loop(torch, lambda i: mx.mx_gemm_mbs_grouped(*a, *b, off, dim, "bf16", out=c), n)
    ms_p = time_loop(torch, lambda i: mx.mx_gemm_mbs_grouped(a[0], a[1], None, b[0], b[1], None, off, dim, "bf16", out=c), n)

    def step(i):
        mx.mx_quantize_mbs(xa, "oas", *a)
        mx.mx_gemm_mbs_grouped(*a, *b, off, dim, "bf16", out=c)

    ms_s = time_loop(torch, step, n)
    ms_qw = time_loop(torch, lambda i: mx.mx_quantize_mbs(xw, "oas", *b), n)
    loads = np.diff(np.asarray(offsets)).astype(int).tolist()
    tg, tp = flops / (ms_g * 1e-3) / 1e12, flops / (ms_p * 1e-3) / 1e12
    # the same routing and the same K in MXFP8 / MXFP6 through the grouped entry point of those formats
    elem_grouped = {"K": dim}
    for elem in ("e4m3", "e2m3"):
        ea, eb = mx.mx_quantize_elem(xa, elem, "oas"), mx.mx_quantize_elem(xw, elem, "oas")
        ms_e = time_loop(torch, lambda i: mx.mx_gemm_mbs_elem_grouped(elem, *ea, elem, *eb, off, dim, "bf16", out=c), n)
        elem_grouped[elem + "_grouped_gemm_mbs_tflops"] = round(flops / (ms_e * 1e-3) / 1e12, 1)
        del ea, eb
    return {
        "mxfp8_mxfp6_grouped": elem_grouped,
        "workload": "32 experts of 2880x2880 N(0,0.02^2), 8192 tokens x 2880 (Student-t(4), 1%% channels x20) routed top-4, "
                    "P(e) ~ (e+1)^-1.1; %d rows in expert order" % rows,
        "kernel": mx.gemm_plan(rows, dim, dim, True, True, True),
        "grouped_gemm_mbs_tflops": round(tg, 1), "grouped_gemm_mbs_frac_of_peak": round(tg / metrics.MFMA_FP4_PEAK_TFLOPS, 4),
        "grouped_gemm_plain_tflops": round(tp, 1), "mbs_overhead": round(metrics.overhead_fraction(tp, tg), 4),
        "step_tflops": round(flops / (ms_s * 1e-3) / 1e12, 1), "ms_per_step": round(ms_s, 4),
        "quantize_expert_weights_gbps": round(xw.numel() * metrics.QUANT_BYTES_PER_ELT_MBS / (ms_qw * 1e-3) / 1e9, 1),
        "expert_load_histogram": loads,
    }


def decode_extras(mx, torch, synth, np):
    """The decode configuration (16 activation rows, K = 4096, weights quantized offline): one step = quantize
    the activations + few-row MBS GEMM, as two launches and as the one fused launch.  The steps are replayed
    from a HIP graph (a launch from Python costs as much as these kernels run) that walks over enough copies
    of the weights to exceed the 256 MB Infinity Cache, so the weights stream from HBM."""
    res = {}
    for n, copies in ((4096, 32), (14336, 10)):
        a_bits, w_bits = synth.decode_skinny(n, 4096)
        xa = torch.from_numpy(a_bits.view(np.int16)).view(torch.bfloat16).cuda()
        w0 = mx.mx_quantize_mbs(torch.from_numpy(w_bits.view(np.int16)).view(torch.bfloat16).cuda(), "oas")
        ws = [tuple(t.clone() for t in w0) for _ in range(copies)]
        aq = mx.mx_quantize_mbs(xa, "oas")
        c = torch.empty((16, n), dtype=torch.bfloat16, device="cuda")
        mx.mx_gemm_mbs(*aq, *ws[0], "bf16", out=c)
        mx.mx_gemm_mbs_quantize_a(xa, "oas", *ws[0], "bf16", out=c)
        torch.cuda.synchronize()

        def two(i):
            mx.mx_quantize_mbs(xa, "oas", *aq)
            mx.mx_gemm_mbs(*aq, *ws[i], "bf16", out=c)

        def fused(i):
            mx.mx_gemm_mbs_quantize_a(xa, "oas", *ws[i], "bf16", out=c)

        entry = {}
        for name, fn in (("quantize_then_gemm", two), ("fused", fused)):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for i in range(copies):
                    fn(i)
            us = time_loop(torch, lambda i: graph.replay(), 20, warm=5) * 1e3 / copies
            entry[name + "_us"] = round(us, 2)
        wbytes = n * 4096 * 0.5390625
        entry["fused_weight_gbps"] = round(wbytes / entry["fused_us"] / 1e3, 1)
        res["N=%d" % n] = entry
        del ws
    res["bound"] = "hbm (weights streamed once: 0.539 B per weight element)"
    return res


def square_shapes(mx, torch, synth, np, metrics):
    """Plain and MBS GEMM on the square shapes M = N = K of the paper's Tab. 4 (its numbers are for another
    machine and are context only): TFLOP/s and the overhead 1 - MBS/plain per shape, and their average."""
    res, overheads = {}, []
    for n in (512, 1024, 2048, 4096, 8192):
        a = mx.mx_quantize_mbs(torch.from_numpy(synth.activations_student_t(n, n, 4.0, 0.01, 20.0, 11).view(np.int16)).view(torch.bfloat16).cuda(), "oas")
        b = mx.mx_quantize_mbs(torch.from_numpy(synth.gaussian(n, n, 0.02, 12).view(np.int16)).view(torch.bfloat16).cuda(), "oas")
        c = torch.empty((n, n), dtype=torch.bfloat16, device="cuda")
        iters = 200 if n <= 2048 else 50
        warm = 20 if n <= 1024 else 150   # the larger shapes only show their rate at sustained clocks
        ms_p = time_loop(torch, lambda i: mx.mx_gemm(a[0], a[1], b[0], b[1], "bf16", out=c), iters, warm)
        ms_m = time_loop(torch, lambda i: mx.mx_gemm_mbs(*a, *b, "bf16", out=c), iters, warm)
        tp, tm = 2.0 * n ** 3 / ms_p / 1e9, 2.0 * n ** 3 / ms_m / 1e9
        overheads.append(metrics.overhead_fraction(tp, tm))
        res[str(n)] = {"plain_tflops": round(tp, 1), "mbs_tflops": round(tm, 1), "overhead": round(overheads[-1], 4)}
    res["average_overhead"] = round(sum(overheads) / len(overheads), 4)
    res["paper_context"] = "Tab. 4 (NVIDIA B200): overheads 14.84, 9.01, 0.17, 2.42, 4.73 %, average 6.2 %"
    return res


def cpu_baseline(np, synth, a_bits, w_bits, M, N, K, brief):
    """The CPU oracle as it stands, timed on a bounded sample of the same workload (about 20-30 s in all): with
    all its threads, and on one thread.  Whole-step time is extrapolated linearly from the two rates."""
    import oracle

    oracle.build()
    threads = oracle.num_threads()
    flops = 2.0 * M * N * K

    def legs(rows_q, rows_g, wq=None):
        t0 = time.perf_counter()
        w = oracle.quantize(w_bits[:rows_q], "oas", mbs=True)
        tq = time.perf_counter() - t0
        a = oracle.quantize(a_bits[:rows_g], "oas", mbs=True)
        wq = w if wq is None else wq
        t0 = time.perf_counter()
        oracle.gemm(a, wq, rows=np.arange(rows_g))
        tg = time.perf_counter() - t0
        return rows_q * K / tq, 2.0 * rows_g * N * K / tg, tq, tg, wq

    q_rate, g_rate, tq, tg, wq_all = legs(N, 24)        # all of W; 24 output rows, all N columns
    est_step_s = (M + N) * K / q_rate + flops / g_rate
    res = {
        "value": round(flops / est_step_s / 1e12, 6),
        "unit": "TFLOP/s",
        "cores": threads,
        "kind": "oracle",
        "sample": "quantize %d of %d W rows (%.2f s), fp64 GEMM of %d of %d output rows (%.2f s); whole-step time "
                  "extrapolated linearly from the two rates" % (N, N, tq, 24, M, tg),
        "quantize_melem_per_s": round(q_rate / 1e6, 2),
        "gemm_gflops": round(g_rate / 1e9, 3),
    }
    old = oracle.set_num_threads(1)
    try:
        q1, g1, tq1, tg1, _ = legs(512, 2, wq_all)
    finally:
        oracle.set_num_threads(old)
    res["single_thread"] = {
        "value": round(flops / ((M + N) * K / q1 + flops / g1) / 1e12, 6), "unit": "TFLOP/s", "cores": 1,
        "sample": "quantize 512 W rows (%.2f s), fp64 GEMM of 2 output rows (%.2f s)" % (tq1, tg1),
        "quantize_melem_per_s": round(q1 / 1e6, 2), "gemm_gflops": round(g1 / 1e9, 3),
    }
    if brief:
        return res
    # the quantizer oracle on a bounded sample of every configuration's tensors
    per_cfg = {}
    tiny_a, tiny_w = synth.tiny(0)
    dec_a, _ = synth.decode_skinny(16, 4096)
    a8, w8 = synth.llama8b_ffn_up(1024, 2048, 4096)
    moe_w = synth.gaussian(2048, 2880, 0.02, 7)
    for name, bits in (("tiny A 64x512", tiny_a), ("tiny W 256x512", tiny_w), ("llama3-8b A 1024x4096", a8), ("llama3-8b W 2048x4096", w8),
                       ("decode A 16x4096", dec_a), ("llama3-70b A 2048x8192", a_bits[:2048]), ("llama3-70b W 2048x8192", w_bits[:2048]),
                       ("moe expert W 2048x2880", moe_w)):
        t0 = time.perf_counter()
        oracle.quantize(bits, "oas", mbs=True)
        per_cfg[name] = round(bits.size / (time.perf_counter() - t0) / 1e6, 1)
    res["quantize_melem_per_s_by_tensor"] = per_cfg
    x = a_bits[:QSNR_ROWS]
    ref = oracle.bf16_to_f64(x)
    ladder = {}
    for name, rule, mbs in QSNR_LADDER:
        q = oracle.quantize(x, rule, mbs=mbs)
        ladder[name] = round(oracle.qsnr_db(ref, oracle.dequantize(q[0], q[1], q[2])), 3)
    res["qsnr_db_oracle"] = ladder
    xw = w_bits[:QSNR_ROWS]
    refw = oracle.bf16_to_f64(xw)
    ladder_w = {}
    for name, q in (("+oas", oracle.quantize(xw, "oas")), ("+oas+mbs-s", oracle.quantize(xw, "oas", mbs=True)),
                    ("+oas+mbs-d", oracle.quantize_mbs_dynamic(xw, "oas")),
                    ("+oas+mbs-d(table)", oracle.quantize_mbs_dynamic_lut(xw, oracle.mbs_lut(), "oas"))):
        ladder_w[name] = round(oracle.qsnr_db(refw, oracle.dequantize(q[0], q[1], q[2])), 3)
    res["qsnr_db_oracle_weights"] = ladder_w
    a_s, w_s = a_bits[:QSNR_AB_ROWS], w_bits[:QSNR_AB_COLS]
    ref_ab = oracle.matmul_bf16(a_s, w_s)
    ladder_ab = {}
    for name, rule, mbs in QSNR_AB_LADDER:
        qa_ = oracle.quantize(a_s, rule, mbs=mbs != "none")
        qw_ = oracle.quantize_mbs_dynamic(w_s, rule) if mbs == "hybrid" else oracle.quantize(w_s, rule, mbs=mbs != "none")
        ladder_ab[name] = round(oracle.qsnr_db(ref_ab, oracle.gemm(qa_, qw_)), 3)
    res["qsnr_ab_db_oracle"] = ladder_ab
    return res


if __name__ == "__main__":
    main()
