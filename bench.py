#!/usr/bin/env python3
"""Benchmark of the MXFP4 OAS+MBS hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input resident in HBM:
    quantize A and W (OAS + MBS-S, one launch)  ->  C = A.W^T with the MBS correction (bf16 out)
on the Llama-3-8B FFN up-projection shape (A 4096x4096, W 14336x4096).  Prints ONE JSON line.

`value` is 2*M*N*K divided by the wall time of a whole step (quantizers included), at the sustained
rate: the device is first brought out of its idle clocks by an untimed run of the same step.  The roofline
object is for the dominant kernel, the MBS GEMM, timed with HIP events on the launch stream inside
the timed region.  The CPU oracle is timed on a bounded sample as a reported baseline.
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

M, N, K = 4096, 14336, 4096
WORKLOAD = "llama3-8b-ffn-up: A 4096x4096 bf16 Student-t(4) + 1% outlier channels x20, W 14336x4096 bf16 N(0,0.02^2)"


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=300)
    p.add_argument("--warmup", type=int, default=100)
    p.add_argument("--prewarm-ms", type=float, default=150.0,
                   help="untimed run of the step before the warm-up steps, so that the device has left its idle "
                        "clocks (it takes about 100 steps, 30 ms, from a cold start); 0 disables it")
    p.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    p.add_argument("--no-extras", action="store_true", help="skip plain-GEMM / dequantize / QSNR side measurements")
    return p.parse_args()


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
    dev = torch.device("cuda:0")

    def to_dev(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)

    a_bits, w_bits = synth.llama8b_ffn_up(M, N, K)
    # Distinct buffers rotated per step so that bf16 inputs are read from HBM, not from the 256 MB
    # Infinity Cache: 8 x 32 MiB of A, 5 x 112 MiB of W, 3 x 112 MiB of C.
    xa = [to_dev(a_bits) for _ in range(8)]
    xw = [to_dev(w_bits) for _ in range(5)]
    qa = [tuple(torch.empty(s, dtype=torch.uint8, device=dev) for s in ((M, K // 2), (M, K // 32), (M, K // 128)))
          for _ in xa]
    qw = [tuple(torch.empty(s, dtype=torch.uint8, device=dev) for s in ((N, K // 2), (N, K // 32), (N, K // 128)))
          for _ in xw]
    cs = [torch.empty((M, N), dtype=torch.bfloat16, device=dev) for _ in range(3)]

    def step(i, ev=None):
        # ev: 3 events bracketing the quantizer launch and the GEMM launch
        a, w, c = i % len(xa), i % len(xw), i % len(cs)
        if ev:
            ev[0].record()
        mx.mx_quantize_mbs_pair(xa[a], xw[w], "oas", qa[a], qw[w])     # both GEMM operands, one launch
        if ev:
            ev[1].record()
        mx.mx_gemm_mbs(qa[a][0], qa[a][1], qa[a][2], qw[w][0], qw[w][1], qw[w][2], "bf16", out=cs[c])
        if ev:
            ev[2].record()

    # From idle the device needs some tens of milliseconds of work before its clocks settle; the number of
    # interest is the sustained rate, so that ramp is kept out of the timed region (and reported).
    prewarm_steps = 0
    t_pre = time.perf_counter()
    while (time.perf_counter() - t_pre) * 1e3 < args.prewarm_ms:
        for i in range(10):
            step(prewarm_steps + i)
        torch.cuda.synchronize()
        prewarm_steps += 10
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    def avg(j):
        return sum(e[j].elapsed_time(e[j + 1]) for e in events) / len(events)

    ms_q, ms_gemm = avg(0), avg(1)
    flops = metrics.gemm_flops(M, N, K)
    value = flops / (ms_per_step * 1e-3) / 1e12
    gemm_tflops = flops / (ms_gemm * 1e-3) / 1e12
    bpe = metrics.QUANT_BYTES_PER_ELT_MBS
    q_gbps = (M + N) * K * bpe / (ms_q * 1e-3) / 1e9

    out = {
        "metric": "OAS+MBS MXFP4 GEMM TFLOP/s (whole step: quantize A and W, MBS GEMM)",
        "value": round(value, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "mxfp4 (E2M1 x E8M0/32, fp32 accumulate, bf16 out)",
        "data": "synthetic",
        "config": {"workload": WORKLOAD, "M": M, "N": N, "K": K, "rule": "oas", "mbs": "static/128",
                   "buffers": "inputs rotated over %d A / %d W / %d C buffers" % (len(xa), len(xw), len(cs)),
                   "prewarm_steps": prewarm_steps},
        "roofline": {
            "kernel": "gemm_ring_kernel<256x128 tile, MBS> (mx_gemm_mbs)",
            "bound": "mfma",
            "achieved": round(gemm_tflops, 2),
            "peak": metrics.MFMA_FP4_PEAK_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(gemm_tflops / metrics.MFMA_FP4_PEAK_TFLOPS, 4),
            "traffic": metrics.GEMM_MBS_TRAFFIC_BYTES,
            "algorithmic_operand_bytes": metrics.gemm_operand_bytes(M, N, K, mbs=True) + M * N * 2,
            "avg_launch_ms": round(ms_gemm, 4),
        },
        "quantize": {
            "bound": "hbm", "bytes_per_element": bpe, "peak": metrics.HBM_PEAK_GBPS, "unit": "GB/s",
            "kernel": "quantize_kernel<mbs> on A and W in one launch (mx_quantize_mbs_pair)",
            "ms": round(ms_q, 4), "achieved": round(q_gbps, 1), "frac": round(q_gbps / metrics.HBM_PEAK_GBPS, 4),
        },
    }

    if not args.no_extras:
        out["extras"] = extras(mx, torch, metrics, xa, xw, qa, qw, cs, flops, gemm_tflops, args)
        out["extras"]["decode_m16_k4096"] = decode_extras(mx, torch, synth, np)
        out["extras"]["square_shapes"] = square_shapes(mx, torch, synth, np, metrics)
        out["extras"]["mxfp8_e4m3"] = mxfp8_extras(mx, torch, xa, xw, cs, flops, args)
        out["extras"]["mxfp6_e2m3"] = mxfp8_extras(mx, torch, xa, xw, cs, flops, args, elem="e2m3")
        out["extras"]["qsnr_db_gpu"] = qsnr_ladder_gpu(mx, torch, xa[0][:QSNR_ROWS])
        out["extras"]["qsnr_db_gpu_weights"] = qsnr_weights_gpu(mx, torch, xw[0][:QSNR_ROWS])
        out["extras"]["qsnr_ab_db_gpu"] = qsnr_ab_gpu(mx, torch, xa[0], xw[0])
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(np, a_bits, w_bits, flops, metrics)
    print(json.dumps(out))


QSNR_ROWS = 256  # rows of the activation tensor the QSNR ladder is computed on, by both paths
QSNR_LADDER = (("mxfp4", "ocp", False), ("+oas", "oas", False), ("+mbs", "ocp", True), ("+oas+mbs", "oas", True))


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


def mxfp8_extras(mx, torch, xa, xw, cs, flops, args, elem="e4m3"):
    """The same step in MXFP8 (E4M3 elements) or MXFP6 (E2M3, packed codes), OAS and MBS restated on the element
    format's own constants: both quantizers, then the MBS GEMM; and QSNR(AB) of the plain OCP rule against
    OAS + MBS-S on the product sample."""
    n = max(5, min(args.steps, 100))
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
    res = {"step_tflops": round(flops / (ms_step * 1e-3) / 1e12, 1), "ms_per_step": round(ms_step, 4),
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
    return res


def qsnr_weights_gpu(mx, torch, x):
    """QSNR (dB) of the weight tensor with OAS alone, with the static MBS word and with the searched one
    (MBS-Dynamic, the weight half of the paper's MBS-Hybrid, Sec. 4.3.1 and 4.4), through the HIP kernels."""
    res = {}
    ref = x.to(torch.float64)
    for name, q in (("+oas", mx.mx_quantize(x, "oas") + (None,)), ("+oas+mbs-s", mx.mx_quantize_mbs(x, "oas")),
                    ("+oas+mbs-d", mx.mx_quantize_mbs_dynamic(x, "oas"))):
        back = mx.mx_dequantize(q[0], q[1], q[2], "f32").to(torch.float64)
        res[name] = round(float(10.0 * torch.log10((ref * ref).sum() / ((ref - back) ** 2).sum())), 3)
    res["sample"] = "first %d rows of W" % QSNR_ROWS
    return res


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


def extras(mx, torch, metrics, xa, xw, qa, qw, cs, flops, gemm_tflops, args):  # noqa: C901
    """Side measurements outside the timed region: plain MXFP4 GEMM on the same shape (for the
    Tab. 4 style overhead), a device copy as the achievable-HBM yardstick, the dequantizer."""
    n = max(5, min(args.steps, 100))
    res = {}
    # operands quantized without MBS for the plain kernel (same codes layout, OCP rule)
    pa = mx.mx_quantize(xa[0], "ocp")
    pw = mx.mx_quantize(xw[0], "ocp")
    ms_plain = time_loop(torch, lambda i: mx.mx_gemm(pa[0], pa[1], pw[0], pw[1], "bf16", out=cs[i % len(cs)]), n)
    ms_mbs = time_loop(torch, lambda i: mx.mx_gemm_mbs(qa[0][0], qa[0][1], qa[0][2], qw[0][0], qw[0][1], qw[0][2],
                                                        "bf16", out=cs[i % len(cs)]), n)
    plain_tflops = flops / (ms_plain * 1e-3) / 1e12
    mbs_tflops = flops / (ms_mbs * 1e-3) / 1e12
    res["gemm_plain_tflops"] = round(plain_tflops, 2)
    res["gemm_mbs_tflops"] = round(mbs_tflops, 2)
    res["gemm_mbs_overhead"] = round(metrics.overhead_fraction(plain_tflops, mbs_tflops), 4)
    # what the matrix cores sustain with nothing else going on: the practical ceiling for these clocks and
    # this power limit (the published peak assumes 2.4 GHz, which random operand bits do not reach)
    res["mfma_issue_only_tflops"] = {"constant_operands": round(mx.mfma_rate(False), 1),
                                     "random_operands": round(mx.mfma_rate(True), 1)}
    res["paper_context"] = "paper reports 6.2% average MBS GEMM overhead on NVIDIA B200 / CUTLASS 4.3.0 (other hardware)"
    # copy yardstick: read + write of the same byte count as one W tensor
    src, dst = xw[1], xw[2]
    ms_copy = time_loop(torch, lambda i: dst.copy_(src), n)
    res["copy_gbps"] = round(2 * src.numel() * 2 / (ms_copy * 1e-3) / 1e9, 1)
    # plain-rule quantizer and dequantizer throughput (algorithmic bytes)
    ms_q = time_loop(torch, lambda i: mx.mx_quantize(xw[i % len(xw)], "ocp", pw[0], pw[1]), n)
    res["quantize_plain_W_gbps"] = round(xw[0].numel() * metrics.QUANT_BYTES_PER_ELT_PLAIN / (ms_q * 1e-3) / 1e9, 1)
    # the step's quantizer launch on its own (back to back, inputs rotating): its rate without the GEMM between launches
    ms_pair = time_loop(torch, lambda i: mx.mx_quantize_mbs_pair(xa[i % len(xa)], xw[i % len(xw)], "oas", qa[i % len(qa)], qw[i % len(qw)]), n)
    res["quantize_pair_alone_gbps"] = round((xa[0].numel() + xw[0].numel()) * metrics.QUANT_BYTES_PER_ELT_MBS / (ms_pair * 1e-3) / 1e9, 1)
    # MBS-Dynamic (offline weight quantization: 17 evaluations of the window instead of one)
    ms_s = time_loop(torch, lambda i: mx.mx_quantize_mbs(xw[i % len(xw)], "oas", *qw[i % len(qw)]), n)
    ms_dyn = time_loop(torch, lambda i: mx.mx_quantize_mbs_dynamic(xw[i % len(xw)], "oas", 0, 16, 16, *qw[i % len(qw)]), n)
    res["quantize_dynamic_W"] = {"ms": round(ms_dyn, 4), "static_ms": round(ms_s, 4), "slowdown_vs_static": round(ms_dyn / ms_s, 2),
                                 "gbps": round(xw[0].numel() * metrics.QUANT_BYTES_PER_ELT_MBS / (ms_dyn * 1e-3) / 1e9, 1),
                                 "candidates": "static word + 16 equally spaced",
                                 "paper_context": "paper reports its MBS-D kernel 2.5-3x slower than MBS-S (NVIDIA B200)"}
    # the timing loop above rewrote qw with searched words: put the static ones back for what follows
    for i in range(len(qw)):
        mx.mx_quantize_mbs(xw[i % len(xw)], "oas", *qw[i])
    deq = torch.empty((xw[0].shape[0], xw[0].shape[1]), dtype=torch.bfloat16, device=xw[0].device)
    ms_d = time_loop(torch, lambda i: mx.mx_dequantize(qw[i % len(qw)][0], qw[i % len(qw)][1], qw[i % len(qw)][2],
                                                       "bf16", out=deq), n)
    res["dequantize_W_gbps"] = round(xw[0].numel() * metrics.QUANT_BYTES_PER_ELT_MBS / (ms_d * 1e-3) / 1e9, 1)
    return res


def cpu_baseline(np, a_bits, w_bits, flops, metrics):
    """The CPU oracle as it stands, timed on a bounded sample of the same workload."""
    import oracle

    oracle.build()
    threads = oracle.num_threads()
    rows_q = N                                      # the whole W tensor gives the quantizer rate
    t0 = time.perf_counter()
    w = oracle.quantize(w_bits, "oas", mbs=True)
    tq = time.perf_counter() - t0
    q_rate = rows_q * K / tq                        # elements / s
    a = oracle.quantize(a_bits[:256], "oas", mbs=True)
    rows = np.arange(0, 256)                        # 256 output rows, all N columns (about 10-15 s)
    t0 = time.perf_counter()
    oracle.gemm(a, w, rows=rows)
    tg = time.perf_counter() - t0
    g_rate = 2.0 * len(rows) * N * K / tg           # flop / s
    est_step_s = (M + N) * K / q_rate + flops / g_rate
    x = a_bits[:QSNR_ROWS]
    ref = oracle.bf16_to_f64(x)
    ladder = {}
    for name, rule, mbs in QSNR_LADDER:
        q = oracle.quantize(x, rule, mbs=mbs)
        ladder[name] = round(oracle.qsnr_db(ref, oracle.dequantize(q[0], q[1], q[2])), 3)
    xw = w_bits[:QSNR_ROWS]
    refw = oracle.bf16_to_f64(xw)
    ladder_w = {}
    for name, q in (("+oas", oracle.quantize(xw, "oas")), ("+oas+mbs-s", oracle.quantize(xw, "oas", mbs=True)),
                    ("+oas+mbs-d", oracle.quantize_mbs_dynamic(xw, "oas"))):
        ladder_w[name] = round(oracle.qsnr_db(refw, oracle.dequantize(q[0], q[1], q[2])), 3)
    a_s, w_s = a_bits[:QSNR_AB_ROWS], w_bits[:QSNR_AB_COLS]
    ref_ab = oracle.matmul_bf16(a_s, w_s)
    ladder_ab = {}
    for name, rule, mbs in QSNR_AB_LADDER:
        qa_ = oracle.quantize(a_s, rule, mbs=mbs != "none")
        qw_ = oracle.quantize_mbs_dynamic(w_s, rule) if mbs == "hybrid" else oracle.quantize(w_s, rule, mbs=mbs != "none")
        ladder_ab[name] = round(oracle.qsnr_db(ref_ab, oracle.gemm(qa_, qw_)), 3)
    return {
        "qsnr_db_oracle": ladder,
        "qsnr_db_oracle_weights": ladder_w,
        "qsnr_ab_db_oracle": ladder_ab,
        "value": round(flops / est_step_s / 1e12, 6),
        "unit": "TFLOP/s",
        "cores": threads,
        "kind": "oracle",
        "sample": "quantize %d of %d W rows (%.2f s), fp64 GEMM of %d of %d output rows (%.2f s); whole-step time "
                  "extrapolated linearly from the two rates" % (rows_q, N, tq, len(rows), M, tg),
        "quantize_melem_per_s": round(q_rate / 1e6, 2),
        "gemm_gflops": round(g_rate / 1e9, 3),
    }


if __name__ == "__main__":
    main()
