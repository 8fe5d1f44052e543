"""Host-side bookkeeping for the benchmark: throughput, roofline and overhead conventions."""
from __future__ import annotations

# MI355X published peaks used as roofline denominators.
HBM_PEAK_GBPS = 8000.0            # HBM3E
MFMA_FP4_PEAK_TFLOPS = 10066.0    # 256 CU x 4 SIMD x 4096 FLOP/clk x 2.4 GHz (dense MXFP4)

# Algorithmic HBM bytes per quantized element: bf16 in, packed FP4 + E8M0/32 (+ MBS word/128) out.
QUANT_BYTES_PER_ELT_PLAIN = 2.0 + 0.5 + 1.0 / 32.0
QUANT_BYTES_PER_ELT_MBS = QUANT_BYTES_PER_ELT_PLAIN + 1.0 / 128.0


def gemm_flops(M: int, N: int, K: int) -> float:
    """FP4 multiply-add work of C = A.B^T counted as 2 FLOP per MAC."""
    return 2.0 * M * N * K


def overhead_fraction(tflops_plain: float, tflops_mbs: float) -> float:
    """GEMM overhead of the MBS kernel over the plain MXFP4 kernel, in the convention of the
    paper's Tab. 4: 1 - TFLOPS_MBS / TFLOPS_plain (e.g. 35.90 -> 30.57 is 14.84 %)."""
    return 1.0 - tflops_mbs / tflops_plain


def gemm_operand_bytes(M: int, N: int, K: int, mbs: bool) -> float:
    """Algorithmic operand bytes of one GEMM launch: each code, E8M0 byte and MBS word read once."""
    per_elt = 0.5 + 1.0 / 32.0 + (1.0 / 128.0 if mbs else 0.0)
    return (M + N) * K * per_elt


# HBM traffic of one MBS GEMM launch on the bench shape (bytes), from the FETCH_SIZE and WRITE_SIZE counter
# runs whose summaries are kept under profiles/ (scaled by the copy-kernel calibration stated there).
GEMM_MBS_TRAFFIC_BYTES = int((202.7 + 144.4) * 2 ** 20)  # read 202.7 MiB + written 144.4 MiB
