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


# ---- secondary bound of the MBS GEMM: vector-ALU instruction issue -----------------------------------
# Measured on this device: beside matrix instructions a SIMD issues one fp32 vector instruction per 4.6 clocks,
# whichever of its wavefronts it comes from (packed fp32 is off in this build), and every matrix instruction holds
# the same issue port for about 12 clocks.  One macro block of a 32 x 32 output fragment is two 32x32x64 matrix
# instructions = 2 * 32 * 32 * 128 FLOP; the correction adds `valu_per_fragment` vector instructions to it and
# brings the matrix instructions per fragment to `mfma_per_fragment`.
SIMDS = 256 * 4
CLOCK_GHZ = 2.4
VALU_ISSUE_CLOCKS = 4.6
MFMA_ISSUE_CLOCKS = 12
FRAGMENT_FLOP = 2.0 * 32 * 32 * 128


def valu_issue_ceiling_tflops(valu_per_fragment: float, mfma_per_fragment: float = 2.0) -> float:
    """TFLOP/s at which the vector-issue port of every SIMD is busy all the time, at the published clock."""
    clocks = valu_per_fragment * VALU_ISSUE_CLOCKS + mfma_per_fragment * MFMA_ISSUE_CLOCKS
    return FRAGMENT_FLOP / clocks * SIMDS * CLOCK_GHZ * 1e9 / 1e12


def read_profile_value(path: str, key: str):
    """A `key = number` line of a committed rocprofv3 summary under profiles/ (None if the file or key is missing)."""
    try:
        with open(path) as f:
            for line in f:
                if line.strip().startswith(key) and "=" in line:
                    return float(line.split("=", 1)[1].split()[0])
    except OSError:
        pass
    return None
