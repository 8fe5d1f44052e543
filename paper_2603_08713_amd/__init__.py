"""MI355X-native MXFP4 quantization with Overflow-Aware Scaling and Macro Block Scaling, and the
block-scaled GEMM with the MBS correction.

This package is argument marshalling only: every step runs in the HIP kernels of ``libmx4.so``
(C ABI declared in ``include/mx4.h``).  PyTorch provides device memory and streams.  There is no
CPU fallback: if the library is missing, importing :mod:`paper_2603_08713_amd.binding` members that
need it raises.
"""
from .binding import (  # noqa: F401
    MX_OUT_BF16, MX_OUT_F32, MX_RULE_FLOOR, MX_RULE_OAS, MX_RULE_OCP, MxError, elem_code_bytes, load_library, forced, gemm_plan,
    mx_dequantize, mx_dequantize_elem, mx_gemm, mx_gemm_mbs, mx_gemm_mbs_elem, mx_gemm_mbs_elem_grouped, mx_gemm_mbs_grouped, mx_gemm_mbs_quantize_a, mx_quantize,
    mx_quantize_elem, mx_quantize_elem_mbs_dynamic, mx_quantize_mbs,
    mx_mbs_lut_build, mx_quantize_mbs_dynamic, mx_quantize_mbs_dynamic_lut, mx_quantize_mbs_dynamic_lut_static, mx_quantize_mbs_pair, mx_quantize_oas, mx_status_string, mx_version,
)
