// Development entry points of libmx4.so (private: not part of the public ABI in include/mx4.h).
//
// Each is a public entry point with one more argument that picks, for this call only, an implementation the
// dispatcher would not pick by itself, so that the tests can hold every rounding implementation of the
// quantizers and every form and tile shape of the GEMM kernels to the same reference results.  They keep no state: the library
// has no process-wide switches, and a call here never changes what a public entry point does.
#pragma once

#include "mx4.h"

#ifdef __cplusplus
extern "C" {
#endif

// mx_quantize (use_mbs == 0, mbs ignored) or mx_quantize_mbs (use_mbs != 0) with the rounding implementation
// chosen: hw_convert != 0 = the hardware fp32 -> E2M1 convert instruction (what the public entry points use),
// 0 = ordinary arithmetic.  Both must give identical codes.
int mx_internal_quantize(const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule, int use_mbs,
                         int hw_convert, uint8_t* codes, uint8_t* scales, uint8_t* mbs, void* stream);

// mx_quantize_elem with the rounding implementation chosen (as above, for the 8-bit formats' converts).
int mx_internal_quantize_elem(mx_elem_t elem, const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule,
                              int use_mbs, int hw_convert, uint8_t* codes, uint8_t* scales, uint8_t* mbs, void* stream);

// mx_gemm (mbs_entry == 0), mx_gemm_mbs (mbs_entry != 0, grouped == 0) or mx_gemm_mbs_grouped (grouped != 0)
// with the kernel form and tile shape forced; force_shape < 0 = automatic, the codes are listed in mx_gemm.hip.
// A shape that cannot take the problem returns MX_EINVAL.
int mx_internal_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs_or_null,
                     const uint8_t* b_codes, const uint8_t* b_scales, const uint8_t* b_mbs_or_null, int grouped,
                     int32_t num_groups, const int64_t* row_offsets, int64_t M, int64_t N, int64_t K, mx_dtype_t c_dtype,
                     void* C, int64_t ldc, int mbs_entry, int force_shape, void* stream);

// Which kernel the dispatcher of mx_gemm / mx_gemm_mbs / mx_gemm_mbs_grouped picks for a problem whose arrays meet the
// fast form's alignment (host only, nothing is launched): a NUL-terminated description into out[cap].
int mx_internal_gemm_plan(int64_t M, int64_t N, int64_t K, int a_has_mbs, int b_has_mbs, int grouped, char* out, int cap);

// mx_gemm_mbs_elem with the kernel chosen by the caller.  force: 0 = as mx_gemm_mbs_elem, 1 = the main kernel's
// general form also where the fast form applies, 2 = the main kernel also where the few-row kernel applies, 3 = the
// few-row kernel (MX_EINVAL where it does not apply).
int mx_internal_gemm_elem(mx_elem_t a_elem, const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs_or_null,
                          mx_elem_t b_elem, const uint8_t* b_codes, const uint8_t* b_scales, const uint8_t* b_mbs_or_null,
                          int64_t M, int64_t N, int64_t K, mx_dtype_t c_dtype, void* C, int64_t ldc, int force,
                          void* stream);

#ifdef __cplusplus
}
#endif
