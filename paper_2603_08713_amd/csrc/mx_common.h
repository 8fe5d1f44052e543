// Shared host/device helpers of the gfx950 MXFP4 library (private; the public ABI is include/mx4.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mx4.h"
#include "mx_constants.h"

namespace mx {

// Returns MX_OK when the current device is gfx950; MX_EUNSUPPORTED otherwise (cached per process).
int check_device();

inline int launch_status() { return hipGetLastError() == hipSuccess ? MX_OK : MX_ELAUNCH; }

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// ---- DPP lane exchanges (all 64 lanes must be active) --------------------------------------------
// quad_perm:[1,0,3,2] / [2,3,0,1] swap neighbours inside each group of four lanes; row_ror:N rotates
// inside each row of 16 lanes.
__device__ __forceinline__ uint32_t dpp_quad_xor1(uint32_t v) {
    return __builtin_amdgcn_update_dpp(0u, v, 0xB1, 0xF, 0xF, true);
}
__device__ __forceinline__ uint32_t dpp_quad_xor2(uint32_t v) {
    return __builtin_amdgcn_update_dpp(0u, v, 0x4E, 0xF, 0xF, true);
}
__device__ __forceinline__ uint32_t dpp_row_ror4(uint32_t v) {
    return __builtin_amdgcn_update_dpp(0u, v, 0x124, 0xF, 0xF, true);
}
__device__ __forceinline__ uint32_t dpp_row_ror8(uint32_t v) {
    return __builtin_amdgcn_update_dpp(0u, v, 0x128, 0xF, 0xF, true);
}

// fp32 -> bf16 bits, round to nearest even; NaN stays NaN.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Two fp32 -> packed bf16 (first value in the low half) with the hardware convert, round to nearest even.
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    typedef float v2f __attribute__((ext_vector_type(2)));
    typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
    const v2f v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, v2bf));
}

}  // namespace mx
