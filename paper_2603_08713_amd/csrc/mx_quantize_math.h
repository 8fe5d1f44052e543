// Device arithmetic shared by the kernels that quantize bf16 to MXFP4 (private; the public ABI is
// include/mx4.h).  Every decision here is exact; see mx_quantize.hip for how the pieces are used.
#pragma once

#include "mx_common.h"

namespace mx {
namespace {

typedef unsigned short us2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
    us2 r = __builtin_elementwise_max(__builtin_bit_cast(us2, a), __builtin_bit_cast(us2, b));
    return __builtin_bit_cast(uint32_t, r);
}

// 8 leading mantissa bits of 6/alpha for alpha = (128 + k) * 2^e (Sec. 4.3.1, Eq. 3):  6*128/(128+k) lies
// in (3, 6]; normalised to [1,2) it is 192/(128+k) for k <= 64 and 384/(128+k) above.
__device__ __forceinline__ uint32_t mbs_word_of_mantissa(uint32_t k) {
    const uint32_t n = 128u + k;
    return (k <= 64u ? 49152u / n : 98304u / n) - 256u;
}
// The same quotient through the hardware reciprocal plus 2^-10: N / (128 + k) is either an integer
// (k = 0, 64) or at least 1/255 away from one, far more than the reciprocal's error.
__device__ __forceinline__ uint32_t mbs_word_of_mantissa_fast(uint32_t k) {
    const float num = k <= 64u ? 49152.0f : 98304.0f;
    const float quo = fmaf(num, __builtin_amdgcn_rcpf((float)(128u + k)), 0x1.0p-10f);
    return (uint32_t)quo - 256u;
}
// Static word of a macro block from the bf16 magnitude bits of its absmax (0 for an all-zero block); a
// subnormal absmax is normalised first.
__device__ __forceinline__ uint32_t mbs_word_of_absmax(uint32_t mmax) {
    if (mmax == 0) return 0;
    uint32_t k = mmax & 0x7Fu;
    if ((mmax >> 7) == 0) k = (k << (__clz(k) - 24)) & 0x7Fu;
    return mbs_word_of_mantissa(k);
}

// Added to the fp32 pattern of the scaled absmax, this bumps the exponent field exactly when the mantissa
// exceeds the rule's threshold (Sec. 4.2: FLOOR 1.5, OAS 1.75, OCP never).
inline uint32_t rule_carry(int rule) {
    return rule == MX_RULE_FLOOR ? 0x3FFFFFu : rule == MX_RULE_OAS ? 0x1FFFFFu : 0u;
}

// ---- all-integer arithmetic, exact for every finite bf16 input including subnormals and huge values ----
// E8M0 byte of a block whose absmax has the bf16 magnitude bits amax (non-zero), scaled by F = u / 256.
__device__ __forceinline__ int exact_scale_byte(uint32_t amax, uint32_t u, int rule) {
    const uint32_t ea = amax >> 7;
    const uint32_t na = ea ? (128u | (amax & 0x7Fu)) : (amax & 0x7Fu);
    const int ex = (int)(ea ? ea : 1u) - 134;            // absmax = na * 2^ex
    const uint32_t P = na * u;                           // absmax * F = P * 2^(ex-8)
    const int msb = 31 - __clz(P);
    const int p = ex - 8 + msb;                          // floor(log2(absmax * F))
    bool low = true;                                     // mantissa at or below the threshold
    if (rule == MX_RULE_FLOOR) low = 2u * P <= (3u << msb);
    else if (rule == MX_RULE_OAS) low = 4u * P <= (7u << msb);
    const int s = low ? 2 - p : 1 - p;
    return min(max(127 - s, 0), 254);
}
// E2M1 code of the bf16 pattern h scaled by F = u / 256 and by 2^s: nearest, ties to the even code,
// saturating; the sign bit is copied.
__device__ __forceinline__ uint32_t exact_code(uint32_t h, uint32_t u, int s) {
    const uint32_t a = h & 0x7FFFu, e = a >> 7;
    const uint32_t n = e ? (128u | (a & 0x7Fu)) : (a & 0x7Fu);
    const int sh = (int)(e ? e : 1u) - 134 - 8 + s + 2;  // |x| F 2^s = n u 2^sh quarter units
    uint32_t T = n * u;
    int r = 0;
    if (sh >= 0) T <<= min(sh, 8); else r = min(-sh, 18);
    // thresholds 1/4, 3/4, 5/4, 7/4, 5/2, 7/2, 5 in quarter units; ties go to the even code
    const uint32_t c = (T > (1u << r)) + (T >= (3u << r)) + (T > (5u << r)) + (T >= (7u << r)) +
                       (T > (10u << r)) + (T >= (14u << r)) + (T > (20u << r));
    return c | ((h >> 12) & 8u);
}

}  // namespace
}  // namespace mx
