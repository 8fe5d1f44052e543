// Dequantizer: x_hat = value(code) * 2^(E-127) / F  (Sec. 4.3.1).  One lane expands one dword of
// eight E2M1 codes; the fp32 result is correctly rounded (value * 2^(E-127) is exact, the division
// by F is IEEE), the bf16 result is that fp32 value rounded to nearest even.
#include "mx_common.h"

namespace mx {
namespace {

constexpr int kThreads = 256;

// fp32 pattern of an E2M1 magnitude index: {0, .5, 1, 1.5, 2, 3, 4, 6}.
__device__ __forceinline__ float e2m1_value(uint32_t code) {
    const uint32_t m = code & 7u;
    uint32_t bits = m >= 2u ? (m + 252u) << 22 : (m ? 0x3F000000u : 0u);
    return __uint_as_float(bits | ((code & 8u) << 28));
}

template <bool kBf16>
__global__ __launch_bounds__(kThreads) void dequantize_kernel(const uint8_t* codes, const uint8_t* scales,
                                                              const uint8_t* mbs, int64_t rows, int64_t K,
                                                              void* out, int64_t ldo) {
    const int64_t per_row = K >> 3;  // dwords of codes per row
    const int64_t total = rows * per_row;
    const int64_t nmac = (K + kMacro - 1) / kMacro;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * kThreads) {
        const int64_t r = i / per_row, d = i - r * per_row;  // element column = 8 d
        const uint32_t c = *reinterpret_cast<const uint32_t*>(codes + r * (K >> 1) + d * 4);
        const uint32_t E = scales[r * (K >> 5) + (d >> 2)];
        const float F = mbs ? 1.0f + (float)mbs[r * nmac + (d >> 4)] * (1.0f / 256.0f) : 1.0f;
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            // divide in the middle of the exponent range, then apply the rest of the power of two
            const int e = (int)E - 127, ec = min(max(e, -100), 100);
            float y = ldexpf(e2m1_value((c >> (4 * j)) & 15u), ec);
            if (mbs) y = y / F;
            y = ldexpf(y, e - ec);
            v[j] = E == 255u ? __uint_as_float(0x7FC00000u) : y;
        }
        if constexpr (kBf16) {
            uint32_t w[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = f32_to_bf16_bits(v[2 * j]) | (f32_to_bf16_bits(v[2 * j + 1]) << 16);
            uint16_t* o = static_cast<uint16_t*>(out) + r * ldo + d * 8;
            if ((reinterpret_cast<uintptr_t>(o) & 15) == 0) {
                *reinterpret_cast<uint4*>(o) = make_uint4(w[0], w[1], w[2], w[3]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) { o[2 * j] = (uint16_t)w[j]; o[2 * j + 1] = (uint16_t)(w[j] >> 16); }
            }
        } else {
            float* o = static_cast<float*>(out) + r * ldo + d * 8;
            if ((reinterpret_cast<uintptr_t>(o) & 15) == 0) {
                reinterpret_cast<float4*>(o)[0] = make_float4(v[0], v[1], v[2], v[3]);
                reinterpret_cast<float4*>(o)[1] = make_float4(v[4], v[5], v[6], v[7]);
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) o[j] = v[j];
            }
        }
    }
}

}  // namespace
}  // namespace mx

extern "C" int mx_dequantize(const uint8_t* codes, const uint8_t* scales, const uint8_t* mbs_or_null,
                             int64_t rows, int64_t K, mx_dtype_t out_dtype, void* out, int64_t ldo,
                             void* stream) {
    using namespace mx;
    if (rows < 0 || K < 0 || (K % kBlock) != 0 || ldo < K) return MX_EINVAL;
    if (out_dtype != MX_OUT_F32 && out_dtype != MX_OUT_BF16) return MX_EINVAL;
    if (rows == 0 || K == 0) return MX_OK;
    if (!codes || !scales || !out) return MX_ENULL;
    if (!aligned(codes, 16) || !aligned(out, out_dtype == MX_OUT_F32 ? 4 : 2)) return MX_EALIGN;
    if (int st = check_device()) return st;
    const int64_t total = rows * (K >> 3);
    int64_t blocks = (total + kThreads - 1) / kThreads;
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (out_dtype == MX_OUT_BF16)
        hipLaunchKernelGGL(dequantize_kernel<true>, dim3((unsigned)blocks), dim3(kThreads), 0, s, codes, scales,
                           mbs_or_null, rows, K, out, ldo);
    else
        hipLaunchKernelGGL(dequantize_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), 0, s, codes, scales,
                           mbs_or_null, rows, K, out, ldo);
    return launch_status();
}
