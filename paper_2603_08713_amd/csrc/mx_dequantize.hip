// Dequantizer: x_hat = value(code) * 2^(E-127) / F  (Sec. 4.3.1).  The fp32 result is correctly rounded (value
// * 2^(E-127) is exact, the division by F is IEEE), the bf16 result is that fp32 value rounded to nearest even.
//
// A lane expands two runs of 8 codes, a wavefront 1024 consecutive elements of a row.
// An E2M1 magnitude is 2^k or 1.5 * 2^k, and scaling by a power of two commutes with rounding, so a run needs
// only two divisions, 1/F and 1.5/F (F is shared by its 8 elements), and every element is one of the two
// quotients with k + E - 127 added to its exponent field.  That holds while the result stays a normal number:
// lanes whose scale byte is outside [8, 247] (and NaN blocks) take the element-by-element route.
#include "mx_common.h"

namespace mx {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kLaneElems = 16, kChunk = kWave * kLaneElems;

// fp32 pattern of an E2M1 magnitude index: {0, .5, 1, 1.5, 2, 3, 4, 6}.
__device__ __forceinline__ float e2m1_value(uint32_t code) {
    const uint32_t m = code & 7u;
    uint32_t bits = m >= 2u ? (m + 252u) << 22 : (m ? 0x3F000000u : 0u);
    return __uint_as_float(bits | ((code & 8u) << 28));
}

// One element through fp64, valid for every scale byte: the product is exact, the quotient is rounded at 53 bits
// and once more to fp32 (to a subnormal where the result is one), which never differs from a single rounding here
// (the exact quotient of a 2-bit by a 9-bit integer has no run of 28 equal bits after its leading 25).
__device__ __forceinline__ float dequantize_element(uint32_t code, uint32_t E, float F, bool divide) {
    double y = (double)e2m1_value(code) * __longlong_as_double((long long)(E + 896u) << 52);  // 2^(E-127)
    if (divide) y = y / (double)F;
    return E == 255u ? __uint_as_float(0x7FC00000u) : (float)y;
}

struct DequantArgs {
    const uint8_t *codes, *scales, *mbs;
    void* out;
    int64_t K, ldo, nmac;
    uint32_t chunks_per_row, total_chunks;
    int vec_out;  // every output row starts 16-byte aligned
};

template <bool kBf16>
__global__ __launch_bounds__(kThreads) void dequantize_kernel(DequantArgs q) {
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6));
    const uint32_t nwaves = gridDim.x * (kThreads / kWave);
    for (uint32_t c = wave; c < q.total_chunks; c += nwaves) {
        const uint32_t row = c / q.chunks_per_row, col0 = (c - row * q.chunks_per_row) * kChunk + lane * 8;
        // two runs of 8 elements, 512 apart: every load and store instruction of the wavefront covers one
        // contiguous piece of the row
        uint32_t cw[2], E[2], m8[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t col = col0 + u * 512;
            cw[u] = 0; E[u] = 127; m8[u] = 0;
            if (col < q.K) {
                cw[u] = *reinterpret_cast<const uint32_t*>(q.codes + (int64_t)row * (q.K >> 1) + (col >> 1));
                E[u] = q.scales[(int64_t)row * (q.K >> 5) + (col >> 5)];
                if (q.mbs) m8[u] = q.mbs[(int64_t)row * q.nmac + (col >> 7)];
            }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t col = col0 + u * 512;
            if (col >= q.K) continue;  // no cross-lane operations below
            const float F = __uint_as_float(0x3F800000u | (m8[u] << 15));  // 1 + m8/256
            float v[8];
            if (E[u] >= 8u && E[u] <= 247u) {
                const uint32_t r1 = __float_as_uint(1.0f / F), r3 = __float_as_uint(1.5f / F);  // m8 = 0: exactly 1 and 1.5
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t code = (cw[u] >> (4 * j)) & 15u, m = code & 7u;
                    // magnitudes: 1 -> 0.5, 2 -> 1, 3 -> 1.5, 4 -> 2, 5 -> 3, 6 -> 4, 7 -> 6
                    const uint32_t quo = (m & 1u) && m > 1u ? r3 : r1;
                    const uint32_t bits = quo + (((m >> 1) + E[u] - 128u) << 23);
                    v[j] = __uint_as_float((m ? bits : 0u) | ((code & 8u) << 28));
                }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = dequantize_element((cw[u] >> (4 * j)) & 15u, E[u], F, q.mbs != nullptr);
            }
            if constexpr (kBf16) {
                uint32_t w[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) w[j] = pack_bf16(v[2 * j], v[2 * j + 1]);
                uint16_t* o = static_cast<uint16_t*>(q.out) + (int64_t)row * q.ldo + col;
                if (q.vec_out) {
                    __builtin_nontemporal_store(u32x4{w[0], w[1], w[2], w[3]}, reinterpret_cast<u32x4*>(o));
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) { o[2 * j] = (uint16_t)w[j]; o[2 * j + 1] = (uint16_t)(w[j] >> 16); }
                }
            } else {
                float* o = static_cast<float*>(q.out) + (int64_t)row * q.ldo + col;
                if (q.vec_out) {
                    __builtin_nontemporal_store(f32x4{v[0], v[1], v[2], v[3]}, reinterpret_cast<f32x4*>(o));
                    __builtin_nontemporal_store(f32x4{v[4], v[5], v[6], v[7]}, reinterpret_cast<f32x4*>(o) + 1);
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j) o[j] = v[j];
                }
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
    DequantArgs q;
    q.codes = codes;
    q.scales = scales;
    q.mbs = mbs_or_null;
    q.out = out;
    q.K = K;
    q.ldo = ldo;
    q.nmac = (K + kMacro - 1) / kMacro;
    const int64_t cpr = (K + kChunk - 1) / kChunk;
    if (cpr * rows >= ((int64_t)1 << 32)) return MX_EINVAL;  // chunk ids are 32-bit
    q.chunks_per_row = (uint32_t)cpr;
    q.total_chunks = (uint32_t)(cpr * rows);
    const int64_t esz = out_dtype == MX_OUT_F32 ? 4 : 2;
    q.vec_out = aligned(out, 16) && (ldo * esz) % 16 == 0;
    int64_t blocks = ((int64_t)q.total_chunks + (kThreads / kWave) - 1) / (kThreads / kWave);
    if (blocks > (int64_t)1 << 22) blocks = (int64_t)1 << 22;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (out_dtype == MX_OUT_BF16)
        hipLaunchKernelGGL(dequantize_kernel<true>, dim3((unsigned)blocks), dim3(kThreads), 0, s, q);
    else
        hipLaunchKernelGGL(dequantize_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), 0, s, q);
    return launch_status();
}
