// Dequantizer for the 8-bit and 6-bit MX element formats: x_hat = value(code) * 2^(E-127) / F  (Sec. 4.3.1, with
// the element formats of the OCP MX specification; 6-bit codes packed, 8 codes in 6 bytes).  The fp32 result is defined through fp64: value * 2^(E-127) is
// exact, the quotient is rounded at 53 bits and once more to fp32; the bf16 result is that fp32 value rounded to
// nearest even.  A block whose scale byte is 255 (non-finite input) gives NaN.  Where every intermediate is a
// normal fp32 number (scale byte in [64, 230]) fp32 arithmetic gives the same bits without a division per element:
// with r = 1 / F (one IEEE division per run of 8), q = t * r is corrected once by the exact remainder,
// q' = fma(fma(-q, F, t), r, q), which is the correctly rounded quotient for every pair of code value and MBS
// word - checked with exact rationals on the host (tests/test_abi_cpu.py); a power-of-two scale commutes with
// rounding.  Other scale bytes take the fp64 route element by element.
//
// A lane expands two runs of 8 codes, 512 apart; a wavefront 1024 consecutive elements of a row, so that every
// load and store instruction of the wavefront covers one contiguous piece of the row.  (8 codes of a 6-bit format
// are 6 bytes, 2-byte aligned: three 16-bit loads.)
#include "mx_common.h"

namespace mx {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kDq8Threads = 256;
constexpr int kDq8Chunk = kWave * 16;

// Value of a code as fp32 (exact).  E4M3: S.EEEE.MMM, bias 7; E5M2: S.EEEEE.MM, bias 15; E2M3: S.EE.MMM, bias 1;
// E3M2: S.EEE.MM, bias 3; subnormals m * 2^(1 - bias - mbits).  The 8-bit codes past the largest finite one are
// not produced by the quantizer; every 6-bit code is a number.
template <int kElem>
struct ElemBits {
    static constexpr int kBits = kElem == MX_ELEM_E4M3 || kElem == MX_ELEM_E5M2 ? 8 : 6;
    static constexpr int kMbits = kElem == MX_ELEM_E4M3 || kElem == MX_ELEM_E2M3 ? 3 : 2;
    static constexpr int kBias = kElem == MX_ELEM_E4M3 ? 7 : kElem == MX_ELEM_E5M2 ? 15 : kElem == MX_ELEM_E2M3 ? 1 : 3;
};
template <int kElem>
__device__ __forceinline__ float fp8_magnitude(uint32_t code) {
    using T = ElemBits<kElem>;
    const uint32_t mag = code & ((1u << (T::kBits - 1)) - 1u);
    const uint32_t e = mag >> T::kMbits, m = mag & ((1u << T::kMbits) - 1u);
    const uint32_t normal = ((e + 127u - T::kBias) << 23) | (m << (23 - T::kMbits));
    const float sub = (float)m * __uint_as_float((uint32_t)(127 + 1 - T::kBias - T::kMbits) << 23);
    return e ? __uint_as_float(normal) : sub;
}
template <int kElem>
__device__ __forceinline__ uint32_t fp8_sign(uint32_t code) {  // the sign as bit 31
    return ((code >> (ElemBits<kElem>::kBits - 1)) & 1u) << 31;
}
template <int kElem>
__device__ __forceinline__ float fp8_value(uint32_t code) {
    return __uint_as_float(__float_as_uint(fp8_magnitude<kElem>(code)) | fp8_sign<kElem>(code));
}

// code j of a lane's run of 8: a byte of the 64 bits, or 6 bits of the 48
template <int kElem>
__device__ __forceinline__ uint32_t run_code(uint2 w, int j) {
    if constexpr (kElem == MX_ELEM_E4M3 || kElem == MX_ELEM_E5M2) {
        return ((j < 4 ? w.x : w.y) >> (8 * (j & 3))) & 0xFFu;
    } else {
        const uint64_t all = ((uint64_t)w.y << 32) | w.x;
        return (uint32_t)(all >> (6 * j)) & 0x3Fu;
    }
}

struct Dequant8Args {
    const uint8_t *codes, *scales, *mbs;
    void* out;
    int64_t K, ldo, nmac;
    uint32_t chunks_per_row, total_chunks;
    int vec_out;  // every output row starts 16-byte aligned
};

template <int kElem, bool kBf16>
__global__ __launch_bounds__(kDq8Threads) void dequantize8_kernel(Dequant8Args q) {
    constexpr bool kSix = kElem == MX_ELEM_E2M3 || kElem == MX_ELEM_E3M2;
    const int64_t row_bytes = kSix ? q.K / 4 * 3 : q.K;
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(blockIdx.x * (kDq8Threads / kWave) + (threadIdx.x >> 6));
    const uint32_t nwaves = gridDim.x * (kDq8Threads / kWave);
    for (uint32_t c = wave; c < q.total_chunks; c += nwaves) {
        const uint32_t row = c / q.chunks_per_row, col0 = (c - row * q.chunks_per_row) * kDq8Chunk + lane * 8;
        uint2 cw[2];
        uint32_t E[2], m8[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t col = col0 + u * 512;
            cw[u] = make_uint2(0, 0); E[u] = 127; m8[u] = 0;
            if (col < q.K) {
                if constexpr (kSix) {
                    const uint16_t* p = reinterpret_cast<const uint16_t*>(q.codes + (int64_t)row * row_bytes + (col >> 3) * 6);
                    cw[u] = make_uint2((uint32_t)p[0] | ((uint32_t)p[1] << 16), p[2]);
                } else {
                    cw[u] = *reinterpret_cast<const uint2*>(q.codes + (int64_t)row * row_bytes + col);
                }
                E[u] = q.scales[(int64_t)row * (q.K >> 5) + (col >> 5)];
                if (q.mbs) m8[u] = q.mbs[(int64_t)row * q.nmac + (col >> 7)];
            }
        }
        // 6-bit codes: the hardware expands 32 at a time (v_cvt_scalef32_pk32_f32_fp6 / _bf6; measured: result
        // register e is the code in bits 6 e .. 6 e + 5, every code exact, the sign of a zero kept, the scale operand
        // multiplies); the lane's two runs are 16 of them.  The instruction is issued with an early-clobber result:
        // it writes its 32 result registers while its six source registers are still being read.
        float six[16];
        if constexpr (kSix) {
            typedef float v32f __attribute__((ext_vector_type(32)));
            typedef uint32_t v6u __attribute__((ext_vector_type(6)));
            const v6u packed = {cw[0].x, cw[0].y | (cw[1].x << 16), (cw[1].x >> 16) | (cw[1].y << 16), 0u, 0u, 0u};
            v32f all;
            if constexpr (kElem == MX_ELEM_E2M3) asm("v_cvt_scalef32_pk32_f32_fp6 %0, %1, 1.0" : "=&v"(all) : "v"(packed));
            else asm("v_cvt_scalef32_pk32_f32_bf6 %0, %1, 1.0" : "=&v"(all) : "v"(packed));
#pragma unroll
            for (int j = 0; j < 16; ++j) six[j] = all[j];
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t col = col0 + u * 512;
            if (col >= q.K) continue;
            float v[8];
            if (E[u] >= 64u && E[u] <= 230u) {
#pragma clang fp contract(off)
                const float F = __uint_as_float(0x3F800000u | (m8[u] << 15));  // 1 + m8/256
                const float scale = __uint_as_float(E[u] << 23);               // 2^(E-127)
                const float r = 1.0f / F;                                      // IEEE division (m8 = 0: exactly 1)
                if constexpr (kSix) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float t = six[8 * u + j] * scale;                // exact
                        const float q0 = t * r;
                        const float rem = __builtin_fmaf(-q0, F, t);           // exact
                        v[j] = __builtin_copysignf(__builtin_fmaf(rem, r, q0), t);  // (the sign of a zero)
                    }
                } else {
                    // 8-bit codes: the hardware convert expands two at a time and applies the scale (exact)
                    typedef float v2f __attribute__((ext_vector_type(2)));
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t word = i < 2 ? cw[u].x : cw[u].y;
                        v2f t;
                        if constexpr (kElem == MX_ELEM_E4M3) {
                            t = (i & 1) ? __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(word, scale, true)
                                        : __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(word, scale, false);
                        } else {
                            t = (i & 1) ? __builtin_amdgcn_cvt_scalef32_pk_f32_bf8(word, scale, true)
                                        : __builtin_amdgcn_cvt_scalef32_pk_f32_bf8(word, scale, false);
                        }
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            const float th = h ? t.y : t.x;
                            const float q0 = th * r;
                            const float rem = __builtin_fmaf(-q0, F, th);      // exact
                            v[2 * i + h] = __builtin_copysignf(__builtin_fmaf(rem, r, q0), th);  // (the sign of a zero)
                        }
                    }
                }
            } else {
                const double F = 1.0 + (double)m8[u] * (1.0 / 256.0);
                const double scale = __longlong_as_double((long long)(E[u] + 896u) << 52);  // 2^(E-127)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t code = run_code<kElem>(cw[u], j);
                    double y = (double)fp8_value<kElem>(code) * scale;
                    if (q.mbs) y = y / F;
                    v[j] = E[u] == 255u ? __uint_as_float(0x7FC00000u) : (float)y;
                }
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
                    // (ordinary stores: each of the two instructions covers only every other 16 bytes of the
                    // wavefront's piece of the row, and streamed past the caches such writes ran at half the rate)
                    *reinterpret_cast<f32x4*>(o) = f32x4{v[0], v[1], v[2], v[3]};
                    *(reinterpret_cast<f32x4*>(o) + 1) = f32x4{v[4], v[5], v[6], v[7]};
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

extern "C" int mx_dequantize_elem(mx_elem_t elem, const uint8_t* codes, const uint8_t* scales, const uint8_t* mbs_or_null,
                                  int64_t rows, int64_t K, mx_dtype_t out_dtype, void* out, int64_t ldo, void* stream) {
    using namespace mx;
    if ((int)elem <= MX_ELEM_E2M1 || (int)elem > MX_ELEM_E3M2) return MX_EINVAL;
    if (rows < 0 || K < 0 || (K % kBlock) != 0 || ldo < K) return MX_EINVAL;
    if (out_dtype != MX_OUT_F32 && out_dtype != MX_OUT_BF16) return MX_EINVAL;
    if (rows == 0 || K == 0) return MX_OK;
    if (!codes || !scales || !out) return MX_ENULL;
    if (!aligned(codes, 8) || !aligned(out, out_dtype == MX_OUT_F32 ? 4 : 2)) return MX_EALIGN;
    if (int st = check_device()) return st;
    Dequant8Args q;
    q.codes = codes; q.scales = scales; q.mbs = mbs_or_null;
    q.out = out;
    q.K = K; q.ldo = ldo; q.nmac = (K + kMacro - 1) / kMacro;
    const int64_t cpr = (K + kDq8Chunk - 1) / kDq8Chunk;
    if (cpr * rows >= ((int64_t)1 << 32)) return MX_EINVAL;  // chunk ids are 32-bit
    q.chunks_per_row = (uint32_t)cpr;
    q.total_chunks = (uint32_t)(cpr * rows);
    const int64_t esz = out_dtype == MX_OUT_F32 ? 4 : 2;
    q.vec_out = aligned(out, 16) && (ldo * esz) % 16 == 0;
    int64_t blocks = ((int64_t)q.total_chunks + (kDq8Threads / kWave) - 1) / (kDq8Threads / kWave);
    if (blocks > (int64_t)1 << 22) blocks = (int64_t)1 << 22;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)blocks), block(kDq8Threads);
    const bool bf = out_dtype == MX_OUT_BF16;
    switch (elem) {
    case MX_ELEM_E4M3:
        if (bf) hipLaunchKernelGGL((dequantize8_kernel<MX_ELEM_E4M3, true>), grid, block, 0, s, q);
        else hipLaunchKernelGGL((dequantize8_kernel<MX_ELEM_E4M3, false>), grid, block, 0, s, q);
        break;
    case MX_ELEM_E5M2:
        if (bf) hipLaunchKernelGGL((dequantize8_kernel<MX_ELEM_E5M2, true>), grid, block, 0, s, q);
        else hipLaunchKernelGGL((dequantize8_kernel<MX_ELEM_E5M2, false>), grid, block, 0, s, q);
        break;
    case MX_ELEM_E2M3:
        if (bf) hipLaunchKernelGGL((dequantize8_kernel<MX_ELEM_E2M3, true>), grid, block, 0, s, q);
        else hipLaunchKernelGGL((dequantize8_kernel<MX_ELEM_E2M3, false>), grid, block, 0, s, q);
        break;
    default:
        if (bf) hipLaunchKernelGGL((dequantize8_kernel<MX_ELEM_E3M2, true>), grid, block, 0, s, q);
        else hipLaunchKernelGGL((dequantize8_kernel<MX_ELEM_E3M2, false>), grid, block, 0, s, q);
        break;
    }
    return launch_status();
}
