// Dequantizer: x_hat = value(code) * 2^(E-127) / F  (Sec. 4.3.1).  The fp32 result is correctly rounded (value
// * 2^(E-127) is exact, the division by F is IEEE), the bf16 result is that fp32 value rounded to nearest even.
//
// A lane expands four runs of 8 codes, 512 elements apart; a wavefront 2048 consecutive elements of a row, so that
// every code load and every store of the wavefront covers one contiguous piece of the row.  The 64 E8M0 bytes
// and 16 MBS words of those elements are fetched once, one byte per lane, and handed to the lanes that need
// them through the LDS crossbar (ds_bpermute): a load instruction occupies the texture-address unit for its 64
// lanes however few bytes each lane asks for, and fetching a byte of each kind per lane and run made that unit,
// not the memory, the limit.
// The hardware convert expands two codes at a time and applies the block scale (exact).  The division by F costs
// one IEEE division per run of 8 (F is shared by them): with r = RN(1 / F), q = RN(t r) is corrected once by the
// exact remainder, q' = RN(q + (t - q F) r), which is the correctly rounded quotient for every E2M1 magnitude
// (mantissa 1 or 1.5) and every MBS word - checked with exact rationals on the host (tests/test_abi_cpu.py); a
// power-of-two scale commutes with all of it.  That holds while every intermediate is a normal number: lanes whose
// scale byte is outside [64, 230] (and NaN blocks) take the element-by-element route.
#include "mx_common.h"

namespace mx {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kRuns = 4, kLaneElems = 8 * kRuns, kChunk = kWave * kLaneElems;

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
        // lane l fetches E8M0 byte l and (l < 16) MBS word l of the chunk; run u of lane l wants byte 16 u + l / 4
        // and word 4 u + l / 16
        const uint32_t chunk0 = col0 - lane * 8;
        uint32_t my_e = 127, my_m8 = 0;
        if (chunk0 + lane * 32 < q.K) my_e = q.scales[(int64_t)row * (q.K >> 5) + (chunk0 >> 5) + lane];
        if (q.mbs && lane < 16 && chunk0 + lane * 128 < q.K) my_m8 = q.mbs[(int64_t)row * q.nmac + (chunk0 >> 7) + lane];
        uint32_t cw[kRuns], E[kRuns], m8[kRuns];
#pragma unroll
        for (int u = 0; u < kRuns; ++u) {
            const uint32_t col = col0 + u * 512;
            cw[u] = 0;
            if (col < q.K) cw[u] = *reinterpret_cast<const uint32_t*>(q.codes + (int64_t)row * (q.K >> 1) + (col >> 1));
            E[u] = (uint32_t)__builtin_amdgcn_ds_bpermute((int)((16 * u + (lane >> 2)) * 4), (int)my_e);
            m8[u] = (uint32_t)__builtin_amdgcn_ds_bpermute((int)((4 * u + (lane >> 4)) * 4), (int)my_m8);
        }
#pragma unroll
        for (int u = 0; u < kRuns; ++u) {
            const uint32_t col = col0 + u * 512;
            if (col >= q.K) continue;  // no cross-lane operations below
            const float F = __uint_as_float(0x3F800000u | (m8[u] << 15));  // 1 + m8/256
            float v[8];
            if (E[u] >= 64u && E[u] <= 230u) {
#pragma clang fp contract(off)
                typedef float v2f __attribute__((ext_vector_type(2)));
                const float r = 1.0f / F;                         // IEEE division, once per run (m8 = 0: exactly 1)
                const float scale = __uint_as_float(E[u] << 23);  // 2^(E-127)
                auto quotient = [&](float t) __attribute__((always_inline)) {  // t / F, correctly rounded (see the header)
                    const float q0 = t * r;
                    const float rem = __builtin_fmaf(-q0, F, t);  // exact
                    return __builtin_copysignf(__builtin_fmaf(rem, r, q0), t);  // (the sign of a zero)
                };
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    v2f t;  // codes 2 i and 2 i + 1 (byte i of the dword) times the scale: exact
                    if (i == 0) t = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(cw[u], scale, 0);
                    if (i == 1) t = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(cw[u], scale, 1);
                    if (i == 2) t = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(cw[u], scale, 2);
                    if (i == 3) t = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(cw[u], scale, 3);
                    v[2 * i] = quotient(t.x);
                    v[2 * i + 1] = quotient(t.y);
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
                    // (ordinary stores: a lane's 32 bytes take two instructions, each of which covers only every
                    // other 16 bytes of the wavefront's piece of the row; streamed past the caches such half-line
                    // writes ran at less than half the rate)
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
