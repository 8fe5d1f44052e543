// Quantizer for the 8-bit and 6-bit MX element formats (E4M3, E5M2; E2M3, E3M2) with Overflow-Aware Scaling and
// static Macro Block Scaling for gfx950 (Sec. 1, footnote: the methods carry over to MXFP6 / MXFP8).
//
// The rules of Sec. 4.2 and 4.3.1 are restated with the element format's constants in place of E2M1's 6 and 1:
// V = vm * 2^emax, the largest finite magnitude (vm = 1.75, for E2M3 1.875), and h = 2^(emax - mbits - 1), half the
// spacing of the top binade.  In terms of the mantissa t of the (MBS-scaled) block absmax, written t * 2^p:
//   OCP    stored exponent p - emax                        FLOOR  one more when t > vm
//   OAS    one more when t > vm + h / 2^emax               MBS-S  m8 = 8 leading mantissa bits of V / absmax128
// Work decomposition and exactness arguments are those of the MXFP4 quantizer (mx_quantize.hip): a lane owns 8
// consecutive bf16, 4 lanes a block, 16 lanes a macro block, a wavefront 512 elements of a row; x * F is exact
// in fp32 and so is its product with the power-of-two block scale; the block exponent is read off the fp32
// pattern of absmax * F with a carry; blocks that could leave fp32's normal range, or hold Inf/NaN, take a
// wave-uniform detour through all-integer arithmetic.
// Output: 8-bit codes one per byte; 6-bit codes packed, element k of a row in bits 6 k .. 6 k + 5 of the row's
// bytes (a block is 24 bytes, which three of its four lanes store, 8 bytes each, after a DPP exchange).
#include "mx_internal.h"
#include "mx_quantize_math.h"

namespace mx {
namespace {

constexpr int kChunk8 = 512;   // elements per wavefront step
constexpr int kUnroll8 = 4;    // chunks in flight per wavefront
constexpr int kThreads8 = 256;

template <int kElem>
struct Fp8;
// kFloorNum / 2^kFloorShift = vm, kOasNum / 2^kOasShift = vm + h / 2^emax; kCarry* = 2^23 - 1 - their mantissa bits;
// MBS word: floor(kMbsNum / (128 + k)) - 256 for k <= kMbsSplit, twice the numerator above (256 vm 128 = kMbsNum).
template <>
struct Fp8<MX_ELEM_E4M3> {
    static constexpr int kBits = 8, kEmax = 8, kMbits = 3, kBias = 7, kMaxCode = 0x7E;
    static constexpr uint32_t kMaxBits = 0x43E00000u;  // 448.0f
    static constexpr uint32_t kCarryFloor = 0x1FFFFFu, kCarryOas = 0x17FFFFu;
    static constexpr uint32_t kFloorNum = 7, kFloorShift = 2, kOasNum = 29, kOasShift = 4;  // 1.75, 1.8125
    static constexpr uint32_t kMbsNum = 57344, kMbsSplit = 96;
};
template <>
struct Fp8<MX_ELEM_E5M2> {
    static constexpr int kBits = 8, kEmax = 15, kMbits = 2, kBias = 15, kMaxCode = 0x7B;
    static constexpr uint32_t kMaxBits = 0x47600000u;  // 57344.0f
    static constexpr uint32_t kCarryFloor = 0x1FFFFFu, kCarryOas = 0x0FFFFFu;
    static constexpr uint32_t kFloorNum = 7, kFloorShift = 2, kOasNum = 15, kOasShift = 3;  // 1.75, 1.875
    static constexpr uint32_t kMbsNum = 57344, kMbsSplit = 96;
};
template <>
struct Fp8<MX_ELEM_E2M3> {
    static constexpr int kBits = 6, kEmax = 2, kMbits = 3, kBias = 1, kMaxCode = 0x1F;
    static constexpr uint32_t kMaxBits = 0x40F00000u;  // 7.5f
    static constexpr uint32_t kCarryFloor = 0x0FFFFFu, kCarryOas = 0x07FFFFu;
    static constexpr uint32_t kFloorNum = 15, kFloorShift = 3, kOasNum = 31, kOasShift = 4;  // 1.875, 1.9375
    static constexpr uint32_t kMbsNum = 61440, kMbsSplit = 112;
};
template <>
struct Fp8<MX_ELEM_E3M2> {
    static constexpr int kBits = 6, kEmax = 4, kMbits = 2, kBias = 3, kMaxCode = 0x1F;
    static constexpr uint32_t kMaxBits = 0x41E00000u;  // 28.0f
    static constexpr uint32_t kCarryFloor = 0x1FFFFFu, kCarryOas = 0x0FFFFFu;
    static constexpr uint32_t kFloorNum = 7, kFloorShift = 2, kOasNum = 15, kOasShift = 3;  // 1.75, 1.875
    static constexpr uint32_t kMbsNum = 57344, kMbsSplit = 96;
};

struct Quant8Args {
    const uint16_t* x;
    uint8_t *codes, *scales, *mbs;
    int64_t K, ldx, nmac;
    uint32_t chunks_per_row, total_chunks;
    uint32_t carry;
    int rule;
    int scales_dword;
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// 8 leading mantissa bits of V / alpha for alpha = (128 + k) * 2^e, V = vm * 2^emax: 128 vm / (128 + k) lies in
// (vm / 2, vm]; normalised to [1, 2) it is 128 vm / (128 + k) for 128 + k <= 128 vm and twice that above.  The
// quotient is taken with the hardware reciprocal plus 2^-10 (an integer, or at least 1/255 away from one).
template <typename T>
__device__ __forceinline__ uint32_t mbs8_word_of_mantissa(uint32_t k) {
    const float num = k <= T::kMbsSplit ? (float)T::kMbsNum : (float)(2 * T::kMbsNum);
    const float quo = fmaf(num, __builtin_amdgcn_rcpf((float)(128u + k)), 0x1.0p-10f);
    return (uint32_t)quo - 256u;
}
template <typename T>
__device__ __forceinline__ uint32_t mbs8_word_of_absmax(uint32_t mmax) {
    if (mmax == 0) return 0;
    uint32_t k = mmax & 0x7Fu;
    if ((mmax >> 7) == 0) k = (k << (__clz(k) - 24)) & 0x7Fu;
    const uint32_t n = 128u + k;
    return (k <= T::kMbsSplit ? T::kMbsNum / n : 2 * T::kMbsNum / n) - 256u;
}

// ---- all-integer arithmetic, exact for every finite bf16 input ----
template <typename T>
__device__ __forceinline__ int exact_scale_byte8(uint32_t amax, uint32_t u, int rule) {
    const uint32_t ea = amax >> 7;
    const uint32_t na = ea ? (128u | (amax & 0x7Fu)) : (amax & 0x7Fu);
    const int ex = (int)(ea ? ea : 1u) - 134;  // absmax = na * 2^ex
    const uint32_t P = na * u;                 // absmax * F = P * 2^(ex - 8)
    const int msb = 31 - __clz(P);
    const int p = ex - 8 + msb;                // floor(log2(absmax * F))
    bool low = true;                           // mantissa at or below the rule's threshold
    if (rule == MX_RULE_FLOOR) low = (P << T::kFloorShift) <= (T::kFloorNum << msb);
    else if (rule == MX_RULE_OAS) low = (P << T::kOasShift) <= (T::kOasNum << msb);
    const int s = low ? T::kEmax - p : T::kEmax - 1 - p;
    return min(max(127 - s, 0), 254);
}
// Code of the bf16 pattern h scaled by F = u / 256 and by 2^s: nearest, ties to even, saturating, sign copied.
template <typename T>
__device__ __forceinline__ uint32_t exact_code8(uint32_t h, uint32_t u, int s) {
    const uint32_t sign = (h >> 15) << (T::kBits - 1);
    const uint32_t a = h & 0x7FFFu, e = a >> 7;
    const uint32_t n = e ? (128u | (a & 0x7Fu)) : (a & 0x7Fu);
    const uint32_t Tv = n * u;  // |x| F 2^s = Tv * 2^e2
    if (Tv == 0) return sign;
    const int e2 = (int)(e ? e : 1u) - 134 - 8 + s;
    const int p = 31 - __clz(Tv) + e2;
    if (p > T::kEmax) return (uint32_t)T::kMaxCode | sign;
    const int ey = max(p, 1 - T::kBias);       // binade whose spacing applies (subnormals share the lowest)
    const int shift = e2 - (ey - T::kMbits);   // in units of that spacing the value is Tv * 2^shift
    uint32_t q;
    if (shift >= 0) {
        q = Tv << shift;                       // at most 2^(mbits + 1)
    } else {
        const int r = min(-shift, 20);
        const uint32_t q0 = Tv >> r, rem = Tv & ((1u << r) - 1u), half = 1u << (r - 1);
        q = q0 + ((rem > half || (rem == half && (q0 & 1u))) ? 1u : 0u);
    }
    const uint32_t code = ((uint32_t)(ey + T::kBias) << T::kMbits) + q - (1u << T::kMbits);
    return min(code, (uint32_t)T::kMaxCode) | sign;
}

struct Chunk8 {
    uint32_t lo, hi;  // 8 codes of this lane: 8 bytes, or 48 bits (32 in lo, 16 in hi) for the 6-bit formats
    uint32_t E, m8;
};

// code i of the lane's 8 goes to bits kBits * i of the 64-bit pair (lo, hi)
template <typename T>
__device__ __forceinline__ void put_code(uint32_t& lo, uint32_t& hi, int i, uint32_t code) {
    const int bit = T::kBits * i;
    if (bit < 32) lo |= code << bit;
    if (bit + T::kBits > 32) hi |= bit >= 32 ? code << (bit - 32) : code >> (32 - bit);
}

// (m8_given >= 0 replaces the static word: the searched word of MBS-Dynamic)
template <typename T>
__device__ __noinline__ Chunk8 quantize_chunk8_exact(u32x4 v, int rule, int use_mbs, int m8_given = -1) {
    uint32_t h[8] = {v.x & 0xFFFFu, v.x >> 16, v.y & 0xFFFFu, v.y >> 16,
                     v.z & 0xFFFFu, v.z >> 16, v.w & 0xFFFFu, v.w >> 16};
    uint32_t amax = 0, nf = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t a = h[i] & 0x7FFFu;
        if (a >= 0x7F80u) nf = 1; else amax = max(amax, a);
    }
    nf |= dpp_quad_xor1(nf);
    nf |= dpp_quad_xor2(nf);
    amax = max(amax, dpp_quad_xor1(amax));
    amax = max(amax, dpp_quad_xor2(amax));
    uint32_t mmax = amax;
    mmax = max(mmax, dpp_row_ror4(mmax));
    mmax = max(mmax, dpp_row_ror8(mmax));
    uint32_t m8 = use_mbs ? mbs8_word_of_absmax<T>(mmax) : 0u;
    if (m8_given >= 0) m8 = (uint32_t)m8_given;
    const uint32_t u = 256u + m8;
    const int E = nf ? 255 : amax == 0 ? 127 : exact_scale_byte8<T>(amax, u, rule);
    uint32_t lo = 0, hi = 0;
    if (!nf) {
#pragma unroll
        for (int i = 0; i < 8; ++i) put_code<T>(lo, hi, i, exact_code8<T>(h[i], u, 127 - E));
    }
    return {lo, hi, (uint32_t)E, m8};
}

// |t| (already scaled) to the format's grid with ordinary arithmetic: adding 1.5 * 2^(23 - mbits + ey), ey the
// binade of min(|t|, V) (not below the lowest normal one), leaves t in units of that binade's spacing in the low
// mantissa bits of the sum, rounded to nearest even.
template <typename T>
__device__ __forceinline__ uint32_t code8_alu(float t) {
    const uint32_t tb = __float_as_uint(t);
    const float y = fminf(__uint_as_float(tb & 0x7FFFFFFFu), __uint_as_float(T::kMaxBits));
    const uint32_t ey = max(__float_as_uint(y) >> 23, (uint32_t)(127 + 1 - T::kBias));
    const float w = y + __uint_as_float(((ey + 23u - T::kMbits) << 23) | 0x400000u);
    const uint32_t q = __float_as_uint(w) & ((1u << (T::kMbits + 2)) - 1u);
    return (((ey - 127u + T::kBias) << T::kMbits) + q - (1u << T::kMbits)) | ((tb >> 31) << (T::kBits - 1));
}

// The scale byte, the MBS word and the multiplier F * 2^(127 - E) of the lane's block, in fp32 arithmetic; `odd`
// (uniform over the wavefront) says that some block of the chunk lies outside the range where that arithmetic is
// exact (exponent field of its absmax outside [24, 249], or Inf/NaN) and the chunk must take the all-integer route.
struct Scale8 {
    uint32_t E, m8;
    float mult;
    bool odd;
};

template <int kElem, bool kMbs>
__device__ __forceinline__ Scale8 chunk_scale8(u32x4 v, const Quant8Args& q) {
    using T = Fp8<kElem>;
    uint32_t m = pk_max_u16(pk_max_u16(v.x & 0x7FFF7FFFu, v.y & 0x7FFF7FFFu),
                            pk_max_u16(v.z & 0x7FFF7FFFu, v.w & 0x7FFF7FFFu));
    uint32_t amax = max(m & 0xFFFFu, m >> 16);
    amax = max(amax, dpp_quad_xor1(amax));
    amax = max(amax, dpp_quad_xor2(amax));
    const bool odd = (amax >= (250u << 7)) || (amax != 0 && amax < (24u << 7));
    if (__builtin_amdgcn_ballot_w64(odd) != 0) return {0u, 0u, 0.0f, true};

    uint32_t m8 = 0;
    if constexpr (kMbs) {
        uint32_t mmax = max(amax, dpp_row_ror4(amax));
        mmax = max(mmax, dpp_row_ror8(mmax));
        m8 = mmax ? mbs8_word_of_mantissa<T>(mmax & 0x7Fu) : 0u;
    }
    const float scaled_max = __uint_as_float(amax << 16) * __uint_as_float(0x3F800000u | (m8 << 15));  // exact
    uint32_t E = ((__float_as_uint(scaled_max) + q.carry) >> 23) - (uint32_t)T::kEmax;
    E = amax ? E : 127u;
    return {E, m8, __uint_as_float(((254u - E) << 23) | (m8 << 15)), false};
}

template <int kElem, bool kHwCvt, bool kMbs>
__device__ __forceinline__ Chunk8 quantize_chunk8(u32x4 v, const Quant8Args& q) {
    using T = Fp8<kElem>;
    const Scale8 sc = chunk_scale8<kElem, kMbs>(v, q);
    if (sc.odd) return quantize_chunk8_exact<T>(v, q.rule, kMbs);
    const uint32_t E = sc.E, m8 = sc.m8;
    const float mult = sc.mult;
    const float vmax = __uint_as_float(T::kMaxBits);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t out[2] = {0, 0};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float t0 = __uint_as_float(w[i] << 16) * mult;          // exact
        const float t1 = __uint_as_float(w[i] & 0xFFFF0000u) * mult;
        if constexpr (kHwCvt && T::kBits == 8) {
            // hardware fp32 -> FP8 pair convert (nearest even); the clamp makes saturation explicit
            const float c0 = __builtin_amdgcn_fmed3f(t0, -vmax, vmax), c1 = __builtin_amdgcn_fmed3f(t1, -vmax, vmax);
            if constexpr (kElem == MX_ELEM_E4M3) {
                if (i % 2 == 0) out[i / 2] = __builtin_amdgcn_cvt_pk_fp8_f32(c0, c1, out[i / 2], false);
                else out[i / 2] = __builtin_amdgcn_cvt_pk_fp8_f32(c0, c1, out[i / 2], true);
            } else {
                if (i % 2 == 0) out[i / 2] = __builtin_amdgcn_cvt_pk_bf8_f32(c0, c1, out[i / 2], false);
                else out[i / 2] = __builtin_amdgcn_cvt_pk_bf8_f32(c0, c1, out[i / 2], true);
            }
        } else {
            put_code<T>(out[0], out[1], 2 * i, code8_alu<T>(t0));
            put_code<T>(out[0], out[1], 2 * i + 1, code8_alu<T>(t1));
        }
    }
    return {out[0], out[1], E, m8};
}

// Four chunks at once through the 32-element hardware convert (v_cvt_scalef32_2xpk16_fp6_f32 / _bf6_f32; measured
// on the device: result element 2 i is the i-th value of the first operand, element 2 i + 1 the i-th of the second,
// element e in bits 6 e .. 6 e + 5; nearest even, subnormals kept, saturating at the largest finite magnitude; the
// scale operand divides).  A dword of the input holds two consecutive elements, so the low halves of all dwords go
// to the first operand and the high halves to the second.  Returns false, with nothing done, if a chunk has to
// leave fp32 arithmetic (uniform over the wavefront).
template <int kElem, bool kMbs>
__device__ __forceinline__ bool quantize_chunks6_hw(const u32x4 (&v)[kUnroll8], const Quant8Args& q, Chunk8 (&res)[kUnroll8]) {
    typedef float v16f __attribute__((ext_vector_type(16)));
    typedef uint32_t v6u __attribute__((ext_vector_type(6)));
    Scale8 sc[kUnroll8];
    bool odd = false;
#pragma unroll
    for (int u = 0; u < kUnroll8; ++u) {
        sc[u] = chunk_scale8<kElem, kMbs>(v[u], q);
        odd |= sc[u].odd;
    }
    if (odd) return false;
    v16f even, uneven;
#pragma unroll
    for (int u = 0; u < kUnroll8; ++u) {
        const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            even[4 * u + i] = __uint_as_float(w[i] << 16) * sc[u].mult;            // exact
            uneven[4 * u + i] = __uint_as_float(w[i] & 0xFFFF0000u) * sc[u].mult;
        }
    }
    // The instruction writes its six result registers while it still reads its 32 source registers, so the result
    // must not share registers with the sources.  The compiler's builtin does not know that (its register
    // allocation put the result inside the second operand, and the elements read after the overwrite came out
    // as zero), hence the instruction itself with an early-clobber result.
    v6u r;
    if constexpr (kElem == MX_ELEM_E2M3) asm("v_cvt_scalef32_2xpk16_fp6_f32 %0, %1, %2, 1.0" : "=&v"(r) : "v"(even), "v"(uneven));
    else asm("v_cvt_scalef32_2xpk16_bf6_f32 %0, %1, %2, 1.0" : "=&v"(r) : "v"(even), "v"(uneven));
    // chunk u: bits 48 u .. 48 u + 47 of the 192
    res[0] = {r[0], r[1] & 0xFFFFu, sc[0].E, sc[0].m8};
    res[1] = {(r[1] >> 16) | (r[2] << 16), r[2] >> 16, sc[1].E, sc[1].m8};
    res[2] = {r[3], r[4] & 0xFFFFu, sc[2].E, sc[2].m8};
    res[3] = {(r[4] >> 16) | (r[5] << 16), r[5] >> 16, sc[3].E, sc[3].m8};
    return true;
}

// A chunk's results to memory: the lane's codes, its block's scale byte, its macro block's word.  Every lane of the
// wavefront takes part in the exchanges; only valid lanes (inside the row) store.
template <int kElem, bool kMbs>
__device__ __forceinline__ void store_chunk8(const Quant8Args& q, const Chunk8& res, uint32_t lane, uint32_t row, uint32_t col,
                                             bool valid) {
    // scales of the macro block gathered into one dword across the row of 16 lanes
    uint32_t ew = res.E << (8 * ((lane >> 2) & 3));
    if ((lane & 3) != 0) ew = 0;
    ew |= dpp_row_ror4(ew);
    ew |= dpp_row_ror8(ew);
    // 6-bit formats: the block's 4 x 48 bits gathered into six dwords (every lane fetches its three
    // neighbours' bits; the block's first lanes store)
    uint32_t six[6] = {0, 0, 0, 0, 0, 0};
    if constexpr (Fp8<kElem>::kBits == 6) {
        uint32_t lo[4], hi[4];
        lo[0] = __builtin_amdgcn_update_dpp(0u, res.lo, 0x00, 0xF, 0xF, true);  // quad_perm: [0,0,0,0]
        hi[0] = __builtin_amdgcn_update_dpp(0u, res.hi, 0x00, 0xF, 0xF, true);
        lo[1] = __builtin_amdgcn_update_dpp(0u, res.lo, 0x55, 0xF, 0xF, true);  // [1,1,1,1]
        hi[1] = __builtin_amdgcn_update_dpp(0u, res.hi, 0x55, 0xF, 0xF, true);
        lo[2] = __builtin_amdgcn_update_dpp(0u, res.lo, 0xAA, 0xF, 0xF, true);  // [2,2,2,2]
        hi[2] = __builtin_amdgcn_update_dpp(0u, res.hi, 0xAA, 0xF, 0xF, true);
        lo[3] = __builtin_amdgcn_update_dpp(0u, res.lo, 0xFF, 0xF, 0xF, true);  // [3,3,3,3]
        hi[3] = __builtin_amdgcn_update_dpp(0u, res.hi, 0xFF, 0xF, 0xF, true);
        six[0] = lo[0];
        six[1] = hi[0] | (lo[1] << 16);
        six[2] = (lo[1] >> 16) | (hi[1] << 16);
        six[3] = lo[2];
        six[4] = hi[2] | (lo[3] << 16);
        six[5] = (lo[3] >> 16) | (hi[3] << 16);
    }
    if (!valid) return;
    const uint32_t kblk = col >> 5;
    uint8_t* srow = q.scales + (int64_t)row * (q.K >> 5);
    if constexpr (Fp8<kElem>::kBits == 6) {
        // lanes 0, 1, 2 of the block store 8 bytes each: one instruction covers the block's 24 bytes
        const uint32_t part = lane & 3;
        if (part < 3) {
            uint2* dst = reinterpret_cast<uint2*>(q.codes + (int64_t)row * (q.K / 4 * 3) + (int64_t)kblk * 24);
            dst[part] = make_uint2(part == 0 ? six[0] : part == 1 ? six[2] : six[4],
                                   part == 0 ? six[1] : part == 1 ? six[3] : six[5]);
        }
    } else {
        *reinterpret_cast<uint2*>(q.codes + (int64_t)row * q.K + col) = make_uint2(res.lo, res.hi);
    }
    if (q.scales_dword) {
        if ((lane & 15) == 0) *reinterpret_cast<uint32_t*>(srow + kblk) = ew;
    } else if ((lane & 3) == 0) {
        srow[kblk] = (uint8_t)res.E;
    }
    if (kMbs && (lane & 15) == 0) q.mbs[(int64_t)row * q.nmac + (col >> 7)] = (uint8_t)res.m8;
}

template <int kElem, bool kHwCvt, bool kMbs>
__global__ __launch_bounds__(kThreads8) void quantize8_kernel(Quant8Args q) {
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(blockIdx.x * (kThreads8 / kWave) + (threadIdx.x >> 6));
    const uint32_t nwaves = gridDim.x * (kThreads8 / kWave);
    for (uint32_t c0 = wave * kUnroll8; c0 < q.total_chunks; c0 += nwaves * kUnroll8) {
        u32x4 v[kUnroll8];
        uint32_t row[kUnroll8], col[kUnroll8];
        bool valid[kUnroll8];
        uint32_t r = c0 / q.chunks_per_row, cc = c0 - r * q.chunks_per_row;
#pragma unroll
        for (int u = 0; u < kUnroll8; ++u) {
            row[u] = r;
            col[u] = cc * kChunk8 + lane * 8;
            valid[u] = c0 + u < q.total_chunks && col[u] < q.K;
            v[u] = u32x4{0, 0, 0, 0};
            if (valid[u])
                v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(q.x + (int64_t)r * q.ldx + col[u]));
            if (++cc == q.chunks_per_row) { cc = 0; ++r; }
        }
        if constexpr (kHwCvt && Fp8<kElem>::kBits == 6) {
            // 6-bit formats: the hardware converts 32 fp32 values at a time, which is what a lane holds over the
            // kUnroll8 chunks in flight (8 each, every chunk with its own multiplier).
            static_assert(kUnroll8 == 4, "four chunks of eight elements fill one convert");
            Chunk8 res[kUnroll8];
            if (!quantize_chunks6_hw<kElem, kMbs>(v, q, res)) {
#pragma unroll
                for (int u = 0; u < kUnroll8; ++u) res[u] = quantize_chunk8<kElem, false, kMbs>(v[u], q);
            }
#pragma unroll
            for (int u = 0; u < kUnroll8; ++u) {
                if (c0 + u >= q.total_chunks) break;  // wave-uniform
                store_chunk8<kElem, kMbs>(q, res[u], lane, row[u], col[u], valid[u]);
            }
        } else {
#pragma unroll
            for (int u = 0; u < kUnroll8; ++u) {
                if (c0 + u >= q.total_chunks) break;  // wave-uniform
                const Chunk8 res = quantize_chunk8<kElem, kHwCvt, kMbs>(v[u], q);
                store_chunk8<kElem, kMbs>(q, res, lane, row[u], col[u], valid[u]);
            }
        }
    }
}

// ---- MBS-Dynamic (Sec. 4.3.3, Sec. 5.3) on these formats ----
// As for MXFP4: per macro block the word is searched among
//     m_j = (m_static + (cand_first + j) * cand_stride) mod 256,  j = 0 .. cand_count - 1,
// for the least sum of squared errors of the 1x128 block, measured directly.  The scaled element t = x F 2^s is
// exact in fp32, its grid value comes out of the rounding addition of code8_alu (the sum minus the added constant),
// and their difference is exact.  The cost has a fixed order of operations so that the minimum is reproducible:
// fused multiply-adds over the lane's 8 elements in order, pairwise sums over the 4 lanes of a block, an exact
// rescale from the block's binade to the macro block's, pairwise sums over the 4 blocks, one multiplication by
// the reciprocal of F^2 (within an ulp).  The static word is the incumbent; a candidate replaces the current choice only with a strictly
// smaller cost.  The search runs where fp32 holds every intermediate exactly (exponent field of the macro-block
// absmax in [64, 249], no Inf/NaN in it); a block whose own absmax is zero or more than 30 binades below
// contributes nothing.
struct Dyn8Args {
    Quant8Args q;
    int cand_first, cand_count, cand_stride;
};

struct Cand8 {
    uint32_t lo, hi, E;
    float cost;
};

template <int kCtrl>
__device__ __forceinline__ float dpp_f(float v) {
    return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), kCtrl, 0xF, 0xF, true));
}

// Codes, scale byte and macro-block cost of word m.  xf: the lane's 8 elements; amax: bf16 magnitude bits of the
// block's absmax; counts: the block contributes to the cost; e128: exponent field of the macro block's absmax.  The
// cost is uniform over the 16 lanes of the macro block.
template <typename T>
__device__ __forceinline__ Cand8 eval_candidate8(const float (&xf)[8], uint32_t amax, bool counts, uint32_t e128, uint32_t m,
                                                 uint32_t carry) {
#pragma clang fp contract(off)
    const float F = __uint_as_float(0x3F800000u | (m << 15));
    const float scaled_max = __uint_as_float(amax << 16) * F;  // exact
    uint32_t E = ((__float_as_uint(scaled_max) + carry) >> 23) - (uint32_t)T::kEmax;
    E = amax ? E : 127u;
    const float mult = __uint_as_float(((254u - E) << 23) | (m << 15));  // F * 2^(127 - E)
    const float vmax = __uint_as_float(T::kMaxBits);
    uint32_t lo = 0, hi = 0;
    float acc = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float t = xf[i] * mult;  // exact
        const uint32_t tb = __float_as_uint(t);
        const float a = __uint_as_float(tb & 0x7FFFFFFFu);
        const float y = fminf(a, vmax);
        const uint32_t ey = max(__float_as_uint(y) >> 23, (uint32_t)(127 + 1 - T::kBias));
        const float magic = __uint_as_float(((ey + 23u - T::kMbits) << 23) | 0x400000u);
        const float w = y + magic;     // y to the spacing of its binade, nearest even
        const uint32_t qbits = __float_as_uint(w) & ((1u << (T::kMbits + 2)) - 1u);
        const uint32_t code = (((ey - 127u + T::kBias) << T::kMbits) + qbits - (1u << T::kMbits)) | ((tb >> 31) << (T::kBits - 1));
        put_code<T>(lo, hi, i, code);
        const float r = a - (w - magic);  // exact: the grid value is within a factor 2 of |t|, or |t| is tiny
        acc = __builtin_fmaf(r, r, acc);
    }
    // block sum, then from units of the block's binade to units of the macro block's: 4^(E + emax - e128)
    acc = counts ? acc : 0.0f;
    acc = acc + dpp_f<0xB1>(acc);   // quad_perm [1,0,3,2]
    acc = acc + dpp_f<0x4E>(acc);   // quad_perm [2,3,0,1]
    const float rescale = __uint_as_float(counts ? (127u + 2u * (E + (uint32_t)T::kEmax - e128)) << 23 : 0x3F800000u);
    acc = acc * rescale;
    acc = acc + dpp_f<0x141>(acc);  // lane i <-> 7 - i inside each half row: the neighbouring block
    acc = acc + dpp_f<0x140>(acc);  // lane i <-> 15 - i inside each row: the neighbouring pair of blocks
    return {lo, hi, E, acc * __builtin_amdgcn_rcpf(F * F)};
}

template <int kElem>
__global__ __launch_bounds__(kThreads8) void quantize8_dynamic_kernel(Dyn8Args d) {
    using T = Fp8<kElem>;
    const Quant8Args& q = d.q;
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(blockIdx.x * (kThreads8 / kWave) + (threadIdx.x >> 6));
    const uint32_t nwaves = gridDim.x * (kThreads8 / kWave);
    for (uint32_t c = wave; c < q.total_chunks; c += nwaves) {
        const uint32_t row = c / q.chunks_per_row, col = (c - row * q.chunks_per_row) * kChunk8 + lane * 8;
        const bool valid = col < q.K;
        u32x4 v = {0, 0, 0, 0};
        if (valid) v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(q.x + (int64_t)row * q.ldx + col));
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};

        // absmax over the finite elements of the lane, block and macro block; Inf/NaN flag of the macro block
        uint32_t amax = 0, nf = 0;
        float xf[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t lo = w[i] & 0x7FFFu, hi = (w[i] >> 16) & 0x7FFFu;
            if (lo >= 0x7F80u) nf = 1; else amax = max(amax, lo);
            if (hi >= 0x7F80u) nf = 1; else amax = max(amax, hi);
            xf[2 * i] = __uint_as_float(w[i] << 16);
            xf[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
        nf |= dpp_quad_xor1(nf);
        nf |= dpp_quad_xor2(nf);
        const uint32_t nf_block = nf;
        nf |= dpp_row_ror4(nf);
        nf |= dpp_row_ror8(nf);
        amax = max(amax, dpp_quad_xor1(amax));
        amax = max(amax, dpp_quad_xor2(amax));
        uint32_t mmax = max(amax, dpp_row_ror4(amax));
        mmax = max(mmax, dpp_row_ror8(mmax));

        const uint32_t m_static = mbs8_word_of_absmax<T>(mmax);
        const uint32_t e128 = mmax >> 7;
        const bool searchable = !nf && e128 >= 64u && e128 <= 249u;
        const bool counts = amax != 0 && (amax >> 7) + 30u >= e128;

        Cand8 best = eval_candidate8<T>(xf, amax, counts, e128, m_static, q.carry);
        uint32_t m_best = m_static;
        for (int j = 0; j < d.cand_count; ++j) {
            const uint32_t step = (uint32_t)((d.cand_first + j) * d.cand_stride) & 255u;
            if (step == 0) continue;  // the static word again: it cannot beat itself (uniform over the launch)
            uint32_t m = (m_static + step) & 255u;
            m = searchable ? m : m_static;
            const Cand8 cand = eval_candidate8<T>(xf, amax, counts, e128, m, q.carry);
            if (cand.cost < best.cost) {
                best = cand;
                m_best = m;
            }
        }

        // the fp32 route gave valid codes unless some block of this wavefront lies outside its range (Inf/NaN, or an
        // absmax exponent field outside [24, 249]); then the all-integer path redoes the chunk with the chosen word
        const bool odd = nf_block || (amax >= (250u << 7)) || (amax != 0 && amax < (24u << 7));
        Chunk8 res = {best.lo, best.hi, best.E, m_best};
        if (__builtin_amdgcn_ballot_w64(odd) != 0) res = quantize_chunk8_exact<T>(v, q.rule, 1, (int)m_best);
        store_chunk8<kElem, true>(q, res, lane, row, col, valid);
    }
}

template <int kElem>
void launch8(const Quant8Args& q, int use_mbs, bool hwcvt, dim3 grid, hipStream_t s) {
    const dim3 block(kThreads8);
    if (hwcvt) {
        if (use_mbs) hipLaunchKernelGGL((quantize8_kernel<kElem, true, true>), grid, block, 0, s, q);
        else hipLaunchKernelGGL((quantize8_kernel<kElem, true, false>), grid, block, 0, s, q);
    } else {
        if (use_mbs) hipLaunchKernelGGL((quantize8_kernel<kElem, false, true>), grid, block, 0, s, q);
        else hipLaunchKernelGGL((quantize8_kernel<kElem, false, false>), grid, block, 0, s, q);
    }
}

// Argument checks and launch parameters shared by the entry points: MX_OK with *nothing = true when there is
// nothing to do.
int prepare_quantize_elem(int elem, const void* x, int64_t rows, int64_t K, int64_t ldx, int rule, int use_mbs,
                          uint8_t* codes, uint8_t* scales, uint8_t* mbs, Quant8Args& q, bool* nothing) {
    *nothing = false;
    if (elem < MX_ELEM_E2M1 || elem > MX_ELEM_E3M2 || elem == MX_ELEM_E2M1) return MX_EINVAL;
    if (rows < 0 || K < 0 || (K % kBlock) != 0 || ldx < K) return MX_EINVAL;
    if (K > (int64_t)1 << 30) return MX_EINVAL;  // a lane's column inside its row is a 32-bit number
    if (rule != MX_RULE_OCP && rule != MX_RULE_FLOOR && rule != MX_RULE_OAS) return MX_EINVAL;
    if (rows == 0 || K == 0) { *nothing = true; return MX_OK; }
    if (!x || !codes || !scales || (use_mbs && !mbs)) return MX_ENULL;
    if (!aligned(x, 16) || (ldx % 8) != 0 || !aligned(codes, 8)) return MX_EALIGN;
    const int64_t chunks_per_row = (K + kChunk8 - 1) / kChunk8, total = rows * chunks_per_row;
    if (total >= ((int64_t)1 << 32) - kUnroll8 || rows >= ((int64_t)1 << 31)) return MX_EINVAL;  // 32-bit chunk ids
    if (int st = check_device()) return st;
    q.x = static_cast<const uint16_t*>(x);
    q.codes = codes; q.scales = scales; q.mbs = mbs;
    q.K = K; q.ldx = ldx; q.nmac = (K + kMacro - 1) / kMacro;
    q.chunks_per_row = (uint32_t)chunks_per_row;
    q.total_chunks = (uint32_t)total;
    q.rule = rule;
    q.scales_dword = (K % kMacro) == 0 && aligned(scales, 4);
    const uint32_t carry_floor[5] = {0, Fp8<MX_ELEM_E4M3>::kCarryFloor, Fp8<MX_ELEM_E5M2>::kCarryFloor,
                                     Fp8<MX_ELEM_E2M3>::kCarryFloor, Fp8<MX_ELEM_E3M2>::kCarryFloor};
    const uint32_t carry_oas[5] = {0, Fp8<MX_ELEM_E4M3>::kCarryOas, Fp8<MX_ELEM_E5M2>::kCarryOas,
                                   Fp8<MX_ELEM_E2M3>::kCarryOas, Fp8<MX_ELEM_E3M2>::kCarryOas};
    q.carry = rule == MX_RULE_FLOOR ? carry_floor[elem] : rule == MX_RULE_OAS ? carry_oas[elem] : 0u;
    return MX_OK;
}

int launch_quantize_elem(int elem, const void* x, int64_t rows, int64_t K, int64_t ldx, int rule, int use_mbs,
                         uint8_t* codes, uint8_t* scales, uint8_t* mbs, void* stream, bool hwcvt = true) {
    Quant8Args q;
    bool nothing;
    if (int st = prepare_quantize_elem(elem, x, rows, K, ldx, rule, use_mbs, codes, scales, mbs, q, &nothing)) return st;
    if (nothing) return MX_OK;
    const int64_t total = q.total_chunks;
    const int64_t waves = (total + kUnroll8 - 1) / kUnroll8;
    int64_t blocks = (waves + (kThreads8 / kWave) - 1) / (kThreads8 / kWave);
    if (blocks > (1 << 22)) blocks = 1 << 22;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)blocks);
    if (elem == MX_ELEM_E4M3) launch8<MX_ELEM_E4M3>(q, use_mbs, hwcvt, grid, s);
    else if (elem == MX_ELEM_E5M2) launch8<MX_ELEM_E5M2>(q, use_mbs, hwcvt, grid, s);
    else if (elem == MX_ELEM_E2M3) launch8<MX_ELEM_E2M3>(q, use_mbs, hwcvt, grid, s);
    else launch8<MX_ELEM_E3M2>(q, use_mbs, hwcvt, grid, s);
    return launch_status();
}

int launch_quantize_elem_dynamic(int elem, const void* x, int64_t rows, int64_t K, int64_t ldx, int rule, int cand_first,
                                 int cand_count, int cand_stride, uint8_t* codes, uint8_t* scales, uint8_t* mbs,
                                 void* stream) {
    if (cand_count < 0 || cand_count > 256 || cand_first < -65536 || cand_first > 65536 || cand_stride < -65536 ||
        cand_stride > 65536)
        return MX_EINVAL;
    Dyn8Args d;
    bool nothing;
    if (int st = prepare_quantize_elem(elem, x, rows, K, ldx, rule, 1, codes, scales, mbs, d.q, &nothing)) return st;
    if (nothing) return MX_OK;
    d.cand_first = cand_first; d.cand_count = cand_count; d.cand_stride = cand_stride;
    int64_t blocks = ((int64_t)d.q.total_chunks + (kThreads8 / kWave) - 1) / (kThreads8 / kWave);
    if (blocks > (1 << 22)) blocks = 1 << 22;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)blocks), block(kThreads8);
    if (elem == MX_ELEM_E4M3) hipLaunchKernelGGL(quantize8_dynamic_kernel<MX_ELEM_E4M3>, grid, block, 0, s, d);
    else if (elem == MX_ELEM_E5M2) hipLaunchKernelGGL(quantize8_dynamic_kernel<MX_ELEM_E5M2>, grid, block, 0, s, d);
    else if (elem == MX_ELEM_E2M3) hipLaunchKernelGGL(quantize8_dynamic_kernel<MX_ELEM_E2M3>, grid, block, 0, s, d);
    else hipLaunchKernelGGL(quantize8_dynamic_kernel<MX_ELEM_E3M2>, grid, block, 0, s, d);
    return launch_status();
}

}  // namespace
}  // namespace mx

extern "C" {

int mx_quantize_elem_mbs_dynamic(mx_elem_t elem, const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule,
                                 int32_t cand_first, int32_t cand_count, int32_t cand_stride, uint8_t* codes,
                                 uint8_t* scales, uint8_t* mbs, void* stream) {
    return mx::launch_quantize_elem_dynamic((int)elem, x_bf16, rows, K, ldx, (int)rule, cand_first, cand_count, cand_stride,
                                            codes, scales, mbs, stream);
}

int mx_quantize_elem(mx_elem_t elem, const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule,
                     int use_mbs, uint8_t* codes, uint8_t* scales, uint8_t* mbs, void* stream) {
    return mx::launch_quantize_elem((int)elem, x_bf16, rows, K, ldx, (int)rule, use_mbs, codes, scales, mbs, stream);
}

int mx_internal_quantize_elem(mx_elem_t elem, const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule,
                              int use_mbs, int hw_convert, uint8_t* codes, uint8_t* scales, uint8_t* mbs, void* stream) {
    return mx::launch_quantize_elem((int)elem, x_bf16, rows, K, ldx, (int)rule, use_mbs, codes, scales, mbs, stream,
                                    hw_convert != 0);
}

}  // extern "C"
