// MXFP4 GEMM  C = A * B^T  for a handful of activation rows (decode): bound by streaming the weights once.
//
// A workgroup owns 16 FN columns of C (16 FN rows of B) and all M <= 16 FM rows of A; its eight wavefronts
// split K between them in groups of four macro blocks and add their partial results through LDS at the
// end.  FN is chosen so that the launch has about one workgroup per compute unit: then every weight byte
// of a typical projection is requested in a single round trip to memory.  Nothing is staged through LDS:
// no byte of B is used twice, and A (a few KB per macro block column) stays in the L2.
//
// v_mfma_scale_f32_16x16x128_f8f6f4 is one macro block deep.  Here the activations feed srcA and the
// weights srcB (lane = 16 q + r holds row r, k-block q of either), so D[4 q + i][r] leaves a lane with
// C[m = 4 q + i][n = r]: sigma_B of the lane's own weight row is a per-lane scalar, computed from the MBS
// word the lane fetched itself, and the four sigma_A values come from a small LDS table that the workgroup
// fills once (one reciprocal per activation row and macro block).  Per lane and group of four macro
// blocks: four 16-byte code pieces per fragment, the 16 E8M0 bytes of the row as one 16-byte piece (each
// instruction takes its byte by shifting), the row's four MBS words as one dword.
//
// Fused form (activations quantized inside this kernel, Sec. 4.3 / 5.3): instead of
// codes the lane fetches the 32 bf16 of its row and k-block (four 16-byte pieces), which is exactly one
// E8M0 block, so its absmax needs no exchange; the macro-block absmax is the maximum over the four lanes
// 16 apart.  MBS word, scale byte and codes follow the quantizer's arithmetic to the bit, the 16 bytes of
// codes are the matrix instruction's operand as they stand, and sigma_A goes through a small LDS table
// private to the wavefront (each wavefront quantizes exactly the K range it multiplies).  No quantized
// activation is ever written to memory, and one launch does the work of two.
#include "mx_gemm_shared.h"
#include "mx_quantize_math.h"

namespace mx {
namespace {

constexpr int kSkinnyWaves = 8, kSkinnyThreads = kSkinnyWaves * kWave;
constexpr int kSkinnyGroup = 4;  // macro blocks per load group

struct SkinnyArgs {
    GemmArgs g;
    // fused form only: bf16 activations [M, ldx], the scale rule and whether MBS-Static words are formed
    const uint16_t* x;
    int64_t ldx;
    int rule;
    uint32_t carry;
    int a_mbs;
};

__device__ __forceinline__ uint32_t lane_xor(uint32_t v, int lane, int mask) {
    return (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ mask) << 2, (int)v);
}

struct Block32 {
    v4i codes;
    uint32_t E, m8;
};

// One 32-element block per lane (raw: its bf16 pairs), the four lanes 16, 32, 48 apart forming a macro
// block.  All-integer arithmetic: exact for subnormal and huge values, Inf and NaN.
__device__ __noinline__ Block32 quantize_block32_exact(v4i r0, v4i r1, v4i r2, v4i r3, int rule, int use_mbs, int lane) {
    const v4i raw[4] = {r0, r1, r2, r3};
    uint32_t amax = 0, nf = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t w = (uint32_t)raw[i / 4][i % 4], lo = w & 0x7FFFu, hi = (w >> 16) & 0x7FFFu;
        if (lo >= 0x7F80u) nf = 1; else amax = max(amax, lo);
        if (hi >= 0x7F80u) nf = 1; else amax = max(amax, hi);
    }
    uint32_t mmax = max(amax, lane_xor(amax, lane, 16));
    mmax = max(mmax, lane_xor(mmax, lane, 32));
    const uint32_t m8 = use_mbs ? mbs_word_of_absmax(mmax) : 0u;
    const uint32_t u = 256u + m8;
    const int E = nf ? 255 : amax == 0 ? 127 : exact_scale_byte(amax, u, rule);
    const int s = 127 - E;
    Block32 out = {v4i{0, 0, 0, 0}, (uint32_t)E, m8};
    if (!nf) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint32_t w = (uint32_t)raw[i / 4][i % 4];
            const uint32_t pair = exact_code(w & 0xFFFFu, u, s) | (exact_code(w >> 16, u, s) << 4);
            out.codes[i / 4] |= (int)(pair << (8 * (i % 4)));
        }
    }
    return out;
}

__device__ __forceinline__ Block32 quantize_block32(const v4i (&raw)[4], int rule, uint32_t carry, int use_mbs, int lane) {
    uint32_t m = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) m = pk_max_u16(m, (uint32_t)raw[i / 4][i % 4] & 0x7FFF7FFFu);
    const uint32_t amax = max(m & 0xFFFFu, m >> 16);
    // exponent field outside [24, 249] (or Inf/NaN): leave fp32 arithmetic, wave-uniformly
    const bool odd = (amax >= (250u << 7)) || (amax != 0 && amax < (24u << 7));
    if (__builtin_amdgcn_ballot_w64(odd) != 0) return quantize_block32_exact(raw[0], raw[1], raw[2], raw[3], rule, use_mbs, lane);
    uint32_t m8 = 0;
    if (use_mbs) {
        uint32_t mmax = max(amax, lane_xor(amax, lane, 16));
        mmax = max(mmax, lane_xor(mmax, lane, 32));
        m8 = mmax ? mbs_word_of_mantissa_fast(mmax & 0x7Fu) : 0u;
    }
    // absmax * F is exact in fp32; exponent field + carry gives the stored byte; multiplier F * 2^(127-E)
    const float scaled_max = __uint_as_float(amax << 16) * __uint_as_float(0x3F800000u | (m8 << 15));
    uint32_t E = ((__float_as_uint(scaled_max) + carry) >> 23) - 2u;
    E = amax ? E : 127u;
    const float mult = __uint_as_float(((254u - E) << 23) | (m8 << 15));
    Block32 out = {v4i{0, 0, 0, 0}, E, m8};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint32_t c = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t w = (uint32_t)raw[i][j];
            const float t0 = __uint_as_float(w << 16) * mult, t1 = __uint_as_float(w & 0xFFFF0000u) * mult;
            if (j == 0) c = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c, t0, t1, 1.0f, 0);
            if (j == 1) c = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c, t0, t1, 1.0f, 1);
            if (j == 2) c = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c, t0, t1, 1.0f, 2);
            if (j == 3) c = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c, t0, t1, 1.0f, 3);
        }
        out.codes[i] = (int)c;
    }
    return out;
}

// FM, FN: 16-row fragments of A and of B per workgroup
template <int FM, int FN, bool kFused>
__global__ __launch_bounds__(kSkinnyThreads) void gemm_skinny_kernel(SkinnyArgs args) {
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const GemmArgs& g = args.g;
    // a null array means sigma = 1
    const bool sigma_a = kFused ? args.a_mbs != 0 : g.a_mbs != nullptr, sigma_b = g.b_mbs != nullptr;
    const int K = (int)g.K, nmac = K / kMacro, ngroups = nmac / kSkinnyGroup;
    const int row_bytes = K >> 1, scale_bytes = K >> 5;
    const int tid = threadIdx.x, l = tid & 63, r = l & 15, q = l >> 4;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t n0 = (int64_t)blockIdx.x * (16 * FN);

    // fused: the bf16 rows as one buffer ending with the last row's K elements; rows past M read zero
    const Operand opa = make_operand(g.a_codes, g.a_scales, g.a_mbs, 0, g.M, FM * 16, g.K);  // (fused: not used)
    const __amdgpu_buffer_rsrc_t opx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(args.x), 0, kFused ? (int)(((g.M - 1) * args.ldx + g.K) * 2) : 0, 0x00020000);
    const int x_off = r * (int)args.ldx * 2 + q * 64;  // fused: this lane's block of row r, fragment 0, macro block 0
    const Operand opb = make_operand(g.b_codes, g.b_scales, g.b_mbs, n0, g.N, FN * 16, g.K);
    // per-lane offsets of row r of fragment 0: codes of k-block q, scales, MBS words; rows past the operand
    // are out of range and read zero
    const int code_off = r * row_bytes + q * 16, scale_off = r * scale_bytes, m8_off = r * nmac;

    struct Group {
        v4i wc[FN][kSkinnyGroup], ws[FN], ac[FM][kSkinnyGroup], as[FM];
        uint32_t wm8[FN];
    };
    auto load_group = [&](Group& d, int grp) {
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int t = 0; t < kSkinnyGroup; ++t)
                d.wc[j][t] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(opb.codes, code_off + j * 16 * row_bytes,
                                                                                          (grp * kSkinnyGroup + t) * 64, 0));
            d.ws[j] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(opb.scales, scale_off + j * 16 * scale_bytes, grp * 16, 0));
            d.wm8[j] = __builtin_amdgcn_raw_buffer_load_b32(opb.mbs, m8_off + j * 16 * nmac, grp * 4, 0);  // no words: zero
        }
        if constexpr (!kFused) {
#pragma unroll
            for (int f = 0; f < FM; ++f) {
#pragma unroll
                for (int t = 0; t < kSkinnyGroup; ++t)
                    d.ac[f][t] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(opa.codes, code_off + f * 16 * row_bytes,
                                                                                              (grp * kSkinnyGroup + t) * 64, 0));
                d.as[f] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(opa.scales, scale_off + f * 16 * scale_bytes, grp * 16, 0));
            }
        }
    };
    // LDS: partial results [wave][fragment pair][lane] float4, then the sigma_A table: [macro block][FM * 16]
    // for all of K, or (fused) one [macro block of the group][FM * 16] table per wavefront
    v4f* red = reinterpret_cast<v4f*>(smem);
    float* sig_a = reinterpret_cast<float*>(smem + kSkinnyWaves * FM * FN * kWave * 16);
    // fused: the bf16 of fragment f for the four macro blocks of a group
    typedef v4i RawGroup[kSkinnyGroup][4];
    auto load_raw = [&](RawGroup& raw, int grp, auto f_) {
        constexpr int f = decltype(f_)::value;
#pragma unroll
        for (int t = 0; t < kSkinnyGroup; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                raw[t][j] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(
                                                        opx, x_off + f * 16 * (int)args.ldx * 2 + j * 16, (grp * kSkinnyGroup + t) * 256, 0));
    };
    // fused: quantize them; codes into d.ac, the scale byte into d.as[f][t] (byte 0 is the lane's own block),
    // sigma_A into this wavefront's table
    auto quantize_raw = [&](Group& d, RawGroup& raw, auto f_) {
        constexpr int f = decltype(f_)::value;
        float* sig_w = sig_a + w * (kSkinnyGroup * FM * 16);
#pragma unroll
        for (int t = 0; t < kSkinnyGroup; ++t) {
            const Block32 b = quantize_block32(raw[t], args.rule, args.carry, args.a_mbs, l);
            d.ac[f][t] = b.codes;
            d.as[f][t] = (int)b.E;
            if (sigma_a && q == 0) sig_w[t * (FM * 16) + f * 16 + r] = __builtin_amdgcn_rcpf(1.0f + (float)b.m8 * (1.0f / 256.0f));
        }
    };

    // this wavefront's groups; the first one is requested before anything else happens
    const int per_wave = (ngroups + kSkinnyWaves - 1) / kSkinnyWaves;
    const int first = w * per_wave, last = min(first + per_wave, ngroups);
    Group d;
    RawGroup raw;
    // fused: the activations of a group are fetched (from the L2) and quantized before its weights are
    // requested, so the raw activations and the weights never hold registers at the same time
    if (kFused && first < last) load_raw(raw, first, std::integral_constant<int, 0>{});
    if (!kFused && first < last) load_group(d, first);

    if (!kFused && sigma_a) {
        for (int idx = tid; idx < nmac * FM * 16; idx += kSkinnyThreads) {
            const int gm = idx / (FM * 16), m = idx % (FM * 16);
            const uint32_t m8 = m < g.M ? g.a_mbs[(int64_t)m * nmac + gm] : 0u;
            sig_a[idx] = __builtin_amdgcn_rcpf(1.0f + (float)m8 * (1.0f / 256.0f));
        }
        __syncthreads();
    }

    v4f acc[FM][FN];
#pragma unroll
    for (int f = 0; f < FM; ++f)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[f][j] = v4f{0.f, 0.f, 0.f, 0.f};
    for (int grp = first; grp < last; ++grp) {
        if constexpr (kFused) {
            if (grp != first) load_raw(raw, grp, std::integral_constant<int, 0>{});
            static_for<FM>([&](auto f_) {
                constexpr int f = decltype(f_)::value;
                quantize_raw(d, raw, f_);
                if constexpr (f + 1 < FM) load_raw(raw, grp, std::integral_constant<int, f + 1>{});
            });
            load_group(d, grp);
        }
        // fused: the table holds this group only and belongs to this wavefront
        const float* sig_g = kFused ? sig_a + w * (kSkinnyGroup * FM * 16) : sig_a + grp * kSkinnyGroup * (FM * 16);
#pragma unroll
        for (int t = 0; t < kSkinnyGroup; ++t) {
            v4f sm[FM];
#pragma unroll
            for (int f = 0; f < FM; ++f) {
                sm[f] = v4f{1.f, 1.f, 1.f, 1.f};
                if (sigma_a) sm[f] = *reinterpret_cast<const v4f*>(sig_g + t * (FM * 16) + f * 16 + q * 4);
            }
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const uint32_t sw = (uint32_t)d.ws[j][t] >> (8 * q);  // the instruction reads byte 0
                // F = 1 + m8/256 is exact, the reciprocal within an ulp; m8 = 0 (also: no words) gives exactly 1
                const float sn = __builtin_amdgcn_rcpf(1.0f + (float)((d.wm8[j] >> (8 * t)) & 0xFFu) * (1.0f / 256.0f));
#pragma unroll
                for (int f = 0; f < FM; ++f) {
                    const uint32_t sa = kFused ? (uint32_t)d.as[f][t] : (uint32_t)d.as[f][t] >> (8 * q);
                    const v4f zero = {0.f, 0.f, 0.f, 0.f};
                    const v4f p = mfma_fp4(d.ac[f][t], d.wc[j][t], zero, sa, sw);  // D[4 q + i][r]: m = 4 q + i, n = r
                    if (sigma_a || sigma_b) acc[f][j] += p * (sm[f] * sn);
                    else acc[f][j] += p;
                }
            }
        }
        if (!kFused && grp + 1 < last) load_group(d, grp + 1);
    }

    // ---- add the eight partial results, store --------------------------------------------------------
#pragma unroll
    for (int f = 0; f < FM; ++f)
#pragma unroll
        for (int j = 0; j < FN; ++j) red[((w * FM + f) * FN + j) * kWave + l] = acc[f][j];
    __syncthreads();
    if (w != 0) return;
#pragma unroll
    for (int f = 0; f < FM; ++f) {
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            v4f sum = red[(f * FN + j) * kWave + l];
#pragma unroll
            for (int o = 1; o < kSkinnyWaves; ++o) sum += red[((o * FM + f) * FN + j) * kWave + l];
            const int64_t n = n0 + j * 16 + r;
            if (n >= g.N) continue;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t m = f * 16 + q * 4 + i;
                if (m >= g.M) continue;
                if (g.c_bf16) static_cast<uint16_t*>(g.C)[m * g.ldc + n] = (uint16_t)f32_to_bf16_bits(sum[i]);
                else static_cast<float*>(g.C)[m * g.ldc + n] = sum[i];
            }
        }
    }
}

template <int FM, int FN, bool kFused>
int launch_skinny_variant(const SkinnyArgs& a, hipStream_t s) {
    const GemmArgs& g = a.g;
    const int64_t blocks = (g.N + 16 * FN - 1) / (16 * FN);
    if (blocks > (int64_t)1 << 30) return MX_EINVAL;
    size_t lds = (size_t)kSkinnyWaves * FM * FN * kWave * 16;
    if (kFused) lds += a.a_mbs ? (size_t)kSkinnyWaves * kSkinnyGroup * FM * 16 * 4 : 0;
    else lds += g.a_mbs ? (size_t)(g.K / kMacro) * FM * 16 * 4 : 0;
    hipLaunchKernelGGL((gemm_skinny_kernel<FM, FN, kFused>), dim3((unsigned)blocks), dim3(kSkinnyThreads), lds, s, a);
    return launch_status();
}

// about one workgroup per compute unit; at most four fragment pairs each (32 KiB of partial results in LDS)
template <int FM, bool kFused>
int launch_skinny_columns(const SkinnyArgs& a, hipStream_t s) {
    const int64_t frags = (a.g.N + 15) / 16;
    if constexpr (FM == 1) {
        if (frags > 2 * 256) return launch_skinny_variant<1, 4, kFused>(a, s);
    }
    if constexpr (FM <= 2) {
        if (frags > 256) return launch_skinny_variant<FM, 2, kFused>(a, s);
    }
    return launch_skinny_variant<FM, 1, kFused>(a, s);
}

template <bool kFused>
int launch_skinny_rows(const SkinnyArgs& a, hipStream_t s) {
    if (a.g.M <= 16) return launch_skinny_columns<1, kFused>(a, s);
    if (a.g.M <= 32) return launch_skinny_columns<2, kFused>(a, s);
    return launch_skinny_columns<4, kFused>(a, s);
}

}  // namespace

// M <= 64, K % 512 == 0, K <= 8192, 16-byte aligned scale arrays, 4-byte aligned MBS arrays, not grouped; the
// caller has checked all of them.
int launch_gemm_skinny(const GemmArgs& g, bool use_mbs, hipStream_t s) {
    SkinnyArgs a = {};
    a.g = g;
    if (!use_mbs) a.g.a_mbs = a.g.b_mbs = nullptr;
    return launch_skinny_rows<false>(a, s);
}

// The same with A given as bf16 [M, ldx] and quantized inside the kernel (rule, MBS-Static words if a_mbs); the
// a_* members of g are not used.  Also requires x 16-byte aligned, ldx % 8 == 0 and the rows of x to span
// less than 2 GiB; the caller has checked these.
int launch_gemm_skinny_fused(const GemmArgs& g, const void* x, int64_t ldx, int rule, bool a_mbs, hipStream_t s) {
    SkinnyArgs a = {};
    a.g = g;
    a.g.a_codes = a.g.a_scales = a.g.a_mbs = nullptr;
    a.x = static_cast<const uint16_t*>(x);
    a.ldx = ldx;
    a.rule = rule;
    a.carry = rule_carry(rule);
    a.a_mbs = a_mbs ? 1 : 0;
    return launch_skinny_rows<true>(a, s);
}

}  // namespace mx
