// GEMM  C = A * B^T  with the Macro Block Scaling correction for a handful of activation rows (decode) and operands
// in the 8-bit and 6-bit MX element formats (Sec. 1, footnote: the methods carry over to MXFP6 and MXFP8): bound by
// streaming the weights once, like the MXFP4 few-row kernel, whose arrangement this one keeps.
//
// A workgroup owns 16 FN columns of C (16 FN rows of B) and all M <= 16 FM rows of A; its eight wavefronts split K
// between them in groups of four macro blocks and add their partial results through LDS at the end.  Nothing is
// staged through LDS: no byte of B is used twice, and A stays in the L2.
//
// v_mfma_scale_f32_16x16x128_f8f6f4 is one macro block deep; the activations feed srcA and the weights srcB, so
// D[4 q + i][r] leaves lane 16 q + r with C[m = 4 q + i][n = r]: sigma_B of the lane's own weight row is a per-lane
// scalar and the four sigma_A values come from an LDS table.  Operand layout, as measured on the device (the same
// for srcA and srcB):
//   8-bit: lane 16 q + r holds, of row r, bytes 16 q .. 16 q + 15 of the macro block in its first four registers
//          and bytes 64 + 16 q .. in its last four; the instruction's 32-element block b (bytes 32 b .. 32 b + 31)
//          is scaled by the E8M0 byte that lane group b supplies, so lane 16 q + r supplies the byte of block q of
//          row r although its own elements belong to blocks q / 2 and 2 + q / 2.
//   6-bit: as for FP4, lane 16 q + r holds the whole block q of row r (24 bytes, six registers) and its own byte.
#include "mx_gemm_shared.h"

namespace mx {
namespace {

constexpr int kSkinnyWaves = 8, kSkinnyThreads = kSkinnyWaves * kWave;
constexpr int kSkinnyGroup = 4;  // macro blocks per load group

typedef int v2i __attribute__((ext_vector_type(2)));

// FM, FN: 16-row fragments of A and of B per workgroup; kFmtA / kFmtB: the matrix instruction's format selectors
// (0 = E4M3, 1 = E5M2, 2 = E2M3, 3 = E3M2)
template <int kFmtA, int kFmtB, int FM, int FN>
__global__ __launch_bounds__(kSkinnyThreads) void gemm_skinny_elem_kernel(GemmArgs g) {
    constexpr bool kSix = kFmtA >= 2;
    static_assert(kSix == (kFmtB >= 2), "6-bit operands: both or neither");
    constexpr int kMacroBytes = kSix ? 96 : 128;  // code bytes of a row per macro block
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    // a null array means sigma = 1
    const bool sigma_a = g.a_mbs != nullptr, sigma_b = g.b_mbs != nullptr;
    const int K = (int)g.K, nmac = K / kMacro, ngroups = nmac / kSkinnyGroup;
    const int row_bytes = kSix ? K / 4 * 3 : K, scale_bytes = K >> 5;
    const int tid = threadIdx.x, l = tid & 63, r = l & 15, q = l >> 4;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t n0 = (int64_t)blockIdx.x * (16 * FN);

    // buffer resources sized to the valid rows: rows past the end read zero
    const int kRsrcFlags = 0x00020000;
    const int64_t a_rows = min((int64_t)(FM * 16), g.M), b_rows = min((int64_t)(FN * 16), g.N - n0);
    auto rsrc = [&](const uint8_t* base, int64_t row0, int64_t rows, int per_row) {
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(base) + row0 * per_row, 0, (int)(rows * per_row), kRsrcFlags);
    };
    const __amdgpu_buffer_rsrc_t a_codes = rsrc(g.a_codes, 0, a_rows, row_bytes), b_codes = rsrc(g.b_codes, n0, b_rows, row_bytes);
    const __amdgpu_buffer_rsrc_t a_scales = rsrc(g.a_scales, 0, a_rows, scale_bytes), b_scales = rsrc(g.b_scales, n0, b_rows, scale_bytes);
    // (no words: an empty buffer, every word reads 0)
    const __amdgpu_buffer_rsrc_t b_mbs = rsrc(g.b_mbs ? g.b_mbs : g.b_codes, g.b_mbs ? n0 : 0, g.b_mbs ? b_rows : 0, nmac);
    // per-lane offsets of row r of fragment 0: the lane's codes of macro block 0, scales, MBS words
    const int code_off = r * row_bytes + (kSix ? 24 : 16) * q, scale_off = r * scale_bytes, m8_off = r * nmac;

    struct Group {
        v8i wc[FN][kSkinnyGroup], ac[FM][kSkinnyGroup];
        v4i ws[FN], as[FM];
        uint32_t wm8[FN];
    };
    // the lane's operand registers of macro block mb of the row at voff
    auto load_codes = [&](const __amdgpu_buffer_rsrc_t& codes, int voff, int mb) {
        const int soff = mb * kMacroBytes;
        if constexpr (kSix) {
            const v4i lo = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(codes, voff, soff, 0));
            const v2i hi = __builtin_bit_cast(v2i, __builtin_amdgcn_raw_buffer_load_b64(codes, voff + 16, soff, 0));
            return v8i{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, 0, 0};
        } else {
            const v4i lo = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(codes, voff, soff, 0));
            const v4i hi = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(codes, voff + 64, soff, 0));
            return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    };
    auto load_group = [&](Group& d, int grp) {
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int t = 0; t < kSkinnyGroup; ++t) d.wc[j][t] = load_codes(b_codes, code_off + j * 16 * row_bytes, grp * kSkinnyGroup + t);
            d.ws[j] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(b_scales, scale_off + j * 16 * scale_bytes, grp * 16, 0));
            d.wm8[j] = __builtin_amdgcn_raw_buffer_load_b32(b_mbs, m8_off + j * 16 * nmac, grp * 4, 0);
        }
#pragma unroll
        for (int f = 0; f < FM; ++f) {
#pragma unroll
            for (int t = 0; t < kSkinnyGroup; ++t) d.ac[f][t] = load_codes(a_codes, code_off + f * 16 * row_bytes, grp * kSkinnyGroup + t);
            d.as[f] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(a_scales, scale_off + f * 16 * scale_bytes, grp * 16, 0));
        }
    };
    // LDS: partial results [wave][fragment pair][lane] float4, then the sigma_A table [macro block][FM * 16]
    v4f* red = reinterpret_cast<v4f*>(smem);
    float* sig_a = reinterpret_cast<float*>(smem + kSkinnyWaves * FM * FN * kWave * 16);

    // this wavefront's groups (K <= 8192: at most two), each requested whole before its first matrix instruction.
    // (Requested inside the loop: with the first group's loads ahead of the loop and the next group's at its end,
    // the compiler's register allocation overwrote the operands of a group's fourth macro block before use.)
    const int per_wave = (ngroups + kSkinnyWaves - 1) / kSkinnyWaves;
    const int first = w * per_wave, last = min(first + per_wave, ngroups);

    if (sigma_a) {
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
        Group d;
        load_group(d, grp);
        const float* sig_g = sig_a + grp * kSkinnyGroup * (FM * 16);
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
                const uint32_t sw = (uint32_t)d.ws[j][t] >> (8 * q);  // the instruction reads byte 0: block q of the row
                // F = 1 + m8/256 is exact, the reciprocal within an ulp; m8 = 0 (also: no words) gives exactly 1
                const float sn = __builtin_amdgcn_rcpf(1.0f + (float)((d.wm8[j] >> (8 * t)) & 0xFFu) * (1.0f / 256.0f));
#pragma unroll
                for (int f = 0; f < FM; ++f) {
                    const uint32_t sa = (uint32_t)d.as[f][t] >> (8 * q);
                    const v4f zero = {0.f, 0.f, 0.f, 0.f};
                    const v4f p = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(d.ac[f][t], d.wc[j][t], zero, kFmtA, kFmtB, 0,
                                                                                    (int)sa, 0, (int)sw);
                    if (sigma_a || sigma_b) acc[f][j] += p * (sm[f] * sn);
                    else acc[f][j] += p;
                }
            }
        }
    }

    // ---- add the eight partial results, store ----
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

template <int kFmtA, int kFmtB, int FM, int FN>
int launch_variant(const GemmArgs& g, hipStream_t s) {
    const int64_t blocks = (g.N + 16 * FN - 1) / (16 * FN);
    if (blocks > (int64_t)1 << 30) return MX_EINVAL;
    const size_t lds = (size_t)kSkinnyWaves * FM * FN * kWave * 16 + (g.a_mbs ? (size_t)(g.K / kMacro) * FM * 16 * 4 : 0);
    hipLaunchKernelGGL((gemm_skinny_elem_kernel<kFmtA, kFmtB, FM, FN>), dim3((unsigned)blocks), dim3(kSkinnyThreads), lds, s, g);
    return launch_status();
}

// about one workgroup per compute unit where the weight has the rows for it; at most two fragment pairs each (a
// group of four macro blocks of an 8-bit fragment is 32 registers)
template <int kFmtA, int kFmtB>
int launch_formats(const GemmArgs& g, hipStream_t s) {
    const int64_t frags = (g.N + 15) / 16;
    if (g.M <= 16) return frags > 256 ? launch_variant<kFmtA, kFmtB, 1, 2>(g, s) : launch_variant<kFmtA, kFmtB, 1, 1>(g, s);
    if (g.M <= 32) return launch_variant<kFmtA, kFmtB, 2, 1>(g, s);
    return launch_variant<kFmtA, kFmtB, 4, 1>(g, s);
}

}  // namespace

// M <= 64, K % 512 == 0, K <= 8192, 16-byte aligned code and scale arrays, 4-byte aligned MBS arrays, both operands
// 8-bit or both 6-bit, not grouped; the caller has checked all of them.
int launch_gemm_skinny_elem(const GemmArgs& g, int a_elem, int b_elem, hipStream_t s) {
    const bool six = a_elem == MX_ELEM_E2M3 || a_elem == MX_ELEM_E3M2;
    const bool a2 = a_elem == MX_ELEM_E5M2 || a_elem == MX_ELEM_E3M2, b2 = b_elem == MX_ELEM_E5M2 || b_elem == MX_ELEM_E3M2;
    if (six) {
        if (!a2 && !b2) return launch_formats<2, 2>(g, s);
        if (!a2 && b2) return launch_formats<2, 3>(g, s);
        if (a2 && !b2) return launch_formats<3, 2>(g, s);
        return launch_formats<3, 3>(g, s);
    }
    if (!a2 && !b2) return launch_formats<0, 0>(g, s);
    if (!a2 && b2) return launch_formats<0, 1>(g, s);
    if (a2 && !b2) return launch_formats<1, 0>(g, s);
    return launch_formats<1, 1>(g, s);
}

}  // namespace mx
