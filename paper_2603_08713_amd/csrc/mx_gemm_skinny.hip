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
#include "mx_gemm_shared.h"

namespace mx {
namespace {

constexpr int kSkinnyWaves = 8, kSkinnyThreads = kSkinnyWaves * kWave;
constexpr int kSkinnyGroup = 4;  // macro blocks per load group

// FM, FN: 16-row fragments of A and of B per workgroup
template <int FM, int FN>
__global__ __launch_bounds__(kSkinnyThreads) void gemm_skinny_kernel(GemmArgs g) {
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const bool sigma_a = g.a_mbs != nullptr, sigma_b = g.b_mbs != nullptr;  // a null array means sigma = 1
    const int K = (int)g.K, nmac = K / kMacro, ngroups = nmac / kSkinnyGroup;
    const int row_bytes = K >> 1, scale_bytes = K >> 5;
    const int tid = threadIdx.x, l = tid & 63, r = l & 15, q = l >> 4;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t n0 = (int64_t)blockIdx.x * (16 * FN);

    const Operand opa = make_operand(g.a_codes, g.a_scales, g.a_mbs, 0, g.M, FM * 16, g.K);
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
#pragma unroll
        for (int f = 0; f < FM; ++f) {
#pragma unroll
            for (int t = 0; t < kSkinnyGroup; ++t)
                d.ac[f][t] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(opa.codes, code_off + f * 16 * row_bytes,
                                                                                          (grp * kSkinnyGroup + t) * 64, 0));
            d.as[f] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(opa.scales, scale_off + f * 16 * scale_bytes, grp * 16, 0));
        }
    };

    // this wavefront's groups; the first one is requested before anything else happens
    const int per_wave = (ngroups + kSkinnyWaves - 1) / kSkinnyWaves;
    const int first = w * per_wave, last = min(first + per_wave, ngroups);
    Group d;
    if (first < last) load_group(d, first);

    // LDS: partial results [wave][fragment pair][lane] float4, then the sigma_A table [macro block][FM * 16]
    v4f* red = reinterpret_cast<v4f*>(smem);
    float* sig_a = reinterpret_cast<float*>(smem + kSkinnyWaves * FM * FN * kWave * 16);
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
#pragma unroll
        for (int t = 0; t < kSkinnyGroup; ++t) {
            v4f sm[FM];
#pragma unroll
            for (int f = 0; f < FM; ++f) {
                sm[f] = v4f{1.f, 1.f, 1.f, 1.f};
                if (sigma_a) sm[f] = *reinterpret_cast<const v4f*>(sig_a + (grp * kSkinnyGroup + t) * (FM * 16) + f * 16 + q * 4);
            }
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const uint32_t sw = (uint32_t)d.ws[j][t] >> (8 * q);  // the instruction reads byte 0
                // F = 1 + m8/256 is exact, the reciprocal within an ulp; m8 = 0 (also: no words) gives exactly 1
                const float sn = __builtin_amdgcn_rcpf(1.0f + (float)((d.wm8[j] >> (8 * t)) & 0xFFu) * (1.0f / 256.0f));
#pragma unroll
                for (int f = 0; f < FM; ++f) {
                    const uint32_t sa = (uint32_t)d.as[f][t] >> (8 * q);
                    const v4f zero = {0.f, 0.f, 0.f, 0.f};
                    const v4f p = mfma_fp4(d.ac[f][t], d.wc[j][t], zero, sa, sw);  // D[4 q + i][r]: m = 4 q + i, n = r
                    if (sigma_a || sigma_b) acc[f][j] += p * (sm[f] * sn);
                    else acc[f][j] += p;
                }
            }
        }
        if (grp + 1 < last) load_group(d, grp + 1);
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

template <int FM, int FN>
int launch_skinny_variant(const GemmArgs& g, hipStream_t s) {
    const int64_t blocks = (g.N + 16 * FN - 1) / (16 * FN);
    if (blocks > (int64_t)1 << 30) return MX_EINVAL;
    const size_t lds = (size_t)kSkinnyWaves * FM * FN * kWave * 16 + (g.a_mbs ? (size_t)(g.K / kMacro) * FM * 16 * 4 : 0);
    hipLaunchKernelGGL((gemm_skinny_kernel<FM, FN>), dim3((unsigned)blocks), dim3(kSkinnyThreads), lds, s, g);
    return launch_status();
}

// about one workgroup per compute unit; at most four fragment pairs each (32 KiB of partial results in LDS)
template <int FM>
int launch_skinny_columns(const GemmArgs& g, hipStream_t s) {
    const int64_t frags = (g.N + 15) / 16;
    if constexpr (FM == 1) {
        if (frags > 2 * 256) return launch_skinny_variant<1, 4>(g, s);
    }
    if constexpr (FM <= 2) {
        if (frags > 256) return launch_skinny_variant<FM, 2>(g, s);
    }
    return launch_skinny_variant<FM, 1>(g, s);
}

}  // namespace

// M <= 64, K % 512 == 0, K <= 8192, 16-byte aligned scale arrays, 4-byte aligned MBS arrays, not grouped; the
// caller has checked all of them.
int launch_gemm_skinny(const GemmArgs& g, bool use_mbs, hipStream_t s) {
    GemmArgs h = g;
    if (!use_mbs) h.a_mbs = h.b_mbs = nullptr;
    if (h.M <= 16) return launch_skinny_columns<1>(h, s);
    if (h.M <= 32) return launch_skinny_columns<2>(h, s);
    return launch_skinny_columns<4>(h, s);
}

}  // namespace mx
