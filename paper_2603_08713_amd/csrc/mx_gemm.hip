// Block-scaled MXFP4 GEMM  C = A * B^T  with the Macro Block Scaling correction, for gfx950: argument checks and
// the choice of kernel.  The kernels are the main template (mx_gemm_ring.h: fast form in mx_gemm_wide.hip and
// mx_gemm_mbs.hip, general forms in mx_gemm_general.hip and mx_gemm_wide.hip) and the few-row kernel
// (mx_gemm_skinny.hip).
#include "mx_gemm_shared.h"
#include "mx_internal.h"

#include <stdio.h>

namespace mx {
namespace {

// force_shape (mx_internal_gemm only; the public entry points pass -1 = automatic): 2 / 6 / 7 = fast form without
// MBS on 256x256 / 256x128 / 128x128 tiles, 3 / 4 = fast form with MBS on 256x128 / 128x128 tiles, 5 = few-row
// kernel, 8 / 9 = general form (2-byte pieces) on 256x128 / 128x128 tiles, 10 = general form (single bytes) on
// 128x128 tiles.
// Which kernel form and tile shape (the codes above) takes a problem.  Tiles run in rounds of one per compute
// unit: rounds x tile area / efficiency (the small tile reaches about 0.8 of the large tile's rate per output
// with MBS, 0.85 / 0.72 without; measured) picks the tile.
int choose_shape(int64_t M, int64_t N, bool use_mbs, bool ring_ok, bool pairs_ok, bool skinny_ok) {
    const int64_t t256x128 = ((M + 255) / 256) * ((N + 127) / 128), t128 = ((M + 127) / 128) * ((N + 127) / 128);
    const double big = 2.0 * ((t256x128 + 255) / 256) / (use_mbs ? 1.0 : 0.85),
                 small = ((t128 + 255) / 256) / (use_mbs ? 0.8 : 0.72);
    if (skinny_ok) return 5;
    if (ring_ok) return use_mbs ? (big <= small ? 3 : 4) : 2;  // (without MBS the launcher also has 256 x 256 tiles)
    if (pairs_ok) return big <= small ? 8 : 9;
    return 10;
}

int launch_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs, const uint8_t* b_codes,
                const uint8_t* b_scales, const uint8_t* b_mbs, int num_groups, const int64_t* row_offsets,
                bool grouped, int64_t M, int64_t N, int64_t K, int c_dtype, void* C, int64_t ldc, bool mbs_entry,
                void* stream, int force_shape = -1) {
    if (M < 0 || N < 0 || K < 0 || (K % kBlock) != 0 || ldc < N) return MX_EINVAL;
    if (c_dtype != MX_OUT_F32 && c_dtype != MX_OUT_BF16) return MX_EINVAL;
    if (grouped && num_groups < 0) return MX_EINVAL;
    // (a tile's rows times the bytes of a row must fit the 32-bit offsets of the buffer loads)
    if (K > (int64_t)1 << 22 || M > (int64_t)1 << 30 || N > (int64_t)1 << 30 ||
        (grouped && (int64_t)num_groups * N > (int64_t)1 << 40))
        return MX_EINVAL;
    if (M == 0 || N == 0 || (grouped && num_groups == 0)) return MX_OK;
    if (!C || (grouped && !row_offsets)) return MX_ENULL;
    if (K > 0 && (!a_codes || !a_scales || !b_codes || !b_scales)) return MX_ENULL;
    const size_t esz = c_dtype == MX_OUT_F32 ? 4 : 2;
    if (!aligned(C, esz) || (K > 0 && (!aligned(a_codes, 16) || !aligned(b_codes, 16)))) return MX_EALIGN;
    if (int st = check_device()) return st;

    GemmArgs g;
    g.a_codes = a_codes; g.a_scales = a_scales; g.a_mbs = a_mbs;
    g.b_codes = b_codes; g.b_scales = b_scales; g.b_mbs = b_mbs;
    g.C = C; g.row_offsets = row_offsets;
    g.M = M; g.N = N; g.K = K; g.ldc = ldc;
    g.num_groups = grouped ? num_groups : 0;
    g.tiles_m = g.tiles_n = 0;
    g.c_bf16 = c_dtype == MX_OUT_BF16;
    g.vec_store16 = aligned(C, 16) && (ldc * esz) % 16 == 0;
    g.vec_store8 = aligned(C, 8) && (ldc * esz) % 8 == 0;
    g.vec_store4 = aligned(C, 4) && (ldc * esz) % 4 == 0;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool use_mbs = mbs_entry && (a_mbs || b_mbs);
    // Fast form: K in whole groups of four macro blocks and aligned per-row arrays.
    const bool ring_ok = !grouped && K > 0 && (K % 512) == 0 && aligned(a_scales, 16) && aligned(b_scales, 16) &&
                         (!use_mbs || ((!a_mbs || aligned(a_mbs, 4)) && (!b_mbs || aligned(b_mbs, 4))));
    // General form with 2-byte pieces of E8M0 bytes: rows of them on even addresses; else single bytes.
    const bool pairs_ok = K > 0 && (K % 64) == 0 && aligned(a_scales, 2) && aligned(b_scales, 2);
    const bool skinny_ok = ring_ok && M <= 64 && K <= 8192;
    int shape = choose_shape(M, N, use_mbs, ring_ok, pairs_ok, skinny_ok);
    if (force_shape >= 0) shape = force_shape;
    // (the checks below only matter for forced shapes)
    if (shape == 5) return skinny_ok ? launch_gemm_skinny(g, use_mbs, s) : MX_EINVAL;
    if (shape == 8 || shape == 9) {
        if (!pairs_ok) return MX_EINVAL;
        return use_mbs ? launch_gemm_mbs_general(g, shape - 8, false, s) : launch_gemm_wide_general(g, shape - 8, false, s);
    }
    if (shape == 10) return use_mbs ? launch_gemm_mbs_general(g, 1, true, s) : launch_gemm_wide_general(g, 1, true, s);
    const bool plain_shape = shape == 2 || shape == 6 || shape == 7;
    if (shape < 2 || shape > 7 || !ring_ok || plain_shape == use_mbs) return MX_EINVAL;
    if (plain_shape) return launch_gemm_wide(g, force_shape < 0 ? 0 : shape == 2 ? 1 : shape == 6 ? 2 : 3, s);
    return launch_gemm_mbs_ring(g, shape == 4, s);
}

// Few-row GEMM with A given as bf16 and quantized inside the kernel (mx_gemm_skinny.hip).
int launch_gemm_quantize_a(const void* a_bf16, int64_t lda, int rule, int a_use_mbs, const uint8_t* b_codes,
                           const uint8_t* b_scales, const uint8_t* b_mbs, int64_t M, int64_t N, int64_t K, int c_dtype,
                           void* C, int64_t ldc, void* stream) {
    if (M < 0 || N < 0 || K < 0 || (K % kBlock) != 0 || ldc < N || lda < K) return MX_EINVAL;
    if (c_dtype != MX_OUT_F32 && c_dtype != MX_OUT_BF16) return MX_EINVAL;
    if (rule != MX_RULE_OCP && rule != MX_RULE_FLOOR && rule != MX_RULE_OAS) return MX_EINVAL;
    if (N > (int64_t)1 << 30) return MX_EINVAL;
    if (M == 0 || N == 0) return MX_OK;
    if (!C || !a_bf16 || !b_codes || !b_scales) return MX_ENULL;
    const size_t esz = c_dtype == MX_OUT_F32 ? 4 : 2;
    if (!aligned(C, esz) || !aligned(a_bf16, 16) || (lda % 8) != 0 || !aligned(b_codes, 16)) return MX_EALIGN;
    // what the few-row kernel covers; larger problems take mx_quantize_mbs + mx_gemm_mbs
    if (M > 64 || K == 0 || (K % 512) != 0 || K > 8192 || !aligned(b_scales, 16) || (b_mbs && !aligned(b_mbs, 4)) ||
        ((M - 1) * lda + K) * 2 >= (int64_t)1 << 31)
        return MX_EUNSUPPORTED;
    if (int st = check_device()) return st;
    GemmArgs g = {};
    g.b_codes = b_codes; g.b_scales = b_scales; g.b_mbs = b_mbs;
    g.C = C;
    g.M = M; g.N = N; g.K = K; g.ldc = ldc;
    g.c_bf16 = c_dtype == MX_OUT_BF16;
    return launch_gemm_skinny_fused(g, a_bf16, lda, rule, a_use_mbs != 0, static_cast<hipStream_t>(stream));
}

}  // namespace
}  // namespace mx

extern "C" {

int mx_gemm_mbs_quantize_a(const void* a_bf16, int64_t lda, mx_rule_t rule, int a_use_mbs, const uint8_t* b_codes,
                           const uint8_t* b_scales, const uint8_t* b_mbs_or_null, int64_t M, int64_t N, int64_t K,
                           mx_dtype_t c_dtype, void* C, int64_t ldc, void* stream) {
    return mx::launch_gemm_quantize_a(a_bf16, lda, (int)rule, a_use_mbs, b_codes, b_scales, b_mbs_or_null, M, N, K,
                                      (int)c_dtype, C, ldc, stream);
}

int mx_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes, const uint8_t* b_scales,
            int64_t M, int64_t N, int64_t K, mx_dtype_t c_dtype, void* C, int64_t ldc, void* stream) {
    return mx::launch_gemm(a_codes, a_scales, nullptr, b_codes, b_scales, nullptr, 0, nullptr, false, M, N, K,
                           (int)c_dtype, C, ldc, false, stream);
}

int mx_gemm_mbs(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs_or_null,
                const uint8_t* b_codes, const uint8_t* b_scales, const uint8_t* b_mbs_or_null, int64_t M, int64_t N,
                int64_t K, mx_dtype_t c_dtype, void* C, int64_t ldc, void* stream) {
    return mx::launch_gemm(a_codes, a_scales, a_mbs_or_null, b_codes, b_scales, b_mbs_or_null, 0, nullptr, false, M,
                           N, K, (int)c_dtype, C, ldc, true, stream);
}

int mx_gemm_mbs_grouped(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs_or_null,
                        const uint8_t* b_codes, const uint8_t* b_scales, const uint8_t* b_mbs_or_null,
                        int32_t num_groups, const int64_t* row_offsets, int64_t M_total, int64_t N, int64_t K,
                        mx_dtype_t c_dtype, void* C, int64_t ldc, void* stream) {
    return mx::launch_gemm(a_codes, a_scales, a_mbs_or_null, b_codes, b_scales, b_mbs_or_null, num_groups,
                           row_offsets, true, M_total, N, K, (int)c_dtype, C, ldc, true, stream);
}

int mx_internal_gemm_plan(int64_t M, int64_t N, int64_t K, int a_has_mbs, int b_has_mbs, int grouped, char* out, int cap) {
    if (!out || cap <= 0 || M < 0 || N < 0 || K < 0 || (K % mx::kBlock) != 0) return MX_EINVAL;
    const bool use_mbs = a_has_mbs || b_has_mbs;
    const bool ring_ok = !grouped && K > 0 && (K % 512) == 0, pairs_ok = K > 0 && (K % 64) == 0;
    const int shape = mx::choose_shape(M, N, use_mbs, ring_ok, pairs_ok, ring_ok && M <= 64 && K <= 8192);
    const char* sides = a_has_mbs && b_has_mbs ? "MBS words on A and B" : a_has_mbs ? "MBS words on A" : b_has_mbs ? "MBS words on B" : "no MBS";
    const char* what;
    switch (shape) {
        case 2: what = mx::describe_gemm_wide(M, N); break;
        case 3: what = a_has_mbs && b_has_mbs ? "gemm_ring_kernel, fast form, 256x128 tile, 8 wavefronts of 64x64"
                                              : "gemm_ring_kernel, fast form, 256x128 tile, 8 wavefronts of 128x32"; break;
        case 4: what = "gemm_ring_kernel, fast form, 128x128 tile, 8 wavefronts of 64x32"; break;
        case 5: what = "gemm_skinny_kernel (few rows)"; break;
        case 8: what = use_mbs ? "gemm_ring_kernel, general form (2-byte scale pieces), 256x128 tile, 8 wavefronts" : "gemm_ring_kernel, general form (2-byte scale pieces), 256x128 tile, 4 wavefronts"; break;
        case 9: what = "gemm_ring_kernel, general form (2-byte scale pieces), 128x128 tile"; break;
        default: what = "gemm_ring_kernel, general form (single scale bytes), 128x128 tile"; break;
    }
    snprintf(out, (size_t)cap, "%s; %s", what, sides);
    return MX_OK;
}

int mx_internal_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs_or_null,
                     const uint8_t* b_codes, const uint8_t* b_scales, const uint8_t* b_mbs_or_null, int grouped,
                     int32_t num_groups, const int64_t* row_offsets, int64_t M, int64_t N, int64_t K, mx_dtype_t c_dtype,
                     void* C, int64_t ldc, int mbs_entry, int force_shape, void* stream) {
    return mx::launch_gemm(a_codes, a_scales, a_mbs_or_null, b_codes, b_scales, b_mbs_or_null, num_groups, row_offsets,
                           grouped != 0, M, N, K, (int)c_dtype, C, ldc, mbs_entry != 0, stream, force_shape);
}

}  // extern "C"
