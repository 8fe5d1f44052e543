/*
 * mx4.h -- C ABI of the MI355X (gfx950) library for MXFP4 quantization with Overflow-Aware
 * Scaling (OAS) and static Macro Block Scaling (MBS-S), and the block-scaled GEMM that consumes
 * those operands and applies the MBS correction in its fp32 accumulation.  The same for the 8-bit
 * MX element formats (MXFP8) through the *_elem entry points at the end.
 *
 * Conventions common to every entry point
 *   - Every pointer argument is a DEVICE pointer owned by the caller (the library never allocates,
 *     frees or keeps them), except `stream`, which is a hipStream_t passed as void* (NULL = the
 *     default stream).
 *   - Calls are asynchronous on `stream`, never synchronise with the host, and return an int:
 *     MX_OK, or a negative error code, in which case nothing was launched.
 *   - Arguments are checked before the GPU is touched, so argument errors are reported even
 *     without a GPU.  A call with zero rows / M / N is a valid no-op.
 *   - Quantization always runs along K, the contraction dimension, for both GEMM operands
 *     (A is [M,K], B is [N,K], the product is C = A * B^T; Sec. 4.3.2).
 *
 * Canonical layouts (row-major, the surface on which bit-exactness is judged)
 *   codes   uint8 [rows, K/2]        two E2M1 codes per byte, element 2j in the low nibble;
 *                                    code = sign<<3 | index into {0,.5,1,1.5,2,3,4,6} (Sec. 2.2)
 *   scales  uint8 [rows, K/32]       E8M0, bias 127: the de-quantization scale 2^(E-127) shared
 *                                    by 32 elements (Sec. 2.2); 255 = NaN (non-finite input block)
 *   mbs     uint8 [rows, ceil(K/128)] the 8 stored mantissa bits m8 of the macro-block factor
 *                                    F = 1 + m8/256 in [1,2), one per 1x128 window (Sec. 4.3.1)
 *   x       bf16  [rows, ldx]        input, K <= ldx (elements)
 * A value is reconstructed as  x_hat = value(code) * 2^(E-127) / F   (Sec. 4.3.1).
 *
 * Alignment: x must be 16-byte aligned and ldx a multiple of 8; codes must be 16-byte aligned;
 * scales, mbs: no requirement.  C must be aligned to its element size.
 */
#ifndef MX4_H
#define MX4_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define MX_OK 0
#define MX_EINVAL (-1)        /* negative size, K % 32 != 0, ld < K (or < N), bad enum value      */
#define MX_ENULL (-2)         /* a required pointer is NULL                                       */
#define MX_EALIGN (-3)        /* pointer or leading dimension violates the alignment above        */
#define MX_EUNSUPPORTED (-4)  /* no HIP device, device is not gfx950, or a shape the entry point does not cover */
#define MX_ELAUNCH (-5)       /* the HIP runtime rejected the launch                              */

/* Rule that picks the power-of-two scale of a 32-element block from its absmax (Sec. 4.2). */
typedef enum {
    MX_RULE_OCP = 0,   /* MXFP4-OCP: shared exponent floor(log2 absmax) - 2, absmax -> [4, 8)      */
    MX_RULE_FLOOR = 1, /* "standard": 6/absmax with the mantissa masked off, absmax -> (3, 6]      */
    MX_RULE_OAS = 2    /* Overflow-Aware Scaling: FLOOR, doubled when absmax lands in (3, 3.5],
                          absmax -> (3.5, 7]                                                       */
} mx_rule_t;

typedef enum { MX_OUT_F32 = 0, MX_OUT_BF16 = 1 } mx_dtype_t;

/* Plain MXFP4 quantization of `rows` rows of K bf16 values with the given scale rule, no MBS
 * (Sec. 2.2 for the format, Sec. 4.2 for the rules).  Elements round to the nearest E2M1 value,
 * ties to the even code, saturating at +-6; the sign bit is copied from the input, also for
 * values that round to zero.  An all-zero block stores E = 127.  A block holding Inf/NaN stores
 * E = 255 and zero codes.  Writes codes [rows,K/2] and scales [rows,K/32]. */
int mx_quantize(const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule,
                uint8_t* codes, uint8_t* scales, void* stream);

/* mx_quantize with MX_RULE_OAS (Sec. 4.2). */
int mx_quantize_oas(const void* x_bf16, int64_t rows, int64_t K, int64_t ldx,
                    uint8_t* codes, uint8_t* scales, void* stream);

/* MBS-Static quantization (Sec. 4.3.1, Eq. 3; Sec. 5.3): per 1x128 window, m8 = the 8 leading
 * mantissa bits of 6/absmax128; every element of the window is multiplied by F = 1 + m8/256 and
 * each 32-element block is then quantized as in mx_quantize with `rule` (MX_RULE_OAS is the
 * paper's MBS-S) on its scaled absmax.  A last window shorter than 128 uses the elements that
 * exist.  Additionally writes mbs [rows, ceil(K/128)].  Non-finite elements are ignored when the
 * window absmax is taken. */
int mx_quantize_mbs(const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule,
                    uint8_t* codes, uint8_t* scales, uint8_t* mbs, void* stream);

/* mx_quantize_mbs for two tensors that share K -- the two operands of one GEMM (Sec. 4.3.2: both A and
 * B carry MBS words) -- in a single launch; outputs identical to two mx_quantize_mbs calls.  Either
 * tensor may have zero rows. */
int mx_quantize_mbs_pair(const void* x0_bf16, int64_t rows0, int64_t ldx0,
                         uint8_t* codes0, uint8_t* scales0, uint8_t* mbs0,
                         const void* x1_bf16, int64_t rows1, int64_t ldx1,
                         uint8_t* codes1, uint8_t* scales1, uint8_t* mbs1,
                         int64_t K, mx_rule_t rule, void* stream);

/* MBS-Dynamic quantization (Sec. 4.3.3, Sec. 5.3; meant for weights, which are quantized
 * offline: MBS-Hybrid = this for B, mx_quantize_mbs for A): as mx_quantize_mbs, but the word of each
 * window is searched for the least sum of squared errors of the window among the static word and
 *     m_j = (m_static + (cand_first + j) * cand_stride) mod 256,   j = 0 .. cand_count-1
 * (the paper searches 16 candidates and does not list them; cand_first 0, cand_count 16,
 * cand_stride 16 spaces them equally over all factors).  0 <= cand_count <= 256, |cand_first| and
 * |cand_stride| <= 65536, else MX_EINVAL.  The sum of squared errors is evaluated in fp32 in a fixed
 * order of operations, so the result is deterministic; ties keep the static word, then the lowest j.
 * Windows holding Inf/NaN, and windows whose absmax is below 2^-63 or at least 2^123, keep the static
 * word.  Outputs as mx_quantize_mbs; mx_gemm_mbs consumes them unchanged. */
int mx_quantize_mbs_dynamic(const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule,
                            int32_t cand_first, int32_t cand_count, int32_t cand_stride,
                            uint8_t* codes, uint8_t* scales, uint8_t* mbs, void* stream);

/* The table MBS-Dynamic reads in the paper (Sec. 4.3.3, Eq. 5): squared relative errors
 * T[v, m_j] ~ ((x_hat - x) / x)^2 of an element whose magnitude in its block's scaled domain is v = |x| SF, under
 * candidate word m_j.  Two tables of 64 points x 16 slots in fp16 (the paper gives this shape, not the contents);
 * here slot j is the word 16 j (factor 1 + j/16); the "normal" table (v >= 1) is indexed by the 6 leading
 * mantissa bits of v, the "sub-normal" one (v < 1) by floor(64 v); an entry is the squared relative error at the
 * middle of its bin, computed in fp64 and rounded once to fp16.  Writes lut_fp16[(table * 64 + p) * 16 + j]
 * (2048 fp16 bit patterns = 4096 bytes, DEVICE memory, 16-byte aligned; table 0 = sub-normal). */
int mx_mbs_lut_build(uint16_t* lut_fp16, void* stream);

/* MBS-Dynamic quantization through that table (Sec. 4.3.3, Eq. 4-6): per 1x128 window the candidate j* of least
 * sum_i x_i^2 T[v_ij, j] (Eq. 6; v_ij taken with the local scale the rule derives from the block's absmax times
 * 1 + j/16; sums in fp32; ties to the lowest j) gives the word 16 j*.  With keep_static != 0 the static word of
 * Eq. 3 is kept instead whenever its own sum of squared errors, evaluated directly, is not larger than that of
 * the picked word, so that no window comes out worse than with mx_quantize_mbs (not in the paper: the table has
 * no slot for the static word).  lut_fp16: the table in the layout above (mx_mbs_lut_build fills it; a caller
 * may pass its own), DEVICE memory, 16-byte aligned, read during the call.  Windows holding Inf/NaN, and windows
 * whose absmax is below 2^-63 or at least 2^123, keep the static word.  Outputs as mx_quantize_mbs. */
int mx_quantize_mbs_dynamic_lut(const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule,
                                const uint16_t* lut_fp16, int keep_static,
                                uint8_t* codes, uint8_t* scales, uint8_t* mbs, void* stream);

/* mx_quantize_mbs_dynamic_lut for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid it) and so have no buffer to hand in for the table: the table lives in
 * a 4 KiB array inside the library's code object, one copy per GPU, held until the process ends.  The array's
 * size does not depend on the input, so the limits on rows and K are those of mx_quantize_mbs_dynamic_lut and
 * are reported the same way (MX_EINVAL and the other codes, before anything is launched).  The call allocates
 * nothing: it writes the whole table on `stream` (the kernel of mx_mbs_lut_build, so its contents are those
 * bits) and then runs the kernel of mx_quantize_mbs_dynamic_lut on it; outputs are bit-identical to that entry
 * point given a table from mx_mbs_lut_build.  All calls on one GPU share that GPU's array: calls that overlap on
 * one GPU (different streams, or threads) race on it, though every writer stores the same values.  The array's
 * address on a device is looked up by the first call on that device that has work to do (rows > 0 and K > 0); a
 * caller that captures graphs makes that first call before the capture begins.
 * x, codes, scales, mbs: DEVICE memory of the caller, as for mx_quantize_mbs. */
int mx_quantize_mbs_dynamic_lut_static(const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule,
                                       int keep_static,
                                       uint8_t* codes, uint8_t* scales, uint8_t* mbs, void* stream);

/* Reconstruct x_hat = value(code) * 2^(E-127) / F (Sec. 4.3.1) into out [rows, ldo] of
 * `out_dtype` (fp32: correctly rounded; bf16: that fp32 value rounded to nearest even).
 * mbs_or_null == NULL means F = 1.  E = 255 gives NaN. */
int mx_dequantize(const uint8_t* codes, const uint8_t* scales, const uint8_t* mbs_or_null,
                  int64_t rows, int64_t K, mx_dtype_t out_dtype, void* out, int64_t ldo,
                  void* stream);

/* Plain MXFP4 GEMM, C[M,N] = A[M,K] * B[N,K]^T with A, B given as codes + E8M0 scales
 * (the baseline the MBS kernel is measured against, Sec. 5.3 / Tab. 4).  fp32 accumulation on the
 * block-scaled MFMA; C is written as c_dtype with leading dimension ldc >= N (elements).
 * Limits (all GEMM entry points): K <= 2^22, M and N <= 2^30, else MX_EINVAL. */
int mx_gemm(const uint8_t* a_codes, const uint8_t* a_scales,
            const uint8_t* b_codes, const uint8_t* b_scales,
            int64_t M, int64_t N, int64_t K, mx_dtype_t c_dtype, void* C, int64_t ldc,
            void* stream);

/* GEMM with the MBS correction (Sec. 4.3.2, App. E): for every 128-deep macro block g the
 * block-scaled partial product P_g is multiplied by sigma_A[i,g] * sigma_B[j,g], sigma = 1/F, and
 * accumulated in fp32:  C[i,j] = sum_g P_g[i,j] * sigma_A[i,g] * sigma_B[j,g].
 * a_mbs_or_null / b_mbs_or_null == NULL means that operand carries no MBS words (sigma = 1). */
int mx_gemm_mbs(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs_or_null,
                const uint8_t* b_codes, const uint8_t* b_scales, const uint8_t* b_mbs_or_null,
                int64_t M, int64_t N, int64_t K, mx_dtype_t c_dtype, void* C, int64_t ldc,
                void* stream);

/* Few-row (decode) form with the activations quantized inside the GEMM kernel (Sec. 4.3, Sec. 5.3): C = Q(A) * B^T where Q is mx_quantize_mbs(rule) if a_use_mbs != 0,
 * else mx_quantize(rule), applied inside the GEMM kernel to a_bf16 [M, lda] (bf16, row-major, 16-byte
 * aligned, lda % 8 == 0, lda >= K); the quantized activations are never written to memory.  The result
 * is bit-identical to mx_quantize_mbs / mx_quantize followed by mx_gemm_mbs on the same weights.
 * Covers M <= 64, K % 512 == 0, 0 < K <= 8192, b_scales 16-byte aligned, b_mbs 4-byte aligned; anything
 * else returns MX_EUNSUPPORTED and nothing is launched (use the two calls). */
int mx_gemm_mbs_quantize_a(const void* a_bf16, int64_t lda, mx_rule_t rule, int a_use_mbs,
                           const uint8_t* b_codes, const uint8_t* b_scales, const uint8_t* b_mbs_or_null,
                           int64_t M, int64_t N, int64_t K, mx_dtype_t c_dtype, void* C, int64_t ldc,
                           void* stream);

/* Grouped (mixture-of-experts) form of mx_gemm_mbs (Sec. 5.1: every expert's linear layers are
 * quantized): the rows of A and C are grouped, group e owning rows
 * row_offsets[e] .. row_offsets[e+1]-1 (row_offsets: DEVICE int64 [num_groups+1], non-decreasing,
 * row_offsets[0] = 0, row_offsets[num_groups] <= M_total), and is multiplied with its own weight
 * B_e [N,K]; the b_* arrays hold the num_groups weights stacked along rows ([num_groups*N, ...]).
 * Empty groups are allowed.  Rows of C at or beyond row_offsets[num_groups] are not written. */
int mx_gemm_mbs_grouped(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs_or_null,
                        const uint8_t* b_codes, const uint8_t* b_scales, const uint8_t* b_mbs_or_null,
                        int32_t num_groups, const int64_t* row_offsets,
                        int64_t M_total, int64_t N, int64_t K, mx_dtype_t c_dtype, void* C,
                        int64_t ldc, void* stream);

/* ---- the 8-bit and 6-bit MX element formats (Sec. 1, footnote: the methods carry over to MXFP6 / MXFP8) ----
 * The paper works MXFP4 through and only states that OAS and MBS generalise; these entry points restate
 * each rule with the element format's own constants in place of E2M1's 6 and 1: V, its largest finite
 * magnitude, and h, half the spacing of its top binade.
 *   MX_RULE_FLOOR  block absmax -> (V/2, V]            MX_RULE_OCP  shared exponent floor(log2 absmax) - emax
 *   MX_RULE_OAS    FLOOR, doubled when the absmax lands at or below (V + h)/2: absmax -> ((V + h)/2, V + h]
 *   MBS-Static     m8 = the 8 leading mantissa bits of V / (absmax of the 1x128 window)
 * Elements round to the nearest value of the format, ties to the even code, saturating at +-V; the sign
 * bit is copied.  Formats as in the OCP MX specification: E4M3 (S.EEEE.MMM, bias 7, V = 448, h = 16), E5M2
 * (S.EEEEE.MM, bias 15, V = 57344, h = 4096), E2M3 (S.EE.MMM, bias 1, V = 7.5, h = 0.25), E3M2 (S.EEE.MM, bias 3,
 * V = 28, h = 2).  Layout of the codes: 8-bit formats uint8 [rows, K], one element per byte; 6-bit formats
 * uint8 [rows, 3K/4], packed: element k of a row occupies bits 6k .. 6k+5 of the row's bytes taken as one
 * little-endian number (a 32-element block is 24 bytes).  Scales and mbs as for MXFP4.  MX_ELEM_E2M1 names the
 * 4-bit format of the other entry points and is not accepted here. */
typedef enum {
    MX_ELEM_E2M1 = 0,
    MX_ELEM_E4M3 = 1,
    MX_ELEM_E5M2 = 2,
    MX_ELEM_E2M3 = 3,
    MX_ELEM_E3M2 = 4
} mx_elem_t;

/* mx_quantize (use_mbs = 0, mbs ignored) or mx_quantize_mbs (use_mbs != 0) into an 8-bit or 6-bit element
 * format.  Alignment: x 16 bytes and ldx a multiple of 8, codes 8 bytes.  K % 32 == 0. */
int mx_quantize_elem(mx_elem_t elem, const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule,
                     int use_mbs, uint8_t* codes, uint8_t* scales, uint8_t* mbs, void* stream);

/* mx_quantize_mbs_dynamic into an 8-bit or 6-bit element format (Sec. 4.3.3, Sec. 5.3; Sec. 1, footnote): as
 * mx_quantize_elem with use_mbs != 0, but the word of each 1x128 window is searched for the least sum of squared
 * errors of the window among the static word and  m_j = (m_static + (cand_first + j) * cand_stride) mod 256,
 * j = 0 .. cand_count-1.  Candidate limits, evaluation order (fp32, fixed), tie rule (the static word, then the
 * lowest j) and the windows that keep the static word (Inf/NaN inside, absmax below 2^-63 or at least 2^123) as for
 * mx_quantize_mbs_dynamic; alignment as for mx_quantize_elem.  mx_gemm_mbs_elem consumes the outputs unchanged. */
int mx_quantize_elem_mbs_dynamic(mx_elem_t elem, const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule,
                                 int32_t cand_first, int32_t cand_count, int32_t cand_stride,
                                 uint8_t* codes, uint8_t* scales, uint8_t* mbs, void* stream);

/* mx_dequantize for an 8-bit or 6-bit element format: out[r, k] = value(code) * 2^(E-127) / F, F = 1 without MBS
 * words (Sec. 4.3.1).  The fp32 result is the quotient evaluated in fp64 and rounded once more; the bf16 result is
 * that fp32 value rounded to nearest even; a block with E = 255 gives NaN.  Codes in the layout mx_quantize_elem
 * writes (6-bit: packed, [rows, 3K/4]).  Alignment: codes 8 bytes, out its element size; ldo >= K in elements. */
int mx_dequantize_elem(mx_elem_t elem, const uint8_t* codes, const uint8_t* scales, const uint8_t* mbs_or_null,
                       int64_t rows, int64_t K, mx_dtype_t out_dtype, void* out, int64_t ldo, void* stream);

/* mx_gemm_mbs for operands in 8-bit or in 6-bit element formats (A's and B's may differ, but both are 8-bit or
 * both 6-bit): the same sum, the same MBS correction per 128 K-elements (Sec. 4.3.2, which does not depend on
 * the element format), on the same scaled matrix instruction.  Covers K >= 128 in whole macro blocks or ending
 * with half of one (K % 64 == 0; the short last macro block of Sec. 4.3.1's windows, as for the MXFP4 entry
 * points), codes 16-byte aligned, scale arrays 4-byte aligned (2-byte where K % 128 == 64); anything else
 * returns MX_EUNSUPPORTED and nothing is launched.  (K % 512 == 0,
 * 16-byte aligned scale arrays and 4-byte aligned MBS arrays take a faster form of the kernel; with M <= 64 and
 * K <= 8192 besides, a kernel that streams the weights once.)
 *
 * Accumulation contract.  The exact result is  C[m, n] = sum over macro blocks g of sigma_A[m, g] sigma_B[n, g]
 * P_g[m, n],  P_g = the sum over the 128 K-elements of g of the products of the dequantized elements.  What is
 * guaranteed about the computed C:
 *   (1) operands produced by mx_quantize_elem from finite tensors (any rule, with or without MBS words), and more
 *       generally operands in which the 16 products of every aligned group of 16 K-elements lie within 2^13 of
 *       the group's largest one in magnitude, or are zero:  |C - exact| <= 1e-3 * RMS(exact)  over the output, the
 *       bound of the MXFP4 entry points.  (A block's elements share their scale, so within a group the products
 *       of E2M1, E2M3 and of quantized E4M3 / E5M2 / E3M2 data stay inside that window.)
 *   (2) any codes and scale bytes (no block with E = 255):  |C[m, n] - exact[m, n]| <= 2^-11 * sum_k |a_mk| |b_nk|
 *       per output, with a, b the dequantized operands.  The matrix instruction adds the 16 products of such a
 *       group after aligning them to the group's largest exponent and cuts them off about 13 bits below it;
 *       groups, blocks and macro blocks are then added in fp32.  Codes spread uniformly over an 8-bit format's
 *       whole range under widely spread scale bytes reach 3e-3 * RMS: they are inside (2), outside (1).
 *   (3) sums whose products need no alignment (all products of a group equal in exponent, or exact in 13 bits
 *       below the largest) are exact up to the fp32 additions across groups.
 * The fp32 output carries the accumulated value; the bf16 output is that value rounded to nearest even. */
int mx_gemm_mbs_elem(mx_elem_t a_elem, const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs_or_null,
                     mx_elem_t b_elem, const uint8_t* b_codes, const uint8_t* b_scales, const uint8_t* b_mbs_or_null,
                     int64_t M, int64_t N, int64_t K, mx_dtype_t c_dtype, void* C, int64_t ldc, void* stream);

/* mx_gemm_mbs_grouped for operands in 8-bit or in 6-bit element formats (Sec. 5.3, the MoE case; formats,
 * conditions on K and alignment, and the accumulation contract as for mx_gemm_mbs_elem): group e owns rows
 * row_offsets[e] .. row_offsets[e+1]-1 of A and C (row_offsets: DEVICE int64 [num_groups+1], non-decreasing,
 * row_offsets[0] = 0, row_offsets[num_groups] <= M_total; empty groups are allowed) and is multiplied with the
 * e-th of the num_groups [N, K] weights stacked along rows in b_*.  Rows of C at or beyond
 * row_offsets[num_groups] are not written. */
int mx_gemm_mbs_elem_grouped(mx_elem_t a_elem, const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs_or_null,
                             mx_elem_t b_elem, const uint8_t* b_codes, const uint8_t* b_scales, const uint8_t* b_mbs_or_null,
                             int32_t num_groups, const int64_t* row_offsets, int64_t M_total, int64_t N, int64_t K,
                             mx_dtype_t c_dtype, void* C, int64_t ldc, void* stream);

/* Human-readable text for a status code (static storage, host pointer). */
const char* mx_status_string(int status);

/* Library version, major*10000 + minor*100 + patch. */
int mx_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MX4_H */
