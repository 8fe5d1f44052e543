/*
 * mx_oracle.c -- CPU oracle for MXFP4 quantization with Overflow-Aware Scaling (OAS) and
 * Macro Block Scaling (static, MBS-S, and searched, MBS-D), and for the block-scaled GEMM with the
 * MBS correction.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, step-by-step restatement of what the
 * paper defines; only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 * It shares no code, table or constant generator with the HIP library, and the HIP library never
 * calls it.  Nothing here is blocked, fused, vectorised by hand or reordered: each function
 * follows the passage it cites so that it can be checked against the paper by eye.  The only
 * concession to run time is an OpenMP "parallel for" over independent rows.
 *
 * Arithmetic: every real number is a C double.  bf16 inputs, the MBS factor (9 significant
 * bits), their product (17 bits) and any power-of-two multiple of it are exact in a double, so
 * codes, scales and MBS words are decided on exact values; there is no rounding anywhere before
 * the final "nearest E2M1 value" decision.  GEMM and QSNR sums, and the sum of squared errors that
 * MBS-Dynamic minimises, are fp64.
 *
 * Conventions (paper silent; fixed here and used by the tests):
 *   - E2M1 code = sign<<3 | magnitude index into {0, .5, 1, 1.5, 2, 3, 4, 6}   (Sec. 2.2, 3.2)
 *   - two codes per byte, element 2j in the low nibble
 *   - the scale byte E is E8M0 with bias 127 and holds the DE-quantization scale 2^(E-127);
 *     the paper's multiplicative SF (Sec. 4.2) is its reciprocal, SF = 2^s with s = 127 - E
 *   - the MBS word m8 is the 8 stored mantissa bits; factor F = 1 + m8/256 in [1,2) (Sec. 4.3.1)
 *   - parity status: every exported function is pinned by tests/test_oracle_pins.py; the functions
 *     for the other MX element formats (mxo_elem_*, last section) by tests/test_oracle_elem_pins.py
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

#define MXO_RULE_OCP 0   /* MXFP4-OCP rule: absmax -> [4, 8)            (Sec. 4.2, last paragraph) */
#define MXO_RULE_FLOOR 1 /* "standard" no-overflow rule: absmax -> (3, 6] (Sec. 4.2, first paragraph) */
#define MXO_RULE_OAS 2   /* Overflow-Aware Scaling: absmax -> (3.5, 7]    (Sec. 4.2)                  */

static const double E2M1_VALUE[8] = {0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0};

/* ---- number formats (Sec. 2.2) ------------------------------------------------------------- */

/* bf16 is the upper half of an IEEE binary32. */
double mxo_bf16_value(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Value of a 4-bit E2M1 code. */
double mxo_e2m1_decode(int code) {
    double v = E2M1_VALUE[code & 7];
    return (code & 8) ? -v : v;
}

/* Magnitude index (0..7) of the E2M1 value nearest to y >= 0.  Beyond 6 the format saturates
 * (Sec. 4.2: "saturation since the format limit is 6.0").  A value exactly half-way between two
 * neighbours goes to the neighbour whose mantissa bit (= low bit of the index) is 0. */
int mxo_e2m1_nearest(double y) {
    if (y >= 6.0) return 7; /* saturation; also keeps the distances below exact for huge y */
    int best = 0;
    double best_d = fabs(y - E2M1_VALUE[0]);
    for (int c = 1; c < 8; ++c) {
        double d = fabs(y - E2M1_VALUE[c]);
        if (d < best_d || (d == best_d && (c & 1) == 0)) {
            best = c;
            best_d = d;
        }
    }
    return best;
}

/* ---- MBS-Static factor (Sec. 4.3.1, Eq. 3) -------------------------------------------------- */

/* Write 6/alpha = 2^e * (1 + m), 0 <= m < 1, and return the 8 leading bits of m, floor(256 m).
 * Eq. 3 takes these bits out of the fp32 pattern of the quotient; here the quotient is the exact
 * rational, so the result does not depend on how a division would round, and alpha may be so
 * small or so large that the fp32 quotient would overflow or go subnormal.  alpha = 0 -> 0. */
int mxo_mbs_static_m8(double alpha) {
    if (!(alpha > 0.0) || isinf(alpha)) return 0;
    int ex;
    double fr = frexp(alpha, &ex);                 /* alpha = fr * 2^ex, fr in [0.5, 1)          */
    uint64_t n = (uint64_t)ldexp(fr, 53);          /* fr = n / 2^53 exactly                       */
    /* 6/fr lies in (6, 12].  If it is >= 8 the normalised quotient 1+m is (6/fr)/8 = 0.75/fr,
     * otherwise it is (6/fr)/4 = 1.5/fr.  floor(256 * (1+m)) by exact integer division.         */
    unsigned __int128 num;
    if (fr <= 0.75)
        num = (unsigned __int128)192 << 53;        /* 256 * 0.75 / fr = 192 * 2^53 / n            */
    else
        num = (unsigned __int128)384 << 53;        /* 256 * 1.5  / fr = 384 * 2^53 / n            */
    uint64_t q = (uint64_t)(num / n);              /* in [256, 512)                               */
    return (int)q - 256;
}

/* ---- local power-of-two scale (Sec. 4.2) ---------------------------------------------------- */

/* Exponent s of the multiplicative scale SF = 2^s chosen for a block whose (MBS-scaled) absmax
 * is alpha > 0.
 *   FLOOR: SF = 6/alpha with the mantissa masked off, i.e. 2^floor(log2(6/alpha)); the scaled
 *          absmax falls in (3, 6].
 *   OAS:   start from FLOOR; if the scaled absmax is not above 3.5, double SF, which moves
 *          (3, 3.5] to (6, 7] and leaves the rest: scaled absmax in (3.5, 7].
 *   OCP:   the OCP rule, shared exponent floor(log2(alpha)) - 2 (2 = exponent of the largest
 *          E2M1 binade); scaled absmax in [4, 8).
 * Readings: the paper writes the OAS trigger as "[3, 3.5]"; FLOOR never produces exactly 3 and the
 * stated OAS image "(3.5, 7]" needs 3.5 -> 7, so the trigger is (3, 3.5], 3.5 included.       */
int mxo_scale_exponent(double alpha, int rule) {
    int ex;
    double fr = frexp(alpha, &ex); /* alpha = fr * 2^ex, fr in [0.5,1) => floor(log2 alpha) = ex-1 */
    if (rule == MXO_RULE_OCP) return 2 - (ex - 1);
    /* 6/alpha = (6/fr) * 2^-ex with 6/fr in (6, 12]: its floor(log2) is 3-ex when 6/fr >= 8,
     * i.e. when fr <= 0.75 (compared on fr so that no division has to round), else 2-ex.        */
    int s = (fr <= 0.75) ? 3 - ex : 2 - ex;
    if (rule == MXO_RULE_OAS) {
        double scaled_max = ldexp(alpha, s);     /* exact                                        */
        if (scaled_max <= 3.5) s += 1;
    }
    return s;
}

/* Stored E8M0 byte for multiplicative exponent s: E = 127 - s limited to the finite codes
 * [0, 254]; 255 is the format's NaN and is only produced for blocks with non-finite input.    */
int mxo_e8m0_from_exponent(int s) {
    int E = 127 - s;
    if (E < 0) E = 0;
    if (E > 254) E = 254;
    return E;
}

/* ---- quantizer (Sec. 4.2, 4.3.1, 5.3 first paragraph) --------------------------------------- */

static int is_finite_bf16(uint16_t h) { return (h & 0x7F80u) != 0x7F80u; }

/* One macro block of one row, elements [k0, k1): multiply by F = 1 + m8/256, then quantize each
 * sub-block with the chosen rule on its scaled absmax (Sec. 4.3.1; Sec. 5.3: "scale each alpha_i by
 * (1+m8) to obtain ... SF_i").  A sub-block holding a non-finite value gets E = 255 and zero codes.
 * cr / sr are the row's code and scale arrays. */
static void quantize_macro_block(const uint16_t* xr, int64_t k0, int64_t k1, int m8, int rule,
                                 int block, uint8_t* cr, uint8_t* sr) {
    const double F = 1.0 + m8 / 256.0;
    for (int64_t b0 = k0; b0 < k1; b0 += block) {
        int finite = 1;
        double amax = 0.0;
        for (int64_t k = b0; k < b0 + block; ++k) {
            if (!is_finite_bf16(xr[k])) finite = 0;
            else amax = fmax(amax, fabs(mxo_bf16_value(xr[k]) * F));
        }
        int E, s;
        if (!finite) { E = 255; s = 0; }
        else if (amax == 0.0) { E = 127; s = 0; }
        else { E = mxo_e8m0_from_exponent(mxo_scale_exponent(amax, rule)); s = 127 - E; }
        sr[b0 / block] = (uint8_t)E;
        for (int64_t k = b0; k < b0 + block; ++k) {
            int code = 0;
            if (finite) {
                double t = ldexp(mxo_bf16_value(xr[k]) * F, s); /* x * F * SF, exact */
                code = mxo_e2m1_nearest(fabs(t)) | ((xr[k] & 0x8000u) ? 8 : 0);
            }
            if (k & 1) cr[k / 2] = (uint8_t)((cr[k / 2] & 0x0F) | (code << 4));
            else       cr[k / 2] = (uint8_t)code;
        }
    }
}

/* Absmax of the finite elements [k0, k1) of a row (Sec. 4.3.1: alpha_max^128). */
static double macro_absmax(const uint16_t* xr, int64_t k0, int64_t k1) {
    double a128 = 0.0;
    for (int64_t k = k0; k < k1; ++k)
        if (is_finite_bf16(xr[k])) a128 = fmax(a128, fabs(mxo_bf16_value(xr[k])));
    return a128;
}

/* Quantize rows of bf16 along K.
 *   x      [rows, ldx] bf16 bit patterns, row-major, K <= ldx
 *   rule   MXO_RULE_*;  use_mbs 0/1;  block = elements per E8M0 scale (32; 16 = the paper's
 *   "MXFP4-16"); macro = elements per MBS word (128), a multiple of block
 *   codes  [rows, K/2]          scales [rows, K/block]       mbs [rows, ceil(K/macro)] (use_mbs)
 * Per macro block (Sec. 4.3.1): alpha128 = max of the sub-block absmaxes -> m8 (MBS-Static, Eq. 3),
 * then quantize_macro_block.  A last macro block shorter than `macro` uses the elements that
 * exist.  The MBS word is taken from the finite elements of the macro block.
 * Returns 0, or -1 on bad arguments. */
int mxo_quantize(const uint16_t* x, int64_t rows, int64_t K, int64_t ldx, int rule, int use_mbs,
                 int block, int macro, uint8_t* codes, uint8_t* scales, uint8_t* mbs) {
    if (rows < 0 || K < 0 || ldx < K || block <= 0 || (block & 1) || macro % block || K % block)
        return -1;
    if (rule < 0 || rule > 2) return -1;
    const int64_t nblk = K / block, nmac = (K + macro - 1) / macro;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const uint16_t* xr = x + r * ldx;
        for (int64_t g = 0; g < nmac; ++g) {
            const int64_t k0 = g * macro, k1 = (k0 + macro < K) ? k0 + macro : K;
            int m8 = 0;
            if (use_mbs) {
                m8 = mxo_mbs_static_m8(macro_absmax(xr, k0, k1));
                mbs[r * nmac + g] = (uint8_t)m8;
            }
            quantize_macro_block(xr, k0, k1, m8, rule, block, codes + r * (K / 2), scales + r * nblk);
        }
    }
    return 0;
}

/* The same with the MBS words given by the caller (mbs_in [rows, ceil(K/macro)]) instead of derived:
 * what any choice of word means for codes and scales.  Used to examine candidate words. */
int mxo_quantize_given_mbs(const uint16_t* x, int64_t rows, int64_t K, int64_t ldx, int rule,
                           int block, int macro, const uint8_t* mbs_in, uint8_t* codes,
                           uint8_t* scales) {
    if (rows < 0 || K < 0 || ldx < K || block <= 0 || (block & 1) || macro % block || K % block)
        return -1;
    if (rule < 0 || rule > 2) return -1;
    const int64_t nblk = K / block, nmac = (K + macro - 1) / macro;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t g = 0; g < nmac; ++g) {
            const int64_t k0 = g * macro, k1 = (k0 + macro < K) ? k0 + macro : K;
            quantize_macro_block(x + r * ldx, k0, k1, mbs_in[r * nmac + g], rule, block,
                                 codes + r * (K / 2), scales + r * nblk);
        }
    return 0;
}

/* ---- MBS-Dynamic (Sec. 4.3.3, Eq. 4-6; Sec. 5.3) ---------------------------------- */

/* Eq. 6 picks, out of a list of candidate words, the one with the smallest sum of squared errors
 * of the 1x128 block, sum_i (x_hat_i - x_i)^2 = sum_i x_i^2 ((x_hat_i - x_i)/x_i)^2, with
 * x_hat_i the value reconstructed from Q(x_i (1 + m_j) SF) (Eq. 4).  This is that definition
 * written out: the error of every element is taken on exact values (x_hat = q 2^-s / F in fp64,
 * one rounding of the division) and summed in fp64, element by element in order.  The paper's table
 * of approximate squared relative errors (Eq. 5) is a way to evaluate the same sum faster; it is
 * restated separately below (mxo_quantize_mbs_dynamic_lut).
 *
 * The candidate list is not given (the paper says only that there are 16 over a narrow range), so it is a parameter:
 *     m_j = (m_static + (cand_first + j) * cand_stride) mod 256,  j = 0 .. cand_count-1
 * (the factor 1 + m/256 is defined up to a power of two, which the local scales absorb, so the
 * words form a circle).  The static word always competes and is the incumbent; candidates are
 * scanned in the order j = 0, 1, ... and one replaces the current choice only with a strictly
 * smaller sum, so ties keep the static word, then the lowest j.  A macro block that holds a
 * non-finite element has no finite sum and keeps the static word. */

/* Sum of squared errors of the macro block xm[0..n) (n a multiple of block, all elements finite)
 * when it is quantized with word m8: sum_i (x_hat_i - x_i)^2, x_hat_i = value(code_i) 2^(E_b-127) / F.
 * Returns -1 if an element is not finite. */
double mxo_mbs_sse(const uint16_t* xm, int n, int m8, int rule, int block) {
    const double F = 1.0 + m8 / 256.0;
    double sse = 0.0;
    for (int b0 = 0; b0 < n; b0 += block) {
        double amax = 0.0;
        for (int k = b0; k < b0 + block; ++k) {
            if (!is_finite_bf16(xm[k])) return -1.0;
            amax = fmax(amax, fabs(mxo_bf16_value(xm[k]) * F));
        }
        int s = 0;
        if (amax > 0.0) s = 127 - mxo_e8m0_from_exponent(mxo_scale_exponent(amax, rule));
        for (int k = b0; k < b0 + block; ++k) {
            const double x = mxo_bf16_value(xm[k]);
            const double t = ldexp(x * F, s);                                  /* Eq. 4's argument, exact */
            double q = E2M1_VALUE[mxo_e2m1_nearest(fabs(t))];
            if (xm[k] & 0x8000u) q = -q;
            const double x_hat = ldexp(q, -s) / F;
            sse += (x_hat - x) * (x_hat - x);
        }
    }
    return sse;
}

/* The same sum for every macro block of a tensor under caller-given words: sse_out [rows, ceil(K/macro)]
 * (-1 for a macro block holding a non-finite element).  What a test needs to judge any choice of words. */
int mxo_mbs_sse_rows(const uint16_t* x, int64_t rows, int64_t K, int64_t ldx, int rule, int block,
                     int macro, const uint8_t* mbs_in, double* sse_out) {
    if (rows < 0 || K < 0 || ldx < K || block <= 0 || (block & 1) || macro % block || K % block)
        return -1;
    if (rule < 0 || rule > 2) return -1;
    const int64_t nmac = (K + macro - 1) / macro;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t g = 0; g < nmac; ++g) {
            const int64_t k0 = g * macro, k1 = (k0 + macro < K) ? k0 + macro : K;
            sse_out[r * nmac + g] = mxo_mbs_sse(x + r * ldx + k0, (int)(k1 - k0), mbs_in[r * nmac + g], rule, block);
        }
    return 0;
}

/* Quantize with MBS-Dynamic words (Eq. 6 with the true error).  Arguments as mxo_quantize plus the
 * candidate list.  Returns 0 or -1. */
int mxo_quantize_mbs_dynamic(const uint16_t* x, int64_t rows, int64_t K, int64_t ldx, int rule,
                             int block, int macro, int cand_first, int cand_count, int cand_stride,
                             uint8_t* codes, uint8_t* scales, uint8_t* mbs) {
    if (rows < 0 || K < 0 || ldx < K || block <= 0 || (block & 1) || macro % block || K % block)
        return -1;
    if (rule < 0 || rule > 2 || cand_count < 0 || cand_count > 256) return -1;
    const int64_t nblk = K / block, nmac = (K + macro - 1) / macro;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const uint16_t* xr = x + r * ldx;
        for (int64_t g = 0; g < nmac; ++g) {
            const int64_t k0 = g * macro, k1 = (k0 + macro < K) ? k0 + macro : K;
            const int m_static = mxo_mbs_static_m8(macro_absmax(xr, k0, k1));
            int best = m_static;
            double best_sse = mxo_mbs_sse(xr + k0, (int)(k1 - k0), m_static, rule, block);
            if (best_sse >= 0.0) {
                for (int j = 0; j < cand_count; ++j) {
                    const int m = (int)(((int64_t)m_static + (int64_t)(cand_first + j) * cand_stride) & 255);
                    const double c = mxo_mbs_sse(xr + k0, (int)(k1 - k0), m, rule, block);
                    if (c < best_sse) { best_sse = c; best = m; }
                }
            }
            mbs[r * nmac + g] = (uint8_t)best;
            quantize_macro_block(xr, k0, k1, best, rule, block, codes + r * (K / 2), scales + r * nblk);
        }
    }
    return 0;
}

/* ---- MBS-Dynamic through the table of Eq. 5 (Sec. 4.3.3) --------------------- */

/* Eq. 5-6 replace the error of every element by a tabulated squared RELATIVE error
 *     T[v, m_j]  ~  ((x_hat - x) / x)^2,    v = |x| SF   (the element in the block's scaled domain, before the
 *                                                        candidate factor is applied; SF = 2^s is the local scale
 *                                                        that the rule derives from the block's absmax times F_j)
 * so that a candidate's sum of squared errors is  sum_i x_i^2 T[v_ij, m_j]  (Eq. 6): one table read and one
 * multiply-add per element and candidate.  The paper gives the table's size, not its contents: two tables
 * ("sub-normal" v < 1 and "normal" v >= 1) of 64 points x 16 slots in fp16.  Reading taken here:
 *   - the 16 slots ARE the 16 candidates, absolute words m_j = 16 j (factors F_j = 1 + j/16): the relative
 *     error depends on the factor itself, so a table with 16 slots can only serve 16 fixed factors;
 *   - normal table: point p = the 6 leading mantissa bits of v.  E2M1 has one mantissa bit in every binade and
 *     nothing saturates below 7 (a block's scaled absmax never exceeds 7 under OAS), so the relative error of
 *     v F_j repeats from binade to binade and the mantissa is all that matters.  The entry is the squared
 *     relative error at the middle of the bin, v = 1 + (p + 1/2)/64;
 *   - sub-normal table: point p = floor(64 v), entry at v = (p + 1/2)/64 (the grid below 1 is {0, 1/2, 1}: the
 *     error is not periodic there);
 *   - entries are rounded to fp16 (nearest even); the caller passes the 2 x 64 x 16 table as fp16 bit patterns,
 *     index (table * 64 + p) * 16 + j, table 0 = sub-normal.
 * mxo_mbs_lut_entry is the definition of an entry in fp64 (the rounding to fp16 is the caller's).  */
double mxo_mbs_lut_entry(int table, int p, int j) {
    const double F = 1.0 + j / 16.0;
    const double v = table ? 1.0 + (p + 0.5) / 64.0 : (p + 0.5) / 64.0;
    const double t = v * F;                              /* below 4: no saturation */
    const double q = E2M1_VALUE[mxo_e2m1_nearest(t)];
    const double rel = (q / F - v) / v;
    return rel * rel;
}

static double half_bits_value(uint16_t h) { /* fp16 bit pattern -> value (finite patterns) */
    const int e = (h >> 10) & 31, m = h & 1023;
    const double v = e ? ldexp(1024.0 + m, e - 25) : ldexp((double)m, -24);
    return (h & 0x8000u) ? -v : v;
}

/* Point of the table for a scaled magnitude v > 0: *table = 1 (normal) with the 6 leading mantissa bits,
 * or 0 (sub-normal) with floor(64 v). */
static int lut_point(double v, int* table) {
    if (v >= 1.0) {
        int ex;
        const double fr = frexp(v, &ex);                 /* v = fr 2^ex, fr in [0.5, 1): mantissa 2 fr in [1, 2) */
        *table = 1;
        return (int)floor((2.0 * fr - 1.0) * 64.0);
    }
    *table = 0;
    return (int)floor(v * 64.0);
}

/* Eq. 6's sum for candidate j (word 16 j) on the macro block xm[0..n), all elements finite:
 * sum_i x_i^2 T[v_ij, j] in fp64, elements in order.  Returns -1 if an element is not finite. */
double mxo_mbs_lut_cost(const uint16_t* xm, int n, int j, int rule, int block, const uint16_t* lut) {
    const double F = 1.0 + j / 16.0;
    double cost = 0.0;
    for (int b0 = 0; b0 < n; b0 += block) {
        double amax = 0.0;
        for (int k = b0; k < b0 + block; ++k) {
            if (!is_finite_bf16(xm[k])) return -1.0;
            amax = fmax(amax, fabs(mxo_bf16_value(xm[k]) * F));
        }
        if (amax == 0.0) continue;
        const int s = 127 - mxo_e8m0_from_exponent(mxo_scale_exponent(amax, rule));
        for (int k = b0; k < b0 + block; ++k) {
            const double x = mxo_bf16_value(xm[k]);
            if (x == 0.0) continue;
            int table;
            const int p = lut_point(ldexp(fabs(x), s), &table);
            cost += x * x * half_bits_value(lut[(table * 64 + p) * 16 + j]);
        }
    }
    return cost;
}

/* Quantize with the word the table picks: j* = argmin_j of Eq. 6's sum over the 16 candidates (ties: the lowest
 * j), word 16 j*.  With keep_static != 0 the static word of Eq. 3 is kept instead whenever its TRUE sum of squared
 * errors (mxo_mbs_sse) is not larger than that of the picked word, so that the result is never worse than MBS-S
 * (not in the paper: the table cannot price the static word, which is not one of its 16 slots).  A macro block
 * holding a non-finite element keeps the static word.  Arguments otherwise as mxo_quantize. */
int mxo_quantize_mbs_dynamic_lut(const uint16_t* x, int64_t rows, int64_t K, int64_t ldx, int rule, int block,
                                 int macro, const uint16_t* lut, int keep_static, uint8_t* codes,
                                 uint8_t* scales, uint8_t* mbs) {
    if (rows < 0 || K < 0 || ldx < K || block <= 0 || (block & 1) || macro % block || K % block || !lut)
        return -1;
    if (rule < 0 || rule > 2) return -1;
    const int64_t nblk = K / block, nmac = (K + macro - 1) / macro;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const uint16_t* xr = x + r * ldx;
        for (int64_t g = 0; g < nmac; ++g) {
            const int64_t k0 = g * macro, k1 = (k0 + macro < K) ? k0 + macro : K;
            const int n = (int)(k1 - k0);
            const int m_static = mxo_mbs_static_m8(macro_absmax(xr, k0, k1));
            int best = m_static;
            double best_cost = mxo_mbs_lut_cost(xr + k0, n, 0, rule, block, lut);
            if (best_cost >= 0.0) {
                int jbest = 0;
                for (int j = 1; j < 16; ++j) {
                    const double c = mxo_mbs_lut_cost(xr + k0, n, j, rule, block, lut);
                    if (c < best_cost) { best_cost = c; jbest = j; }
                }
                best = 16 * jbest;
                if (keep_static && mxo_mbs_sse(xr + k0, n, m_static, rule, block) <= mxo_mbs_sse(xr + k0, n, best, rule, block))
                    best = m_static;
            }
            mbs[r * nmac + g] = (uint8_t)best;
            quantize_macro_block(xr, k0, k1, best, rule, block, codes + r * (K / 2), scales + r * nblk);
        }
    }
    return 0;
}

/* ---- dequantizer (Sec. 4.3.1: value = code * 2^(E-127) / F) --------------------------------- */

static double scale_value(int E) { return (E == 255) ? NAN : ldexp(1.0, E - 127); }

/* out [rows, K] fp64.  mbs may be NULL (F = 1). */
int mxo_dequantize(const uint8_t* codes, const uint8_t* scales, const uint8_t* mbs, int64_t rows,
                   int64_t K, int block, int macro, double* out) {
    if (rows < 0 || K < 0 || block <= 0 || macro % block || K % block) return -1;
    const int64_t nblk = K / block, nmac = (K + macro - 1) / macro;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < K; ++k) {
            int byte = codes[r * (K / 2) + k / 2];
            int code = (k & 1) ? (byte >> 4) : (byte & 15);
            double F = mbs ? 1.0 + mbs[r * nmac + k / macro] / 256.0 : 1.0;
            out[r * K + k] = mxo_e2m1_decode(code) * scale_value(scales[r * nblk + k / block]) / F;
        }
    return 0;
}

/* ---- GEMM with MBS (Sec. 4.3.2; App. E: the MBS scales are applied every 128 K-elements) ----- */

/* C[t, j] for the listed rows i = row_idx[t] of A (all rows if row_idx is NULL, then nrows = M):
 *   C[i,j] = sum over macro blocks g of
 *            ( sum_{k in g} a_ik 2^(Ea-127) * b_jk 2^(Eb-127) ) * sigma_A[i,g] * sigma_B[j,g],
 * sigma = 1/F (Sec. 4.3.2).  A is [M,K], B is [N,K] (the product is A B^T), a_mbs / b_mbs may be
 * NULL.  Output [nrows, N] fp64. */
int mxo_gemm_rows(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs,
                  const uint8_t* b_codes, const uint8_t* b_scales, const uint8_t* b_mbs,
                  int64_t M, int64_t N, int64_t K, int block, int macro,
                  const int64_t* row_idx, int64_t nrows, double* C) {
    if (M < 0 || N < 0 || K < 0 || block <= 0 || macro % block || K % block) return -1;
    const int64_t nblk = K / block, nmac = (K + macro - 1) / macro;
    for (int64_t t = 0; t < nrows; ++t)
        if (row_idx && (row_idx[t] < 0 || row_idx[t] >= M)) return -1;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t t = 0; t < nrows; ++t)
        for (int64_t j = 0; j < N; ++j) {
            const int64_t i = row_idx ? row_idx[t] : t;
            double c = 0.0;
            for (int64_t g = 0; g < nmac; ++g) {
                const int64_t k0 = g * macro, k1 = (k0 + macro < K) ? k0 + macro : K;
                double p = 0.0;
                for (int64_t k = k0; k < k1; ++k) {
                    int ab = a_codes[i * (K / 2) + k / 2], bb = b_codes[j * (K / 2) + k / 2];
                    int ac = (k & 1) ? (ab >> 4) : (ab & 15), bc = (k & 1) ? (bb >> 4) : (bb & 15);
                    double av = mxo_e2m1_decode(ac) * scale_value(a_scales[i * nblk + k / block]);
                    double bv = mxo_e2m1_decode(bc) * scale_value(b_scales[j * nblk + k / block]);
                    p += av * bv;
                }
                double Fa = a_mbs ? 1.0 + a_mbs[i * nmac + g] / 256.0 : 1.0;
                double Fb = b_mbs ? 1.0 + b_mbs[j * nmac + g] / 256.0 : 1.0;
                c += p * (1.0 / Fa) * (1.0 / Fb);
            }
            C[t * N + j] = c;
        }
    return 0;
}

/* Product of the unquantized bf16 tensors, the reference signal of QSNR(AB) (Eq. 2):
 * C[t, j] = sum_k A[row_idx[t], k] * B[j, k] in fp64. */
int mxo_matmul_bf16_rows(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb, int64_t M,
                         int64_t N, int64_t K, const int64_t* row_idx, int64_t nrows, double* C) {
    if (M < 0 || N < 0 || K < 0 || lda < K || ldb < K) return -1;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t t = 0; t < nrows; ++t)
        for (int64_t j = 0; j < N; ++j) {
            const int64_t i = row_idx ? row_idx[t] : t;
            double c = 0.0;
            for (int64_t k = 0; k < K; ++k)
                c += mxo_bf16_value(A[i * lda + k]) * mxo_bf16_value(B[j * ldb + k]);
            C[t * N + j] = c;
        }
    return 0;
}

/* ---- the other MX element formats (Sec. 1, footnote: the methods carry over to MXFP6 / MXFP8) ---- */

/* The paper works MXFP4 through and says only that OAS and MBS generalise.  The reading taken here
 * restates each rule with the element format's own constants in place of E2M1's:
 *   V      largest finite magnitude (E2M1: 6)            = vm * 2^emax, vm in [1, 2)
 *   h      half of the spacing of the format's top binade (E2M1: 1) = 2^(emax - mbits - 1)
 *   FLOOR: SF = 2^floor(log2(V/alpha)), scaled absmax in (V/2, V]
 *   OAS:   from FLOOR; a scaled absmax of at most (V + h)/2 doubles SF: scaled absmax in
 *          ((V + h)/2, V + h].  V + h is where E2M1's 7 comes from: saturating a value of (V, V + h]
 *          to V costs no more than rounding inside the top binade does.
 *   OCP:   shared exponent floor(log2 alpha) - emax, scaled absmax in [2^emax, 2^(emax+1))
 *   MBS-S: m8 = 8 leading mantissa bits of V/alpha128, so that the macro-block absmax lands on V
 * Element formats as in the OCP MX specification: E4M3 (bias 7; S.1111.111 is NaN, so V = 448),
 * E5M2 (bias 15; exponent field 31 is Inf/NaN, V = 57344), E2M3 (bias 1, V = 7.5) and E3M2 (bias 3,
 * V = 28) with every code finite, and E2M1 itself, which must reproduce mxo_quantize.
 * Codes are stored one per byte (sign in the format's top bit), whatever the format's width.
 * Parity status: pinned by tests/test_oracle_elem_pins.py; no value of the paper covers these
 * formats, so what is pinned is this reading against exact arithmetic and a library's FP8 types. */
#define MXO_ELEM_E2M1 0
#define MXO_ELEM_E4M3 1
#define MXO_ELEM_E5M2 2
#define MXO_ELEM_E2M3 3
#define MXO_ELEM_E3M2 4

typedef struct {
    int ebits, mbits, bias;
    int max_code; /* magnitude code of V */
} elem_format;

static const elem_format ELEM[5] = {
    {2, 1, 1, 0x07}, /* E2M1: 1.5 * 2^2            */
    {4, 3, 7, 0x7E}, /* E4M3: 1.75 * 2^8, 0x7F NaN */
    {5, 2, 15, 0x7B}, /* E5M2: 1.75 * 2^15, exponent 31 Inf/NaN */
    {2, 3, 1, 0x1F}, /* E2M3: 1.875 * 2^2          */
    {3, 2, 3, 0x1F}, /* E3M2: 1.75 * 2^4           */
};

int mxo_elem_bits(int fmt) { return (fmt < 0 || fmt > 4) ? -1 : 1 + ELEM[fmt].ebits + ELEM[fmt].mbits; }

/* Value of magnitude code c (sign stripped): subnormal m * 2^(1-bias-mbits) when the exponent field
 * is 0, else (1 + m/2^mbits) * 2^(e-bias). */
static double elem_magnitude(const elem_format* f, int c) {
    const int e = c >> f->mbits, m = c & ((1 << f->mbits) - 1);
    if (e == 0) return ldexp((double)m, 1 - f->bias - f->mbits);
    return ldexp((double)((1 << f->mbits) + m), e - f->bias - f->mbits);
}

/* Value of a stored code (sign bit = bit ebits+mbits).  Codes above the largest finite magnitude
 * (E4M3's NaN, E5M2's Inf/NaN) decode to NaN; the quantizer never produces them. */
double mxo_elem_decode(int fmt, int code) {
    if (fmt < 0 || fmt > 4) return NAN;
    const elem_format* f = &ELEM[fmt];
    const int sign_bit = 1 << (f->ebits + f->mbits), c = code & (sign_bit - 1);
    if (c > f->max_code) return NAN;
    const double v = elem_magnitude(f, c);
    return (code & sign_bit) ? -v : v;
}

double mxo_elem_max(int fmt) { return (fmt < 0 || fmt > 4) ? NAN : elem_magnitude(&ELEM[fmt], ELEM[fmt].max_code); }

/* Magnitude code of the format's value nearest to y >= 0: saturating at V, a tie to the code with
 * an even mantissa.  Plain search over every finite code. */
int mxo_elem_nearest(int fmt, double y) {
    if (fmt < 0 || fmt > 4) return -1;
    const elem_format* f = &ELEM[fmt];
    if (y >= elem_magnitude(f, f->max_code)) return f->max_code;
    int best = 0;
    double best_d = fabs(y - elem_magnitude(f, 0));
    for (int c = 1; c <= f->max_code; ++c) {
        const double d = fabs(y - elem_magnitude(f, c));
        if (d < best_d || (d == best_d && (c & 1) == 0)) {
            best = c;
            best_d = d;
        }
    }
    return best;
}

/* emax and the mantissa vm of V = vm * 2^emax. */
static double elem_vmax_parts(const elem_format* f, int* emax) {
    int ex;
    const double fr = frexp(elem_magnitude(f, f->max_code), &ex); /* V = fr * 2^ex, fr in [0.5, 1) */
    *emax = ex - 1;
    return 2.0 * fr;
}

/* Exponent s of SF = 2^s for a block of (MBS-scaled) absmax alpha > 0 under the rules above. */
int mxo_elem_scale_exponent(int fmt, double alpha, int rule) {
    const elem_format* f = &ELEM[fmt];
    int emax, ex;
    const double vm = elem_vmax_parts(f, &emax);
    const double fr = frexp(alpha, &ex); /* alpha = fr * 2^ex */
    if (rule == MXO_RULE_OCP) return emax - (ex - 1);
    /* V/alpha = (vm / (2 fr)) * 2^(emax - ex + 1) with vm/(2 fr) in (vm/2, vm]: its floor(log2) is
     * emax - ex + 1 when vm/(2 fr) >= 1, i.e. fr <= vm/2 (compared so that no division rounds). */
    int s = (fr <= vm / 2.0) ? emax - ex + 1 : emax - ex;
    if (rule == MXO_RULE_OAS) {
        const double V = elem_magnitude(f, f->max_code), h = ldexp(1.0, emax - f->mbits - 1);
        if (ldexp(alpha, s) <= (V + h) / 2.0) s += 1; /* all exact */
    }
    return s;
}

/* MBS-Static word: the 8 leading mantissa bits of V/alpha, by exact integer division. */
int mxo_elem_mbs_static_m8(int fmt, double alpha) {
    if (!(alpha > 0.0) || isinf(alpha)) return 0;
    const elem_format* f = &ELEM[fmt];
    int emax, ex;
    const double vm = elem_vmax_parts(f, &emax);
    const double fr = frexp(alpha, &ex);
    const uint64_t n = (uint64_t)ldexp(fr, 53);               /* fr = n / 2^53                 */
    /* normalised quotient 1+m = vm/(2 fr) when that is >= 1, else vm/fr; 256 vm is an integer     */
    const unsigned __int128 vm256 = (unsigned __int128)(uint64_t)(256.0 * vm);
    const unsigned __int128 num = (fr <= vm / 2.0) ? (vm256 << 52) : (vm256 << 53);
    return (int)(uint64_t)(num / n) - 256;
}

/* One macro block xr[k0..k1) of a row under word m8 into element format fmt: scale bytes into
 * scales_row[k / block], codes (one per byte) into codes_row[k]. */
static void elem_quantize_macro_block(int fmt, const uint16_t* xr, int64_t k0, int64_t k1, int m8, int rule,
                                      int block, uint8_t* codes_row, uint8_t* scales_row) {
    const elem_format* f = &ELEM[fmt];
    const int sign_bit = 1 << (f->ebits + f->mbits);
    const double F = 1.0 + m8 / 256.0;
    for (int64_t b0 = k0; b0 < k1; b0 += block) {
        int finite = 1;
        double amax = 0.0;
        for (int64_t k = b0; k < b0 + block; ++k) {
            if (!is_finite_bf16(xr[k])) finite = 0;
            else amax = fmax(amax, fabs(mxo_bf16_value(xr[k]) * F));
        }
        int E, s;
        if (!finite) { E = 255; s = 0; }
        else if (amax == 0.0) { E = 127; s = 0; }
        else { E = mxo_e8m0_from_exponent(mxo_elem_scale_exponent(fmt, amax, rule)); s = 127 - E; }
        scales_row[b0 / block] = (uint8_t)E;
        for (int64_t k = b0; k < b0 + block; ++k) {
            int code = 0;
            if (finite) {
                const double t = ldexp(mxo_bf16_value(xr[k]) * F, s); /* exact */
                code = mxo_elem_nearest(fmt, fabs(t)) | ((xr[k] & 0x8000u) ? sign_bit : 0);
            }
            codes_row[k] = (uint8_t)code;
        }
    }
}

/* Quantize rows of bf16 into element format fmt: as mxo_quantize, with codes [rows, K] one per byte. */
int mxo_elem_quantize(int fmt, const uint16_t* x, int64_t rows, int64_t K, int64_t ldx, int rule,
                      int use_mbs, int block, int macro, uint8_t* codes, uint8_t* scales, uint8_t* mbs) {
    if (fmt < 0 || fmt > 4 || rows < 0 || K < 0 || ldx < K || block <= 0 || macro % block || K % block)
        return -1;
    if (rule < 0 || rule > 2) return -1;
    const int64_t nblk = K / block, nmac = (K + macro - 1) / macro;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const uint16_t* xr = x + r * ldx;
        for (int64_t g = 0; g < nmac; ++g) {
            const int64_t k0 = g * macro, k1 = (k0 + macro < K) ? k0 + macro : K;
            int m8 = 0;
            if (use_mbs) {
                m8 = mxo_elem_mbs_static_m8(fmt, macro_absmax(xr, k0, k1));
                mbs[r * nmac + g] = (uint8_t)m8;
            }
            elem_quantize_macro_block(fmt, xr, k0, k1, m8, rule, block, codes + r * K, scales + r * nblk);
        }
    }
    return 0;
}

/* The same with caller-chosen words mbs_in [rows, ceil(K/macro)] (what a test needs to judge any choice of
 * words, and what MBS-Dynamic ends with). */
int mxo_elem_quantize_given_mbs(int fmt, const uint16_t* x, int64_t rows, int64_t K, int64_t ldx, int rule,
                                int block, int macro, const uint8_t* mbs_in, uint8_t* codes, uint8_t* scales) {
    if (fmt < 0 || fmt > 4 || rows < 0 || K < 0 || ldx < K || block <= 0 || macro % block || K % block)
        return -1;
    if (rule < 0 || rule > 2) return -1;
    const int64_t nblk = K / block, nmac = (K + macro - 1) / macro;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t g = 0; g < nmac; ++g) {
            const int64_t k0 = g * macro, k1 = (k0 + macro < K) ? k0 + macro : K;
            elem_quantize_macro_block(fmt, x + r * ldx, k0, k1, mbs_in[r * nmac + g], rule, block, codes + r * K,
                                      scales + r * nblk);
        }
    return 0;
}

/* MBS-Dynamic for the element formats (Sec. 4.3.3, Eq. 6 with the true error; Sec. 1, footnote).  The
 * definition does not depend on the element format: among the static word and the candidates
 * m_j = (m_static + (cand_first + j) * cand_stride) mod 256 the word with the least sum of squared
 * errors of the 1x128 block wins, ties to the static word, then to the lowest j (see mxo_mbs_sse and
 * mxo_quantize_mbs_dynamic above, which these two restate with the format's rules and grid). */
double mxo_elem_mbs_sse(int fmt, const uint16_t* xm, int n, int m8, int rule, int block) {
    const double F = 1.0 + m8 / 256.0;
    double sse = 0.0;
    for (int b0 = 0; b0 < n; b0 += block) {
        double amax = 0.0;
        for (int k = b0; k < b0 + block; ++k) {
            if (!is_finite_bf16(xm[k])) return -1.0;
            amax = fmax(amax, fabs(mxo_bf16_value(xm[k]) * F));
        }
        int s = 0;
        if (amax > 0.0) s = 127 - mxo_e8m0_from_exponent(mxo_elem_scale_exponent(fmt, amax, rule));
        for (int k = b0; k < b0 + block; ++k) {
            const double x = mxo_bf16_value(xm[k]);
            const double t = ldexp(x * F, s); /* exact */
            double q = elem_magnitude(&ELEM[fmt], mxo_elem_nearest(fmt, fabs(t)));
            if (xm[k] & 0x8000u) q = -q;
            const double x_hat = ldexp(q, -s) / F;
            sse += (x_hat - x) * (x_hat - x);
        }
    }
    return sse;
}

int mxo_elem_mbs_sse_rows(int fmt, const uint16_t* x, int64_t rows, int64_t K, int64_t ldx, int rule, int block,
                          int macro, const uint8_t* mbs_in, double* sse_out) {
    if (fmt < 0 || fmt > 4 || rows < 0 || K < 0 || ldx < K || block <= 0 || macro % block || K % block)
        return -1;
    if (rule < 0 || rule > 2) return -1;
    const int64_t nmac = (K + macro - 1) / macro;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t g = 0; g < nmac; ++g) {
            const int64_t k0 = g * macro, k1 = (k0 + macro < K) ? k0 + macro : K;
            sse_out[r * nmac + g] = mxo_elem_mbs_sse(fmt, x + r * ldx + k0, (int)(k1 - k0), mbs_in[r * nmac + g], rule, block);
        }
    return 0;
}

int mxo_elem_quantize_mbs_dynamic(int fmt, const uint16_t* x, int64_t rows, int64_t K, int64_t ldx, int rule,
                                  int block, int macro, int cand_first, int cand_count, int cand_stride,
                                  uint8_t* codes, uint8_t* scales, uint8_t* mbs) {
    if (fmt < 0 || fmt > 4 || rows < 0 || K < 0 || ldx < K || block <= 0 || macro % block || K % block)
        return -1;
    if (rule < 0 || rule > 2 || cand_count < 0 || cand_count > 256) return -1;
    const int64_t nblk = K / block, nmac = (K + macro - 1) / macro;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const uint16_t* xr = x + r * ldx;
        for (int64_t g = 0; g < nmac; ++g) {
            const int64_t k0 = g * macro, k1 = (k0 + macro < K) ? k0 + macro : K;
            const int m_static = mxo_elem_mbs_static_m8(fmt, macro_absmax(xr, k0, k1));
            int best = m_static;
            double best_sse = mxo_elem_mbs_sse(fmt, xr + k0, (int)(k1 - k0), m_static, rule, block);
            if (best_sse >= 0.0) {
                for (int j = 0; j < cand_count; ++j) {
                    const int m = (int)(((int64_t)m_static + (int64_t)(cand_first + j) * cand_stride) & 255);
                    const double c = mxo_elem_mbs_sse(fmt, xr + k0, (int)(k1 - k0), m, rule, block);
                    if (c < best_sse) { best_sse = c; best = m; }
                }
            }
            mbs[r * nmac + g] = (uint8_t)best;
            elem_quantize_macro_block(fmt, xr, k0, k1, best, rule, block, codes + r * K, scales + r * nblk);
        }
    }
    return 0;
}

/* out [rows, K] fp64 = code value * 2^(E-127) / F. */
int mxo_elem_dequantize(int fmt, const uint8_t* codes, const uint8_t* scales, const uint8_t* mbs,
                        int64_t rows, int64_t K, int block, int macro, double* out) {
    if (fmt < 0 || fmt > 4 || rows < 0 || K < 0 || block <= 0 || macro % block || K % block) return -1;
    const int64_t nblk = K / block, nmac = (K + macro - 1) / macro;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < K; ++k) {
            const double F = mbs ? 1.0 + mbs[r * nmac + k / macro] / 256.0 : 1.0;
            out[r * K + k] = mxo_elem_decode(fmt, codes[r * K + k]) * scale_value(scales[r * nblk + k / block]) / F;
        }
    return 0;
}

/* mxo_gemm_rows for operands in element formats fmt_a and fmt_b (Sec. 4.3.2 unchanged: the MBS
 * correction does not depend on the element format). */
int mxo_elem_gemm_rows(int fmt_a, const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs,
                       int fmt_b, const uint8_t* b_codes, const uint8_t* b_scales, const uint8_t* b_mbs,
                       int64_t M, int64_t N, int64_t K, int block, int macro,
                       const int64_t* row_idx, int64_t nrows, double* C) {
    if (fmt_a < 0 || fmt_a > 4 || fmt_b < 0 || fmt_b > 4) return -1;
    if (M < 0 || N < 0 || K < 0 || block <= 0 || macro % block || K % block) return -1;
    const int64_t nblk = K / block, nmac = (K + macro - 1) / macro;
    for (int64_t t = 0; t < nrows; ++t)
        if (row_idx && (row_idx[t] < 0 || row_idx[t] >= M)) return -1;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t t = 0; t < nrows; ++t)
        for (int64_t j = 0; j < N; ++j) {
            const int64_t i = row_idx ? row_idx[t] : t;
            double c = 0.0;
            for (int64_t g = 0; g < nmac; ++g) {
                const int64_t k0 = g * macro, k1 = (k0 + macro < K) ? k0 + macro : K;
                double p = 0.0;
                for (int64_t k = k0; k < k1; ++k) {
                    const double av = mxo_elem_decode(fmt_a, a_codes[i * K + k]) * scale_value(a_scales[i * nblk + k / block]);
                    const double bv = mxo_elem_decode(fmt_b, b_codes[j * K + k]) * scale_value(b_scales[j * nblk + k / block]);
                    p += av * bv;
                }
                const double Fa = a_mbs ? 1.0 + a_mbs[i * nmac + g] / 256.0 : 1.0;
                const double Fb = b_mbs ? 1.0 + b_mbs[j * nmac + g] / 256.0 : 1.0;
                c += p * (1.0 / Fa) * (1.0 / Fb);
            }
            C[t * N + j] = c;
        }
    return 0;
}

/* ---- QSNR (Sec. 3.1, Eq. 1-2) --------------------------------------------------------------- */

/* 10 log10( ||ref||^2 / ||ref - test||^2 ); +inf when test reproduces ref. */
double mxo_qsnr_db(const double* ref, const double* test, int64_t n) {
    double sig = 0.0, noise = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        sig += ref[i] * ref[i];
        double d = ref[i] - test[i];
        noise += d * d;
    }
    if (noise == 0.0) return INFINITY;
    return 10.0 * log10(sig / noise);
}

/* Number of OpenMP threads a parallel region here uses (reported beside the CPU baseline). */
#ifdef _OPENMP
#include <omp.h>
int mxo_num_threads(void) { return omp_get_max_threads(); }
/* Number of threads the row loops use from now on (for timing the oracle on one core); returns the old number. */
int mxo_set_num_threads(int n) { int old = omp_get_max_threads(); if (n > 0) omp_set_num_threads(n); return old; }
#else
int mxo_num_threads(void) { return 1; }
int mxo_set_num_threads(int n) { (void)n; return 1; }
#endif
