// MXFP4 quantizer with Overflow-Aware Scaling and static Macro Block Scaling for gfx950.
//
// Work decomposition (one pass over the tensor, Sec. 4.3: no second traversal is needed because
// the macro block is local):  a lane owns 8 consecutive bf16 (one 16-byte load), 4 lanes own a
// 32-element block, a row of 16 lanes owns a 1x128 macro block, a wavefront owns 512 consecutive
// elements of one tensor row.  Block and macro-block maxima are DPP reductions over the bf16
// magnitude bits (integer order == magnitude order); no LDS traffic is needed for them.
//
// Arithmetic is arranged so that every decision is exact:
//   - MBS word (Sec. 4.3.1, Eq. 3): the 8 leading mantissa bits of 6/absmax128 depend only on
//     the 7 mantissa bits k of the bf16 absmax: floor(N / (128 + k)) - 256 with N = 49152 or 98304.
//     The quotient is taken with the hardware reciprocal plus 2^-10: N / (128 + k) is either an
//     integer (k = 0, 64) or at least 1/255 away from one, far more than the reciprocal's error.
//   - x * F (F = 1 + m8/256) has at most 17 significant bits and is exact in fp32, and so is its
//     product with the power-of-two block scale.
//   - the block exponent is read off the fp32 pattern of absmax * F with a carry trick: adding
//     (2^23 - 1 - threshold) to the pattern bumps the exponent field exactly when the mantissa
//     exceeds the rule's threshold (Sec. 4.2: FLOOR 1.5, OAS 1.75, OCP never).
// Blocks whose magnitudes are so small or so large that fp32 products could leave the normal
// range, and blocks holding Inf/NaN, take a wave-uniform detour through an all-integer path.
#include "mx_internal.h"
#include "mx_quantize_math.h"

#include <mutex>

// The table of Eq. 5 for callers that cannot allocate: one copy per GPU inside the library's code object, held
// until the process ends.  In host code `scratch` is only a stand-in for the symbol; the per-device address
// comes from hipGetSymbolAddress, is looked up once per device with that device current, and is what every
// launch and kernel argument below uses.
static __device__ __align__(256) uint16_t scratch[2048];

namespace mx {
namespace {

constexpr int kChunk = 512;        // elements per wavefront step
constexpr int kUnroll = 4;         // chunks in flight per wavefront
constexpr int kThreads = 256;
constexpr int64_t kMaxK = (int64_t)1 << 30;  // a lane's column inside its row is a 32-bit number

struct QuantArgs {
    const uint16_t* x;
    uint8_t* codes;
    uint8_t* scales;
    uint8_t* mbs;
    int64_t K, ldx, nmac;
    uint32_t chunks_per_row, total_chunks;
    uint32_t carry;  // 2^23 - 1 - mantissa threshold of the rule, 0 for OCP
    int rule;
    int use_mbs;
    int scales_dword;  // scales of a macro block can be stored as one aligned dword
    // optional second tensor with the same K, quantized by the same launch: its chunks follow the first
    // tensor's, whose count is rounded up to a whole batch (split) so that no batch straddles the two
    const uint16_t* x2;
    uint8_t *codes2, *scales2, *mbs2;
    int64_t ldx2;
    uint32_t split, total_chunks2;
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Round |t| (t already multiplied by the block scale) to the E2M1 grid, nearest-even, saturating.
// Adding 1.5 * 2^(22 + e), e = max(exponent(t), 0), leaves t in units of the grid step of its
// binade in the low mantissa bits of the sum.
__device__ __forceinline__ uint32_t e2m1_code_alu(float t) {
    const uint32_t tb = __float_as_uint(t);
    const float y = fminf(__uint_as_float(tb & 0x7FFFFFFFu), 6.0f);
    const uint32_t ey = max(__float_as_uint(y) >> 23, 127u);
    const float w = y + __uint_as_float(((ey + 22u) << 23) | 0x400000u);
    const uint32_t mag = (__float_as_uint(w) & 0xFu) + 2u * (ey - 127u);
    return mag | ((tb >> 28) & 8u);
}

struct ChunkResult {
    uint32_t codes;  // 8 E2M1 codes of this lane
    uint32_t E;      // E8M0 byte of this lane's block
    uint32_t m8;     // MBS word of this lane's macro block
};

// All-integer path, exact for every bf16 input including subnormals, huge values and Inf/NaN.
// m8_given >= 0 replaces the static word (the searched word of MBS-Dynamic).
__device__ __noinline__ ChunkResult quantize_chunk_exact(u32x4 v, int rule, int use_mbs, int m8_given = -1) {
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

    uint32_t m8 = use_mbs ? mbs_word_of_absmax(mmax) : 0u;
    if (m8_given >= 0) m8 = (uint32_t)m8_given;
    const uint32_t u = 256u + m8;  // F = u / 256

    const int E = nf ? 255 : amax == 0 ? 127 : exact_scale_byte(amax, u, rule);
    const int s = 127 - E;
    uint32_t codes = 0;
    if (!nf) {
#pragma unroll
        for (int i = 0; i < 8; ++i) codes |= exact_code(h[i], u, s) << (4 * i);
    }
    return {codes, (uint32_t)E, m8};
}

template <bool kHwCvt, bool kMbs>
__device__ __forceinline__ ChunkResult quantize_chunk(u32x4 v, const QuantArgs& q) {
    // lane, block and macro-block absmax on the magnitude bits
    uint32_t m = pk_max_u16(pk_max_u16(v.x & 0x7FFF7FFFu, v.y & 0x7FFF7FFFu),
                            pk_max_u16(v.z & 0x7FFF7FFFu, v.w & 0x7FFF7FFFu));
    uint32_t amax = max(m & 0xFFFFu, m >> 16);
    amax = max(amax, dpp_quad_xor1(amax));
    amax = max(amax, dpp_quad_xor2(amax));

    // exponent field outside [24, 249] (or Inf/NaN): leave fp32 arithmetic, wave-uniformly
    const bool odd = (amax >= (250u << 7)) || (amax != 0 && amax < (24u << 7));
    if (__builtin_amdgcn_ballot_w64(odd) != 0) return quantize_chunk_exact(v, q.rule, kMbs);

    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t codes = 0;
    if constexpr (!kMbs && kHwCvt) {
        // no MBS: the block exponent comes straight off the bf16 absmax, and the hardware converts
        // bf16 pairs with the block scale applied (x / 2^(E-127), nearest-even, saturating)
        uint32_t E = (((amax << 16) + q.carry) >> 23) - 2u;
        E = amax ? E : 127u;
        const float scale = __uint_as_float(E << 23);
        typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
        codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(codes, __builtin_bit_cast(v2bf, w[0]), scale, 0);
        codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(codes, __builtin_bit_cast(v2bf, w[1]), scale, 1);
        codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(codes, __builtin_bit_cast(v2bf, w[2]), scale, 2);
        codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(codes, __builtin_bit_cast(v2bf, w[3]), scale, 3);
        return {codes, E, 0u};
    } else {
        uint32_t m8 = 0;
        if constexpr (kMbs) {
            uint32_t mmax = max(amax, dpp_row_ror4(amax));
            mmax = max(mmax, dpp_row_ror8(mmax));
            m8 = mmax ? mbs_word_of_mantissa_fast(mmax & 0x7Fu) : 0u;
        }
        // absmax * F is exact in fp32; exponent field + carry gives the stored byte
        const float scaled_max = __uint_as_float(amax << 16) * __uint_as_float(0x3F800000u | (m8 << 15));
        uint32_t E = ((__float_as_uint(scaled_max) + q.carry) >> 23) - 2u;
        E = amax ? E : 127u;
        // multiplier F * 2^(127-E): exponent field 254-E under F's mantissa
        const float mult = __uint_as_float(((254u - E) << 23) | (m8 << 15));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float t0 = __uint_as_float(w[i] << 16) * mult;
            const float t1 = __uint_as_float(w[i] & 0xFFFF0000u) * mult;
            if constexpr (kHwCvt) {
                // hardware fp32 -> E2M1 pair convert (scale 1: the block scale is already applied)
                if (i == 0) codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, t0, t1, 1.0f, 0);
                if (i == 1) codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, t0, t1, 1.0f, 1);
                if (i == 2) codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, t0, t1, 1.0f, 2);
                if (i == 3) codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, t0, t1, 1.0f, 3);
            } else {
                codes |= (e2m1_code_alu(t0) | (e2m1_code_alu(t1) << 4)) << (8 * i);
            }
        }
        return {codes, E, m8};
    }
}

template <bool kHwCvt, bool kMbs>
__global__ __launch_bounds__(kThreads) void quantize_kernel(QuantArgs q) {
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6));
    const uint32_t nwaves = gridDim.x * (kThreads / kWave);

    // chunk ids are wave-uniform: (row, chunk-in-row) is found once per batch of kUnroll chunks and then
    // stepped, so the division stays off the per-element path
    for (uint32_t g0 = wave * kUnroll; g0 < q.split + q.total_chunks2; g0 += nwaves * kUnroll) {
        // which tensor (wave-uniform)
        const bool second = g0 >= q.split;
        const uint16_t* x = second ? q.x2 : q.x;
        uint8_t* codes = second ? q.codes2 : q.codes;
        uint8_t* scales = second ? q.scales2 : q.scales;
        uint8_t* mbs = second ? q.mbs2 : q.mbs;
        const int64_t ldx = second ? q.ldx2 : q.ldx;
        const uint32_t total = second ? q.total_chunks2 : q.total_chunks;
        const uint32_t c0 = second ? g0 - q.split : g0;
        if (c0 >= total) continue;
        u32x4 v[kUnroll];
        uint32_t row[kUnroll], col[kUnroll];
        bool valid[kUnroll];
        uint32_t r = c0 / q.chunks_per_row, cc = c0 - r * q.chunks_per_row;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            row[u] = r;
            col[u] = cc * kChunk + lane * 8;
            valid[u] = c0 + u < total && col[u] < q.K;
            v[u] = u32x4{0, 0, 0, 0};
            if (valid[u]) {
                const uint16_t* rowp = x + (int64_t)r * ldx;  // uniform base + 32-bit lane offset
                v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(rowp + col[u]));
            }
            if (++cc == q.chunks_per_row) { cc = 0; ++r; }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            if (c0 + u >= total) break;  // wave-uniform
            const ChunkResult res = quantize_chunk<kHwCvt, kMbs>(v[u], q);
            // scales of the macro block gathered into one dword across the row of 16 lanes
            uint32_t ew = res.E << (8 * ((lane >> 2) & 3));
            if ((lane & 3) != 0) ew = 0;
            ew |= dpp_row_ror4(ew);
            ew |= dpp_row_ror8(ew);
            if (!valid[u]) continue;
            const uint32_t kblk = col[u] >> 5;
            uint8_t* srow = scales + (int64_t)row[u] * (q.K >> 5);
            uint8_t* crow = codes + (int64_t)row[u] * (q.K >> 1);
            *reinterpret_cast<uint32_t*>(crow + (col[u] >> 1)) = res.codes;
            if (q.scales_dword) {
                if ((lane & 15) == 0) *reinterpret_cast<uint32_t*>(srow + kblk) = ew;
            } else if ((lane & 3) == 0) {
                srow[kblk] = (uint8_t)res.E;
            }
            if (kMbs && (lane & 15) == 0) mbs[(int64_t)row[u] * q.nmac + (col[u] >> 7)] = (uint8_t)res.m8;
        }
    }
}

// ---- MBS-Dynamic (Sec. 4.3.1, Sec. 5.3) ----------------------------------------------------
// Per macro block the word is searched among the candidates
//     m_j = (m_static + (cand_first + j) * cand_stride) mod 256,  j = 0 .. cand_count - 1,
// for the least sum of squared errors of the 1x128 block.  The paper reads squared relative errors from a
// table; here the error is measured directly: the hardware converts the scaled pair to E2M1 and back, the
// difference is exact in fp32, and its squares are accumulated.  So that the minimum is reproducible the
// cost has a fixed order of operations: fused multiply-adds over the lane's 8 elements in order, pairwise
// sums over the 4 lanes of a block, an exact rescale from the block's binade to the macro block's,
// pairwise sums over the 4 blocks, one multiplication by the reciprocal of F^2 (within an ulp).  The static word is the
// incumbent; a candidate replaces the current choice only with a strictly smaller cost.  The search runs
// where fp32 holds every intermediate exactly (exponent field of the macro-block absmax in [64, 249], no
// Inf/NaN in it); a block whose own absmax is zero or more than 30 binades below contributes nothing.
struct DynArgs {
    QuantArgs q;
    int cand_first, cand_count, cand_stride;
};

__device__ __forceinline__ float dpp_quad_xor1_f(float v) { return __uint_as_float(dpp_quad_xor1(__float_as_uint(v))); }
__device__ __forceinline__ float dpp_quad_xor2_f(float v) { return __uint_as_float(dpp_quad_xor2(__float_as_uint(v))); }
// lane i <-> 7 - i inside each half row, lane i <-> 15 - i inside each row: on values that are uniform
// over aligned groups of 4 (resp. 8) lanes these exchange neighbouring groups
__device__ __forceinline__ float dpp_half_mirror_f(float v) {
    return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), 0x141, 0xF, 0xF, true));
}
__device__ __forceinline__ float dpp_mirror_f(float v) {
    return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), 0x140, 0xF, 0xF, true));
}

struct Candidate {
    uint32_t codes, E;
    float cost;
};

// Codes, scale byte and macro-block cost of word m.  xf: the lane's 8 elements; amax: bf16 magnitude bits
// of the block's absmax; counts: the block contributes to the cost; e128: exponent field of the macro
// block's absmax.  The cost is uniform over the 16 lanes of the macro block.
__device__ __forceinline__ Candidate eval_candidate(const float (&xf)[8], uint32_t amax, bool counts, uint32_t e128,
                                                    uint32_t m, uint32_t carry) {
#pragma clang fp contract(off)
    const float F = __uint_as_float(0x3F800000u | (m << 15));
    const float scaled_max = __uint_as_float(amax << 16) * F;  // exact
    uint32_t E = ((__float_as_uint(scaled_max) + carry) >> 23) - 2u;
    E = amax ? E : 127u;
    const float mult = __uint_as_float(((254u - E) << 23) | (m << 15));  // F * 2^(127 - E)
    uint32_t codes = 0;
    float acc = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float t0 = xf[2 * i] * mult, t1 = xf[2 * i + 1] * mult;  // exact
        typedef float v2f __attribute__((ext_vector_type(2)));
        v2f q;
        if (i == 0) { codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, t0, t1, 1.0f, 0); q = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 0); }
        if (i == 1) { codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, t0, t1, 1.0f, 1); q = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 1); }
        if (i == 2) { codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, t0, t1, 1.0f, 2); q = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 2); }
        if (i == 3) { codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, t0, t1, 1.0f, 3); q = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 3); }
        const float r0 = t0 - q.x, r1 = t1 - q.y;  // exact: the grid value is within a factor 2 of t, or t is tiny
        acc = __builtin_fmaf(r0, r0, acc);
        acc = __builtin_fmaf(r1, r1, acc);
    }
    // block sum, then from units of the block's binade to units of the macro block's: 4^(E - e128)
    acc = counts ? acc : 0.0f;
    acc = acc + dpp_quad_xor1_f(acc);
    acc = acc + dpp_quad_xor2_f(acc);
    const float rescale = __uint_as_float(counts ? (127u + 2u * (E - e128)) << 23 : 0x3F800000u);
    acc = acc * rescale;
    acc = acc + dpp_half_mirror_f(acc);
    acc = acc + dpp_mirror_f(acc);
    return {codes, E, acc * __builtin_amdgcn_rcpf(F * F)};
}

__global__ __launch_bounds__(kThreads) void quantize_dynamic_kernel(DynArgs d) {
    const QuantArgs& q = d.q;
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6));
    const uint32_t nwaves = gridDim.x * (kThreads / kWave);
    for (uint32_t c = wave; c < q.total_chunks; c += nwaves) {
        const uint32_t row = c / q.chunks_per_row, col = (c - row * q.chunks_per_row) * kChunk + lane * 8;
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

        // static word (Eq. 3) from the mantissa of the absmax, a subnormal absmax normalised first
        const uint32_t m_static = mbs_word_of_absmax(mmax);
        const uint32_t e128 = mmax >> 7;
        const bool searchable = !nf && e128 >= 64u && e128 <= 249u;
        const bool counts = amax != 0 && (amax >> 7) + 30u >= e128;

        Candidate best = eval_candidate(xf, amax, counts, e128, m_static, q.carry);
        uint32_t m_best = m_static;
        for (int j = 0; j < d.cand_count; ++j) {
            const uint32_t step = (uint32_t)((d.cand_first + j) * d.cand_stride) & 255u;
            if (step == 0) continue;  // the static word again: it cannot beat itself (uniform over the launch)
            uint32_t m = (m_static + step) & 255u;
            m = searchable ? m : m_static;
            const Candidate cand = eval_candidate(xf, amax, counts, e128, m, q.carry);
            if (cand.cost < best.cost) {
                best = cand;
                m_best = m;
            }
        }

        // the fp32 route gave valid codes unless some block of this wavefront lies outside its range
        // (Inf/NaN, or an absmax exponent field outside [24, 249]); then the all-integer path redoes the
        // chunk with the chosen word
        const bool odd = nf_block || (amax >= (250u << 7)) || (amax != 0 && amax < (24u << 7));
        ChunkResult res = {best.codes, best.E, m_best};
        if (__builtin_amdgcn_ballot_w64(odd) != 0) res = quantize_chunk_exact(v, q.rule, 1, (int)m_best);

        uint32_t ew = res.E << (8 * ((lane >> 2) & 3));
        if ((lane & 3) != 0) ew = 0;
        ew |= dpp_row_ror4(ew);
        ew |= dpp_row_ror8(ew);
        if (!valid) continue;
        const uint32_t kblk = col >> 5;
        uint8_t* srow = q.scales + (int64_t)row * (q.K >> 5);
        uint8_t* crow = q.codes + (int64_t)row * (q.K >> 1);
        *reinterpret_cast<uint32_t*>(crow + (col >> 1)) = res.codes;
        if (q.scales_dword) {
            if ((lane & 15) == 0) *reinterpret_cast<uint32_t*>(srow + kblk) = ew;
        } else if ((lane & 3) == 0) {
            srow[kblk] = (uint8_t)res.E;
        }
        if ((lane & 15) == 0) q.mbs[(int64_t)row * q.nmac + (col >> 7)] = (uint8_t)res.m8;
    }
}

// ---- MBS-Dynamic through the table of Eq. 5 (Sec. 4.3.3) ----------------------------
// Eq. 5-6 price a candidate factor by a table of squared relative errors, T[v, m_j] ~ ((x_hat - x) / x)^2 with
// v = |x| SF the element in its block's scaled domain, so that a candidate's sum of squared errors is
// sum_i x_i^2 T[v_ij, m_j].  The table is 2 x 64 points x 16 slots of fp16 (4 KiB, held in LDS): slot j is the
// candidate word 16 j; the "normal" table (v >= 1) is indexed by the 6 leading mantissa bits of v (E2M1's relative
// error repeats from binade to binade), the "sub-normal" one (v < 1) by floor(64 v); an entry is the squared
// relative error at the middle of its bin.  A point's 16 slots lie side by side, so one element costs two 16-byte
// LDS reads and sixteen multiply-adds that take the fp16 entry as it stands (v_fma_mix_f32) for all candidates.
// The candidates only differ in F_j = 1 + j/16 < 2, so a block's local scale takes at most two values over them,
// SF and SF/2 from some j on: both points of an element are priced and each candidate takes the sum that
// belongs to its scale.
struct LutArgs {
    QuantArgs q;
    const uint16_t* lut;
    int keep_static;
};

typedef _Float16 h8 __attribute__((ext_vector_type(8)));

// fp64 -> fp16 bit pattern, round to nearest even (values in [0, 2): no overflow)
__device__ __forceinline__ uint32_t f64_to_f16_bits(double v) {
    const uint64_t u = (uint64_t)__double_as_longlong(v);
    const int e = (int)((u >> 52) & 0x7FF) - 1023;  // v = 1.m * 2^e
    if ((u << 1) == 0) return 0;
    uint64_t m = (u & 0xFFFFFFFFFFFFFull) | (1ull << 52);  // 53 bits, value m * 2^(e - 52)
    int shift;                                              // result = round(m >> shift) in units of the fp16 ulp
    uint32_t base;
    if (e >= -14) { shift = 42; base = (uint32_t)(e + 15 - 1) << 10; }  // normal: 10 mantissa bits, the leading 1 adds to the exponent field
    else { shift = 42 + (-14 - e); base = 0; }                           // subnormal: ulp 2^-24
    if (shift > 63) return 0;
    const uint64_t q = m >> shift, rem = m & ((1ull << shift) - 1), half = 1ull << (shift - 1);
    const uint64_t r = q + ((rem > half || (rem == half && (q & 1))) ? 1 : 0);
    return base + (uint32_t)r;
}

// Entry (table, p, j) of the table, as defined above, in fp64 and rounded once to fp16.
__global__ void mbs_lut_build_kernel(uint16_t* lut) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= 2048) return;
    const int j = idx & 15, p = (idx >> 4) & 63, table = idx >> 10;
    const double F = 1.0 + j / 16.0;
    const double v = table ? 1.0 + (p + 0.5) / 64.0 : (p + 0.5) / 64.0;
    const double t = v * F;  // below 4: the E2M1 grid {0, .5, 1, 1.5, 2, 3, 4}, ties to the even code
    double qv;
    if (t <= 0.25) qv = 0.0;
    else if (t < 0.75) qv = 0.5;
    else if (t <= 1.25) qv = 1.0;
    else if (t < 1.75) qv = 1.5;
    else if (t <= 2.5) qv = 2.0;
    else if (t < 3.5) qv = 3.0;
    else qv = 4.0;
    const double rel = (qv / F - v) / v;
    lut[idx] = (uint16_t)f64_to_f16_bits(rel * rel);
}

__device__ __forceinline__ float dpp_row_ror4_f(float v) { return __uint_as_float(dpp_row_ror4(__float_as_uint(v))); }
__device__ __forceinline__ float dpp_row_ror8_f(float v) { return __uint_as_float(dpp_row_ror8(__float_as_uint(v))); }

__global__ __launch_bounds__(kThreads) void quantize_dynamic_lut_kernel(LutArgs d) {
    __shared__ __attribute__((aligned(16))) uint16_t table[2048];
    reinterpret_cast<u32x4*>(table)[threadIdx.x] = reinterpret_cast<const u32x4*>(d.lut)[threadIdx.x];  // 256 threads x 16 B
    __syncthreads();
    const QuantArgs& q = d.q;
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6));
    const uint32_t nwaves = gridDim.x * (kThreads / kWave);
    for (uint32_t c = wave; c < q.total_chunks; c += nwaves) {
        const uint32_t row = c / q.chunks_per_row, col = (c - row * q.chunks_per_row) * kChunk + lane * 8;
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

        const uint32_t m_static = mbs_word_of_absmax(mmax);
        const uint32_t e128 = mmax >> 7;
        const bool searchable = !nf && e128 >= 64u && e128 <= 249u;
        // (a block more than 30 binades below its window prices at nothing: its x^2 is below 2^-60 of the window's)
        const bool counts = amax != 0 && (amax >> 7) + 30u >= e128;

        // the block's scale byte without a factor, and from which candidate on it is one higher (scale halved)
        const float amax_f = __uint_as_float(amax << 16);
        const uint32_t E0 = ((__float_as_uint(amax_f) + q.carry) >> 23) - 2u;
        uint32_t halved = 0;  // bit j: candidate j quantizes this block with SF / 2
#pragma unroll
        for (int j = 1; j < 16; ++j) {
            const float scaled = amax_f * __uint_as_float(0x3F800000u | ((uint32_t)j << 19));  // absmax * (1 + j/16), exact
            const uint32_t Ej = ((__float_as_uint(scaled) + q.carry) >> 23) - 2u;
            halved |= (Ej != E0 ? 1u : 0u) << j;
        }
        // elements in the block's scaled domain, v = |x| 2^(127 - E0), and, for the sums, in the window's: xn = x 2^(127 - e128)
        const float to_block = __uint_as_float(counts ? (254u - E0) << 23 : 0u);
        const float to_window = __uint_as_float(searchable ? (254u - e128) << 23 : 0u);
        float cost_hi[16], cost_lo[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) cost_hi[j] = cost_lo[j] = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float vh = __builtin_fabsf(xf[i]) * to_block;  // exact; at most 8
            const float xn = xf[i] * to_window, x2 = xn * xn;
            const uint32_t vb = __float_as_uint(vh);
            // points of v and of v / 2: normal table rows 64 .. 127 by the mantissa, sub-normal rows 0 .. 63 by floor(64 v)
            const uint32_t mant = (vb >> 17) & 63u;
            const uint32_t sub = (uint32_t)(vh * 64.0f);  // (only used below 1)
            const uint32_t row_hi = vh >= 1.0f ? 64u + mant : sub;
            const uint32_t row_lo = vh >= 2.0f ? 64u + mant : vh >= 1.0f ? 32u + (mant >> 1) : sub >> 1;
            const h8* ph = reinterpret_cast<const h8*>(table + row_hi * 16);
            const h8* pl = reinterpret_cast<const h8*>(table + row_lo * 16);
            const h8 h0 = ph[0], h1 = ph[1], l0 = pl[0], l1 = pl[1];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                cost_hi[j] = __builtin_fmaf(x2, (float)h0[j], cost_hi[j]);
                cost_hi[8 + j] = __builtin_fmaf(x2, (float)h1[j], cost_hi[8 + j]);
                cost_lo[j] = __builtin_fmaf(x2, (float)l0[j], cost_lo[j]);
                cost_lo[8 + j] = __builtin_fmaf(x2, (float)l1[j], cost_lo[8 + j]);
            }
        }
        // every candidate takes the sum of its scale, then the sums of the window's 16 lanes are added up
        float cost[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) cost[j] = (halved >> j) & 1u ? cost_lo[j] : cost_hi[j];
        // (step by step over all candidates: sixteen independent chains leave no wait state between an add and the next)
#pragma unroll
        for (int j = 0; j < 16; ++j) cost[j] += dpp_quad_xor1_f(cost[j]);
#pragma unroll
        for (int j = 0; j < 16; ++j) cost[j] += dpp_quad_xor2_f(cost[j]);
#pragma unroll
        for (int j = 0; j < 16; ++j) cost[j] += dpp_row_ror4_f(cost[j]);
#pragma unroll
        for (int j = 0; j < 16; ++j) cost[j] += dpp_row_ror8_f(cost[j]);
        uint32_t j_best = 0;
        float best = cost[0];
#pragma unroll
        for (int j = 1; j < 16; ++j) {
            if (cost[j] < best) {
                best = cost[j];
                j_best = (uint32_t)j;
            }
        }
        uint32_t m_pick = searchable ? 16u * j_best : m_static;
        // codes and scale byte of the picked word; with keep_static the static word stays unless the picked one's
        // true sum of squared errors (the fp32 sum of the exact search) is smaller
        Candidate cand = eval_candidate(xf, amax, counts, e128, m_pick, q.carry);
        if (d.keep_static && m_pick != m_static) {
            const Candidate stat = eval_candidate(xf, amax, counts, e128, m_static, q.carry);
            if (stat.cost <= cand.cost) {
                cand = stat;
                m_pick = m_static;
            }
        }
        const bool odd = nf_block || (amax >= (250u << 7)) || (amax != 0 && amax < (24u << 7));
        ChunkResult res = {cand.codes, cand.E, m_pick};
        if (__builtin_amdgcn_ballot_w64(odd) != 0) res = quantize_chunk_exact(v, q.rule, 1, (int)m_pick);

        uint32_t ew = res.E << (8 * ((lane >> 2) & 3));
        if ((lane & 3) != 0) ew = 0;
        ew |= dpp_row_ror4(ew);
        ew |= dpp_row_ror8(ew);
        if (!valid) continue;
        const uint32_t kblk = col >> 5;
        uint8_t* srow = q.scales + (int64_t)row * (q.K >> 5);
        uint8_t* crow = q.codes + (int64_t)row * (q.K >> 1);
        *reinterpret_cast<uint32_t*>(crow + (col >> 1)) = res.codes;
        if (q.scales_dword) {
            if ((lane & 15) == 0) *reinterpret_cast<uint32_t*>(srow + kblk) = ew;
        } else if ((lane & 3) == 0) {
            srow[kblk] = (uint8_t)res.E;
        }
        if ((lane & 15) == 0) q.mbs[(int64_t)row * q.nmac + (col >> 7)] = (uint8_t)res.m8;
    }
}

int launch_filled(const QuantArgs& q, int use_mbs, void* stream, bool hwcvt = true);

// argument checks and the fields common to both quantizer kernels; MX_OK with *empty set means nothing to do
int fill_quant_args(QuantArgs& q, bool* empty, const void* x, int64_t rows, int64_t K, int64_t ldx, int rule, int use_mbs,
                    uint8_t* codes, uint8_t* scales, uint8_t* mbs, bool device_check = true) {
    *empty = true;
    if (rows < 0 || K < 0 || (K % kBlock) != 0 || ldx < K || K > kMaxK) return MX_EINVAL;
    if (rule != MX_RULE_OCP && rule != MX_RULE_FLOOR && rule != MX_RULE_OAS) return MX_EINVAL;
    if (rows == 0 || K == 0) return MX_OK;
    if (!x || !codes || !scales || (use_mbs && !mbs)) return MX_ENULL;
    if (!aligned(x, 16) || (ldx % 8) != 0 || !aligned(codes, 16)) return MX_EALIGN;
    if (device_check)
        if (int st = check_device()) return st;
    q.x = static_cast<const uint16_t*>(x);
    q.codes = codes;
    q.scales = scales;
    q.mbs = mbs;
    q.K = K;
    q.ldx = ldx;
    const int64_t cpr = (K + kChunk - 1) / kChunk;
    if (cpr * rows >= ((int64_t)1 << 32)) return MX_EINVAL;  // chunk ids are 32-bit
    q.chunks_per_row = (uint32_t)cpr;
    q.total_chunks = (uint32_t)(cpr * rows);
    q.nmac = (K + kMacro - 1) / kMacro;
    q.rule = rule;
    q.use_mbs = use_mbs;
    q.carry = rule_carry(rule);
    q.scales_dword = (K % kMacro) == 0 && aligned(scales, 4);
    q.x2 = nullptr;
    q.codes2 = q.scales2 = q.mbs2 = nullptr;
    q.ldx2 = 0;
    q.split = q.total_chunks;
    q.total_chunks2 = 0;
    *empty = false;
    return MX_OK;
}

int launch_quantize(const void* x, int64_t rows, int64_t K, int64_t ldx, int rule, int use_mbs,
                    uint8_t* codes, uint8_t* scales, uint8_t* mbs, void* stream, bool hwcvt = true) {
    QuantArgs q;
    bool empty;
    if (int st = fill_quant_args(q, &empty, x, rows, K, ldx, rule, use_mbs, codes, scales, mbs)) return st;
    if (empty) return MX_OK;
    return launch_filled(q, use_mbs, stream, hwcvt);
}

// Two tensors with the same K (the two operands of a GEMM) in one launch: the smaller one no longer pays
// for a launch and a ramp of its own.
int launch_quantize_pair(const void* x0, int64_t rows0, int64_t ldx0, uint8_t* codes0, uint8_t* scales0, uint8_t* mbs0,
                         const void* x1, int64_t rows1, int64_t ldx1, uint8_t* codes1, uint8_t* scales1, uint8_t* mbs1,
                         int64_t K, int rule, void* stream) {
    QuantArgs q0, q1;
    bool empty0, empty1;
    if (int st = fill_quant_args(q0, &empty0, x0, rows0, K, ldx0, rule, 1, codes0, scales0, mbs0, false)) return st;
    if (int st = fill_quant_args(q1, &empty1, x1, rows1, K, ldx1, rule, 1, codes1, scales1, mbs1, false)) return st;
    if (empty0 && empty1) return MX_OK;
    if (int st = check_device()) return st;
    if (empty0) return launch_filled(q1, 1, stream);
    if (empty1) return launch_filled(q0, 1, stream);
    const int64_t split = ((int64_t)q0.total_chunks + kUnroll - 1) / kUnroll * kUnroll;
    if (split + q1.total_chunks >= ((int64_t)1 << 32)) return MX_EINVAL;  // chunk ids are 32-bit
    q0.x2 = q1.x;
    q0.codes2 = q1.codes;
    q0.scales2 = q1.scales;
    q0.mbs2 = q1.mbs;
    q0.ldx2 = q1.ldx;
    q0.split = (uint32_t)split;
    q0.total_chunks2 = q1.total_chunks;
    q0.scales_dword = q0.scales_dword && q1.scales_dword;
    return launch_filled(q0, 1, stream);
}

int launch_filled(const QuantArgs& q, int use_mbs, void* stream, bool hwcvt) {
    const int64_t waves_needed = ((int64_t)q.split + q.total_chunks2 + kUnroll - 1) / kUnroll;
    int64_t blocks = (waves_needed + (kThreads / kWave) - 1) / (kThreads / kWave);
    // one batch of kUnroll chunks per wavefront (the hardware balances the workgroups); the loop in
    // the kernel only matters beyond this cap
    const int64_t max_blocks = 1 << 22;
    if (blocks > max_blocks) blocks = max_blocks;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)blocks), block(kThreads);
    if (hwcvt) {
        if (use_mbs) hipLaunchKernelGGL((quantize_kernel<true, true>), grid, block, 0, s, q);
        else hipLaunchKernelGGL((quantize_kernel<true, false>), grid, block, 0, s, q);
    } else {
        if (use_mbs) hipLaunchKernelGGL((quantize_kernel<false, true>), grid, block, 0, s, q);
        else hipLaunchKernelGGL((quantize_kernel<false, false>), grid, block, 0, s, q);
    }
    return launch_status();
}

int launch_quantize_dynamic(const void* x, int64_t rows, int64_t K, int64_t ldx, int rule, int cand_first,
                            int cand_count, int cand_stride, uint8_t* codes, uint8_t* scales, uint8_t* mbs,
                            void* stream) {
    constexpr int kCandLimit = 1 << 16;  // keeps (cand_first + j) * cand_stride inside 32 bits
    if (cand_count < 0 || cand_count > 256 || cand_first < -kCandLimit || cand_first > kCandLimit ||
        cand_stride < -kCandLimit || cand_stride > kCandLimit)
        return MX_EINVAL;
    DynArgs d;
    bool empty;
    if (int st = fill_quant_args(d.q, &empty, x, rows, K, ldx, rule, 1, codes, scales, mbs)) return st;
    if (empty) return MX_OK;
    d.cand_first = cand_first;
    d.cand_count = cand_count;
    d.cand_stride = cand_stride;
    // one chunk per wavefront and step: the kernel is bound by arithmetic, not by loads in flight
    int64_t blocks = ((int64_t)d.q.total_chunks + (kThreads / kWave) - 1) / (kThreads / kWave);
    const int64_t max_blocks = 1 << 20;
    if (blocks > max_blocks) blocks = max_blocks;
    hipLaunchKernelGGL(quantize_dynamic_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, static_cast<hipStream_t>(stream), d);
    return launch_status();
}

int launch_quantize_dynamic_lut(const void* x, int64_t rows, int64_t K, int64_t ldx, int rule, const uint16_t* lut,
                                int keep_static, uint8_t* codes, uint8_t* scales, uint8_t* mbs, void* stream) {
    LutArgs d;
    bool empty;
    if (int st = fill_quant_args(d.q, &empty, x, rows, K, ldx, rule, 1, codes, scales, mbs, false)) return st;
    if (empty) return MX_OK;
    if (!lut) return MX_ENULL;
    if (!aligned(lut, 16)) return MX_EALIGN;
    if (int st = check_device()) return st;
    d.lut = lut;
    d.keep_static = keep_static != 0;
    int64_t blocks = ((int64_t)d.q.total_chunks + (kThreads / kWave) - 1) / (kThreads / kWave);
    const int64_t max_blocks = 1 << 20;
    if (blocks > max_blocks) blocks = max_blocks;
    hipLaunchKernelGGL(quantize_dynamic_lut_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, static_cast<hipStream_t>(stream), d);
    return launch_status();
}

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
uint16_t* g_scratch_ptr[kMaxDevices];  // guarded by g_scratch_mutex; null until looked up

int scratch_for_current_device(uint16_t** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return MX_ELAUNCH;
    if (dev < 0 || dev >= kMaxDevices) return MX_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return MX_ELAUNCH;
        }
        g_scratch_ptr[dev] = static_cast<uint16_t*>(p);
    }
    *out = g_scratch_ptr[dev];
    return MX_OK;
}

}  // namespace
}  // namespace mx

extern "C" {

int mx_quantize_mbs_dynamic_lut_static(const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule,
                                       int keep_static, uint8_t* codes, uint8_t* scales, uint8_t* mbs,
                                       void* stream) {
    // argument errors first, as in the entry point this one is a variant of (nothing is launched on an error)
    {
        mx::QuantArgs probe;
        bool empty;
        if (int st = mx::fill_quant_args(probe, &empty, x_bf16, rows, K, ldx, (int)rule, 1, codes, scales, mbs, false)) return st;
        if (empty) return MX_OK;
    }
    if (int st = mx::check_device()) return st;
    uint16_t* table = nullptr;
    if (int st = mx::scratch_for_current_device(&table)) return st;
    // The array keeps whatever the last call on this GPU left, and a first call finds it zero: every call
    // writes the whole table on its own stream in front of the kernel that reads it.
    hipLaunchKernelGGL(mx::mbs_lut_build_kernel, dim3(8), dim3(256), 0, static_cast<hipStream_t>(stream), table);
    if (int st = mx::launch_status()) return st;
    return mx::launch_quantize_dynamic_lut(x_bf16, rows, K, ldx, (int)rule, table, keep_static, codes, scales, mbs, stream);
}

int mx_mbs_lut_build(uint16_t* lut_fp16, void* stream) {
    if (!lut_fp16) return MX_ENULL;
    if (!mx::aligned(lut_fp16, 16)) return MX_EALIGN;
    if (int st = mx::check_device()) return st;
    hipLaunchKernelGGL(mx::mbs_lut_build_kernel, dim3(8), dim3(256), 0, static_cast<hipStream_t>(stream), lut_fp16);
    return mx::launch_status();
}

int mx_quantize_mbs_dynamic_lut(const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule,
                                const uint16_t* lut_fp16, int keep_static, uint8_t* codes, uint8_t* scales,
                                uint8_t* mbs, void* stream) {
    return mx::launch_quantize_dynamic_lut(x_bf16, rows, K, ldx, (int)rule, lut_fp16, keep_static, codes, scales, mbs, stream);
}

int mx_quantize(const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule,
                uint8_t* codes, uint8_t* scales, void* stream) {
    return mx::launch_quantize(x_bf16, rows, K, ldx, (int)rule, 0, codes, scales, nullptr, stream);
}

int mx_quantize_oas(const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, uint8_t* codes,
                    uint8_t* scales, void* stream) {
    return mx::launch_quantize(x_bf16, rows, K, ldx, MX_RULE_OAS, 0, codes, scales, nullptr, stream);
}

int mx_quantize_mbs(const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule,
                    uint8_t* codes, uint8_t* scales, uint8_t* mbs, void* stream) {
    return mx::launch_quantize(x_bf16, rows, K, ldx, (int)rule, 1, codes, scales, mbs, stream);
}

int mx_quantize_mbs_pair(const void* x0_bf16, int64_t rows0, int64_t ldx0, uint8_t* codes0, uint8_t* scales0,
                         uint8_t* mbs0, const void* x1_bf16, int64_t rows1, int64_t ldx1, uint8_t* codes1,
                         uint8_t* scales1, uint8_t* mbs1, int64_t K, mx_rule_t rule, void* stream) {
    return mx::launch_quantize_pair(x0_bf16, rows0, ldx0, codes0, scales0, mbs0, x1_bf16, rows1, ldx1, codes1, scales1,
                                    mbs1, K, (int)rule, stream);
}

int mx_quantize_mbs_dynamic(const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule,
                            int32_t cand_first, int32_t cand_count, int32_t cand_stride, uint8_t* codes,
                            uint8_t* scales, uint8_t* mbs, void* stream) {
    return mx::launch_quantize_dynamic(x_bf16, rows, K, ldx, (int)rule, cand_first, cand_count, cand_stride, codes,
                                       scales, mbs, stream);
}

int mx_internal_quantize(const void* x_bf16, int64_t rows, int64_t K, int64_t ldx, mx_rule_t rule, int use_mbs,
                         int hw_convert, uint8_t* codes, uint8_t* scales, uint8_t* mbs, void* stream) {
    return mx::launch_quantize(x_bf16, rows, K, ldx, (int)rule, use_mbs ? 1 : 0, codes, scales, mbs, stream, hw_convert != 0);
}

}  // extern "C"
