// Block-scaled MXFP4 GEMM  C = A * B^T  with the Macro Block Scaling correction, for gfx950.
//
// The contraction runs on v_mfma_scale_f32_16x16x128_f8f6f4 in FP4 mode.  One instruction is
// exactly one macro block deep (128 K-elements = 4 E8M0 blocks), which is the granularity at
// which the MBS correction has to be applied (App. E): with MBS every instruction starts from a
// zero accumulator and its 16x16 partial product is folded into the running fp32 result as
//     acc[i,j] += P_g[i,j] * sigma_A[i,g] * sigma_B[j,g],      sigma = 1/(1 + m8/256)   (Sec. 4.3.2)
// on the vector ALUs; without MBS the instructions chain their accumulators.
//
// Operand mapping of the instruction (64 lanes, lane = 16 q + r):
//   srcA: 16 rows x 128 k;  lane holds row r, k-block q: 32 FP4 = 16 bytes (4 of the 8 operand VGPRs)
//   srcB: 16 cols x 128 k;  lane holds col r, k-block q
//   scale operands: one E8M0 byte per lane (for its row/col and k-block), picked out of a VGPR
//                   by a per-instruction byte selector
//   D:    lane holds D[4 q + i][r], i = 0..3
// The weight matrix B feeds srcA and the activation matrix A feeds srcB, so that a lane ends up
// with four consecutive n of one output row m and stores them as one vector.
//
// Tiling: a workgroup of NWM x NWN wavefronts computes a TM x TN tile of C, each wavefront
// FM x FN 16x16 fragments.  FP4 operands are so small next to the MFMA rate (4096 FLOP/clk/SIMD)
// that the tile has to be large for the L2 to keep up: a T x T tile moves 1/(2T) bytes per FLOP.
// K advances in stages of 256 elements (two macro blocks, one 128-byte line per row and operand),
// double-buffered in LDS.  The codes go from global memory straight into LDS (buffer loads with
// the LDS bit) as a row-major image with XOR-swizzled 16-byte chunks: eight lanes fetch one full
// 128-byte line, and the 16-byte fragment reads of the multiply phase are bank-conflict free.
// Buffer resources are sized to the tile's valid rows, so ragged tiles read zeros without a branch.  The E8M0 bytes and the sigma values
// are staged through registers: the scales are regrouped so that one dword holds the bytes of
// four fragments for a given lane (the instruction's byte selector then picks the fragment), and
// the MBS words are turned into fp32 sigma once per (row, macro block).
#include <utility>

#include "mx_common.h"

namespace mx {
namespace {

constexpr int kStageK = 256;  // K elements per pipeline stage
constexpr int kStageMacros = kStageK / kMacro;
constexpr int kFragBytes = 1024;  // 16 rows x 128 FP4
constexpr int kGroupM = 8;        // tile-rows walked together for L2 reuse

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;

template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Tile shape: NWM x NWN wavefronts, each FM x FN fragments of 16 x 16 outputs.
template <int NWM_, int NWN_, int FM_, int FN_, int NBUF_>
struct Shape {
    static constexpr int NWM = NWM_, NWN = NWN_, FM = FM_, FN = FN_;
    static constexpr int NBUF = NBUF_;  // code stages in LDS; NBUF - 1 stages are in flight while one is multiplied
    static constexpr int NW = NWM * NWN, NT = NW * kWave;
    static constexpr int TM = NWM * FM * 16, TN = NWN * FN * 16;
    // LDS map: NBUF x [codes m | n], then 2 x [scale_m | scale_n | sigma_m | sigma_n]
    static constexpr int kCodesStage = (TM + TN) * (kStageK / 2);
    static constexpr int kSmallBase = NBUF * kCodesStage;
    static constexpr int kScaleM = 0;                                // u32 [macro][TM/64][64]
    static constexpr int kScaleN = kScaleM + kStageMacros * TM * 4;  // u32 [macro][TN/64][64]
    static constexpr int kSigmaM = kScaleN + kStageMacros * TN * 4;  // f32 [macro][TM]
    static constexpr int kSigmaN = kSigmaM + kStageMacros * TM * 4;  // f32 [macro][TN]
    static constexpr int kSmallStage = kSigmaN + kStageMacros * TN * 4;
    static constexpr int kLdsBytes = kSmallBase + 2 * kSmallStage;
    static_assert(FM == 2 || FM % 4 == 0, "fragment count per wave: 2 or a multiple of 4");
    static_assert(FN == 2 || FN % 4 == 0, "fragment count per wave: 2 or a multiple of 4");
    static_assert((TM / 8) % NW == 0 && (TN / 8) % NW == 0, "8-row loads per wave");
    static_assert(TM % 64 == 0 && TN % 64 == 0, "scale dwords group four fragments");
    static_assert(NBUF == 2 || NBUF == 3, "double or triple buffering");
    static_assert(kLdsBytes <= 160 * 1024, "LDS capacity of a gfx950 compute unit");
};

struct GemmArgs {
    const uint8_t *a_codes, *a_scales, *a_mbs;
    const uint8_t *b_codes, *b_scales, *b_mbs;
    void* C;
    const int64_t* row_offsets;  // grouped mode only
    int64_t M, N, K, ldc;
    int num_groups;              // 0 = plain GEMM
    int tiles_m, tiles_n;        // tile grid (tiles_m is an upper bound in grouped mode)
    int c_bf16;
    int vec_store;               // C rows allow 4-element vector stores
};

// One operand (A or B) of the tile as the loader sees it: buffer resources rebased to the tile's first
// row and sized to its valid rows, so that rows past the end read as zero without any branch.
struct Operand {
    __amdgpu_buffer_rsrc_t codes, scales, mbs;
    int row_bytes;    // K / 2
    int scale_bytes;  // K / 32
    int nmac;         // ceil(K / 128)
};

__device__ __forceinline__ Operand make_operand(const uint8_t* codes, const uint8_t* scales, const uint8_t* mbs,
                                                int64_t row0, int64_t row_end, int tile_rows, int64_t K) {
    Operand op;
    const int64_t rows = row_end > row0 ? (row_end - row0 < tile_rows ? row_end - row0 : tile_rows) : 0;
    op.row_bytes = (int)(K >> 1);
    op.scale_bytes = (int)(K >> 5);
    op.nmac = (int)((K + kMacro - 1) / kMacro);
    const int kRsrcFlags = 0x00020000;  // raw buffer, 32-bit data format
    op.codes = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(codes) + row0 * op.row_bytes, 0,
                                                 (int)(rows * op.row_bytes), kRsrcFlags);
    op.scales = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(scales) + row0 * op.scale_bytes, 0,
                                                  (int)(rows * op.scale_bytes), kRsrcFlags);
    op.mbs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(mbs ? mbs + row0 * op.nmac : codes), 0,
                                               mbs ? (int)(rows * op.nmac) : 0, kRsrcFlags);
    return op;
}

constexpr int kOob = 0x7FFFFFF0;  // byte offset beyond any buffer: the load returns zero

// Codes of one stage straight into LDS.  The LDS image of an operand is row-major, 128 bytes (the
// stage's 256 k) per row, with the eight 16-byte chunks of a row XOR-swizzled by (row >> 1) & 7:
// chunk c of row r sits at r * 128 + ((c ^ ((r >> 1) & 7)) * 16).  A wavefront-wide load covers 8 rows;
// lane l writes LDS slot l (hardware order) and therefore fetches row l / 8, chunk (l % 8) ^ swizzle:
// eight lanes read one full 128-byte line of global memory, and the later fragment reads (16 lanes =
// 16 consecutive rows, one chunk each) hit 16 distinct 16-byte bank groups.
template <int kRows, int NW, bool kRaggedK>
__device__ __forceinline__ void load_codes(const Operand& op, uint8_t* lds_codes, int64_t K, int k0, int tid) {
    const int w = tid >> 6, l = tid & 63;
    constexpr int kLoads = kRows / 8 / NW;
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
        const int row0 = (i * NW + w) * 8;
        const int row = row0 + (l >> 3);
        const int c = (l & 7) ^ ((row >> 1) & 7);
        int voff = row * op.row_bytes + c * 16;
        if (kRaggedK && k0 + c * kBlock >= K) voff = kOob;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(op.codes, (lds_ptr_t)(lds_codes + row0 * (kStageK / 2)), 16, voff,
                                                 k0 >> 1, 0, 0);
    }
}

struct Small {
    uint32_t scale;  // the four E8M0 bytes of one (row, macro block)
    uint32_t m8;
};

// (row, macro block) pair p of the stage: its four E8M0 bytes and its MBS word.
template <int kRows, bool kMbs, bool kScaleDword>
__device__ __forceinline__ Small load_small(const Operand& op, int64_t K, int k0, int p) {
    const int row = p >> 1;  // two lanes share a row, i.e. a cache line of scales
    const int g = k0 / kMacro + (p & 1);
    Small r;
    const int off = row * op.scale_bytes + g * 4;
    const bool have = g * kMacro < K && p < kRows * kStageMacros;
    if (kScaleDword) {
        r.scale = __builtin_amdgcn_raw_buffer_load_b32(op.scales, have ? off : kOob, 0, 0);
    } else {
        // rows are not dword aligned or the last macro block is short: byte loads, absent blocks read 0
        r.scale = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int o = have && g * kMacro + j * kBlock < K ? off + j : kOob;
            r.scale |= (uint32_t)__builtin_amdgcn_raw_buffer_load_b8(op.scales, o, 0, 0) << (8 * j);
        }
    }
    r.m8 = 0;
    if (kMbs) r.m8 = __builtin_amdgcn_raw_buffer_load_b8(op.mbs, have ? row * op.nmac + g : kOob, 0, 0);
    return r;
}

// Scale bytes regrouped: dword [macro][row / 64][16 q + row % 16] byte (row / 16) % 4 = E8M0 of k-block q.
template <int kRows, bool kMbs>
__device__ __forceinline__ void store_small(const Small& v, uint8_t* scale, uint8_t* sigma, int p) {
    if (p >= kRows * kStageMacros) return;
    const int row = p >> 1, mb = p & 1;
    const int group = row >> 6, frag = (row >> 4) & 3, r = row & 15;
    uint8_t* sb = scale + ((mb * (kRows / 64) + group) * kWave) * 4;
#pragma unroll
    for (int q = 0; q < 4; ++q) sb[(q * 16 + r) * 4 + frag] = (uint8_t)(v.scale >> (8 * q));
    // sigma = 1/F to within an ulp (the hardware reciprocal); F = 1 + m8/256 is exact
    if (kMbs) reinterpret_cast<float*>(sigma)[mb * kRows + row] = __builtin_amdgcn_rcpf(1.0f + (float)v.m8 * (1.0f / 256.0f));
}

template <int kSelN, int kSelM>
__device__ __forceinline__ v4f mfma_fp4(v4i n_frag, v4i m_frag, v4f c, uint32_t scale_n, uint32_t scale_m) {
    const v8i a = __builtin_shufflevector(n_frag, n_frag, 0, 1, 2, 3, -1, -1, -1, -1);
    const v8i b = __builtin_shufflevector(m_frag, m_frag, 0, 1, 2, 3, -1, -1, -1, -1);
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 4 /*A: FP4*/, 4 /*B: FP4*/, kSelN,
                                                            (int)scale_n, kSelM, (int)scale_m);
}

// kMbs: apply the per-macro-block correction; kScaleDword: the four E8M0 bytes of a macro block are an
// aligned dword (K % 128 == 0, 4-byte aligned scale arrays); kRaggedK: K is not a multiple of the stage.
template <typename S, bool kMbs, bool kScaleDword, bool kRaggedK>
__global__ __launch_bounds__(S::NT, 2) void gemm_kernel(GemmArgs g) {
    constexpr int FM = S::FM, FN = S::FN, TM = S::TM, TN = S::TN, NT = S::NT, NW = S::NW;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- which tile --------------------------------------------------------------------------
    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tiles and
    // walk tiles in bands of kGroupM tile-rows so that concurrently running workgroups share
    // operand panels in their XCD's L2.
    const int total = g.tiles_m * g.tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int linear = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || linear >= total) return;
    const int band = kGroupM * g.tiles_n;
    const int first_m = (linear / band) * kGroupM;
    const int band_rows = min(g.tiles_m - first_m, kGroupM);
    int tm = first_m + (linear % band) % band_rows;
    const int tn = (linear % band) / band_rows;

    int64_t a_row0 = (int64_t)tm * TM, a_end = g.M;
    int64_t b_row0 = (int64_t)tn * TN, b_end = g.N;
    if (g.num_groups > 0) {
        // tm counts tiles over all groups; find the group that owns it
        int e = 0;
        int64_t lo = 0, hi = 0;
        bool found = false;
        for (; e < g.num_groups; ++e) {
            lo = g.row_offsets[e];
            hi = g.row_offsets[e + 1];
            const int nt = (int)((hi - lo + TM - 1) / TM);
            if (tm < nt) { found = true; break; }
            tm -= nt;
        }
        if (!found) return;
        a_row0 = lo + (int64_t)tm * TM;
        a_end = hi;
        b_row0 += (int64_t)e * g.N;
        b_end = (int64_t)e * g.N + g.N;
    }
    const Operand opa = make_operand(g.a_codes, g.a_scales, g.a_mbs, a_row0, a_end, TM, g.K);
    const Operand opb = make_operand(g.b_codes, g.b_scales, g.b_mbs, b_row0, b_end, TN, g.K);

    const int tid = threadIdx.x, l = tid & 63, w = tid >> 6;
    const int wm = w % S::NWM, wn = w / S::NWM;  // position of this wavefront in the tile

    v4f acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};

    constexpr int kPairsM = (TM * kStageMacros + NT - 1) / NT, kPairsN = (TN * kStageMacros + NT - 1) / NT;
    constexpr int kDepth = S::NBUF - 1;  // code stages in flight
    // Direct-to-LDS loads one wavefront issues per stage.  They complete in order, so "at most
    // (kDepth - 1) stages' worth outstanding" means the oldest stage in flight has landed.
    constexpr int kDmaPerStage = (TM + TN) / 8 / NW;
    constexpr int kWaitOps = (kDepth - 1) * kDmaPerStage;
    static_assert(kWaitOps < 64, "vmcnt is a 6-bit counter");
    // s_waitcnt vmcnt(kWaitOps) lgkmcnt(0): the landed stage plus this wavefront's own LDS stores
    constexpr int kWaitImm = (kWaitOps & 0xF) | ((kWaitOps >> 4) << 14) | 0x0070;

    auto issue_codes = [&](int s) {
        uint8_t* cbase = smem + (s % S::NBUF) * S::kCodesStage;
        const int k0 = s * kStageK;
        load_codes<TM, NW, kRaggedK>(opa, cbase, g.K, k0, tid);
        load_codes<TN, NW, kRaggedK>(opb, cbase + TM * (kStageK / 2), g.K, k0, tid);
    };
    auto issue_small = [&](int s, Small (&sa)[kPairsM], Small (&sb)[kPairsN]) {
        const int k0 = s * kStageK;
#pragma unroll
        for (int i = 0; i < kPairsM; ++i) sa[i] = load_small<TM, kMbs, kScaleDword>(opa, g.K, k0, i * NT + tid);
#pragma unroll
        for (int i = 0; i < kPairsN; ++i) sb[i] = load_small<TN, kMbs, kScaleDword>(opb, g.K, k0, i * NT + tid);
    };
    // Publish stage s: its scales and sigmas go to small slot s % 2 (last read two stages ago); its
    // codes have landed once at most kWaitOps younger direct-to-LDS loads are outstanding.
    auto commit_stage = [&](int s, const Small (&sa)[kPairsM], const Small (&sb)[kPairsN]) {
        uint8_t* sbase = smem + S::kSmallBase + (s & 1) * S::kSmallStage;
#pragma unroll
        for (int i = 0; i < kPairsM; ++i)
            store_small<TM, kMbs>(sa[i], sbase + S::kScaleM, sbase + S::kSigmaM, i * NT + tid);
#pragma unroll
        for (int i = 0; i < kPairsN; ++i)
            store_small<TN, kMbs>(sb[i], sbase + S::kScaleN, sbase + S::kSigmaN, i * NT + tid);
        __builtin_amdgcn_s_waitcnt(kWaitImm);
        // Workgroup barrier as a bare instruction: the compiler's own barrier intrinsic forces a wait for
        // ALL outstanding vector-memory operations, which would drain the younger stages still in flight.
        asm volatile("s_barrier" ::: "memory");
    };

    // byte offset of this lane's 16 bytes inside a 16-row block of the swizzled LDS image, per macro block
    int frag_off[kStageMacros];
#pragma unroll
    for (int mb = 0; mb < kStageMacros; ++mb)
        frag_off[mb] = (l & 15) * (kStageK / 2) + (((mb * 4 + (l >> 4)) ^ ((l & 15) >> 1)) * 16);

    const int nstages = (int)((g.K + kStageK - 1) / kStageK);
    if (nstages > 0) {
        Small sa[kPairsM], sb[kPairsN];
        issue_codes(0);
        issue_small(0, sa, sb);
#pragma unroll
        for (int d = 1; d < kDepth; ++d) issue_codes(d);
        commit_stage(0, sa, sb);
    }

    for (int s = 0; s < nstages; ++s) {
        const uint8_t* cm = smem + (s % S::NBUF) * S::kCodesStage;
        const uint8_t* cn = cm + TM * (kStageK / 2);
        const uint8_t* sm_base = smem + S::kSmallBase + (s & 1) * S::kSmallStage;
        // The register-staged scales of the next stage first, then the codes of stage s + kDepth into
        // the buffer that was read last in the previous iteration (every wavefront is past the barrier
        // that ended it).  In this order, "the scales have arrived" implies that every older
        // direct-to-LDS load has landed too.  Unconditional, so that the loop body stays one basic
        // block: past the end of K the loads are out of range or land in rows nobody reads.
        Small sa[kPairsM], sb[kPairsN];
        issue_small(s + 1, sa, sb);
        issue_codes(s + kDepth);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mb = 0; mb < kStageMacros; ++mb) {
            v4i m_frag[FM], n_frag[FN];
            float sig_m[FM];
            v4f sig_n[FN];
            uint32_t scl_m[(FM + 3) / 4], scl_n[(FN + 3) / 4];
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                m_frag[i] = *reinterpret_cast<const v4i*>(cm + (wm * FM + i) * (16 * kStageK / 2) + frag_off[mb]);
                if constexpr (kMbs)
                    sig_m[i] = reinterpret_cast<const float*>(sm_base + S::kSigmaM)[mb * TM + (wm * FM + i) * 16 + (l & 15)];
            }
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                n_frag[j] = *reinterpret_cast<const v4i*>(cn + (wn * FN + j) * (16 * kStageK / 2) + frag_off[mb]);
                if constexpr (kMbs)
                    sig_n[j] = *reinterpret_cast<const v4f*>(sm_base + S::kSigmaN +
                                                             (mb * TN + (wn * FN + j) * 16 + (l >> 4) * 4) * 4);
            }
            // scale dwords: group = (first fragment) / 4; a 2-fragment wave uses half a dword
#pragma unroll
            for (int d = 0; d < (FM + 3) / 4; ++d) {
                const int group = (wm * FM) / 4 + d;
                scl_m[d] = reinterpret_cast<const uint32_t*>(sm_base + S::kScaleM)[(mb * (TM / 64) + group) * kWave + l];
                if (FM == 2) scl_m[d] >>= 16 * (wm & 1);
            }
#pragma unroll
            for (int d = 0; d < (FN + 3) / 4; ++d) {
                const int group = (wn * FN) / 4 + d;
                scl_n[d] = reinterpret_cast<const uint32_t*>(sm_base + S::kScaleN)[(mb * (TN / 64) + group) * kWave + l];
                if (FN == 2) scl_n[d] >>= 16 * (wn & 1);
            }
            static_for<FM>([&](auto mi) {
                static_for<FN>([&](auto ni) {
                    constexpr int i = decltype(mi)::value, j = decltype(ni)::value;
                    if constexpr (kMbs) {
                        const v4f zero = {0.f, 0.f, 0.f, 0.f};
                        const v4f p = mfma_fp4<j % 4, i % 4>(n_frag[j], m_frag[i], zero, scl_n[j / 4], scl_m[i / 4]);
                        const float sa_ = sig_m[i];
                        acc[i][j].x = fmaf(p.x, sa_ * sig_n[j].x, acc[i][j].x);
                        acc[i][j].y = fmaf(p.y, sa_ * sig_n[j].y, acc[i][j].y);
                        acc[i][j].z = fmaf(p.z, sa_ * sig_n[j].z, acc[i][j].z);
                        acc[i][j].w = fmaf(p.w, sa_ * sig_n[j].w, acc[i][j].w);
                    } else {
                        acc[i][j] = mfma_fp4<j % 4, i % 4>(n_frag[j], m_frag[i], acc[i][j], scl_n[j / 4], scl_m[i / 4]);
                    }
                });
            });
        }
        // keep the multiply phase ahead of the wait for the next stage's loads
        __builtin_amdgcn_sched_barrier(0);
        commit_stage(s + 1, sa, sb);
    }

    // ---- epilogue: lane holds C[m][n .. n+3] for each of its fragments ------------------------------
    const int64_t n_base = (int64_t)tn * TN + wn * FN * 16 + (l >> 4) * 4;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int64_t m = a_row0 + (wm * FM + i) * 16 + (l & 15);
        if (m >= a_end) continue;
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int64_t n = n_base + j * 16;
            if (n >= g.N) continue;
            const v4f v = acc[i][j];
            if (g.c_bf16) {
                uint16_t* o = static_cast<uint16_t*>(g.C) + m * g.ldc + n;
                const uint32_t b0 = f32_to_bf16_bits(v.x), b1 = f32_to_bf16_bits(v.y);
                const uint32_t b2 = f32_to_bf16_bits(v.z), b3 = f32_to_bf16_bits(v.w);
                if (g.vec_store && n + 3 < g.N) {
                    *reinterpret_cast<uint2*>(o) = make_uint2(b0 | (b1 << 16), b2 | (b3 << 16));
                } else {
                    o[0] = (uint16_t)b0;
                    if (n + 1 < g.N) o[1] = (uint16_t)b1;
                    if (n + 2 < g.N) o[2] = (uint16_t)b2;
                    if (n + 3 < g.N) o[3] = (uint16_t)b3;
                }
            } else {
                float* o = static_cast<float*>(g.C) + m * g.ldc + n;
                if (g.vec_store && n + 3 < g.N) {
                    *reinterpret_cast<v4f*>(o) = v;
                } else {
                    o[0] = v.x;
                    if (n + 1 < g.N) o[1] = v.y;
                    if (n + 2 < g.N) o[2] = v.z;
                    if (n + 3 < g.N) o[3] = v.w;
                }
            }
        }
    }
}

template <typename S, bool kMbs, bool kScaleDword, bool kRaggedK>
int launch_variant(GemmArgs g, bool grouped, hipStream_t s) {
    const int64_t tiles_m = (g.M + S::TM - 1) / S::TM + (grouped ? g.num_groups : 0);
    const int64_t tiles_n = (g.N + S::TN - 1) / S::TN;
    if (tiles_m * tiles_n > (int64_t)1 << 30) return MX_EINVAL;
    g.tiles_m = (int)tiles_m;
    g.tiles_n = (int)tiles_n;
    const unsigned blocks = (unsigned)(((tiles_m * tiles_n + 7) / 8) * 8);
    static bool attr_set = false;  // dynamic LDS above 64 KiB needs an opt-in once per process
    auto* fn = gemm_kernel<S, kMbs, kScaleDword, kRaggedK>;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                                S::kLdsBytes) != hipSuccess) {
            (void)hipGetLastError();
            return MX_ELAUNCH;
        }
        attr_set = true;
    }
    hipLaunchKernelGGL(fn, dim3(blocks), dim3(S::NT), S::kLdsBytes, s, g);
    return launch_status();
}

template <typename S>
int launch_shape(const GemmArgs& g, bool grouped, bool use_mbs, bool dword, bool ragged, hipStream_t s) {
    if (use_mbs) {
        if (!dword) return launch_variant<S, true, false, true>(g, grouped, s);
        return ragged ? launch_variant<S, true, true, true>(g, grouped, s)
                      : launch_variant<S, true, true, false>(g, grouped, s);
    }
    if (!dword) return launch_variant<S, false, false, true>(g, grouped, s);
    return ragged ? launch_variant<S, false, true, true>(g, grouped, s)
                  : launch_variant<S, false, true, false>(g, grouped, s);
}

using Shape128 = Shape<2, 4, 4, 2, 3>;      // 8 waves, 128 x 128 tile, 64 x 32 per wave, 3 code stages
using Shape256x128 = Shape<4, 2, 4, 4, 3>;  // 8 waves, 256 x 128 tile, 64 x 64 per wave, 3 code stages
using Shape256 = Shape<2, 4, 8, 4, 2>;      // 8 waves, 256 x 256 tile, 128 x 64 per wave, 2 code stages

int g_force_shape = -1;  // development switch: 0 = 128x128, 1 = 256x128, 2 = 256x256

int launch_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs, const uint8_t* b_codes,
                const uint8_t* b_scales, const uint8_t* b_mbs, int num_groups, const int64_t* row_offsets,
                bool grouped, int64_t M, int64_t N, int64_t K, int c_dtype, void* C, int64_t ldc, bool mbs_entry,
                void* stream) {
    if (M < 0 || N < 0 || K < 0 || (K % kBlock) != 0 || ldc < N) return MX_EINVAL;
    if (c_dtype != MX_OUT_F32 && c_dtype != MX_OUT_BF16) return MX_EINVAL;
    if (grouped && num_groups < 0) return MX_EINVAL;
    if (K > (int64_t)1 << 24 || M > (int64_t)1 << 30 || N > (int64_t)1 << 30 ||
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
    g.vec_store = aligned(C, 4 * esz) && (ldc % 4) == 0;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool use_mbs = mbs_entry && (a_mbs || b_mbs);
    const bool dword = (K % kMacro) == 0 && aligned(a_scales, 4) && aligned(b_scales, 4);
    const bool ragged = (K % kStageK) != 0;

    // Tile shape: large tiles need enough of them to fill 256 compute units.
    int shape = 0;
    const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256), t256x128 = ((M + 255) / 256) * ((N + 127) / 128);
    if (t256 >= 512 && !use_mbs) shape = 2;  // with MBS the 128 x 64 wave tile runs out of registers
    else if (t256x128 >= 512) shape = 1;
    if (grouped) shape = 0;
    if (g_force_shape >= 0) shape = g_force_shape;
    if (shape == 2) return launch_shape<Shape256>(g, grouped, use_mbs, dword, ragged, s);
    if (shape == 1) return launch_shape<Shape256x128>(g, grouped, use_mbs, dword, ragged, s);
    return launch_shape<Shape128>(g, grouped, use_mbs, dword, ragged, s);
}

}  // namespace
}  // namespace mx

extern "C" {

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

// Development switch (not part of the public ABI): force a tile shape, -1 = automatic.
void mx_internal_set_gemm_shape(int shape) { mx::g_force_shape = shape; }

}  // extern "C"
