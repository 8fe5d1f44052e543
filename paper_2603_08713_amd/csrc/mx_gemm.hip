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
//   scale operands: one E8M0 byte per lane (for its row/col and k-block), byte 0 of a VGPR here
//   D:    lane holds D[4 q + i][r], i = 0..3
// The weight matrix B feeds srcA and the activation matrix A feeds srcB, so that a lane ends up
// with four consecutive n of one output row m and stores them as one vector.
//
// Tiling: a workgroup of NWM x NWN wavefronts computes a TM x TN tile of C, each wavefront
// FM x FN 16x16 fragments.  FP4 operands are so small next to the MFMA rate (4096 FLOP/clk/SIMD)
// that the tile has to be large for the L2 to keep up: a T x T tile moves 1/(2T) bytes per FLOP.
//
// Data movement: K advances in stages of 256 elements (two macro blocks, one 128-byte line per row
// and operand).  Everything a stage needs travels from global memory straight into LDS with buffer
// loads that carry the LDS bit, so no vector register ever waits on global memory:
//   codes   three stages in LDS (two in flight while one is multiplied), row-major with XOR-swizzled
//           16-byte chunks: eight lanes fetch one full 128-byte line, and the 16-byte fragment reads
//           of the multiply phase are bank-conflict free;
//   scales  the 8 E8M0 bytes per row and stage, two slots; each lane later picks its own byte;
//   MBS     the 2 words per row and stage, three slots; one stage ahead of their use they are turned
//           into fp32 sigma values (two slots) by the workgroup.
// The loads of a stage are issued a few at a time between the matrix instructions, because the
// memory pipeline of a compute unit accepts them far more slowly than a wavefront can issue them.
// Buffer resources are sized to the tile's valid rows, so ragged tiles read zeros without a branch.
// The loop is software-pipelined by one macro block: while the matrix cores work on one macro block
// the LDS reads of the next one are in flight; the barrier that publishes stage s + 1 sits between the
// two macro blocks of stage s.
#include "mx_gemm_shared.h"

namespace mx {
namespace {

constexpr int kStageK = 256;  // K elements per pipeline stage
constexpr int kStageMacros = kStageK / kMacro;
constexpr int kRowStage = kStageK / 2;  // code bytes per row and stage
constexpr int kGroupM = 8;              // tile-rows walked together for L2 reuse
constexpr int kCodeBufs = 3, kSigmaBufs = 2;

// Tile shape: NWM x NWN wavefronts, each FM x FN fragments of kFrag x kFrag outputs (16: one 16x16x128
// instruction per fragment pair and macro block; 32: two chained 32x32x64 instructions).
template <int NWM_, int NWN_, int FM_, int FN_, int kFrag_>
struct Shape {
    static constexpr int NWM = NWM_, NWN = NWN_, FM = FM_, FN = FN_, kFrag = kFrag_;
    static constexpr int NW = NWM * NWN, NT = NW * kWave;
    static constexpr int TM = NWM * FM * kFrag, TN = NWN * FN * kFrag;
    static constexpr int kRows = TM + TN;  // rows of A followed by rows of B
    static_assert((TM / 8) % NW == 0 && (TN / 8) % NW == 0, "8-row code loads: operand fixed per load index");
};

// LDS map and direct-to-LDS load counts of one kernel variant.  A direct-to-LDS load always writes one
// dword per lane, also when it fetches a single byte (zero-extended), so the byte-wise fallbacks
// (kScaleDword / kM8Quad false) cost four LDS bytes per byte and only fit the smaller tile.
//   kScaleDword: the four E8M0 bytes of a macro block are an aligned dword (K % 128 == 0, aligned array)
//   kM8Quad:     the MBS words of two stages are an aligned dword (K % 512 == 0, aligned arrays)
template <typename S, bool kMbs, bool kScaleDword, bool kM8Quad>
struct Layout {
    static constexpr int NW = S::NW, kRows = S::kRows;
    // E8M0 slots: with three, the scales of stage s + 2 can be requested as early as its codes; the MBS
    // variants need the LDS for the sigma tables and request them one phase later into two slots
    static constexpr int kScaleBufs = kMbs ? 2 : 3;
    // loads per wavefront and stage (every wavefront issues the same number)
    static constexpr int kCodeDma = kRows / 8 / NW;                                              // 8 rows x 128 B
    static constexpr int kScaleDma = ceil_div(kScaleDword ? kRows * 2 : kRows * 8, kWave * NW);  // 64 lanes each
    static constexpr int kM8Dma = ceil_div(kM8Quad ? kRows : kRows * 2, kWave * NW);
    static constexpr int kScaleStride = kScaleDword ? 1 : 4;  // LDS bytes per E8M0 byte
    static constexpr int kCodesStage = kRows * kRowStage;
    static constexpr int kScaleStage = kRows * 8 * kScaleStride;          // [row][8 E8M0 bytes of the stage]
    static constexpr int kM8Stage = !kMbs ? 0 : kM8Quad ? kRows * 4 : kRows * 2 * 4;  // quad: [row] dword = words of 2 stages
    static constexpr int kM8Bufs = kM8Quad ? 2 : 3;
    static constexpr int kSigmaStage = kMbs ? kRows * 8 : 0;              // f32 [macro][row]
    static constexpr int kScaleBase = kCodeBufs * kCodesStage;
    static constexpr int kM8Base = kScaleBase + kScaleBufs * kScaleStage;
    static constexpr int kSigmaBase = kM8Base + kM8Bufs * kM8Stage;
    static constexpr int kDummy = kSigmaBase + kSigmaBufs * kSigmaStage;  // target of padding loads
    static constexpr int kLdsBytes = kDummy + 256;
    static_assert(kLdsBytes <= 160 * 1024, "LDS capacity of a gfx950 compute unit");
};

// kMbs: apply the per-macro-block correction; kFast: aligned dword loads of scales and MBS words (see
// Layout), otherwise byte loads; kRaggedK: K is not a multiple of the stage.
template <typename S, bool kMbs, bool kFast, bool kRaggedK>
__global__ __launch_bounds__(S::NT, 2) void gemm_kernel(GemmArgs g) {
    constexpr int FM = S::FM, FN = S::FN, TM = S::TM, TN = S::TN, NT = S::NT, NW = S::NW, kRows = S::kRows;
    constexpr int kFrag = S::kFrag;
    constexpr int kSub = kFrag == 32 ? 2 : 1;  // matrix instructions per fragment pair and macro block
    static_assert(kFrag == 16 || (kFrag == 32 && !kMbs), "the MBS path is written for 16 x 16 fragments");
    constexpr bool kScaleDword = kFast, kM8Quad = kFast;
    using L = Layout<S, kMbs, kScaleDword, kM8Quad>;
    constexpr int kScaleBufs = L::kScaleBufs;
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
    const int K = (int)g.K;
    const int row_bytes = K >> 1, scale_bytes = K >> 5, nmac = (K + kMacro - 1) / kMacro;

    const int tid = threadIdx.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront index, kept in a scalar register
    const int wm = w % S::NWM, wn = w / S::NWM;              // position of this wavefront in the tile

    // ---- per-lane byte offsets of the direct-to-LDS loads (constant over the K loop) ----------------
    // Codes: load i of wavefront w covers the 8 rows (i * NW + w) * 8 .. + 7 of the A-then-B row space;
    // lane l writes LDS slot l of that 1-KiB block (hardware order) and fetches row l / 8, chunk
    // (l % 8) ^ ((row >> 1) & 7): chunk c of row r lives at r * 128 + ((c ^ ((r >> 1) & 7)) * 16).
    constexpr int kCodeDma = L::kCodeDma;
    int code_off[kCodeDma], code_chunk[kCodeDma];
#pragma unroll
    for (int i = 0; i < kCodeDma; ++i) {
        const int row = ((i * NW + w) * 8 + (l >> 3)) - (i * NW * 8 < TM ? 0 : TM);  // row within its operand
        code_chunk[i] = (l & 7) ^ ((row >> 1) & 7);
        code_off[i] = row * row_bytes + code_chunk[i] * 16;
    }
    // Scales: dword loads fetch (row, macro block) pair p = (i * NW + w) * 64 + l, byte loads fetch byte
    // p of the [row][8] image.  MBS words: byte loads of pair p.  Loads past the image are padding.
    constexpr int kScaleDma = L::kScaleDma;
    int scale_off[kScaleDma], scale_sub[kScaleDma];  // sub = k-block (byte loads) or macro block (dword loads)
    bool scale_is_a[kScaleDma], scale_pad[kScaleDma];
#pragma unroll
    for (int i = 0; i < kScaleDma; ++i) {
        const int p = (i * NW + w) * kWave + l;
        const int grow = kScaleDword ? p >> 1 : p >> 3;  // row in the A-then-B row space
        scale_sub[i] = kScaleDword ? p & 1 : p & 7;
        scale_is_a[i] = (i * NW + w) * kWave < (kScaleDword ? TM * 2 : TM * 8);
        scale_pad[i] = (i * NW + w) * kWave >= (kScaleDword ? kRows * 2 : kRows * 8);
        const int row = grow - (scale_is_a[i] ? 0 : TM);
        scale_off[i] = scale_pad[i] ? kOob : row * scale_bytes + scale_sub[i] * (kScaleDword ? 4 : 1);
    }
    // MBS words: quad mode fetches one dword per row (the words of two stages), byte mode one byte per
    // (row, macro block) pair.
    constexpr int kM8Dma = L::kM8Dma;
    int m8_off[kM8Dma];
    bool m8_is_a[kM8Dma], m8_pad[kM8Dma];
#pragma unroll
    for (int i = 0; i < kM8Dma; ++i) {
        const int p = (i * NW + w) * kWave + l;
        m8_is_a[i] = (i * NW + w) * kWave < (kM8Quad ? TM : TM * 2);
        m8_pad[i] = (i * NW + w) * kWave >= (kM8Quad ? kRows : kRows * 2);
        const int row = (kM8Quad ? p : p >> 1) - (m8_is_a[i] ? 0 : TM);
        m8_off[i] = m8_pad[i] ? kOob : row * nmac + (kM8Quad ? 0 : p & 1);
    }

    // The loop requests up to three stages past the last one so that every wavefront's load count stays
    // fixed; those requests are sent out of range (they read zero and touch no memory).
    const int nstages = (K + kStageK - 1) / kStageK;
    auto dma_scale = [&](int s, auto i_) {  // load i of the E8M0 bytes of stage s
        constexpr int i = decltype(i_)::value;
        uint8_t* base = smem + L::kScaleBase + (s % kScaleBufs) * L::kScaleStage;
        int voff = s < nstages ? scale_off[i] : kOob;
        // past the end of K the block does not exist: read zero (2^-127), never a stray NaN scale
        if (kRaggedK && (kScaleDword ? (s * kStageMacros + scale_sub[i]) * kMacro : (s * 8 + scale_sub[i]) * kBlock) >= K)
            voff = kOob;
        uint8_t* dst = scale_pad[i] ? smem + L::kDummy : base + (i * NW + w) * 256;  // one dword per lane
        __builtin_amdgcn_raw_ptr_buffer_load_lds(scale_is_a[i] ? opa.scales : opb.scales, (lds_ptr_t)dst,
                                                 kScaleDword ? 4 : 1, voff, s * 8, 0, 0);
    };
    auto dma_scales = [&](int s) { static_for<kScaleDma>([&](auto i_) { dma_scale(s, i_); }); };
    auto dma_code = [&](int s, auto i_) {  // load i of the codes of stage s
        constexpr int i = decltype(i_)::value;
        uint8_t* base = smem + (s % kCodeBufs) * L::kCodesStage;
        int voff = s < nstages ? code_off[i] : kOob;
        if (kRaggedK && s * kStageK + code_chunk[i] * kBlock >= K) voff = kOob;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(i * NW * 8 < TM ? opa.codes : opb.codes,
                                                 (lds_ptr_t)(base + (i * NW + w) * 1024), 16, voff, s * kRowStage, 0, 0);
    };
    // Quad mode: the words of stages 2t and 2t + 1 as one dword per row into slot t % 2; issued every
    // iteration so that each wavefront's load count stays fixed, odd calls go to the padding area.
    // Byte mode: the words of stage s, one zero-extended byte per dword, into slot s % 3.
    auto dma_m8 = [&](int s) {
#pragma unroll
        for (int i = 0; i < kM8Dma; ++i) {
            if constexpr (kM8Quad) {
                const bool real = (s & 1) == 0 && !m8_pad[i];
                uint8_t* dst = real ? smem + L::kM8Base + ((s >> 1) & 1) * L::kM8Stage + (i * NW + w) * 256 : smem + L::kDummy;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(m8_is_a[i] ? opa.mbs : opb.mbs, (lds_ptr_t)dst, 4,
                                                         (s & 1) == 0 && s < nstages ? m8_off[i] : kOob, s * kStageMacros, 0, 0);
            } else {
                uint8_t* dst = m8_pad[i] ? smem + L::kDummy : smem + L::kM8Base + (s % 3) * L::kM8Stage + (i * NW + w) * 256;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(m8_is_a[i] ? opa.mbs : opb.mbs, (lds_ptr_t)dst, 1,
                                                         s < nstages ? m8_off[i] : kOob, s * kStageMacros, 0, 0);
            }
        }
    };
    // MBS words of stage s (landed) -> fp32 sigma = 1/F, F = 1 + m8/256 exact, reciprocal within an ulp.
    auto convert_sigma = [&](int s) {
        const uint32_t* raw = reinterpret_cast<const uint32_t*>(
            smem + L::kM8Base + (kM8Quad ? (s >> 1) & 1 : s % 3) * L::kM8Stage);
        float* sig = reinterpret_cast<float*>(smem + L::kSigmaBase + (s % kSigmaBufs) * L::kSigmaStage);
        const int g0 = s * kStageMacros;
#pragma unroll
        for (int i = 0; i < ceil_div(kRows * 2, NT); ++i) {
            // pair (row p / 2 of the A-then-B row space, macro block p % 2); threads past the last pair redo
            // pair 0 and store to the padding area, which keeps the loop body free of branches
            const int q = i * NT + tid;
            const bool live = kRows * 2 % NT == 0 || q < kRows * 2;
            const int p = live ? q : 0;
            uint32_t m8 = kM8Quad ? (raw[p >> 1] >> (8 * ((s & 1) * 2 + (p & 1)))) & 0xFFu : raw[p] & 0xFFu;
            // a macro block past the end of K has no word (the row's next bytes belong to other blocks)
            if (g0 + (p & 1) >= nmac) m8 = 0;
            float* dst = live ? sig + (p & 1) * kRows + (p >> 1) : reinterpret_cast<float*>(smem + L::kDummy);
            *dst = __builtin_amdgcn_rcpf(1.0f + (float)m8 * (1.0f / 256.0f));
        }
    };

    // ---- operands of one macro block in registers ---------------------------------------------------
    // Lane coordinates inside a fragment: row lr; k-block lq of the instruction's blocks (4 of 32 elements
    // for the 16-row form, 2 for the 32-row form).  The two instructions of a 32-row fragment pair split the
    // macro block so that lane half lq takes blocks 2 lq (first instruction) and 2 lq + 1 (second): its two
    // E8M0 bytes are then neighbours and come with one 16-bit LDS read, selected per instruction by op_sel.
    const int lr = l & (kFrag - 1), lq = l / kFrag;
    constexpr int kSclRegs = (kFrag == 32 && !kScaleDword) ? 2 : 1;
    struct Frags {
        v4i m[FM][kSub], n[FN][kSub];
        uint32_t scl_m[FM][kSclRegs], scl_n[FN][kSclRegs];
        float sig_m[FM];
        v4f sig_n[FN];
    };
    // byte offset of this lane's 16 bytes inside a fragment's rows of the swizzled code image
    int frag_off[kStageMacros][kSub];
#pragma unroll
    for (int mb = 0; mb < kStageMacros; ++mb)
#pragma unroll
        for (int kk = 0; kk < kSub; ++kk)
            frag_off[mb][kk] = lr * kRowStage + (((mb * 4 + lq * kSub + kk) ^ ((lr >> 1) & 7)) * 16);
    // this lane's first E8M0 byte inside a fragment's rows of the [row][8] scale image (+ 4 * macro block)
    const int lane_scale = (lr * 8 + lq * kSub) * L::kScaleStride;

    auto read_frags = [&](Frags& f, int s, auto mb_) {
        constexpr int mb = decltype(mb_)::value;
        const uint8_t* cm = smem + (s % kCodeBufs) * L::kCodesStage;
        const uint8_t* cn = cm + TM * kRowStage;
        // (typed as an LDS pointer: the byte load then zero-extends by itself)
        const lds_byte_ptr_t sc = (lds_byte_ptr_t)(smem + L::kScaleBase + (s % kScaleBufs) * L::kScaleStage + lane_scale +
                                                   mb * 4 * L::kScaleStride);
        const float* sig = reinterpret_cast<const float*>(smem + L::kSigmaBase + (s % kSigmaBufs) * L::kSigmaStage) + mb * kRows;
        auto read_scales = [&](uint32_t (&dst)[kSclRegs], int row0) {
            const lds_byte_ptr_t q = sc + row0 * 8 * L::kScaleStride;
            if constexpr (kFrag == 32 && kScaleDword) dst[0] = *(lds_half_ptr_t)q;
            else
#pragma unroll
                for (int kk = 0; kk < kSclRegs; ++kk) dst[kk] = q[kk * L::kScaleStride];
        };
#pragma unroll
        for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int kk = 0; kk < kSub; ++kk)
                f.m[i][kk] = *reinterpret_cast<const v4i*>(cm + (wm * FM + i) * (kFrag * kRowStage) + frag_off[mb][kk]);
            read_scales(f.scl_m[i], (wm * FM + i) * kFrag);
            if constexpr (kMbs) f.sig_m[i] = sig[(wm * FM + i) * 16 + lr];
        }
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int kk = 0; kk < kSub; ++kk)
                f.n[j][kk] = *reinterpret_cast<const v4i*>(cn + (wn * FN + j) * (kFrag * kRowStage) + frag_off[mb][kk]);
            read_scales(f.scl_n[j], TM + (wn * FN + j) * kFrag);
            if constexpr (kMbs) f.sig_n[j] = *reinterpret_cast<const v4f*>(sig + TM + (wn * FN + j) * 16 + lq * 4);
        }
    };

    using acc_t = std::conditional_t<kFrag == 32, v16f, v4f>;
    acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < kFrag * kFrag / kWave; ++e) acc[i][j][e] = 0.f;

    constexpr int kMfmas = FM * FN * kSub;  // matrix instructions per macro block
    Frags f0, f1;

    // Plain path: FM x FN matrix instructions on one macro block, accumulating in place; `between(t)` runs
    // after instruction t and is where the loads of later stages are slipped in.
    // The two instructions of a 32-row fragment pair are FM * FN instructions apart, so none waits for its
    // predecessor's result.
    auto multiply = [&](const Frags& f, auto&& between) {
        static_for<kMfmas>([&](auto t_) {
            constexpr int kk = decltype(t_)::value / (FM * FN), i = decltype(t_)::value % (FM * FN) / FN,
                          j = decltype(t_)::value % FN;
            if constexpr (kFrag == 32) {
                constexpr int sel = kSclRegs == 1 ? kk : 0, reg = kSclRegs == 1 ? 0 : kk;
                acc[i][j] = mfma_fp4_wide<sel, sel>(f.n[j][kk], f.m[i][kk], acc[i][j], f.scl_n[j][reg], f.scl_m[i][reg]);
            } else {
                acc[i][j] = mfma_fp4(f.n[j][0], f.m[i][0], acc[i][j], f.scl_n[j][0], f.scl_m[i][0]);
            }
            between(t_);
        });
    };

    // MBS path (Sec. 4.3, Fig. 6): each matrix instruction yields the partial sums of one macro block, which
    // the vector ALU folds into the accumulators as acc += p * (sigma_m * sigma_n).  A product is consumed
    // kDepth instructions after it was issued, so the vector work never waits on the matrix pipeline.  Unit u
    // of an iteration is instruction u % kMfmas of macro block u / kMfmas (f0, then f1); units past
    // 2 * kMfmas belong to the next iteration's f0.
    constexpr int kDepth = 2;
    static_assert((2 * kMfmas) % kDepth == 0, "ring slots must line up across iterations");
    v4f prod[kDepth];
    auto issue = [&](auto u_) {
        constexpr int u = decltype(u_)::value, t = u % kMfmas, i = t / FN, j = t % FN;
        const Frags& f = ((u / kMfmas) & 1) ? f1 : f0;
        const v4f zero = {0.f, 0.f, 0.f, 0.f};
        prod[u % kDepth] = mfma_fp4(f.n[j][0], f.m[i][0], zero, f.scl_n[j][0], f.scl_m[i][0]);
    };
    auto retire = [&](auto u_) {
        constexpr int u = decltype(u_)::value, t = u % kMfmas, i = t / FN, j = t % FN;
        const Frags& f = ((u / kMfmas) & 1) ? f1 : f0;
        const v4f p = prod[u % kDepth];
        const float sm = f.sig_m[i];
        acc[i][j].x = fmaf(p.x, sm * f.sig_n[j].x, acc[i][j].x);
        acc[i][j].y = fmaf(p.y, sm * f.sig_n[j].y, acc[i][j].y);
        acc[i][j].z = fmaf(p.z, sm * f.sig_n[j].z, acc[i][j].z);
        acc[i][j].w = fmaf(p.w, sm * f.sig_n[j].w, acc[i][j].w);
    };
    // one macro block of the MBS path: units base .. base + kMfmas - 1 retire, the units kDepth ahead issue
    auto multiply_mbs = [&](auto base_, auto&& between) {
        constexpr int base = decltype(base_)::value;
        static_for<kMfmas>([&](auto t_) {
            constexpr int t = decltype(t_)::value;
            retire(std::integral_constant<int, base + t>{});
            issue(std::integral_constant<int, base + t + kDepth>{});
            __builtin_amdgcn_sched_barrier(0);
            between(t_);
        });
    };
    using C0 = std::integral_constant<int, 0>;
    using C1 = std::integral_constant<int, 1>;

    // ---- prologue: stages 0 and 1 (and the MBS words of stage 2) -------------------------------------
    if (nstages > 0) {
        static_for<kCodeDma>([&](auto i_) { dma_code(0, i_); });
        dma_scales(0);
        static_for<kCodeDma>([&](auto i_) { dma_code(1, i_); });
        dma_scales(1);
        if constexpr (kMbs) {
            dma_m8(0);
            dma_m8(1);  // quad mode: padding
            dma_m8(2);
        }
        __builtin_amdgcn_s_waitcnt(wait_imm(0));
        bare_barrier();
        if constexpr (kMbs) {
            convert_sigma(0);
            convert_sigma(1);
            __builtin_amdgcn_s_waitcnt(wait_imm(0));
            bare_barrier();
        }
        read_frags(f0, 0, C0{});
        if constexpr (kMbs) static_for<kDepth>([&](auto u_) { issue(u_); });
    }

    // Loads of later stages slipped in between the matrix instructions, split evenly over the two phases so
    // that the texture-address path sees a steady stream.  The codes of stage s + 2 go into the buffer stage
    // s - 1 was read from (those reads completed before the barrier of the previous iteration), part in
    // phase A and the rest in phase B.  Phase A also takes the MBS words of stage s + 3 (slot of stage s,
    // converted two iterations ago).  Phase B, after the barrier, takes the scales of stage s + 2: with two
    // scale slots (MBS) that is the slot of stage s, whose bytes were all read before the barrier.
    constexpr int kM8Loads = kMbs ? kM8Dma : 0;
    constexpr int kCodesA = (kCodeDma + kScaleDma - kM8Loads + 1) / 2 < 0 ? 0
                            : (kCodeDma + kScaleDma - kM8Loads + 1) / 2 > kCodeDma ? kCodeDma
                            : (kCodeDma + kScaleDma - kM8Loads + 1) / 2;
    constexpr int kSlotsA = kCodesA + (kMbs ? 1 : 0);               // calls slipped into phase A
    constexpr int kSlotsB = kCodeDma - kCodesA + kScaleDma;          // calls slipped into phase B
    constexpr int kLoadsA = kCodesA + kM8Loads;                      // load instructions of phase A
    static_assert(kLoadsA < 64, "vmcnt is a 6-bit counter");
    auto load_a = [&](int s, auto n_) {
        constexpr int n = decltype(n_)::value;
        if constexpr (n < kCodesA) dma_code(s + 2, n_);
        else dma_m8(s + 3);
    };
    auto load_b = [&](int s, auto n_) {
        constexpr int n = decltype(n_)::value;
        if constexpr (n < kCodeDma - kCodesA) dma_code(s + 2, std::integral_constant<int, kCodesA + n>{});
        else dma_scale(s + 2, std::integral_constant<int, n - (kCodeDma - kCodesA)>{});
    };
    // after matrix instruction t of a phase, issue the loads whose evenly spread position is t
    auto slip = [&](auto t_, auto count_, auto&& issue) {
        constexpr int t = decltype(t_)::value, count = decltype(count_)::value;
        static_for<count>([&](auto n_) {
            constexpr int n = decltype(n_)::value;
            if constexpr ((n * kMfmas) / count == t) {
                issue(n_);
                __builtin_amdgcn_sched_barrier(0);
            }
        });
    };

    for (int s = 0; s < nstages; ++s) {
        // Past the end of K the loads below are out of range or land in rows nobody reads; issuing them
        // unconditionally keeps the loop body one basic block.
        // f0 was requested a whole phase ago: waiting for it first keeps the matrix instructions below from
        // queueing behind the reads of f1, which all wavefronts issue at once
        __builtin_amdgcn_s_waitcnt(kWaitLds);
        read_frags(f1, s, C1{});
        __builtin_amdgcn_sched_barrier(0);
        auto loads_a = [&](auto t_) {
            slip(t_, std::integral_constant<int, kSlotsA>{}, [&](auto n_) { load_a(s, n_); });
        };
        if constexpr (kMbs) multiply_mbs(std::integral_constant<int, 0>{}, loads_a);
        else multiply(f0, loads_a);
        __builtin_amdgcn_sched_barrier(0);
        // publish stage s + 1: everything issued before this iteration has landed
        __builtin_amdgcn_s_waitcnt(wait_imm(kLoadsA));
        bare_barrier();
        if constexpr (kMbs) convert_sigma(s + 2);  // into the slot of stage s, all of whose reads are done
        read_frags(f0, s + 1, C0{});
        __builtin_amdgcn_sched_barrier(0);
        auto loads_b = [&](auto t_) {
            slip(t_, std::integral_constant<int, kSlotsB>{}, [&](auto n_) { load_b(s, n_); });
        };
        if constexpr (kMbs) multiply_mbs(std::integral_constant<int, kMfmas>{}, loads_b);
        else multiply(f1, loads_b);
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- epilogue: a lane holds, per fragment, row m = lr and groups of four consecutive n --------------
    // (16-row form: the group starting at 4 lq; 32-row form: the groups starting at 8 g + 4 lq, g = 0..3)
    constexpr int kGroups = kFrag == 32 ? 4 : 1;
    const int64_t n_base = (int64_t)tn * TN + wn * FN * kFrag + lq * 4;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int64_t m = a_row0 + (wm * FM + i) * kFrag + lr;
        if (m >= a_end) continue;
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int gq = 0; gq < kGroups; ++gq) {
                const int64_t n = n_base + j * kFrag + gq * 8;
                if (n >= g.N) continue;
                const v4f v = {acc[i][j][gq * 4], acc[i][j][gq * 4 + 1], acc[i][j][gq * 4 + 2], acc[i][j][gq * 4 + 3]};
                store_c4(g, m, n, v);
            }
        }
    }
}

template <typename S, bool kMbs, bool kFast, bool kRaggedK>
int launch_variant(GemmArgs g, bool grouped, hipStream_t s) {
    using L = Layout<S, kMbs, kFast, kFast>;
    const int64_t tiles_m = (g.M + S::TM - 1) / S::TM + (grouped ? g.num_groups : 0);
    const int64_t tiles_n = (g.N + S::TN - 1) / S::TN;
    if (tiles_m * tiles_n > (int64_t)1 << 30) return MX_EINVAL;
    g.tiles_m = (int)tiles_m;
    g.tiles_n = (int)tiles_n;
    const unsigned blocks = (unsigned)(((tiles_m * tiles_n + 7) / 8) * 8);
    static bool attr_set = false;  // dynamic LDS above 64 KiB needs an opt-in once per process
    auto* fn = gemm_kernel<S, kMbs, kFast, kRaggedK>;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                                L::kLdsBytes) != hipSuccess) {
            (void)hipGetLastError();
            return MX_ELAUNCH;
        }
        attr_set = true;
    }
    hipLaunchKernelGGL(fn, dim3(blocks), dim3(S::NT), L::kLdsBytes, s, g);
    return launch_status();
}

// SMbs / SPlain: the same tile with 16-row fragments (MBS path) and 32-row fragments (plain path)
template <typename SMbs, typename SPlain, bool kFast>
int launch_shape(const GemmArgs& g, bool grouped, bool use_mbs, bool ragged, hipStream_t s) {
    static_assert(SMbs::TM == SPlain::TM && SMbs::TN == SPlain::TN && SMbs::NT == SPlain::NT, "one tile, two fragment sizes");
    if (use_mbs)
        return ragged ? launch_variant<SMbs, true, kFast, true>(g, grouped, s)
                      : launch_variant<SMbs, true, kFast, false>(g, grouped, s);
    return ragged ? launch_variant<SPlain, false, kFast, true>(g, grouped, s)
                  : launch_variant<SPlain, false, kFast, false>(g, grouped, s);
}

// 8 wavefronts each; 128 x 128 tile with 64 x 32 per wavefront, 256 x 128 tile with 64 x 64 per wavefront
using Shape128 = Shape<2, 4, 4, 2, 16>;
using Shape128Wide = Shape<2, 4, 2, 1, 32>;
using Shape256x128 = Shape<4, 2, 4, 4, 16>;
using Shape256x128Wide = Shape<4, 2, 2, 2, 32>;

constexpr int64_t kRingMinTiles = 8;  // 128 x 128 tiles a problem needs before the main kernels take it
int g_force_shape = -1;  // development switch: 0 / 1 = generic kernel on 128x128 / 256x128 tiles, 2 / 6 / 7 = main plain kernel on 256x256 / 256x128 / 128x128 tiles, 3 / 4 = main MBS kernel on 256x128 / 128x128 tiles, 5 = few-row kernel, 8 / 9 = general form of the main kernels on 256x128 / 128x128 tiles

int launch_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs, const uint8_t* b_codes,
                const uint8_t* b_scales, const uint8_t* b_mbs, int num_groups, const int64_t* row_offsets,
                bool grouped, int64_t M, int64_t N, int64_t K, int c_dtype, void* C, int64_t ldc, bool mbs_entry,
                void* stream) {
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
    g.vec_store = aligned(C, 4 * esz) && (ldc % 4) == 0;
    g.vec_store16 = aligned(C, 16) && (ldc * esz) % 16 == 0;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool use_mbs = mbs_entry && (a_mbs || b_mbs);
    const bool ragged = (K % kStageK) != 0;
    // Fast variant: scales of a macro block and MBS words of two stages are aligned dwords.
    bool fast = (K % kMacro) == 0 && aligned(a_scales, 4) && aligned(b_scales, 4);
    if (use_mbs) fast = fast && (K % (2 * kStageK)) == 0 && (!a_mbs || aligned(a_mbs, 4)) && (!b_mbs || aligned(b_mbs, 4));

    // Tile shape: the large tile needs enough tiles to fill 256 compute units, and the fast variant
    // (the byte-wise fallback does not fit its LDS).
    int shape = 0;
    const int64_t t256x128 = ((M + 255) / 256) * ((N + 127) / 128);
    if (t256x128 >= 512) shape = 1;
    if (grouped) shape = 0;
    // The main kernels need K in whole groups of four macro blocks, aligned per-row arrays and enough tiles
    // for every compute unit; everything else (grouped, ragged K, small problems) stays here.
    const bool ring_ok = !grouped && K > 0 && (K % 512) == 0 && aligned(a_scales, 16) && aligned(b_scales, 16) &&
                         (!use_mbs || ((!a_mbs || aligned(a_mbs, 4)) && (!b_mbs || aligned(b_mbs, 4))));
    // (plain: the launcher picks 256 x 256, 256 x 128 or 128 x 128 tiles by how many fill the device; MBS:
    // 256 x 128 tiles when they fill it, else 128 x 128)
    const int64_t t128 = ((M + 127) / 128) * ((N + 127) / 128);
    if (ring_ok && !use_mbs && t128 >= kRingMinTiles) shape = 2;
    if (ring_ok && use_mbs && t128 >= kRingMinTiles) {
        // rounds of one tile per compute unit x tile area / efficiency (the small tile reaches about 0.8 of the
        // large tile's rate per output, measured)
        const double big = 2.0 * ((t256x128 + 255) / 256), small = 1.25 * ((t128 + 255) / 256);
        shape = big <= small ? 3 : 4;
    }
    // The general form of the main kernels: any K % 64 == 0, scale rows on even addresses, grouped or not.
    const bool gen_ok = K > 0 && (K % 64) == 0 && aligned(a_scales, 2) && aligned(b_scales, 2);
    if (!ring_ok && gen_ok && t128 >= kRingMinTiles) {
        const double big = 2.0 * ((t256x128 + 255) / 256) / (use_mbs ? 1.0 : 0.85),
                     small = ((t128 + 255) / 256) / (use_mbs ? 0.8 : 0.72);
        shape = big <= small ? 8 : 9;
    }
    const bool skinny_ok = ring_ok && M <= 64 && K <= 8192;
    if (skinny_ok) shape = 5;
    if (g_force_shape >= 0) shape = g_force_shape;
    if (shape == 5) {
        if (!skinny_ok) return MX_EINVAL;  // only reachable through the development switch
        return launch_gemm_skinny(g, use_mbs, s);
    }
    if (shape == 8 || shape == 9) {
        if (!gen_ok) return MX_EINVAL;  // only reachable through the development switch
        return use_mbs ? launch_gemm_mbs_general(g, shape - 8, s) : launch_gemm_wide_general(g, shape - 8, s);
    }
    if (grouped && shape >= 2) return MX_EINVAL;  // only reachable through the development switch
    if (shape >= 2) {
        const bool plain_shape = shape == 2 || shape == 6 || shape == 7;
        if (shape > 7 || !ring_ok || plain_shape == use_mbs) return MX_EINVAL;  // only reachable through the development switch
        // (forced through the development switch: 2 = 256 x 256 only, 6 = 256 x 128 only, 7 = 128 x 128 only)
        if (plain_shape) return launch_gemm_wide(g, g_force_shape < 0 ? 0 : shape == 2 ? 1 : shape == 6 ? 2 : 3, s);
        return launch_gemm_mbs_ring(g, shape == 4, s);
    }
    if (!fast) return launch_shape<Shape128, Shape128Wide, false>(g, grouped, use_mbs, ragged, s);
    if (shape >= 1) return launch_shape<Shape256x128, Shape256x128Wide, true>(g, grouped, use_mbs, ragged, s);
    return launch_shape<Shape128, Shape128Wide, true>(g, grouped, use_mbs, ragged, s);
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

// Development switch (not part of the public ABI): force a tile shape, -1 = automatic.
void mx_internal_set_gemm_shape(int shape) { mx::g_force_shape = shape; }

}  // extern "C"
