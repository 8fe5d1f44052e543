// Block-scaled MXFP4 GEMM  C = A * B^T  on v_mfma_scale_f32_32x32x64_f8f6f4: the main kernel template
// (private; instantiated by mx_gemm_wide.hip without MBS, by mx_gemm_mbs.hip with MBS and by
// mx_gemm_general.hip in its general form with MBS).
//
// What limits the instruction in practice is instruction issue and data movement, not the matrix pipeline:
//   * every scaled matrix instruction keeps the vector-ALU issue port busy for about 12 clocks whatever its
//     size, so the 32x32x64 form (32 clocks in the pipeline) leaves issue slots where the 16x16x128 form
//     (16 clocks) leaves none;
//   * a direct-to-LDS load holds up its wavefront while the texture-address unit, shared by the four
//     SIMDs, works through its 64 lanes - 16 clocks for 16 bytes per lane, but 64 clocks for 4 bytes per
//     lane - so everything is fetched in 16-byte pieces and the wavefronts issue at different slots.
//
// Tiling: NWM x NWN wavefronts, each FM x FN fragments of 32 x 32 outputs.  The weight matrix feeds srcA
// and the activation matrix srcB, so a lane ends up with groups of four consecutive n of one output row m.
// Operand mapping (lane = 32 h + r): srcA/srcB hold row r, k-block h of the instruction's two 32-element
// blocks (16 bytes of FP4); the scale operand is one E8M0 byte per lane; D[8 (j / 4) + 4 h + j % 4][r] is
// result register j.  The two instructions of a fragment pair split the macro block so that lane half h
// takes blocks 2 h and 2 h + 1: its two E8M0 bytes are neighbours, one 16-bit LDS read fetches both and
// op_sel picks the byte.
//
// Pipeline: K advances one macro block (128 elements: 64 code bytes, 4 E8M0 bytes, one MBS word per row)
// per stage through a ring of four LDS code slots.  While stage s is multiplied out of registers, stage
// s + 1 is read from LDS into the other register set; every other stage issues the loads of stages s + 3 and
// s + 4 together, line by line, into the slots the stages s - 1 and s have left (mx_gemm_schedule.h: a memory
// line holds two stages of a row, and its two halves are cheaper requested back to back than a stage apart).
// Only those stages open with a wait for the wavefront's loads and the workgroup's barrier, which publishes
// stages s + 1 and s + 2 and, because every wavefront has finished reading stage s by then, frees the two slots;
// the stages between read what is published already, so the wavefronts may drift up to two stages apart.
// E8M0 bytes and MBS words travel per group of four stages: a row's 16 scale bytes as one 16-byte piece, its
// 4 words as one dword (two LDS slots each); the general form, for K and row addresses that do not allow such
// pieces, is described at RingShape.  With MBS a wavefront keeps one set of fragment registers and reads a
// fragment's next contents from LDS right behind the last pair that uses it; a stage must not begin with a
// fragment requested at the end of the stage before (the wait for the LDS would stand in front of its first
// matrix instruction), which the pair order of the 64 x 64 arrangement avoids (kSnake below).
//
// MBS (Sec. 4.3.2, App. E): the two instructions of a fragment pair start from a zero accumulator and
// yield the partial sums of one macro block, which the vector ALUs fold into the running result as
//     acc[m, n] += P[m, n] * sigma_A[m, g] * sigma_B[n, g],      sigma = 1 / (1 + m8 / 256).
// The sigma values of stages s + 2 and s + 3 are computed by the workgroup during a stage s without a barrier
// (one reciprocal per row and stage) into two of four LDS tables, which the next stage's barrier publishes.
// With words on one operand only, a wavefront folds a product in while the next pair's instructions run.
//
// Where both operands carry words, the surface S = sigma_A (x) sigma_B of Sec. 4.3.2 is itself a matrix product
// with K = 1, and the matrix cores form it: one v_mfma_f32_32x32x1_2b_f32 takes sigma_B[n] on its rows and, in
// its two blocks, sigma_A[m] of two neighbouring A fragments on its columns, and returns both fragments'
// 32 x 32 products RN(sigma_A sigma_B) in exactly the register layout of the partial sums.  That halves the
// vector work per output (one multiply-add, acc += P * S) at the price of half a matrix instruction more per
// fragment.  Measured on this device: beside matrix instructions a SIMD issues one fp32 vector instruction per
// 4.6 clocks whichever of its wavefronts it comes from, and a matrix instruction holds the same port for 12,
// so the two vector operations per output and macro block of App. B, Eq. 7 cost about 150 issue clocks per
// fragment against the 64 its two matrix instructions take; with the surface on the matrix cores it is
// 16 x 4.6 + 2.5 x 12 = 104 against 96.  A wavefront that issues matrix instructions only and one that issues
// multiply-adds only slow each other down badly (2.5 times), so every product instruction is followed by 8 of
// the multiply-adds that fold the pair BEFORE in.
//
// LDS image of a stage: codes [row][64 B] with the 16-byte chunk c of row r at position
// c ^ ((r >> 2) & 3), which keeps the 16-lane groups of a fragment read on distinct banks and lets four
// lanes of a load fetch one contiguous 64-byte piece of a row.
#pragma once

#include "mx_gemm_schedule.h"
#include "mx_gemm_shared.h"

namespace mx {
namespace {

template <typename S>
__global__ __launch_bounds__(S::NT) void gemm_ring_kernel(GemmArgs g) {
    constexpr int FM = S::FM, FN = S::FN, TM = S::TM, TN = S::TN, NW = S::NW, NT = S::NT, kRows = S::kRows;
    constexpr int kCodeDma = S::kCodeDma, kRowDma = S::kRowDma, kScaleDma = S::kScaleDma, kM8Dma = S::kM8Dma;
    constexpr bool kMbs = S::kMbs, kSigmaA = (S::kSides & 1) != 0, kSigmaB = (S::kSides & 2) != 0;
    // sigma_A (x) sigma_B on the matrix cores: both sides carry words, one B fragment, A fragments in couples
    constexpr bool kSurface = S::kSurface;
    constexpr int kCouples = FM / 2 * FN;  // surfaces per stage
    // Two A fragments against two B fragments: the pairs of a stage run (A0, B0), (A1, B0), (A1, B1), (A0, B1), so
    // that a fragment is read again from LDS right after its last pair and every fragment of the next stage has been
    // requested at least two pairs before its first use.  A0 alone is used by the last pair and by the next stage's
    // first: it has two register sets, taken in turn by stage parity.
    constexpr bool kSnake = kSurface && FM == 2 && FN == 2;
    // The other arrangements with MBS have one B fragment, which every pair of a stage uses: read again behind the
    // last pair, it would be waited for at the start of the next stage.  With the surface (two A fragments, two
    // pairs) all fragments have two register sets, taken in turn, and the next stage's are requested behind the
    // first pair; with words on one operand the B fragment alone has two.
    constexpr bool kDoubleAll = kSurface && !kSnake, kDoubleB = kMbs && !kSurface && FN == 1;
    // The loop over the stages that issue loads takes two groups of four stages per turn (see run below).
    constexpr bool kTwoGroups = kSnake && !S::kGen;
    // sigma = 1 / (1 + m8 / 256) read from a table of its 256 values instead of computed per row and stage
    constexpr bool kSigmaLut = kSnake && !S::kGen;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- which tile: workgroups are dealt round-robin to the 8 XCDs; each XCD gets a contiguous run of
    // tiles, walked in bands of kRingGroupM tile-rows so that concurrent workgroups share panels in its L2
    // (grouped: the launch took an upper bound of the tile-rows; the tiles are dealt out over the real number)
    int tiles_m = g.tiles_m;
    if constexpr (S::kGen) {
        if (g.num_groups > 0) tiles_m = grouped_tile_rows(g.row_offsets, g.num_groups, TM, (int)(threadIdx.x & 63));
    }
    const int total = tiles_m * g.tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int linear = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || linear >= total) return;
    const int band = kRingGroupM * g.tiles_n;
    const int first_m = (linear / band) * kRingGroupM;
    const int band_rows = min(tiles_m - first_m, kRingGroupM);
    const int tm = first_m + (linear % band) % band_rows;
    const int tn = (linear % band) / band_rows;
    // Rows of A and C this tile covers and the rows of B it multiplies with.  Grouped (general form only):
    // tile-rows are counted group by group; group e owns rows row_offsets[e] .. row_offsets[e + 1] - 1 and
    // the e-th of the stacked [N, K] weights.
    int64_t a_row0 = (int64_t)tm * TM, a_end = g.M, b_row0 = (int64_t)tn * TN, b_end = g.N;
    if constexpr (S::kGen) {
        if (g.num_groups > 0) {
            GroupOfTileRow gr;
            if (!grouped_find(g.row_offsets, g.num_groups, TM, (int)(threadIdx.x & 63), tm, gr)) return;
            a_row0 = gr.lo + (int64_t)(tm - gr.first) * TM;
            a_end = gr.hi;
            b_row0 = (int64_t)gr.group * g.N + (int64_t)tn * TN;
            b_end = (int64_t)(gr.group + 1) * g.N;
        }
    }

    const int K = (int)g.K;
    // general form: K in stages of 128 (the last one possibly half), padded to whole groups of four stages
    const int row_bytes = K >> 1, scale_bytes = K >> 5, nmac = (K + kMacro - 1) / kMacro;
    const int nstages = S::kGen ? (nmac + kRingGroup - 1) / kRingGroup * kRingGroup : K / kRingStageK;
    const int ngroups = nstages / kRingGroup;
    const Operand opa = make_operand(g.a_codes, g.a_scales, g.a_mbs, a_row0, a_end, TM, g.K);
    const Operand opb = make_operand(g.b_codes, g.b_scales, g.b_mbs, b_row0, b_end, TN, g.K);

    const int tid = threadIdx.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w % S::NWM, wn = w / S::NWM;
    const int lr = l & 31, lh = l >> 5;

    // ---- per-lane byte offsets of the direct-to-LDS loads (constant over the K loop) ----------------
    // Codes: load i of wavefront w covers rows (i * NW + w) * 16 .. + 15 of the A-then-B row space; lane l
    // writes LDS slot l of that 1-KiB block and fetches row l / 4, chunk (l % 4) ^ ((row >> 2) & 3).
    int code_off[kCodeDma];
#pragma unroll
    for (int i = 0; i < kCodeDma; ++i) {
        const int row = ((i * NW + w) * 16 + (l >> 2)) - (i * NW * 16 < TM ? 0 : TM);  // row within its operand
        code_off[i] = row * row_bytes + (((l & 3) ^ ((row >> 2) & 3)) * 16);
    }
    // Per-row loads, fast form: load i of wavefront w serves row (i * NW + w) * 64 + l with the 16 E8M0 bytes, or
    // the 4 MBS words, of a group of four stages; rows past the tile are padding and read zero.
    int scale_off[kRowDma], m8_off[kRowDma];
    bool row_is_a[kRowDma];
#pragma unroll
    for (int i = 0; i < kRowDma; ++i) {
        const int grow = (i * NW + w) * kWave + l;
        row_is_a[i] = (i * NW + w) * kWave < TM;
        const int row = grow - (row_is_a[i] ? 0 : TM);
        scale_off[i] = grow >= kRows ? kOob : row * scale_bytes;
        m8_off[i] = grow >= kRows ? kOob : row * nmac;
    }
    // General forms: E8M0 load i of wavefront w serves rows (i * NW + w) * 8 .. + 7, lane l pair l % 8 of the
    // group's 8 pairs of bytes of row l / 8 (or rows (i * NW + w) * 4 .. + 3, lane l byte l % 16 of row l / 16);
    // MBS load i serves rows (i * NW + w) * 16 .. + 15, lane l word l % 4 of row l / 4.
    const int gen_code_col = ((l & 3) ^ ((l >> 4) & 3)) * 16;  // this lane's chunk of the 64-byte stage piece
    const int gen_scale_col = S::kBytes ? l & 15 : (l & 7) * 2;
    const int gen_scale_off = (S::kBytes ? w * 4 + (l >> 4) : w * 8 + (l >> 3)) * scale_bytes + gen_scale_col;
    const int gen_m8_off = (w * 16 + (l >> 2)) * nmac + (l & 3), gen_m8_col = l & 3;

    // A stage or group past the end of K is never used; its loads (the pipeline issues them regardless, into
    // slots that are no longer read) fetch the last one again, so that no address leaves the operands.
    // (The offsets and resources are passed as named copies: handed over as array elements or conditional
    // expressions, the host pass of the compiler drops the kernel.)
    auto dma_code = [&](int s, auto i_) {  // load i of the codes of stage s
        constexpr int i = decltype(i_)::value;
        uint8_t* dst = smem + S::kCodesBase + (s % kRingSlots) * S::kCodesStage + (i * NW + w) * 1024;
        int voff = code_off[i];
        if constexpr (S::kGen) {
            // chunks at or past the end of K (half of the last stage, all of a padding stage) read zero
            if (s * kRingRowStage + gen_code_col >= row_bytes) voff = kOob;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(i * NW * 16 < TM ? opa.codes : opb.codes, (lds_ptr_t)dst, 16, voff,
                                                     s * kRingRowStage, 0, 0);
        } else {
            __builtin_amdgcn_raw_ptr_buffer_load_lds(i * NW * 16 < TM ? opa.codes : opb.codes, (lds_ptr_t)dst, 16, voff,
                                                     min(s, nstages - 1) * kRingRowStage, 0, 0);
        }
    };
    auto dma_scale = [&](int grp, auto i_) {  // load i of the E8M0 bytes of stages 4 grp .. 4 grp + 3
        constexpr int i = decltype(i_)::value;
        if constexpr (S::kGen) {
            constexpr int kPer = S::kScaleRowsPerLoad;
            constexpr bool is_a = i * NW * kPer < TM;
            uint8_t* dst = smem + S::kScaleBase + (grp & 1) * S::kScaleGroup + (i * NW + w) * 256;
            // (the row goes into the per-lane offset, which is what the hardware checks against the valid rows)
            const int in_range = gen_scale_off + (i * NW * kPer - (is_a ? 0 : TM)) * scale_bytes;
            const int voff = grp * 16 + gen_scale_col < scale_bytes ? in_range : kOob;  // past K: zero
            const __amdgpu_buffer_rsrc_t rsrc = is_a ? opa.scales : opb.scales;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)dst, S::kBytes ? 1 : 2, voff, grp * 16, 0, 0);
        } else {
            uint8_t* dst = smem + S::kScaleBase + (grp & 1) * S::kScaleGroup + (i * NW + w) * 1024;
            const int voff = scale_off[i];
            const __amdgpu_buffer_rsrc_t rsrc = row_is_a[i] ? opa.scales : opb.scales;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)dst, 16, voff, min(grp, ngroups - 1) * 16, 0, 0);
        }
    };
    auto dma_m8 = [&](int grp, auto i_) {  // load i of the MBS words of stages 4 grp .. 4 grp + 3
        constexpr int i = decltype(i_)::value;
        if constexpr (S::kGen) {
            constexpr bool is_a = i * NW * 16 < TM;
            uint8_t* dst = smem + S::kM8Base + (grp & 1) * S::kM8Group + (i * NW + w) * 256;
            const int in_range = gen_m8_off + (i * NW * 16 - (is_a ? 0 : TM)) * nmac;
            const int voff = grp * 4 + gen_m8_col < nmac ? in_range : kOob;  // past K: zero
            const __amdgpu_buffer_rsrc_t rsrc = is_a ? opa.mbs : opb.mbs;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)dst, 1, voff, grp * 4, 0, 0);
        } else {
            uint8_t* dst = smem + S::kM8Base + (grp & 1) * S::kM8Group + (i * NW + w) * 256;
            const int voff = m8_off[i];
            const __amdgpu_buffer_rsrc_t rsrc = row_is_a[i] ? opa.mbs : opb.mbs;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)dst, 4, voff, min(grp, ngroups - 1) * 4, 0, 0);
        }
    };
    // MBS words of stage s -> fp32 sigma = 1/F, F = 1 + m8/256 exact, reciprocal within an ulp.  Thread p serves
    // row p (whose words its own wavefront has loaded, so its own wait covers them); threads past the last row
    // redo row 0 and store to the padding area, which keeps the stage body free of branches.  The words are read
    // from LDS at the start of a stage (load_words: those of stages s and s + 1, s even, which share a group) and
    // converted at its end (store_sigma), so that the conversion does not wait for the LDS.
    constexpr int kConv = ceil_div(kRows, NT);
    struct RawWords {
        uint32_t first[kConv], second[kConv];
    };
    // (gp_: the parity of stage s's group where the caller knows it at compile time, -1 where it does not: a known
    // parity turns the slot's address into a constant of the LDS instruction)
    auto load_words = [&](int s, RawWords& r, auto gp_) {
        constexpr int gp = decltype(gp_)::value;
        const uint32_t* raw = reinterpret_cast<const uint32_t*>(smem + S::kM8Base + (gp < 0 ? (s / kRingGroup) & 1 : gp) * S::kM8Group);
#pragma unroll
        for (int i = 0; i < kConv; ++i) {
            const int q = i * NT + tid;  // (a side without words reads zero and stores sigma = 1, which nobody reads)
            const int p = (kRows % NT == 0 || q < kRows) ? q : 0;
            // fast form: a row's four words in one dword; general form: one word per dword, [row][4]
            r.first[i] = S::kGen ? raw[p * kRingGroup + s % kRingGroup] : raw[p];
            r.second[i] = S::kGen ? raw[p * kRingGroup + s % kRingGroup + 1] : r.first[i];
        }
    };
    auto store_sigma = [&](int s, const uint32_t (&words)[kConv]) {
        float* sig = reinterpret_cast<float*>(smem + S::kSigmaBase + (s % kSigmaSlots) * S::kSigmaStage);
#pragma unroll
        for (int i = 0; i < kConv; ++i) {
            const int q = i * NT + tid;
            const bool live = kRows % NT == 0 || q < kRows;
            const uint32_t m8 = S::kGen ? words[i] & 0xFFu : (words[i] >> (8 * (s % kRingGroup))) & 0xFFu;
            float* dst = live ? sig + (live ? q : 0) : reinterpret_cast<float*>(smem + S::kDummy);
            *dst = __builtin_amdgcn_rcpf(1.0f + (float)m8 * (1.0f / 256.0f));
        }
    };
    // The same through a table of the 256 possible values (kSigmaLut): the reciprocal runs at a quarter of the
    // vector rate and the conversion has two more vector instructions in front of it, all on the issue port that
    // bounds the MBS path; a table read costs the port one LDS instruction.  lookup_sigma requests the values of
    // stage s, store_looked_up writes them to the stage's table later in the stage.
    auto lookup_sigma = [&](int s, const uint32_t (&words)[kConv], float (&val)[kConv]) {
        const uint8_t* tab = smem + S::kRcpBase;
#pragma unroll
        for (int i = 0; i < kConv; ++i) {
            const uint32_t at = S::kGen ? (words[i] & 0xFFu) << 2 : ((words[i] >> (8 * (s % kRingGroup))) & 0xFFu) << 2;
            val[i] = *reinterpret_cast<const float*>(tab + at);
        }
    };
    auto store_looked_up = [&](int s, const float (&val)[kConv]) {
        float* sig = reinterpret_cast<float*>(smem + S::kSigmaBase + (s % kSigmaSlots) * S::kSigmaStage);
#pragma unroll
        for (int i = 0; i < kConv; ++i) {
            const int q = i * NT + tid;
            const bool live = kRows % NT == 0 || q < kRows;
            float* dst = live ? sig + (live ? q : 0) : reinterpret_cast<float*>(smem + S::kDummy);
            *dst = val[i];
        }
    };
    auto convert_sigma_pair = [&](int s) {  // stages s and s + 1 at once (prologue)
        RawWords r;
        load_words(s, r, std::integral_constant<int, -1>{});
        store_sigma(s, r.first);
        store_sigma(s + 1, r.second);
    };

    // ---- operands of one macro block in registers ----------------------------------------------------
    struct Frags {
        v4i m[FM][2], n[FN][2];
        uint32_t scl_m[FM], scl_n[FN];
    };
    // sigma values in registers: this lane's output row of each A fragment, per stage parity, and its 16
    // output columns of a B fragment.  Pairs run B fragment by B fragment; while one fragment's FM pairs
    // are folded in, the next fragment's values (of this or of the next stage) arrive in the other set.
    float sig_m[2][FM > kCouples ? FM : kCouples];
    v4f sig_n[2][4];
    // With the surface on the matrix cores a lane supplies, per stage, sigma_B of B row lr (to both blocks) and,
    // per couple c of A fragments, sigma_A of row lr of fragment 2 c + lh (block lh); `surface` holds the two
    // products of the current couple, registers 16 b .. 16 b + 15 for fragment 2 c + b.
    float sig_n1[2][FN];
#pragma unroll
    for (int j = 0; j < FN; ++j) sig_n1[0][j] = sig_n1[1][j] = 0.f;
    // Two surfaces are alive at a time, those of consecutive couples, but never more than three of their four
    // halves: a couple's first fragment is folded in (and its half dead) before the next couple's surface is
    // issued.  Couples alternate between `surf_a`, which keeps its first fragment in its upper half, and
    // `surf_b`, which keeps it in its lower half, so that the two can share those 16 registers.
    v32f surf_a, surf_b;
#pragma unroll
    for (int e = 0; e < 32; ++e) surf_a[e] = surf_b[e] = 0.f;
    // (zeros: the first stage folds in the "last product of the stage before", which is zero times these)
#pragma unroll
    for (int par = 0; par < 2; ++par) {
#pragma unroll
        for (int i = 0; i < (FM > kCouples ? FM : kCouples); ++i) sig_m[par][i] = 0.f;
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) sig_n[par][gq] = v4f{0.f, 0.f, 0.f, 0.f};
    }
    // This lane's 16 bytes inside a fragment's 32 rows, per instruction of the pair, with the wavefront's
    // first row of A (index 0) or of B (index 1) folded in.  The LDS read instruction adds a 16-bit constant
    // to its address register; ring slot, fragment and operand are compile-time constants, so with a second
    // copy of each base 64 KiB up every code read is a bare instruction (no address arithmetic on the
    // vector ALU, which the MBS path has no cycles to spare for).  The empty asm keeps the compiler from
    // folding the copies back into one base plus additions.
    int code_base[2][2][2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const int in_frag = lr * kRingRowStage + (((lh * 2 + kk) ^ ((lr >> 2) & 3)) * 16);
        code_base[0][kk][0] = wm * FM * 32 * kRingRowStage + in_frag;
        code_base[1][kk][0] = (TM + wn * FN * 32) * kRingRowStage + in_frag;
#pragma unroll
        for (int o = 0; o < 2; ++o) {
            code_base[o][kk][1] = code_base[o][kk][0] + 65536;
            asm volatile("" : "+v"(code_base[o][kk][0]));
            asm volatile("" : "+v"(code_base[o][kk][1]));
        }
    }
    const int lane_scale = S::kBytes ? lr * 64 + lh * 8 : S::kGen ? lr * 32 + lh * 4 : lr * 16 + lh * 2;

    // LDS read `idx` of the kReads that fetch the fragments of a stage in ring slot `slot`: per fragment (A's
    // FM, then B's FN) the two 16-byte code pieces and the 16-bit scale pair.
    constexpr int kReads = (FM + FN) * 3;
    auto read_item = [&](Frags& f, int s, auto slot_, auto idx_, auto gp_) {
        constexpr int idx = decltype(idx_)::value, fr = idx / 3, part = idx % 3, slot = decltype(slot_)::value;
        constexpr int gp = decltype(gp_)::value;  // parity of stage s's group, -1: not known at compile time
        constexpr bool is_m = fr < FM;
        constexpr int q = is_m ? fr : fr - FM;
        if constexpr (part < 2) {
            constexpr int off = S::kCodesBase + slot * S::kCodesStage + q * 32 * kRingRowStage, hi = off > 65535 - 16 ? 1 : 0;
            const v4i v = *reinterpret_cast<const v4i*>(smem + code_base[is_m ? 0 : 1][part][hi] + (off - hi * 65536));
            if constexpr (is_m) f.m[q][part] = v;
            else f.n[q][part] = v;
        } else {
            const int row0 = is_m ? (wm * FM + q) * 32 : TM + (wn * FN + q) * 32;  // in the A-then-B row space
            // fast form: [row][16 bytes of the group]; general forms: [row][8 pairs], one pair per dword, or
            // [row][16 bytes], one byte per dword (the lane's two bytes come as two dwords and are packed)
            uint32_t v;
            const uint8_t* grp_base = smem + S::kScaleBase + (gp < 0 ? (s / kRingGroup) & 1 : gp) * S::kScaleGroup;
            if constexpr (S::kBytes) {
                // (a plain vector type: before a read through HIP's uint2 the compiler waits for every
                // outstanding direct-to-LDS load)
                typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                const u32x2 two = *reinterpret_cast<const u32x2*>(grp_base + (s % kRingGroup) * 16 + lane_scale + row0 * 64);
                v = (two.x & 0xFFu) | ((two.y & 0xFFu) << 8);
            } else if constexpr (S::kGen) {
                v = *(lds_half_ptr_t)(grp_base + (s % kRingGroup) * 8 + lane_scale + row0 * 32);
            } else {
                v = *(lds_half_ptr_t)(grp_base + (s % kRingGroup) * 4 + lane_scale + row0 * 16);
            }
            if constexpr (is_m) f.scl_m[q] = v;
            else f.scl_n[q] = v;
        }
    };
    // sigma values of stage s: one float per A fragment, four float4 per B fragment (columns 8 g + 4 h .. + 3)
    auto read_sigma_m = [&](int s, auto par_) {
        if constexpr (!kSigmaA) return;
        const float* sig = reinterpret_cast<const float*>(smem + S::kSigmaBase + (s % kSigmaSlots) * S::kSigmaStage);
        if constexpr (kSurface) {
            // The couples of all stages, counted on, alternate between surf_a (first fragment in block 1, so lane
            // half h supplies fragment 2 c + 1 - h) and surf_b (lane half h supplies fragment 2 c + h); couple
            // j FM / 2 + c has the parity of c, plus the stage's when a stage has an odd number of couples.
            constexpr int par = decltype(par_)::value;
#pragma unroll
            for (int g = 0; g < kCouples; ++g) {
                const int c = g % (FM / 2);
                // (kSnake: the second couple runs A1 first, so its halves are the other way round)
                const bool swap = (((kCouples % 2 == 1 ? par : 0) + g) % 2 == 0) != (kSnake && g == 1);
                sig_m[par][g] = sig[(wm * FM + 2 * c) * 32 + (swap ? l ^ 32 : l)];
            }
#pragma unroll
            for (int j = 0; j < FN; ++j) sig_n1[par][j] = sig[TM + (wn * FN + j) * 32 + lr];
        } else {
#pragma unroll
            for (int i = 0; i < FM; ++i) sig_m[decltype(par_)::value][i] = sig[(wm * FM + i) * 32 + lr];
        }
    };
    auto read_sigma_n = [&](int s, auto j_, auto set_) {
        constexpr int j = decltype(j_)::value, set = decltype(set_)::value;
        if constexpr (!kSigmaB || kSurface) return;
        const float* sig = reinterpret_cast<const float*>(smem + S::kSigmaBase + (s % kSigmaSlots) * S::kSigmaStage);
#pragma unroll
        for (int gq = 0; gq < 4; ++gq)
            sig_n[set][gq] = *reinterpret_cast<const v4f*>(sig + TM + (wn * FN + j) * 32 + gq * 8 + lh * 4);
    };

    v16f acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // ---- loads per stage (mx_gemm_schedule.h) ----------------------------------------------------------
    using Sched = RingSchedule<kCodeDma, kScaleDma, kMbs ? kM8Dma : 0>;
    static_assert(Sched::kSlots == kRingSlots && Sched::kGroup == kRingGroup, "the schedule is written for this ring");
    static_assert(Sched::prologue_count() < 64 && Sched::issue_count(1) + Sched::issue_count(3) < 64, "vmcnt is a 6-bit counter");
    // load n of those a stage of this phase issues (s: the issuing stage)
    auto issue_load = [&](int s, auto phase_, auto n_) {
        constexpr LoadItem it = Sched::issue_item(decltype(phase_)::value, decltype(n_)::value);
        using Index = std::integral_constant<int, it.index>;
        if constexpr (it.kind == kLoadCode) dma_code(s + it.what, Index{});
        else if constexpr (it.kind == kLoadScale) dma_scale(s / kRingGroup + it.what, Index{});
        else dma_m8(s / kRingGroup + it.what, Index{});
    };

    // ---- prologue: fill the ring, fetch the operands of stage 0 --------------------------------------
    static_for<Sched::prologue_count()>([&](auto n_) {
        constexpr LoadItem it = Sched::prologue_item(decltype(n_)::value);
        using Index = std::integral_constant<int, it.index>;
        if constexpr (it.kind == kLoadCode) dma_code(it.what, Index{});
        else if constexpr (it.kind == kLoadScale) dma_scale(it.what, Index{});
        else dma_m8(it.what, Index{});
    });
    if constexpr (kSigmaLut) {
        static_assert(NT >= 256, "one thread per table entry");
        if (tid < 256) reinterpret_cast<float*>(smem + S::kRcpBase)[tid] = __builtin_amdgcn_rcpf(1.0f + (float)tid * (1.0f / 256.0f));
        __builtin_amdgcn_s_waitcnt(kWaitLds);  // the barrier below publishes the table
    }
    __builtin_amdgcn_s_waitcnt(wait_imm(Sched::prologue_wait_first()));
    bare_barrier();
    Frags f0, f1;
    Frags alt;  // the second register set of A fragment 0 (kSnake: m[0], scl_m[0]) or of the B fragment (kDoubleB: n[0], scl_n[0])
    if constexpr (kMbs) {
        convert_sigma_pair(0);
        __builtin_amdgcn_s_waitcnt(kWaitLds);
        bare_barrier();
        read_sigma_m(0, std::integral_constant<int, 0>{});
        read_sigma_n(0, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    }
    static_for<kReads>([&](auto idx_) { read_item(f0, 0, std::integral_constant<int, 0>{}, idx_, std::integral_constant<int, 0>{}); });

    // ---- the matrix instructions of one stage ---------------------------------------------------------
    // Plain: instruction t is half kk = t / (FM FN) of fragment pair (i, j); the two halves of a pair are
    // FM FN instructions apart, so none waits for its predecessor.  MBS: pair q = (j, i) takes two
    // instructions, the first from a zero accumulator and the second on top of it; the instructions of pair
    // q + 1 are issued before the product of pair q is folded into the accumulators (two product register
    // sets), and the SIMD's other wavefront fills what gaps remain.
    constexpr int kPairs = FM * FN, kMfmas = kPairs * 2;
    // The product of a stage's last pair is folded in at the start of the next stage, behind that stage's first
    // matrix instructions: otherwise every stage would begin with the vector ALUs waiting for the first product
    // and end with the matrix pipeline idle behind the last one, in both wavefronts of a SIMD at once (the
    // barrier keeps them in step).  Needs the sigma registers of the stage before (they alternate by stage
    // parity when FN = 1) and a product register set that the next stage's first pair does not take.
    constexpr bool kDefer = kMbs && !kSurface && FN == 1 && kPairs % 2 == 0;
    v16f prod[2];
#pragma unroll
    for (int e = 0; e < 16; ++e) prod[0][e] = prod[1][e] = 0.f;
    auto product = [&](const Frags& f, auto q_, auto par_) {
        constexpr int q = decltype(q_)::value, j = q / FM, i = q % FM;
        constexpr bool other = kDoubleB && decltype(par_)::value == 1;  // odd stages: the B fragment sits in `alt`
        const v4i n0 = other ? alt.n[0][0] : f.n[j][0], n1 = other ? alt.n[0][1] : f.n[j][1];
        const uint32_t sn = other ? alt.scl_n[0] : f.scl_n[j];
        v16f zero;
#pragma unroll
        for (int e = 0; e < 16; ++e) zero[e] = 0.f;
        prod[q % 2] = mfma_fp4_wide<0, 0>(n0, f.m[i][0], zero, sn, f.scl_m[i]);
        prod[q % 2] = mfma_fp4_wide<1, 1>(n1, f.m[i][1], prod[q % 2], sn, f.scl_m[i]);
    };
    // The surface of couple g of the stage with parity par: g = j FM / 2 + c is A fragments 2 c and 2 c + 1 against
    // B fragment j.  Consecutive couples alternate between the two buffers; a stage with an odd number of couples
    // (one) alternates by stage parity as well.
    auto issue_surface = [&](auto par_, auto g_) {
        constexpr int par = decltype(par_)::value, g = decltype(g_)::value, j = g / (FM / 2);
        v32f zero;
#pragma unroll
        for (int e = 0; e < 32; ++e) zero[e] = 0.f;
        const v32f v = __builtin_amdgcn_mfma_f32_32x32x1f32(sig_n1[par][j], sig_m[par][g], zero, 0, 0, 0);
        if constexpr (((kCouples % 2 == 1 ? par : 0) + g) % 2 == 0) surf_a = v;
        else surf_b = v;
    };
    // Half `half` (8 of the 16 multiply-adds) of folding the product of pair q = j FM + i of the stage with parity
    // par in.
    auto fold = [&](auto par_, auto q_, auto half_) {
        constexpr int par = decltype(par_)::value, q = decltype(q_)::value, half = decltype(half_)::value;
        constexpr int i = kSnake ? (q == 1 || q == 2 ? 1 : 0) : q % FM, j = q / FM, g = j * (FM / 2) + i / 2;
        constexpr bool in_a = ((kCouples % 2 == 1 ? par : 0) + g) % 2 == 0;
        constexpr bool first = kSnake ? q % 2 == 0 : i % 2 == 0;  // the couple's fragment that is folded in first
        constexpr int base = in_a ? (first ? 16 : 0) : (first ? 0 : 16);
#pragma unroll
        for (int e = half * 8; e < half * 8 + 8; ++e)
            acc[i][j][e] = fmaf(prod[q % 2][e], in_a ? surf_a[base + e] : surf_b[base + e], acc[i][j][e]);
    };
    auto retire = [&](auto par_, auto q_) {
        constexpr int q = decltype(q_)::value, j = q / FM, i = q % FM;
        const float sm = sig_m[decltype(par_)::value][i];
        // sigma set of B fragment j of this stage: fragments alternate sets, counted over all stages
        constexpr int set = FN == 1 ? decltype(par_)::value : j % 2;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float sn = sig_n[set][e / 4][e % 4];
            acc[i][j][e] = fmaf(prod[q % 2][e], kSigmaA && kSigmaB ? sm * sn : kSigmaA ? sm : sn, acc[i][j][e]);
        }
    };

    // One stage: multiply stage s out of `cur`; slipped in between the matrix instructions, the LDS reads of
    // stage s + 1 into `next` and, with kIssue, this stage's loads.  The wavefronts issue their loads at
    // different instruction slots (kLate 0 or 1).
    // gp_: the parity of the stage's group of four (which of the two slots its E8M0 bytes and MBS words sit in) where
    // the caller knows it at compile time, -1 where it does not.
    auto stage = [&](int s, const Frags& cur, Frags& next, auto phase_, auto late_, auto issue_, auto gp_) {
        constexpr int kPhase = decltype(phase_)::value, kLate = decltype(late_)::value, kGp = decltype(gp_)::value;
        using NextGp = std::integral_constant<int, kGp < 0 ? -1 : kPhase == 3 ? 1 - kGp : kGp>;    // of stage s + 1
        using WordsGp = std::integral_constant<int, kGp < 0 ? -1 : kPhase >= 2 ? 1 - kGp : kGp>;   // of stage s + 2
        using Par = std::integral_constant<int, kPhase % 2>;       // stage parity: kRingGroup is even
        using NextPar = std::integral_constant<int, 1 - kPhase % 2>;
        using NextSlot = std::integral_constant<int, (kPhase + 1) % kRingSlots>;  // stage s sits in slot s % 4 = kPhase
        static_assert(kRingSlots == kRingGroup, "the phase of a stage is also its ring slot");
        constexpr bool kIssue = decltype(issue_)::value;
        constexpr int kN = Sched::issue_count(kPhase);
        // A stage that issues loads: everything this wavefront has requested has landed (the stages s + 1 and
        // s + 2, the E8M0 bytes and MBS words of the groups they belong to), own LDS traffic is done, and behind the
        // barrier every wavefront has finished stage s - 1.  (Stages past the last request keep the barrier.)
        if constexpr (Sched::has_barrier(kPhase)) {
            __builtin_amdgcn_s_waitcnt(wait_imm(Sched::wait_count(kPhase)));
            bare_barrier();
        }
        // a stage without a barrier converts the words of the stages s + 2 and s + 3 at its end (published by the
        // next stage's barrier, into the tables that the stages s - 2 and s - 1 were read from)
        constexpr bool kConvert = kMbs && !Sched::has_barrier(kPhase);
        RawWords words;
        if constexpr (kConvert) load_words(s + 2, words, WordsGp{});
        float looked_up[2][kConv];
        auto convert = [&]() {
            if constexpr (kConvert && kSigmaLut) {
                store_looked_up(s + 2, looked_up[0]);
                store_looked_up(s + 3, looked_up[1]);
            } else if constexpr (kConvert) {
                store_sigma(s + 2, words.first);
                store_sigma(s + 3, words.second);
            }
        };
        auto slip = [&](auto t_) {  // after matrix instruction t: LDS reads and loads whose turn it is
            constexpr int t = decltype(t_)::value;
            if constexpr (!kMbs) {
                static_for<kReads>([&](auto r_) {
                    if constexpr ((decltype(r_)::value * kMfmas) / kReads == t) read_item(next, s + 1, NextSlot{}, r_, NextGp{});
                });
            }
            if constexpr (kMbs && t == kMfmas / 2) read_sigma_m(s + 1, NextPar{});
            if constexpr (kIssue) {
                static_for<kN>([&](auto n_) {
                    constexpr int n = decltype(n_)::value, slot = (n * kMfmas) / kN + kLate;
                    if constexpr ((slot < kMfmas ? slot : kMfmas - 1) == t) {
                        issue_load(s, phase_, n_);
                    }
                });
            }
        };
        if constexpr (kSnake) {
            // As the branch below (every product instruction followed by half of the multiply-adds of the pair
            // before, the surface instruction by loads and table work), in the pair order given at kSnake, with
            // the LDS reads of a fragment's next contents right behind its last pair.
            using I0 = std::integral_constant<int, 0>;
            using I1 = std::integral_constant<int, 1>;
            constexpr int par = kPhase % 2;
            read_sigma_m(s + 1, NextPar{});
            auto refill = [&](Frags& dst, auto f_) {  // fragment f of stage s + 1: two code pieces and the E8M0 pair
                static_for<3>([&](auto part_) {
                    read_item(dst, s + 1, NextSlot{}, std::integral_constant<int, decltype(f_)::value * 3 + decltype(part_)::value>{}, NextGp{});
                });
            };
            static_for<4>([&](auto q_) {
                constexpr int q = decltype(q_)::value, i = (q == 1 || q == 2) ? 1 : 0, j = q / 2;
                using Before = std::integral_constant<int, (q + 3) % 4>;
                using BeforePar = std::conditional_t<q == 0, NextPar, Par>;  // the last pair of the stage before
                // A0 of this stage sits in `cur` (even stages) or in `alt` (odd stages)
                const v4i m0 = i == 0 && par == 1 ? alt.m[0][0] : cur.m[i][0], m1 = i == 0 && par == 1 ? alt.m[0][1] : cur.m[i][1];
                const uint32_t sm = i == 0 && par == 1 ? alt.scl_m[0] : cur.scl_m[i];
                v16f zero;
#pragma unroll
                for (int e = 0; e < 16; ++e) zero[e] = 0.f;
                prod[q % 2] = mfma_fp4_wide<0, 0>(cur.n[j][0], m0, zero, cur.scl_n[j], sm);
                __builtin_amdgcn_sched_barrier(0);
                fold(BeforePar{}, Before{}, I0{});
                __builtin_amdgcn_sched_barrier(0);
                prod[q % 2] = mfma_fp4_wide<1, 1>(cur.n[j][1], m1, prod[q % 2], cur.scl_n[j], sm);
                __builtin_amdgcn_sched_barrier(0);
                fold(BeforePar{}, Before{}, I1{});
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (q % 2 == 1) {
                    constexpr int shadow = q / 2;
                    if constexpr (shadow == 0) issue_surface(Par{}, I1{});
                    else issue_surface(NextPar{}, I0{});
                    __builtin_amdgcn_sched_barrier(0);
                }
                // last pairs: B0 after pair 1, A1 after pair 2, B1 and this stage's A0 after pair 3; the next stage's
                // A0 goes to the other register set and is requested with B0
                if constexpr (q == 1) {
                    refill(next, std::integral_constant<int, FM + 0>{});
                    if constexpr (par == 0) refill(alt, I0{});
                    else refill(next, I0{});
                }
                if constexpr (q == 2) refill(next, I1{});
                if constexpr (q == 3) refill(next, std::integral_constant<int, FM + 1>{});
                if constexpr (q % 2 == 1) {
                    constexpr int shadow = q / 2;
                    if constexpr (kIssue) {
                        static_for<kN>([&](auto n_) {
                            if constexpr ((decltype(n_)::value * 2) / kN == shadow) issue_load(s, phase_, n_);
                        });
                    }
                    if constexpr (shadow == 0 && kConvert && kSigmaLut) {
                        lookup_sigma(s + 2, words.first, looked_up[0]);
                        lookup_sigma(s + 3, words.second, looked_up[1]);
                    }
                    if constexpr (shadow == 1) convert();
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        } else if constexpr (kSurface) {
            // Two wavefronts share a SIMD's matrix pipeline and its vector issue port well only if each of them
            // mixes its matrix and vector instructions finely (measured: one wavefront issuing matrix
            // instructions only and one issuing multiply-adds only slow each other down by a factor of 2.5,
            // while two that each follow every matrix instruction with a few multiply-adds lose nothing).  So
            // every product instruction is followed by 8 of the 16 multiply-adds that fold the pair BEFORE in
            // (its product is complete by then), and the long surface instruction by this wavefront's LDS reads,
            // loads and table work, which need no vector issue slots.  A couple's surface is issued a whole pair
            // before its first use, right after the first fragment of the couple before has been folded in.
            using I0 = std::integral_constant<int, 0>;
            using I1 = std::integral_constant<int, 1>;
            constexpr int kShadows = kCouples;
            read_sigma_m(s + 1, NextPar{});  // published by this stage's barrier or the one before; the next stage's first surface needs it
            static_for<kPairs>([&](auto q_) {
                constexpr int q = decltype(q_)::value, i = q % FM, j = q / FM;
                using Before = std::integral_constant<int, (q + kPairs - 1) % kPairs>;
                using BeforePar = std::conditional_t<q == 0, NextPar, Par>;  // the last pair of the stage before
                v16f zero;
#pragma unroll
                for (int e = 0; e < 16; ++e) zero[e] = 0.f;
                prod[q % 2] = mfma_fp4_wide<0, 0>(cur.n[j][0], cur.m[i][0], zero, cur.scl_n[j], cur.scl_m[i]);
                __builtin_amdgcn_sched_barrier(0);
                fold(BeforePar{}, Before{}, I0{});
                __builtin_amdgcn_sched_barrier(0);
                prod[q % 2] = mfma_fp4_wide<1, 1>(cur.n[j][1], cur.m[i][1], prod[q % 2], cur.scl_n[j], cur.scl_m[i]);
                __builtin_amdgcn_sched_barrier(0);
                fold(BeforePar{}, Before{}, I1{});
                __builtin_amdgcn_sched_barrier(0);
                // (two register sets: the next stage's fragments are requested behind the first pair)
                if constexpr (kDoubleAll && q == 0) static_for<kReads>([&](auto idx_) { read_item(next, s + 1, NextSlot{}, idx_, NextGp{}); });
                if constexpr (q % 2 == 1) {
                    constexpr int shadow = q / 2;
                    if constexpr (shadow + 1 < kShadows) issue_surface(Par{}, std::integral_constant<int, shadow + 1>{});
                    else issue_surface(NextPar{}, I0{});
                    __builtin_amdgcn_sched_barrier(0);
                    // in its shadow: refill the fragments whose last pair lies in this couple with the next stage's
                    // data (A fragment i serves the pairs (0, i) .. (FN - 1, i), B fragment j the pairs (j, 0) ..
                    // (j, FM - 1)), this stage's loads, and at the end the table work
                    if constexpr (!kDoubleAll) static_for<FM + FN>([&](auto f_) {
                        constexpr int f = decltype(f_)::value;
                        constexpr int last = f < FM ? (FN - 1) * FM + f : (f - FM) * FM + FM - 1;  // last pair that reads it
                        if constexpr (last == q || last == q - 1) static_for<3>([&](auto part_) {
                            read_item(next, s + 1, NextSlot{}, std::integral_constant<int, f * 3 + decltype(part_)::value>{}, NextGp{});
                        });
                    });
                    if constexpr (kIssue) {
                        static_for<kN>([&](auto n_) {
                            if constexpr ((decltype(n_)::value * kShadows) / kN == shadow) issue_load(s, phase_, n_);
                        });
                    }
                    if constexpr (shadow == kShadows - 1) convert();
                    __builtin_amdgcn_sched_barrier(0);
                }
            });
        } else if constexpr (kMbs) {
            // The MBS path keeps one set of fragment registers (`cur` and `next` are the same object): a
            // fragment is refilled with the next stage's data right after the instructions of the last pair
            // that uses it have been issued.
            auto issue = [&](auto p_) {  // the instructions of pair p, then the refills it makes possible
                constexpr int pj = decltype(p_)::value / FM, pi = decltype(p_)::value % FM;
                product(cur, p_, Par{});
                if constexpr (kDoubleB) {
                    // the next stage's B fragment into the register set this stage does not use, behind the first pair
                    if constexpr (decltype(p_)::value == 0) static_for<3>([&](auto part_) {
                        using Idx = std::integral_constant<int, FM * 3 + decltype(part_)::value>;
                        if constexpr (kPhase % 2 == 0) read_item(alt, s + 1, NextSlot{}, Idx{}, NextGp{});
                        else read_item(next, s + 1, NextSlot{}, Idx{}, NextGp{});
                    });
                } else if constexpr (pi == FM - 1) static_for<3>([&](auto part_) {
                    read_item(next, s + 1, NextSlot{}, std::integral_constant<int, (FM + pj) * 3 + decltype(part_)::value>{}, NextGp{});
                });
                if constexpr (pj == FN - 1) static_for<3>([&](auto part_) {
                    read_item(next, s + 1, NextSlot{}, std::integral_constant<int, pi * 3 + decltype(part_)::value>{}, NextGp{});
                });
            };
            issue(std::integral_constant<int, 0>{});
            // (behind the first pair's instructions: the LDS round trip of the MBS words then overlaps their run)
            convert();
            if constexpr (kDefer) {
                __builtin_amdgcn_sched_barrier(0);
                retire(NextPar{}, std::integral_constant<int, kPairs - 1>{});  // (the other parity: the stage before)
                __builtin_amdgcn_sched_barrier(0);
            }
            static_for<kPairs>([&](auto q_) {
                constexpr int q = decltype(q_)::value, j = q / FM, i = q % FM;
                // (behind the last use of the couple before: the product folded in just above)
                if constexpr (q + 1 < kPairs) issue(std::integral_constant<int, q + 1>{});
                // first pair of a B fragment: request the sigma values of the next one into the other set
                if constexpr (i == 0) {
                    using OtherSet = std::integral_constant<int, FN == 1 ? 1 - kPhase % 2 : (j + 1) % 2>;
                    if constexpr (j + 1 < FN) read_sigma_n(s, std::integral_constant<int, j + 1>{}, OtherSet{});
                    else read_sigma_n(s + 1, std::integral_constant<int, 0>{}, OtherSet{});
                }
                slip(std::integral_constant<int, 2 * q>{});
                slip(std::integral_constant<int, 2 * q + 1>{});
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (!(kDefer && q == kPairs - 1)) retire(Par{}, q_);
                __builtin_amdgcn_sched_barrier(0);
            });
        } else {
            static_for<kMfmas>([&](auto t_) {
                constexpr int t = decltype(t_)::value, kk = t / kPairs, i = t % kPairs / FN, j = t % FN;
                acc[i][j] = mfma_fp4_wide<kk, kk>(cur.n[j][kk], cur.m[i][kk], acc[i][j], cur.scl_n[j], cur.scl_m[i]);
                slip(t_);
                __builtin_amdgcn_sched_barrier(0);
            });
        }
    };
    // Stages whose iteration still has a stage s + 4 to request, rounded up to whole groups (the extra ones
    // fetch the last stage again into slots that are no longer read); the rest runs without loads.
    const int n_issue = (max(nstages - kRingSlots, 0) + kRingGroup - 1) / kRingGroup * kRingGroup;
    auto run = [&](auto late_) {
        using Yes = std::integral_constant<bool, true>;
        using No = std::integral_constant<bool, false>;
        using P0 = std::integral_constant<int, 0>;
        using P1 = std::integral_constant<int, 1>;
        using P2 = std::integral_constant<int, 2>;
        using P3 = std::integral_constant<int, 3>;
        Frags& fa = f0;
        Frags& fb = kMbs && !kDoubleAll ? f0 : f1;  // the MBS path refills one set in place (kDoubleAll aside)
        using G0 = std::integral_constant<int, 0>;
        using G1 = std::integral_constant<int, 1>;
        using Gx = std::integral_constant<int, -1>;
        int s = 0;
        if constexpr (kTwoGroups) {
            // two groups per turn: which of the two slots a group's E8M0 bytes and MBS words sit in is then a
            // constant of the LDS instructions that read them, which saves the vector ALUs the address additions
            for (; s + 8 <= n_issue; s += 8) {
                stage(s, fa, fb, P0{}, late_, Yes{}, G0{});
                stage(s + 1, fb, fa, P1{}, late_, Yes{}, G0{});
                stage(s + 2, fa, fb, P2{}, late_, Yes{}, G0{});
                stage(s + 3, fb, fa, P3{}, late_, Yes{}, G0{});
                stage(s + 4, fa, fb, P0{}, late_, Yes{}, G1{});
                stage(s + 5, fb, fa, P1{}, late_, Yes{}, G1{});
                stage(s + 6, fa, fb, P2{}, late_, Yes{}, G1{});
                stage(s + 7, fb, fa, P3{}, late_, Yes{}, G1{});
            }
        }
        for (; s < n_issue; s += 4) {
            stage(s, fa, fb, P0{}, late_, Yes{}, Gx{});
            stage(s + 1, fb, fa, P1{}, late_, Yes{}, Gx{});
            stage(s + 2, fa, fb, P2{}, late_, Yes{}, Gx{});
            stage(s + 3, fb, fa, P3{}, late_, Yes{}, Gx{});
        }
        for (; s < nstages; s += 4) {  // nstages is a multiple of the group
            stage(s, fa, fb, P0{}, late_, No{}, Gx{});
            stage(s + 1, fb, fa, P1{}, late_, No{}, Gx{});
            stage(s + 2, fa, fb, P2{}, late_, No{}, Gx{});
            stage(s + 3, fb, fa, P3{}, late_, No{}, Gx{});
        }
    };
    // (with one wavefront per SIMD every stalled load stalls the matrix pipeline: half of the wavefronts issue
    // theirs one slot later; with two per SIMD the second copy of the loop is not worth its registers)
    if constexpr (kSurface) issue_surface(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    if (NW == 8 || w % 4 < 2) run(std::integral_constant<int, 0>{});
    else run(std::integral_constant<int, 1>{});
    // (the last stage is the fourth of its group: parity 1)
    if constexpr (kDefer) retire(std::integral_constant<int, 1>{}, std::integral_constant<int, kPairs - 1>{});
    if constexpr (kSurface) {
        fold(std::integral_constant<int, 1>{}, std::integral_constant<int, kPairs - 1>{}, std::integral_constant<int, 0>{});
        fold(std::integral_constant<int, 1>{}, std::integral_constant<int, kPairs - 1>{}, std::integral_constant<int, 1>{});
    }

    // ---- epilogue ------------------------------------------------------------------------------------
    // A lane holds, per fragment, output row lr and the column groups 8 g + 4 h .. + 3.  Each wavefront
    // passes its block through its own piece of LDS, 32 output rows at a time, so that the global stores
    // cover whole row segments (16 bytes per lane, consecutive lanes along n).
    __builtin_amdgcn_s_waitcnt(wait_imm(0));
    bare_barrier();  // every wavefront's loads have landed and all LDS reads are done: the LDS is free
    constexpr int kCols = FN * 32;
    uint8_t* stg = smem + w * S::kStageRegion;
    const int64_t m0 = a_row0 + wm * FM * 32, n0 = (int64_t)tn * TN + wn * kCols;
    auto flush = [&](auto bf16_) {
        constexpr bool kBf16 = decltype(bf16_)::value;
        constexpr int esz = kBf16 ? 2 : 4, per = 16 / esz;  // bytes per element, elements per lane and store
        constexpr int pitch = kCols * esz + 16;             // bytes per staged row; the pad spreads the rows over the banks
        constexpr int lanes_per_row = kCols * esz / 16, rows_per_pass = kWave / lanes_per_row;
        const int rd_row = l / lanes_per_row, rd_chunk = l % lanes_per_row;
        const int64_t n = n0 + rd_chunk * per;
        const bool whole = g.vec_store16 && n + per <= g.N;
        static_for<FM>([&](auto i_) {
            constexpr int i = decltype(i_)::value;
            static_for<FN * 4>([&](auto q_) {
                constexpr int j = decltype(q_)::value / 4, gq = decltype(q_)::value % 4;
                const int col = j * 32 + gq * 8 + lh * 4;
                const v4f v = {acc[i][j][gq * 4], acc[i][j][gq * 4 + 1], acc[i][j][gq * 4 + 2], acc[i][j][gq * 4 + 3]};
                if constexpr (kBf16)
                    *reinterpret_cast<uint2*>(stg + lr * pitch + col * 2) = make_uint2(pack_bf16(v.x, v.y), pack_bf16(v.z, v.w));
                else
                    *reinterpret_cast<v4f*>(stg + lr * pitch + col * 4) = v;
            });
            __builtin_amdgcn_s_waitcnt(kWaitLds);
            static_for<32 / rows_per_pass>([&](auto p_) {
                const int row = decltype(p_)::value * rows_per_pass + rd_row;
                const v4i v = *reinterpret_cast<const v4i*>(stg + row * pitch + rd_chunk * 16);
                const int64_t m = m0 + i * 32 + row;
                if (m < a_end && n < g.N) {
                    uint8_t* o = static_cast<uint8_t*>(g.C) + (m * g.ldc + n) * esz;
                    if (whole) {
                        __builtin_nontemporal_store(v, reinterpret_cast<v4i*>(o));
                    } else {
                        // rows of C that start on 8-byte but not on 16-byte boundaries: the halves of the piece that
                        // lie inside the row go out as 8-byte stores, the rest element by element
#pragma unroll
                        for (int half = 0; half < 2; ++half) {
                            if (g.vec_store8 && n + (half + 1) * (per / 2) <= g.N) {
                                typedef int v2i_t __attribute__((ext_vector_type(2)));
                                reinterpret_cast<v2i_t*>(o)[half] = v2i_t{v[2 * half], v[2 * half + 1]};
                                continue;
                            }
                            if constexpr (kBf16) {
                                // (rows on 4-byte boundaries: two elements at a time where both lie inside the row)
#pragma unroll
                                for (int d = 2 * half; d < 2 * half + 2; ++d) {
                                    if (g.vec_store4 && n + 2 * d + 1 < g.N) {
                                        reinterpret_cast<int*>(o)[d] = v[d];
                                    } else {
                                        if (n + 2 * d < g.N) reinterpret_cast<uint16_t*>(o)[2 * d] = (uint16_t)(uint32_t)v[d];
                                        if (n + 2 * d + 1 < g.N) reinterpret_cast<uint16_t*>(o)[2 * d + 1] = (uint16_t)((uint32_t)v[d] >> 16);
                                    }
                                }
                            } else {
#pragma unroll
                                for (int e = 2 * half; e < 2 * half + 2; ++e)
                                    if (n + e < g.N) reinterpret_cast<int*>(o)[e] = v[e];
                            }
                        }
                    }
                }
            });
            __builtin_amdgcn_s_waitcnt(kWaitLds);  // the rows are in registers before the next block overwrites them
        });
    };
    if (g.c_bf16) flush(std::integral_constant<bool, true>{});
    else flush(std::integral_constant<bool, false>{});
}

template <typename S>
int launch_ring(GemmArgs g, hipStream_t s) {
    // grouped: every group may end with a partial tile-row, so this is an upper bound (the surplus exits)
    const int64_t tiles_m = g.num_groups > 0 ? g.M / S::TM + g.num_groups : (g.M + S::TM - 1) / S::TM;
    const int64_t tiles_n = (g.N + S::TN - 1) / S::TN;
    if (g.num_groups > 0 && !S::kGen) return MX_EINVAL;
    if (tiles_m * tiles_n > (int64_t)1 << 30) return MX_EINVAL;
    g.tiles_m = (int)tiles_m;
    g.tiles_n = (int)tiles_n;
    const unsigned blocks = (unsigned)(((tiles_m * tiles_n + 7) / 8) * 8);
    auto* fn = gemm_ring_kernel<S>;
    static LdsOptIn opt_in;  // one per kernel instantiation
    if (int st = opt_in.ensure(reinterpret_cast<const void*>(fn), S::kLdsBytes)) return st;
    hipLaunchKernelGGL(fn, dim3(blocks), dim3(S::NT), S::kLdsBytes, s, g);
    return launch_status();
}

}  // namespace
}  // namespace mx
