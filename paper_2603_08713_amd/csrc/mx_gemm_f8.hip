// Block-scaled GEMM  C = A * B^T  with the Macro Block Scaling correction for operands in the 8-bit and 6-bit MX
// element formats (E4M3, E5M2, E2M3, E3M2; Sec. 1, footnote: the methods carry over to MXFP6 and MXFP8), on
// v_mfma_scale_f32_32x32x64_f8f6f4.
//
// The sum and the correction are those of the MXFP4 kernels (Sec. 4.3.2, App. E): per macro block of 128
// K-elements two matrix instructions start from a zero accumulator, and the vector ALUs fold their result in as
//     acc[m, n] += P[m, n] * sigma_A[m, g] * sigma_B[n, g],      sigma = 1 / (1 + m8 / 256).
// What differs is the balance.  An 8-bit operand is twice the bytes and the instruction runs twice as long, so
// per matrix instruction the vector ALUs have twice the time for the same correction, and LDS and L2 carry twice
// the bytes per output: a wavefront therefore owns 64 x 64 outputs (2 x 2 fragments, 1 KiB of LDS reads per
// matrix instruction) and a workgroup of eight wavefronts 256 x 128.
//
// Operand mapping (lane = 32 h + r), as measured on the device: srcA takes the weight matrix, srcB the
// activations; a lane holds row r; its first four operand registers hold 16 elements of the instruction's first
// 32-element block and its last four 16 elements of the second block (lane half h: elements 16 h .. 16 h + 15 of
// each); the first block is scaled by the E8M0 byte that lane half 0 supplies, the second by lane half 1's.
// Instruction kk of a macro block takes blocks 2 kk and 2 kk + 1: lane half h shifts the row's dword of four
// E8M0 bytes right by 8 h and op_sel picks byte 2 kk.  D[8 (j / 4) + 4 h + j % 4][r] is result register j.
//
// Pipeline: one macro block per stage through a ring of three LDS slots per operand (256 resp. 128 rows x 128 B).
// The registers hold the fragments of stage s while the loads of stages s + 1 and s + 2 are in flight; the
// barrier at the start of stage s publishes stage s + 1 and, because every wavefront read stage s out of its slot
// during stage s - 1, frees that slot for the loads of stage s + 3.  A fragment is refilled from stage s + 1 right
// after the last matrix instruction that reads it has been issued.  Code rows go straight into LDS, 8 rows x
// 128 B per instruction; LDS image of a stage: [row][128 B], the 16-byte piece c of row r at position
// c ^ ((r >> 1) & 7), which spreads the 16 lanes of a fragment read over all banks.
//
// E8M0 bytes and MBS words are a fraction of the bytes but not of the load instructions: a load of 4 bytes per
// lane from 64 different rows costs the texture-address unit as much as four loads of 16 bytes per lane, and
// fetched per stage they alone would take three times as long as the matrix instructions.  The fast form
// (K % 512 == 0, 16-byte aligned E8M0 rows, 4-byte aligned MBS rows) therefore fetches them per group of four
// stages: a row's 16 E8M0 bytes as one 16-byte piece into one of two LDS buffers, its four MBS words as one dword
// into a register of the thread that owns the row.  That thread turns the word of stage s + 1 into
// sigma = 1 / (1 + m8 / 256) during stage s, into one of two LDS tables that the barrier publishes.  The general
// form (any K % 64 == 0 from 128 on) fetches one dword of E8M0 bytes and one MBS word per lane and stage into registers and
// keeps a sigma table per wavefront.
//
// 6-bit operands (E2M3, E3M2; codes packed 32 to 24 bytes) run the fast form of the same template.  As for FP4, a
// lane half holds one whole block per instruction (instruction kk: block kk + 2 h) with the lane's own E8M0
// byte.  A stage is 96 bytes of a row; so that no 128-byte line of memory is fetched twice, the ring slots hold
// planes instead of stages: slot L = bytes 128 L .. + 127 of the 384 that a group of four stages takes of each
// row, loaded during stage L + 1 of the group before.  Details at the places marked kSix.  Their general form (any
// K % 64 == 0 from 128 on) keeps a stage per ring slot like the 8-bit one: the 96 bytes of a row sit in places 0 .. 5 of the
// row's eight 16-byte places, a quarter of the lanes of a code load fetch nothing, and a stage's bytes straddle the
// 128-byte lines of memory, so half of the lines are fetched twice (from the L2).
//
// Grouped problems (mx_gemm_mbs_elem_grouped) run the general form: a tile-row belongs to one group, whose rows of
// A and C and whose weight the workgroup looks up in row_offsets.
#include "mx_gemm_f8_schedule.h"
#include "mx_gemm_shared.h"
#include "mx_internal.h"

namespace mx {
namespace {

// kFmtA / kFmtB: the matrix instruction's format selector of tensor A / B (0 = E4M3, 1 = E5M2).
template <int kFmtA, int kFmtB, bool kMbs, bool kFast>
__global__ __launch_bounds__(F8Shape<kFast>::NT) void gemm_f8_kernel(GemmArgs g) {
    using S = F8Shape<kFast>;
    constexpr int FM = S::FM, FN = S::FN, TM = S::TM, TN = S::TN, NW = S::NW, kCodeDma = S::kCodeDma;
    // 6-bit codes (format selectors 2, 3) come packed, 24 bytes per block; both operands have the same width
    constexpr bool kSix = kFmtA >= 2;
    static_assert(kSix == (kFmtB >= 2), "6-bit operands: both or neither");
    // fast form: ring slots hold planes; general form: a slot holds a stage, six of a row's eight 16-byte places used
    constexpr bool kSixPlanes = kSix && kFast, kSixGen = kSix && !kFast;
    constexpr int kRowStage = kSix ? 96 : kF8RowStage;  // code bytes per row and stage
    // loads a wavefront makes per stage: what the stage's wait counts (a count that assumed more would let the
    // youngest loads of the stage it is about to read stay in flight)
    using Sched = F8Schedule<kSixPlanes ? kF8Six : kFast ? kF8Fast : kF8General, kMbs>;
    constexpr int kLoads = Sched::kLoads;
    static_assert(kLoads == S::kLoads - (kFast || kMbs ? 0 : 2) && Sched::kCodeDma == kCodeDma, "the schedule describes this kernel");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- which tile: workgroups are dealt round-robin to the 8 XCDs; each XCD gets a contiguous run of tiles,
    // walked in bands of kF8GroupM tile-rows so that concurrent workgroups share panels in its L2
    // (grouped: the launch took an upper bound of the tile-rows; the tiles are dealt out over the real number)
    int tiles_m = g.tiles_m;
    if constexpr (!kFast) {
        if (g.num_groups > 0) tiles_m = grouped_tile_rows(g.row_offsets, g.num_groups, TM, (int)(threadIdx.x & 63));
    }
    const int total = tiles_m * g.tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int linear = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || linear >= total) return;
    const int band = kF8GroupM * g.tiles_n;
    const int first_m = (linear / band) * kF8GroupM;
    const int band_rows = min(tiles_m - first_m, kF8GroupM);
    const int tm = first_m + (linear % band) % band_rows;
    const int tn = (linear % band) / band_rows;
    // Rows of A and C this tile covers and the rows of B it multiplies with.  Grouped (general form only): tile-rows
    // are counted group by group; group e owns rows row_offsets[e] .. row_offsets[e + 1] - 1 and the e-th of the
    // stacked [N, K] weights.
    int64_t a_row0 = (int64_t)tm * TM, a_end = g.M, b_row0 = (int64_t)tn * TN, b_end = g.N;
    if constexpr (!kFast) {
        if (g.num_groups > 0) {
            GroupOfTileRow gr;
            if (!grouped_find(g.row_offsets, g.num_groups, TM, (int)(threadIdx.x & 63), tm, gr)) return;
            a_row0 = gr.lo + (int64_t)(tm - gr.first) * TM;
            a_end = gr.hi;
            b_row0 = (int64_t)gr.group * g.N + (int64_t)tn * TN;
            b_end = (int64_t)(gr.group + 1) * g.N;
        }
    }

    // general form: K may end with half a macro block (K % 128 == 64): the last stage then holds two blocks of
    // every row; the pieces of its codes past the end of the row are fetched out of range (zeros), and its E8M0 dword
    // is fetched two bytes early, so that it ends with the row, and shifted down when it is used
    const int K = (int)g.K, scale_bytes = K >> 5, nmac = (K + kMacro - 1) / kMacro, nstages = nmac;
    const bool half_tail = !kFast && (K % kMacro) != 0;
    const int row_bytes = kSix ? K / 4 * 3 : K;
    // buffer resources rebased to the tile's first row and sized to its valid rows: rows past the end read zero
    const int kRsrcFlags = 0x00020000;
    const int64_t a_rows = min((int64_t)TM, a_end - a_row0), b_rows = min((int64_t)TN, b_end - b_row0);
    const __amdgpu_buffer_rsrc_t a_codes = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(g.a_codes) + a_row0 * row_bytes, 0, (int)(a_rows * row_bytes), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t b_codes = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(g.b_codes) + b_row0 * row_bytes, 0, (int)(b_rows * row_bytes), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t a_scales = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(g.a_scales) + a_row0 * scale_bytes, 0, (int)(a_rows * scale_bytes), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t b_scales = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(g.b_scales) + b_row0 * scale_bytes, 0, (int)(b_rows * scale_bytes), kRsrcFlags);
    // (an operand without MBS words gets an empty buffer: its words read 0, sigma = 1)
    const __amdgpu_buffer_rsrc_t a_mbs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(g.a_mbs ? g.a_mbs + a_row0 * nmac : g.a_codes), 0, g.a_mbs ? (int)(a_rows * nmac) : 0, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t b_mbs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(g.b_mbs ? g.b_mbs + b_row0 * nmac : g.b_codes), 0, g.b_mbs ? (int)(b_rows * nmac) : 0, kRsrcFlags);

    const int tid = threadIdx.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w % S::NWM, wn = w / S::NWM;
    const int lr = l & 31, lh = l >> 5;

    // ---- per-lane byte offsets of the loads (constant over the K loop; the stage goes into the scalar offset) ----
    // Codes: load i of wavefront w covers rows (i * NW + w) * 8 .. + 7 of the A-then-B row space; lane l writes LDS
    // position l of that 1-KiB block and fetches row l / 8, piece (l % 8) ^ ((row >> 1) & 7).
    // (load i adds i * NW * 8 whole rows, which leaves (row >> 1) & 7 as it is; the row has to stay in the per-lane
    // offset, the only part of the address the hardware checks against the buffer's valid rows)
    // 6-bit codes: a stage is 96 bytes of a row, which would straddle the 128-byte lines of the memory system; the
    // unit of loading is therefore a plane, 128 bytes of every row, a third of the group of four stages (384 bytes
    // a row).  Ring slot L holds plane L of the current group, in the 8-bit layout, and is loaded again, with the
    // next group's plane, during stage L + 1 of the group, after the last fragment that reads it has been fetched.
    // (6-bit general form: a slot holds a stage like an 8-bit one; a row's places 6 and 7 are never read, and the
    // lanes that would fill them fetch nothing)
    const int code_row0 = w * 8 + (l >> 3);
    const int code_piece = (l & 7) ^ ((code_row0 >> 1) & 7);
    const bool code_idle = kSixGen && code_piece >= 6;
    const int code_off0 = code_row0 * row_bytes + code_piece * 16;
    // (last stage: the lane's piece lies past the end of the row)
    const int tail_soff = (nstages - 1) * kRowStage;
    const bool code_past_tail = !kFast && tail_soff + code_piece * 16 >= row_bytes;
    // general form: a lane's E8M0 dword per fragment and stage, and the MBS word of the row it converts
    const int scale_off_a0 = (wm * FM * 32 + lr) * scale_bytes, scale_off_b0 = (wn * FN * 32 + lr) * scale_bytes;
    const int m8_off_a = (wm * FM * 32 + l) * nmac, m8_off_b = (wn * FN * 32 + l) * nmac;
    // fast form: thread t < kRows owns row t of the A-then-B row space (wavefronts 0 .. 3: A, 4 and 5: B)
    const bool owner_is_a = w * kWave < TM;
    const int own_row = tid - (owner_is_a ? 0 : TM);
    const int own_scale_off = tid < S::kRows ? own_row * scale_bytes : kOob, own_m8_off = tid < S::kRows ? own_row * nmac : kOob;

    struct Pref {  // general form: what a stage needs besides its codes
        uint32_t sa[FM], sb[FN];
        uint32_t ma, mb;
    };
    Pref pref[kFast ? 1 : kF8Slots];
    uint32_t own_m8[kF8Slots] = {0u, 0u, 0u};  // fast form: the owned row's four MBS words of group g, in g % 3

    // load i of the codes that start soff bytes into their rows into ring slot `slot`
    auto issue_code = [&](int soff, auto slot_, auto i_) __attribute__((always_inline)) {
        constexpr int slot = decltype(slot_)::value, i = decltype(i_)::value, kLoadsA = TM / 8 / NW;
        const bool idle = code_idle || (!kFast && code_past_tail && soff == tail_soff);
        if constexpr (i < kLoadsA) {
            uint8_t* dst = smem + S::kBaseA + slot * S::kStageA + (i * NW + w) * 1024;
            const int voff = idle ? kOob : code_off0 + i * NW * 8 * row_bytes;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(a_codes, (lds_ptr_t)dst, 16, voff, soff, 0, 0);
        } else if constexpr (i < kCodeDma) {
            uint8_t* dst = smem + S::kBaseB + slot * S::kStageB + ((i - kLoadsA) * NW + w) * 1024;
            const int voff = idle ? kOob : code_off0 + (i - kLoadsA) * NW * 8 * row_bytes;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(b_codes, (lds_ptr_t)dst, 16, voff, soff, 0, 0);
        }
    };
    // Fast form: E8M0 bytes and MBS words of the four stages of group grp, the E8M0 bytes into LDS buffer grp % 2
    // ([row][16]), the words into own_m8[grp % 3].  Wavefronts 6 and 7 own no rows: their loads are out of range
    // and their 16-byte pieces (zeros) go to a spare KiB, which keeps the sequence free of branches.
    const int ngroups = nstages / S::kGroup;
    const bool owns = w * kWave < S::kRows;
    const __amdgpu_buffer_rsrc_t own_scales = owner_is_a ? a_scales : b_scales, own_mbs = owner_is_a ? a_mbs : b_mbs;
    auto issue_group = [&](int grp, auto mod3_) __attribute__((always_inline)) {  // mod3_: grp % 3
        const int gg = min(grp, ngroups - 1);
        uint8_t* dst = smem + (owns ? S::kSmallBase + (grp & 1) * S::kScaleGroup + w * 1024 : S::kSpare);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(own_scales, (lds_ptr_t)dst, 16, own_scale_off, gg * 16, 0, 0);
        own_m8[decltype(mod3_)::value] = __builtin_amdgcn_raw_buffer_load_b32(own_mbs, own_m8_off, gg * 4, 0);
    };
    // General form: E8M0 dwords and MBS words of stage st into the registers of ring slot `slot`.
    auto issue_regs = [&](int st, auto slot_) __attribute__((always_inline)) {
        constexpr int slot = decltype(slot_)::value;
        if constexpr (!kFast) {
            const int scale_soff = st * 4 - (half_tail && st == nstages - 1 ? 2 : 0);
            static_for<FM>([&](auto i_) {
                const int voff = scale_off_a0 + decltype(i_)::value * 32 * scale_bytes;
                pref[slot].sa[decltype(i_)::value] = __builtin_amdgcn_raw_buffer_load_b32(a_scales, voff, scale_soff, 0);
            });
            static_for<FN>([&](auto j_) {
                const int voff = scale_off_b0 + decltype(j_)::value * 32 * scale_bytes;
                pref[slot].sb[decltype(j_)::value] = __builtin_amdgcn_raw_buffer_load_b32(b_scales, voff, scale_soff, 0);
            });
            if constexpr (kMbs) {
                pref[slot].ma = __builtin_amdgcn_raw_buffer_load_b8(a_mbs, m8_off_a, st, 0);
                pref[slot].mb = __builtin_amdgcn_raw_buffer_load_b8(b_mbs, m8_off_b, st, 0);
            }
        }
    };
    // All loads of stage s at once (prologue).  The stage's waits count loads: the empty asm keeps the compiler from
    // mixing the loads of two stages.
    auto issue = [&](int s, auto slot_) __attribute__((always_inline)) {
        const int st = min(s, nstages - 1);
        asm volatile("" ::: "memory");
        issue_regs(st, slot_);
        static_for<kCodeDma>([&](auto i_) { issue_code(st * kRowStage, slot_, i_); });
        asm volatile("" ::: "memory");
    };

    v16f acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // general form: this wavefront's sigma table; fast form: the workgroup's two tables, [row] of the A-then-B space
    float* sig = reinterpret_cast<float*>(smem + S::kSigmaBase + (kFast ? 0 : w * S::kSigmaWave));
    // The LDS read instruction adds a 16-bit constant to its address register: with the wavefront's first row
    // folded into the register, ring slot and fragment are that constant, and A's third slot, which lies more
    // than 64 KiB up, gets a second copy of the registers (the empty asm keeps the compiler from folding the
    // copies back into one base plus additions).
    int frag_b[2][2], frag_a[2][2], frag_a_hi[2][2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int part = 0; part < 2; ++part) {
            // 8-bit: piece 2 (2 kk + part) + lh of row lr, swizzled (6-bit operands have registers of their own)
            const int piece = lr * kF8RowStage + (((2 * (2 * kk + part) + lh) ^ ((lr >> 1) & 7)) * 16);
            frag_b[kk][part] = S::kBaseB + wn * FN * 32 * kF8RowStage + piece;
            frag_a[kk][part] = S::kBaseA + wm * FM * 32 * kF8RowStage + piece;
            frag_a_hi[kk][part] = frag_a[kk][part] + 65536;
            asm volatile("" : "+v"(frag_b[kk][part]));
            asm volatile("" : "+v"(frag_a[kk][part]));
            asm volatile("" : "+v"(frag_a_hi[kk][part]));
        }

    // 6-bit: the lane's blocks kk + 2 lh of stage q of the group are the 48 bytes from 96 q + 48 lh of the row's
    // 384, that is the 16-byte pieces 6 q + 3 lh .. + 2 of the group's 24 (eight to a plane, swizzled like the
    // 8-bit pieces): instruction 0 reads the first piece and half of the second, instruction 1 the other half and
    // the third.
    int six_a[kSixPlanes ? 4 : 1][3], six_b[kSixPlanes ? 4 : 1][3];
    if constexpr (kSixPlanes) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                const int piece = 6 * q + 3 * lh + c, plane = piece >> 3;
                const int at = lr * kF8RowStage + (((piece & 7) ^ ((lr >> 1) & 7)) * 16);
                six_b[q][c] = S::kBaseB + plane * S::kStageB + wn * FN * 32 * kF8RowStage + at;
                six_a[q][c] = S::kBaseA + plane * S::kStageA + wm * FM * 32 * kF8RowStage + at;
                asm volatile("" : "+v"(six_b[q][c]));
                asm volatile("" : "+v"(six_a[q][c]));
            }
    }

    // 6-bit, general form: the stage's six pieces sit at places 0 .. 5 of the row's eight, swizzled like the 8-bit
    // pieces; the lane's blocks are pieces 3 lh .. 3 lh + 2.  Slot and fragment go into the instruction's constant,
    // with a second copy of the registers for A's third slot as above.
    int gsix_b[3], gsix_a[3], gsix_a_hi[3];
    if constexpr (kSixGen) {
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            const int at = lr * kF8RowStage + (((3 * lh + c) ^ ((lr >> 1) & 7)) * 16);
            gsix_b[c] = S::kBaseB + wn * FN * 32 * kF8RowStage + at;
            gsix_a[c] = S::kBaseA + wm * FM * 32 * kF8RowStage + at;
            gsix_a_hi[c] = gsix_a[c] + 65536;
            asm volatile("" : "+v"(gsix_b[c]));
            asm volatile("" : "+v"(gsix_a[c]));
            asm volatile("" : "+v"(gsix_a_hi[c]));
        }
    }

    // Operands of one macro block in registers.  They are refilled in place: a fragment takes the next stage's
    // data right after the last matrix instruction that reads it has been issued.
    v8i fa[FM][2], fb[FN][2];
    // (slot_: the ring slot; for 6-bit operands the stage's place in its group.  LDS reads go through plain vector
    // types: before a read through one of HIP's vector structs, uint2 say, the compiler puts a wait for every
    // outstanding direct-to-LDS load.)
    auto read_frag = [&](auto slot_, auto is_a_, auto idx_, auto kk_) __attribute__((always_inline)) {
        constexpr int slot = decltype(slot_)::value, idx = decltype(idx_)::value, kk = decltype(kk_)::value;
        constexpr bool is_a = decltype(is_a_)::value;
        v8i v;
        if constexpr (kSix) {
            // (fast form: slot_ is the stage's place in its group; general form: the ring slot, in the constant)
            constexpr int off = kSixGen ? (is_a ? slot * S::kStageA : slot * S::kStageB) : 0;
            constexpr bool far = kSixGen && is_a && off + idx * 32 * kF8RowStage >= 65536;
            const int* at = kSixGen ? (is_a ? (far ? gsix_a_hi : gsix_a) : gsix_b) : (is_a ? six_a[slot] : six_b[slot]);
            constexpr int row0 = idx * 32 * kF8RowStage + (far ? off - 65536 : off);
            // The middle piece is read once, whole, into registers 4 .. 7 of instruction 0's operand (the matrix
            // instruction takes six registers of a 6-bit operand; the last two ride along) and its second half is
            // copied into registers 0 and 1 of instruction 1's operand by patch_frags(), once the read has
            // landed: three 16-byte reads per fragment instead of two and two 8-byte reads, which the LDS serves
            // no faster than 16-byte ones (two lanes of a 32-lane pass share a bank pair).
            if constexpr (kk == 0) {
                const v4i p0 = *reinterpret_cast<const v4i*>(smem + at[0] + row0);
                const v4i p1 = *reinterpret_cast<const v4i*>(smem + at[1] + row0);
                v = __builtin_shufflevector(p0, p1, 0, 1, 2, 3, 4, 5, 6, 7);
            } else {
                const v8i old = is_a ? fa[idx][1] : fb[idx][1];
                const v4i p2 = *reinterpret_cast<const v4i*>(smem + at[2] + row0);
                v = v8i{old[0], old[1], p2.x, p2.y, p2.z, p2.w, old[6], old[7]};
            }
        } else {
            constexpr int off = (is_a ? slot * S::kStageA : slot * S::kStageB) + idx * 32 * kF8RowStage;
            constexpr bool far = is_a && off >= 65536;  // past the range of the instruction's constant
            const int b0 = is_a ? (far ? frag_a_hi[kk][0] : frag_a[kk][0]) : frag_b[kk][0];
            const int b1 = is_a ? (far ? frag_a_hi[kk][1] : frag_a[kk][1]) : frag_b[kk][1];
            const v4i lo = *reinterpret_cast<const v4i*>(smem + b0 + (far ? off - 65536 : off));
            const v4i hi = *reinterpret_cast<const v4i*>(smem + b1 + (far ? off - 65536 : off));
            v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
        if constexpr (is_a) fa[idx][kk] = v;
        else fb[idx][kk] = v;
    };
    using IsA = std::integral_constant<bool, true>;
    using IsB = std::integral_constant<bool, false>;
    // 6-bit: second half of every fragment's middle piece into its place (after the wait for the fragment reads)
    auto patch_frags = [&]() __attribute__((always_inline)) {
        if constexpr (kSix) {
#pragma unroll
            for (int i = 0; i < FM; ++i) { fa[i][1][0] = fa[i][0][6]; fa[i][1][1] = fa[i][0][7]; }
#pragma unroll
            for (int j = 0; j < FN; ++j) { fb[j][1][0] = fb[j][0][6]; fb[j][1][1] = fb[j][0][7]; }
        }
    };

    // E8M0 operands of a stage.  8-bit: lane half h supplies the byte of block 2 kk + h, i.e. bytes h and 2 + h of the
    // row's four, so the dword goes in shifted right by 8 h and op_sel picks byte 0 or 2.  6-bit: the lane's own
    // block kk + 2 h: shifted right by 16 h, op_sel picks byte 0 or 1.
    constexpr int kSclShift = kSix ? 16 : 8, kSel1 = kSix ? 1 : 2;  // op_sel of a macro block's second instruction
    uint32_t scl_a[FM], scl_b[FN];
    const int lane_scale_a = S::kSmallBase + (wm * FM * 32 + lr) * 16, lane_scale_b = S::kSmallBase + (TM + wn * FN * 32 + lr) * 16;
    auto read_scales_fast = [&](int s) __attribute__((always_inline)) {  // stage s out of its group's LDS buffer
        const int at = ((s / S::kGroup) & 1) * S::kScaleGroup + (s % S::kGroup) * 4;
#pragma unroll
        for (int i = 0; i < FM; ++i)
            scl_a[i] = *reinterpret_cast<const uint32_t*>(smem + lane_scale_a + at + i * 32 * 16) >> (kSclShift * lh);
#pragma unroll
        for (int j = 0; j < FN; ++j)
            scl_b[j] = *reinterpret_cast<const uint32_t*>(smem + lane_scale_b + at + j * 32 * 16) >> (kSclShift * lh);
    };
    // fast form: the owner of a row turns its MBS word of stage s into sigma, into table s % 2
    auto convert_sigma_fast = [&](int s, auto mod3_) __attribute__((always_inline)) {  // mod3_: (s / 4) % 3
        const uint32_t words = own_m8[decltype(mod3_)::value];
        const uint32_t m8 = (words >> (8 * (s % S::kGroup))) & 0xFFu;
        // (threads that own no row store to the spare KiB: no branch)
        float* dst = tid < S::kRows ? sig + (s & 1) * S::kRows + tid : reinterpret_cast<float*>(smem + S::kSpare) + l;
        *dst = __builtin_amdgcn_rcpf(1.0f + (float)m8 * (1.0f / 256.0f));
    };

    // MBS: the product of a stage's last pair is folded into the accumulators at the start of the next stage, behind
    // that stage's first matrix instructions (otherwise every stage begins with the vector ALUs waiting for the
    // first product and ends with the matrix pipeline idle behind the last, in both wavefronts of a SIMD at once);
    // it waits in prod[1] with its sigma values.  The first stage folds in zeros.  (Fast form only: the general
    // form has no registers to spare for it.)
    constexpr bool kDefer = kMbs && kFast;
    v16f prod[2];
    float last_sm = 0.f;
    uint32_t last_sn[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int e = 0; e < 16; ++e) prod[0][e] = prod[1][e] = 0.f;
    // acc[i][j] += prod[which] * sm * sn (sn: the lane's four sigma_B registers of the fragment, fetched by DPP)
    auto fold = [&](auto i_, auto j_, auto which_, float sm, const uint32_t (&sn)[4]) __attribute__((always_inline)) {
        constexpr int i = decltype(i_)::value, j = decltype(j_)::value, which = decltype(which_)::value;
        // sigma_A * sigma_B with the DPP fetch folded into the multiply (written out: the compiler keeps the
        // fetch as a move of its own); four products at a time, so that no multiply-add follows the
        // multiply it depends on directly (the compiler would put a wait state between the two)
        static_for<4>([&](auto gq_) {
            constexpr int gq = decltype(gq_)::value;
            float w0, w1, w2, w3;
            asm("v_mul_f32_dpp %0, %1, %2 quad_perm:[0,0,0,0] row_mask:0xf bank_mask:0xf bound_ctrl:1" : "=v"(w0) : "v"(sn[gq]), "v"(sm));
            asm("v_mul_f32_dpp %0, %1, %2 quad_perm:[1,1,1,1] row_mask:0xf bank_mask:0xf bound_ctrl:1" : "=v"(w1) : "v"(sn[gq]), "v"(sm));
            asm("v_mul_f32_dpp %0, %1, %2 quad_perm:[2,2,2,2] row_mask:0xf bank_mask:0xf bound_ctrl:1" : "=v"(w2) : "v"(sn[gq]), "v"(sm));
            asm("v_mul_f32_dpp %0, %1, %2 quad_perm:[3,3,3,3] row_mask:0xf bank_mask:0xf bound_ctrl:1" : "=v"(w3) : "v"(sn[gq]), "v"(sm));
            acc[i][j][4 * gq + 0] = fmaf(prod[which][4 * gq + 0], w0, acc[i][j][4 * gq + 0]);
            acc[i][j][4 * gq + 1] = fmaf(prod[which][4 * gq + 1], w1, acc[i][j][4 * gq + 1]);
            acc[i][j][4 * gq + 2] = fmaf(prod[which][4 * gq + 2], w2, acc[i][j][4 * gq + 2]);
            acc[i][j][4 * gq + 3] = fmaf(prod[which][4 * gq + 3], w3, acc[i][j][4 * gq + 3]);
        });
    };
    using LastI = std::integral_constant<int, FM - 1>;
    using LastJ = std::integral_constant<int, FN - 1>;
    using Prod1 = std::integral_constant<int, 1>;
    static_assert((FM * FN) % 2 == 0, "the last pair's product waits in prod[1], which the next stage's first pair leaves alone");

    // One stage.  On entry the registers hold the fragments (fast form: and the E8M0 operands) of stage s; the
    // loads of stages s + 1 and s + 2 are in flight.
    auto stage = [&](int s, auto slot_, auto phase_) __attribute__((always_inline)) {
        constexpr int slot = decltype(slot_)::value;
        constexpr int p = decltype(phase_)::value % S::kGroup;  // fast form: the stage's place in its group
        using Next = std::integral_constant<int, kSixPlanes ? (p + 1) % S::kGroup : (slot + 1) % kF8Slots>;
        // own loads of stage s + 1 have landed (those of stage s + 2 may still fly; the fast form's group loads
        // are requested ahead of a stage's codes, so they have landed a stage after their request); own LDS
        // traffic is done.  (The count is only right if every load of the earlier issue() calls has been issued
        // by now: the empty asm keeps the compiler from moving one across.)
        // 6-bit: the pieces the next stage's fragments come from belong to planes requested two stages ago or
        // earlier; since then came one stage's plane (six loads) or, before the group's second stage, the group
        // loads (of which the second may still fly).
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(wait_imm(Sched::stage_wait(p)));
        bare_barrier();
        patch_frags();
        if constexpr (kFast) {
            // (t: the stage's place in the turn of the loop, 3 groups of 4 stages)
            constexpr int t = decltype(phase_)::value;
            if constexpr (kMbs) convert_sigma_fast(s + 1, std::integral_constant<int, (t + 1) / S::kGroup % 3>{});  // (past the end: a table nobody reads)
            if constexpr (t % S::kGroup == 0) issue_group(s / S::kGroup + 1, std::integral_constant<int, (t / S::kGroup + 1) % 3>{});
        } else {
            // what this stage needs of its prefetched registers, before the loads of stage s + 3 take them over
            // (half a macro block at the end of K: the dword was fetched two bytes early; shifted down, the bytes of
            // the two blocks that do not exist read 0, a finite scale for their zero codes)
            const uint32_t early = half_tail && s == nstages - 1 ? 16u : 0u;
#pragma unroll
            for (int i = 0; i < FM; ++i) scl_a[i] = (pref[slot].sa[i] >> early) >> (kSclShift * lh);
#pragma unroll
            for (int j = 0; j < FN; ++j) scl_b[j] = (pref[slot].sb[j] >> early) >> (kSclShift * lh);
            if constexpr (kMbs) {
                sig[l] = __builtin_amdgcn_rcpf(1.0f + (float)pref[slot].ma * (1.0f / 256.0f));
                sig[64 + l] = __builtin_amdgcn_rcpf(1.0f + (float)pref[slot].mb * (1.0f / 256.0f));
            }
        }
        // the loads of stage s + 3: registers now (general form), the codes one by one behind the matrix
        // instructions - a direct-to-LDS load holds its wavefront up for as long as the texture-address unit needs
        // for its 64 lanes, and six in a row from all eight wavefronts would stall the matrix pipeline
        const int st3 = min(s + 3, nstages - 1);
        issue_regs(st3, slot_);
        // (6-bit: plane p - 1 of the next group, which the last group fetches from itself again; nothing in the
        // group's first stage)
        using CodeSlot = std::integral_constant<int, kSixPlanes ? (p > 0 ? p - 1 : 0) : slot>;
        const int code_soff = kSixPlanes ? min(s / S::kGroup + 1, ngroups - 1) * (S::kGroup * kRowStage) + (p - 1) * 128 : st3 * kRowStage;
        auto issue_next = [&](auto i_) __attribute__((always_inline)) {
            if constexpr (!kSixPlanes || p > 0) issue_code(code_soff, CodeSlot{}, i_);
        };

        // sigma of this lane's output row per A fragment; of its 16 output columns per B fragment, kept as four
        // registers: lane l holds the value of column 8 gq + 4 h + l % 4, and the multiply fetches column i from
        // lane i of its group of four (DPP quad_perm), a quarter of the LDS traffic of reading all sixteen into
        // every lane
        float sig_m[FM];
        uint32_t sig_n[FN][4];
        if constexpr (kMbs) {
            const float* sa = kFast ? sig + (s & 1) * S::kRows + wm * FM * 32 : sig;
            const float* sb = kFast ? sig + (s & 1) * S::kRows + TM + wn * FN * 32 : sig + 64;
#pragma unroll
            for (int i = 0; i < FM; ++i) sig_m[i] = sa[i * 32 + lr];
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) sig_n[j][gq] = __float_as_uint(sb[j * 32 + gq * 8 + lh * 4 + (l & 3)]);
        }
        if constexpr (kMbs) {
            constexpr int kPairs = FM * FN;
            auto product = [&](auto q_) __attribute__((always_inline)) {  // the instructions of pair q, then the refills they make possible
                constexpr int q = decltype(q_)::value, j = q / FM, i = q % FM;
                v16f zero;
#pragma unroll
                for (int e = 0; e < 16; ++e) zero[e] = 0.f;
                prod[q % 2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[j][0], fa[i][0], zero, kFmtB, kFmtA, 0,
                                                                                (int)scl_b[j], 0, (int)scl_a[i]);
                issue_next(std::integral_constant<int, 2 * q>{});
                prod[q % 2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[j][1], fa[i][1], prod[q % 2], kFmtB, kFmtA,
                                                                                kSel1, (int)scl_b[j], kSel1, (int)scl_a[i]);
                issue_next(std::integral_constant<int, 2 * q + 1>{});
                if constexpr (i == FM - 1) {
                    read_frag(Next{}, IsB{}, std::integral_constant<int, j>{}, std::integral_constant<int, 0>{});
                    read_frag(Next{}, IsB{}, std::integral_constant<int, j>{}, std::integral_constant<int, 1>{});
                }
                if constexpr (j == FN - 1) {
                    read_frag(Next{}, IsA{}, std::integral_constant<int, i>{}, std::integral_constant<int, 0>{});
                    read_frag(Next{}, IsA{}, std::integral_constant<int, i>{}, std::integral_constant<int, 1>{});
                }
            };
            product(std::integral_constant<int, 0>{});
            if constexpr (kDefer) {
                __builtin_amdgcn_sched_barrier(0);
                fold(LastI{}, LastJ{}, Prod1{}, last_sm, last_sn);  // the stage before
                __builtin_amdgcn_sched_barrier(0);
            }
            static_for<kPairs>([&](auto q_) {
                constexpr int q = decltype(q_)::value, j = q / FM, i = q % FM;
                if constexpr (q + 1 < kPairs) product(std::integral_constant<int, q + 1>{});
                // (every instruction of the stage has its E8M0 operands: the next stage's may replace them)
                if constexpr (kFast && q + 1 == kPairs - 1) read_scales_fast(s + 1);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (q + 1 < kPairs || !kDefer) {
                    fold(std::integral_constant<int, i>{}, std::integral_constant<int, j>{}, std::integral_constant<int, q % 2>{}, sig_m[i], sig_n[j]);
                } else {
                    last_sm = sig_m[i];
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq) last_sn[gq] = sig_n[j][gq];
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        } else {
            // instruction t: half kk = t / (FM FN) of pair (i, j); a fragment half is refilled after its last use
            static_for<2 * FM * FN>([&](auto t_) {
                constexpr int t = decltype(t_)::value, kk = t / (FM * FN), i = t % (FM * FN) / FN, j = t % FN;
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[j][kk], fa[i][kk], acc[i][j], kFmtB, kFmtA, kSel1 * kk,
                                                                             (int)scl_b[j], kSel1 * kk, (int)scl_a[i]);
                issue_next(t_);
                if constexpr (i == FM - 1) read_frag(Next{}, IsB{}, std::integral_constant<int, j>{}, std::integral_constant<int, kk>{});
                if constexpr (j == FN - 1) read_frag(Next{}, IsA{}, std::integral_constant<int, i>{}, std::integral_constant<int, kk>{});
                if constexpr (kFast && t == 2 * FM * FN - 1) read_scales_fast(s + 1);
                __builtin_amdgcn_sched_barrier(0);
            });
        }
    };

    // ---- prologue: three stages of loads in flight, the fragments of stage 0 into registers ----
    if constexpr (kFast) issue_group(0, std::integral_constant<int, 0>{});
    if constexpr (kSixPlanes) {  // the three planes of group 0
        static_for<kF8Slots>([&](auto L_) {
            static_for<kCodeDma>([&](auto i_) { issue_code(decltype(L_)::value * 128, L_, i_); });
        });
        asm volatile("" ::: "memory");
    } else {
        issue(0, std::integral_constant<int, 0>{});
        issue(1, std::integral_constant<int, 1>{});
        issue(2, std::integral_constant<int, 2>{});
    }
    __builtin_amdgcn_s_waitcnt(wait_imm(Sched::prologue_wait()));
    if constexpr (kFast && kMbs) {
        convert_sigma_fast(0, std::integral_constant<int, 0>{});
        __builtin_amdgcn_s_waitcnt(kWaitLds);
    }
    bare_barrier();
    static_for<2>([&](auto kk_) {
        static_for<FN>([&](auto j_) { read_frag(std::integral_constant<int, 0>{}, IsB{}, j_, kk_); });
        static_for<FM>([&](auto i_) { read_frag(std::integral_constant<int, 0>{}, IsA{}, i_, kk_); });
    });
    patch_frags();
    if constexpr (kFast) read_scales_fast(0);
    // The loop body is a whole number of turns of the ring and, in the fast form, of groups, so that ring slot and
    // place in the group are compile-time constants; what is left of K follows after the loop, as the first
    // stages of one more turn.  (A loop body with early exits would also make the compiler assume the shortest
    // path between a register load and its use, and wait for far too much.)
    constexpr int kTurn = kFast ? kF8Slots * S::kGroup : kF8Slots;
    constexpr int kStep = kFast ? S::kGroup : 1;  // the stage count is a multiple of this
    auto run = [&](int s0, auto first_, auto count_) __attribute__((always_inline)) {
        static_for<decltype(count_)::value>([&](auto t_) {
            constexpr int t = decltype(first_)::value + decltype(t_)::value;
            stage(s0 + t, std::integral_constant<int, t % kF8Slots>{}, std::integral_constant<int, t>{});
        });
    };
    using Zero = std::integral_constant<int, 0>;
    using Step = std::integral_constant<int, kStep>;
    int s = 0;
    for (; s + kTurn <= nstages; s += kTurn) run(s, Zero{}, std::integral_constant<int, kTurn>{});
    if (s < nstages) {
        run(s, Zero{}, Step{});
        if (s + kStep < nstages) run(s, Step{}, Step{});
    }

    if constexpr (kDefer) fold(LastI{}, LastJ{}, Prod1{}, last_sm, last_sn);  // the last stage's last pair

    // ---- epilogue ----
    // A lane holds, per fragment, output row lr and the column groups 8 g + 4 h .. + 3.  Each wavefront passes its
    // block through its own piece of LDS, 32 output rows at a time, so that the global stores cover whole row
    // segments (16 bytes per lane, consecutive lanes along n).
    __builtin_amdgcn_s_waitcnt(wait_imm(0));
    bare_barrier();  // every wavefront's loads have landed and all LDS reads are done: the LDS is free
    constexpr int kCols = FN * 32;
    uint8_t* stg = smem + w * S::kStageRegion;
    const int64_t m0 = a_row0 + wm * FM * 32, n0 = (int64_t)tn * TN + wn * kCols;
    auto flush = [&](auto bf16_) __attribute__((always_inline)) {
        constexpr bool kBf16 = decltype(bf16_)::value;
        constexpr int esz = kBf16 ? 2 : 4, per = 16 / esz;
        constexpr int pitch = kCols * esz + 16;  // the pad spreads the staged rows over the banks
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

template <int kFmtA, int kFmtB, bool kMbs, bool kFast>
int launch_f8_kernel(const GemmArgs& g, unsigned blocks, hipStream_t s) {
    using S = F8Shape<kFast>;
    auto* fn = gemm_f8_kernel<kFmtA, kFmtB, kMbs, kFast>;
    static LdsOptIn opt_in;  // one per kernel instantiation
    if (int st = opt_in.ensure(reinterpret_cast<const void*>(fn), S::kLdsBytes)) return st;
    hipLaunchKernelGGL(fn, dim3(blocks), dim3(S::NT), S::kLdsBytes, s, g);
    return launch_status();
}

template <int kFmtA, int kFmtB>
int launch_f8(GemmArgs g, bool use_mbs, bool force_general, hipStream_t s) {
    using S = F8Shape<true>;
    // grouped: every group may end with a partial tile-row, so this is an upper bound (the surplus exits)
    const int64_t tiles_m = g.num_groups > 0 ? g.M / S::TM + g.num_groups : (g.M + S::TM - 1) / S::TM;
    const int64_t tiles_n = (g.N + S::TN - 1) / S::TN;
    if (tiles_m * tiles_n > (int64_t)1 << 30) return MX_EINVAL;
    g.tiles_m = (int)tiles_m;
    g.tiles_n = (int)tiles_n;
    const unsigned blocks = (unsigned)(((tiles_m * tiles_n + 7) / 8) * 8);
    // fast form: E8M0 bytes and MBS words travel per group of four stages, as 16-byte pieces and dwords
    // (grouped problems take the general form: a group's rows of E8M0 bytes and MBS words start anywhere)
    const bool fast = !force_general && g.num_groups == 0 && (g.K % 512) == 0 && aligned(g.a_scales, 16) && aligned(g.b_scales, 16) &&
                      (!g.a_mbs || aligned(g.a_mbs, 4)) && (!g.b_mbs || aligned(g.b_mbs, 4));
    if (fast)
        return use_mbs ? launch_f8_kernel<kFmtA, kFmtB, true, true>(g, blocks, s) : launch_f8_kernel<kFmtA, kFmtB, false, true>(g, blocks, s);
    return use_mbs ? launch_f8_kernel<kFmtA, kFmtB, true, false>(g, blocks, s) : launch_f8_kernel<kFmtA, kFmtB, false, false>(g, blocks, s);
}

// force: 0 = automatic, 1 = the main kernel's general form, 2 = the main kernel in the form the problem allows, 3 = the
// few-row kernel
int launch_gemm_elem(int a_elem, const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs, int b_elem,
                     const uint8_t* b_codes, const uint8_t* b_scales, const uint8_t* b_mbs, int num_groups,
                     const int64_t* row_offsets, bool grouped, int64_t M, int64_t N, int64_t K, int c_dtype, void* C,
                     int64_t ldc, void* stream, int force = 0) {
    if (a_elem <= MX_ELEM_E2M1 || a_elem > MX_ELEM_E3M2 || b_elem <= MX_ELEM_E2M1 || b_elem > MX_ELEM_E3M2) return MX_EINVAL;
    if (M < 0 || N < 0 || K < 0 || (K % kBlock) != 0 || ldc < N) return MX_EINVAL;
    if (c_dtype != MX_OUT_F32 && c_dtype != MX_OUT_BF16) return MX_EINVAL;
    if (grouped && num_groups < 0) return MX_EINVAL;
    // (a tile's rows times the bytes of a row must fit the 32-bit offsets of the buffer loads)
    if (K > (int64_t)1 << 22 || M > (int64_t)1 << 30 || N > (int64_t)1 << 30 ||
        (grouped && (int64_t)num_groups * N > (int64_t)1 << 40))
        return MX_EINVAL;
    if (M == 0 || N == 0 || (grouped && num_groups == 0)) return MX_OK;
    if (!C || (grouped && !row_offsets) || (K > 0 && (!a_codes || !a_scales || !b_codes || !b_scales))) return MX_ENULL;
    const size_t esz = c_dtype == MX_OUT_F32 ? 4 : 2;
    if (!aligned(C, esz)) return MX_EALIGN;
    const bool a8 = a_elem == MX_ELEM_E4M3 || a_elem == MX_ELEM_E5M2, b8 = b_elem == MX_ELEM_E4M3 || b_elem == MX_ELEM_E5M2;
    // K in whole macro blocks, or ending with half of one (the general form; rows of E8M0 bytes then start on even
    // addresses only)
    const bool half_tail = (K % kMacro) != 0;
    if (a8 != b8 || K == 0 || (K % (kMacro / 2)) != 0 || K < kMacro || !aligned(a_codes, 16) || !aligned(b_codes, 16) ||
        !aligned(a_scales, half_tail ? 2 : 4) || !aligned(b_scales, half_tail ? 2 : 4))
        return MX_EUNSUPPORTED;
    if (int st = check_device()) return st;
    GemmArgs g = {};
    g.a_codes = a_codes; g.a_scales = a_scales; g.a_mbs = a_mbs;
    g.b_codes = b_codes; g.b_scales = b_scales; g.b_mbs = b_mbs;
    g.C = C; g.row_offsets = row_offsets;
    g.M = M; g.N = N; g.K = K; g.ldc = ldc;
    g.num_groups = grouped ? num_groups : 0;
    g.c_bf16 = c_dtype == MX_OUT_BF16;
    g.vec_store16 = aligned(C, 16) && (ldc * esz) % 16 == 0;
    g.vec_store8 = aligned(C, 8) && (ldc * esz) % 8 == 0;
    g.vec_store4 = aligned(C, 4) && (ldc * esz) % 4 == 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool use_mbs = a_mbs || b_mbs;
    const bool force_general = force == 1;
    // few activation rows: the weights are streamed once, nothing is staged (mx_gemm_skinny_f8.hip)
    const bool skinny_ok = !grouped && M <= 64 && (K % 512) == 0 && K <= 8192 && aligned(a_scales, 16) && aligned(b_scales, 16) &&
                           (!a_mbs || aligned(a_mbs, 4)) && (!b_mbs || aligned(b_mbs, 4));
    if (force == 3 && !skinny_ok) return MX_EINVAL;
    if (skinny_ok && (force == 0 || force == 3)) return launch_gemm_skinny_elem(g, a_elem, b_elem, s);
    if (!a8) {
        const bool a32 = a_elem == MX_ELEM_E3M2, b32 = b_elem == MX_ELEM_E3M2;
        if (!a32 && !b32) return launch_f8<2, 2>(g, use_mbs, force_general, s);
        if (!a32 && b32) return launch_f8<2, 3>(g, use_mbs, force_general, s);
        if (a32 && !b32) return launch_f8<3, 2>(g, use_mbs, force_general, s);
        return launch_f8<3, 3>(g, use_mbs, force_general, s);
    }
    const bool a5 = a_elem == MX_ELEM_E5M2, b5 = b_elem == MX_ELEM_E5M2;
    if (!a5 && !b5) return launch_f8<0, 0>(g, use_mbs, force_general, s);
    if (!a5 && b5) return launch_f8<0, 1>(g, use_mbs, force_general, s);
    if (a5 && !b5) return launch_f8<1, 0>(g, use_mbs, force_general, s);
    return launch_f8<1, 1>(g, use_mbs, force_general, s);
}

}  // namespace
}  // namespace mx

extern "C" int mx_gemm_mbs_elem(mx_elem_t a_elem, const uint8_t* a_codes, const uint8_t* a_scales,
                                const uint8_t* a_mbs_or_null, mx_elem_t b_elem, const uint8_t* b_codes,
                                const uint8_t* b_scales, const uint8_t* b_mbs_or_null, int64_t M, int64_t N, int64_t K,
                                mx_dtype_t c_dtype, void* C, int64_t ldc, void* stream) {
    return mx::launch_gemm_elem((int)a_elem, a_codes, a_scales, a_mbs_or_null, (int)b_elem, b_codes, b_scales,
                                b_mbs_or_null, 0, nullptr, false, M, N, K, (int)c_dtype, C, ldc, stream);
}

extern "C" int mx_gemm_mbs_elem_grouped(mx_elem_t a_elem, const uint8_t* a_codes, const uint8_t* a_scales,
                                        const uint8_t* a_mbs_or_null, mx_elem_t b_elem, const uint8_t* b_codes,
                                        const uint8_t* b_scales, const uint8_t* b_mbs_or_null, int32_t num_groups,
                                        const int64_t* row_offsets, int64_t M_total, int64_t N, int64_t K,
                                        mx_dtype_t c_dtype, void* C, int64_t ldc, void* stream) {
    return mx::launch_gemm_elem((int)a_elem, a_codes, a_scales, a_mbs_or_null, (int)b_elem, b_codes, b_scales,
                                b_mbs_or_null, num_groups, row_offsets, true, M_total, N, K, (int)c_dtype, C, ldc, stream);
}

extern "C" int mx_internal_gemm_elem(mx_elem_t a_elem, const uint8_t* a_codes, const uint8_t* a_scales,
                                     const uint8_t* a_mbs_or_null, mx_elem_t b_elem, const uint8_t* b_codes,
                                     const uint8_t* b_scales, const uint8_t* b_mbs_or_null, int64_t M, int64_t N,
                                     int64_t K, mx_dtype_t c_dtype, void* C, int64_t ldc, int force, void* stream) {
    return mx::launch_gemm_elem((int)a_elem, a_codes, a_scales, a_mbs_or_null, (int)b_elem, b_codes, b_scales,
                                b_mbs_or_null, 0, nullptr, false, M, N, K, (int)c_dtype, C, ldc, stream, force);
}
