// Block-scaled GEMM  C = A * B^T  with the Macro Block Scaling correction for operands in the 8-bit MX element
// formats (E4M3, E5M2; Sec. 1, footnote: the methods carry over to MXFP8), on v_mfma_scale_f32_32x32x64_f8f6f4.
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
// Pipeline: one macro block per stage through a ring of three LDS slots (256 + 128 rows x 128 B each).  The
// loads of stage s + 2 - code rows straight into LDS, 8 rows x 128 B per instruction; E8M0 dwords and MBS words
// into registers - are issued when stage s starts, after the barrier that publishes stage s and frees the slot
// of stage s - 1.  LDS image of a stage: [row][128 B], the 16-byte piece c of row r at position
// c ^ ((r >> 1) & 7), which spreads the 16 lanes of a fragment read over all banks.  Each wavefront turns its own
// 64 + 64 MBS words into fp32 sigma values in a private LDS table, so no second barrier is needed.
#include "mx_gemm_shared.h"

namespace mx {
namespace {

constexpr int kF8Slots = 3;
constexpr int kF8RowStage = kMacro;  // code bytes per row and stage
constexpr int kF8GroupM = 4;         // tile-rows walked together for L2 reuse

struct F8Shape {
    static constexpr int NWM = 4, NWN = 2, FM = 2, FN = 2, NW = NWM * NWN, NT = NW * kWave;
    static constexpr int TM = NWM * FM * 32, TN = NWN * FN * 32, kRows = TM + TN;
    static constexpr int kCodeDma = kRows / 8 / NW;        // per wavefront and stage: 8 rows x 128 B per load
    static constexpr int kRegLoads = FM + FN + 2;          // E8M0 dwords and MBS words per lane and stage
    static constexpr int kLoads = kCodeDma + kRegLoads;
    static constexpr int kStage = kRows * kF8RowStage;
    static constexpr int kSigmaBase = kF8Slots * kStage;
    static constexpr int kSigmaWave = (FM + FN) * 32 * 4;  // per wavefront: sigma of its A rows, then of its B rows
    static constexpr int kLdsBytes = kSigmaBase + NW * kSigmaWave;
    static constexpr int kStageRegion = 32 * (FN * 32 * 4 + 16);  // per wavefront, epilogue staging
    static_assert((TM / 8) % NW == 0 && (TN / 8) % NW == 0, "operand fixed per load index");
    static_assert(kLdsBytes <= 160 * 1024 && NW * kStageRegion <= kLdsBytes, "LDS capacity of a gfx950 compute unit");
    static_assert(2 * kLoads < 64, "vmcnt is a 6-bit counter");
};

// kFmtA / kFmtB: the matrix instruction's format selector of tensor A / B (0 = E4M3, 1 = E5M2).
template <int kFmtA, int kFmtB, bool kMbs>
__global__ __launch_bounds__(F8Shape::NT) void gemm_f8_kernel(GemmArgs g) {
    using S = F8Shape;
    constexpr int FM = S::FM, FN = S::FN, TM = S::TM, TN = S::TN, NW = S::NW, kCodeDma = S::kCodeDma;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- which tile: workgroups are dealt round-robin to the 8 XCDs; each XCD gets a contiguous run of tiles,
    // walked in bands of kF8GroupM tile-rows so that concurrent workgroups share panels in its L2
    const int total = g.tiles_m * g.tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int linear = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || linear >= total) return;
    const int band = kF8GroupM * g.tiles_n;
    const int first_m = (linear / band) * kF8GroupM;
    const int band_rows = min(g.tiles_m - first_m, kF8GroupM);
    const int tm = first_m + (linear % band) % band_rows;
    const int tn = (linear % band) / band_rows;
    const int64_t a_row0 = (int64_t)tm * TM, b_row0 = (int64_t)tn * TN;

    const int K = (int)g.K, scale_bytes = K >> 5, nmac = K / kMacro, nstages = nmac;
    // buffer resources rebased to the tile's first row and sized to its valid rows: rows past the end read zero
    const int kRsrcFlags = 0x00020000;
    const int64_t a_rows = min((int64_t)TM, g.M - a_row0), b_rows = min((int64_t)TN, g.N - b_row0);
    const __amdgpu_buffer_rsrc_t a_codes = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(g.a_codes) + a_row0 * K, 0, (int)(a_rows * K), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t b_codes = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(g.b_codes) + b_row0 * K, 0, (int)(b_rows * K), kRsrcFlags);
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
    int code_off[kCodeDma];
#pragma unroll
    for (int i = 0; i < kCodeDma; ++i) {
        const int row = ((i * NW + w) * 8 + (l >> 3)) - (i * NW * 8 < TM ? 0 : TM);  // row within its operand
        code_off[i] = row * K + (((l & 7) ^ ((row >> 1) & 7)) * 16);
    }
    int scale_off_a[FM], scale_off_b[FN];
#pragma unroll
    for (int i = 0; i < FM; ++i) scale_off_a[i] = ((wm * FM + i) * 32 + lr) * scale_bytes;
#pragma unroll
    for (int j = 0; j < FN; ++j) scale_off_b[j] = ((wn * FN + j) * 32 + lr) * scale_bytes;
    const int m8_off_a = (wm * FM * 32 + l) * nmac, m8_off_b = (wn * FN * 32 + l) * nmac;

    struct Pref {  // what a stage needs besides its codes
        uint32_t sa[FM], sb[FN];
        uint32_t ma, mb;
    };
    Pref pref[kF8Slots];

    // Loads of stage s into ring slot `slot`.  A stage past the end of K is never used; its loads fetch the last
    // one again (into a slot that is no longer read), so that every stage issues the same number of loads.
    auto issue = [&](int s, auto slot_) {
        constexpr int slot = decltype(slot_)::value;
        const int st = min(s, nstages - 1);
        asm volatile("" ::: "memory");
        static_for<kCodeDma>([&](auto i_) {
            constexpr int i = decltype(i_)::value;
            uint8_t* dst = smem + slot * S::kStage + (i * NW + w) * 1024;
            const int voff = code_off[i];
            if constexpr (i * NW * 8 < TM)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(a_codes, (lds_ptr_t)dst, 16, voff, st * kF8RowStage, 0, 0);
            else
                __builtin_amdgcn_raw_ptr_buffer_load_lds(b_codes, (lds_ptr_t)dst, 16, voff, st * kF8RowStage, 0, 0);
        });
        static_for<FM>([&](auto i_) {
            const int voff = scale_off_a[decltype(i_)::value];
            pref[slot].sa[decltype(i_)::value] = __builtin_amdgcn_raw_buffer_load_b32(a_scales, voff, st * 4, 0);
        });
        static_for<FN>([&](auto j_) {
            const int voff = scale_off_b[decltype(j_)::value];
            pref[slot].sb[decltype(j_)::value] = __builtin_amdgcn_raw_buffer_load_b32(b_scales, voff, st * 4, 0);
        });
        pref[slot].ma = __builtin_amdgcn_raw_buffer_load_b8(a_mbs, m8_off_a, st, 0);
        pref[slot].mb = __builtin_amdgcn_raw_buffer_load_b8(b_mbs, m8_off_b, st, 0);
        // (the waits below count loads: keep the compiler from mixing the loads of two stages)
        asm volatile("" ::: "memory");
    };

    v16f acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    float* sig = reinterpret_cast<float*>(smem + S::kSigmaBase + w * S::kSigmaWave);
    // this lane's 16-byte pieces inside a fragment's 32 rows: instruction kk, register half `part` takes the
    // piece lh of block 2 kk + part, i.e. piece 2 (2 kk + part) + lh of row lr
    int piece_off[2][2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int part = 0; part < 2; ++part)
            piece_off[kk][part] = lr * kF8RowStage + (((2 * (2 * kk + part) + lh) ^ ((lr >> 1) & 7)) * 16);

    auto stage = [&](int s, auto slot_) {
        constexpr int slot = decltype(slot_)::value;
        // own loads of stage s have landed (those of stage s + 1 may still fly); own LDS traffic is done.  (The
        // count is only right if every load of the previous stage's issue() has been issued by now: the empty
        // asm keeps the compiler from moving one across.)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(wait_imm(S::kLoads));
        bare_barrier();  // stage s is published; every wavefront has left stage s - 1, whose slot is free
        issue(s + 2, std::integral_constant<int, (slot + 2) % kF8Slots>{});

        float sig_m[FM];
        v4f sig_n[FN][4];
        if constexpr (kMbs) {
            sig[l] = __builtin_amdgcn_rcpf(1.0f + (float)pref[slot].ma * (1.0f / 256.0f));
            sig[64 + l] = __builtin_amdgcn_rcpf(1.0f + (float)pref[slot].mb * (1.0f / 256.0f));
        }
        // fragments of the stage
        v8i fa[FM][2], fb[FN][2];
        const uint8_t* base = smem + slot * S::kStage;
        static_for<FN>([&](auto j_) {
            constexpr int j = decltype(j_)::value;
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const uint8_t* p = base + (TM + (wn * FN + j) * 32) * kF8RowStage;
                const v4i lo = *reinterpret_cast<const v4i*>(p + piece_off[kk][0]);
                const v4i hi = *reinterpret_cast<const v4i*>(p + piece_off[kk][1]);
                fb[j][kk] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        });
        static_for<FM>([&](auto i_) {
            constexpr int i = decltype(i_)::value;
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const uint8_t* p = base + ((wm * FM + i) * 32) * kF8RowStage;
                const v4i lo = *reinterpret_cast<const v4i*>(p + piece_off[kk][0]);
                const v4i hi = *reinterpret_cast<const v4i*>(p + piece_off[kk][1]);
                fa[i][kk] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        });
        if constexpr (kMbs) {
#pragma unroll
            for (int i = 0; i < FM; ++i) sig_m[i] = sig[i * 32 + lr];
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq)
                    sig_n[j][gq] = *reinterpret_cast<const v4f*>(sig + 64 + j * 32 + gq * 8 + lh * 4);
        }
        // lane half h supplies the E8M0 byte of block 2 kk + h: bytes h and 2 + h of the row's four
        uint32_t scl_a[FM], scl_b[FN];
#pragma unroll
        for (int i = 0; i < FM; ++i) scl_a[i] = pref[slot].sa[i] >> (8 * lh);
#pragma unroll
        for (int j = 0; j < FN; ++j) scl_b[j] = pref[slot].sb[j] >> (8 * lh);

        if constexpr (kMbs) {
            constexpr int kPairs = FM * FN;
            v16f prod[2];
            auto product = [&](auto q_) {
                constexpr int q = decltype(q_)::value, j = q / FM, i = q % FM;
                v16f zero;
#pragma unroll
                for (int e = 0; e < 16; ++e) zero[e] = 0.f;
                prod[q % 2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[j][0], fa[i][0], zero, kFmtB, kFmtA, 0,
                                                                                (int)scl_b[j], 0, (int)scl_a[i]);
                prod[q % 2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[j][1], fa[i][1], prod[q % 2], kFmtB, kFmtA,
                                                                                2, (int)scl_b[j], 2, (int)scl_a[i]);
            };
            product(std::integral_constant<int, 0>{});
            static_for<kPairs>([&](auto q_) {
                constexpr int q = decltype(q_)::value, j = q / FM, i = q % FM;
                if constexpr (q + 1 < kPairs) product(std::integral_constant<int, q + 1>{});
                __builtin_amdgcn_sched_barrier(0);
                const float sm = sig_m[i];
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    acc[i][j][e] = fmaf(prod[q % 2][e], sm * sig_n[j][e / 4][e % 4], acc[i][j][e]);
                __builtin_amdgcn_sched_barrier(0);
            });
        } else {
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
                        acc[i][j] = kk == 0 ? __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                                                  fb[j][0], fa[i][0], acc[i][j], kFmtB, kFmtA, 0, (int)scl_b[j], 0, (int)scl_a[i])
                                            : __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                                                  fb[j][1], fa[i][1], acc[i][j], kFmtB, kFmtA, 2, (int)scl_b[j], 2, (int)scl_a[i]);
        }
    };

    // ---- prologue, main loop ----
    issue(0, std::integral_constant<int, 0>{});
    issue(1, std::integral_constant<int, 1>{});
    // (whole turns of the ring in the loop, the rest after it: a loop body with early exits would make the
    // compiler assume the shortest path between a register load and its use, and wait for far too much)
    int s = 0;
    for (; s + kF8Slots <= nstages; s += kF8Slots) {
        stage(s, std::integral_constant<int, 0>{});
        stage(s + 1, std::integral_constant<int, 1>{});
        stage(s + 2, std::integral_constant<int, 2>{});
    }
    if (s < nstages) {
        stage(s, std::integral_constant<int, 0>{});
        if (s + 1 < nstages) stage(s + 1, std::integral_constant<int, 1>{});
    }

    // ---- epilogue ----
    // A lane holds, per fragment, output row lr and the column groups 8 g + 4 h .. + 3.  Each wavefront passes its
    // block through its own piece of LDS, 32 output rows at a time, so that the global stores cover whole row
    // segments (16 bytes per lane, consecutive lanes along n).
    __builtin_amdgcn_s_waitcnt(wait_imm(0));
    bare_barrier();  // every wavefront's loads have landed and all LDS reads are done: the LDS is free
    constexpr int kCols = FN * 32;
    uint8_t* stg = smem + w * S::kStageRegion;
    const int64_t m0 = a_row0 + wm * FM * 32, n0 = b_row0 + wn * kCols;
    auto flush = [&](auto bf16_) {
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
                if (m < g.M && n < g.N) {
                    uint8_t* o = static_cast<uint8_t*>(g.C) + (m * g.ldc + n) * esz;
                    if (whole) {
                        __builtin_nontemporal_store(v, reinterpret_cast<v4i*>(o));
                    } else {
#pragma unroll
                        for (int e = 0; e < per; ++e) {
                            if (n + e >= g.N) break;
                            if constexpr (kBf16) reinterpret_cast<uint16_t*>(o)[e] = (uint16_t)((uint32_t)v[e >> 1] >> ((e & 1) * 16));
                            else reinterpret_cast<int*>(o)[e] = v[e];
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

template <int kFmtA, int kFmtB, bool kMbs>
int launch_f8_kernel(const GemmArgs& g, unsigned blocks, hipStream_t s) {
    using S = F8Shape;
    static bool attr_set = false;  // dynamic LDS above 64 KiB needs an opt-in once per process
    auto* fn = gemm_f8_kernel<kFmtA, kFmtB, kMbs>;
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

template <int kFmtA, int kFmtB>
int launch_f8(GemmArgs g, bool use_mbs, hipStream_t s) {
    using S = F8Shape;
    const int64_t tiles_m = (g.M + S::TM - 1) / S::TM, tiles_n = (g.N + S::TN - 1) / S::TN;
    if (tiles_m * tiles_n > (int64_t)1 << 30) return MX_EINVAL;
    g.tiles_m = (int)tiles_m;
    g.tiles_n = (int)tiles_n;
    const unsigned blocks = (unsigned)(((tiles_m * tiles_n + 7) / 8) * 8);
    return use_mbs ? launch_f8_kernel<kFmtA, kFmtB, true>(g, blocks, s) : launch_f8_kernel<kFmtA, kFmtB, false>(g, blocks, s);
}

int launch_gemm_elem(int a_elem, const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs, int b_elem,
                     const uint8_t* b_codes, const uint8_t* b_scales, const uint8_t* b_mbs, int64_t M, int64_t N,
                     int64_t K, int c_dtype, void* C, int64_t ldc, void* stream) {
    if (a_elem <= MX_ELEM_E2M1 || a_elem > MX_ELEM_E3M2 || b_elem <= MX_ELEM_E2M1 || b_elem > MX_ELEM_E3M2) return MX_EINVAL;
    if (M < 0 || N < 0 || K < 0 || (K % kBlock) != 0 || ldc < N) return MX_EINVAL;
    if (c_dtype != MX_OUT_F32 && c_dtype != MX_OUT_BF16) return MX_EINVAL;
    // (a tile's rows times the bytes of a row must fit the 32-bit offsets of the buffer loads)
    if (K > (int64_t)1 << 22 || M > (int64_t)1 << 30 || N > (int64_t)1 << 30) return MX_EINVAL;
    if (M == 0 || N == 0) return MX_OK;
    if (!C || (K > 0 && (!a_codes || !a_scales || !b_codes || !b_scales))) return MX_ENULL;
    const size_t esz = c_dtype == MX_OUT_F32 ? 4 : 2;
    if (!aligned(C, esz)) return MX_EALIGN;
    const bool fp8 = (a_elem == MX_ELEM_E4M3 || a_elem == MX_ELEM_E5M2) && (b_elem == MX_ELEM_E4M3 || b_elem == MX_ELEM_E5M2);
    if (!fp8 || K == 0 || (K % kMacro) != 0 || !aligned(a_codes, 16) || !aligned(b_codes, 16) || !aligned(a_scales, 4) ||
        !aligned(b_scales, 4))
        return MX_EUNSUPPORTED;
    if (int st = check_device()) return st;
    GemmArgs g = {};
    g.a_codes = a_codes; g.a_scales = a_scales; g.a_mbs = a_mbs;
    g.b_codes = b_codes; g.b_scales = b_scales; g.b_mbs = b_mbs;
    g.C = C;
    g.M = M; g.N = N; g.K = K; g.ldc = ldc;
    g.c_bf16 = c_dtype == MX_OUT_BF16;
    g.vec_store16 = aligned(C, 16) && (ldc * esz) % 16 == 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool use_mbs = a_mbs || b_mbs;
    const bool a5 = a_elem == MX_ELEM_E5M2, b5 = b_elem == MX_ELEM_E5M2;
    if (!a5 && !b5) return launch_f8<0, 0>(g, use_mbs, s);
    if (!a5 && b5) return launch_f8<0, 1>(g, use_mbs, s);
    if (a5 && !b5) return launch_f8<1, 0>(g, use_mbs, s);
    return launch_f8<1, 1>(g, use_mbs, s);
}

}  // namespace
}  // namespace mx

extern "C" int mx_gemm_mbs_elem(mx_elem_t a_elem, const uint8_t* a_codes, const uint8_t* a_scales,
                                const uint8_t* a_mbs_or_null, mx_elem_t b_elem, const uint8_t* b_codes,
                                const uint8_t* b_scales, const uint8_t* b_mbs_or_null, int64_t M, int64_t N, int64_t K,
                                mx_dtype_t c_dtype, void* C, int64_t ldc, void* stream) {
    return mx::launch_gemm_elem((int)a_elem, a_codes, a_scales, a_mbs_or_null, (int)b_elem, b_codes, b_scales,
                                b_mbs_or_null, M, N, K, (int)c_dtype, C, ldc, stream);
}
