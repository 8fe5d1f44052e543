// Block-scaled MXFP4 GEMM  C = A * B^T  without the MBS correction: the large-tile kernel for gfx950.
//
// Without MBS nothing but the matrix cores touches the accumulators, so the kernel is built around
// what limits v_mfma_scale_f32_32x32x64_f8f6f4 in practice: instruction issue and data movement.
//   * Four wavefronts per workgroup, one per SIMD, each owning a 128 x 128 (FM x FN fragments of 32 x 32)
//     block of the 256 x 256 tile.  The 16 accumulator fragments (256 registers) live in the accumulation
//     half of the register file; the operand fragments of two macro blocks in the other half.  The large
//     register tile reads each LDS byte for 4 matrix instructions.
//   * K advances one macro block (128 elements, 64 code bytes and 4 E8M0 bytes per row) per stage through
//     a ring of four LDS slots.  While stage s is multiplied out of registers, stage s + 1 is read from
//     LDS into the other register set and the direct-to-LDS loads of stage s + 4 are issued into the slot
//     stage s has just left: three stages are in flight, enough to cover a miss in the L2.
//   * One workgroup barrier per stage.  It publishes stage s + 1 and, because every wavefront has
//     finished reading stage s by then, frees its slot.
//
// Operand mapping of the instruction (lane = 32 h + r): srcA/srcB hold row r, k-block h of the
// instruction's two 32-element blocks (16 bytes of FP4); the scale operand is one E8M0 byte per lane;
// D[8 (j / 4) + 4 h + j % 4][r] is result register j.  The two instructions of a fragment pair split
// the macro block so that lane half h takes blocks 2 h and 2 h + 1: its two E8M0 bytes are neighbours
// in the row's scale dword, one 16-bit LDS read fetches both and op_sel picks the byte.  As in the
// other kernel the weight matrix feeds srcA, so a lane ends up with groups of four consecutive n of one
// output row m.
//
// LDS image of a stage: codes [row][64 B] with the 16-byte chunk c of row r at position
// c ^ ((r >> 2) & 3), which keeps the 16-lane groups of a fragment read on distinct banks and lets four
// lanes of a load fetch one contiguous 64-byte piece of a row; scales [row] dwords.
#include "mx_gemm_shared.h"

namespace mx {
namespace {

constexpr int kWideStageK = kMacro;            // K elements per stage
constexpr int kWideRowStage = kWideStageK / 2;  // code bytes per row and stage
constexpr int kWideSlots = 4;
constexpr int kWideGroup = 4;                   // stages per 16-byte piece of a row's E8M0 bytes
constexpr int kWideGroupM = 4;                  // tile-rows walked together for L2 reuse

template <int NWM_, int NWN_, int FM_, int FN_>
struct WideShape {
    static constexpr int NWM = NWM_, NWN = NWN_, FM = FM_, FN = FN_;
    static constexpr int NW = NWM * NWN, NT = NW * kWave;
    static constexpr int TM = NWM * FM * 32, TN = NWN * FN * 32;
    static constexpr int kRows = TM + TN;
    static constexpr int kCodeDma = kRows / 16 / NW;   // 16 rows x 64 B per load
    static constexpr int kScaleDma = ceil_div(kRows, kWave * NW);  // 64 rows x 16 B per load, once per group
    static constexpr int kCodesStage = kRows * kWideRowStage;
    static constexpr int kScaleGroup = kScaleDma * NW * kWave * 16;
    static constexpr int kScaleBase = kWideSlots * kCodesStage;
    static constexpr int kLdsBytes = kScaleBase + 2 * kScaleGroup;
    static_assert(NW == 4, "one wavefront per SIMD");
    static_assert((TM / 16) % NW == 0 && (TN / 16) % NW == 0, "16-row code loads: operand fixed per load index");
    static_assert(kLdsBytes <= 160 * 1024, "LDS capacity of a gfx950 compute unit");
    static_assert(FM * FN * 16 <= 256, "accumulators fill at most the accumulation registers");
};

template <typename S>
__global__ __launch_bounds__(S::NT) void gemm_wide_kernel(GemmArgs g) {
    constexpr int FM = S::FM, FN = S::FN, TM = S::TM, TN = S::TN, NW = S::NW, kRows = S::kRows;
    constexpr int kCodeDma = S::kCodeDma, kScaleDma = S::kScaleDma;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- which tile: XCD-contiguous runs, bands of kWideGroupM tile-rows (as in the other kernel) -------
    const int total = g.tiles_m * g.tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int linear = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || linear >= total) return;
    const int band = kWideGroupM * g.tiles_n;
    const int first_m = (linear / band) * kWideGroupM;
    const int band_rows = min(g.tiles_m - first_m, kWideGroupM);
    const int tm = first_m + (linear % band) % band_rows;
    const int tn = (linear % band) / band_rows;
    const int64_t a_row0 = (int64_t)tm * TM, b_row0 = (int64_t)tn * TN;

    const int K = (int)g.K;
    const int row_bytes = K >> 1, scale_bytes = K >> 5;
    const int nstages = K / kWideStageK, ngroups = nstages / kWideGroup;
    const Operand opa = make_operand(g.a_codes, g.a_scales, nullptr, a_row0, g.M, TM, g.K);
    const Operand opb = make_operand(g.b_codes, g.b_scales, nullptr, b_row0, g.N, TN, g.K);

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
    // Scales: load i of wavefront w fetches, for row (i * NW + w) * 64 + l, the 16 E8M0 bytes of a group of
    // four stages (one 16-byte piece per lane costs the memory pipeline a quarter of four dword loads);
    // rows past the tile are padding and read zero.
    int scale_off[kScaleDma];
    bool scale_is_a[kScaleDma];
#pragma unroll
    for (int i = 0; i < kScaleDma; ++i) {
        const int grow = (i * NW + w) * kWave + l;
        scale_is_a[i] = (i * NW + w) * kWave < TM;
        scale_off[i] = grow >= kRows ? kOob : (grow - (scale_is_a[i] ? 0 : TM)) * scale_bytes;
    }

    // A stage past the end of K is never multiplied; its loads (the pipeline issues them regardless, into
    // slots that are no longer read) fetch the last stage again, so that no address leaves the operands.
    auto dma_code = [&](int s, auto i_) {  // load i of the codes of stage s
        constexpr int i = decltype(i_)::value;
        uint8_t* dst = smem + (s % kWideSlots) * S::kCodesStage + (i * NW + w) * 1024;
        const int voff = code_off[i];  // (a named copy: passed as an array element the host pass drops the kernel)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(i * NW * 16 < TM ? opa.codes : opb.codes, (lds_ptr_t)dst, 16, voff,
                                                 min(s, nstages - 1) * kWideRowStage, 0, 0);
    };
    auto dma_scale = [&](int grp, auto i_) {  // load i of the E8M0 bytes of stages 4 grp .. 4 grp + 3
        constexpr int i = decltype(i_)::value;
        uint8_t* dst = smem + S::kScaleBase + (grp & 1) * S::kScaleGroup + (i * NW + w) * 1024;
        const int voff = scale_off[i];  // (named copies, as above)
        const __amdgpu_buffer_rsrc_t rsrc = scale_is_a[i] ? opa.scales : opb.scales;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)dst, 16, voff, min(grp, ngroups - 1) * 16, 0, 0);
    };

    // ---- operand fragments of one macro block in registers ----------------------------------------
    struct Frags {
        v4i m[FM][2], n[FN][2];
        uint32_t scl_m[FM], scl_n[FN];
    };
    int frag_off[2];  // this lane's 16 bytes inside a fragment's 32 rows, per instruction of the pair
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) frag_off[kk] = lr * kWideRowStage + (((lh * 2 + kk) ^ ((lr >> 2) & 3)) * 16);
    const int lane_scale = lr * 16 + lh * 2;

    // LDS read `idx` of the kReads that fetch the fragments of stage s: per fragment (A's FM, then B's FN) the
    // two 16-byte code pieces and the 16-bit scale pair.
    constexpr int kReads = (FM + FN) * 3;
    auto read_item = [&](Frags& f, int s, auto idx_) {
        constexpr int idx = decltype(idx_)::value, fr = idx / 3, part = idx % 3;
        constexpr bool is_m = fr < FM;
        constexpr int q = is_m ? fr : fr - FM;
        const int row0 = is_m ? (wm * FM + q) * 32 : TM + (wn * FN + q) * 32;  // in the A-then-B row space
        if constexpr (part < 2) {
            const v4i v = *reinterpret_cast<const v4i*>(smem + (s % kWideSlots) * S::kCodesStage + row0 * kWideRowStage +
                                                        frag_off[part]);
            if constexpr (is_m) f.m[q][part] = v;
            else f.n[q][part] = v;
        } else {
            const uint32_t v = *(lds_half_ptr_t)(smem + S::kScaleBase + ((s / kWideGroup) & 1) * S::kScaleGroup +
                                                 (s % kWideGroup) * 4 + lane_scale + row0 * 16);
            if constexpr (is_m) f.scl_m[q] = v;
            else f.scl_n[q] = v;
        }
    };

    v16f acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // ---- prologue: fill the ring, fetch the fragments of stage 0 -------------------------------------
    static_assert(kWideSlots * kCodeDma + kScaleDma < 64, "vmcnt is a 6-bit counter");
    static_for<kScaleDma>([&](auto i_) { dma_scale(0, i_); });
    static_for<kWideSlots * kCodeDma>([&](auto t_) {
        constexpr int t = decltype(t_)::value;
        dma_code(t / kCodeDma, std::integral_constant<int, t % kCodeDma>{});
    });
    __builtin_amdgcn_s_waitcnt(wait_imm((kWideSlots - 1) * kCodeDma));
    bare_barrier();
    Frags f0, f1;
    static_for<kReads>([&](auto idx_) { read_item(f0, 0, idx_); });

    // One stage: publish stage s + 1; multiply stage s out of `cur`; after each matrix instruction issue one
    // LDS read of stage s + 1 into `next` and, with kIssue, the loads of stage s + 4 (into the slot of stage
    // s); the first stage of a group (kPhase 0) also requests the scales of the next group, into the slot
    // the previous group left two stages ago.  The two instructions of a fragment pair are FM * FN
    // instructions apart, so none waits for its predecessor.  A direct-to-LDS load holds up its wavefront
    // while the texture-address unit, which the four SIMDs share, works through its 64 lanes: the
    // wavefronts therefore issue theirs at different instruction slots, two wavefronts per slot.
    constexpr int kMfmas = FM * FN * 2;
    static_assert(kReads <= kMfmas, "one LDS read per matrix instruction");
    auto stage = [&](int s, const Frags& cur, Frags& next, auto phase_, auto late_, auto issue_) {
        constexpr int kPhase = decltype(phase_)::value, kLate = decltype(late_)::value;
        constexpr bool kIssue = decltype(issue_)::value;
        constexpr int kLoads = kCodeDma + (kPhase == 0 ? kScaleDma : 0);
        // Own loads of stage s + 1 (and, before the last stage of a group, of the next group's scales) have
        // landed; the loads issued in the last two stages may still fly.  Own reads of `cur` are done.
        constexpr int kYounger = 2 * kCodeDma + (kPhase == 1 || kPhase == 2 ? kScaleDma : 0);
        __builtin_amdgcn_s_waitcnt(wait_imm(kIssue ? kYounger : 0));
        bare_barrier();
        static_for<kMfmas>([&](auto t_) {
            constexpr int t = decltype(t_)::value, kk = t / (FM * FN), i = t % (FM * FN) / FN, j = t % FN;
            acc[i][j] = mfma_fp4_wide<kk, kk>(cur.n[j][kk], cur.m[i][kk], acc[i][j], cur.scl_n[j], cur.scl_m[i]);
            if constexpr (t < kReads) read_item(next, s + 1, t_);
            if constexpr (kIssue) {
                static_for<kLoads>([&](auto n_) {
                    constexpr int n = decltype(n_)::value, slot = (n * kMfmas) / kLoads + kLate;
                    if constexpr ((slot < kMfmas ? slot : kMfmas - 1) == t) {
                        if constexpr (n < kCodeDma) dma_code(s + kWideSlots, n_);
                        else dma_scale(s / kWideGroup + 1, std::integral_constant<int, n - kCodeDma>{});
                    }
                });
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    // Stages whose iteration still has a stage s + 4 to request, rounded up to whole groups (the extra ones
    // fetch the last stage again into slots that are no longer read); the rest runs without loads.
    const int n_issue = (max(nstages - kWideSlots, 0) + kWideGroup - 1) / kWideGroup * kWideGroup;
    auto run = [&](auto late_) {
        using Yes = std::integral_constant<bool, true>;
        using No = std::integral_constant<bool, false>;
        using P0 = std::integral_constant<int, 0>;
        using P1 = std::integral_constant<int, 1>;
        using P2 = std::integral_constant<int, 2>;
        using P3 = std::integral_constant<int, 3>;
        int s = 0;
        for (; s < n_issue; s += 4) {
            stage(s, f0, f1, P0{}, late_, Yes{});
            stage(s + 1, f1, f0, P1{}, late_, Yes{});
            stage(s + 2, f0, f1, P2{}, late_, Yes{});
            stage(s + 3, f1, f0, P3{}, late_, Yes{});
        }
        for (; s < nstages; s += 4) {  // nstages is a multiple of the group
            stage(s, f0, f1, P0{}, late_, No{});
            stage(s + 1, f1, f0, P1{}, late_, No{});
            stage(s + 2, f0, f1, P2{}, late_, No{});
            stage(s + 3, f1, f0, P3{}, late_, No{});
        }
    };
    if (w < 2) run(std::integral_constant<int, 0>{});
    else run(std::integral_constant<int, 1>{});

    // ---- epilogue ------------------------------------------------------------------------------------
    // A lane holds, per fragment, output row lr and the column groups 8 g + 4 h .. + 3.  Each wavefront
    // passes its block through its own piece of LDS, 32 output rows at a time, so that the global stores
    // cover whole row segments (16 bytes per lane, consecutive lanes along n).
    __builtin_amdgcn_s_waitcnt(wait_imm(0));
    bare_barrier();  // every wavefront's loads have landed and all fragment reads are done: the LDS is free
    constexpr int kCols = FN * 32;
    uint8_t* stg = smem + w * (32 * (kCols * 4 + 16));
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
                if (m < g.M && n < g.N) {
                    uint8_t* o = static_cast<uint8_t*>(g.C) + (m * g.ldc + n) * esz;
                    if (whole) {
                        *reinterpret_cast<v4i*>(o) = v;
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

template <typename S>
int launch_wide_variant(GemmArgs g, hipStream_t s) {
    const int64_t tiles_m = (g.M + S::TM - 1) / S::TM, tiles_n = (g.N + S::TN - 1) / S::TN;
    if (tiles_m * tiles_n > (int64_t)1 << 30) return MX_EINVAL;
    g.tiles_m = (int)tiles_m;
    g.tiles_n = (int)tiles_n;
    const unsigned blocks = (unsigned)(((tiles_m * tiles_n + 7) / 8) * 8);
    static bool attr_set = false;  // dynamic LDS above 64 KiB needs an opt-in once per process
    auto* fn = gemm_wide_kernel<S>;
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

}  // namespace

// Plain (no MBS, not grouped) GEMM on 256 x 256 tiles.  Requires K % 512 == 0, K > 0 and 16-byte aligned scale
// arrays (the E8M0 bytes of four stages are fetched as one 16-byte piece); the caller has checked both.
int launch_gemm_wide(const GemmArgs& g, hipStream_t s) {
    using S = WideShape<2, 2, 4, 4>;
    return launch_wide_variant<S>(g, s);
}

}  // namespace mx
