// Tile shape and load schedule of the GEMM kernel for 8-bit and 6-bit operands (mx_gemm_f8.hip): what the kernel
// keeps in LDS, which loads a wavefront issues in a stage, in which order, and how many of its youngest loads may
// still be in flight when a stage starts.  Plain constexpr C++ with no device code, so that a host program can
// replay the schedule of every form and check it (tests/schedule_check.cpp).
//
// K advances one macro block (a "stage") at a time through three LDS code slots per operand.  A wavefront's loads
// complete in the order it issued them; a stage starts with s_waitcnt vmcnt(n) and the workgroup's barrier, after
// which the codes of stage s + 1 (read from LDS during stage s) and, in the fast forms, the E8M0 bytes of that
// stage's group of four must have landed.
//
// Three forms:
//   general (8-bit and 6-bit, any K % 128 == 0): a stage issues, for stage s + 3, one dword of E8M0 bytes per fragment and
//       (with MBS words) one word per operand into registers, then the code loads into slot s % 3, which the stage
//       itself has left.  What was issued during the stage before may fly.
//   fast (8-bit, K % 512 == 0, aligned rows): E8M0 bytes and MBS words travel per group of four stages: the first
//       stage of a group issues the next group's two loads (16 bytes of E8M0 per row into one of two LDS buffers,
//       the row's four words into a register) ahead of its code loads.
//   six (6-bit, the fast form's conditions): a stage is 96 bytes of a row; the unit of loading is a plane, 128
//       bytes of every row, a third of a group's 384.  Slot L holds plane L of the current group and is loaded
//       again, with the next group's plane L, during stage L + 1 of the group; the group's first stage issues the
//       group loads only.  The fragments of stage q of a group are the 16-byte pieces 6 q .. 6 q + 5 of the
//       group's 24, i.e. planes (6 q) / 8 .. (6 q + 5) / 8.
#pragma once

#include "mx_constants.h"

namespace mx {

constexpr int kF8Slots = 3;
constexpr int kF8RowStage = kMacro;  // code bytes per row and stage (8-bit)
constexpr int kF8GroupM = 4;         // tile-rows walked together for L2 reuse

template <bool kFast_>
struct F8Shape {
    static constexpr bool kFast = kFast_;
    static constexpr int NWM = 4, NWN = 2, FM = 2, FN = 2, NW = NWM * NWN, NT = NW * kWave;
    static constexpr int TM = NWM * FM * 32, TN = NWN * FN * 32, kRows = TM + TN;
    static constexpr int kCodeDma = kRows / 8 / NW;                     // per wavefront and stage: 8 rows x 128 B per load
    static constexpr int kRegLoads = kFast ? 0 : FM + FN + 2;           // general form: E8M0 dwords and MBS words per lane and stage
    static constexpr int kLoads = kCodeDma + kRegLoads;                 // (the general form without MBS loads no words: two fewer)
    static constexpr int kGroup = 4;                                    // fast form: stages per 16-byte piece of E8M0 bytes
    static constexpr int kStageA = TM * kF8RowStage, kStageB = TN * kF8RowStage, kStage = kStageA + kStageB;
    static constexpr int kBaseB = 0, kBaseA = kF8Slots * kStageB;       // the ring slots of B, then those of A
    static constexpr int kSmallBase = kF8Slots * kStage;
    // fast form: two buffers of [row][16 E8M0 bytes], two tables of [row] sigma; general form: a table per wavefront
    static constexpr int kScaleGroup = kRows * 16, kSigmaTable = kRows * 4;
    static constexpr int kSigmaBase = kSmallBase + (kFast ? 2 * kScaleGroup : 0);
    static constexpr int kSigmaWave = (FM + FN) * 32 * 4;
    static constexpr int kSpare = kSigmaBase + 2 * kSigmaTable;         // fast form: 1 KiB nobody reads
    static constexpr int kLdsBytes = kFast ? kSpare + 1024 : kSigmaBase + NW * kSigmaWave;
    static constexpr int kStageRegion = 32 * (FN * 32 * 4 + 16);        // per wavefront, epilogue staging
    static_assert((TM / 8) % NW == 0 && (TN / 8) % NW == 0, "operand fixed per load index");
    static_assert(kRows % kWave == 0 && TM % kWave == 0, "fast form: a wavefront's rows belong to one operand");
    static_assert(kLdsBytes <= 160 * 1024 && NW * kStageRegion <= kLdsBytes, "LDS capacity of a gfx950 compute unit");
    static_assert(kCodeDma <= 2 * FM * FN - 2 && 3 * kLoads + 4 < 64, "vmcnt is a 6-bit counter");
};

// ---- load schedule ----------------------------------------------------------------------------------------------
enum F8Form { kF8General = 0, kF8Fast = 1, kF8Six = 2 };
// codes: `what` is the stage (8-bit forms) or the plane counted over all groups, 3 g + L (six); group loads: the
// group; register loads of the general form: the stage.  Only kF8Code and kF8GroupScale write LDS.
enum F8LoadKind { kF8Code = 0, kF8GroupScale = 1, kF8GroupWords = 2, kF8RegScale = 3, kF8RegWords = 4 };
struct F8LoadItem {
    int kind, what, index;
};

template <int kForm, bool kMbs>
struct F8Schedule {
    using S = F8Shape<kForm != kF8General>;
    static constexpr int kCodeDma = S::kCodeDma, kGroup = S::kGroup;
    static constexpr int kRegScales = kForm == kF8General ? S::FM + S::FN : 0;
    static constexpr int kRegWords = kForm == kF8General && kMbs ? 2 : 0;
    static constexpr int kLoads = kCodeDma + kRegScales + kRegWords;  // per stage, 8-bit forms

    // ---- the loop: loads that stage s issues, in order.  p = s % kGroup; `what` relative as noted.
    static constexpr int issue_count(int p) {
        if (kForm == kF8General) return kLoads;
        if (kForm == kF8Fast) return (p == 0 ? 2 : 0) + kCodeDma;
        return p == 0 ? 2 : kCodeDma;
    }
    // General: registers, then codes of stage s + 3.  Fast: at p == 0 the E8M0 bytes and the words of group
    // s / 4 + 1, then the codes of stage s + 3.  Six: at p == 0 the group loads of group s / 4 + 1; at p > 0 plane
    // p - 1 of group s / 4 + 1.
    static constexpr F8LoadItem issue_item(int p, int n) {
        if (kForm == kF8General) {
            if (n < kRegScales) return F8LoadItem{kF8RegScale, 3, n};
            if (n < kRegScales + kRegWords) return F8LoadItem{kF8RegWords, 3, n - kRegScales};
            return F8LoadItem{kF8Code, 3, n - kRegScales - kRegWords};
        }
        if (p == 0 && n < 2) return F8LoadItem{n == 0 ? kF8GroupScale : kF8GroupWords, 1, 0};
        if (kForm == kF8Fast) return F8LoadItem{kF8Code, 3, n - (p == 0 ? 2 : 0)};
        return F8LoadItem{kF8Code, 3 + (p - 1), n};  // plane 3 (g + 1) + p - 1, counted from 3 g
    }
    // Loads that may still be in flight when stage s starts.  8-bit forms: what the stage before issued for stage
    // s + 2 (its codes; in the fast form the group loads go ahead of a stage's codes and have landed a stage after
    // their request).  Six: the planes the next stage's fragments come from were requested two stages ago or
    // earlier; since then came one stage's plane, or, before a group's second stage, the group loads, of which the
    // second (the words, into a register) may fly.
    static constexpr int stage_wait(int p) {
        if (kForm == kF8Six) return p == 1 ? 1 : kCodeDma;
        return kLoads;
    }

    // ---- the prologue: fast forms first the group loads of group 0; then the codes (general: all loads) of stages
    // 0, 1, 2 (six: planes 0, 1, 2 of group 0)
    static constexpr int prologue_count() { return (kForm == kF8General ? 0 : 2) + 3 * (kForm == kF8General ? kLoads : kCodeDma); }
    static constexpr F8LoadItem prologue_item(int n) {
        if (kForm != kF8General) {
            if (n < 2) return F8LoadItem{n == 0 ? kF8GroupScale : kF8GroupWords, 0, 0};
            n -= 2;
            return F8LoadItem{kF8Code, n / kCodeDma, n % kCodeDma};
        }
        const int st = n / kLoads, k = n % kLoads;
        if (k < kRegScales) return F8LoadItem{kF8RegScale, st, k};
        if (k < kRegScales + kRegWords) return F8LoadItem{kF8RegWords, st, k - kRegScales};
        return F8LoadItem{kF8Code, st, k - kRegScales - kRegWords};
    }
    // before the first LDS reads (codes of stage 0, fast forms: E8M0 bytes of group 0): the loads of stages 1 and 2
    // may fly; six: everything has to land, stage 0's fragments aside the planes hold stages 1 .. 3 too
    static constexpr int prologue_wait() { return kForm == kF8Six ? 0 : 2 * kLoads; }
};

}  // namespace mx
