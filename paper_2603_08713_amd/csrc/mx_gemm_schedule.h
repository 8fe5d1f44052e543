// Tile shapes and load schedule of the main GEMM kernel template (mx_gemm_ring.h): what a shape keeps in LDS, which
// direct-to-LDS loads a stage issues, in which order, and how many of a wavefront's loads may still be in flight
// when a stage starts.  Plain constexpr C++ with no device code, so that a host program can replay the schedule of
// every instantiated shape and check it (tests/schedule_check.cpp).
//
// K advances one macro block (a "stage": 64 code bytes per row) at a time through a ring of four LDS code slots;
// E8M0 bytes and MBS words travel per group of four stages through two slots each.  A memory line holds the code
// bytes of TWO consecutive stages of a row, and the vector cache is far too small to keep a line from one stage to
// the next, so the loads of stages 2 t and 2 t + 1 are issued together, line by line: the two halves of a line are
// then requested back to back (measured 6 % faster on the kernel without MBS than one stage per stage).  Stages
// of phase 1 and 3 (phase = stage mod 4) issue the code
// loads of stages s + 3 and s + 4, whose slots the stages s - 1 and s have left; phase 1 issues the E8M0 bytes of
// the next group in front of them, phase 3 the MBS words of the group after next.  Phases 0 and 2 issue nothing.
//
// A wavefront's loads complete in the order it issued them.  The workgroup synchronises every other stage only,
// at the start of the stages that issue loads (phases 1 and 3): there a wavefront waits for all of its loads
// (what it issued two stages earlier, the codes of stages s + 1 and s + 2 among them, is everything outstanding)
// and passes the barrier, which publishes them and, because every wavefront has finished stage s - 1, frees the
// slots of stages s - 1 and s for this stage's loads.  The stage after (phase 0 or 2) reads what that barrier
// published and issues nothing, so it needs neither wait nor barrier, and the wavefronts of a workgroup may drift up
// to two stages apart (measured: 6 % faster with MBS than a barrier per stage, results bit-identical).
#pragma once

#include "mx_constants.h"

namespace mx {

constexpr int ceil_div(int a, int b) { return (a + b - 1) / b; }

// ---- tile shapes of the kernel template and what they hold in LDS -------------------------------------------
constexpr int kRingStageK = kMacro;             // K elements per stage
constexpr int kRingRowStage = kRingStageK / 2;  // code bytes per row and stage
constexpr int kRingSlots = 4;
constexpr int kRingGroup = 4;                   // stages per 16-byte piece of a row's E8M0 bytes
constexpr int kRingGroupM = 4;                  // tile-rows walked together for L2 reuse
constexpr int kSigmaSlots = 4;                  // as many as ring slots: a stage's table index is a compile-time constant

// kSides: which operands carry MBS words (0 none, 1 A only, 2 B only, 3 both).
// kForm: 0 = fast form, which wants K % 512 == 0 and 16-byte (E8M0) / 4-byte (MBS) aligned rows, so that a row's
// bytes of four stages travel as one piece per lane.  1, 2 = general forms for everything else, grouped problems
// included: E8M0 bytes travel as 2-byte pieces (1: any K % 64 == 0, rows of E8M0 bytes on even addresses; one
// piece per lane and pair of blocks) or as single bytes (2: any K % 32 == 0, any address), MBS words as single
// bytes, each piece in an LDS dword of its own; the last stage may be partly empty and the stage count is
// padded to whole groups with stages that read zeros.
template <int NWM_, int NWN_, int FM_, int FN_, int kSides_, int kForm_ = 0>
struct RingShape {
    static constexpr int NWM = NWM_, NWN = NWN_, FM = FM_, FN = FN_, kSides = kSides_;
    static constexpr bool kMbs = kSides != 0, kGen = kForm_ != 0, kBytes = kForm_ == 2;
    // (couples of A fragments against one B fragment at a time; instantiated with one and with two B fragments)
    static constexpr bool kSurface = kSides == 3 && FM_ % 2 == 0 && (FN_ == 1 || FN_ == 2);
    static constexpr int NW = NWM * NWN, NT = NW * kWave;
    static constexpr int TM = NWM * FM * 32, TN = NWN * FN * 32;
    static constexpr int kRows = TM + TN;             // rows of A followed by rows of B
    static constexpr int kCodeDma = kRows / 16 / NW;  // per wavefront and stage: 16 rows x 64 B per load
    // per wavefront and group of four stages: E8M0 bytes (fast: one row per lane; general: 8 rows x 8 pairs or
    // 4 rows x 16 bytes per load) and MBS words (fast: one row per lane; general: 16 rows x 4 words per load)
    static constexpr int kRowDma = ceil_div(kRows, kWave * NW);
    static constexpr int kScaleRowsPerLoad = kBytes ? 4 : 8;  // general forms
    static constexpr int kScaleDma = kGen ? kRows / kScaleRowsPerLoad / NW : kRowDma;
    static constexpr int kM8Dma = kGen ? kRows / 16 / NW : kRowDma;
    static constexpr int kRowsPadded = kRowDma * NW * kWave;
    static constexpr int kCodesStage = kRows * kRingRowStage;
    static constexpr int kScaleGroup = kBytes ? kRows * 64 : kGen ? kRows * 32 : kRowsPadded * 16;
    static constexpr int kM8Group = !kMbs ? 0 : kGen ? kRows * 16 : kRowsPadded * 4;
    static constexpr int kSigmaStage = kMbs ? kRows * 4 : 0;
    // The small arrays come first: their addresses then fit the 16-bit constant of an LDS instruction.
    static constexpr int kM8Base = 0;
    static constexpr int kSigmaBase = kM8Base + 2 * kM8Group;
    // the 256 values sigma can take, 1 / (1 + m8 / 256) in fp32 (kernels that look sigma up instead of computing it)
    static constexpr int kRcpBase = kSigmaBase + kSigmaSlots * kSigmaStage;
    static constexpr int kRcpBytes = kMbs ? 1024 : 0;
    static constexpr int kScaleBase = (kRcpBase + kRcpBytes + 16383) / 16384 * 16384;
    static constexpr int kDummy = kScaleBase + 2 * kScaleGroup;  // target of padding stores
    static constexpr int kCodesBase = kDummy + 256;
    static constexpr int kLdsBytes = kCodesBase + kRingSlots * kCodesStage;
    static_assert(kCodesBase % 64 == 0 && kCodesBase < 65536, "code rows stay 64-byte aligned; small arrays below 64 KiB");
    static constexpr int kStageRegion = 32 * (FN * 32 * 4 + 16);  // per wavefront, epilogue staging
    static_assert(NW == 4 || NW == 8, "one or two wavefronts per SIMD");
    static_assert((TM / 16) % NW == 0 && (TN / 16) % NW == 0, "16-row code loads: operand fixed per load index");
    static_assert(!kGen || (TM % 128 == 0 && TN % 128 == 0 && kRows % (16 * NW) == 0), "general forms: operand fixed per load index");
    static_assert(kLdsBytes <= 160 * 1024, "LDS capacity of a gfx950 compute unit");
    static_assert(NW * kStageRegion <= kLdsBytes, "epilogue staging fits the LDS of the main loop");
    static_assert(FM * FN * 16 <= 256, "accumulators fill at most the accumulation registers");
    static_assert(!kMbs || FN == 1 || FN % 2 == 0, "MBS path: sigma sets line up across stages");
};

// ---- load schedule ----------------------------------------------------------------------------------------------
enum LoadKind { kLoadCode = 0, kLoadScale = 1, kLoadWords = 2 };

// kind; what: the stage (codes) or the group (E8M0 bytes, MBS words), counted from the issuing stage s (codes:
// s + what) or its group s / 4 (others: s / 4 + what) in the loop, absolute in the prologue; index: which of the
// wavefront's loads of that kind for that stage or group.
struct LoadItem {
    int kind, what, index;
};

template <int kCodeDma, int kScaleDma, int kWordDma>
struct RingSchedule {
    static constexpr int kGroup = 4, kSlots = 4;

    // ---- the loop ----
    static constexpr int issue_count(int phase) {
        return phase == 1 ? kScaleDma + 2 * kCodeDma : phase == 3 ? kWordDma + 2 * kCodeDma : 0;
    }
    static constexpr LoadItem issue_item(int phase, int n) {
        const int small = phase == 1 ? kScaleDma : kWordDma;
        if (n < small) return phase == 1 ? LoadItem{kLoadScale, 1, n} : LoadItem{kLoadWords, 2, n};
        const int k = n - small;  // the two stages of a line alternate
        return LoadItem{kLoadCode, 3 + (k & 1), k >> 1};
    }
    // Stages of phase 1 and 3 open with a wait and the workgroup's barrier; the others with neither.
    static constexpr bool has_barrier(int phase) { return phase % 2 == 1; }
    // Loads that may be in flight when such a stage passes its wait: none.  The youngest outstanding loads are the
    // codes of stage s + 2, which the stage after this one reads before the next barrier.
    static constexpr int wait_count(int phase) { return has_barrier(phase) ? 0 : 63; }

    // ---- the prologue: what the loop would have issued before stage 0 ----
    // E8M0 bytes and MBS words of group 0, the codes of stages 0 and 1 line by line, then (as a stage of phase 3
    // would) the MBS words of group 1 and the codes of stages 2 and 3.
    static constexpr int prologue_count() { return kScaleDma + 2 * kWordDma + 4 * kCodeDma; }
    static constexpr LoadItem prologue_item(int n) {
        if (n < kScaleDma) return LoadItem{kLoadScale, 0, n};
        n -= kScaleDma;
        if (n < kWordDma) return LoadItem{kLoadWords, 0, n};
        n -= kWordDma;
        if (n < 2 * kCodeDma) return LoadItem{kLoadCode, n & 1, n >> 1};
        n -= 2 * kCodeDma;
        if (n < kWordDma) return LoadItem{kLoadWords, 1, n};
        n -= kWordDma;
        return LoadItem{kLoadCode, 2 + (n & 1), n >> 1};
    }
    // before the prologue's barrier, which stands in for the barrier of a stage of phase 3: everything that the
    // stages 0 (no barrier of its own) and the conversions read has landed - the E8M0 bytes and MBS words of
    // group 0, the codes of stages 0 and 1; the second batch may fly
    static constexpr int prologue_wait_first() { return kWordDma + 2 * kCodeDma; }
};

}  // namespace mx
