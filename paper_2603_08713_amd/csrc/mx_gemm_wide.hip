// Plain (no MBS) MXFP4 GEMM on 256 x 256 tiles: four wavefronts, one per SIMD, each owning a 128 x 128
// block whose 16 accumulator fragments (256 registers) live in the accumulation half of the register
// file.  Nothing but the matrix cores touches them, so this translation unit is compiled without the
// VGPR form of the matrix instructions.  The large register tile reads each LDS byte for four instructions.
#include "mx_gemm_ring.h"

namespace mx {

// Requires K % 512 == 0, K > 0 and 16-byte aligned scale arrays (the E8M0 bytes of four stages are fetched
// as one 16-byte piece); the caller has checked both.
//
// All tiles cost the same, so the launch runs in rounds of one tile per compute unit and a last round that
// fills only part of the chip costs as much as a full one.  The columns of C are therefore split in two
// launches where that saves time: 256 x 256 tiles for as many columns as make whole rounds, 256 x 128 tiles
// (half the cost each) for the rest.
int launch_gemm_wide(const GemmArgs& g, bool allow_split, hipStream_t s) {
    using Main = RingShape<2, 2, 4, 4, 0>;
    using Tail = RingShape<2, 2, 4, 2, 0>;
    constexpr int64_t kUnits = 256;  // compute units of the device
    const int64_t tiles_m = (g.M + Main::TM - 1) / Main::TM, cols = (g.N + Main::TN - 1) / Main::TN;
    auto rounds = [&](int64_t tiles) { return (tiles + kUnits - 1) / kUnits; };
    // cost in half-rounds of giving the first c tile columns to the large tile
    auto cost = [&](int64_t c) {
        const int64_t rest = g.N - c * Main::TN > 0 ? (g.N - c * Main::TN + Tail::TN - 1) / Tail::TN : 0;
        return 2 * rounds(c * tiles_m) + rounds(rest * tiles_m);
    };
    int64_t best = cols;
    for (int64_t c = cols; allow_split && c >= 0 && c >= cols - 64; --c)
        if (cost(c) < cost(best)) best = c;
    if (best == cols) return launch_ring<Main>(g, s);
    GemmArgs head = g, tail = g;
    head.N = best * Main::TN;
    tail.N = g.N - head.N;
    tail.b_codes += head.N * (g.K >> 1);
    tail.b_scales += head.N * (g.K >> 5);
    tail.C = static_cast<uint8_t*>(g.C) + head.N * (g.c_bf16 ? 2 : 4);
    if (head.N > 0)
        if (int st = launch_ring<Main>(head, s)) return st;
    return launch_ring<Tail>(tail, s);
}

}  // namespace mx
