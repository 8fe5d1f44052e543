// Plain (no MBS) MXFP4 GEMM, on 256 x 256 tiles where the problem has enough of them: four wavefronts, one per SIMD, each owning a 128 x 128
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
//
// Problems with too few large tiles for the device take 256 x 128 or 128 x 128 tiles throughout (four
// wavefronts of 128 x 64 or 64 x 64).
//
// tile: 0 = choose, 1 = 256 x 256 only, 2 = 256 x 128 only, 3 = 128 x 128 only (development switch).
namespace {

using Main = RingShape<2, 2, 4, 4, 0>;
using Tail = RingShape<2, 2, 4, 2, 0>;
using Small = RingShape<2, 2, 2, 2, 0>;
constexpr int64_t kUnits = 256;  // compute units of the device

// What launch_gemm_wide does with an M x N problem: the tile (1, 2, 3 as above) and, for the large tile, how many
// of its tile columns go to the large tile (the rest to 256 x 128 tiles in a second launch).
struct WidePlan {
    int tile;
    int64_t big_cols, cols;
};

WidePlan plan_wide(int64_t M, int64_t N, int tile) {
    if (tile == 0) {
        // Tiles run in rounds of one per compute unit.  Cost of a launch in units of a 128 x 128 tile's time:
        // rounds x tile area / efficiency, the smaller tiles reaching about 0.85 and 0.78 of the large tile's
        // rate per output (measured; 0.72 is used for the smallest so that an underfilled round of large tiles keeps its edge); the large tile wins ties, and only it is split over two launches.
        auto rounds = [&](int64_t tm, int64_t tn) {
            return (((M + tm - 1) / tm) * ((N + tn - 1) / tn) + kUnits - 1) / kUnits;
        };
        const double c256 = 4.0 * rounds(256, 256), c256x128 = 2.0 * rounds(256, 128) / 0.85,
                     c128 = 1.0 * rounds(128, 128) / 0.72;
        if (c256x128 < c256 && c256x128 <= c128) return {2, 0, 0};
        if (c128 < c256) return {3, 0, 0};
    }
    if (tile == 2 || tile == 3) return {tile, 0, 0};
    const bool allow_split = tile == 0;
    const int64_t tiles_m = (M + Main::TM - 1) / Main::TM, cols = (N + Main::TN - 1) / Main::TN;
    auto rounds = [&](int64_t tiles) { return (tiles + kUnits - 1) / kUnits; };
    // cost in half-rounds of giving the first c tile columns to the large tile
    auto cost = [&](int64_t c) {
        const int64_t rest = N - c * Main::TN > 0 ? (N - c * Main::TN + Tail::TN - 1) / Tail::TN : 0;
        return 2 * rounds(c * tiles_m) + rounds(rest * tiles_m);
    };
    int64_t best = cols;
    for (int64_t c = cols; allow_split && c >= 0 && c >= cols - 64; --c)
        if (cost(c) < cost(best)) best = c;
    return {1, best, cols};
}

}  // namespace

const char* describe_gemm_wide(int64_t M, int64_t N) {
    const WidePlan p = plan_wide(M, N, 0);
    if (p.tile == 2) return "gemm_ring_kernel, fast form, 256x128 tile, 4 wavefronts of 128x64";
    if (p.tile == 3) return "gemm_ring_kernel, fast form, 128x128 tile, 4 wavefronts of 64x64";
    if (p.big_cols == p.cols) return "gemm_ring_kernel, fast form, 256x256 tile, 4 wavefronts of 128x128";
    if (p.big_cols == 0) return "gemm_ring_kernel, fast form, 256x128 tile, 4 wavefronts of 128x64 (all columns)";
    return "gemm_ring_kernel, fast form, 256x256 tile, 4 wavefronts of 128x128, and a second launch on 256x128 tiles for the last columns";
}

int launch_gemm_wide(const GemmArgs& g, int tile, hipStream_t s) {
    const WidePlan p = plan_wide(g.M, g.N, tile);
    if (p.tile == 2) return launch_ring<Tail>(g, s);
    if (p.tile == 3) return launch_ring<Small>(g, s);
    if (p.big_cols == p.cols) return launch_ring<Main>(g, s);
    GemmArgs head = g, tail = g;
    head.N = p.big_cols * Main::TN;
    tail.N = g.N - head.N;
    tail.b_codes += head.N * (g.K >> 1);
    tail.b_scales += head.N * (g.K >> 5);
    tail.C = static_cast<uint8_t*>(g.C) + head.N * (g.c_bf16 ? 2 : 4);
    if (head.N > 0)
        if (int st = launch_ring<Main>(head, s)) return st;
    return launch_ring<Tail>(tail, s);
}

// The general forms (mx_gemm_ring.h: any K, any alignment of the scale arrays, grouped or not) without MBS.
// tile: 0 = 256 x 128, 1 = 128 x 128.  bytes: E8M0 bytes one at a time (128 x 128 tiles only).
int launch_gemm_wide_general(const GemmArgs& g, int tile, bool bytes, hipStream_t s) {
    if (bytes) return launch_ring<RingShape<2, 2, 2, 2, 0, 2>>(g, s);
    if (tile == 0) return launch_ring<RingShape<2, 2, 4, 2, 0, 1>>(g, s);
    return launch_ring<RingShape<2, 2, 2, 2, 0, 1>>(g, s);
}

}  // namespace mx
