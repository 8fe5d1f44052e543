// MXFP4 GEMM with the MBS correction on 256 x 128 tiles: eight wavefronts, two per SIMD.  The vector ALUs
// consume every matrix-instruction result (acc += P * sigma_A * sigma_B), so this translation unit is
// compiled with the VGPR form of the matrix instructions.  With words on both operands a wavefront owns
// 64 x 64 outputs (two A fragments against two B fragments: four fragments to read from LDS per four products)
// and the products sigma_A * sigma_B come from the matrix cores as well (mx_gemm_ring.h; its four pairs run in an
// order that lets every fragment be read again from LDS two pairs before its next use); with words on one
// operand only it owns 128 x 32 (four A fragments against one B fragment), and the 16 per-lane sigma_B values
// of the B fragment, or the lane's sigma_A, are read from LDS once per stage and serve four products.
// Problems with too few 256 x 128 tiles for the device take 128 x 128 tiles (64 x 32 per wavefront).
// Measured at 8192 x 28672 x 8192 with words on both operands, same device, same run: 64 x 64 per wavefront
// 2.42 PFLOP/s, 128 x 32 per wavefront 2.35, the same tile on four wavefronts of 128 x 64 (one per SIMD, operands
// partly in accumulation registers) 2.29.
#include "mx_gemm_ring.h"

namespace mx {

// Requires K % 512 == 0, K > 0, 16-byte aligned scale arrays and 4-byte aligned MBS arrays (a row's words of
// four stages are fetched as one dword); the caller has checked all of them.  A null MBS array means sigma = 1
// for that operand: the one-sided variants fold a product in with one multiply-add per output instead of two
// operations.
int launch_gemm_mbs_ring(const GemmArgs& g, int variant, hipStream_t s) {
    if (variant == 1) {  // 128 x 128 tiles
        if (g.a_mbs && g.b_mbs) return launch_ring<RingShape<2, 4, 2, 1, 3>>(g, s);
        if (g.a_mbs) return launch_ring<RingShape<2, 4, 2, 1, 1>>(g, s);
        return launch_ring<RingShape<2, 4, 2, 1, 2>>(g, s);
    }
    if (g.a_mbs && g.b_mbs) return launch_ring<RingShape<4, 2, 2, 2, 3>>(g, s);
    if (g.a_mbs) return launch_ring<RingShape<2, 4, 4, 1, 1>>(g, s);
    return launch_ring<RingShape<2, 4, 4, 1, 2>>(g, s);
}

}  // namespace mx
