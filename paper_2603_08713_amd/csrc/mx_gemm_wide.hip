// Plain (no MBS) MXFP4 GEMM on 256 x 256 tiles: four wavefronts, one per SIMD, each owning a 128 x 128
// block whose 16 accumulator fragments (256 registers) live in the accumulation half of the register
// file.  Nothing but the matrix cores touches them, so this translation unit is compiled without the
// VGPR form of the matrix instructions.  The large register tile reads each LDS byte for four instructions.
#include "mx_gemm_ring.h"

namespace mx {

// Requires K % 512 == 0, K > 0 and 16-byte aligned scale arrays (the E8M0 bytes of four stages are fetched
// as one 16-byte piece); the caller has checked both.
int launch_gemm_wide(const GemmArgs& g, hipStream_t s) { return launch_ring<RingShape<2, 2, 4, 4, false>>(g, s); }

}  // namespace mx
