// The main GEMM kernel template in its general forms: any K, rows of E8M0 bytes and MBS words at any address,
// and grouped problems (mixture of experts).  E8M0 bytes travel as 2-byte pieces (K % 64 == 0, even addresses) or
// as single bytes, MBS words as single bytes, which costs texture-address time the fast form does not spend,
// so the fast form keeps every problem it can take.  This file holds the kernels with MBS (compiled with the
// VGPR form of the matrix instructions, as in mx_gemm_mbs.hip); those without are in mx_gemm_wide.hip.
#include "mx_gemm_ring.h"

namespace mx {

// K % 64 == 0, K > 0, E8M0 arrays 2-byte aligned (or `bytes`); the caller has checked these.  A null MBS array reads as
// words of zero (sigma = 1, which multiplies exactly), so one instantiation serves one-sided MBS as well.
// tile: 0 = 256 x 128, 1 = 128 x 128.  bytes: E8M0 bytes one at a time (any K % 32 == 0, any address; 128 x 128
// tiles only: one LDS dword per byte does not fit beside the larger tile).
int launch_gemm_mbs_general(const GemmArgs& g, int tile, bool bytes, hipStream_t s) {
    if (bytes) return launch_ring<RingShape<2, 4, 2, 1, 3, 2>>(g, s);
    if (tile == 0) return launch_ring<RingShape<4, 2, 2, 2, 3, 1>>(g, s);
    return launch_ring<RingShape<2, 4, 2, 1, 3, 1>>(g, s);
}

}  // namespace mx
