// Pieces shared by the MXFP4 GEMM kernels (private; the public ABI is include/mx4.h).
#pragma once

#include <atomic>
#include <type_traits>
#include <utility>

#include "mx_common.h"
#include "mx_gemm_schedule.h"

namespace mx {

// Dynamic LDS above 64 KiB needs an opt-in per kernel and device.  The opt-in is idempotent, so two threads
// that both find it missing may both make it; the flag only saves later launches the call.
struct LdsOptIn {
    std::atomic<uint64_t> done{0};  // bit d: made on device d
    int ensure(const void* fn, int bytes) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0) { (void)hipGetLastError(); return MX_ELAUNCH; }
        const uint64_t bit = dev < 64 ? (uint64_t)1 << dev : 0;  // (devices past the 64th opt in on every launch)
        if (done.load(std::memory_order_acquire) & bit) return MX_OK;
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) {
            (void)hipGetLastError();
            return MX_ELAUNCH;
        }
        done.fetch_or(bit, std::memory_order_release);
        return MX_OK;
    }
};

struct GemmArgs {
    const uint8_t *a_codes, *a_scales, *a_mbs;
    const uint8_t *b_codes, *b_scales, *b_mbs;
    void* C;
    const int64_t* row_offsets;  // grouped mode only
    int64_t M, N, K, ldc;
    int num_groups;              // 0 = plain GEMM
    int tiles_m, tiles_n;        // tile grid (tiles_m is an upper bound in grouped mode)
    int c_bf16;
    int vec_store16;             // C rows allow 16-byte vector stores
    int vec_store8;              // C rows allow 8-byte vector stores
    int vec_store4;              // C rows allow 4-byte stores (bf16 output: two elements at a time)
};

// Main kernels (mx_gemm_ring.h), fast form: K % 512 == 0 and aligned scale and MBS arrays, not grouped; without MBS
// (mx_gemm_wide.hip: 256 x 256, 256 x 128 or 128 x 128 tiles) and with MBS (mx_gemm_mbs.hip: 256 x 128 or 128 x 128).
int launch_gemm_wide(const GemmArgs& g, int tile, hipStream_t s);
const char* describe_gemm_wide(int64_t M, int64_t N);  // what launch_gemm_wide(tile = 0) does with an M x N problem
int launch_gemm_mbs_ring(const GemmArgs& g, int variant, hipStream_t s);
// The same kernels in their general forms (any K % 32 == 0, any alignment of the scale arrays, grouped or not),
// defined in mx_gemm_general.hip (with MBS) and mx_gemm_wide.hip (without).  tile: 0 = 256 x 128, 1 = 128 x 128;
// bytes: E8M0 bytes fetched one at a time (needed when K % 64 != 0 or a scale array sits on an odd address;
// 128 x 128 tiles only).
int launch_gemm_mbs_general(const GemmArgs& g, int tile, bool bytes, hipStream_t s);
int launch_gemm_wide_general(const GemmArgs& g, int tile, bool bytes, hipStream_t s);
// Few activation rows (M <= 64, K <= 8192, otherwise the same conditions), defined in mx_gemm_skinny.hip.
int launch_gemm_skinny(const GemmArgs& g, bool use_mbs, hipStream_t s);
int launch_gemm_skinny_fused(const GemmArgs& g, const void* x_bf16, int64_t ldx, int rule, bool a_mbs, hipStream_t s);
// The few-row kernel for operands in the 8-bit or 6-bit element formats (a_elem, b_elem: mx_elem_t), under the same
// conditions, defined in mx_gemm_skinny_f8.hip; an operand without MBS words has a null a_mbs / b_mbs.
int launch_gemm_skinny_elem(const GemmArgs& g, int a_elem, int b_elem, hipStream_t s);

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v32f __attribute__((ext_vector_type(32)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef __attribute__((address_space(3))) const uint16_t* lds_half_ptr_t;

template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}


// One operand (A or B) of the tile as the loader sees it: buffer resources rebased to the tile's first
// row and sized to its valid rows, so that rows past the end read as zero without any branch.
struct Operand {
    __amdgpu_buffer_rsrc_t codes, scales, mbs;
};

__device__ __forceinline__ Operand make_operand(const uint8_t* codes, const uint8_t* scales, const uint8_t* mbs,
                                                int64_t row0, int64_t row_end, int tile_rows, int64_t K) {
    Operand op;
    const int64_t rows = row_end > row0 ? (row_end - row0 < tile_rows ? row_end - row0 : tile_rows) : 0;
    const int64_t row_bytes = K >> 1, scale_bytes = K >> 5, nmac = (K + kMacro - 1) / kMacro;
    const int kRsrcFlags = 0x00020000;  // raw buffer, 32-bit data format
    op.codes = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(codes) + row0 * row_bytes, 0,
                                                 (int)(rows * row_bytes), kRsrcFlags);
    op.scales = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(scales) + row0 * scale_bytes, 0,
                                                  (int)(rows * scale_bytes), kRsrcFlags);
    op.mbs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(mbs ? mbs + row0 * nmac : codes), 0,
                                               mbs ? (int)(rows * nmac) : 0, kRsrcFlags);
    return op;
}

constexpr int kOob = 0x7FFFFFF0;  // byte offset beyond any buffer: the load returns zero

// ---- grouped problems: which rows a tile-row covers ------------------------------------------------------------
// Group e owns rows off[e] .. off[e + 1] - 1 of A and C, the e-th of the stacked weights, and
// ceil(rows / tile_rows) tile-rows; tile-rows are counted group by group.  Every wavefront works this out for
// itself with one group per lane (64 groups per pass): a walk from group to group would be one memory round trip
// per group in front of every tile, and only the kernel can know how many tile-rows there really are - the launch
// takes an upper bound, and tiles dealt out over that bound would leave the last XCDs without work.
__device__ __forceinline__ int wave_scan_add(int x, int lane) {  // inclusive prefix sum over the 64 lanes
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int t = __builtin_amdgcn_ds_bpermute(((lane - d) & 63) << 2, x);
        if (lane >= d) x += t;
    }
    return x;
}
__device__ __forceinline__ int64_t readlane64(int64_t v, int idx) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, idx);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), idx);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}
// tile-rows of all groups together (the same value in every lane)
__device__ __forceinline__ int grouped_tile_rows(const int64_t* off, int num_groups, int tile_rows, int lane) {
    int total = 0;
    for (int base = 0; base < num_groups; base += 64) {
        const int e = base + lane;
        int rows = 0;
        if (e < num_groups) rows = (int)((off[e + 1] - off[e] + tile_rows - 1) / tile_rows);
        total += __builtin_amdgcn_readlane(wave_scan_add(rows, lane), 63);
    }
    return total;
}
struct GroupOfTileRow {
    int group, first;  // the group and its first tile-row
    int64_t lo, hi;    // its rows
};
// the group tile-row tm belongs to (uniform over the wavefront); false if tm lies past the last group
__device__ __forceinline__ bool grouped_find(const int64_t* off, int num_groups, int tile_rows, int lane, int tm,
                                             GroupOfTileRow& out) {
    int before = 0;
    for (int base = 0; base < num_groups; base += 64) {
        const int e = base + lane;
        int64_t lo = 0, hi = 0;
        if (e < num_groups) {
            lo = off[e];
            hi = off[e + 1];
        }
        const int rows = (int)((hi - lo + tile_rows - 1) / tile_rows);
        const int incl = wave_scan_add(rows, lane);
        const uint64_t hit = __builtin_amdgcn_ballot_w64(before + incl > tm);
        if (hit != 0) {
            const int idx = __builtin_amdgcn_readfirstlane(__builtin_ctzll(hit));
            out.group = base + idx;
            out.first = before + __builtin_amdgcn_readlane(incl - rows, idx);
            out.lo = readlane64(lo, idx);
            out.hi = readlane64(hi, idx);
            return true;
        }
        before += __builtin_amdgcn_readlane(incl, 63);
    }
    return false;
}

__device__ __forceinline__ v4f mfma_fp4(v4i n_frag, v4i m_frag, v4f c, uint32_t scale_n, uint32_t scale_m) {
    const v8i a = __builtin_shufflevector(n_frag, n_frag, 0, 1, 2, 3, -1, -1, -1, -1);
    const v8i b = __builtin_shufflevector(m_frag, m_frag, 0, 1, 2, 3, -1, -1, -1, -1);
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 4 /*A: FP4*/, 4 /*B: FP4*/, 0, (int)scale_n,
                                                            0, (int)scale_m);
}

// 32x32x64 form: lane = 32 h + r holds row r, k-block h of the instruction's two blocks; the scale operand is
// byte `sel` of the lane's scale register; D[8 (j / 4) + 4 h + j % 4][r] in result register j.
template <int kSelN, int kSelM>
__device__ __forceinline__ v16f mfma_fp4_wide(v4i n_frag, v4i m_frag, v16f c, uint32_t scale_n, uint32_t scale_m) {
    const v8i a = __builtin_shufflevector(n_frag, n_frag, 0, 1, 2, 3, -1, -1, -1, -1);
    const v8i b = __builtin_shufflevector(m_frag, m_frag, 0, 1, 2, 3, -1, -1, -1, -1);
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 4 /*A: FP4*/, 4 /*B: FP4*/, kSelN, (int)scale_n,
                                                            kSelM, (int)scale_m);
}

// s_waitcnt vmcnt(n) lgkmcnt(0): at most n direct-to-LDS loads outstanding, own LDS traffic done.
constexpr int wait_imm(int n) { return (n & 0xF) | ((n >> 4) << 14) | 0x0070; }
// s_waitcnt lgkmcnt(0) alone: own LDS traffic done, vector-memory operations left in flight.
constexpr int kWaitLds = 0xC07F;

// Workgroup barrier as a bare instruction: the compiler's own barrier intrinsic forces a wait for ALL
// outstanding vector-memory operations, which would drain the younger stages still in flight.
__device__ __forceinline__ void bare_barrier() { asm volatile("s_barrier" ::: "memory"); }

}  // namespace
}  // namespace mx
