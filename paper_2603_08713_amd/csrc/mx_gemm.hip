// Block-scaled MXFP4 GEMM  C = A * B^T  with the Macro Block Scaling correction, for gfx950.
//
// The contraction runs on v_mfma_scale_f32_16x16x128_f8f6f4 in FP4 mode.  One instruction is
// exactly one macro block deep (128 K-elements = 4 E8M0 blocks), which is the granularity at
// which the MBS correction has to be applied (App. E): with MBS every instruction starts from a
// zero accumulator and its 16x16 partial product is folded into the running fp32 result as
//     acc[i,j] += P_g[i,j] * sigma_A[i,g] * sigma_B[j,g],      sigma = 1/(1 + m8/256)   (Sec. 4.3.2)
// on the vector ALUs; without MBS the instructions chain their accumulators.
//
// Operand mapping of the instruction (64 lanes, lane = 16 q + r):
//   srcA: 16 rows x 128 k;  lane holds row r, k-block q: 32 FP4 = 16 bytes (4 of the 8 operand VGPRs)
//   srcB: 16 cols x 128 k;  lane holds col r, k-block q
//   scale operands: one E8M0 byte per lane (for its row/col and k-block), picked out of a VGPR
//                   by a per-instruction byte selector
//   D:    lane holds D[4 q + i][r], i = 0..3
// The weight matrix B feeds srcA and the activation matrix A feeds srcB, so that a lane ends up
// with four consecutive n of one output row m and stores them as one vector.
//
// Tiling: a workgroup of 4 wavefronts computes a 128 x 128 tile of C, each wavefront a 64 x 64
// quadrant (4 x 4 instructions per macro block).  K advances in stages of 256 elements (two macro
// blocks, one 128-byte line per row and operand), double-buffered in LDS: while stage s is being
// multiplied, stage s+1 is in flight from global memory into registers.  In LDS every 16-row x
// 128-k fragment is stored in lane order, so fragment reads are conflict-free 16-byte reads, and
// the E8M0 bytes are regrouped so that one dword holds the scales of the four fragments a
// wavefront combines with a given k-block (the byte selector then picks the fragment).
#include "mx_common.h"

namespace mx {
namespace {

constexpr int kTile = 128;            // rows of A and rows of B per workgroup tile
constexpr int kStageK = 256;          // K elements per pipeline stage
constexpr int kStageMacros = kStageK / kMacro;
constexpr int kThreads = 256;
constexpr int kFragBytes = 1024;      // 16 rows x 128 FP4
constexpr int kGroupM = 8;            // tile-rows walked together for L2 reuse

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

struct GemmArgs {
    const uint8_t *a_codes, *a_scales, *a_mbs;
    const uint8_t *b_codes, *b_scales, *b_mbs;
    void* C;
    const int64_t* row_offsets;  // grouped mode only
    int64_t M, N, K, ldc;
    int num_groups;              // 0 = plain GEMM
    int tiles_m, tiles_n;        // tile grid (tiles_m is an upper bound in grouped mode)
    int c_bf16;
    int vec_store;               // C rows allow 4-element vector stores
};

// LDS map (dynamic, 72 KiB): the two code stages first, so that the direct-to-LDS loads target the
// low 64 KiB, then the small per-stage arrays.
struct __attribute__((aligned(16))) StageCodes {
    uint8_t m[kTile / 16][kStageMacros][kFragBytes];  // A rows (activations): fragment-major, lane order
    uint8_t n[kTile / 16][kStageMacros][kFragBytes];  // B rows (weights)
};
struct __attribute__((aligned(16))) StageSmall {
    uint32_t scale_m[kStageMacros][2][kWave];  // [macro][wave half][lane]: bytes = the 4 fragments of that half
    uint32_t scale_n[kStageMacros][2][kWave];
    float sigma_m[kStageMacros][kTile];
    float sigma_n[kStageMacros][kTile];
};
constexpr int kLdsBytes = 2 * (int)sizeof(StageCodes) + 2 * (int)sizeof(StageSmall);

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// One operand (A or B) of the tile as the loader sees it: buffer resources rebased to the tile's first
// row and sized to its valid rows, so that rows past the end read as zero without any branch.
struct Operand {
    __amdgpu_buffer_rsrc_t codes, scales, mbs;
    int row_bytes;    // K / 2
    int scale_bytes;  // K / 32
    int nmac;         // ceil(K / 128)
    bool has_mbs;
};

__device__ __forceinline__ Operand make_operand(const uint8_t* codes, const uint8_t* scales, const uint8_t* mbs,
                                                int64_t row0, int64_t row_end, int64_t K) {
    Operand op;
    const int64_t rows = row_end > row0 ? (row_end - row0 < kTile ? row_end - row0 : kTile) : 0;
    op.row_bytes = (int)(K >> 1);
    op.scale_bytes = (int)(K >> 5);
    op.nmac = (int)((K + kMacro - 1) / kMacro);
    op.has_mbs = mbs != nullptr;
    const int kRsrcFlags = 0x00020000;  // raw buffer, 32-bit data format
    op.codes = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(codes) + row0 * op.row_bytes, 0,
                                                 (int)(rows * op.row_bytes), kRsrcFlags);
    op.scales = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(scales) + row0 * op.scale_bytes, 0,
                                                  (int)(rows * op.scale_bytes), kRsrcFlags);
    op.mbs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(mbs ? mbs + row0 * op.nmac : codes), 0,
                                               mbs ? (int)(rows * op.nmac) : 0, kRsrcFlags);
    return op;
}

constexpr int kOob = 0x7FFFFFF0;  // byte offset beyond any buffer: the load returns zero

// Codes of one stage straight into LDS.  Each wavefront issues four 1-KiB loads per operand; load i
// of wavefront w fills fragment (16-row block, macro block) = (pair >> 1, pair & 1), pair = 4 i + w,
// lane l fetching row l % 16, 32-element block l / 16 -- which is exactly the lane order the
// instruction wants, so the LDS image needs no further shuffling.
template <bool kRaggedK>
__device__ __forceinline__ void load_codes(const Operand& op, uint8_t (*dst)[kStageMacros][kFragBytes], int64_t K,
                                           int k0, int tid) {
    const int w = tid >> 6, l = tid & 63;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int pair = i * 4 + w;
        const int rb = pair >> 1, mb = pair & 1;
        const int k = mb * kMacro + (l >> 4) * kBlock;  // within the stage
        int voff = (rb * 16 + (l & 15)) * op.row_bytes + (k >> 1);
        if (kRaggedK && k0 + k >= K) voff = kOob;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(op.codes, (lds_ptr_t)(&dst[rb][mb][0]), 16, voff, k0 >> 1, 0, 0);
    }
}

struct Small {
    uint32_t scale;  // the four E8M0 bytes of one (row, macro block)
    uint32_t m8;
};

// One (row, macro block) per thread: its four E8M0 bytes and its MBS word.
template <bool kMbs, bool kScaleDword>
__device__ __forceinline__ Small load_small(const Operand& op, int64_t K, int k0, int tid) {
    const int row = tid & 127;
    const int g = k0 / kMacro + (tid >> 7);
    Small r;
    const int off = row * op.scale_bytes + g * 4;
    if (kScaleDword) {
        r.scale = __builtin_amdgcn_raw_buffer_load_b32(op.scales, g * kMacro < K ? off : kOob, 0, 0);
    } else {
        // rows are not dword aligned or the last macro block is short: byte loads, absent blocks read 0
        r.scale = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int o = g * kMacro + j * kBlock < K ? off + j : kOob;
            r.scale |= (uint32_t)__builtin_amdgcn_raw_buffer_load_b8(op.scales, o, 0, 0) << (8 * j);
        }
    }
    r.m8 = 0;
    if (kMbs) r.m8 = __builtin_amdgcn_raw_buffer_load_b8(op.mbs, g * kMacro < K ? row * op.nmac + g : kOob, 0, 0);
    return r;
}

template <bool kMbs>
__device__ __forceinline__ void store_small(const Small& v, uint32_t (*scale)[2][kWave], float (*sigma)[kTile],
                                            int tid) {
    const int row = tid & 127, mb = tid >> 7;
    const int half = row >> 6, frag = (row >> 4) & 3, r = row & 15;
    uint8_t* sb = reinterpret_cast<uint8_t*>(&scale[mb][half][0]);
#pragma unroll
    for (int q = 0; q < 4; ++q) sb[(q * 16 + r) * 4 + frag] = (uint8_t)(v.scale >> (8 * q));
    if (kMbs) sigma[mb][row] = 1.0f / (1.0f + (float)v.m8 * (1.0f / 256.0f));
}

template <int kSelN, int kSelM>
__device__ __forceinline__ v4f mfma_fp4(v4i n_frag, v4i m_frag, v4f c, uint32_t scale_n, uint32_t scale_m) {
    const v8i a = __builtin_shufflevector(n_frag, n_frag, 0, 1, 2, 3, -1, -1, -1, -1);
    const v8i b = __builtin_shufflevector(m_frag, m_frag, 0, 1, 2, 3, -1, -1, -1, -1);
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 4 /*A: FP4*/, 4 /*B: FP4*/, kSelN,
                                                            (int)scale_n, kSelM, (int)scale_m);
}

template <bool kMbs, int kMi, int kNi>
__device__ __forceinline__ void tile_step(v4f (&acc)[4][4], const v4i (&m_frag)[4], const v4i (&n_frag)[4],
                                          uint32_t sn, uint32_t sm, const float (&sig_m)[4],
                                          const v4f (&sig_n)[4]) {
    if constexpr (kMbs) {
        const v4f zero = {0.f, 0.f, 0.f, 0.f};
        const v4f p = mfma_fp4<kNi, kMi>(n_frag[kNi], m_frag[kMi], zero, sn, sm);
        const float sa = sig_m[kMi];
        acc[kMi][kNi].x = fmaf(p.x, sa * sig_n[kNi].x, acc[kMi][kNi].x);
        acc[kMi][kNi].y = fmaf(p.y, sa * sig_n[kNi].y, acc[kMi][kNi].y);
        acc[kMi][kNi].z = fmaf(p.z, sa * sig_n[kNi].z, acc[kMi][kNi].z);
        acc[kMi][kNi].w = fmaf(p.w, sa * sig_n[kNi].w, acc[kMi][kNi].w);
    } else {
        acc[kMi][kNi] = mfma_fp4<kNi, kMi>(n_frag[kNi], m_frag[kMi], acc[kMi][kNi], sn, sm);
    }
}

template <bool kMbs, int kMi>
__device__ __forceinline__ void tile_row(v4f (&acc)[4][4], const v4i (&m_frag)[4], const v4i (&n_frag)[4],
                                         uint32_t sn, uint32_t sm, const float (&sig_m)[4],
                                         const v4f (&sig_n)[4]) {
    tile_step<kMbs, kMi, 0>(acc, m_frag, n_frag, sn, sm, sig_m, sig_n);
    tile_step<kMbs, kMi, 1>(acc, m_frag, n_frag, sn, sm, sig_m, sig_n);
    tile_step<kMbs, kMi, 2>(acc, m_frag, n_frag, sn, sm, sig_m, sig_n);
    tile_step<kMbs, kMi, 3>(acc, m_frag, n_frag, sn, sm, sig_m, sig_n);
}

// kMbs: apply the per-macro-block correction; kScaleDword: the four E8M0 bytes of a macro block are an
// aligned dword (K % 128 == 0, 4-byte aligned scale arrays); kRaggedK: K is not a multiple of the stage.
template <bool kMbs, bool kScaleDword, bool kRaggedK>
__global__ __launch_bounds__(kThreads, 2) void gemm_kernel(GemmArgs g) {
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    StageCodes* codes = reinterpret_cast<StageCodes*>(smem);
    StageSmall* small = reinterpret_cast<StageSmall*>(smem + 2 * sizeof(StageCodes));

    // ---- which tile --------------------------------------------------------------------------
    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tiles and
    // walk tiles in bands of kGroupM tile-rows so that concurrently running workgroups share
    // operand panels in their XCD's L2.
    const int total = g.tiles_m * g.tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int linear = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || linear >= total) return;
    const int band = kGroupM * g.tiles_n;
    const int first_m = (linear / band) * kGroupM;
    const int band_rows = min(g.tiles_m - first_m, kGroupM);
    int tm = first_m + (linear % band) % band_rows;
    const int tn = (linear % band) / band_rows;

    int64_t a_row0 = (int64_t)tm * kTile, a_end = g.M;
    int64_t b_row0 = (int64_t)tn * kTile, b_end = g.N;
    if (g.num_groups > 0) {
        // tm counts tiles over all groups; find the group that owns it
        int e = 0;
        int64_t lo = 0, hi = 0;
        bool found = false;
        for (; e < g.num_groups; ++e) {
            lo = g.row_offsets[e];
            hi = g.row_offsets[e + 1];
            const int nt = (int)((hi - lo + kTile - 1) / kTile);
            if (tm < nt) { found = true; break; }
            tm -= nt;
        }
        if (!found) return;
        a_row0 = lo + (int64_t)tm * kTile;
        a_end = hi;
        b_row0 += (int64_t)e * g.N;
        b_end = (int64_t)e * g.N + g.N;
    }
    const Operand opa = make_operand(g.a_codes, g.a_scales, g.a_mbs, a_row0, a_end, g.K);
    const Operand opb = make_operand(g.b_codes, g.b_scales, g.b_mbs, b_row0, b_end, g.K);

    const int tid = threadIdx.x, l = tid & 63, w = tid >> 6;
    const int wm = w & 1, wn = w >> 1;  // quadrant of the tile owned by this wavefront

    v4f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};

    const int nstages = (int)((g.K + kStageK - 1) / kStageK);
    if (nstages > 0) {
        load_codes<kRaggedK>(opa, codes[0].m, g.K, 0, tid);
        load_codes<kRaggedK>(opb, codes[0].n, g.K, 0, tid);
        const Small sa = load_small<kMbs, kScaleDword>(opa, g.K, 0, tid);
        const Small sb = load_small<kMbs, kScaleDword>(opb, g.K, 0, tid);
        store_small<kMbs>(sa, small[0].scale_m, small[0].sigma_m, tid);
        store_small<kMbs>(sb, small[0].scale_n, small[0].sigma_n, tid);
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the direct-to-LDS loads have landed
        __syncthreads();
    }

    for (int s = 0; s < nstages; ++s) {
        const StageCodes& cc = codes[s & 1];
        const StageSmall& cs = small[s & 1];
        // Next stage into the other buffer (last read before the barrier that ended the previous
        // iteration).  Unconditional, so that the loop body stays one basic block: past the end of K
        // the loads are out of range and return zeros that nobody reads.
        const int k1 = (s + 1) * kStageK;
        load_codes<kRaggedK>(opa, codes[(s + 1) & 1].m, g.K, k1, tid);
        load_codes<kRaggedK>(opb, codes[(s + 1) & 1].n, g.K, k1, tid);
        const Small sa = load_small<kMbs, kScaleDword>(opa, g.K, k1, tid);
        const Small sb = load_small<kMbs, kScaleDword>(opb, g.K, k1, tid);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mb = 0; mb < kStageMacros; ++mb) {
            v4i m_frag[4], n_frag[4];
            float sig_m[4] = {1.f, 1.f, 1.f, 1.f};
            v4f sig_n[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                m_frag[i] = *reinterpret_cast<const v4i*>(&cc.m[wm * 4 + i][mb][l * 16]);
                n_frag[i] = *reinterpret_cast<const v4i*>(&cc.n[wn * 4 + i][mb][l * 16]);
                if constexpr (kMbs) {
                    sig_m[i] = cs.sigma_m[mb][wm * 64 + i * 16 + (l & 15)];
                    sig_n[i] = *reinterpret_cast<const v4f*>(&cs.sigma_n[mb][wn * 64 + i * 16 + (l >> 4) * 4]);
                } else {
                    sig_n[i] = v4f{1.f, 1.f, 1.f, 1.f};
                }
            }
            const uint32_t sm = cs.scale_m[mb][wm][l];
            const uint32_t sn = cs.scale_n[mb][wn][l];
            tile_row<kMbs, 0>(acc, m_frag, n_frag, sn, sm, sig_m, sig_n);
            tile_row<kMbs, 1>(acc, m_frag, n_frag, sn, sm, sig_m, sig_n);
            tile_row<kMbs, 2>(acc, m_frag, n_frag, sn, sm, sig_m, sig_n);
            tile_row<kMbs, 3>(acc, m_frag, n_frag, sn, sm, sig_m, sig_n);
        }
        // keep the multiply phase ahead of the wait for the next stage's loads
        __builtin_amdgcn_sched_barrier(0);
        StageSmall& ns = small[(s + 1) & 1];
        store_small<kMbs>(sa, ns.scale_m, ns.sigma_m, tid);
        store_small<kMbs>(sb, ns.scale_n, ns.sigma_n, tid);
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the direct-to-LDS loads have landed
        __syncthreads();
    }

    // ---- epilogue: lane holds C[m][n .. n+3] for each of its 4 x 4 fragments -------------------------
    const int64_t n_base = (int64_t)tn * kTile + wn * 64 + (l >> 4) * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t m = a_row0 + wm * 64 + i * 16 + (l & 15);
        if (m >= a_end) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t n = n_base + j * 16;
            if (n >= g.N) continue;
            const v4f v = acc[i][j];
            if (g.c_bf16) {
                uint16_t* o = static_cast<uint16_t*>(g.C) + m * g.ldc + n;
                const uint32_t b0 = f32_to_bf16_bits(v.x), b1 = f32_to_bf16_bits(v.y);
                const uint32_t b2 = f32_to_bf16_bits(v.z), b3 = f32_to_bf16_bits(v.w);
                if (g.vec_store && n + 3 < g.N) {
                    *reinterpret_cast<uint2*>(o) = make_uint2(b0 | (b1 << 16), b2 | (b3 << 16));
                } else {
                    o[0] = (uint16_t)b0;
                    if (n + 1 < g.N) o[1] = (uint16_t)b1;
                    if (n + 2 < g.N) o[2] = (uint16_t)b2;
                    if (n + 3 < g.N) o[3] = (uint16_t)b3;
                }
            } else {
                float* o = static_cast<float*>(g.C) + m * g.ldc + n;
                if (g.vec_store && n + 3 < g.N) {
                    *reinterpret_cast<v4f*>(o) = v;
                } else {
                    o[0] = v.x;
                    if (n + 1 < g.N) o[1] = v.y;
                    if (n + 2 < g.N) o[2] = v.z;
                    if (n + 3 < g.N) o[3] = v.w;
                }
            }
        }
    }
}

template <bool kMbs, bool kScaleDword, bool kRaggedK>
int launch_variant(const GemmArgs& g, unsigned blocks, hipStream_t s) {
    static bool attr_set = false;  // dynamic LDS above 64 KiB needs an opt-in once per process
    auto* fn = gemm_kernel<kMbs, kScaleDword, kRaggedK>;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                                kLdsBytes) != hipSuccess) {
            (void)hipGetLastError();
            return MX_ELAUNCH;
        }
        attr_set = true;
    }
    hipLaunchKernelGGL(fn, dim3(blocks), dim3(kThreads), kLdsBytes, s, g);
    return launch_status();
}

int launch_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs, const uint8_t* b_codes,
                const uint8_t* b_scales, const uint8_t* b_mbs, int num_groups, const int64_t* row_offsets,
                bool grouped, int64_t M, int64_t N, int64_t K, int c_dtype, void* C, int64_t ldc, bool mbs_entry,
                void* stream) {
    if (M < 0 || N < 0 || K < 0 || (K % kBlock) != 0 || ldc < N) return MX_EINVAL;
    if (c_dtype != MX_OUT_F32 && c_dtype != MX_OUT_BF16) return MX_EINVAL;
    if (grouped && num_groups < 0) return MX_EINVAL;
    if (K > (int64_t)1 << 24 || M > (int64_t)1 << 30 || N > (int64_t)1 << 30 || (grouped && (int64_t)num_groups * N > (int64_t)1 << 40))
        return MX_EINVAL;
    if (M == 0 || N == 0 || (grouped && num_groups == 0)) return MX_OK;
    if (!C || (grouped && !row_offsets)) return MX_ENULL;
    if (K > 0 && (!a_codes || !a_scales || !b_codes || !b_scales)) return MX_ENULL;
    const size_t esz = c_dtype == MX_OUT_F32 ? 4 : 2;
    if (!aligned(C, esz) || (K > 0 && (!aligned(a_codes, 16) || !aligned(b_codes, 16)))) return MX_EALIGN;
    if (int st = check_device()) return st;

    GemmArgs g;
    g.a_codes = a_codes; g.a_scales = a_scales; g.a_mbs = a_mbs;
    g.b_codes = b_codes; g.b_scales = b_scales; g.b_mbs = b_mbs;
    g.C = C; g.row_offsets = row_offsets;
    g.M = M; g.N = N; g.K = K; g.ldc = ldc;
    g.num_groups = grouped ? num_groups : 0;
    const int64_t tiles_m = (M + kTile - 1) / kTile + (grouped ? num_groups : 0);
    const int64_t tiles_n = (N + kTile - 1) / kTile;
    if (tiles_m * tiles_n > (int64_t)1 << 30) return MX_EINVAL;
    g.tiles_m = (int)tiles_m;
    g.tiles_n = (int)tiles_n;
    g.c_bf16 = c_dtype == MX_OUT_BF16;
    g.vec_store = aligned(C, 4 * esz) && (ldc % 4) == 0;

    const int total = g.tiles_m * g.tiles_n;
    const unsigned blocks = (unsigned)(((total + 7) / 8) * 8);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool use_mbs = mbs_entry && (a_mbs || b_mbs);
    const bool dword = (K % kMacro) == 0 && aligned(a_scales, 4) && aligned(b_scales, 4);
    const bool ragged = (K % kStageK) != 0;
    if (use_mbs) {
        if (dword) return ragged ? launch_variant<true, true, true>(g, blocks, s) : launch_variant<true, true, false>(g, blocks, s);
        return launch_variant<true, false, true>(g, blocks, s);
    }
    if (dword) return ragged ? launch_variant<false, true, true>(g, blocks, s) : launch_variant<false, true, false>(g, blocks, s);
    return launch_variant<false, false, true>(g, blocks, s);
}

}  // namespace
}  // namespace mx

extern "C" {

int mx_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes, const uint8_t* b_scales,
            int64_t M, int64_t N, int64_t K, mx_dtype_t c_dtype, void* C, int64_t ldc, void* stream) {
    return mx::launch_gemm(a_codes, a_scales, nullptr, b_codes, b_scales, nullptr, 0, nullptr, false, M, N, K,
                           (int)c_dtype, C, ldc, false, stream);
}

int mx_gemm_mbs(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs_or_null,
                const uint8_t* b_codes, const uint8_t* b_scales, const uint8_t* b_mbs_or_null, int64_t M, int64_t N,
                int64_t K, mx_dtype_t c_dtype, void* C, int64_t ldc, void* stream) {
    return mx::launch_gemm(a_codes, a_scales, a_mbs_or_null, b_codes, b_scales, b_mbs_or_null, 0, nullptr, false, M,
                           N, K, (int)c_dtype, C, ldc, true, stream);
}

int mx_gemm_mbs_grouped(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* a_mbs_or_null,
                        const uint8_t* b_codes, const uint8_t* b_scales, const uint8_t* b_mbs_or_null,
                        int32_t num_groups, const int64_t* row_offsets, int64_t M_total, int64_t N, int64_t K,
                        mx_dtype_t c_dtype, void* C, int64_t ldc, void* stream) {
    return mx::launch_gemm(a_codes, a_scales, a_mbs_or_null, b_codes, b_scales, b_mbs_or_null, num_groups,
                           row_offsets, true, M_total, N, K, (int)c_dtype, C, ldc, true, stream);
}

}  // extern "C"
