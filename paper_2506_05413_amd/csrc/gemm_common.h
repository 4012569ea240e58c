// Pieces shared by the compute-bound GEMM kernels (int8-MFMA kernel in gemm_prefill.hip, FP6-MFMA
// kernel in gemm_f6.hip): hand-placed waits, LDS-DMA loads, the transposing epilogue, launch helpers.
#pragma once

#include "sr_common.h"

#include <hip/hip_fp16.h>

namespace sr {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------------
// The DMA loads, their waits and the barrier are inline assembly on purpose: the compiler
// would order every LDS read behind ALL outstanding LDS-DMA loads (vmcnt(0)) and put a full
// fence on every barrier, which serialises the pipeline.  Hazards are handled by hand:
// wait_vmcnt<n>() lets the n youngest loads stay in flight (loads complete in order), and the
// "memory" clobbers keep the compiler from moving LDS accesses across these statements.
// ------------------------------------------------------------------------------------------
template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void barrier_nofence() { asm volatile("s_barrier" ::: "memory"); }

// 64 lanes x 16 bytes: global (base + per-lane 32-bit offset) -> LDS bytes [lds, lds + 1024)
__device__ __forceinline__ void dma16(const uint8_t *base, uint32_t lane_off, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(lane_off), "s"(base)
                 : "memory", "m0");
}

// ------------------------------------------------------------------------------------------
// Epilogue for 32 x 32 MFMA tiles: dequantise, then transpose the wave's WM x WN tile through LDS,
// 32 tokens at a time, so that global memory is written in whole rows of the tile (16 bytes per
// lane, WN * 2 contiguous bytes per token) instead of 8-byte pieces scattered over 32 rows per
// instruction.  In the accumulator layout a lane owns token (l & 31) and, per quad q, the four
// output channels 8q + 4 (l >> 5) .. + 3 of each tile.  `stage` is this wave's private LDS area of
// 32 * (WN * 2 + 16) bytes; the caller has made sure nobody else touches it.  sx[j] is the token
// scale / 256 of this lane's token in row block j, sw[i][q] the four channel scales of quad q of
// column block i (fetched by the caller; unused for the raw int32 output).
// The accumulators are either int32 holding 256 x the sum (int8 MFMA on codes x 16) or fp32
// holding the sum / 64 exactly (FP6 MFMA on codes / 8); sx carries the matching factor.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float acc_f32(int a) { return (float)a; }
__device__ __forceinline__ float acc_f32(float a) { return a; }
__device__ __forceinline__ int acc_i32(int a) { return a >> 8; }
__device__ __forceinline__ int acc_i32(float a) { return (int)(a * 64.f); }

// CG = MFMA column tiles staged at a time (FN by default; fewer where the staging area is small): the rows
// written to memory are then CG * 64 bytes long.
template <int FM, int FN, int CG = FN, typename V16>
__device__ __forceinline__ void store_wave_tile(const V16 (&acc)[FN][FM], uint8_t *stage, int lane, int m_base, int n_base,
                                                int M, int N, const float (&sx)[FM], const float4 (&sw)[FN][4],
                                                void *__restrict__ Yv, int64_t ldy, int out_i32)
{
    constexpr int WN = FN * 32;
    const int fr = lane & 31, fg = lane >> 5;
    if (out_i32) {                                          // raw accumulators: a debugging / test output, stored directly
#pragma unroll
        for (int j = 0; j < FM; ++j)
#pragma unroll
            for (int i = 0; i < FN; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int m = m_base + j * 32 + fr, n = n_base + i * 32 + q * 8 + fg * 4;
                    if (m < M && n < N)
                        *reinterpret_cast<int4 *>(static_cast<int32_t *>(Yv) + (int64_t)m * ldy + n) =
                            make_int4(acc_i32(acc[i][j][4 * q]), acc_i32(acc[i][j][4 * q + 1]), acc_i32(acc[i][j][4 * q + 2]),
                                      acc_i32(acc[i][j][4 * q + 3]));
                }
    } else {
        constexpr int GW = CG * 32;                          // channels per staged group
        constexpr int RS = GW * 2 + 16;
        constexpr int CPR = GW * 2 / 16;
        constexpr int RPI = 64 / CPR;
        const int c = lane % CPR, r0 = lane / CPR;
#pragma unroll
        for (int j = 0; j < FM; ++j) {
#pragma unroll
            for (int i0 = 0; i0 < FN; i0 += CG) {
#pragma unroll
                for (int i = i0; i < i0 + CG && i < FN; ++i)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int nl = (i - i0) * 32 + q * 8 + fg * 4;
                        union { __half h[4]; uint2 u; } o;
                        o.h[0] = __float2half_rn(acc_f32(acc[i][j][4 * q]) * sx[j] * sw[i][q].x);
                        o.h[1] = __float2half_rn(acc_f32(acc[i][j][4 * q + 1]) * sx[j] * sw[i][q].y);
                        o.h[2] = __float2half_rn(acc_f32(acc[i][j][4 * q + 2]) * sx[j] * sw[i][q].z);
                        o.h[3] = __float2half_rn(acc_f32(acc[i][j][4 * q + 3]) * sx[j] * sw[i][q].w);
                        *reinterpret_cast<uint2 *>(stage + fr * RS + nl * 2) = o.u;
                    }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
#pragma unroll
                for (int r = r0; r < 32; r += RPI) {
                    const int m = m_base + j * 32 + r, nloc = i0 * 32 + c * 8, n = n_base + nloc;
                    const u32x4 v = *reinterpret_cast<const u32x4 *>(stage + r * RS + c * 16);
                    // streamed once, never read back by this kernel: keep it from displacing operand panels in L2
                    if (lane < RPI * CPR && nloc < WN && m < M && n < N)
                        __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(static_cast<__half *>(Yv) + (int64_t)m * ldy + n));
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            }
        }
    }
}

// Split of the tile grid over the 8 XCDs (each with its own L2): XCD x = v & 7 gets the rectangle
// (x % xcd_m, x / xcd_m) of an xcd_m x (8 / xcd_m) split and walks it m fastest.  Measured (FETCH_SIZE,
// M = 2048, K = 4096, int8 kernel): two halves in m by four blocks in n reads 112 MB through the fabric at
// N = 14336 where one run of tiles per XCD read 223 MB (half of X then stays in an XCD's 4 MB L2); it was
// also the fastest split at K = 14336.  Otherwise: the split whose rectangles need the fewest operand rows.
// 0 = no remapping.
inline int choose_xcd_split(int tiles_m, int tiles_n, int BM, int BN)
{
    if (tiles_m % 2 == 0 && tiles_n % 4 == 0) return 2;
    int xcd_m = 0;
    int64_t best = 0;
    for (int sm = 1; sm <= 8; sm *= 2) {
        if (tiles_m % sm != 0 || tiles_n % (8 / sm) != 0) continue;
        const int64_t rows = (int64_t)(tiles_m / sm) * BM + (int64_t)(tiles_n / (8 / sm)) * BN;
        if (xcd_m == 0 || rows < best) { xcd_m = sm; best = rows; }
    }
    return xcd_m;
}

// virtual workgroup index -> tile origin under that split
__device__ __forceinline__ void tile_origin(int v, int tiles_m, int tiles_n, int xcd_m, int BM, int BN, int &m0, int &n0)
{
    int tm, tn;
    if (xcd_m > 0) {
        const int x = v & 7, l = v >> 3;
        const int rm = tiles_m / xcd_m, rn = tiles_n / (8 / xcd_m);      // rectangle size in tiles
        // walk: mw tiles in m fastest, then across the rectangle in n, then the next mw rows of tiles -- the ~32
        // tiles an XCD works on at a time then form a block of 8 x 4 tiles instead of a 32 x 1 column
        // (M = 16384, N = 4096, K = 4096 on the FP6 kernel: 148.6 -> 139.5 us)
        const int mw = (rm > 8 && rm % 8 == 0) ? 8 : rm;
        const int a = l % mw, b = (l / mw) % rn, c = l / (mw * rn);
        tm = (x % xcd_m) * rm + c * mw + a;
        tn = (x / xcd_m) * rn + b;
    } else {
        tm = v % tiles_m;
        tn = v / tiles_m;
    }
    m0 = tm * BM;
    n0 = tn * BN;
}

}  // namespace
}  // namespace sr
