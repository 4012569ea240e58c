// INT4 x INT4 GEMM, INT32 accumulation, dequantising epilogue -- compute-bound shapes (M > 16).
//
//   acc[m][n] = sum_k cX[m][k] * cW[n][k],   Y = fp16(acc * dx[m] * dw[n])
//
// (Paper: the quantised forward pass of the linear layer; dequantisation per Eq. (1).)
//
// gfx950 has no 4-bit matrix instruction, so the packed codes are widened to int8 in
// registers and fed to the int8 MFMA.  A nibble is sign-extended for free by leaving it in
// the HIGH half of its byte:
//     lo = (w << 4) & 0xF0F0F0F0      (codes 0,2,4,6 of the dword, each x16)
//     hi =  w       & 0xF0F0F0F0      (codes 1,3,5,7 of the dword, each x16)
// Both operands carry the factor 16, so the accumulator holds 256 * acc exactly
// (256 * 64 * K < 2^31 for K < 131072); the factor leaves by an arithmetic shift (int32
// output) or inside the row scale (fp16 output).  A dot product does not care in which
// order k is visited: X and W only have to permute k identically, and they do because both
// are widened by the same three instructions from the same byte offsets.
//
// What the main kernel is built around (all measured on MI355X):
//  * v_mfma_i32_32x32x32_i8 (8 passes, 32 cycles of the matrix pipe) lets vector-ALU instructions
//    of the same wave issue underneath it; v_mfma_i32_16x16x64_i8 (4 passes) does not.  The
//    widening (4.5 - 6 ALU instructions per MFMA) therefore costs little MFMA time.
//  * Memory instructions hold up the wave that issues them (an LDS-DMA load ~50 cycles, a
//    ds_read_b128 ~25), and with one wave per SIMD a held-up wave idles the matrix pipe: timed
//    per stage, DMA and fragment reads ADD to the MFMA time instead of hiding under it.  Hence
//    (a) two waves per SIMD -- eight waves on a 256 x 128 tile, or two four-wave workgroups of
//    128 x 128 per CU -- and (b) no bursts: a 64-code sub-step is cut into regions of
//    [2 fragment reads, 4-5 MFMAs with the widening of 2 fragments underneath, 1-2 DMA
//    instructions], the DMA of a stage being spread over the sub-steps after the barrier that
//    frees its ring slot.
//  * Both operands stay packed (4 bit) all the way into LDS, and every global access fetches
//    whole 128-byte lines (256 codes per row per stage) -- half-line fetches were re-fetched
//    from L2 each time, an int8 copy of X doubled its traffic and was slower.
//  * Global -> LDS copies use the LDS-DMA form of the global load (no staging registers) into a
//    ring of two stages of 256 codes; one barrier per stage; per 64 codes a register-level
//    software pipeline (LDS reads for t+2, widening for t+1, MFMAs for t).
//  * The epilogue transposes each wave tile through the idle LDS ring and stores whole rows:
//    8-byte stores scattered over 32 rows per instruction cost 14 us per tile, this costs ~5.
//  * LDS rows are XOR-swizzled in 16-byte chunks (applied on the global side of the DMA,
//    which fills LDS linearly): ds_read_b128 of a fragment runs at the full LDS rate
//    (240 B/clk/CU measured with eight waves; one wave alone reaches 33 B/clk).
//  * MFMA operand roles are swapped (A = weight rows, B = token rows): a lane then owns 4
//    consecutive output channels of one token per accumulator quad = one 8-byte store.
//  * Tried and dropped: deeper DMA prefetch (three ring slots: DMA latency is already hidden),
//    dedicated DMA-issuing waves (1, 2 or 4 per workgroup: slower, a wave issues DMA too slowly).
//
// K % 256 != 0 (and any K % 64 == 0) runs on a simpler register-staged kernel further down.
#include "sr_common.h"

#include <hip/hip_fp16.h>
#include <stdlib.h>
#include <type_traits>

namespace sr {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr unsigned HM = 0xF0F0F0F0u;

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
// Epilogue for 32 x 32 MFMA tiles: dequantise, then transpose the wave's WM x WN tile through LDS
// so that global memory is written in whole rows of the tile (16 bytes per lane, WN * esize
// contiguous bytes per token) instead of 8-byte pieces scattered over 32 rows per instruction.
// In the accumulator layout a lane owns token (l & 31) and, per quad q, the four output channels
// 8q + 4 (l >> 5) .. + 3 of each tile.  `stage` is this wave's private LDS area of
// WM * (WN * 2 + 16) bytes; the caller has made sure nobody still reads it.
// ------------------------------------------------------------------------------------------
template <int FM, int FN>
__device__ __forceinline__ void store_wave_tile(const v16i (&acc)[FN][FM], uint8_t *stage, int lane, int m_base, int n_base,
                                                int M, int N, const float *__restrict__ xs,
                                                const float *__restrict__ ws, void *__restrict__ Yv, int64_t ldy,
                                                int out_i32)
{
    constexpr int WM = FM * 32, WN = FN * 32;
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
                            make_int4(acc[i][j][4 * q] >> 8, acc[i][j][4 * q + 1] >> 8, acc[i][j][4 * q + 2] >> 8,
                                      acc[i][j][4 * q + 3] >> 8);
                }
    } else {
        constexpr int RS = WN * 2 + 16;
#pragma unroll
        for (int j = 0; j < FM; ++j) {
            const int m = m_base + j * 32 + fr;
            const float sx = xs[m < M ? m : M - 1] * (1.f / 256.f);
#pragma unroll
            for (int i = 0; i < FN; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int nl = i * 32 + q * 8 + fg * 4;
                    const int n = n_base + nl < N ? n_base + nl : N - 4;
                    const float4 sw = *reinterpret_cast<const float4 *>(ws + n);
                    union { __half h[4]; uint2 u; } o;
                    o.h[0] = __float2half_rn((float)acc[i][j][4 * q] * sx * sw.x);
                    o.h[1] = __float2half_rn((float)acc[i][j][4 * q + 1] * sx * sw.y);
                    o.h[2] = __float2half_rn((float)acc[i][j][4 * q + 2] * sx * sw.z);
                    o.h[3] = __float2half_rn((float)acc[i][j][4 * q + 3] * sx * sw.w);
                    *reinterpret_cast<uint2 *>(stage + (j * 32 + fr) * RS + nl * 2) = o.u;
                }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        constexpr int CPR = WN * 2 / 16;
        constexpr int RPI = 64 / CPR;
        const int c = lane % CPR, r0 = lane / CPR;
#pragma unroll
        for (int r = r0; r < WM; r += RPI) {
            const int m = m_base + r, n = n_base + c * 8;
            const u32x4 v = *reinterpret_cast<const u32x4 *>(stage + r * RS + c * 16);
            // streamed once, never read back by this kernel: keep it from displacing operand panels in L2
            if (lane < RPI * CPR && m < M && n < N)
                __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(static_cast<__half *>(Yv) + (int64_t)m * ldy + n));
        }
    }
}

constexpr int ROWB = 128;  // packed bytes per row per stage (256 codes = one 128-byte line)

template <int BM, int BN, int WGM, int WGN, int STAGES, bool SMOOTH = false>
__global__ __launch_bounds__(WGM * WGN * 64) void gemm_w4a4_kernel(
    const uint8_t *__restrict__ Xq, const float *__restrict__ xs, const uint8_t *__restrict__ Wq,
    const float *__restrict__ ws, int M, int N, int K, void *__restrict__ Yv, int64_t ldy, int out_i32,
    int tiles_m, int tiles_n, int xcd_m)
{
    constexpr int NWAVE = WGM * WGN;
    constexpr int WM = BM / WGM, WN = BN / WGN;      // wave tile
    constexpr int FM = WM / 32, FN = WN / 32;        // 32 x 32 MFMA tiles per wave
    constexpr int REGIONS = (BM + BN) / 8;           // 1 KB DMA regions (8 rows x 128 B) per stage
    constexpr int RPW = REGIONS / NWAVE;             // DMA instructions per wave per stage
    constexpr int X_BYTES = BM * ROWB, STAGE_BYTES = (BM + BN) * ROWB;
    static_assert(REGIONS % NWAVE == 0 && NWAVE % 2 == 0 && WM % 32 == 0 && WN % 32 == 0 && STAGES >= 2 &&
                      (STAGES - 1) * RPW < 64, "tile");

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WGM, wn = wave / WGM;

    // workgroups are dealt round-robin to the 8 XCDs (each with its own L2): XCD x = blockIdx & 7 gets the
    // rectangle (x % xcd_m, x / xcd_m) of an xcd_m x (8 / xcd_m) split of the tile grid and walks it m
    // fastest, so the tiles that run together share few X and W panels (the split is chosen on the host)
    int tm, tn;
    if (xcd_m > 0) {
        const int x = blockIdx.x & 7, l = blockIdx.x >> 3;
        const int rm = tiles_m / xcd_m, rn = tiles_n / (8 / xcd_m);      // rectangle size in tiles
        tm = (x % xcd_m) * rm + l % rm;
        tn = (x / xcd_m) * rn + l / rm;
    } else {
        tm = blockIdx.x % tiles_m;
        tn = blockIdx.x / tiles_m;
    }
    const int m0 = tm * BM, n0 = tn * BN;
    const int Kb = K >> 1;
    const int ns = K / 256;                          // stages

    // ---- DMA sources.  Region q = wave + NWAVE * i holds rows 8q .. 8q+7 of the combined
    // [X rows ; W rows] tile.  Lane l lands in row l >> 3, physical chunk l & 7, and therefore
    // fetches logical chunk (l & 7) ^ swz(row), swz(row) = (row >> 1) & 7 (q and wave have
    // the same parity because NWAVE is even).
    const int dchunk = (lane & 7) ^ ((4 * (wave & 1) + (lane >> 4)) & 7);
    constexpr int XI = BM / 8 / NWAVE;               // the first XI regions of a wave are X rows, the rest W rows
    static_assert((BM / 8) % NWAVE == 0, "X regions must split evenly over the waves");
    uint32_t goff[RPW];
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const int trow = (wave + NWAVE * i) * 8 + (lane >> 3);
        int r;
        if (i < XI) { r = m0 + trow; r = r < M ? r : M - 1; }
        else { r = n0 + trow - BM; r = r < N ? r : N - 1; }
        goff[i] = (uint32_t)r * (uint32_t)Kb + (dchunk << 4);
    }
    const uint32_t smem_base = (uint32_t)(uintptr_t)smem;
    auto issue = [&](int s) {                        // stage s of K -> ring slot s % STAGES
        const uint32_t sb = smem_base + (uint32_t)(s % STAGES) * STAGE_BYTES + wave * 1024;
        const uint8_t *xsrc = Xq + (int64_t)s * ROWB;
        const uint8_t *wsrc = Wq + (int64_t)s * ROWB;
#pragma unroll
        for (int i = 0; i < RPW; ++i) dma16(i < XI ? xsrc : wsrc, goff[i], sb + NWAVE * i * 1024);
    };

    // ---- fragment addresses: lane (r = l & 31, g = l >> 5).  Sub-step p (64 codes) of a stage is
    // chunks 2p, 2p+1 of the row; lane group g takes chunk 2p + g, whose two 8-byte halves are the
    // operands of two consecutive MFMAs (K = 32 each).
    const int fr = lane & 31, fg = lane >> 5;
    const int fz = (fr >> 1) & 7;
    const int xrow = (wm * WM + fr) * ROWB, wrow = X_BYTES + (wn * WN + fr) * ROWB;

    struct Frag { uint4 x[FM]; uint4 w[FN]; };              // packed, as read from LDS
    struct Ops { v4i x[FM][2]; v4i w[FN][2]; };              // widened MFMA operands of one sub-step
    auto load_frags = [&](Frag &f, int slot, int p) {
        const uint8_t *st = smem + slot * STAGE_BYTES + (((2 * p + fg) ^ fz) << 4);
#pragma unroll
        for (int j = 0; j < FM; ++j) f.x[j] = *reinterpret_cast<const uint4 *>(st + xrow + j * 32 * ROWB);
#pragma unroll
        for (int i = 0; i < FN; ++i) f.w[i] = *reinterpret_cast<const uint4 *>(st + wrow + i * 32 * ROWB);
    };

    v16i acc[FN][FM];
#pragma unroll
    for (int i = 0; i < FN; ++i)
#pragma unroll
        for (int j = 0; j < FM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    auto widen = [](const uint4 w, v4i &a0, v4i &a1) {
        a0 = v4i{(int)((w.x << 4) & HM), (int)(w.x & HM), (int)((w.y << 4) & HM), (int)(w.y & HM)};
        a1 = v4i{(int)((w.z << 4) & HM), (int)(w.z & HM), (int)((w.w << 4) & HM), (int)(w.w & HM)};
    };
    auto widen_all = [&](const Frag &f, Ops &o) {
#pragma unroll
        for (int j = 0; j < FM; ++j) widen(f.x[j], o.x[j][0], o.x[j][1]);
#pragma unroll
        for (int i = 0; i < FN; ++i) widen(f.w[i], o.w[i][0], o.w[i][1]);
    };
    auto mfmas = [&](const Ops &o) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < FN; ++i)
#pragma unroll
                for (int j = 0; j < FM; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(o.w[i][h], o.x[j][h], acc[i][j], 0, 0, 0);
    };
    constexpr int NMFMA = 2 * FN * FM;                       // MFMAs per sub-step
    constexpr int NWID = 12 * (FM + FN);                     // widening ALU instructions per sub-step
    constexpr int PER = (NWID + NMFMA - 1) / NMFMA;
    // One sub-step t, three things in flight (a register-level software pipeline):
    //   LDS reads of the packed fragments of sub-step t+2          -> rd
    //   widening of the fragments of sub-step t+1 (read last time) -> nxt, underneath ...
    //   ... the MFMAs of sub-step t (the 8-pass MFMA leaves the ALU port free)
    // The scheduling hints pin that interleaving: reads first, then PER ALU instructions after each MFMA.
    auto sub = [&](auto do_read, auto do_widen, const Ops &cur, Ops &nxt, const Frag &wd, Frag &rd, int slot, int p) {
        __builtin_amdgcn_sched_barrier(0);               // each sub-step is scheduled on its own
        if constexpr (decltype(do_read)::value) load_frags(rd, slot, p);
        mfmas(cur);
        if constexpr (decltype(do_widen)::value) widen_all(wd, nxt);
        if constexpr (decltype(do_read)::value) __builtin_amdgcn_sched_group_barrier(0x100, FM + FN, 0);
#pragma unroll
        for (int k = 0; k < NMFMA; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if constexpr (decltype(do_widen)::value) __builtin_amdgcn_sched_group_barrier(0x002, PER, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    constexpr std::true_type yes{};
    constexpr std::false_type no{};

    Ops o0, o1;
    Frag fa, fb;                                     // fragments of even / odd sub-steps
    int slot = 0;
    if constexpr (SMOOTH) {
        // ---- smooth issue: memory instructions block the issuing wave while their queue is full, and with
        // one wave per SIMD a blocked wave idles the matrix pipe.  So nothing is issued in bursts: a sub-step
        // is cut into NREG regions of [FPR fragment reads, ~NM/NREG MFMAs with the widening of FPR fragments
        // underneath, ONE DMA instruction].  The RPW DMA instructions of a stage are thereby spread over the
        // four sub-steps that follow the barrier which frees their slot (ring of three slots: stage s+3 is
        // issued from the middle of iteration s to the middle of iteration s+1 and first read after barrier s+2).
        // With a ring of two slots the slot is needed again one stage later, so the stage is issued over the two
        // sub-steps after the barrier only (more than one DMA instruction per region).
        static_assert((STAGES == 3 || STAGES == 2) && (FM + FN) % 2 == 0, "smooth schedule");
        constexpr int FPR = 2;                       // fragments per region
        constexpr int NREG = (FM + FN) / FPR;        // regions per sub-step
        constexpr int NR = (STAGES == 3 ? 4 : 2) * NREG;        // regions a stage's DMA is spread over
        constexpr int DPR = (RPW + NR - 1) / NR;     // DMA instructions per region
        constexpr int HALF = 2 * NREG * DPR < RPW ? 2 * NREG * DPR : RPW;   // ... issued in a stage's first two sub-steps
        constexpr int NM = 2 * FM * FN;              // MFMAs per sub-step
        auto region = [&](auto RC, auto PARTC, const Ops &cur, Ops &nxt, const Frag &wd, Frag &rd, int rslot, int p,
                          int dstage, int dslot) {
            constexpr int r = decltype(RC)::value, part = decltype(PARTC)::value;
            constexpr int mlo = r * NM / NREG, mhi = (r + 1) * NM / NREG;
            constexpr int per = (12 * FPR + (mhi - mlo) - 1) / (mhi - mlo);
            __builtin_amdgcn_sched_barrier(0);
            const uint8_t *st = smem + rslot * STAGE_BYTES + (((2 * p + fg) ^ fz) << 4);
#pragma unroll
            for (int q = r * FPR; q < (r + 1) * FPR; ++q) {
                if (q < FM) rd.x[q < FM ? q : 0] = *reinterpret_cast<const uint4 *>(st + xrow + q * 32 * ROWB);
                else rd.w[q < FM ? 0 : q - FM] = *reinterpret_cast<const uint4 *>(st + wrow + (q - FM) * 32 * ROWB);
            }
#pragma unroll
            for (int m = mlo; m < mhi; ++m) {
                const int h = m / (FM * FN), i = (m % (FM * FN)) / FM, j = m % FM;
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(cur.w[i][h], cur.x[j][h], acc[i][j], 0, 0, 0);
            }
#pragma unroll
            for (int q = r * FPR; q < (r + 1) * FPR; ++q) {
                if (q < FM) widen(wd.x[q < FM ? q : 0], nxt.x[q < FM ? q : 0][0], nxt.x[q < FM ? q : 0][1]);
                else widen(wd.w[q < FM ? 0 : q - FM], nxt.w[q < FM ? 0 : q - FM][0], nxt.w[q < FM ? 0 : q - FM][1]);
            }
            __builtin_amdgcn_sched_group_barrier(0x100, FPR, 0);
#pragma unroll
            for (int k = mlo; k < mhi; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, per, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            constexpr int g = part * NREG + r;       // ordinal of this region among those that issue DMA
            if constexpr (g < NR) {
#pragma unroll
                for (int idx = g * DPR; idx < (g + 1) * DPR && idx < RPW; ++idx)
                    dma16((idx < XI ? Xq : Wq) + (int64_t)dstage * ROWB, goff[idx],
                          smem_base + (uint32_t)dslot * STAGE_BYTES + wave * 1024 + NWAVE * idx * 1024);
            }
        };
        auto ssub = [&](auto PARTC, const Ops &cur, Ops &nxt, const Frag &wd, Frag &rd, int rslot, int p, int dstage,
                        int dslot) {
            region(std::integral_constant<int, 0>{}, PARTC, cur, nxt, wd, rd, rslot, p, dstage, dslot);
            if constexpr (NREG >= 2) region(std::integral_constant<int, 1>{}, PARTC, cur, nxt, wd, rd, rslot, p, dstage, dslot);
            if constexpr (NREG >= 3) region(std::integral_constant<int, 2>{}, PARTC, cur, nxt, wd, rd, rslot, p, dstage, dslot);
            if constexpr (NREG >= 4) region(std::integral_constant<int, 3>{}, PARTC, cur, nxt, wd, rd, rslot, p, dstage, dslot);
            static_assert(NREG <= 4, "regions");
        };
        constexpr std::integral_constant<int, 0> P0{};
        constexpr std::integral_constant<int, 1> P1{};
        constexpr std::integral_constant<int, 2> P2{};
        constexpr std::integral_constant<int, 3> P3{};
        // prologue: stages 0 and 1 whole and, with three slots, the first half of stage 2
        issue(0);
        issue(ns > 1 ? 1 : 0);
        if constexpr (STAGES == 3) {
            const int st2 = ns > 2 ? 2 : ns - 1;
#pragma unroll
            for (int i = 0; i < HALF; ++i)
                dma16((i < XI ? Xq : Wq) + (int64_t)st2 * ROWB, goff[i],
                      smem_base + 2u * STAGE_BYTES + wave * 1024 + NWAVE * i * 1024);
            wait_vmcnt<RPW + HALF>();                // stage 0 has landed
        } else {
            wait_vmcnt<RPW>();
        }
        barrier_nofence();
        load_frags(fa, 0, 0);
        load_frags(fb, 0, 1);
        widen_all(fa, o0);
        for (int s = 0; s < ns; ++s) {
            const int nslot = slot == STAGES - 1 ? 0 : slot + 1, pslot = slot == 0 ? STAGES - 1 : slot - 1;
            const int st2 = s + 2 < ns ? s + 2 : ns - 1, st3 = s + 3 < ns ? s + 3 : ns - 1;
            // three slots: second half of stage s+2 -> slot of stage s-1; two slots: these sub-steps issue nothing
            ssub(P2, o0, o1, fb, fa, slot, 2, st2, pslot);
            ssub(P3, o1, o0, fa, fb, slot, 3, st2, pslot);
            // stage s+1 must have landed (with three slots stage s+2, the youngest RPW instructions, may still fly),
            // and every wave's reads of stage s must have returned: its slot takes stage s+STAGES from here on
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(STAGES == 3 ? RPW : 0) : "memory");
            barrier_nofence();
            ssub(P0, o0, o1, fb, fa, nslot, 0, STAGES == 3 ? st3 : st2, slot);
            ssub(P1, o1, o0, fa, fb, nslot, 1, STAGES == 3 ? st3 : st2, slot);
            slot = nslot;
        }
    } else {
    // Every stage runs the same branch-free body.  Past the end of K the pipeline keeps reading (stale,
    // in-bounds) LDS and re-fetching the last stage; those fragments are widened but never multiplied.
    // ---- prologue: two stages in flight; operands of sub-step 0 and fragments of sub-step 1 in registers
#pragma unroll
    for (int q = 0; q < STAGES; ++q) issue(q < ns ? q : ns - 1);
    wait_vmcnt<(STAGES - 1) * RPW>();                // stage 0 has landed, the younger ones may still fly
    barrier_nofence();
    load_frags(fa, 0, 0);
    load_frags(fb, 0, 1);
    widen_all(fa, o0);
    for (int s = 0; s < ns; ++s) {
        const int nslot = slot == STAGES - 1 ? 0 : slot + 1;
        sub(yes, yes, o0, o1, fb, fa, slot, 2);
        sub(yes, yes, o1, o0, fa, fb, slot, 3);
        // stage s+1 (issued STAGES-1 stages ago) must have landed for every wave -- the STAGES-2 younger
        // stages may stay in flight -- and every wave's LDS reads of stage s (the last ones were issued a
        // sub-step ago) must have returned: its slot now takes stage s+STAGES
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((STAGES - 2) * RPW) : "memory");
        barrier_nofence();
        issue(s + STAGES < ns ? s + STAGES : ns - 1);
        sub(yes, yes, o0, o1, fb, fa, nslot, 0);
        sub(yes, yes, o1, o0, fa, fb, nslot, 1);
        slot = nslot;
    }
    }
    wait_vmcnt<0>();                                 // no LDS-DMA write may outlive the workgroup

    // ---- epilogue: every wave transposes its tile through its own part of the (now idle) LDS ring ----
    barrier_nofence();                               // all waves are done reading fragments
    static_assert(NWAVE * WM * (WN * 2 + 16) <= STAGES * STAGE_BYTES, "epilogue staging must fit the ring");
    store_wave_tile<FM, FN>(acc, smem + wave * (WM * (WN * 2 + 16)), lane, m0 + wm * WM, n0 + wn * WN, M, N, xs, ws,
                            Yv, ldy, out_i32);
}

template <int BM, int BN, int WGM, int WGN, int STAGES = 2, bool SMOOTH = false>
hipError_t launch_tile(const uint8_t *Xq, const float *xs, const uint8_t *Wq, const float *ws, int64_t M, int64_t N,
                       int64_t K, void *Y, int64_t ldy, int out_i32, hipStream_t st)
{
    auto kern = gemm_w4a4_kernel<BM, BN, WGM, WGN, STAGES, SMOOTH>;
    constexpr int lds = STAGES * (BM + BN) * ROWB;
    static_assert(lds <= 160 * 1024, "LDS");
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
    }
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((N + BN - 1) / BN);
    // split of the tile grid over the 8 XCDs.  Measured (FETCH_SIZE, M = 2048, K = 4096): two halves in m by four
    // blocks in n reads 112 MB through the fabric at N = 14336 where one run of tiles per XCD read 223 MB (half
    // of X then stays in an XCD's 4 MB L2); it was also the fastest split at K = 14336.  Otherwise: the split
    // whose rectangles need the fewest operand rows.  0 = no remapping.
    int xcd_m = 0;
    if (tiles_m % 2 == 0 && tiles_n % 4 == 0) {
        xcd_m = 2;
    } else {
        int64_t best = 0;
        for (int sm = 1; sm <= 8; sm *= 2) {
            if (tiles_m % sm != 0 || tiles_n % (8 / sm) != 0) continue;
            const int64_t rows = (int64_t)(tiles_m / sm) * BM + (int64_t)(tiles_n / (8 / sm)) * BN;
            if (xcd_m == 0 || rows < best) { xcd_m = sm; best = rows; }
        }
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(WGM * WGN * 64), lds, st, Xq, xs, Wq, ws,
                       (int)M, (int)N, (int)K, Y, ldy, out_i32, tiles_m, tiles_n, xcd_m);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Generic kernel (any K % 64 == 0): 128 x 128 tile, K step of 128 codes, global -> registers
// -> LDS double buffering, v_mfma_i32_16x16x64_i8; a K tail of 64 codes is zero-filled.
// ------------------------------------------------------------------------------------------
constexpr int KB = 64;   // packed bytes of one K step per row (128 codes)

__device__ __forceinline__ int swz_off(int row, int chunk)
{
    return row * KB + ((chunk ^ ((row >> 2) & 3)) << 4);
}

__device__ __forceinline__ void unpack16(const uint4 w, v4i &a0, v4i &a1)
{
        a0[0] = (int)((w.x << 4) & HM); a0[1] = (int)(w.x & HM);
    a0[2] = (int)((w.y << 4) & HM); a0[3] = (int)(w.y & HM);
    a1[0] = (int)((w.z << 4) & HM); a1[1] = (int)(w.z & HM);
    a1[2] = (int)((w.w << 4) & HM); a1[3] = (int)(w.w & HM);
}

template <int BM, int BN>
__global__ __launch_bounds__(256) void gemm_w4a4_generic_kernel(const uint8_t *__restrict__ Xq, const float *__restrict__ xs,
                                                        const uint8_t *__restrict__ Wq, const float *__restrict__ ws,
                                                        int M, int N, int K, void *__restrict__ Yv, int64_t ldy,
                                                        int out_i32, int tiles_m, int tiles_n)
{
    constexpr int WM = BM / 2, WN = BN / 2;          // wave tile
    constexpr int FM = WM / 16, FN = WN / 16;        // MFMA tiles per wave
    constexpr int LX = BM * 4 / 256, LW = BN * 4 / 256;   // 16-byte loads per thread per K step
    static_assert(BM % 64 == 0 && BN % 64 == 0, "tile");

    __shared__ __attribute__((aligned(16))) uint8_t lds[2][(BM + BN) * KB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;

    // ---- workgroup -> tile: workgroups are dealt round-robin to the 8 XCDs, so give each
    // XCD a contiguous run of tiles (neighbours share X / W panels in that XCD's L2).
    int bid = blockIdx.x;
    const int total = tiles_m * tiles_n;
    if ((total & 7) == 0) bid = (bid & 7) * (total >> 3) + (bid >> 3);
    const int tm = bid % tiles_m, tn = bid / tiles_m;
    const int m0 = tm * BM, n0 = tn * BN;

    const int Kb = K >> 1;                          // packed bytes per row
    const int nk = (Kb + KB - 1) / KB;

    // global load coordinates: thread -> (row, 16-byte chunk)
    const int lrow = tid >> 2, lchunk = tid & 3;
    const uint8_t *xg[LX];
    const uint8_t *wg[LW];
#pragma unroll
    for (int i = 0; i < LX; ++i) {
        int r = m0 + lrow + 64 * i;
        r = r < M ? r : M - 1;
        xg[i] = Xq + (int64_t)r * Kb + lchunk * 16;
    }
#pragma unroll
    for (int i = 0; i < LW; ++i) {
        int r = n0 + lrow + 64 * i;
        r = r < N ? r : N - 1;
        wg[i] = Wq + (int64_t)r * Kb + lchunk * 16;
    }

    uint4 px[LX], pw[LW];
    auto gload = [&](int ks) {
        const int kb = ks * KB;
        const bool ok = kb + lchunk * 16 < Kb;      // K tail (K % 128 == 64): zero codes
#pragma unroll
        for (int i = 0; i < LX; ++i)
            px[i] = ok ? *reinterpret_cast<const uint4 *>(xg[i] + kb) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < LW; ++i)
            pw[i] = ok ? *reinterpret_cast<const uint4 *>(wg[i] + kb) : make_uint4(0, 0, 0, 0);
    };
    auto lstore = [&](int stage) {
        uint8_t *xs_l = lds[stage];
        uint8_t *ws_l = lds[stage] + BM * KB;
#pragma unroll
        for (int i = 0; i < LX; ++i)
            *reinterpret_cast<uint4 *>(xs_l + swz_off(lrow + 64 * i, lchunk)) = px[i];
#pragma unroll
        for (int i = 0; i < LW; ++i)
            *reinterpret_cast<uint4 *>(ws_l + swz_off(lrow + 64 * i, lchunk)) = pw[i];
    };

    v4i acc[FN][FM];
#pragma unroll
    for (int i = 0; i < FN; ++i)
#pragma unroll
        for (int j = 0; j < FM; ++j) acc[i][j] = v4i{0, 0, 0, 0};

    const int fr = lane & 15, fg = lane >> 4;       // fragment row / k group of this lane

    gload(0);
    lstore(0);
    __syncthreads();

    for (int ks = 0; ks < nk; ++ks) {
        const int stage = ks & 1;
        if (ks + 1 < nk) gload(ks + 1);

        const uint8_t *xs_l = lds[stage] + (wm * WM) * KB;
        const uint8_t *ws_l = lds[stage] + BM * KB + (wn * WN) * KB;

        v4i xa0[FM], xa1[FM];
#pragma unroll
        for (int j = 0; j < FM; ++j) {
            const uint4 p = *reinterpret_cast<const uint4 *>(xs_l + swz_off(j * 16 + fr, fg));
            unpack16(p, xa0[j], xa1[j]);
        }
#pragma unroll
        for (int i = 0; i < FN; ++i) {
            const uint4 p = *reinterpret_cast<const uint4 *>(ws_l + swz_off(i * 16 + fr, fg));
            v4i wa0, wa1;
            unpack16(p, wa0, wa1);
#pragma unroll
            for (int j = 0; j < FM; ++j) {
                acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa0, xa0[j], acc[i][j], 0, 0, 0);
                acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa1, xa1[j], acc[i][j], 0, 0, 0);
            }
        }

        if (ks + 1 < nk) lstore(stage ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane owns token m, output channels n .. n+3 of each MFMA tile ----------
#pragma unroll
    for (int j = 0; j < FM; ++j) {
        const int m = m0 + wm * WM + j * 16 + fr;
        if (m >= M) continue;
        const float sx = out_i32 ? 0.f : xs[m] * (1.f / 256.f);
#pragma unroll
        for (int i = 0; i < FN; ++i) {
            const int n = n0 + wn * WN + i * 16 + fg * 4;
            if (n >= N) continue;
            const v4i a = acc[i][j];
            if (out_i32) {
                int4 o = make_int4(a[0] >> 8, a[1] >> 8, a[2] >> 8, a[3] >> 8);
                *reinterpret_cast<int4 *>(static_cast<int32_t *>(Yv) + (int64_t)m * ldy + n) = o;
            } else {
                const float4 sw = *reinterpret_cast<const float4 *>(ws + n);
                union { __half h[4]; uint2 u; } o;
                o.h[0] = __float2half_rn((float)a[0] * sx * sw.x);
                o.h[1] = __float2half_rn((float)a[1] * sx * sw.y);
                o.h[2] = __float2half_rn((float)a[2] * sx * sw.z);
                o.h[3] = __float2half_rn((float)a[3] * sx * sw.w);
                *reinterpret_cast<uint2 *>(static_cast<__half *>(Yv) + (int64_t)m * ldy + n) = o.u;
            }
        }
    }
}


}  // namespace

hipError_t launch_gemm_prefill(const uint8_t *Xq, const float *xs, const uint8_t *Wq, const float *ws,
                               int64_t M, int64_t N, int64_t K, void *Y, int64_t ldy, int out_i32,
                               hipStream_t st)
{
    // SMOOTHROT_GEMM_TILE selects a tile configuration by number (tuning aid); unset = heuristic.
    int variant = 0;
    if (const char *env = getenv("SMOOTHROT_GEMM_TILE")) variant = atoi(env);
    if (K % 256 != 0 || variant == 9) {
        constexpr int BM = 128, BN = 128;
        const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((N + BN - 1) / BN);
        hipLaunchKernelGGL((gemm_w4a4_generic_kernel<BM, BN>), dim3((unsigned)(tiles_m * tiles_n)), dim3(256), 0, st,
                           Xq, xs, Wq, ws, (int)M, (int)N, (int)K, Y, ldy, out_i32, tiles_m, tiles_n);
        return hipGetLastError();
    }
    switch (variant) {
        case 1: return launch_tile<256, 128, 2, 2>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);               // burst schedule
        case 3: return launch_tile<128, 128, 2, 2>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);               // burst schedule
        case 10: return launch_tile<256, 128, 2, 2, 3, true>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);     // 4 waves, 3 slots
        case 12: return launch_tile<256, 128, 4, 2, 3, true>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);     // 8 waves, 3 slots
        case 14: return launch_tile<128, 128, 2, 2, 2, true>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);
        case 15: return launch_tile<256, 128, 4, 2, 2, true>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);
        default: break;
    }
    // A launch takes about ceil(tiles / 256) rounds of one tile time each (tile time ~ BM * BN): pick the tile
    // shape with the cheapest schedule; ties go to the larger tile (less L2 traffic, fewer fragment reads).
    //   256 x 128: eight waves (two per SIMD, so that one can issue MFMAs while the other is held up issuing
    //              LDS or DMA instructions), 96 KB of LDS, one workgroup per CU
    //   128 x 128: four waves, 64 KB of LDS, two workgroups per CU
    // both with the smooth (burst-free) instruction schedule and a ring of two stages.
    auto cost = [&](int64_t bm, int64_t bn) {
        const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
        return ((tiles + 255) / 256) * bm * bn;
    };
    const int64_t c256 = cost(256, 128), c128 = cost(128, 128);
    if (c256 <= c128) return launch_tile<256, 128, 4, 2, 2, true>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);
    return launch_tile<128, 128, 2, 2, 2, true>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);
}

}  // namespace sr
