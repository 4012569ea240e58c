// INT4 x INT4 GEMM on the FP6 matrix pipe, compute-bound shapes.
//
//   acc[m][n] = sum_k cX[m][k] * cW[n][k],   Y = fp16(acc * dx[m] * dw[n])
//
// (Paper: the quantised forward pass of the linear layer; dequantisation per Eq. (1).)
//
// gfx950 has no 4-bit integer matrix instruction, and its int8 MFMA sustains ~3.5 POP/s on this
// chip (power).  The scaled-float MFMA family runs 6-bit floats at twice the int8 rate, and the
// 6-bit format E2M3 (sign, 2 exponent bits, 3 mantissa bits, bias 1) holds every INT4 code
// exactly: its first sixteen magnitudes -- the subnormals m/8 and the first binade 1 + m/8 --
// are the linear sequence 0, 1/8, ..., 15/8, so a code c is the 6-bit pattern
//     f6(c) = (c < 0 ? 32 : 0) | |c|            (value c / 8)
// and needs no arithmetic to build.  Products c_x c_w / 64 and their sums are integers / 64 below
// 2^24 / 64 for K < 262144, so the fp32 accumulation is exact in any order; measured on MI355X:
// v_mfma_f32_32x32x64_f8f6f4 reproduces the integer sums bit for bit (K = 14336, random codes and
// the all -8 worst case) and issues at 5.4 - 6.2 POP/s where the int8 MFMA reaches 3.3 - 3.7.
//
// The operands arrive already packed as 6-bit fields in the layout the MFMA wants ("f6 tiles",
// written by pack_f6.hip and by the activation quantiser), so the main loop has no vector-ALU
// work at all: LDS-DMA loads, LDS reads, MFMAs.
//
// f6 tiles of a code matrix [rows, K], K % 128 == 0, rows padded to a multiple of 8:
//   block (R, C) = rows 8R .. 8R+7 x codes 128C .. 128C+127, 768 bytes at ((C * rows/8) + R) * 768
//   (chunk-major: the blocks of all rows for one 128-code chunk are contiguous, so one stage of a tile is
//   two contiguous runs -- BM * 96 bytes of X and BN * 96 bytes of W -- copied by whole-KB LDS-DMA loads).
//   Inside a block, piece (r, t, g) = the 32 codes k = 128C + 64t + 32g + j (j = 0..31) of row
//   8R + r, code j in bits [6j, 6j+6) of a 24-byte little-endian string -- exactly the operand
//   of lane (row, k half g) of MFMA step t.  Its first 16 bytes live at
//       256 t + 128 (g ^ (R & 1)) + 16 r
//   and its last 8 bytes at
//       512 + 128 (g ^ (R & 1)) + 16 r + 8 t
//   i.e. the tails of the two steps share one 16-byte slot of the same (g, r) pattern as the first parts; a
//   32-row fragment (four blocks) then touches every LDS bank once per read.  The compiler reads each step's
//   half of the slot with 8-byte reads paired over two fragments (ds_read2st64_b64).  Measured in one process
//   against the first layout (tails in separate, XOR-swizzled 8-byte slots): M = 2048, N = 14336, K = 4096
//   69.8 -> 65.8 us, 4096 x 4096 x 14336 116.7 -> 108.1 us; forcing whole 16-byte tail reads (ds_read_b128,
//   the other half kept in registers for the next step) was 1 - 5 % slower than leaving the split to the compiler.
//   (The 12-byte form of the LDS-DMA load leaves a 4-byte hole after every lane's data in LDS -- measured -- so
//   stages are copied with the 16-byte form, 1 KB per instruction.)
//
// Kernel structure: persistent workgroups, tile BM x BN, ring of SLOTS stages of 128 codes, one
// barrier per stage, two MFMA steps (64 codes) per stage with the fragment reads of the next
// step issued under the MFMAs of the current one; transposing epilogue shared with the int8
// kernel; scales of a tile fetched by LDS-DMA at the start of the tile.
#include "sr_common.h"
#include "gemm_common.h"

#include <type_traits>

namespace sr {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int BLK = 768;     // bytes of one block (8 rows x 128 codes x 6 bits)

// 64 lanes x 4 bytes -> LDS bytes [lds, lds + 256)
__device__ __forceinline__ void dma4(const void *base, uint32_t lane_off, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds), "v"(lane_off), "s"(base)
                 : "memory", "m0");
}

// The work of one workgroup: tiles v0, v0 + vstep, ... (< total) of the tile grid tiles_m x tiles_n that starts
// at output channel n_off.  CG = MFMA column tiles staged at a time by the epilogue.
// WARM: the workgroup has one wave more than the tile needs.  That wave computes nothing: it reads one word of
// every 128-byte line of the workgroup's share of [warm, warm + 128 warm_lines), a few lines per K stage, so that
// the memory-side cache holds that region when the next kernel asks for it -- the matrix waves are short of L2
// delivery and LDS bandwidth, not of HBM bandwidth, and cannot issue such loads themselves (a wave's loads
// complete in order: a slow load from HBM between the LDS-DMA loads would hold up their counted completion).
// The extra wave joins every barrier of the workgroup, so its loop mirrors the barrier count of the tile loop.
// (Also built and measured for the 256 x 256 configuration, which has no registers for a ninth wave: the
// workgroups that run out of tiles before the last round reading the region instead.  With the 12.6 MB of the
// benchmark's N = 4096 weights behind its N = 14336 launch the step got 2 % slower, not faster; dropped.)
template <int BM, int BN, int WGM, int WGN, int SLOTS, int CG, bool WARM = false>
__device__ __forceinline__ void f6_tiles(
    const uint8_t *__restrict__ X6, const float *__restrict__ xs, const uint8_t *__restrict__ W6,
    const float *__restrict__ ws, const int M, const int N, const int K, void *__restrict__ Yv, const int64_t ldy,
    const int out_i32, const int tiles_m, const int tiles_n, const int xcd_m, const int n_off, const int v0,
    const int vstep, const int total, const uint32_t *__restrict__ warm = nullptr, const int64_t warm_lines = 0)
{
    constexpr int NWAVE = WGM * WGN;
    constexpr int WM = BM / WGM, WN = BN / WGN;      // wave tile
    constexpr int FM = WM / 32, FN = WN / 32;        // 32 x 32 MFMA tiles per wave
    constexpr int X_BYTES = BM / 8 * BLK, STAGE_BYTES = (BM + BN) / 8 * BLK;
    // 1 KB LDS-DMA instructions per stage: NXI for the X run, NWI for the W run; every wave issues XI + WI of
    // them -- where the count does not divide by the waves, the last ones wrap around and copy a KB a second
    // time (same data to the same place), so that all waves keep the same number of loads in flight
    constexpr int NXI = X_BYTES / 1024, NWI = (STAGE_BYTES - X_BYTES) / 1024;
    constexpr int XI = (NXI + NWAVE - 1) / NWAVE, WI = (NWI + NWAVE - 1) / NWAVE;
    constexpr int RPW = XI + WI;
    constexpr int SCALE_OFF = SLOTS * STAGE_BYTES;   // two areas of BM + BN floats behind the ring
    constexpr int NSC = (BM + BN) / 64;              // scale DMA instructions per tile
    static_assert(X_BYTES % 1024 == 0 && STAGE_BYTES % 1024 == 0 && WM % 32 == 0 && WN % 32 == 0 && BM % 64 == 0 &&
                      BN % 64 == 0 && SLOTS >= 2 && SLOTS * RPW < 64, "tile");

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WGM, wn = wave / WGM;
    const int nc = K >> 7;                           // 128-code chunks per row = stages
    if constexpr (WARM) {
        if (wave == NWAVE) {
            // load instruction j of this wave touches lines (j * vstep + v0) * 64 + lane: the workgroups of the
            // launch sweep the region front to back together
            const int64_t per_wg = (warm_lines + (int64_t)vstep * 64 - 1) / ((int64_t)vstep * 64);   // instructions of this wave
            const int my_tiles = (total - v0 + vstep - 1) / vstep;
            // spread evenly over the K stages of this workgroup's tiles (measured inside the benchmark's step, 44 MB
            // behind the M = 2048, N = 4096 GEMM: all loads up front costs the step 2.5 % against one per stage;
            // non-temporal loads are not kept by the memory-side cache; the scope bits make no difference)
            const int per_stage = (int)((per_wg + (int64_t)my_tiles * nc - 1) / ((int64_t)my_tiles * nc));
            int64_t l = (int64_t)v0 * 64 + lane;
            uint32_t word = 0;
            for (int v = v0; v < total; v += vstep) {
                barrier_nofence();
                for (int s = 0; s < nc; ++s) {
                    for (int i = 0; i < per_stage; ++i) {
                        if (l < warm_lines) asm volatile("global_load_dword %0, %1, off" : "=v"(word) : "v"(warm + l * 32) : "memory");
                        l += (int64_t)vstep * 64;
                    }
                    barrier_nofence();
                }
                barrier_nofence();
                if (v + vstep < total) barrier_nofence();
            }
            wait_vmcnt<0>();
            asm volatile("" ::"v"(word));
            return;
        }
    }
    const uint32_t cx_bytes = (uint32_t)((M + 7) >> 3) * BLK, cw_bytes = (uint32_t)((N + 7) >> 3) * BLK;   // one chunk of X / W

    // ---- DMA sources: X instruction q copies bytes [1024 q, 1024 q + 1024) of the stage's X run, W instruction q
    // of its W run; a lane past the end of the operand re-reads the last 16 bytes
    uint32_t goff[RPW], ldst[RPW];
#pragma unroll
    for (int i = 0; i < RPW; ++i)
        ldst[i] = i < XI ? (uint32_t)((wave + NWAVE * i) % NXI) * 1024 : X_BYTES + (uint32_t)((wave + NWAVE * (i - XI)) % NWI) * 1024;
    auto set_sources = [&](int m0, int n0) {
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            uint32_t off;
            if (i < XI) { off = (uint32_t)(m0 >> 3) * BLK + ldst[i] + lane * 16; off = off < cx_bytes ? off : cx_bytes - 16; }
            else { off = (uint32_t)(n0 >> 3) * BLK + (ldst[i] - X_BYTES) + lane * 16; off = off < cw_bytes ? off : cw_bytes - 16; }
            goff[i] = off;
        }
    };
    const uint32_t smem_base = (uint32_t)(uintptr_t)smem;
    auto dma_one = [&](int idx, int s, int slot) {   // instruction idx of this wave, stage s -> ring slot
        dma16((idx < XI ? X6 + (int64_t)s * cx_bytes : W6 + (int64_t)s * cw_bytes), goff[idx],
              smem_base + (uint32_t)slot * STAGE_BYTES + ldst[idx]);
    };
    auto issue = [&](int s, int slot) {
#pragma unroll
        for (int i = 0; i < RPW; ++i) dma_one(i, s, slot);
    };
    // scales of a tile: floats [0, BM) = token scales, [BM, BM + BN) = channel scales, 64 per instruction
    auto issue_scales = [&](int m0, int n0, int area) {
#pragma unroll
        for (int k = 0; k < (NSC + NWAVE - 1) / NWAVE; ++k) {
            const int idx = wave + k * NWAVE;        // wave-uniform
            if (idx < NSC) {
                const int f = idx * 64 + lane;
                const bool is_x = idx < BM / 64;
                int e = is_x ? m0 + f : n0 + f - BM;
                const int last = is_x ? M - 1 : N - 1;
                e = e < last ? e : last;
                const uint32_t dst = smem_base + SCALE_OFF + (uint32_t)area * (BM + BN) * 4 + (uint32_t)idx * 256;
                dma4(is_x ? xs : ws, (uint32_t)e * 4u, (uint32_t)__builtin_amdgcn_readfirstlane((int)dst));
            }
        }
    };

    // ---- fragment addresses: lane (r = l & 31, g = l >> 5) reads row r of a 32-row fragment, k half g
    const int fr = lane & 31, fg = lane >> 5;
    const int rq = fr >> 3;                          // block of the fragment (= R & 3: fragments start at multiples of 32 rows)
    const uint32_t a16 = rq * BLK + ((fg ^ (rq & 1)) << 7) + ((fr & 7) << 4);   // step 0; step 1 at + 256; tails at + 512
    const uint32_t xfrag = (wm * WM / 8) * BLK, wfrag = X_BYTES + (wn * WN / 8) * BLK;

    struct Frags { v8i x[FM]; v8i w[FN]; };
    uint2 tail1[FM + FN];                            // tails of step 1, read together with those of step 0
    // fragment q of a stage, step t: step 0 also fetches the 16 bytes holding both tails.  The W fragments come
    // first and the MFMAs below walk the X fragments in the outer loop, so that the fragments read last in a step
    // are the ones the next step needs last (with X first, the first MFMA of a step waited for the last read).
    auto read_q = [&](Frags &f, int q, uint32_t sbase, int t) {
        const uint32_t base = sbase + (q < FN ? wfrag + q * 4 * BLK : xfrag + (q - FN) * 4 * BLK) + a16;
        v8i &d = q < FN ? f.w[q < FN ? q : 0] : f.x[q < FN ? 0 : q - FN];
        const uint4 lo = *reinterpret_cast<const uint4 *>(smem + base + t * 256);
        d[0] = (int)lo.x; d[1] = (int)lo.y; d[2] = (int)lo.z; d[3] = (int)lo.w;
        if (t == 0) {
            const uint4 tl = *reinterpret_cast<const uint4 *>(smem + base + 512);
            d[4] = (int)tl.x; d[5] = (int)tl.y;
            tail1[q] = make_uint2(tl.z, tl.w);
        } else {
            d[4] = (int)tail1[q].x; d[5] = (int)tail1[q].y;
        }
    };

    v16f acc[FN][FM];

    // ---- one MFMA step (64 codes): the FM * FN MFMAs on `cur`, the reads of the next step's FM + FN fragments
    // into `nxt` and a share of the DMA of a later stage, cut into regions of [2 fragment reads, a slice of the
    // MFMAs, some DMA instructions] so that no memory instruction queue sees a burst.
    // regions per step: fragments read in pairs -- measured against 1, 2 and FM + FN regions (M = 2048, N = 14336,
    // K = 4096: 68.9, 63.1, 65.7 us against 62.0 us)
    constexpr int NREG = (FM + FN + 1) / 2;
    constexpr int FPRG = (FM + FN + NREG - 1) / NREG;   // fragments read per region
    constexpr int NM = FM * FN;                      // MFMAs per step
    // (Tried: the two waves of a SIMD issuing their DMA in different steps, so that they are not held up at the
    // same moments -- 1 - 2 % slower.)
    constexpr int HALF = SLOTS == 2 ? RPW : (RPW + 1) / 2;      // DMA instructions issued in the step after the barrier
    auto step = [&](auto PART, const Frags &cur, Frags &nxt, uint32_t rbase, int t, int dstage, int dslot) {
        constexpr int part = decltype(PART)::value;             // 0: step after the barrier, 1: step before it
        constexpr int dlo = part == 0 ? 0 : HALF, dhi = part == 0 ? HALF : RPW;
        constexpr int DPR = (dhi - dlo + NREG - 1) / NREG;
#pragma unroll
        for (int r = 0; r < NREG; ++r) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = r * FPRG; q < (r + 1) * FPRG && q < FM + FN; ++q) read_q(nxt, q, rbase, t);
            const int mlo = r * NM / NREG, mhi = (r + 1) * NM / NREG;
#pragma unroll
            for (int m = mlo; m < mhi; ++m) {
                const int j = m / FN, i = m % FN;
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(cur.w[i], cur.x[j], acc[i][j], 2, 2, 0, 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int idx = dlo + r * DPR; idx < dlo + (r + 1) * DPR && idx < dhi; ++idx) dma_one(idx, dstage, dslot);
        }
    };
    constexpr std::integral_constant<int, 0> AFTER{};
    constexpr std::integral_constant<int, 1> BEFORE{};

    // epilogue staging: one piece = 32 tokens x CG * 32 channels of fp16 per wave, in the last ring slot
    constexpr int PIECE = 32 * (CG * 64 + 16);
    static_assert(NWAVE * PIECE <= STAGE_BYTES, "epilogue staging must fit one ring slot");

    int v = v0;
    int m0, n0;
    tile_origin(v, tiles_m, tiles_n, xcd_m, BM, BN, m0, n0);
    n0 += n_off;
    set_sources(m0, n0);
    // order of a wave's loads at the start of every tile: stage 0, scales, stages 1 .. SLOTS-2, first part of
    // stage SLOTS-1 (its second part is issued by the first step of the loop)
    int area = 0;
    issue(0, 0);
    issue_scales(m0, n0, area);
#pragma unroll
    for (int q = 1; q < SLOTS - 1; ++q) issue(q < nc ? q : nc - 1, q);
#pragma unroll
    for (int i = 0; i < HALF; ++i) dma_one(i, SLOTS - 1 < nc ? SLOTS - 1 : nc - 1, SLOTS - 1);
    for (;;) {
#pragma unroll
        for (int i = 0; i < FN; ++i)
#pragma unroll
            for (int j = 0; j < FM; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

        // Stage 0 (and the scales) have landed once at most (SLOTS-2) RPW + HALF of this wave's memory operations
        // are outstanding: loads complete in order among themselves and that many loads are younger, so an
        // unfinished older load would leave more outstanding -- however many stores of the previous tile are
        // still on their way (stores and loads may overtake each other).
        wait_vmcnt<(SLOTS - 2) * RPW + HALF>();
        barrier_nofence();
        Frags fa, fb;                                // fragments of step 0 / step 1 of a stage
#pragma unroll
        for (int q = 0; q < FM + FN; ++q) read_q(fa, q, 0, 0);
        int slot = 0;
        // Every stage runs the same branch-free body.  Past the end of K the pipeline keeps reading (stale,
        // in-bounds) LDS and re-fetching the last stage; those fragments are never multiplied.
        for (int s = 0; s < nc; ++s) {
            const int nslot = slot == SLOTS - 1 ? 0 : slot + 1, pslot = slot == 0 ? SLOTS - 1 : slot - 1;
            const int sa = s + SLOTS - 1 < nc ? s + SLOTS - 1 : nc - 1, sb = s + SLOTS < nc ? s + SLOTS : nc - 1;
            // step 0 of stage s; reads step 1; second part of the DMA of stage s+SLOTS-1 -> slot of stage s-1
            step(BEFORE, fa, fb, (uint32_t)slot * STAGE_BYTES, 1, sa, pslot);
            // stage s+1 must have landed (the SLOTS-2 younger stages may stay in flight), and every wave's
            // reads of stage s must have returned: its slot takes stage s+SLOTS from here on
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((SLOTS - 2) * RPW) : "memory");
            barrier_nofence();
            // step 1 of stage s; reads step 0 of stage s+1; first part of the DMA of stage s+SLOTS
            step(AFTER, fb, fa, (uint32_t)nslot * STAGE_BYTES, 0, sb, slot);
            slot = nslot;
        }

        // ---- tile boundary
        const int vn = v + vstep;
        const bool more = vn < total;
        wait_vmcnt<0>();                             // no LDS-DMA write is in flight any more ...
        barrier_nofence();                           // ... and all waves are done reading fragments
        int m1 = 0, n1 = 0;
        if (more) {                                  // the next tile's first stages fly during the epilogue
            tile_origin(vn, tiles_m, tiles_n, xcd_m, BM, BN, m1, n1);
            n1 += n_off;
            set_sources(m1, n1);
            issue(0, 0);
            issue_scales(m1, n1, area ^ 1);
#pragma unroll
            for (int q = 1; q < SLOTS - 1; ++q) issue(q < nc ? q : nc - 1, q);
        }
        {
            const float *sc = reinterpret_cast<const float *>(smem + SCALE_OFF) + area * (BM + BN);
            float sx[FM];
            float4 sw[FN][4];
#pragma unroll
            for (int j = 0; j < FM; ++j) sx[j] = sc[wm * WM + j * 32 + fr] * 64.f;      // both operands carried a factor 1/8
#pragma unroll
            for (int i = 0; i < FN; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    sw[i][q] = *reinterpret_cast<const float4 *>(sc + BM + wn * WN + i * 32 + q * 8 + fg * 4);
            store_wave_tile<FM, FN, CG>(acc, smem + (SLOTS - 1) * STAGE_BYTES + wave * PIECE, lane, m0 + wm * WM, n0 + wn * WN,
                                    M, N, sx, sw, Yv, ldy, out_i32);
        }
        if (!more) break;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        barrier_nofence();                           // every wave has read its staging back: the last slot is free
#pragma unroll
        for (int i = 0; i < HALF; ++i) dma_one(i, SLOTS - 1 < nc ? SLOTS - 1 : nc - 1, SLOTS - 1);
        v = vn;
        m0 = m1;
        n0 = n1;
        area ^= 1;
    }
    wait_vmcnt<0>();
}

constexpr int f6_lds_bytes(int BM, int BN, int SLOTS) { return SLOTS * (BM + BN) / 8 * BLK + 2 * (BM + BN) * 4 + 256; }   // ring, two scale areas, slack

template <int BM, int BN, int WGM, int WGN, int SLOTS, int WG_PER_CU>
__global__ __launch_bounds__(WGM * WGN * 64, WGM * WGN * WG_PER_CU / 4) void gemm_f6_kernel(
    const uint8_t *__restrict__ X6, const float *__restrict__ xs, const uint8_t *__restrict__ W6,
    const float *__restrict__ ws, int M, int N, int K, void *__restrict__ Yv, int64_t ldy, int out_i32,
    int tiles_m, int tiles_n, int xcd_m)
{
    f6_tiles<BM, BN, WGM, WGN, SLOTS, BN / WGN / 32>(X6, xs, W6, ws, M, N, K, Yv, ldy, out_i32, tiles_m, tiles_n, xcd_m, 0,
                                                     (int)blockIdx.x, (int)gridDim.x, tiles_m * tiles_n);
}

// The same with a ninth wave that warms the memory-side cache (one workgroup per CU: three waves then share the
// first SIMD, which the register budget of the 64 x 64 wave tile allows and that of the 128 x 64 one does not).
template <int BM, int BN, int WGM, int WGN, int SLOTS>
__global__ __launch_bounds__((WGM * WGN + 1) * 64) void gemm_f6_warm_kernel(
    const uint8_t *__restrict__ X6, const float *__restrict__ xs, const uint8_t *__restrict__ W6,
    const float *__restrict__ ws, int M, int N, int K, void *__restrict__ Yv, int64_t ldy, int out_i32,
    int tiles_m, int tiles_n, int xcd_m, const uint32_t *__restrict__ warm, int64_t warm_lines)
{
    f6_tiles<BM, BN, WGM, WGN, SLOTS, BN / WGN / 32, true>(X6, xs, W6, ws, M, N, K, Yv, ldy, out_i32, tiles_m, tiles_n, xcd_m,
                                                           0, (int)blockIdx.x, (int)gridDim.x, tiles_m * tiles_n, warm,
                                                           warm_lines);
}

template <int BM, int BN, int WGM, int WGN, int SLOTS, int WG_PER_CU, bool CAN_WARM = false>
hipError_t launch_f6(const uint8_t *X6, const float *xs, const uint8_t *W6, const float *ws, int64_t M, int64_t N,
                     int64_t K, void *Y, int64_t ldy, int out_i32, hipStream_t st, const void *warm = nullptr,
                     size_t warm_bytes = 0)
{
    auto kern = gemm_f6_kernel<BM, BN, WGM, WGN, SLOTS, WG_PER_CU>;
    constexpr int lds = f6_lds_bytes(BM, BN, SLOTS);
    static_assert(lds * WG_PER_CU <= 160 * 1024, "LDS");
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
    }
    bool warms = false;
    if constexpr (CAN_WARM) {
        static_assert(WG_PER_CU == 1, "the extra wave is budgeted for one workgroup per CU");
        warms = warm && warm_bytes >= 128;
        if (int64_t w; tuned(kTuneGemmWarm, w) && w == 0) warms = false;
        if (warms && lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_f6_warm_kernel<BM, BN, WGM, WGN, SLOTS>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            if (e != hipSuccess) return e;
        }
    }
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((N + BN - 1) / BN);
    int xcd_m = choose_xcd_split(tiles_m, tiles_n, BM, BN);
    if (int64_t f; tuned(kTuneGemmXcdM, f)) {                         // force the split (0 = none)
        if (f == 0 || ((f == 1 || f == 2 || f == 4 || f == 8) && tiles_m % f == 0 && tiles_n % (8 / f) == 0)) xcd_m = (int)f;
    }
    int64_t grid = (int64_t)compute_units() * WG_PER_CU;
    if (int64_t g; tuned(kTuneGemmGrid, g) && g > 0) grid = g / 8 * 8;
    if (grid < 8) grid = 8;
    const int64_t total = (int64_t)tiles_m * tiles_n;
    if (grid > total) grid = total;
    // the raw int32 output takes no scales (they may be NULL): the kernel still fetches M and N floats it then
    // ignores, from the start of the operand arrays (at least 96 M and 96 N bytes, 16-byte aligned)
    if (out_i32) {
        xs = reinterpret_cast<const float *>(X6);
        ws = reinterpret_cast<const float *>(W6);
    }
    if constexpr (CAN_WARM) {
        if (warms) {
            hipLaunchKernelGGL((gemm_f6_warm_kernel<BM, BN, WGM, WGN, SLOTS>), dim3((unsigned)grid), dim3((WGM * WGN + 1) * 64),
                               lds, st, X6, xs, W6, ws, (int)M, (int)N, (int)K, Y, ldy, out_i32, tiles_m, tiles_n, xcd_m,
                               static_cast<const uint32_t *>(warm), (int64_t)(warm_bytes / 128));
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(WGM * WGN * 64), lds, st, X6, xs, W6, ws,
                       (int)M, (int)N, (int)K, Y, ldy, out_i32, tiles_m, tiles_n, xcd_m);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Repacking of canonical INT4 codes (two per byte along K) into f6 tiles.  One thread per piece
// (row, 128-code chunk, step t, half g): 16 bytes in, 24 bytes out.  Rows >= rows (padding of
// the last block) are written as zeros.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pack_f6_kernel(const uint8_t *__restrict__ Q4, int rows, int K,
                                                      uint8_t *__restrict__ T6, int64_t pieces)
{
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= pieces) return;
    // piece index: [C][R][t][g][r] with r fastest, so that the 16-byte parts of neighbouring threads are neighbours
    const int r = (int)(p & 7), g = (int)((p >> 3) & 1), t = (int)((p >> 4) & 1);
    const int64_t bc = p >> 5;                      // C * row_blocks + R = index of the block in memory
    const int64_t rb = ((int64_t)rows + 7) >> 3;
    const int C = (int)(bc / rb);
    const int64_t R = bc % rb;
    const int64_t row = R * 8 + r;
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    if (row < rows) {
        const uint4 q = *reinterpret_cast<const uint4 *>(Q4 + row * (int64_t)(K >> 1) + C * 64 + t * 32 + g * 16);
        w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
    }
    uint32_t o[6] = {0u, 0u, 0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        const uint32_t nib = (w[j >> 3] >> ((j & 7) * 4)) & 15u;
        const uint32_t f = nib < 8u ? nib : (32u | (16u - nib));          // sign-magnitude 6-bit field
        const int bit = 6 * j;
        o[bit >> 5] |= f << (bit & 31);
        if ((bit & 31) > 26) o[(bit >> 5) + 1] |= f >> (32 - (bit & 31));
    }
    uint8_t *blk = T6 + bc * BLK;
    const int Rl = (int)(R & 3);
    *reinterpret_cast<uint4 *>(blk + 256 * t + 128 * (g ^ (Rl & 1)) + 16 * r) = make_uint4(o[0], o[1], o[2], o[3]);
    *reinterpret_cast<uint2 *>(blk + 512 + 128 * (g ^ (Rl & 1)) + 16 * r + 8 * t) = make_uint2(o[4], o[5]);
}

}  // namespace

hipError_t launch_pack_f6(const uint8_t *Q4, int64_t rows, int64_t K, uint8_t *T6, hipStream_t st)
{
    const int64_t pieces = ((rows + 7) / 8) * 8 * (K / 128) * 4;
    hipLaunchKernelGGL(pack_f6_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st, Q4, (int)rows, (int)K, T6,
                       pieces);
    return hipGetLastError();
}

hipError_t launch_gemm_f6(const uint8_t *X6, const float *xs, const uint8_t *W6, const float *ws, int64_t M, int64_t N,
                          int64_t K, void *Y, int64_t ldy, int out_i32, hipStream_t st, const void *warm, size_t warm_bytes)
{
    // the tile knob selects a tile configuration by number; not set = heuristic
    int variant = 0;
    if (int64_t t; tuned(kTuneGemmTile, t)) variant = (int)t;
    switch (variant) {
        case 61: return launch_f6<256, 256, 2, 4, 3, 1>(X6, xs, W6, ws, M, N, K, Y, ldy, out_i32, st);
        case 63: return launch_f6<256, 128, 2, 2, 2, 2>(X6, xs, W6, ws, M, N, K, Y, ldy, out_i32, st);
        case 64: return launch_f6<256, 256, 2, 4, 2, 1>(X6, xs, W6, ws, M, N, K, Y, ldy, out_i32, st);
        case 65: return launch_f6<256, 128, 4, 2, 4, 1, true>(X6, xs, W6, ws, M, N, K, Y, ldy, out_i32, st, warm, warm_bytes);
        case 66: return launch_f6<256, 128, 4, 2, 3, 1>(X6, xs, W6, ws, M, N, K, Y, ldy, out_i32, st);
        default: break;
    }
    // 256 x 256 tiles (eight waves of 128 x 64) run ~15 % faster per output than 256 x 128 tiles (eight waves of
    // 64 x 64: more LDS traffic per MFMA), so the small tile is taken only where it saves whole rounds:
    // measured at M = 2048, K = 4096: N = 14336 63.8 us against 77.6 us; N = 4096 (128 big tiles on 256 CUs)
    // 28.9 us against 24.3 us.  Four-wave workgroups (one wave per SIMD) lost everywhere.  N = 14336 at M = 2048 is
    // 448 big tiles = 1.75 rounds; a launch mixing one round of 256-wide with one round of 192-wide tiles (every CU
    // then works 1.75 tile times) was built and measured: 63.3 us against 61.9 us -- the second, three-quarters
    // filled round of the plain schedule already runs faster (fewer CUs draw power and share L2), so it was dropped.
    const int64_t cus = compute_units();
    const int64_t tm = (M + 255) / 256;
    auto rounds = [&](int64_t tiles) { return (tiles + cus - 1) / cus; };
    const int64_t cost_big = rounds(tm * ((N + 255) / 256)) * 256 * 256 * 85;
    const int64_t cost_small = rounds(tm * ((N + 127) / 128)) * 256 * 128 * 100;
    if (cost_big <= cost_small) return launch_f6<256, 256, 2, 4, 3, 1>(X6, xs, W6, ws, M, N, K, Y, ldy, out_i32, st);
    return launch_f6<256, 128, 4, 2, 4, 1, true>(X6, xs, W6, ws, M, N, K, Y, ldy, out_i32, st, warm, warm_bytes);
}

}  // namespace sr
