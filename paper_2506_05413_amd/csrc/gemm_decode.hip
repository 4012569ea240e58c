// INT4 x INT4 GEMM for M <= 16 tokens (decode): weight-streaming kernels.
//
// Same arithmetic as the compute-bound kernel (exact INT32 accumulation, dequantising
// epilogue; paper Eq. (1) and the quantised forward pass), but the cost is reading the
// packed weights once from HBM.  No scratch memory in global memory: partial sums are
// integers, reduced on chip through LDS (order-free, exact).
//
// What all three kernels share, each point measured on the 29 MB of a 4096 x 14336 weight:
//  * eight neighbouring lanes read one whole 128-byte line of a weight row (5.7 us against
//    6.9 us when an instruction touches 16 rows x 64 bytes: the memory pipe merges only what
//    neighbouring lanes ask for);
//  * every load of a wave is issued before the first one is used, unconditionally (a load
//    under a branch makes the compiler wait for all of them at once), non-temporal for W;
//  * nothing that waits on memory precedes the weight loads: a CU accepts loads only as fast
//    as earlier ones return, so the last load of a kernel is issued when most of the data has
//    already arrived, and whatever precedes the loads delays the whole stream;
//  * the dequantisation factors are fetched first and multiplied last.
//
//  M <= 2   gemm_decode_dot_kernel: v_dot8_i32_i4 multiplies eight packed 4-bit codes of W
//           with eight of X directly -- no widening at all.  A workgroup owns 8..16 output
//           channels, its waves take interleaved 128-byte slabs of K.  (One microsecond per
//           further token: it loses to the MFMA kernels from 3 tokens on.)
//  M <= 16  int8 MFMA 16x16x64 on codes widened to code * 16; lines are brought into operand
//           order through wave-private LDS buffers.
//           gemm_decode_kernel: a workgroup per 16 channels, activations re-read per workgroup.
//           gemm_decode_stream_kernel: one workgroup per CU, activations widened once and kept
//           in registers while the workgroup's weights stream past.
#include "gemm_common.h"


namespace sr {
namespace {

__device__ __forceinline__ void unpack16(const u32x4 w, v4i &a0, v4i &a1)
{
    constexpr unsigned HM = 0xF0F0F0F0u;     // nibble kept in the high half of its byte = code * 16
    a0[0] = (int)((w.x << 4) & HM); a0[1] = (int)(w.x & HM);
    a0[2] = (int)((w.y << 4) & HM); a0[3] = (int)(w.y & HM);
    a1[0] = (int)((w.z << 4) & HM); a1[1] = (int)(w.z & HM);
    a1[2] = (int)((w.w << 4) & HM); a1[3] = (int)(w.w & HM);
}

constexpr int SLAB = 128;    // packed bytes per row per slab (256 codes)

// ------------------------------------------------------------------------------------------
// MFMA kernel for up to 8 * SETS tokens.
// v_mfma_i32_16x16x64_i8 wants lane l to hold 16 bytes of operand row (l & 15); loading that
// layout directly touches 16 rows x 64 bytes per instruction, and the two half-line requests
// of a row are not merged on their way to L2 (three times the L2 requests of the data).  So
// an operand "row" i of the MFMA is used as (real row i & 7, K half i >> 3): a fragment is
// 8 rows x 128 bytes, lane (i = l & 15, g = l >> 4) holding the 16-byte chunk 4 (i >> 3) + g
// of row (i & 7), for the weights and for the activations alike.  Of the 16 x 16 products
// only the two diagonal 8 x 8 blocks (same K half on both sides) mean anything; the matrix
// pipe has time to spare here.  The result of (channel r, token t) is the sum of the
// accumulator entries [r][t] and [r + 8][t + 8], taken when the waves' partial sums are
// reduced through LDS.  G groups of 16 output channels share the activation fragments (the
// dispatcher uses G = 1: two groups measured slower once the loads were in line order).
//
// The loads themselves do NOT use the fragment's lane order (neighbouring lanes on different
// rows: measured 0.8 - 2.7 us slower per call, the memory pipe merges only what neighbouring
// lanes ask for).  Eight neighbouring lanes fetch one whole 128-byte line (lane 8 r + c:
// chunk c of row r); each 1 KB piece is then written to a wave-private LDS buffer and read
// back in fragment order.  A staged row is 144 bytes apart from the next, so the eight rows
// that one chunk index touches fall on distinct banks.  No workgroup barrier is involved: a
// wave's LDS accesses execute in program order.
// ------------------------------------------------------------------------------------------
template <int NW, int G, int SETS, int UNR>
__global__ __launch_bounds__(NW * 64) void gemm_decode_kernel(const uint8_t *__restrict__ Xq, const float *__restrict__ xs,
                                                              const uint8_t *__restrict__ Wq, const float *__restrict__ ws,
                                                              int M, int N, int K, void *__restrict__ Yv, int64_t ldy,
                                                              int out_i32)
{
    constexpr int NA = 2 * G;                               // weight row sets of 8 channels
    constexpr int XROW = 144;                               // bytes from one staged row to the next
    __shared__ int red[NW][2][NA][SETS][4][16];
    __shared__ __attribute__((aligned(16))) uint8_t stage[NW][NA + SETS][8 * XROW];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r8 = lane >> 3, chunk = (lane & 7) * 16;      // load order: row of the set, byte offset inside a slab
    uint8_t *const st_put = &stage[wave][0][0] + r8 * XROW + chunk;
    // fragment order: lane (i = l & 15, g = l >> 4) takes chunk 4 (i >> 3) + g of row i & 7
    const uint8_t *const st_get = &stage[wave][0][0] + (lane & 7) * XROW + (4 * ((lane >> 3) & 1) + (lane >> 4)) * 16;
    const int n0 = blockIdx.x * (16 * G);
    const int Kb = K >> 1;
    const int nslab = (Kb + SLAB - 1) / SLAB;

    const uint8_t *wrow[NA];
#pragma unroll
    for (int a = 0; a < NA; ++a) {
        int n = n0 + 8 * a + r8;
        n = n < N ? n : N - 1;                             // a ragged last workgroup re-reads the last row
        wrow[a] = Wq + (int64_t)n * Kb + chunk;
    }
    const uint8_t *xrow[SETS];
    bool xok[SETS];
#pragma unroll
    for (int b = 0; b < SETS; ++b) {
        xok[b] = 8 * b + r8 < M;
        xrow[b] = Xq + (int64_t)(xok[b] ? 8 * b + r8 : 0) * Kb + chunk;
    }

    // Output o of the workgroup = (token o / (16 G), channel o % (16 G)).  Its dequantisation factors are fetched
    // now (a load issued after the reduction would put one more memory latency at the end of every workgroup)
    // and multiplied only at the end (a product taken here would make the wave wait before its weight loads).
    constexpr int NOUT = NA * SETS * 64, PER = (NOUT + NW * 64 - 1) / (NW * 64);
    float fx[PER], fw[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int o = threadIdx.x + k * NW * 64, m = o / (16 * G), n = n0 + o % (16 * G);
        const bool valid = !out_i32 && o < NOUT && m < M && n < N;
        fx[k] = valid ? xs[m] : 0.f;
        fw[k] = valid ? ws[n] : 0.f;
    }

    v4i acc[NA][SETS];
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int b = 0; b < SETS; ++b) acc[a][b] = v4i{0, 0, 0, 0};
    const u32x4 zero = {0u, 0u, 0u, 0u};

    for (int s0 = wave * UNR; s0 < nslab; s0 += NW * UNR) {
        // Every load is issued unconditionally (so that the waits below can count them): a lane whose chunk lies
        // beyond K re-reads the first bytes of its row, and its activation fragment is cleared instead.
        u32x4 w[UNR][NA], x[UNR][SETS];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const bool ok = (s0 + u) < nslab && (s0 + u) * SLAB + chunk < Kb;  // K % 256 != 0: the last slab is half empty
            const int off = ok ? (s0 + u) * SLAB : -chunk;
#pragma unroll
            for (int a = 0; a < NA; ++a)
                w[u][a] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wrow[a] + off));
#pragma unroll
            for (int b = 0; b < SETS; ++b) {
                x[u][b] = *reinterpret_cast<const u32x4 *>(xrow[b] + off);
                if (!(ok && xok[b])) x[u][b] = zero;
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            // load order -> fragment order through the wave's staging buffers
#pragma unroll
            for (int a = 0; a < NA; ++a) *reinterpret_cast<u32x4 *>(st_put + a * 8 * XROW) = w[u][a];
#pragma unroll
            for (int b = 0; b < SETS; ++b) *reinterpret_cast<u32x4 *>(st_put + (NA + b) * 8 * XROW) = x[u][b];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            u32x4 wf[NA], xf[SETS];
#pragma unroll
            for (int a = 0; a < NA; ++a) wf[a] = *reinterpret_cast<const u32x4 *>(st_get + a * 8 * XROW);
#pragma unroll
            for (int b = 0; b < SETS; ++b) xf[b] = *reinterpret_cast<const u32x4 *>(st_get + (NA + b) * 8 * XROW);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            v4i xa0[SETS], xa1[SETS];
#pragma unroll
            for (int b = 0; b < SETS; ++b) unpack16(xf[b], xa0[b], xa1[b]);
#pragma unroll
            for (int a = 0; a < NA; ++a) {
                v4i wa0, wa1;
                unpack16(wf[a], wa0, wa1);
#pragma unroll
                for (int b = 0; b < SETS; ++b) {
                    acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa0, xa0[b], acc[a][b], 0, 0, 0);
                    acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa1, xa1[b], acc[a][b], 0, 0, 0);
                }
            }
        }
    }

    // accumulator entry [i][j] sits in lane (j, i >> 2), register i & 3.  Output (channel 8 a + r, token 8 b + t)
    // = entries [r][t] + [r + 8][t + 8]: lane t + 16 (r >> 2) and the lane 40 above it.  Both halves go to LDS
    // as they are (no lane exchange) and are added with the waves' partial sums.
    {
        const int half = lane >> 5, l2 = lane - 40 * half;             // upper half: lanes 40..47, 56..63 -> 0..7, 16..23
        const bool holds = half ? (lane & 8) != 0 : (lane & 8) == 0;
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
            for (int b = 0; b < SETS; ++b)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (holds) red[wave][half][a][b][v][(l2 & 7) + 8 * (l2 >> 4)] = acc[a][b][v];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int o = threadIdx.x + k * NW * 64;
        const int m = o / (16 * G), nn = o % (16 * G), n = n0 + nn;
        if (o >= NOUT || m >= M || n >= N) continue;
        const int t = m & 7, b = m >> 3, r = nn & 7, a = nn >> 3;
        int sum = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) sum += red[w][0][a][b][r & 3][t + 8 * (r >> 2)] + red[w][1][a][b][r & 3][t + 8 * (r >> 2)];
        sum >>= 8;                                         // both operands carried the factor 16
        if (out_i32) static_cast<int32_t *>(Yv)[(int64_t)m * ldy + n] = sum;
        else static_cast<__half *>(Yv)[(int64_t)m * ldy + n] = __float2half_rn((float)sum * fx[k] * fw[k]);
    }
}

// ------------------------------------------------------------------------------------------
// Streaming MFMA kernel for 3 .. 16 tokens: the activations are widened once per workgroup.
// One workgroup of 16 waves per CU.  A wave owns SPW slabs of K (slab sb0 + 16 i + wave) and
// keeps their activation fragments, already widened to int8, in registers; the workgroup owns
// UPW "units" of 8 output channels per pass, and a wave's whole share of their weights
// (UPW x SPW loads of 1 KB, eight neighbouring lanes per 128-byte line) is in flight at once.
// Two units at a time go through the wave's two LDS staging buffers and come back as ONE
// ordinary operand of v_mfma_i32_16x16x64_i8 (operand row i = channel i & 7 of unit i >> 3,
// lane group g = 16-byte chunk 4 h + g of the slab, h = 0, 1), are widened, and meet the
// resident activation fragments (row = token) in the matrix pipe: every entry of the 16 x 16
// product is used.  Per weight load this leaves 12 vector-ALU instructions and no activation
// traffic at all, where the kernel above re-reads and re-widens the activations in every
// workgroup.  Every wave leaves its integer partial sums in LDS as they are (16 bytes per lane)
// and the first waves add the 16 copies (exact, order-free; measured against ds_add into one
// copy: 8.1 -> 7.9 us at 16 tokens, and nothing to clear).
// Units of one 128-byte output line go to workgroups of the same XCD (blockIdx & 7), so that
// a line of Y is assembled in one L2.
// ------------------------------------------------------------------------------------------
template <int SPW, int UPW>
__global__ __launch_bounds__(1024) void gemm_decode_stream_kernel(const uint8_t *__restrict__ Xq, const float *__restrict__ xs,
                                                                   const uint8_t *__restrict__ Wq, const float *__restrict__ ws,
                                                                   int M, int N, int K, void *__restrict__ Yv, int64_t ldy,
                                                                   int out_i32)
{
    constexpr int NW = 16, XROW = 144, PAIRS = (UPW + 1) / 2;
    static_assert(UPW <= 8, "one output per thread and pass");
    extern __shared__ __attribute__((aligned(16))) v4i red[];          // [NW][PAIRS][64]: a wave's accumulators as they are
    __shared__ __attribute__((aligned(16))) uint8_t stage[NW][2][8 * XROW];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r8 = lane >> 3, chunk = (lane & 7) * 16;      // load order: row of the piece, byte offset inside a slab
    uint8_t *const st_put = &stage[wave][0][0] + r8 * XROW + chunk;
    // fragment order: lane (i = l & 15, g = l >> 4) takes chunk 4 h + g of row i & 7 of piece i >> 3
    const uint8_t *const st_get = &stage[wave][(lane >> 3) & 1][0] + (lane & 7) * XROW + (lane >> 4) * 16;
    const int Kb = K >> 1, nslab = (Kb + SLAB - 1) / SLAB, units = N >> 3;
    const int xcd = blockIdx.x & 7, wg = blockIdx.x >> 3, WGX = gridDim.x >> 3;
    const u32x4 zero = {0u, 0u, 0u, 0u};
    // e-th unit of this XCD: output lines (8 units each) are dealt to the XCDs in turn
    auto unit_of = [xcd](int e) { return ((e >> 3) * 8 + xcd) * 8 + (e & 7); };
    // two pieces in load order -> the two K halves of one operand in fragment order, widened
    auto to_fragments = [&](const u32x4 p0, const u32x4 p1, v4i (&f)[2][2]) {
        *reinterpret_cast<u32x4 *>(st_put) = p0;
        *reinterpret_cast<u32x4 *>(st_put + 8 * XROW) = p1;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const u32x4 h0 = *reinterpret_cast<const u32x4 *>(st_get);
        const u32x4 h1 = *reinterpret_cast<const u32x4 *>(st_get + 64);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        unpack16(h0, f[0][0], f[0][1]);
        unpack16(h1, f[1][0], f[1][1]);
    };
    // Outputs of a pass: thread (q = t >> 6, l = t & 63) of the first PAIRS waves adds the 16 waves' copies of
    // accumulator lane l of pair q.  Entry [i][tok] (operand row i, token tok) sits in lane tok + 16 (i >> 2),
    // register i & 3: the thread owns token l & 15 and the four channels 4 ((l >> 4) & 1) .. + 3 of unit slot
    // 2 q + (l >> 5).
    const int oq = threadIdx.x >> 6, om = lane & 15, oj = 2 * oq + (lane >> 5), orow = 4 * ((lane >> 4) & 1);

    for (int e0 = wg; unit_of(e0) < units; e0 += WGX * UPW) {
        const int ou = unit_of(e0 + oj * WGX), on = 8 * ou + orow;
        const bool ovalid = oq < PAIRS && oj < UPW && om < M && ou < units;
        // dequantisation factors, fetched ahead of the weights and multiplied only at the end (a product taken
        // here would make the wave wait for them before it issues its weight loads)
        const float fx = (ovalid && !out_i32) ? xs[om] : 0.f;
        const float4 fw = (ovalid && !out_i32) ? *reinterpret_cast<const float4 *>(ws + on) : make_float4(0.f, 0.f, 0.f, 0.f);

        const uint8_t *wrow[UPW];
#pragma unroll
        for (int j = 0; j < UPW; ++j) {
            const int u = unit_of(e0 + j * WGX);
            const int n = u < units ? 8 * u + r8 : N - 1;  // a missing unit re-reads the last row; its sums are dropped
            wrow[j] = Wq + (int64_t)n * Kb + chunk;
        }
        v4i acc[PAIRS];
#pragma unroll
        for (int q = 0; q < PAIRS; ++q) acc[q] = v4i{0, 0, 0, 0};

        for (int sb0 = 0; sb0 < nslab; sb0 += NW * SPW) {
            // Every load is unconditional (the compiler then counts them in its waits): a lane whose chunk lies
            // beyond K re-reads the first bytes of its row, and its activation chunk is cleared instead.
            u32x4 x[SPW][2], w[PAIRS * 2][SPW];
            int off[SPW];
#pragma unroll
            for (int i = 0; i < SPW; ++i) {
                const int sl = sb0 + i * NW + wave;
                const bool ok = sl < nslab && sl * SLAB + chunk < Kb;
                off[i] = ok ? sl * SLAB : -chunk;
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    const int m = 8 * b + r8;
                    x[i][b] = *reinterpret_cast<const u32x4 *>(Xq + (int64_t)(m < M ? m : 0) * Kb + chunk + off[i]);
                    if (!(ok && m < M)) x[i][b] = zero;
                }
            }
#pragma unroll
            for (int j = 0; j < PAIRS * 2; ++j)
#pragma unroll
                for (int i = 0; i < SPW; ++i)
                    w[j][i] = j < UPW ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wrow[j < UPW ? j : 0] + off[i])) : zero;

            v4i xa[SPW][2][2];
#pragma unroll
            for (int i = 0; i < SPW; ++i) to_fragments(x[i][0], x[i][1], xa[i]);
#pragma unroll
            for (int q = 0; q < PAIRS; ++q)
#pragma unroll
                for (int i = 0; i < SPW; ++i) {
                    v4i wa[2][2];
                    to_fragments(w[2 * q][i], w[2 * q + 1][i], wa);
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        acc[q] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa[h][0], xa[i][h][0], acc[q], 0, 0, 0);
                        acc[q] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa[h][1], xa[i][h][1], acc[q], 0, 0, 0);
                    }
                }
        }

        // every wave leaves its accumulators in LDS as they are (16 bytes per lane and pair, no atomics, nothing
        // to clear); the outputs are summed by the first PAIRS waves
#pragma unroll
        for (int q = 0; q < PAIRS; ++q) red[(wave * PAIRS + q) * 64 + lane] = acc[q];
        __syncthreads();
        if (ovalid) {
            v4i sum = red[oq * 64 + lane];
#pragma unroll
            for (int w = 1; w < NW; ++w) sum += red[(w * PAIRS + oq) * 64 + lane];
            sum >>= 8;                                      // both operands carried the factor 16
            if (out_i32) {
                *reinterpret_cast<v4i *>(static_cast<int32_t *>(Yv) + (int64_t)om * ldy + on) = sum;
            } else {
                union { __half h[4]; uint2 u; } o;
                o.h[0] = __float2half_rn((float)sum[0] * fx * fw.x);
                o.h[1] = __float2half_rn((float)sum[1] * fx * fw.y);
                o.h[2] = __float2half_rn((float)sum[2] * fx * fw.z);
                o.h[3] = __float2half_rn((float)sum[3] * fx * fw.w);
                *reinterpret_cast<uint2 *>(static_cast<__half *>(Yv) + (int64_t)om * ldy + on) = o.u;
            }
        }
        __syncthreads();                                    // red[] is written again by the next pass
    }
}

// ------------------------------------------------------------------------------------------
// Dot-product kernel for M <= MT tokens.  lane -> (row r = l >> 3 of an 8-row group, chunk
// c = l & 7 of a 128-byte slab).  A workgroup owns G consecutive 8-row groups; a wave loads the
// X chunks of its slabs once and reuses them for all G groups, so X costs M / G loads per
// weight load.  NW waves take interleaved slabs, U slabs at a time.
// ------------------------------------------------------------------------------------------
template <int MT, int NW, int U, int G>
__global__ __launch_bounds__(NW * 64) void gemm_decode_dot_kernel(const uint8_t *__restrict__ Xq, const float *__restrict__ xs,
                                                                  const uint8_t *__restrict__ Wq, const float *__restrict__ ws,
                                                                  int M, int N, int K, void *__restrict__ Yv, int64_t ldy,
                                                                  int out_i32)
{
    __shared__ int red[NW][MT][G * 8];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane >> 3, c = lane & 7;
    const int n0 = blockIdx.x * (8 * G);
    const int Kb = K >> 1;
    const int nslab = (Kb + SLAB - 1) / SLAB;
    const uint8_t *wp = Wq + (int64_t)(n0 + r) * Kb + c * 16;
    const uint8_t *xp = Xq + c * 16;
    const u32x4 zero = {0u, 0u, 0u, 0u};

    // the dequantisation factors of this thread's output (token t / (8 G), channel t % (8 G)), fetched ahead of
    // the weights so that their latency does not follow the reduction, multiplied only at the end
    static_assert(MT * G * 8 <= NW * 64, "one output per thread at most");
    float fx = 0.f, fw = 0.f;
    {
        const int m = threadIdx.x / (G * 8), n = n0 + threadIdx.x % (G * 8);
        if (!out_i32 && m < MT && m < M && n < N) { fx = xs[m]; fw = ws[n]; }
    }

    int acc[G][MT];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[g][m] = 0;

    for (int s0 = wave; s0 < nslab; s0 += NW * U) {
        u32x4 w[G][U], x[U][MT];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int off = (s0 + NW * u) * SLAB;
            const bool ok = (s0 + NW * u) < nslab && off + c * 16 < Kb;
#pragma unroll
            for (int g = 0; g < G; ++g)
                w[g][u] = ok ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wp + (int64_t)g * 8 * Kb + off)) : zero;
#pragma unroll
            for (int m = 0; m < MT; ++m)
                x[u][m] = (ok && m < M) ? *reinterpret_cast<const u32x4 *>(xp + (int64_t)m * Kb + off) : zero;
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int m = 0; m < MT; ++m) {
                    int a = acc[g][m];
                    a = __builtin_amdgcn_sdot8((int)w[g][u].x, (int)x[u][m].x, a, false);
                    a = __builtin_amdgcn_sdot8((int)w[g][u].y, (int)x[u][m].y, a, false);
                    a = __builtin_amdgcn_sdot8((int)w[g][u].z, (int)x[u][m].z, a, false);
                    a = __builtin_amdgcn_sdot8((int)w[g][u].w, (int)x[u][m].w, a, false);
                    acc[g][m] = a;
                }
    }
    // the 8 lanes of a row, then the waves
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            int v = acc[g][m];
            v = sum_of_8_lanes(v);
            if (c == 0) red[wave][m][g * 8 + r] = v;
        }
    __syncthreads();
    if (const int t = threadIdx.x; t < MT * G * 8) {
        const int m = t / (G * 8), j = t % (G * 8), n = n0 + j;
        if (m < M && n < N) {
            int sum = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) sum += red[w][m][j];
            if (out_i32) static_cast<int32_t *>(Yv)[(int64_t)m * ldy + n] = sum;
            else static_cast<__half *>(Yv)[(int64_t)m * ldy + n] = __float2half_rn((float)sum * fx * fw);
        }
    }
}

template <int MT, int U, int G>
hipError_t launch_dot(const uint8_t *Xq, const float *xs, const uint8_t *Wq, const float *ws, int64_t M, int64_t N,
                      int64_t K, void *Y, int64_t ldy, int out_i32, hipStream_t st)
{
    if (N % (8 * G) != 0) {                              // N % 16 == 0 is guaranteed: fall back to 2 groups
        if constexpr (G > 2) return launch_dot<MT, U, 2>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);
    }
    const unsigned blocks = (unsigned)(N / (8 * G));
    const int nslab = (int)((K / 2 + SLAB - 1) / SLAB);
    // more waves per workgroup for long rows, so that every CU keeps ~100 KB of weights in flight
    if (nslab >= 32)
        hipLaunchKernelGGL((gemm_decode_dot_kernel<MT, 8, U, G>), dim3(blocks), dim3(512), 0, st, Xq, xs, Wq, ws,
                           (int)M, (int)N, (int)K, Y, ldy, out_i32);
    else
        hipLaunchKernelGGL((gemm_decode_dot_kernel<MT, 4, U, G>), dim3(blocks), dim3(256), 0, st, Xq, xs, Wq, ws,
                           (int)M, (int)N, (int)K, Y, ldy, out_i32);
    return hipGetLastError();
}

template <int SPW, int UPW>
hipError_t launch_stream(const uint8_t *Xq, const float *xs, const uint8_t *Wq, const float *ws, int64_t M, int64_t N,
                         int64_t K, void *Y, int64_t ldy, int out_i32, int wgx, hipStream_t st)
{
    auto kern = gemm_decode_stream_kernel<SPW, UPW>;
    constexpr int lds = 16 * ((UPW + 1) / 2) * 64 * 16;               // the waves' accumulators
    // with the 36 KB of static staging buffers the workgroup needs up to 100 KB of LDS
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(8 * wgx), dim3(1024), lds, st, Xq, xs, Wq, ws, (int)M, (int)N, (int)K, Y, ldy, out_i32);
    return hipGetLastError();
}

// one workgroup per CU, 8 XCDs; the units a workgroup takes per pass are bounded by the loads a wave keeps in flight
hipError_t launch_stream_any(const uint8_t *Xq, const float *xs, const uint8_t *Wq, const float *ws, int64_t M, int64_t N,
                             int64_t K, void *Y, int64_t ldy, int out_i32, hipStream_t st)
{
    const int wgx = compute_units() >= 8 ? compute_units() / 8 : 1;
    const int nslab = (int)((K / 2 + SLAB - 1) / SLAB);
    const int64_t lines = (N / 8 + 7) / 8, per_xcd = 8 * ((lines + 7) / 8);
    const int need = (int)((per_xcd + wgx - 1) / wgx);
    const int spw = nslab <= 16 ? 1 : 2;                  // more slabs per wave would not fit the register file
    const int cap = spw == 1 ? 8 : 3;
    const int upw = need < cap ? need : cap;
#define SR_STREAM(S, U) if (spw == S && upw == U) return launch_stream<S, U>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, wgx, st)
    SR_STREAM(1, 1); SR_STREAM(1, 2); SR_STREAM(1, 3); SR_STREAM(1, 4); SR_STREAM(1, 5); SR_STREAM(1, 6); SR_STREAM(1, 7); SR_STREAM(1, 8);
    SR_STREAM(2, 1); SR_STREAM(2, 2); SR_STREAM(2, 3);
#undef SR_STREAM
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_gemm_decode(const uint8_t *Xq, const float *xs, const uint8_t *Wq, const float *ws,
                              int64_t M, int64_t N, int64_t K, void *Y, int64_t ldy, int out_i32, hipStream_t st)
{
    // the decode-kernel knob = 1 (dot, M <= 2 only), 2 (MFMA, workgroup per 16 channels) or 3 (streaming MFMA)
    // forces a kernel (tuning and test aid); not set = the choice measured below.
    int force = 0;
    if (int64_t f; tuned(kTuneDecodeKernel, f)) force = (int)f;
    const int nslab = (int)((K / 2 + SLAB - 1) / SLAB);

    // measured (4096 -> 14336): dot kernel 6.2 / 7.0 us for M = 1 / 2 (one more microsecond per further token),
    // MFMA kernels 7.0 - 7.2 us for 3 .. 8 tokens
    if (force == 1 ? M <= 2 : (force == 0 && M <= 2)) {
        if (M <= 1) return launch_dot<1, 4, 1>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);
        return launch_dot<2, 4, 2>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);
    }
    // The streaming kernel wins where every one of its 16 waves has a slab of K (K >= 4096) and a wave can keep
    // its whole share of K in registers (K <= 8192), except with few tokens and so many channels that a workgroup
    // per 16 channels fills the chip several times over (4096 -> 14336: 6.7 against 7.7 us for M <= 8; at 16
    // tokens 8.2 against 7.9 us the other way round).  Shorter rows leave waves idle (1024 -> 14336 at 16 tokens:
    // 6.0 against 4.5 us).
    const bool few_tokens_many_channels = M <= 8 && nslab <= 16 && N >= 8192;
    if (force == 3 || (force == 0 && nslab >= 16 && nslab <= 32 && !few_tokens_many_channels))
        return launch_stream_any(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);

    const unsigned blocks = (unsigned)(N / 16);
#define SR_DEC(NW, SS, UU)                                                                                               \
    hipLaunchKernelGGL((gemm_decode_kernel<NW, 1, SS, UU>), dim3(blocks), dim3(NW * 64), 0, st, Xq, xs, Wq, ws, (int)M, \
                       (int)N, (int)K, Y, ldy, out_i32)
    // long rows: more waves per workgroup, so that a wave has most of its K range in flight at once
    if (nslab > 16) {
        if (M <= 8) SR_DEC(8, 1, 4); else SR_DEC(8, 2, 2);
    } else {
        if (M <= 8) SR_DEC(4, 1, 2); else SR_DEC(4, 2, 1);
    }
#undef SR_DEC
    return hipGetLastError();
}

}  // namespace sr
