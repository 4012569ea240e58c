// INT4 x INT4 GEMM for M <= 16 tokens (decode): weight-streaming kernels.
//
// Same arithmetic as the compute-bound kernel (exact INT32 accumulation, dequantising
// epilogue; paper Eq. (1) and the quantised forward pass), but the cost is reading the
// packed weights once from HBM.  No scratch memory, no atomics: partial sums are integers,
// reduced on chip (order-free, exact).
//
//  M <= 2   gemm_decode_dot_kernel: v_dot8_i32_i4 multiplies eight packed 4-bit codes of W
//           with eight of X directly -- no widening at all.  Eight lanes read one whole
//           128-byte line of a weight row (measured: 5.7 us for the 29 MB of a 4096 x 14336
//           weight against 6.9 us when an instruction touches 16 rows x 64 bytes); a
//           workgroup owns 8..16 output channels, its waves take interleaved 128-byte slabs of K.
//           (The M dot products per weight dword make it lose to the MFMA kernel from 3 tokens on.)
//  M <= 16  gemm_decode_kernel: int8 MFMA 16x16x64 with operand rows re-interpreted so that
//           weights and activations are both loaded as whole lines (see the kernel).
#include "sr_common.h"

#include <hip/hip_fp16.h>

namespace sr {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

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
// MFMA kernel for up to 8 * SETS tokens, every load a whole 128-byte line per row.
// v_mfma_i32_16x16x64_i8 wants lane l to hold 16 bytes of operand row (l & 15); loading that
// layout directly touches 16 rows x 64 bytes per instruction, and the two half-line requests
// of a row are not merged on their way to L2 (three times the L2 requests of the data).  So
// an operand "row" i of the MFMA is used as (real row i & 7, K half i >> 3): lane
// (i = l & 15, g = l >> 4) loads the 16-byte chunk 4 (i >> 3) + g of row (i & 7) -- 8 rows x
// 128 bytes per instruction, for the weights and for the activations alike.  Of the 16 x 16
// products only the two diagonal 8 x 8 blocks (same K half on both sides) mean anything; the
// matrix pipe has time to spare here.  The result of (channel r, token t) is the sum of the
// accumulator entries [r][t] and [r + 8][t + 8], taken when the waves' partial sums are
// reduced through LDS.  G groups of 16 output channels share the activation fragments.
// ------------------------------------------------------------------------------------------
template <int NW, int G, int SETS, int UNR>
__global__ __launch_bounds__(NW * 64) void gemm_decode_kernel(const uint8_t *__restrict__ Xq, const float *__restrict__ xs,
                                                              const uint8_t *__restrict__ Wq, const float *__restrict__ ws,
                                                              int M, int N, int K, void *__restrict__ Yv, int64_t ldy,
                                                              int out_i32)
{
    constexpr int NA = 2 * G;                               // weight row sets of 8 channels
    __shared__ int red[NW][NA][SETS][4][16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r8 = lane & 7, kh = (lane >> 3) & 1, fg = lane >> 4;
    const int chunk = (4 * kh + fg) * 16;                   // byte offset of this lane's chunk inside a slab
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

    v4i acc[NA][SETS];
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int b = 0; b < SETS; ++b) acc[a][b] = v4i{0, 0, 0, 0};
    const u32x4 zero = {0u, 0u, 0u, 0u};

    for (int s0 = wave * UNR; s0 < nslab; s0 += NW * UNR) {
        u32x4 w[UNR][NA], x[UNR][SETS];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int off = (s0 + u) * SLAB;
            const bool ok = (s0 + u) < nslab && off + chunk < Kb;      // K % 256 != 0: the last slab is half empty
#pragma unroll
            for (int a = 0; a < NA; ++a)
                w[u][a] = ok ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wrow[a] + off)) : zero;
#pragma unroll
            for (int b = 0; b < SETS; ++b)
                x[u][b] = (ok && xok[b]) ? *reinterpret_cast<const u32x4 *>(xrow[b] + off) : zero;
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            v4i xa0[SETS], xa1[SETS];
#pragma unroll
            for (int b = 0; b < SETS; ++b) unpack16(x[u][b], xa0[b], xa1[b]);
#pragma unroll
            for (int a = 0; a < NA; ++a) {
                v4i wa0, wa1;
                unpack16(w[u][a], wa0, wa1);
#pragma unroll
                for (int b = 0; b < SETS; ++b) {
                    acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa0, xa0[b], acc[a][b], 0, 0, 0);
                    acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa1, xa1[b], acc[a][b], 0, 0, 0);
                }
            }
        }
    }

    // accumulator entry [i][j] sits in lane (j, i >> 2), register i & 3.  Output (channel 8 a + r, token 8 b + t)
    // = entries [r][t] + [r + 8][t + 8]: lane t + 16 (r >> 2) and the lane 40 above it.
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int b = 0; b < SETS; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int both = acc[a][b][v] + __shfl(acc[a][b][v], (lane + 40) & 63, 64);
                if (lane < 32 && !(lane & 8)) red[wave][a][b][v][(lane & 7) + 8 * (lane >> 4)] = both;
            }
    __syncthreads();
    for (int o = threadIdx.x; o < NA * SETS * 64; o += NW * 64) {
        const int t = o & 7, r = (o >> 3) & 7, ab = o >> 6, b = ab % SETS, a = ab / SETS;
        const int m = 8 * b + t, n = n0 + 8 * a + r;
        if (m >= M || n >= N) continue;
        int sum = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) sum += red[w][a][b][r & 3][t + 8 * (r >> 2)];
        sum >>= 8;                                         // both operands carried the factor 16
        if (out_i32) static_cast<int32_t *>(Yv)[(int64_t)m * ldy + n] = sum;
        else static_cast<__half *>(Yv)[(int64_t)m * ldy + n] = __float2half_rn((float)sum * xs[m] * ws[n]);
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
            v += __shfl_xor(v, 1, 64);
            v += __shfl_xor(v, 2, 64);
            v += __shfl_xor(v, 4, 64);
            if (c == 0) red[wave][m][g * 8 + r] = v;
        }
    __syncthreads();
    for (int t = threadIdx.x; t < MT * G * 8; t += NW * 64) {
        const int m = t / (G * 8), j = t % (G * 8), n = n0 + j;
        if (m >= M) continue;
        int sum = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) sum += red[w][m][j];
        if (out_i32) static_cast<int32_t *>(Yv)[(int64_t)m * ldy + n] = sum;
        else static_cast<__half *>(Yv)[(int64_t)m * ldy + n] = __float2half_rn((float)sum * xs[m] * ws[n]);
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

}  // namespace

hipError_t launch_gemm_decode(const uint8_t *Xq, const float *xs, const uint8_t *Wq, const float *ws,
                              int64_t M, int64_t N, int64_t K, void *Y, int64_t ldy, int out_i32, hipStream_t st)
{
    // measured (4096 -> 14336): dot kernel 6.2 / 7.1 / 8.4 us for M = 1 / 2 / 3, MFMA kernel 7.5 - 7.9 us for M <= 4
    if (M <= 1) return launch_dot<1, 4, 1>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);
    if (M <= 2) return launch_dot<2, 4, 2>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);
    // groups of 16 channels per workgroup: two (activation fragments shared) once there are many tokens and
    // still a few workgroups per CU
    const int64_t groups = N / 16;
    const int G = (M >= 8 && groups >= 800) ? 2 : 1;
    const unsigned blocks = (unsigned)((groups + G - 1) / G);
#define SR_DEC(NW, GG, SS, UU)                                                                                           \
    hipLaunchKernelGGL((gemm_decode_kernel<NW, GG, SS, UU>), dim3(blocks), dim3(NW * 64), 0, st, Xq, xs, Wq, ws, (int)M, \
                       (int)N, (int)K, Y, ldy, out_i32)
    // enough waves per workgroup that a wave has most of its K range in flight at once
    if (K >= 8192) {
        if (M <= 8) { if (G == 2) SR_DEC(8, 2, 1, 4); else SR_DEC(8, 1, 1, 4); }
        else { if (G == 2) SR_DEC(8, 2, 2, 2); else SR_DEC(8, 1, 2, 4); }
    } else {
        if (M <= 8) { if (G == 2) SR_DEC(4, 2, 1, 4); else SR_DEC(4, 1, 1, 4); }
        else { if (G == 2) SR_DEC(4, 2, 2, 2); else SR_DEC(4, 1, 2, 4); }
    }
#undef SR_DEC
    return hipGetLastError();
}

}  // namespace sr
