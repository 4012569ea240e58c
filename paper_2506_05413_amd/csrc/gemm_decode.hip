// INT4 x INT4 GEMM for M <= 16 tokens (decode): weight-streaming kernels.
//
// Same arithmetic as the compute-bound kernel (exact INT32 accumulation, dequantising
// epilogue; paper Eq. (1) and the quantised forward pass), but the cost is reading the
// packed weights once from HBM.  No scratch memory, no atomics: partial sums are integers,
// reduced on chip (order-free, exact).
//
//  M <= 4   gemm_decode_dot_kernel: v_dot8_i32_i4 multiplies eight packed 4-bit codes of W
//           with eight of X directly -- no widening at all.  Eight lanes read one whole
//           128-byte line of a weight row (measured: 5.7 us for the 29 MB of a 4096 x 14336
//           weight against 6.9 us when an instruction touches 16 rows x 64 bytes); a
//           workgroup owns 8..32 output channels, its waves take interleaved 128-byte slabs of K.
//           (Beyond 4 tokens the M dot products per weight dword cost more than the MFMA path.)
//  M <= 16  gemm_decode_kernel: one workgroup owns 16 output channels; its waves split K,
//           issue all their 16-byte weight loads up front and multiply on the int8 MFMA with
//           the <= 16 token rows as the second operand (the MFMA needs lane = row mod 16,
//           hence the 64-byte pieces).
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
constexpr int UNR = 4;       // slabs in flight per wave iteration

template <int NW>
__global__ __launch_bounds__(NW * 64) void gemm_decode_kernel(const uint8_t *__restrict__ Xq, const float *__restrict__ xs,
                                                              const uint8_t *__restrict__ Wq, const float *__restrict__ ws,
                                                              int M, int N, int K, void *__restrict__ Yv, int64_t ldy,
                                                              int out_i32)
{
    __shared__ int red[NW][4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int fr = lane & 15, fg = lane >> 4;
    const int n0 = blockIdx.x * 16;
    const int Kb = K >> 1;
    const int nslab = (Kb + SLAB - 1) / SLAB;

    const uint8_t *wrow = Wq + (int64_t)(n0 + fr) * Kb + fg * 16;
    const bool xrow_ok = fr < M;
    const uint8_t *xrow = Xq + (int64_t)(xrow_ok ? fr : 0) * Kb + fg * 16;

    v4i acc = {0, 0, 0, 0};
    const u32x4 zero = {0u, 0u, 0u, 0u};

    for (int s0 = wave * UNR; s0 < nslab; s0 += NW * UNR) {
        u32x4 w[UNR][2], x[UNR][2];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int off = (s0 + u) * SLAB + h * 64;          // byte offset of this lane's chunk - fg*16
                const bool ok = (s0 + u) < nslab && off + fg * 16 < Kb;
                w[u][h] = ok ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wrow + off)) : zero;
                x[u][h] = (ok && xrow_ok) ? *reinterpret_cast<const u32x4 *>(xrow + off) : zero;
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                v4i wa0, wa1, xa0, xa1;
                unpack16(w[u][h], wa0, wa1);
                unpack16(x[u][h], xa0, xa1);
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa0, xa0, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa1, xa1, acc, 0, 0, 0);
            }
        }
    }

#pragma unroll
    for (int v = 0; v < 4; ++v) red[wave][v][lane] = acc[v];
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        int s = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += red[w][v][lane];
        acc[v] = s;
    }
    // lane owns token m = fr, output channels n0 + 4*fg .. +3
    const int m = fr, n = n0 + fg * 4;
    if (m >= M) return;
    if (out_i32) {
        *reinterpret_cast<int4 *>(static_cast<int32_t *>(Yv) + (int64_t)m * ldy + n) =
            make_int4(acc[0] >> 8, acc[1] >> 8, acc[2] >> 8, acc[3] >> 8);
    } else {
        const float sx = xs[m] * (1.f / 256.f);
        const float4 sw = *reinterpret_cast<const float4 *>(ws + n);
        union { __half h[4]; uint2 u; } o;
        o.h[0] = __float2half_rn((float)acc[0] * sx * sw.x);
        o.h[1] = __float2half_rn((float)acc[1] * sx * sw.y);
        o.h[2] = __float2half_rn((float)acc[2] * sx * sw.z);
        o.h[3] = __float2half_rn((float)acc[3] * sx * sw.w);
        *reinterpret_cast<uint2 *>(static_cast<__half *>(Yv) + (int64_t)m * ldy + n) = o.u;
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
    if (M <= 1) return launch_dot<1, 4, 1>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);
    if (M <= 2) return launch_dot<2, 4, 2>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);
    if (M <= 4) {
        // row groups per workgroup: reuse of the X chunks against enough workgroups to fill 256 CUs
        if (N >= 32 * 400) return launch_dot<4, 2, 4>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);
        if (N >= 16 * 400) return launch_dot<4, 4, 2>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);
        return launch_dot<4, 4, 1>(Xq, xs, Wq, ws, M, N, K, Y, ldy, out_i32, st);
    }
    const unsigned blocks = (unsigned)(N / 16);
    // enough waves per block that a wave streams ~2 KB of its 16 rows' K range at once
    if (K >= 8192)
        hipLaunchKernelGGL(gemm_decode_kernel<8>, dim3(blocks), dim3(512), 0, st, Xq, xs, Wq, ws, (int)M, (int)N,
                           (int)K, Y, ldy, out_i32);
    else
        hipLaunchKernelGGL(gemm_decode_kernel<4>, dim3(blocks), dim3(256), 0, st, Xq, xs, Wq, ws, (int)M, (int)N,
                           (int)K, Y, ldy, out_i32);
    return hipGetLastError();
}

}  // namespace sr
