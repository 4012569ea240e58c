// INT4 x INT4 GEMM, INT32 accumulation, dequantising epilogue -- compute-bound shapes.
//
//   acc[m][n] = sum_k cX[m][k] * cW[n][k],   Y = fp16(acc * dx[m] * dw[n])
//
// (Paper: the quantised forward pass of the linear layer; dequantisation per Eq. (1).)
//
// There is no 4-bit matrix instruction on gfx950, so the packed nibbles are widened
// to int8 in registers and fed to v_mfma_i32_16x16x64_i8.  A nibble is sign-extended
// for free by leaving it in the HIGH half of its byte:
//     lo = (w << 4) & 0xF0F0F0F0      (codes 0,2,4,6 of the dword, each x16)
//     hi =  w       & 0xF0F0F0F0      (codes 1,3,5,7 of the dword, each x16)
// Both operands are scaled by 16, so the accumulator holds 256 * acc exactly
// (|256 * acc| <= 256 * 64 * K < 2^31 for K < 131072); the factor is removed by an
// arithmetic shift (int32 output) or folded into the row scale (fp16 output).
// A dot product does not care in which order k is visited, so X and W only have to
// permute k identically -- which they do, because both are unpacked by the same code
// from the same byte offsets.
//
// Tiling: 256 threads = 4 waves (2 x 2), block tile BM x BN, wave tile (BM/2) x (BN/2)
// built from 16 x 16 MFMA tiles, K step of 128 codes (64 packed bytes per row).
// Global -> registers -> LDS double buffering; LDS rows are 64 bytes with the 16-byte
// chunk index XOR-swizzled by (row >> 2) & 3 so that both the 16-byte stores and the
// 16-byte fragment loads are bank-conflict free.
//
// MFMA operand roles are swapped (A operand = weight rows, B operand = token rows):
// a lane then owns 4 consecutive output channels of one token, i.e. one 8-byte store.
#include "sr_common.h"

#include <hip/hip_fp16.h>

namespace sr {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int KB = 64;   // packed bytes of one K step per row (128 codes)

__device__ __forceinline__ int swz_off(int row, int chunk)
{
    return row * KB + ((chunk ^ ((row >> 2) & 3)) << 4);
}

__device__ __forceinline__ void unpack16(const uint4 w, v4i &a0, v4i &a1)
{
    constexpr unsigned HM = 0xF0F0F0F0u;
    a0[0] = (int)((w.x << 4) & HM); a0[1] = (int)(w.x & HM);
    a0[2] = (int)((w.y << 4) & HM); a0[3] = (int)(w.y & HM);
    a1[0] = (int)((w.z << 4) & HM); a1[1] = (int)(w.z & HM);
    a1[2] = (int)((w.w << 4) & HM); a1[3] = (int)(w.w & HM);
}

template <int BM, int BN>
__global__ __launch_bounds__(256) void gemm_w4a4_kernel(const uint8_t *__restrict__ Xq, const float *__restrict__ xs,
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
    constexpr int BM = 128, BN = 128;
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((N + BN - 1) / BN);
    hipLaunchKernelGGL((gemm_w4a4_kernel<BM, BN>), dim3((unsigned)(tiles_m * tiles_n)), dim3(256), 0, st,
                       Xq, xs, Wq, ws, (int)M, (int)N, (int)K, Y, ldy, out_i32, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace sr
