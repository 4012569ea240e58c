// Offline helpers: calibration absmax, smoothing factors, and the fp16 transpose (which also collects the weight's
// row maxima) that turns the weight fold into a row-wise rotation + quantisation.
// (Paper, section "Methodology": s_j = max|X_j|^alpha / max|W_j|^(1-alpha), calibrated
// offline; Lambda = diag(s) goes into the weights.)
#include "sr_common.h"

#include <hip/hip_fp16.h>

namespace sr {
namespace {

typedef unsigned short us8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ us8 abs_bits(uint4 v)
{
    v.x &= 0x7FFF7FFFu; v.y &= 0x7FFF7FFFu; v.z &= 0x7FFF7FFFu; v.w &= 0x7FFF7FFFu;
    union { uint4 u; us8 s; } c;
    c.u = v;
    return c.s;
}

__device__ __forceinline__ float half_bits_to_float(unsigned short b)
{
    return __half2float(__ushort_as_half(b));
}

// Column-wise max |x| over a slab of rows.  |fp16| bit patterns of finite values order
// like unsigned integers, so the running maximum is kept as packed u16 and is exact.
// Block = CG column groups (8 columns each: CG * 16 contiguous bytes per row) x 256 / CG row lanes.
// Narrow, tall blocks keep the number of atomics per channel small: the atomics on the K shared
// addresses, not the reads, were what bounded a wide-block version.
template <int CG>
__global__ __launch_bounds__(256) void calib_absmax_kernel(const __half *__restrict__ X, int64_t T, int K,
                                                            int64_t ldx, float *__restrict__ absmax,
                                                            int64_t rows_per_block)
{
    constexpr int RL = 256 / CG;                         // row lanes
    __shared__ us8 part[RL][CG];
    const int tx = threadIdx.x % CG, ty = threadIdx.x / CG;
    const int col = (blockIdx.x * CG + tx) * 8;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
    const int64_t r1 = (r0 + rows_per_block < T) ? r0 + rows_per_block : T;
    us8 acc = {0, 0, 0, 0, 0, 0, 0, 0};
    if (col < K) {
        const __half *p = X + col;
        int64_t r = r0 + ty;
        for (; r + RL * 7 < r1; r += RL * 8) {           // 8 loads in flight
            uint4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const uint4 *>(p + (r + RL * u) * ldx);
#pragma unroll
            for (int u = 0; u < 8; ++u) acc = __builtin_elementwise_max(acc, abs_bits(v[u]));
        }
        for (; r < r1; r += RL)
            acc = __builtin_elementwise_max(acc, abs_bits(*reinterpret_cast<const uint4 *>(p + r * ldx)));
    }
    part[ty][tx] = acc;
    __syncthreads();
    for (int s = RL / 2; s >= 1; s >>= 1) {
        if (ty < s) part[ty][tx] = __builtin_elementwise_max(part[ty][tx], part[ty + s][tx]);
        __syncthreads();
    }
    if (threadIdx.x < CG * 8) {                          // one channel per thread
        const int c = (blockIdx.x * CG) * 8 + threadIdx.x;
        if (c < K) {
            const float f = half_bits_to_float(part[0][threadIdx.x >> 3][threadIdx.x & 7]);
            // non-negative floats order like their bit patterns
            atomicMax(reinterpret_cast<unsigned int *>(absmax + c), __float_as_uint(f));
        }
    }
}

// s_j = max(a_j, 1e-5)^alpha / max(w_j, 1e-5)^(1 - alpha), in double (K values only).
__global__ void smooth_factors_kernel(const float *__restrict__ act_absmax, const float *__restrict__ w_rowmax,
                                      int K, double alpha, float *__restrict__ s, float *__restrict__ inv_s)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= K) return;
    double sj = 1.0;
    if (act_absmax) {
        const double a = fmax((double)act_absmax[j], 1e-5);
        const double w = fmax((double)w_rowmax[j], 1e-5);
        sj = pow(a, alpha) / pow(w, 1.0 - alpha);
    }
    s[j] = (float)sj;
    if (inv_s) inv_s[j] = (float)(1.0 / sj);
}

// Wt[n][k] = W[k][n] in tiles of 64 x 64 through LDS, 16 bytes per lane on both sides, and -- on the way -- the row
// maxima w_rowmax[k] = max_n |W[k][n]| of the smoothing-factor formula, so that W is read once for both.
//   load   lane (row r = t / 8, chunk c = t % 8) fetches the eight values W[k0 + r][n0 + 8 c ..]: a wave reads eight
//          whole 128-byte rows of the tile; their maximum over the eight lanes of a row goes to w_rowmax with ONE
//          atomic per row and tile (bit patterns of non-negative floats order like unsigned integers; the caller
//          clears w_rowmax first)
//   LDS    row pitch 72 values; the 16-byte chunk c of row k sits at chunk position (c + k / 8) % 8, so that the
//          transposed reads below touch every bank once
//   store  lane (n = t / 8, chunk kc = t % 8) gathers W[k0 + 8 kc .. + 7][n0 + n] with eight 2-byte reads and writes
//          16 bytes of row n of Wt: eight lanes fill one 128-byte line
// K % 64 == 0 for every supported Hadamard order; N % 16 == 0, so a chunk of 8 columns is inside or outside N whole.
__global__ __launch_bounds__(256) void transpose_absmax_f16_kernel(const unsigned short *__restrict__ W, int K, int N,
                                                                   int64_t ldw, unsigned short *__restrict__ Wt,
                                                                   float *__restrict__ w_rowmax)
{
    constexpr int PITCH = 72;
    __shared__ __attribute__((aligned(16))) unsigned short tile[64 * PITCH];
    const int k0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    const int t = threadIdx.x;
    {
        const int c = t & 7;
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int r = (t >> 3) + 32 * pass;
            const int n = n0 + 8 * c;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (n < N) v = *reinterpret_cast<const uint4 *>(W + (int64_t)(k0 + r) * ldw + n);
            *reinterpret_cast<uint4 *>(tile + r * PITCH + 8 * ((c + (r >> 3)) & 7)) = v;
            if (w_rowmax) {
                const us8 a = abs_bits(v);
                unsigned short m = 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) m = a[e] > m ? a[e] : m;
                int mi = (int)m;                          // maximum over the 8 lanes of the row (lanes 8 q .. 8 q + 7)
                mi = max(mi, lane_perm<0xB1>(mi));
                mi = max(mi, lane_perm<0x4E>(mi));
                mi = max(mi, lane_perm<0x141>(mi));
                if (c == 0 && mi != 0)
                    atomicMax(reinterpret_cast<unsigned int *>(w_rowmax + k0 + r), __float_as_uint(half_bits_to_float((unsigned short)mi)));
            }
        }
    }
    __syncthreads();
    {
        const int kc = t & 7;
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int nl = (t >> 3) + 32 * pass;
            if (n0 + nl < N) {
                union { uint4 u; unsigned short h[8]; } o;
                const int pos = 8 * (((nl >> 3) + kc) & 7) + (nl & 7);      // where column nl sits in the rows of chunk kc
#pragma unroll
                for (int u = 0; u < 8; ++u) o.h[u] = tile[(8 * kc + u) * PITCH + pos];
                *reinterpret_cast<uint4 *>(Wt + (int64_t)(n0 + nl) * K + k0 + 8 * kc) = o.u;
            }
        }
    }
}

__global__ __launch_bounds__(256) void zero_f32_kernel(float *__restrict__ p, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

}  // namespace

template <int CG>
hipError_t launch_calib(const void *X, int64_t T, int64_t K, int64_t ldx, float *absmax_io, hipStream_t st, int64_t wgs)
{
    constexpr int RL = 256 / CG;
    const unsigned gx = (unsigned)((K + CG * 8 - 1) / (CG * 8));
    // about `wgs` workgroups, at least one row per row lane each
    int64_t gy = wgs / gx > 0 ? wgs / gx : 1;
    if (gy > (T + RL - 1) / RL) gy = (T + RL - 1) / RL;
    int64_t rpb = (T + gy - 1) / gy;
    rpb = (rpb + RL - 1) / RL * RL;
    gy = (T + rpb - 1) / rpb;
    hipLaunchKernelGGL(calib_absmax_kernel<CG>, dim3(gx, (unsigned)gy), dim3(256), 0, st,
                       static_cast<const __half *>(X), T, (int)K, ldx, absmax_io, rpb);
    return hipGetLastError();
}

// Measured on K = 4096 (TB/s; strips of 128 bytes per row and 1024 workgroups against strips of 256 bytes and
// 2048 workgroups): T = 2048 2.95 / 2.89 (one short round: the narrower strip ends with fewer atomics),
// T = 16384 4.73 / 5.66, T = 65536 5.10 / 5.64.
hipError_t launch_calib_absmax(const void *X, int64_t T, int64_t K, int64_t ldx, float *absmax_io,
                               hipStream_t st)
{
    if (T >= 8192) return launch_calib<16>(X, T, K, ldx, absmax_io, st, 2048);
    return launch_calib<8>(X, T, K, ldx, absmax_io, st, 1024);
}

hipError_t launch_smooth_factors(const float *act_absmax, const float *w_rowmax, int64_t K, float alpha,
                                 float *s, float *inv_s, hipStream_t st)
{
    hipLaunchKernelGGL(smooth_factors_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st,
                       act_absmax, w_rowmax, (int)K, (double)alpha, s, inv_s);
    return hipGetLastError();
}

hipError_t launch_transpose_absmax_f16(const void *W, int64_t K, int64_t N, int64_t ldw, void *Wt, float *w_rowmax,
                                       hipStream_t st)
{
    if (w_rowmax) {                                      // the maxima are collected with atomicMax: start from zero
        hipLaunchKernelGGL(zero_f32_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, w_rowmax, (int)K);
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(transpose_absmax_f16_kernel, dim3((unsigned)((N + 63) / 64), (unsigned)(K / 64)), dim3(256), 0, st,
                       static_cast<const unsigned short *>(W), (int)K, (int)N, ldw, static_cast<unsigned short *>(Wt),
                       w_rowmax);
    return hipGetLastError();
}

}  // namespace sr
