// Offline helpers: calibration absmax, weight row maxima, smoothing factors and the
// fp16 transpose that turns the weight fold into a row-wise rotation + quantisation.
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

// w_rowmax[j] = max_n |W[j][n]|: one block per input channel j.
__global__ __launch_bounds__(256) void row_absmax_kernel(const __half *__restrict__ W, int N, int64_t ldw,
                                                          float *__restrict__ w_rowmax)
{
    __shared__ us8 part[256];
    const __half *p = W + (int64_t)blockIdx.x * ldw;
    us8 acc = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int c = threadIdx.x * 8; c < N; c += 256 * 8)      // N % 16 == 0: whole 8-groups
        acc = __builtin_elementwise_max(acc, abs_bits(*reinterpret_cast<const uint4 *>(p + c)));
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s >= 1; s >>= 1) {
        if ((int)threadIdx.x < s)
            part[threadIdx.x] = __builtin_elementwise_max(part[threadIdx.x], part[threadIdx.x + s]);
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const us8 a = part[0];
        unsigned short m = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) m = a[e] > m ? a[e] : m;
        w_rowmax[blockIdx.x] = half_bits_to_float(m);
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

// 64 x 64 tile transpose of 16-bit values through LDS.
__global__ __launch_bounds__(256) void transpose_f16_kernel(const unsigned short *__restrict__ W, int K, int N,
                                                             int64_t ldw, unsigned short *__restrict__ Wt)
{
    __shared__ unsigned short tile[64][66];
    const int k0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int r = ty; r < 64; r += 4) {
        const int k = k0 + r, n = n0 + tx;
        tile[r][tx] = (k < K && n < N) ? W[(int64_t)k * ldw + n] : (unsigned short)0;
    }
    __syncthreads();
    for (int r = ty; r < 64; r += 4) {
        const int n = n0 + r, k = k0 + tx;
        if (n < N && k < K) Wt[(int64_t)n * K + k] = tile[tx][r];
    }
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

hipError_t launch_row_absmax(const void *W, int64_t K, int64_t N, int64_t ldw, float *w_rowmax, hipStream_t st)
{
    hipLaunchKernelGGL(row_absmax_kernel, dim3((unsigned)K), dim3(256), 0, st,
                       static_cast<const __half *>(W), (int)N, ldw, w_rowmax);
    return hipGetLastError();
}

hipError_t launch_smooth_factors(const float *act_absmax, const float *w_rowmax, int64_t K, float alpha,
                                 float *s, float *inv_s, hipStream_t st)
{
    hipLaunchKernelGGL(smooth_factors_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st,
                       act_absmax, w_rowmax, (int)K, (double)alpha, s, inv_s);
    return hipGetLastError();
}

hipError_t launch_transpose_f16(const void *W, int64_t K, int64_t N, int64_t ldw, void *Wt, hipStream_t st)
{
    hipLaunchKernelGGL(transpose_f16_kernel, dim3((unsigned)((N + 63) / 64), (unsigned)((K + 63) / 64)),
                       dim3(256), 0, st, static_cast<const unsigned short *>(W), (int)K, (int)N, ldw,
                       static_cast<unsigned short *>(Wt));
    return hipGetLastError();
}

}  // namespace sr
