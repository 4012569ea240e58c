// Measurement kernels: what this chip sustains with nothing else in the way.  They compute nothing of the method;
// bench.py times them beside the real kernels so that every fraction of a published peak can also be read against
// a ceiling measured in the same process on the same box.
//   sr_ceiling_hbm_read   a pure read stream over a buffer (the weight stream of a decode GEMM without the GEMM)
//   sr_ceiling_row_stream the memory traffic of a rotation + quantiser launch (a row in, its codes out) without the rotation
//   sr_ceiling_mfma_f6    a bare issue loop of the FP6 matrix instruction the prefill GEMM uses, on code-valued
//                         operands held in registers (no LDS, no loads, no barriers)
//   sr_ceiling_mfma_i8    the same for the int8 matrix instruction of the canonical-nibble GEMM
//   sr_ceiling_valu_f32   a bare loop of independent fp32 vector additions (the butterflies of the rotation)
#include "../../include/smoothrot.h"
#include "sr_common.h"

namespace sr {
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Every thread keeps INFLIGHT 16-byte loads in flight; a workgroup reads contiguous runs of NT * 16 bytes and
// strides by the grid.  The words are folded into one value that is stored only if it equals a constant no
// buffer of the benchmark produces, so the loads cannot be dropped and nothing is written.
template <int INFLIGHT, bool NT_LOADS>
__global__ __launch_bounds__(1024) void hbm_read_kernel(const u32x4 *__restrict__ src, int64_t n16, uint32_t *__restrict__ sink)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t acc = 0;
    for (; i + (INFLIGHT - 1) * stride < n16; i += INFLIGHT * stride) {
        u32x4 v[INFLIGHT];
#pragma unroll
        for (int k = 0; k < INFLIGHT; ++k)
            v[k] = NT_LOADS ? __builtin_nontemporal_load(src + i + k * stride) : src[i + k * stride];
#pragma unroll
        for (int k = 0; k < INFLIGHT; ++k) acc ^= v[k][0] ^ v[k][1] ^ v[k][2] ^ v[k][3];
    }
    for (; i < n16; i += stride) {
        const u32x4 v = NT_LOADS ? __builtin_nontemporal_load(src + i) : src[i];
        acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    if (acc == 0x9E3779B9u && sink) sink[0] = acc;
}

// The traffic of a rotation + quantiser launch without the rotation: workgroup w of 256 threads reads "row" w of
// `row_bytes` (16-byte loads, all issued up front, as the rotation kernels do), folds it and writes `out_bytes` of
// the fold to "row" w of dst -- same grid, same bytes per workgroup, same dependence of every store on every load of
// the row, no arithmetic to speak of.  lds_bytes of dynamic LDS per workgroup reproduce the occupancy.
__global__ __launch_bounds__(256) void row_stream_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t rows,
                                                         int row16, int out16)
{
    extern __shared__ uint32_t red_s[];
    const int t = threadIdx.x;
    for (int64_t w = blockIdx.x; w < rows; w += gridDim.x) {
        const u32x4 *s = src + w * row16;
        u32x4 acc = {0u, 0u, 0u, 0u};
        u32x4 v[8];
        for (int i0 = 0; i0 < row16; i0 += 8 * 256) {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int i = i0 + k * 256 + t;
                v[k] = i < row16 ? __builtin_nontemporal_load(s + i) : acc;
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) acc ^= v[k];
        }
        // every store depends on every load of the row (as the quantiser's scale does): fold over the workgroup
        uint32_t f = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) f ^= __shfl_xor(f, off, 64);
        if ((t & 63) == 0) red_s[t >> 6] = f;
        __syncthreads();
        f = red_s[0] ^ red_s[1] ^ red_s[2] ^ red_s[3];
        __syncthreads();
        u32x4 *d = dst + w * out16;
        for (int i = t; i < out16; i += 256) {
            const u32x4 o = {f, acc[1], acc[2], (uint32_t)i};
            d[i] = o;
        }
    }
}

// 8 waves per workgroup (two per SIMD, as in the GEMM), 8 independent 32 x 32 accumulators per wave (4 x 2 tiles,
// 128 registers, as in the GEMM's wave tile); operands are 6-bit fields of INT4 codes (sign-magnitude, |c| <= 8)
// loaded once from `codes` so that the multipliers see the switching activity of real operands.
__global__ __launch_bounds__(512, 2) void mfma_f6_loop_kernel(const uint32_t *__restrict__ codes, int iters, float *__restrict__ sink)
{
    v8i a[4], b[2];
    const uint32_t *p = codes + (threadIdx.x & 63) * 6;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int k = 0; k < 8; ++k) a[i][k] = k < 6 ? (int)p[384 * i + k] : 0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int k = 0; k < 8; ++k) b[i][k] = k < 6 ? (int)p[384 * (4 + i) + k] : 0;
    v16f acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 2; ++i)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b[i], a[j], acc[i][j], 2, 2, 0, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) s += acc[i][j][e];
    if (s == 12345.678f && sink) sink[0] = s;            // sums of integers / 64: never this value
}

// the int8 instruction of the canonical-nibble GEMM (32 x 32 x 32, operands = codes * 16 in bytes)
__global__ __launch_bounds__(512, 2) void mfma_i8_loop_kernel(const uint32_t *__restrict__ bytes, int iters, int *__restrict__ sink)
{
    v4i a[4], b[2];
    const uint32_t *p = bytes + (threadIdx.x & 63) * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int k = 0; k < 4; ++k) a[i][k] = (int)p[256 * i + k];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int k = 0; k < 4; ++k) b[i][k] = (int)p[256 * (4 + i) + k];
    v16i acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 2; ++i) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[i], a[j], acc[i][j], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) s ^= acc[i][j][e];
    if (s == 0x7FFFFFFF && sink) sink[0] = s;
}

// One 32-point transform per iteration and lane, in registers: 5 levels x 32 additions / subtractions, then one
// multiplication per value by 1/32 so that the values stay where they started (H H = 32 I): 192 vector
// instructions per iteration and wave, the instruction mix of the rotation kernels' register passes.
__global__ __launch_bounds__(256) void valu_f32_loop_kernel(int iters, float seed, float *__restrict__ sink)
{
    float v[32];
#pragma unroll
    for (int k = 0; k < 32; ++k) v[k] = seed * (float)(k + 1) + (float)(threadIdx.x & 63) * 0.37f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int h = 1; h < 32; h <<= 1)
#pragma unroll
            for (int k = 0; k < 32; ++k)
                if (!(k & h)) {
                    const float x = v[k], y = v[k | h];
                    v[k] = x + y;
                    v[k | h] = x - y;
                }
#pragma unroll
        for (int k = 0; k < 32; ++k) v[k] *= 0.03125f;
        asm volatile("" : "+v"(v[0]));                           // keeps the loop a loop
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 32; ++k) s += v[k];
    if (s == 12345.678f && sink) sink[0] = s;
}

template <int INFLIGHT>
hipError_t launch_read(const void *src, size_t bytes, uint32_t *sink, int grid, int block, int nontemporal, hipStream_t st)
{
    const int64_t n16 = (int64_t)(bytes / 16);
    if (nontemporal)
        hipLaunchKernelGGL((hbm_read_kernel<INFLIGHT, true>), dim3(grid), dim3(block), 0, st, static_cast<const u32x4 *>(src), n16, sink);
    else
        hipLaunchKernelGGL((hbm_read_kernel<INFLIGHT, false>), dim3(grid), dim3(block), 0, st, static_cast<const u32x4 *>(src), n16, sink);
    return hipGetLastError();
}

}  // namespace
}  // namespace sr

extern "C" {

int sr_ceiling_hbm_read(const void *src, size_t bytes, int grid, int block, int in_flight, int nontemporal,
                        uint32_t *sink, void *stream)
{
    if (!src) return SR_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || bytes % 16 != 0) return SR_ERR_ALIGN;
    if (grid < 1 || grid > 65536 || block < 64 || block > 1024 || block % 64 != 0) return SR_ERR_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    switch (in_flight) {
        case 1: e = sr::launch_read<1>(src, bytes, sink, grid, block, nontemporal, st); break;
        case 2: e = sr::launch_read<2>(src, bytes, sink, grid, block, nontemporal, st); break;
        case 4: e = sr::launch_read<4>(src, bytes, sink, grid, block, nontemporal, st); break;
        case 8: e = sr::launch_read<8>(src, bytes, sink, grid, block, nontemporal, st); break;
        case 16: e = sr::launch_read<16>(src, bytes, sink, grid, block, nontemporal, st); break;
        default: return SR_ERR_ARG;
    }
    return e == hipSuccess ? SR_OK : SR_ERR_DEVICE;
}

int sr_ceiling_row_stream(const void *src, void *dst, int64_t rows, int64_t row_bytes, int64_t out_bytes, int grid,
                          int lds_bytes, void *stream)
{
    if (!src || !dst) return SR_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 15u) || row_bytes % 16 != 0 ||
        out_bytes % 16 != 0)
        return SR_ERR_ALIGN;
    if (rows < 1 || row_bytes < 16 || out_bytes < 16 || row_bytes > (1 << 24) || grid < 1 || grid > 65536 || lds_bytes < 64 ||
        lds_bytes > 160 * 1024)
        return SR_ERR_ARG;
    auto kern = sr::row_stream_kernel;
    if (lds_bytes > 48 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess)
        return SR_ERR_DEVICE;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), (size_t)lds_bytes, static_cast<hipStream_t>(stream),
                       static_cast<const sr::u32x4 *>(src), static_cast<sr::u32x4 *>(dst), rows, (int)(row_bytes / 16),
                       (int)(out_bytes / 16));
    return hipGetLastError() == hipSuccess ? SR_OK : SR_ERR_DEVICE;
}

int sr_ceiling_mfma_f6(const void *fields, size_t bytes, int iters, int grid, float *sink, void *stream)
{
    if (!fields) return SR_ERR_NULL;
    if (bytes < 9216 || (reinterpret_cast<uintptr_t>(fields) & 3u)) return SR_ERR_ARG;
    if (iters < 1 || grid < 1 || grid > 65536) return SR_ERR_ARG;
    hipLaunchKernelGGL(sr::mfma_f6_loop_kernel, dim3(grid), dim3(512), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint32_t *>(fields), iters, sink);
    return hipGetLastError() == hipSuccess ? SR_OK : SR_ERR_DEVICE;
}

int sr_ceiling_mfma_i8(const void *operands, size_t bytes, int iters, int grid, int *sink, void *stream)
{
    if (!operands) return SR_ERR_NULL;
    if (bytes < 6144 || (reinterpret_cast<uintptr_t>(operands) & 3u)) return SR_ERR_ARG;
    if (iters < 1 || grid < 1 || grid > 65536) return SR_ERR_ARG;
    hipLaunchKernelGGL(sr::mfma_i8_loop_kernel, dim3(grid), dim3(512), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint32_t *>(operands), iters, sink);
    return hipGetLastError() == hipSuccess ? SR_OK : SR_ERR_DEVICE;
}

int sr_ceiling_valu_f32(int iters, int grid, float *sink, void *stream)
{
    if (iters < 1 || grid < 1 || grid > 65536) return SR_ERR_ARG;
    hipLaunchKernelGGL(sr::valu_f32_loop_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream), iters, 1.0f, sink);
    return hipGetLastError() == hipSuccess ? SR_OK : SR_ERR_DEVICE;
}

}  // extern "C"
