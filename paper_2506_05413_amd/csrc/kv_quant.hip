// Asymmetric 4-bit group quantiser for keys and values (paper: Eq. (1), asymmetric case;
// "Quantization" settings: group size 128, constant clipping ratio 0.95).
//
//   hi = clip * max, lo = clip * min over a group of G consecutive values
//   Delta = (hi - lo) / 15 (1 when the range is empty),  z = -rint(lo / Delta)
//   code  = clamp(rint(v / Delta) + z, 0, 15)
// (divisions by Delta are multiplications by its fp32 reciprocal here)
//
// Pure streaming: 2 bytes read and 0.5 + 8 / G bytes written per value.  Eight lanes x 16 bytes
// cover 64 values, so a group of G values is G / 8 neighbouring lanes: minimum and maximum are
// reduced with lane shuffles inside that lane group, every lane quantises its own eight values
// into one dword, and a wave instruction reads 1 KB and writes 256 B of contiguous memory.
#include "sr_common.h"

#include <hip/hip_fp16.h>

namespace sr {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// LPG = lanes per group = G / 8; CONTIG: rows follow each other without padding; UNROLL 16-byte loads in flight per lane
template <int LPG, bool CONTIG, int UNROLL>
__global__ __launch_bounds__(256) void kv_quant_kernel(const __half *__restrict__ X, int64_t rows, int D, int64_t ldx,
                                                        float clip, uint32_t *__restrict__ Q, float *__restrict__ scale,
                                                        float *__restrict__ zero, int64_t chunks)
{
    // chunk = 8 consecutive values of a row; chunk c -> (row, column) = (c / (D/8), 8 * (c % (D/8)))
    const int cpr = D >> 3;
    const int64_t stride = (int64_t)gridDim.x * 256;
    int64_t c0 = (int64_t)blockIdx.x * 256 * UNROLL + threadIdx.x;
    for (; c0 - threadIdx.x < chunks; c0 += stride * UNROLL) {
        union { u32x4 v; __half h[8]; } raw[UNROLL];
        bool ok[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t c = c0 + 256 * u;
            ok[u] = c < chunks;
            const int64_t cc = ok[u] ? c : chunks - 1;     // in-bounds dummy for the tail lanes
            if (CONTIG) {
                raw[u].v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(X + cc * 8));
            } else {
                const int64_t r = cc / cpr;                // (a 64-bit division per chunk: the padded layout is the slow path)
                const int col = (int)(cc - r * cpr) << 3;
                raw[u].v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(X + r * ldx + col));
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = __half2float(raw[u].h[e]);
            float mx = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
            float mn = fminf(fminf(fminf(v[0], v[1]), fminf(v[2], v[3])), fminf(fminf(v[4], v[5]), fminf(v[6], v[7])));
            // D % G == 0 and chunks % LPG == 0: a lane group never straddles rows or the end of the data
            if constexpr (LPG == 16) {                     // the paper's group of 128 values: no LDS round trips
                mx = max_of_16_lanes(mx);
                mn = min_of_16_lanes(mn);
            } else {
#pragma unroll
                for (int off = LPG / 2; off >= 1; off >>= 1) {
                    mx = fmaxf(mx, __shfl_xor(mx, off, 64));
                    mn = fminf(mn, __shfl_xor(mn, off, 64));
                }
            }
            const float hi = clip * mx, lo = clip * mn;
            const float delta = (hi == lo) ? 1.f : (hi - lo) / 15.f;
            const float inv = 1.f / delta;
            const float z = -rintf(lo * inv);
            uint32_t word = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float code = fminf(fmaxf(rintf(v[e] * inv) + z, 0.f), 15.f);
                word |= (uint32_t)(int)code << (4 * e);
            }
            const int64_t c = c0 + 256 * u;
            if (ok[u]) {
                __builtin_nontemporal_store(word, Q + c);
                if ((threadIdx.x & (LPG - 1)) == 0) {
                    scale[c / LPG] = delta;
                    zero[c / LPG] = z;
                }
            }
        }
    }
}

template <int LPG>
hipError_t launch_lpg(const void *X, int64_t rows, int64_t D, int64_t ldx, float clip, uint8_t *Q, float *scale, float *zero,
                      hipStream_t st)
{
    const int64_t chunks = rows * (D / 8);
    const bool contig = ldx == D || rows == 1;
    // eight loads in flight per lane once that still leaves every CU several workgroups, two otherwise
    const bool big = chunks >= (int64_t)256 * 8 * 2048;
    const int unroll = big ? 8 : 2;
    int64_t blocks = (chunks + 256 * unroll - 1) / (256 * unroll);
    if (blocks > 65536) blocks = 65536;
#define SR_KV(CC, UU)                                                                                                  \
    hipLaunchKernelGGL((kv_quant_kernel<LPG, CC, UU>), dim3((unsigned)blocks), dim3(256), 0, st,                        \
                       static_cast<const __half *>(X), rows, (int)D, ldx, clip, reinterpret_cast<uint32_t *>(Q), scale, \
                       zero, chunks)
    if (contig) { if (big) SR_KV(true, 8); else SR_KV(true, 2); }
    else { if (big) SR_KV(false, 8); else SR_KV(false, 2); }
#undef SR_KV
    return hipGetLastError();
}

}  // namespace

hipError_t launch_kv_quant(const void *X, int64_t rows, int64_t D, int64_t ldx, int64_t group, float clip,
                           uint8_t *Q, float *scale, float *zero, hipStream_t st)
{
    switch (group) {
        case 32: return launch_lpg<4>(X, rows, D, ldx, clip, Q, scale, zero, st);
        case 64: return launch_lpg<8>(X, rows, D, ldx, clip, Q, scale, zero, st);
        case 128: return launch_lpg<16>(X, rows, D, ldx, clip, Q, scale, zero, st);
        case 256: return launch_lpg<32>(X, rows, D, ldx, clip, Q, scale, zero, st);
        case 512: return launch_lpg<64>(X, rows, D, ldx, clip, Q, scale, zero, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sr
