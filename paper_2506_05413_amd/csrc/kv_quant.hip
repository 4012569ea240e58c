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

// LPG = lanes per group = G / 8; CONTIG: rows follow each other without padding; UNROLL 16-byte loads per lane and
// batch.  A thread walks over several batches and fetches the next one before it works on the current one: with
// one batch per thread every wave of the chip loads at the same time and computes at the same time, and the
// ~11 vector instructions per value do not overlap the memory traffic (measured 23 us = 13 us of traffic plus
// 10 us of arithmetic for 32768 x 1024 values).
template <int LPG, bool CONTIG, int UNROLL>
__global__ __launch_bounds__(256) void kv_quant_kernel(const __half *__restrict__ X, int64_t rows, int D, int64_t ldx,
                                                        float clip, uint32_t *__restrict__ Q, float *__restrict__ scale,
                                                        float *__restrict__ zero, int64_t chunks)
{
    // chunk = 8 consecutive values of a row; chunk c -> (row, column) = (c / (D/8), 8 * (c % (D/8)))
    const int cpr = D >> 3;
    const int64_t stride = (int64_t)gridDim.x * 256 * UNROLL;
    union Raw { u32x4 v; __half h[8]; };
    // loads are unconditional (chunks past the end re-read the last one), so that the wait before the first use
    // of a batch leaves the loads of the next batch in flight
    auto load_batch = [&](Raw (&raw)[UNROLL], int64_t c0) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t c = c0 + 256 * u;
            const int64_t cc = c < chunks ? c : chunks - 1;
            if (CONTIG) {
                raw[u].v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(X + cc * 8));
            } else {
                const int64_t r = cc / cpr;                // (a 64-bit division per chunk: the padded layout is the slow path)
                const int col = (int)(cc - r * cpr) << 3;
                raw[u].v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(X + r * ldx + col));
            }
        }
    };
    auto quantise_batch = [&](const Raw (&raw)[UNROLL], int64_t c0) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = __half2float(raw[u].h[e]);
            float mx = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
            float mn = fminf(fminf(fminf(v[0], v[1]), fminf(v[2], v[3])), fminf(fminf(v[4], v[5]), fminf(v[6], v[7])));
            // D % G == 0 and chunks % LPG == 0: a lane group never straddles rows or the end of the data.
            // Lane exchanges inside a row of 16 lanes are operand permutations; only larger groups go through LDS.
            if constexpr (LPG >= 2) { mx = fmaxf(mx, lane_perm<0xB1>(mx)); mn = fminf(mn, lane_perm<0xB1>(mn)); }
            if constexpr (LPG >= 4) { mx = fmaxf(mx, lane_perm<0x4E>(mx)); mn = fminf(mn, lane_perm<0x4E>(mn)); }
            if constexpr (LPG >= 8) { mx = fmaxf(mx, lane_perm<0x141>(mx)); mn = fminf(mn, lane_perm<0x141>(mn)); }
            if constexpr (LPG >= 16) { mx = fmaxf(mx, lane_perm<0x140>(mx)); mn = fminf(mn, lane_perm<0x140>(mn)); }
#pragma unroll
            for (int off = LPG / 2; off >= 16; off >>= 1) {
                mx = fmaxf(mx, __shfl_xor(mx, off, 64));
                mn = fminf(mn, __shfl_xor(mn, off, 64));
            }
            const float hi = clip * mx, lo = clip * mn;
            // two roundings (the constant 1/15, the product) and a reciprocal good to one unit in the last place:
            // Delta and 1 / Delta are within 2e-7 of the quotients, far inside the tolerance of a rounding boundary
            const float delta = (hi == lo) ? 1.f : (hi - lo) * (1.f / 15.f);
            const float inv = __builtin_amdgcn_rcpf(delta);
            const float z = -rintf(lo * inv);
            // rint(v / Delta) + z, clamped to [0, 15]: adding 1.5 * 2^23 rounds v * inv + z to the nearest integer
            // (ties to even) in the low mantissa bits; |z| and |v * inv| stay below 2^16 for fp16 inputs (a group's
            // range is at least one fp16 spacing of its largest value), so z + magic is exact.  The eight fields are
            // packed with the constant still inside and its packed image subtracted once.
            constexpr uint32_t kMagic = 0x4B400000u;
            const float zm = z + __uint_as_float(kMagic);
            uint32_t word = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int bits = (int)__float_as_uint(fmaf(v[e], inv, zm));
                const uint32_t t = (uint32_t)min(max(bits, (int)kMagic), (int)kMagic + 15);
                word += t << (4 * e);
            }
            constexpr uint32_t packed_magic = kMagic * 0x11111111u;      // sum of kMagic << 4 e, modulo 2^32
            word -= packed_magic;
            const int64_t c = c0 + 256 * u;
            if (c < chunks) {
                __builtin_nontemporal_store(word, Q + c);
                if ((threadIdx.x & (LPG - 1)) == 0) {
                    scale[c / LPG] = delta;
                    zero[c / LPG] = z;
                }
            }
        }
    };

    int64_t c0 = (int64_t)blockIdx.x * 256 * UNROLL + threadIdx.x;
    Raw a[UNROLL], b[UNROLL];
    load_batch(a, c0);
    // two batches per trip, so that the buffers swap roles without register copies
    for (; c0 - threadIdx.x < chunks; c0 += 2 * stride) {
        load_batch(b, c0 + stride);
        quantise_batch(a, c0);
        load_batch(a, c0 + 2 * stride);
        if (c0 + stride - threadIdx.x < chunks) quantise_batch(b, c0 + stride);
    }
}

template <int LPG>
hipError_t launch_lpg(const void *X, int64_t rows, int64_t D, int64_t ldx, float clip, uint8_t *Q, float *scale, float *zero,
                      hipStream_t st)
{
    const int64_t chunks = rows * (D / 8);
    const bool contig = ldx == D || rows == 1;
    // four loads per batch (two batches in flight per lane); at most eight workgroups per CU, so that a thread of a
    // large call walks over several batches
    const bool big = chunks >= (int64_t)256 * 4 * 2048;
    const int unroll = big ? 4 : 2;
    int64_t blocks = (chunks + 256 * unroll - 1) / (256 * unroll);
    const int64_t cap = (int64_t)compute_units() * 8;
    if (blocks > cap) blocks = cap;
#define SR_KV(CC, UU)                                                                                                  \
    hipLaunchKernelGGL((kv_quant_kernel<LPG, CC, UU>), dim3((unsigned)blocks), dim3(256), 0, st,                        \
                       static_cast<const __half *>(X), rows, (int)D, ldx, clip, reinterpret_cast<uint32_t *>(Q), scale, \
                       zero, chunks)
    if (contig) { if (big) SR_KV(true, 4); else SR_KV(true, 2); }
    else { if (big) SR_KV(false, 4); else SR_KV(false, 2); }
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
