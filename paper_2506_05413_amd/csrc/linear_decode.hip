// Whole online path of the W4A4 linear layer for a decode step behind one entry point; for ONE token and
// K = 2048 / 4096 in ONE launch:
//     x^ = quantise((x * inv_s) H),   Y = dequantise(x^ W^)
// (Paper: online Hadamard + per-token INT4 of the activations in front of the quantised
// projection, section "Methodology" and Eq. (1); this is the decode step, where a launch and a
// round trip through memory cost as much as the arithmetic.)
//
// A workgroup owns 8 G output channels over all of K.  It first ISSUES the loads of its token row
// and smoothing factors, then of all its weights (they stay in flight in registers), then rotates
// and quantises the row in LDS while the weights travel, and finally multiplies packed codes with
// v_dot8_i32_i4 straight from the registers against the codes in LDS.  Every workgroup repeats
// the rotation, so the grid is kept near one workgroup per CU; and only power-of-two K up to 8192
// is offered, because the rotation of a longer or a 28 * 2^p row takes one workgroup longer than
// the weights take to arrive.  Loads return in order per wave: whatever the rotation needs has to
// be issued BEFORE the weights.  Lane (r = l >> 3, c = l & 7) holds the 16-byte chunk c of a
// 128-byte slab of row r of an 8-row group, so every load instruction reads whole lines; wave w
// takes slabs w, w + 8, ...
#include "fwht_row.h"

namespace sr {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int LD_NT = 512;                 // threads per workgroup
constexpr int LD_NW = LD_NT / 64;
constexpr int LD_MT = 1;                   // tokens per call (two rows lose to the two-call path: measured)

template <int K, int G>
__global__ __launch_bounds__(LD_NT) void linear_decode_kernel(const __half *__restrict__ X, int M, int64_t ldx,
                                                              const float *__restrict__ pre, float clip,
                                                              const uint8_t *__restrict__ Wq,
                                                              const float *__restrict__ ws, int N,
                                                              __half *__restrict__ Y, int64_t ldy,
                                                              uint8_t *__restrict__ Xq_out, float *__restrict__ xs_out)
{
    constexpr int Kb = K / 2;
    constexpr int NSLAB = (Kb + 127) / 128;
    constexpr int U = (NSLAB + LD_NW - 1) / LD_NW;
    static_assert(G * U <= 16, "weights in flight must fit the register file");

    extern __shared__ float row[];                                     // padded_len(K) floats, then the codes
    uint32_t *xq = reinterpret_cast<uint32_t *>(row + padded_len(K));   // [LD_MT][K / 8] packed codes
    __shared__ float red[LD_NW];
    __shared__ float sx[LD_MT];

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int r = lane >> 3, c = lane & 7;
    const int n0 = blockIdx.x * (8 * G);

    // ---- the first token row's loads go first (they are what the rotation waits for) ...
    RowLoad<K, LD_NT> xld;
    row_load<K, LD_NT, true>(X, pre, t, xld);

    // ---- ... the channel scale of this thread's output (fetched now, used last: a load after the reduction would
    // put one more memory latency at the end of the kernel) ...
    static_assert(8 * G <= LD_NT, "one output per thread");
    const float w_scale = (t < 8 * G && n0 + t < N) ? ws[n0 + t] : 0.f;

    // ---- ... then all weight loads of this workgroup, up front, every one unconditional: a load under a
    // branch would make the compiler wait for ALL outstanding loads before the rotation may touch the row, and the
    // rotation would then start when the last weight has arrived instead of running while they travel
    static_assert(NSLAB % LD_NW == 0 && Kb % 128 == 0, "every wave owns whole slabs");
    u32x4 w[G][U];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        // register slot g holds row group (g + workgroup index) mod G: at any moment the workgroups of the
        // chip then ask for different offsets inside their 8 G rows, not all for the same memory channels
        int n = n0 + 8 * ((g + (int)blockIdx.x) % G) + r;
        n = n < N ? n : N - 1;                                          // ragged last workgroup: re-read the last row
        const uint8_t *wp = Wq + (int64_t)n * Kb + c * 16;
#pragma unroll
        for (int u = 0; u < U; ++u)
            w[g][u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wp + (wave + LD_NW * u) * 128));
    }

    // nothing of the rotation may be scheduled ahead of the weight loads (its first instructions wait for the row)
    __builtin_amdgcn_sched_barrier(0);

    // ---- rotate + quantise the token row into LDS (M = 1: the host rejects more) ----------------
    {
        constexpr int m = 0;
        const float amax = rotate_loaded_row_absmax<K, LD_NT>(xld, pre, row, red, t);
        const float delta = (amax == 0.f) ? 1.f : (clip * amax) / 7.f;
        const float inv_delta = 1.f / delta;
        if (t == 0) {
            sx[m] = delta;
            if (xs_out && blockIdx.x == 0) xs_out[m] = delta;
        }
        uint32_t *q = xq + m * (K / 8);
        for (int i = t; i < K / 8; i += LD_NT) {
            const float *src = row + pad(8 * i);
            const float4 a = *reinterpret_cast<const float4 *>(src);
            const float4 b = *reinterpret_cast<const float4 *>(src + 4);
            const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
            const uint32_t code = quant_pack8(v, inv_delta);
            q[i] = code;
            if (Xq_out && blockIdx.x == 0) reinterpret_cast<uint32_t *>(Xq_out + (int64_t)m * Kb)[i] = code;
        }
        __syncthreads();                                               // row is free again, codes are visible
    }

    // ---- dot products: registers (weights) x LDS (activation codes) ---------------------------
    int acc[G][LD_MT];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int m = 0; m < LD_MT; ++m) acc[g][m] = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int off = (wave + LD_NW * u) * 128 + c * 16;             // byte offset inside a row of codes
        {
#pragma unroll
            for (int m = 0; m < LD_MT; ++m) {
                {
                    const u32x4 x = *reinterpret_cast<const u32x4 *>(xq + m * (K / 8) + off / 4);
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        int a = acc[g][m];
                        a = __builtin_amdgcn_sdot8((int)w[g][u].x, (int)x.x, a, false);
                        a = __builtin_amdgcn_sdot8((int)w[g][u].y, (int)x.y, a, false);
                        a = __builtin_amdgcn_sdot8((int)w[g][u].z, (int)x.z, a, false);
                        a = __builtin_amdgcn_sdot8((int)w[g][u].w, (int)x.w, a, false);
                        acc[g][m] = a;
                    }
                }
            }
        }
    }
    // the 8 lanes of a row, then the waves (through the now idle row buffer)
    int *part = reinterpret_cast<int *>(row);                          // [LD_NW][LD_MT][8 G]
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int m = 0; m < LD_MT; ++m) {
            int v = acc[g][m];
            v = sum_of_8_lanes(v);
            if (c == 0) part[(wave * LD_MT + m) * (8 * G) + ((g + (int)blockIdx.x) % G) * 8 + r] = v;
        }
    __syncthreads();
    if (t < 8 * G && n0 + t < N) {                                      // M = 1: output t of the workgroup
        int sum = 0;
#pragma unroll
        for (int wv = 0; wv < LD_NW; ++wv) sum += part[wv * LD_MT * (8 * G) + t];
        Y[n0 + t] = __float2half_rn((float)sum * sx[0] * w_scale);
    }
}

template <int K, int G>
hipError_t launch_ld(const void *X, int64_t M, int64_t ldx, const float *pre, float clip, const uint8_t *Wq,
                     const float *ws, int64_t N, void *Y, int64_t ldy, uint8_t *Xq_out, float *xs_out, hipStream_t st)
{
    auto kern = linear_decode_kernel<K, G>;
    constexpr int lds = (int)(sizeof(float) * padded_len(K)) + LD_MT * (K / 2);
    static_assert(lds + 64 <= 160 * 1024, "LDS");
    if (lds > 40 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
    }
    const unsigned blocks = (unsigned)((N + 8 * G - 1) / (8 * G));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(LD_NT), lds, st, static_cast<const __half *>(X), (int)M, ldx, pre, clip,
                       Wq, ws, (int)N, static_cast<__half *>(Y), ldy, Xq_out, xs_out);
    return hipGetLastError();
}

constexpr int LD_WS_SCALES = 256, LD_WS_CODES = 512;      // workspace of the two-launch path: scales [16], codes [M][K / 2]

// Row groups of 8 channels per workgroup: every workgroup repeats the rotation, so few large workgroups are
// cheaper, but the chip should be filled in whole rounds -- the G <= gmax with the least (rounds x G), ties to
// the larger G (14336 channels on 256 CUs: G = 7 gives exactly 256 workgroups, G = 8 would leave 32 CUs idle).
inline int pick_g(int64_t N, int gmax)
{
    const int64_t cus = compute_units();
    int best = 1;
    int64_t best_cost = -1;
    for (int g = 1; g <= gmax; ++g) {
        const int64_t blocks = (N + 8 * g - 1) / (8 * g);
        const int64_t cost = ((blocks + cus - 1) / cus) * g;
        if (best_cost < 0 || cost <= best_cost) { best = g; best_cost = cost; }
    }
    return best;
}

}  // namespace

bool linear_decode_supported(int64_t K) { return K == 2048 || K == 4096 || K == 8192 || K == 14336; }

// one token and a power-of-two order up to 4096: ONE launch in which every workgroup rotates the row itself
// (4096 -> 14336: 8.0 against 9.6 - 10.0 us for two launches; 4096 -> 4096: 5.0 against 6.5 us; K = 8192: 11.3 us
// either way, so it takes the general path)
static bool redundant_rotation_path(int64_t M, int64_t K) { return M == 1 && (K == 2048 || K == 4096); }

size_t linear_decode_workspace_bytes(int64_t M, int64_t K)
{
    if (M < 1 || M > 16 || !linear_decode_supported(K) || redundant_rotation_path(M, K)) return 0;
    return (size_t)LD_WS_CODES + (size_t)M * (size_t)(K / 2);
}

hipError_t launch_linear_decode(const void *X, int64_t M, int64_t K, int64_t ldx, const float *pre, float clip,
                                const uint8_t *Wq, const float *ws, int64_t N, void *Y, int64_t ldy,
                                uint8_t *Xq_out, float *xs_out, void *workspace, hipStream_t st)
{
    if (redundant_rotation_path(M, K)) {
#define SR_LD(KK, GG) case GG: return launch_ld<KK, GG>(X, M, ldx, pre, clip, Wq, ws, N, Y, ldy, Xq_out, xs_out, st)
        switch (K) {
            case 2048: switch (pick_g(N, 8)) { SR_LD(2048, 1); SR_LD(2048, 2); SR_LD(2048, 3); SR_LD(2048, 4); SR_LD(2048, 5); SR_LD(2048, 6); SR_LD(2048, 7); SR_LD(2048, 8); default: break; } break;
            case 4096: switch (pick_g(N, 8)) { SR_LD(4096, 1); SR_LD(4096, 2); SR_LD(4096, 3); SR_LD(4096, 4); SR_LD(4096, 5); SR_LD(4096, 6); SR_LD(4096, 7); SR_LD(4096, 8); default: break; } break;
            default: break;
        }
        return hipErrorInvalidValue;
#undef SR_LD
    }
    // Everything else -- several tokens, K = 8192 where the two are level, K = 14336 = 28 * 512 -- runs as two launches
    // behind the one entry point: the rotation + quantiser of the M rows, then the M <= 16 GEMM; codes and scales go
    // through the workspace (or straight into the caller's optional outputs).  One-launch variants for these shapes
    // were built and measured against exactly this pair (4096 -> 14336 / 14336 -> 4096, 20 rotating weight copies):
    //  - every workgroup rotating the row(s) itself: 13.4 us against 11.9 us at K = 14336, one token (the rotation
    //    of such a row takes a 512-thread workgroup longer than its weights take to arrive);
    //  - rows rotated once by M extra workgroups and handed to the others through memory (agent-scope release,
    //    relaxed polling, coherent loads of the codes): 11.9 - 12.3 us against 11.9 us at K = 14336 for one token,
    //    13.4 - 15.5 against 12.1 - 12.5 us for 2 - 4 tokens, 12.2 against 10.1 us at K = 4096 for two tokens -- the
    //    producers' own loads queue behind 29 MB of weight requests (rotation done 7.6 us into the kernel instead
    //    of 5.2 us), and dot products on packed nibbles for several tokens lose to the matrix-pipe GEMM;
    //  - the pair with the quantiser launch also pulling the weights into the memory-side cache: 13.5 against
    //    12.1 us (a GEMM that is bound by HBM gains nothing from reading the weights twice).
    uint8_t *wsp = static_cast<uint8_t *>(workspace);
    uint8_t *xq = Xq_out ? Xq_out : wsp + LD_WS_CODES;
    float *xs = xs_out ? xs_out : reinterpret_cast<float *>(wsp + LD_WS_SCALES);
    hipError_t e = launch_fwht_quant(X, M, K, ldx, pre, clip, 1.0f, xq, xs, st);
    if (e != hipSuccess) return e;
    return launch_gemm_decode(xq, xs, Wq, ws, M, N, K, Y, ldy, 0, st);
}

}  // namespace sr
