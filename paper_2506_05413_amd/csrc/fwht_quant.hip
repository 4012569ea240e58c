// Online Hadamard rotation fused with per-row symmetric INT4 quantisation.
//
// One workgroup owns one row (a token of X, or an output channel of the transposed,
// smoothed weight during the fold).  The row is converted to fp32, rotated by
// T(v) = v H on chip and quantised; only the packed codes and one scale per row go
// back to memory.  (Paper: online exact Hadamard before the projection, section
// "Methodology"; quantiser Eq. (1) with per-token / per-channel symmetric scales.)
//
// Rotation schedule.  H = (x) of 2x2 Sylvester factors (and H_28 for K = 28 * 2^p);
// Kronecker factors commute, so the butterflies are grouped into passes of up to four
// index bits that a thread can do entirely in registers on 16 values:
//   pass 1   bits 0-3, straight from the global load (16 contiguous fp16 per group)
//   pass 2.. bits 4-7, 8-11, ... gathered from / scattered to an fp32 row in LDS
//   H_28     28 values at stride 2^p per group, as  y_j = S - 2 * sum_{H[i][j]=-1} v_i
// The LDS row is padded by 4 floats per 64 so that every access pattern above is
// bank-conflict free for K = 4096.
#include "fwht_row.h"
#include "gemm_common.h"      // LDS-DMA load, hand-placed waits, fence-free barrier

namespace sr {
namespace {

// F6: Q receives f6 tiles (operands of the FP6-MFMA GEMM) instead of packed nibbles; K % 128 == 0 then.
// STREAM: the grid is smaller than the number of rows; a workgroup walks over rows w, w + gridDim.x, .. and
// fetches its next row while it rotates the current one (gridDim.x % 64 == 0 for F6, so that the row mapping
// below stays what it is for a grid of one workgroup per row).
template <int K, int NT, bool F6, bool GATE = false, bool STREAM = false>
__global__ __launch_bounds__(NT, STREAM ? 2 * NT / 256 : 1) void fwht_quant_kernel(const __half *__restrict__ X, int64_t ldx, int64_t rows,
                                                        const float *__restrict__ pre, float clip,
                                                        float post_scale, uint8_t *__restrict__ Q,
                                                        float *__restrict__ scale_out,
                                                        const __half *__restrict__ gate, int64_t ldg,
                                                        const uint32_t *__restrict__ warm, int64_t warm_lines)
{
    extern __shared__ float row[];
    __shared__ float red[NT / 64];

    const int t = threadIdx.x;
    // warming the memory-side cache for the kernel that follows (see fwht4096_wave_kernel): the threads of the
    // launch share the lines and read one word of each once the workgroup's first row has left its load registers
    uint32_t warm_acc = 0;
    auto warm_lines_now = [&]() {
        if (warm) {
            const int64_t gt = (int64_t)blockIdx.x * NT + t, nt = (int64_t)gridDim.x * NT;
            for (int64_t l = gt; l < warm_lines; l += nt) warm_acc ^= warm[l * 32];
        }
    };
    // F6: the eight rows of a tile block (768 contiguous bytes per 128 codes) should be written from ONE XCD at
    // about the same time, so that its L2 assembles whole lines: workgroups are dealt round-robin to the 8
    // XCDs, so (virtual) workgroup w = 8 a + x (XCD x) takes row r = a % 8 of row block 8 (a / 8) + x.
    auto row_of = [](int64_t w) -> int64_t {
        if constexpr (F6) {
            const int64_t x = w & 7, a = w >> 3;
            return 64 * (a >> 3) + 8 * x + (a & 7);
        } else {
            return w;
        }
    };
    const int64_t total = F6 ? (rows + 63) / 64 * 64 : rows;      // virtual workgroups; F6: some map past the last row
    auto quantise = [&](int64_t m, float amax) {
        // Delta = clip * absmax / 7 (1 for an all-zero row), Eq. (1) with the signed range
        const float delta = (amax == 0.f) ? 1.f : (clip * amax) / 7.f;
        const float inv_delta = 1.f / delta;
        if (t == 0) scale_out[m] = (amax == 0.f) ? 1.f : delta * post_scale;

        if constexpr (F6) {
            // ---- 32 contiguous values -> one 24-byte piece of a tile (the padding of 4 floats per 64 keeps the
            // 16-byte reads of 16 neighbouring threads on distinct banks) -----------------------------------------
            const int64_t row_blocks = (rows + 7) >> 3;
            for (int p = t; p < K / 32; p += NT) quant_store_f6_piece(row + pad(32 * p), inv_delta, Q, row_blocks, m, p);
        } else {
            // ---- quantise 8 contiguous values -> one packed dword ---------------------------------------------
            uint32_t *q = reinterpret_cast<uint32_t *>(Q + m * (int64_t)(K / 2));
            for (int c = t; c < K / 8; c += NT) {
                const float *src = row + pad(8 * c);
                const float4 a = *reinterpret_cast<const float4 *>(src);
                const float4 b = *reinterpret_cast<const float4 *>(src + 4);
                const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
                q[c] = quant_pack8(v, inv_delta);
            }
        }
    };

    if constexpr (!STREAM) {
        const int64_t m = row_of(blockIdx.x);
        if (m >= rows) return;                           // F6: the grid is rounded up to a multiple of 64
        RowLoad<K, NT> ld;
        row_load<K, NT, false, GATE>(X + m * ldx, pre, t, ld, GATE ? gate + m * ldg : nullptr);
        const float amax = rotate_loaded_row_absmax<K, NT, GATE>(ld, pre, row, red, t, warm_lines_now);
        quantise(m, amax);
    } else {
        // (not with a gate row: twice the registers in flight; measured 15 - 25 % slower than one row per
        // workgroup, also with the prefetch moved behind the Paley pass)
        static_assert(!GATE, "the walking variant takes no gate row");
        const int64_t step = gridDim.x;
        int64_t w = blockIdx.x;
        while (w < total && row_of(w) >= rows) w += step;
        if (w >= total) return;
        RowLoad<K, NT> ld;
        {
            const int64_t m = row_of(w);
            row_load<K, NT, false, GATE>(X + m * ldx, pre, t, ld);
        }
        bool first = true;
        for (;;) {
            const int64_t m = row_of(w);
            int64_t wn = w + step;
            while (wn < total && row_of(wn) >= rows) wn += step;
            const bool more = wn < total;                // uniform over the workgroup
            // the next row is requested as soon as this one has left the registers; the smoothing factors,
            // which come from L2, only after the register-hungry passes
            const int64_t mn = more ? row_of(wn) : m;
            const float amax = rotate_loaded_row_absmax<K, NT, GATE>(ld, pre, row, red, t, [&]() {
                if (more) row_load<K, NT, false, GATE, 1>(X + mn * ldx, pre, t, ld);
                if (first) warm_lines_now();
            });
            first = false;
            if (more) row_load<K, NT, false, GATE, 2>(X + mn * ldx, pre, t, ld);
            quantise(m, amax);
            if (!more) break;
            w = wn;
            __syncthreads();                             // the row buffer is rewritten by the next first pass
        }
    }
    asm volatile("" ::"v"(warm_acc));                    // keeps the warming loads; they returned long ago
}

// ------------------------------------------------------------------------------------------
// Extended row kernel: the same rotation + quantiser with three optional extras
//   gate       x = silu(gate) * X in fp32 before smoothing (the down-projection input of the gated
//              FFN, paper Fig. 2: sigma(gate) (.) up, then 1/s, Hadamard, quantiser)
//   had_mask   head-wise Hadamard: only the selected index bits are transformed (power-of-two K)
//   grid       per-row clipping ratio by linear search over the squared quantisation error
//              (paper, "Quantization" settings for the weights), first minimum in grid order
// Kept apart from the plain kernel so that the hot path carries none of these branches.
// ------------------------------------------------------------------------------------------
template <int K, int NT, bool F6>
__global__ __launch_bounds__(NT) void fwht_quant_ex_kernel(const __half *__restrict__ X, int64_t ldx, int64_t rows,
                                                           const float *__restrict__ pre, float clip,
                                                           float post_scale, uint8_t *__restrict__ Q,
                                                           float *__restrict__ scale_out, const RowExtras ex)
{
    constexpr bool KRON = !is_pow2(K);
    constexpr int P2 = KRON ? K / 28 : K;
    constexpr int LOGP = ilog2(P2);
    constexpr int NW = NT / 64;

    extern __shared__ float row[];
    __shared__ float red[NW];
    __shared__ double err_w[kMaxClipGrid][NW];

    const int t = threadIdx.x;
    int64_t m = blockIdx.x;
    if constexpr (F6) {                                  // rows of a tile block from one XCD (see fwht_quant_kernel)
        const int64_t w = blockIdx.x, x8 = w & 7, a = w >> 3;
        m = 64 * (a >> 3) + 8 * x8 + (a & 7);
        if (m >= rows) return;
    }
    const __half *x = X + m * ldx;
    const __half *gt = ex.gate ? ex.gate + m * ex.ldg : nullptr;
    const uint32_t mask = KRON ? 0xFFFFFFFFu : ex.had_mask;

    // ---- pass 1: bits 0..3 from global ------------------------------------------------
    for (int g = t; g < K / 16; g += NT) {
        union { uint4 u[2]; __half h[16]; } raw, graw;
        raw.u[0] = *reinterpret_cast<const uint4 *>(x + 16 * g);
        raw.u[1] = *reinterpret_cast<const uint4 *>(x + 16 * g + 8);
        float v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = __half2float(raw.h[e]);
        if (gt) {
            graw.u[0] = *reinterpret_cast<const uint4 *>(gt + 16 * g);
            graw.u[1] = *reinterpret_cast<const uint4 *>(gt + 16 * g + 8);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float gv = __half2float(graw.h[e]);
                // silu(g) = g / (1 + exp(-g)); exp(-g) = inf for very negative g gives g * 0 = -0
                v[e] *= gv * __builtin_amdgcn_rcpf(1.f + __expf(-gv));
            }
        }
        if (pre) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 s = *reinterpret_cast<const float4 *>(pre + 16 * g + 4 * q);
                v[4 * q + 0] *= s.x; v[4 * q + 1] *= s.y; v[4 * q + 2] *= s.z; v[4 * q + 3] *= s.w;
            }
        }
        butterflies_masked<4>(v, mask & 15u);
        float *dst = row + pad(16 * g);
#pragma unroll
        for (int q = 0; q < 4; ++q)
            *reinterpret_cast<float4 *>(dst + 4 * q) = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
    }
    __syncthreads();

    lds_passes_masked<K, NT, 4, LOGP>(row, t, mask);

    if constexpr (KRON) {
        for (int g = t; g < P2; g += NT) {
            float v[28], o[28];
            float *col = row + pad(g);
#pragma unroll
            for (int i = 0; i < 28; ++i) v[i] = col[strided<P2>(g, i)];
            h28_program(v, o);
#pragma unroll
            for (int j = 0; j < 28; ++j) col[strided<P2>(g, j)] = o[j];
        }
        __syncthreads();
    }

    // ---- row absmax (own sweep: the last transforming pass depends on the mask) -----------------
    float amax = 0.f;
    for (int c = t; c < K / 8; c += NT) {
        const float *src = row + pad(8 * c);
        const float4 a = *reinterpret_cast<const float4 *>(src);
        const float4 b = *reinterpret_cast<const float4 *>(src + 4);
        amax = fmaxf(amax, fmaxf(fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))),
                                 fmaxf(fmaxf(fabsf(b.x), fabsf(b.y)), fmaxf(fabsf(b.z), fabsf(b.w)))));
    }
    amax = max_of_wave(amax);
    if ((t & 63) == 0) red[t >> 6] = amax;
    __syncthreads();
    amax = red[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) amax = fmaxf(amax, red[w]);

    // ---- clipping-ratio search: err_r = sum_j (y_j - Delta_r * code_r(y_j))^2 for every ratio -------
    if (ex.n_grid > 0 && amax != 0.f) {
        for (int i = 0; i < ex.n_grid; ++i) {
            const float d = (ex.grid[i] * amax) / 7.f;
            const float inv = 1.f / d;
            double acc = 0.0;
            for (int c = t; c < K / 8; c += NT) {
                const float *src = row + pad(8 * c);
                const float4 a = *reinterpret_cast<const float4 *>(src);
                const float4 b = *reinterpret_cast<const float4 *>(src + 4);
                const float y[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
                float part = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float code = fminf(fmaxf(rintf(y[e] * inv), -8.f), 7.f);
                    const float r = fmaf(-d, code, y[e]);
                    part = fmaf(r, r, part);
                }
                acc += (double)part;
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
            if ((t & 63) == 0) err_w[i][t >> 6] = acc;
        }
        __syncthreads();
        double best = 0.0;
        int best_i = 0;
        for (int i = 0; i < ex.n_grid; ++i) {               // every thread takes the same decision
            double e = 0.0;
#pragma unroll
            for (int w = 0; w < NW; ++w) e += err_w[i][w];
            if (i == 0 || e < best) { best = e; best_i = i; }
        }
        clip = ex.grid[best_i];
    } else if (ex.n_grid > 0) {
        clip = ex.grid[0];
    }
    if (ex.ratio_out && t == 0) ex.ratio_out[m] = clip;

    const float delta = (amax == 0.f) ? 1.f : (clip * amax) / 7.f;
    const float inv_delta = 1.f / delta;
    if (t == 0) scale_out[m] = (amax == 0.f) ? 1.f : delta * post_scale;

    if constexpr (F6) {
        for (int p = t; p < K / 32; p += NT) quant_store_f6_piece(row + pad(32 * p), inv_delta, Q, (rows + 7) >> 3, m, p);
    } else {
        uint32_t *q = reinterpret_cast<uint32_t *>(Q + m * (int64_t)(K / 2));
        for (int c = t; c < K / 8; c += NT) {
            const float *src = row + pad(8 * c);
            const float4 a = *reinterpret_cast<const float4 *>(src);
            const float4 b = *reinterpret_cast<const float4 *>(src + 4);
            const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
            q[c] = quant_pack8(v, inv_delta);
        }
    }
}

// ------------------------------------------------------------------------------------------
// K = 4096: one WAVE per row, no workgroup barriers.  A lane holds 64 fp32 values, so six index
// bits are butterflied in registers at a time and only one transposition separates the two
// halves of the transform:
//   phase 1  lane l loads the 16-byte chunks l, l+64, ..: registers = index bits {0,1,2,9,10,11}
//   LDS      wave-private transposition (row padded by 8 floats per 512: conflict-free both ways)
//   phase 2  lane (e = l & 7, j = l >> 3) holds elements 512 j + 8 r + e: registers = bits 3..8
//   row absmax by a wave reduction, Delta, then back through LDS to the natural order, where a
//   lane quantises 8 consecutive values into one packed dword.
// ------------------------------------------------------------------------------------------

// MASKED: head-wise transform -- only the index bits set in had_mask are butterflied (uniform branches).
// STAGED (with factors, full transform): the 16 KB of smoothing factors reach the four waves of a workgroup through
// LDS -- ONE copy per workgroup by LDS-DMA instead of 16 vector loads per wave, a quarter of the traffic on the
// CU's vector-memory path, which every row load of the launch has to share.  The copies are inline assembly with a
// hand-counted wait, so that the order (factors, then the row) and the wait (factors have landed while the row is
// still in flight) are what is written here, not what the compiler's scheduler makes of them.
template <bool HAS_PRE, bool F6, bool MASKED = false, bool STAGED = false>
__global__ __launch_bounds__(256) void fwht4096_wave_kernel(const __half *__restrict__ X, int64_t ldx, int64_t rows,
                                                            const float *__restrict__ pre, float clip, float post_scale,
                                                            uint8_t *__restrict__ Q, float *__restrict__ scale_out,
                                                            uint32_t had_mask, const uint32_t *__restrict__ warm,
                                                            int64_t warm_lines)
{
    constexpr int K = 4096, ROWF = F6 ? K + 576 : K + 64;   // floats per wave-private row incl. padding
    extern __shared__ __attribute__((aligned(16))) float smem_rows[];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int64_t m = (int64_t)blockIdx.x * 4 + wave;
    if constexpr (F6) {
        // both halves of a tile block (8 rows) from the same XCD: workgroup w = 8 a + x (XCD x) takes half
        // a % 2 of row block 8 (a / 2) + x (see the workgroup-per-row kernel)
        const int64_t w = blockIdx.x, x = w & 7, a = w >> 3;
        m = 8 * (8 * (a >> 1) + x) + 4 * (a & 1) + wave;
    }
    static_assert(!STAGED || (HAS_PRE && !MASKED), "the staged variant is the plain transform with factors");
    if constexpr (!STAGED) {
        if (m >= rows) return;                           // no barrier below: waves are independent
    }
    float *buf = smem_rows + wave * ROWF;
    const __half *x = X + m * ldx;

    // ---- phase 1 --------------------------------------------------------------------------
    // every load of the row first (the scheduling barrier keeps the compiler from sinking each load to its use,
    // which serialised the memory round trips), then the arithmetic, chunk by chunk as the data arrives
    uint4 rx[8];
    u32x4 rxa[8];                                        // STAGED: the row as loaded by inline assembly
    float4 rs[8][2];
    if constexpr (STAGED) {
        const bool active = m < rows;                    // a wave past the last row still helps with the factors
        // wave w copies KB 4 w .. 4 w + 3 of the factors into the staging area, which overlays the row buffers
        // (nobody writes those before the second barrier).  KB q = half h = q & 1 of the 512 factors j = q >> 1:
        // lane l fetches the four factors 512 j + 8 l + 4 h .., so that the reads below are contiguous per lane.
        const uint32_t stage = (uint32_t)(uintptr_t)smem_rows;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int q = __builtin_amdgcn_readfirstlane(4 * wave + i);
            dma16(reinterpret_cast<const uint8_t *>(pre), (uint32_t)((512 * (q >> 1) + 8 * lane + 4 * (q & 1)) * 4),
                  (uint32_t)__builtin_amdgcn_readfirstlane((int)(stage + q * 1024)));
        }
        // The row's loads are inline assembly too: ordinary loads from a read-only argument float freely in the
        // compiler's schedule (it sank them below both barriers, past the wait that counts on them).  The compiler
        // takes rxa[] for defined where the statement stands; every use goes through the wait statements below.
        const uint64_t xa = (uint64_t)(uintptr_t)(active ? x : X);          // wave-uniform: into scalar registers
        const uint32_t xlo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)xa);
        const uint32_t xhi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(xa >> 32));
        const __half *xr = reinterpret_cast<const __half *>((uint64_t)xlo | ((uint64_t)xhi << 32));
#pragma unroll
        for (int j = 0; j < 8; ++j)
            asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(rxa[j]) : "v"((uint32_t)((512 * j + 8 * lane) * 2)), "s"(xr) : "memory");
        wait_vmcnt<8>();
        barrier_nofence();                               // all 16 KB of factors are in LDS
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            rs[j][0] = *reinterpret_cast<const float4 *>(reinterpret_cast<const uint8_t *>(smem_rows) + (2 * j) * 1024 + lane * 16);
            rs[j][1] = *reinterpret_cast<const float4 *>(reinterpret_cast<const uint8_t *>(smem_rows) + (2 * j + 1) * 1024 + lane * 16);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        barrier_nofence();                               // every wave holds its factors: the row buffers are free
        if (!active) {
            wait_vmcnt<0>();                             // (its loads read row 0; nothing may be in flight at the end)
            return;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            rx[j] = *reinterpret_cast<const uint4 *>(x + 512 * j + 8 * lane);
            if (HAS_PRE) {
                rs[j][0] = *reinterpret_cast<const float4 *>(pre + 512 * j + 8 * lane);
                rs[j][1] = *reinterpret_cast<const float4 *>(pre + 512 * j + 8 * lane + 4);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    float v[64];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if constexpr (STAGED) {
            // chunk j has landed once at most 7 - j younger loads are outstanding (loads complete in order)
            if (j == 0) asm volatile("s_waitcnt vmcnt(7)" : "+v"(rxa[0]));
            if (j == 1) asm volatile("s_waitcnt vmcnt(6)" : "+v"(rxa[1]));
            if (j == 2) asm volatile("s_waitcnt vmcnt(5)" : "+v"(rxa[2]));
            if (j == 3) asm volatile("s_waitcnt vmcnt(4)" : "+v"(rxa[3]));
            if (j == 4) asm volatile("s_waitcnt vmcnt(3)" : "+v"(rxa[4]));
            if (j == 5) asm volatile("s_waitcnt vmcnt(2)" : "+v"(rxa[5]));
            if (j == 6) asm volatile("s_waitcnt vmcnt(1)" : "+v"(rxa[6]));
            if (j == 7) asm volatile("s_waitcnt vmcnt(0)" : "+v"(rxa[7]));
            rx[j] = make_uint4(rxa[j][0], rxa[j][1], rxa[j][2], rxa[j][3]);
        }
        union { uint4 u; half2v h[4]; } raw;
        raw.u = rx[j];
        float f[8];
        if (HAS_PRE) {
            const float4 s0 = rs[j][0], s1 = rs[j][1];
            f[0] = s0.x; f[1] = s0.y; f[2] = s0.z; f[3] = s0.w;
            f[4] = s1.x; f[5] = s1.y; f[6] = s1.z; f[7] = s1.w;
        }
        if constexpr (MASKED) {                         // index bit 0 may be unselected: values as they are
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                v[8 * j + e] = (float)raw.h[e >> 1][e & 1];
                if (HAS_PRE) v[8 * j + e] *= f[e];
            }
        } else {                                        // conversion, factor and index bit 0 in one go
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (HAS_PRE) pair_level(raw.h[e], f[2 * e], f[2 * e + 1], v[8 * j + 2 * e], v[8 * j + 2 * e + 1]);
                else pair_level(raw.h[e], v[8 * j + 2 * e], v[8 * j + 2 * e + 1]);
            }
        }
        // (STAGED: keeps the arithmetic of chunk j between the waits for chunks j and j + 1 -- the compiler
        // otherwise gathers the eight waits in front of all of it)
        if constexpr (STAGED) {
            float *vj = v + 8 * j;
            float blk[8] = {vj[0], vj[1], vj[2], vj[3], vj[4], vj[5], vj[6], vj[7]};
            butterflies_from<3, 2>(blk);                 // index bits 1, 2 inside the chunk, as soon as it is there
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                vj[e] = blk[e];
                asm volatile("" : "+v"(vj[e]));          // pins the arithmetic here (it would be sunk to its first use)
            }
        }
    }
    if constexpr (MASKED) butterflies_masked<6>(v, (had_mask & 7u) | (((had_mask >> 9) & 7u) << 3));   // register bits = index bits 0,1,2,9,10,11
    else if constexpr (STAGED) butterflies_from<6, 8>(v);   // bits 1, 2 were done chunk by chunk
    else butterflies_from<6, 2>(v);
    // Warming the memory-side cache for the kernel that follows (its weights): the waves of the launch share the
    // 128-byte lines of [warm, warm + 128 warm_lines) and read one word of each -- with ordinary loads, so that the
    // lines are allocated -- now that the row's own loads have returned; the words are never looked at.
    uint32_t warm_acc = 0;
    if (warm) {
        const int64_t gw = (int64_t)blockIdx.x * 4 + wave, nw = (int64_t)gridDim.x * 4;
        for (int64_t l = gw * 64 + lane; l < warm_lines; l += nw * 64) warm_acc ^= warm[l * 32];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        float *d = buf + 520 * j + 8 * lane;             // element 512 j + 8 l + e lives at 520 j + 8 l + e
        *reinterpret_cast<float4 *>(d) = make_float4(v[8 * j], v[8 * j + 1], v[8 * j + 2], v[8 * j + 3]);
        *reinterpret_cast<float4 *>(d + 4) = make_float4(v[8 * j + 4], v[8 * j + 5], v[8 * j + 6], v[8 * j + 7]);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");

    // ---- phase 2 --------------------------------------------------------------------------
    const float *src = buf + 520 * (lane >> 3) + (lane & 7);
#pragma unroll
    for (int r = 0; r < 64; ++r) v[r] = src[8 * r];
    if constexpr (MASKED) butterflies_masked<6>(v, (had_mask >> 3) & 63u);                            // index bits 3..8
    else butterflies<6>(v);
    float amax = 0.f;
#pragma unroll
    for (int r = 0; r < 64; r += 2) amax = fmaxf(fmaxf(amax, fabsf(v[r])), fabsf(v[r + 1]));
    amax = max_of_wave(amax);
    const float delta = (amax == 0.f) ? 1.f : (clip * amax) / 7.f;
    const float inv_delta = 1.f / delta;
    if (lane == 0) scale_out[m] = (amax == 0.f) ? 1.f : delta * post_scale;

    if constexpr (F6) {
        // ---- f6 tiles: every lane converts two pieces of 32 consecutive values (quant_store_f6_piece) -----------
        // Back through LDS with 4 floats of padding per 32 and 8 per 512 (element i at i + 4 (i >> 5) + 8 (i >> 9)):
        // the scattered writes below and the 16-byte reads of 32 values per lane are both free of bank conflicts.
        float *dst = buf + 584 * (lane >> 3) + (lane & 7);
#pragma unroll
        for (int r = 0; r < 64; ++r) dst[8 * r + 4 * (r >> 2)] = v[r];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        const int64_t row_blocks = (rows + 7) >> 3;
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int p = lane + 64 * pass;                  // piece p of the row: k = 32 p .. 32 p + 31
            quant_store_f6_piece(buf + 36 * p + 8 * (p >> 4), inv_delta, Q, row_blocks, m, p);
        }
    } else {
        float *dst = buf + 520 * (lane >> 3) + (lane & 7);
#pragma unroll
        for (int r = 0; r < 64; ++r) dst[8 * r] = v[r];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");

        // ---- quantise: 8 consecutive values -> one dword ---------------------------------------
        uint32_t *q = reinterpret_cast<uint32_t *>(Q + m * (int64_t)(K / 2));
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float *s8 = buf + 520 * j + 8 * lane;
            const float4 a = *reinterpret_cast<const float4 *>(s8);
            const float4 b = *reinterpret_cast<const float4 *>(s8 + 4);
            const float y[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
            q[64 * j + lane] = quant_pack8(y, inv_delta);
        }
    }
    asm volatile("" ::"v"(warm_acc));                    // keeps the warming loads; they returned long ago
}

// ------------------------------------------------------------------------------------------
// K = 4096, one row per workgroup of four waves, two passes of SIX index bits each: four bits in registers
// (16 values per thread) and two across neighbouring lanes by DPP.  A single wave of this chip issues a vector
// instruction every ~5 cycles however independent its instructions are, and two waves per SIMD double that: the
// wave-per-row kernel above leaves a row's ~1150 instructions to ONE wave (2.5 us after the row has arrived, with
// two waves per SIMD at 2048 rows), this one to four waves of ~300 each, eight waves per SIMD -- with the same LDS
// traffic (the row goes through LDS twice), where the general workgroup-per-row kernel needs three passes of four
// bits and three round trips.
//
// Thread t holds x[16 t .. 16 t + 15]: index bits 0..3 in registers, bits 4, 5 in lane bits 0, 1.  A butterfly
// across lanes is ONE instruction per value, v <- v + c * v[partner] (v_fmac_f32 with a DPP source, c = +1 in
// the lane whose bit is clear, -1 in the other): the lane with the bit clear gets a + b, the other b - a -- the
// difference with its sign flipped.  The flip is not undone on the spot: every later step is linear and pairs
// only lanes with equal flips, so a value simply carries the sign (-1)^(number of set bits among the lane bits
// used so far); row maxima ignore it, and the quantiser multiplies by 1/Delta anyway, so it multiplies by
// -1/Delta where the sign is -1 (exact).  Pass 2 reads c + 64 r + 1024 q for r = 0..15 (c = t >> 2: index bits
// 0..5, q = t & 3: bits 10, 11 in lane bits 0, 1; registers: bits 6..9), all written by threads with lane bits
// 0, 1 = (t >> 6) & 3 -- one sign per thread from pass 1 -- and writes them back where it read them.
// LDS layout: element i at i + 4 (i >> 5) + 8 (i >> 10) floats: the 16-byte writes of pass 1, the 4-byte
// accesses of pass 2 (a half-wave covers eight consecutive c and four q: banks c + 8 q, all 32) and the 16-byte
// reads of the quantiser are all free of bank conflicts.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ int wg4096_pos(int i) { return i + ((i >> 5) << 2) + ((i >> 10) << 3); }
constexpr int kWg4096Floats = 4096 + 4 * 128 + 8 * 4;

// v[e] += c * v[e] of the lane with lane bit 0 (QP = 0xB1) or lane bit 1 (QP = 0x4E) flipped, for 16 values.
// (Inline assembly: the two wait states a DPP read needs after a vector write of the same register are given
// by the s_nop in front; inside the block no instruction reads what its predecessor wrote.)
template <int QP>
__device__ __forceinline__ void lane_butterfly16(float (&v)[16], float c)
{
    static_assert(QP == 0xB1 || QP == 0x4E, "quad permutations [1,0,3,2] and [2,3,0,1]");
#define SR_DPP_FMAC(i) "v_fmac_f32_dpp %" #i ", %" #i ", %16 quad_perm:[%17,%18,%19,%20] row_mask:0xf bank_mask:0xf\n\t"
    asm("s_nop 1\n\t"
        SR_DPP_FMAC(0) SR_DPP_FMAC(1) SR_DPP_FMAC(2) SR_DPP_FMAC(3) SR_DPP_FMAC(4) SR_DPP_FMAC(5) SR_DPP_FMAC(6) SR_DPP_FMAC(7)
        SR_DPP_FMAC(8) SR_DPP_FMAC(9) SR_DPP_FMAC(10) SR_DPP_FMAC(11) SR_DPP_FMAC(12) SR_DPP_FMAC(13) SR_DPP_FMAC(14) SR_DPP_FMAC(15)
        : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]),
          "+v"(v[8]), "+v"(v[9]), "+v"(v[10]), "+v"(v[11]), "+v"(v[12]), "+v"(v[13]), "+v"(v[14]), "+v"(v[15])
        : "v"(c), "n"(QP & 3), "n"((QP >> 2) & 3), "n"((QP >> 4) & 3), "n"((QP >> 6) & 3));
#undef SR_DPP_FMAC
}

// (Measured and dropped: 2, 4 or 8 rows per workgroup, one after the other, all loads issued up front and two LDS
// buffers taking turns, so that a row would arrive while the one before it is computed -- 9.7 / 10.8 / 13.8 us
// against 9.0 us at 2048 rows, worse at every row count below 16384.)
template <bool HAS_PRE, bool F6>
__global__ __launch_bounds__(256) void fwht4096_wg_kernel(const __half *__restrict__ X, int64_t ldx, int64_t rows,
                                                          const float *__restrict__ pre, float clip, float post_scale,
                                                          uint8_t *__restrict__ Q, float *__restrict__ scale_out,
                                                          const uint32_t *__restrict__ warm, int64_t warm_lines)
{
    constexpr int K = 4096;
    extern __shared__ __attribute__((aligned(16))) float smem_rows[];
    __shared__ float red[4];
    float *row = smem_rows;
    const int t = threadIdx.x, lane = t & 63;
    int64_t m = blockIdx.x;
    if constexpr (F6) {
        // the eight rows of a tile block from the same XCD: workgroup w = 8 a + x (XCD x) takes row a % 8 of
        // block 8 (a / 8) + x
        const int64_t w = blockIdx.x, x = w & 7, a = w >> 3;
        m = 8 * (8 * (a >> 3) + x) + (a & 7);
    }
    if (m >= rows) return;                               // the whole workgroup: no barrier is left behind
    const __half *x = X + m * ldx;

    // ---- pass 1: index bits 0..5 ------------------------------------------------------------------
    uint4 rx[2];
    float4 rs[4];
    rx[0] = *reinterpret_cast<const uint4 *>(x + 16 * t);
    rx[1] = *reinterpret_cast<const uint4 *>(x + 16 * t + 8);
    if (HAS_PRE) {
#pragma unroll
        for (int q = 0; q < 4; ++q) rs[q] = *reinterpret_cast<const float4 *>(pre + 16 * t + 4 * q);
    }
    const float c0 = (lane & 1) ? -1.f : 1.f, c1 = (lane & 2) ? -1.f : 1.f;
    float v[16];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        union { uint4 u; half2v h[4]; } raw;
        raw.u = rx[j];
        if (HAS_PRE) {
            const float4 s0 = rs[2 * j], s1 = rs[2 * j + 1];
            pair_level(raw.h[0], s0.x, s0.y, v[8 * j], v[8 * j + 1]);
            pair_level(raw.h[1], s0.z, s0.w, v[8 * j + 2], v[8 * j + 3]);
            pair_level(raw.h[2], s1.x, s1.y, v[8 * j + 4], v[8 * j + 5]);
            pair_level(raw.h[3], s1.z, s1.w, v[8 * j + 6], v[8 * j + 7]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) pair_level(raw.h[e], v[8 * j + 2 * e], v[8 * j + 2 * e + 1]);
        }
    }
    butterflies_from<4, 2>(v);
    lane_butterfly16<0xB1>(v, c0);
    lane_butterfly16<0x4E>(v, c1);
    {
        float *d = row + wg4096_pos(16 * t);
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<float4 *>(d + 4 * q) = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
    }
    // (barriers without the fence of __syncthreads: that would also wait for the warming loads below)
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    barrier_nofence();
    // warming the memory-side cache for the kernel that follows (see fwht4096_wave_kernel): one word of every
    // 128-byte line of the region, shared among the threads of the launch, ordinary loads, never looked at
    uint32_t warm_acc = 0;
    if (warm) {
        const int64_t nthreads = (int64_t)gridDim.x * 256;
        for (int64_t l = (int64_t)blockIdx.x * 256 + t; l < warm_lines; l += nthreads) warm_acc ^= warm[l * 32];
    }

    // ---- pass 2: index bits 6..11 -----------------------------------------------------------------
    float *col = row + wg4096_pos((t >> 2) + 1024 * (t & 3));
#pragma unroll
    for (int r = 0; r < 16; ++r) v[r] = col[72 * r];     // element + 64 r sits 64 r + 4 * 2 r floats further
    butterflies<4>(v);
    lane_butterfly16<0xB1>(v, c0);
    lane_butterfly16<0x4E>(v, c1);
    float amax = 0.f;
#pragma unroll
    for (int r = 0; r < 16; r += 2) amax = fmaxf(fmaxf(amax, fabsf(v[r])), fabsf(v[r + 1]));
#pragma unroll
    for (int r = 0; r < 16; ++r) col[72 * r] = v[r];     // the same thread read these: nothing to wait for
    amax = max_of_wave(amax);
    if (lane == 0) red[t >> 6] = amax;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    barrier_nofence();
    amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float delta = (amax == 0.f) ? 1.f : (clip * amax) / 7.f;
    const float inv_delta = 1.f / delta;
    if (t == 0) scale_out[m] = (amax == 0.f) ? 1.f : delta * post_scale;

    // ---- quantise.  The 16 values of group g = i >> 4 carry the sign (-1)^(popcount(g & 3) + popcount(g >> 6)):
    // lane bits 0, 1 of their writer in pass 1 were g & 3, in pass 2 g >> 6.
    auto signed_inv = [&](int g) { return (__builtin_popcount((g & 3) | ((g >> 6) << 2)) & 1) ? -inv_delta : inv_delta; };
    if constexpr (F6) {
        if (t < K / 32) {
            const float *s32 = row + 36 * t + 8 * (t >> 5);
            quant_store_f6_piece(s32, signed_inv(2 * t), signed_inv(2 * t + 1), Q, (rows + 7) >> 3, m, t);
        }
    } else {
        const float *s16 = row + wg4096_pos(16 * t);
        const float sd = signed_inv(t);
        uint32_t *q = reinterpret_cast<uint32_t *>(Q + m * (int64_t)(K / 2));
        uint32_t w2[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const float4 a = *reinterpret_cast<const float4 *>(s16 + 8 * h);
            const float4 b = *reinterpret_cast<const float4 *>(s16 + 8 * h + 4);
            const float y[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
            w2[h] = quant_pack8(y, sd);
        }
        *reinterpret_cast<uint2 *>(q + 2 * t) = make_uint2(w2[0], w2[1]);
    }
    asm volatile("" ::"v"(warm_acc));                    // keeps the warming loads; they returned long ago
}

__global__ __launch_bounds__(256) void fill_f32_kernel(float *__restrict__ dst, int64_t n, float value)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = value;
}

// One workgroup per row -- or, for K = 14336 with 256 threads, no gate row and at least two rounds of rows, as many
// workgroups as the chip holds at once (the fp32 row in LDS allows two per CU), each walking over rows and
// fetching its next row while it works on the current one (2048 rows: 36.2 -> 34.4 us, 16384: 264 -> 243 us).
template <int K, int NT, bool F6, bool GATE>
hipError_t launch_row_kernel(const void *X, int64_t rows, int64_t ldx, const float *pre, float clip, float post_scale,
                             uint8_t *Q, float *scale_out, const __half *gate, int64_t ldg, hipStream_t st,
                             const void *warm = nullptr, size_t warm_bytes = 0)
{
    constexpr size_t lds = sizeof(float) * padded_len(K);
    const int64_t total = F6 ? (rows + 63) / 64 * 64 : rows;
    int64_t grid = total;
    bool stream = false;
    if constexpr (K == 14336 && NT == 256 && !GATE) {
        const int64_t resident = (int64_t)compute_units() * (int64_t)(160 * 1024 / lds) / 64 * 64;
        stream = resident >= 64 && total >= 2 * resident;
        if (int64_t f; tuned(kTuneFwhtStream, f)) stream = resident >= 64 && f != 0;
        if (stream) grid = resident < total ? resident : total;
    }
    auto kern = stream ? fwht_quant_kernel<K, NT, F6, GATE, (K == 14336 && NT == 256 && !GATE)> : fwht_quant_kernel<K, NT, F6, GATE, false>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    // the hint is honoured from 256 workgroups on (a launch of a few rows cannot move megabytes on the side)
    const bool warms = warm && warm_bytes >= 128 && grid >= 256;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NT), lds, st,
                       static_cast<const __half *>(X), ldx, rows, pre, clip, post_scale, Q, scale_out, gate, ldg,
                       warms ? static_cast<const uint32_t *>(warm) : nullptr, (int64_t)(warm_bytes / 128));
    return hipGetLastError();
}

template <int K, bool F6 = false, int NT_FORCE = 0>
hipError_t launch_one(const void *X, int64_t rows, int64_t ldx, const float *pre, float clip,
                      float post_scale, uint8_t *Q, float *scale_out, hipStream_t st,
                      const void *warm = nullptr, size_t warm_bytes = 0)
{
    constexpr int groups = K / 16;
    constexpr int NT = NT_FORCE ? NT_FORCE : (groups >= 256 ? 256 : (groups >= 128 ? 128 : 64));
    // Long rows: more threads per row where they pay (measured, one row / 2048 rows, 256 threads against the
    // choice below).  K = 8192: 5.6 -> 4.1 us / 19.2 -> 16.3 us; 16384: 9.0 -> 6.0 / 46.6 -> 34.4; 28672 (one
    // workgroup per CU whatever its size): 23.5 -> 9.7 / 257 -> 87; 32768: 24.9 -> 19.9 / 276 -> 222.  K = 14336
    // and 7168 only while every row still has a CU to itself (14336: 8.0 -> 6.1 us for one row with 1024 threads,
    // 9.7 -> 7.9 us for 256 rows with 512, but 42 -> 57 us for 2048 rows: two small workgroups per CU overlap
    // better than one large one).
    if constexpr (NT_FORCE == 0) {
        if constexpr (K == 8192) return launch_one<K, F6, 512>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st);
        if constexpr (K == 16384 || K == 28672 || K == 32768)
            return launch_one<K, F6, 1024>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st);
        if constexpr (K == 14336) {
            if (rows <= 64) return launch_one<K, F6, 1024>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st);
            if (rows <= 256) return launch_one<K, F6, 512>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st);
        }
        if constexpr (K == 7168) {
            if (rows <= 512) return launch_one<K, F6, 512>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st);
        }
    }
    return launch_row_kernel<K, NT, F6, false>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, nullptr, 0, st, warm, warm_bytes);
}

// silu(gate) * x in front of the plain kernel (no head mask, no clip search)
template <int K, bool F6 = false, int NT_FORCE = 0>
hipError_t launch_one_gated(const void *X, int64_t rows, int64_t ldx, const float *pre, float clip, float post_scale,
                            uint8_t *Q, float *scale_out, const __half *gate, int64_t ldg, hipStream_t st)
{
    constexpr int groups = K / 16;
    constexpr int NT = NT_FORCE ? NT_FORCE : (groups >= 256 ? 256 : (groups >= 128 ? 128 : 64));
    if constexpr (NT_FORCE == 0) {                          // threads per row as in launch_one
        if constexpr (K == 8192) return launch_one_gated<K, F6, 512>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, gate, ldg, st);
        if constexpr (K == 16384 || K == 28672)
            return launch_one_gated<K, F6, 1024>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, gate, ldg, st);
        if constexpr (K == 14336) {
            if (rows <= 64) return launch_one_gated<K, F6, 1024>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, gate, ldg, st);
            if (rows <= 256) return launch_one_gated<K, F6, 512>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, gate, ldg, st);
        }
        if constexpr (K == 7168) {
            if (rows <= 512) return launch_one_gated<K, F6, 512>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, gate, ldg, st);
        }
    }
    return launch_row_kernel<K, NT, F6, true>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, gate, ldg, st);
}

template <int K, bool F6 = false>
hipError_t launch_one_ex(const void *X, int64_t rows, int64_t ldx, const float *pre, float clip,
                         float post_scale, uint8_t *Q, float *scale_out, const RowExtras &ex, hipStream_t st)
{
    constexpr int groups = K / 16;
    constexpr int NT = groups >= 256 ? 256 : (groups >= 128 ? 128 : 64);
    constexpr size_t lds = sizeof(float) * padded_len(K);
    auto kern = fwht_quant_ex_kernel<K, NT, F6>;
    if (lds > 40 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const unsigned grid = F6 ? (unsigned)((rows + 63) / 64 * 64) : (unsigned)rows;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), lds, st,
                       static_cast<const __half *>(X), ldx, rows, pre, clip, post_scale, Q, scale_out, ex);
    return hipGetLastError();
}

}  // namespace

// K = 4096: below this many rows the wave-per-row kernel leaves most of the chip idle (4 rows per workgroup)
// and the workgroup-per-row kernel has the shorter critical path.
constexpr int64_t kWaveKernelMinRows = 1024;   // measured: 3.3 - 4.8 us against 4.2 - 5.9 us up to 512 rows, equal at 1024
constexpr int64_t kWgKernelMaxRows = 3072;     // the two-pass workgroup-per-row kernel up to here (see launch_fwht_quant)

template <bool HAS_PRE, bool F6, bool MASKED = false, bool STAGED = false>
hipError_t launch_wave4096(const void *X, int64_t rows, int64_t ldx, const float *pre, float clip, float post_scale,
                           uint8_t *Q, float *scale_out, hipStream_t st, uint32_t had_mask = 0xFFFFFFFFu,
                           const void *warm = nullptr, size_t warm_bytes = 0)
{
    constexpr size_t lds = 4 * (4096 + (F6 ? 576 : 64)) * sizeof(float);
    const unsigned blocks = F6 ? (unsigned)((rows + 63) / 64 * 16) : (unsigned)((rows + 3) / 4);
    auto kern = fwht4096_wave_kernel<HAS_PRE, F6, MASKED, STAGED>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), lds, st, static_cast<const __half *>(X), ldx, rows, pre, clip,
                       post_scale, Q, scale_out, had_mask, warm_bytes >= 128 ? static_cast<const uint32_t *>(warm) : nullptr,
                       (int64_t)(warm_bytes / 128));
    return hipGetLastError();
}

template <bool HAS_PRE, bool F6>
hipError_t launch_wg4096(const void *X, int64_t rows, int64_t ldx, const float *pre, float clip, float post_scale,
                         uint8_t *Q, float *scale_out, hipStream_t st, const void *warm, size_t warm_bytes)
{
    constexpr size_t lds = kWg4096Floats * sizeof(float);
    const unsigned blocks = F6 ? (unsigned)((rows + 63) / 64 * 64) : (unsigned)rows;
    const bool warms = warm && warm_bytes >= 128 && blocks >= 256;
    hipLaunchKernelGGL((fwht4096_wg_kernel<HAS_PRE, F6>), dim3(blocks), dim3(256), lds, st, static_cast<const __half *>(X), ldx,
                       rows, pre, clip, post_scale, Q, scale_out, warms ? static_cast<const uint32_t *>(warm) : nullptr,
                       (int64_t)(warm_bytes / 128));
    return hipGetLastError();
}

hipError_t launch_fwht_quant(const void *X, int64_t rows, int64_t K, int64_t ldx, const float *pre,
                             float clip, float post_scale, uint8_t *Q, float *scale_out, hipStream_t st, bool f6,
                             const void *warm, size_t warm_bytes)
{
    int pick = 0;
    if (int64_t f; tuned(kTuneFwht4096, f)) pick = (int)f;
    // K = 4096: a workgroup of four waves per row in two passes of six bits up to kWgKernelMaxRows rows (every row
    // count measured from 1 to 3072: 3.1 / 3.4 / 4.7 / 6.1 / 9.0 / 12.5 us for 1 / 64 / 512 / 1024 / 2048 / 3072 rows
    // against 3.5 / 3.7 / 5.3 / 6.8 / 9.5 / 13.4 for the general workgroup-per-row kernel and 4.4 / 5.4 / 6.3 / 7.2 /
    // 9.4 / 14.0 for a wave per row); a wave per row beyond (16384 rows: 52 against 57 us)
    const bool wg_ok = !pre || (reinterpret_cast<uintptr_t>(pre) & 15u) == 0;
    if (K == 4096 && wg_ok && (pick == 5 || (pick == 0 && rows <= kWgKernelMaxRows))) {
        if (pre) return f6 ? launch_wg4096<true, true>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st, warm, warm_bytes)
                           : launch_wg4096<true, false>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st, warm, warm_bytes);
        return f6 ? launch_wg4096<false, true>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st, warm, warm_bytes)
                  : launch_wg4096<false, false>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st, warm, warm_bytes);
    }
    if (K == 4096 && (pick == 1 || pick == 3 || pick == 4 || (pick == 0 && rows > kWaveKernelMinRows))) {
        constexpr uint32_t all = 0xFFFFFFFFu;
        // factors through LDS (one copy per workgroup) unless the knob asks for per-wave vector loads (4)
        if (pre && pick != 4 && (reinterpret_cast<uintptr_t>(pre) & 15u) == 0 && ldx * 2 * rows < (int64_t)1 << 40)
            return f6 ? launch_wave4096<true, true, false, true>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st, all, warm, warm_bytes)
                      : launch_wave4096<true, false, false, true>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st, all, warm, warm_bytes);
        if (pre) return f6 ? launch_wave4096<true, true>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st, all, warm, warm_bytes)
                           : launch_wave4096<true, false>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st, all, warm, warm_bytes);
        return f6 ? launch_wave4096<false, true>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st, all, warm, warm_bytes)
                  : launch_wave4096<false, false>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st, all, warm, warm_bytes);
    }
    if (f6) {
#define SR_CASE(KK) case KK: return launch_one<KK, true>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st, warm, warm_bytes);
        switch (K) {                                    // K % 128 == 0
            SR_CASE(128) SR_CASE(256) SR_CASE(512) SR_CASE(1024) SR_CASE(2048)
            SR_CASE(4096) SR_CASE(8192) SR_CASE(16384) SR_CASE(32768)
            SR_CASE(896) SR_CASE(1792) SR_CASE(3584) SR_CASE(7168) SR_CASE(14336) SR_CASE(28672)
            default: return hipErrorInvalidValue;
        }
#undef SR_CASE
    }
#define SR_CASE(KK) case KK: return launch_one<KK>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st);
    switch (K) {
        SR_CASE(64) SR_CASE(128) SR_CASE(256) SR_CASE(512) SR_CASE(1024) SR_CASE(2048)
        SR_CASE(4096) SR_CASE(8192) SR_CASE(16384) SR_CASE(32768)
        SR_CASE(448) SR_CASE(896) SR_CASE(1792) SR_CASE(3584) SR_CASE(7168) SR_CASE(14336) SR_CASE(28672)
        default: return hipErrorInvalidValue;
    }
#undef SR_CASE
}

hipError_t launch_fwht_quant_ex(const void *X, int64_t rows, int64_t K, int64_t ldx, const float *pre,
                                float clip, float post_scale, uint8_t *Q, float *scale_out,
                                const RowExtras &ex, hipStream_t st, bool f6)
{
    // head-wise transform of many rows of 4096: the wave-per-row kernel with the unselected butterflies skipped
    if (K == 4096 && !ex.gate && ex.n_grid == 0 && rows > kWaveKernelMinRows) {
        // no search: the ratio "chosen" for every row is the fixed one (the wave kernel itself does not report it)
        if (ex.ratio_out) {
            hipLaunchKernelGGL(fill_f32_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, st, ex.ratio_out, rows, clip);
            if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
        }
        if (pre) return f6 ? launch_wave4096<true, true, true>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st, ex.had_mask)
                           : launch_wave4096<true, false, true>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st, ex.had_mask);
        return f6 ? launch_wave4096<false, true, true>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st, ex.had_mask)
                  : launch_wave4096<false, false, true>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, st, ex.had_mask);
    }
    // the gate alone (the FFN down-projection input) goes through the plain kernel: fewer passes over the row
    // than the general kernel below (K = 14336, 2048 rows: 52 against 68 us)
    if (ex.gate && ex.n_grid == 0 && (ex.had_mask == 0xFFFFFFFFu || !is_pow2(K))) {
#define SR_CASE(KK)                                                                                                      \
    case KK:                                                                                                             \
        return f6 ? launch_one_gated<KK, true>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, ex.gate, ex.ldg, st)  \
                  : launch_one_gated<KK, false>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, ex.gate, ex.ldg, st);
        switch (K) {                                    // the FFN widths; other K take the general kernel
            SR_CASE(1024) SR_CASE(2048) SR_CASE(4096) SR_CASE(8192) SR_CASE(16384)
            SR_CASE(3584) SR_CASE(7168) SR_CASE(14336) SR_CASE(28672)
            default: break;
        }
#undef SR_CASE
    }
    if (f6) {
#define SR_CASE(KK) case KK: return launch_one_ex<KK, true>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, ex, st);
        switch (K) {                                    // K % 128 == 0
            SR_CASE(128) SR_CASE(256) SR_CASE(512) SR_CASE(1024) SR_CASE(2048)
            SR_CASE(4096) SR_CASE(8192) SR_CASE(16384) SR_CASE(32768)
            SR_CASE(896) SR_CASE(1792) SR_CASE(3584) SR_CASE(7168) SR_CASE(14336) SR_CASE(28672)
            default: return hipErrorInvalidValue;
        }
#undef SR_CASE
    }
#define SR_CASE(KK) case KK: return launch_one_ex<KK>(X, rows, ldx, pre, clip, post_scale, Q, scale_out, ex, st);
    switch (K) {
        SR_CASE(64) SR_CASE(128) SR_CASE(256) SR_CASE(512) SR_CASE(1024) SR_CASE(2048)
        SR_CASE(4096) SR_CASE(8192) SR_CASE(16384) SR_CASE(32768)
        SR_CASE(448) SR_CASE(896) SR_CASE(1792) SR_CASE(3584) SR_CASE(7168) SR_CASE(14336) SR_CASE(28672)
        default: return hipErrorInvalidValue;
    }
#undef SR_CASE
}

}  // namespace sr
