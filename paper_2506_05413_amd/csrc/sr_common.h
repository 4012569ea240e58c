// Internal declarations shared by the HIP translation units of libsmoothrot.
// (Public interface: include/smoothrot.h.)
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <stddef.h>
#include <atomic>

namespace sr {

// ---- Hadamard order helpers (host) ------------------------------------------------
constexpr bool is_pow2(int64_t v) { return v >= 1 && (v & (v - 1)) == 0; }
constexpr int64_t kMinK = 64, kMaxPow2K = 32768, kMaxKronK = 28672;

inline bool hadamard_supported(int64_t K)
{
    if (K < kMinK) return false;
    if (is_pow2(K)) return K <= kMaxPow2K;
    return K % 28 == 0 && is_pow2(K / 28) && K % 64 == 0 && K <= kMaxKronK;
}

// ---- reductions over lanes without LDS traffic (device) ------------------------------------------
// __shfl_xor compiles to ds_bpermute_b32 here: every step of a reduction then waits for a round trip
// through the LDS crossbar.  DPP lane permutations are operand modifiers of ordinary vector
// instructions.  Controls: 0xB1 / 0x4E = quad_perm [1,0,3,2] / [2,3,0,1] (lane ^ 1, lane ^ 2),
// 0x141 = row_half_mirror (lane i <-> 7 - i of 8), 0x140 = row_mirror (i <-> 15 - i of 16),
// 0x142 / 0x143 = row_bcast15 / row_bcast31 (last lane of a row of 16 / of 32 lanes to the next ones).
template <int CTRL, int ROW_MASK = 0xF> __device__ __forceinline__ int lane_perm(int v)
{
    // all rows enabled: every lane has a source, and the compiler can fold the move into the instruction that uses it
    if constexpr (ROW_MASK == 0xF) return __builtin_amdgcn_mov_dpp(v, CTRL, 0xF, 0xF, true);
    else return __builtin_amdgcn_update_dpp(v, v, CTRL, ROW_MASK, 0xF, false);  // disabled rows keep their own value
}
template <int CTRL, int ROW_MASK = 0xF> __device__ __forceinline__ float lane_perm(float v)
{
    return __int_as_float(lane_perm<CTRL, ROW_MASK>(__float_as_int(v)));
}
// every lane of an aligned group of 8 / 16 lanes receives the group's result
__device__ __forceinline__ int sum_of_8_lanes(int v)
{
    v += lane_perm<0xB1>(v);
    v += lane_perm<0x4E>(v);
    return v + lane_perm<0x141>(v);
}
__device__ __forceinline__ float max_of_16_lanes(float v)
{
    v = fmaxf(v, lane_perm<0xB1>(v));
    v = fmaxf(v, lane_perm<0x4E>(v));
    v = fmaxf(v, lane_perm<0x141>(v));
    return fmaxf(v, lane_perm<0x140>(v));
}
// maximum over the wave, returned to every lane (through lane 63, which collects the four rows)
__device__ __forceinline__ float max_of_wave(float v)
{
    v = max_of_16_lanes(v);
    v = fmaxf(v, lane_perm<0x142, 0xA>(v));
    v = fmaxf(v, lane_perm<0x143, 0xC>(v));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// ---- tuning knobs (host) ---------------------------------------------------------------
// Process-wide overrides of the dispatch heuristics, set through sr_tune_set (include/smoothrot.h): the tests
// use them to run every kernel on every shape, tuning runs to compare variants inside one process.  A knob that
// is not set (kTuneAuto) leaves the measured choice in place.  Relaxed atomics: a launch reads each knob once.
enum { kTuneGemmTile = 0, kTuneGemmGrid, kTuneGemmXcdM, kTuneDecodeKernel, kTuneFwht4096, kTuneFwhtStream,
       kTuneGemmWarm, kTuneCount };
constexpr int64_t kTuneAuto = INT64_MIN;
int64_t tune(int knob);                                  // sr_api.hip
inline bool tuned(int knob, int64_t &v) { v = tune(knob); return v != kTuneAuto; }

// ---- device properties (host) ---------------------------------------------------------
// compute units of the current device (asked once per process and device)
inline int compute_units()
{
    static std::atomic<int> cached[64];                  // zero-initialised; concurrent first calls store the same value
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// ---- launchers (each returns hipGetLastError() of its launches) ------------------

// y = (x * pre) H per row, per-row symmetric INT4, scale_out = delta * post_scale.
// f6: Q receives f6 tiles (see gemm_f6.hip; K % 128 == 0) instead of canonical packed nibbles.
// warm: device memory (4-byte aligned) whose 128-byte lines the launch reads on the side, so that the kernel
// that follows finds them in the memory-side cache; honoured by the K = 4096 wave-per-row kernel and by the default
// workgroup-per-row launches of at least 256 workgroups, ignored elsewhere.
hipError_t launch_fwht_quant(const void *X_f16, int64_t rows, int64_t K, int64_t ldx,
                             const float *pre, float clip, float post_scale,
                             uint8_t *Q, float *scale_out, hipStream_t st, bool f6 = false,
                             const void *warm = nullptr, size_t warm_bytes = 0);

// Optional extras of the row kernel (see fwht_quant.hip).
constexpr int kMaxClipGrid = 32;
struct RowExtras {
    const __half *gate = nullptr;   // x = silu(gate) * X when set; row stride ldg elements
    int64_t ldg = 0;
    uint32_t had_mask = 0xFFFFFFFFu; // index bits that are transformed (power-of-two K only)
    int n_grid = 0;                  // > 0: search the clipping ratio per row over grid[0 .. n_grid)
    float grid[kMaxClipGrid] = {};
    float *ratio_out = nullptr;      // chosen ratio per row
};

hipError_t launch_fwht_quant_ex(const void *X_f16, int64_t rows, int64_t K, int64_t ldx,
                                const float *pre, float clip, float post_scale,
                                uint8_t *Q, float *scale_out, const RowExtras &ex, hipStream_t st, bool f6 = false);

hipError_t launch_calib_absmax(const void *X_f16, int64_t T, int64_t K, int64_t ldx,
                               float *absmax_io, hipStream_t st);

// s / inv_s from calibration and weight maxima (act_absmax may be NULL: s = 1)
hipError_t launch_smooth_factors(const float *act_absmax, const float *w_rowmax, int64_t K,
                                 float alpha, float *s, float *inv_s, hipStream_t st);

// Wt[n][k] = W[k][n] (fp16 bits moved unchanged) and, if w_rowmax is not NULL, w_rowmax[j] = max_n |W[j][n]|
hipError_t launch_transpose_absmax_f16(const void *W_f16, int64_t K, int64_t N, int64_t ldw, void *Wt_f16,
                                       float *w_rowmax, hipStream_t st);

// asymmetric 4-bit group quantiser (keys / values)
hipError_t launch_kv_quant(const void *X_f16, int64_t rows, int64_t D, int64_t ldx, int64_t group, float clip,
                           uint8_t *Q, float *scale, float *zero, hipStream_t st);

// decode step behind one entry point: rotate + quantise up to 16 token rows and multiply (see linear_decode.hip).
// workspace: linear_decode_workspace_bytes(M, K) bytes (0 = none needed).
bool linear_decode_supported(int64_t K);
size_t linear_decode_workspace_bytes(int64_t M, int64_t K);
hipError_t launch_linear_decode(const void *X_f16, int64_t M, int64_t K, int64_t ldx, const float *pre, float clip,
                                const uint8_t *Wq, const float *ws, int64_t N, void *Y_f16, int64_t ldy,
                                uint8_t *Xq_out, float *xs_out, void *workspace, hipStream_t st);

hipError_t launch_gemm_prefill(const uint8_t *Xq, const float *xs, const uint8_t *Wq, const float *ws,
                               int64_t M, int64_t N, int64_t K, void *Y, int64_t ldy, int out_i32,
                               hipStream_t st);

// f6 tiles (see gemm_f6.hip): repacking of canonical INT4 codes, and the GEMM on the FP6 matrix pipe
hipError_t launch_pack_f6(const uint8_t *Q4, int64_t rows, int64_t K, uint8_t *T6, hipStream_t st);
// warm / warm_bytes: a region whose 128-byte lines the launch reads on the side where its tile configuration has a
// wave to spare (256 x 128 tiles); ignored elsewhere
hipError_t launch_gemm_f6(const uint8_t *X6, const float *xs, const uint8_t *W6, const float *ws,
                          int64_t M, int64_t N, int64_t K, void *Y, int64_t ldy, int out_i32,
                          hipStream_t st, const void *warm = nullptr, size_t warm_bytes = 0);

hipError_t launch_gemm_decode(const uint8_t *Xq, const float *xs, const uint8_t *Wq, const float *ws,
                              int64_t M, int64_t N, int64_t K, void *Y, int64_t ldy, int out_i32,
                              hipStream_t st);

}  // namespace sr
