// C ABI of libsmoothrot: host-side argument validation and dispatch.
// Every check happens before the first launch, so an error leaves all outputs untouched.
#include "../../include/smoothrot.h"
#include "sr_common.h"

#include <atomic>

namespace sr {
namespace {
std::atomic<int64_t> g_tune[kTuneCount] = {
    {kTuneAuto}, {kTuneAuto}, {kTuneAuto}, {kTuneAuto}, {kTuneAuto}, {kTuneAuto}, {kTuneAuto}};
static_assert(kTuneCount == 7, "one initialiser per knob");
}
int64_t tune(int knob) { return g_tune[knob].load(std::memory_order_relaxed); }
}  // namespace sr

// ---- device-resident scratch of the entry point that allocates nothing -------------------------------------
// One array per GPU the library is loaded on, held until the process ends.  In host code the array's name is
// only a handle: its device address is asked for once per device (with that device current) and kept.
constexpr size_t kNoallocScratchBytes = (size_t)32 * 1024 * 1024 + 2 * 128 * 1024;   // fold of 16 Mi weights
static __device__ __align__(256) unsigned char scratch[kNoallocScratchBytes];

namespace {

std::atomic<void *> g_scratch_ptr[64];

// device address of `scratch` on the current device (nullptr and *err set if the runtime refuses)
void *scratch_on_current_device(hipError_t *err)
{
    int dev = 0;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= 64) { *err = hipErrorInvalidDevice; return nullptr; }
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (*err != hipSuccess || !p) { if (*err == hipSuccess) *err = hipErrorInvalidSymbol; return nullptr; }
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // two racing first calls store the same address
    return p;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// layout of the fold workspace: [Wt fp16 N*K][s fp32 K][w_rowmax fp32 K]
struct FoldWs { size_t wt, s, wmax, total; };
inline FoldWs fold_ws(int64_t K, int64_t N)
{
    FoldWs w;
    w.wt = 0;
    w.s = round_up((size_t)N * (size_t)K * 2, 256);
    w.wmax = w.s + round_up((size_t)K * 4, 256);
    w.total = w.wmax + round_up((size_t)K * 4, 256);
    return w;
}

inline int dev(hipError_t e) { return e == hipSuccess ? SR_OK : SR_ERR_DEVICE; }

}  // namespace

extern "C" {

const char *sr_status_str(int status)
{
    switch (status) {
        case SR_OK: return "ok";
        case SR_ERR_NULL: return "a required pointer is NULL";
        case SR_ERR_SHAPE: return "bad shape (negative size, N not a multiple of 16, or leading dimension too small)";
        case SR_ERR_UNSUPPORTED_K: return "unsupported K (need 2^p or 28*2^p, 64 <= K <= 32768)";
        case SR_ERR_ALIGN: return "pointer not 16-byte aligned or leading dimension not a multiple of 8";
        case SR_ERR_ARG: return "argument out of range (alpha in [0,1], clip in (0,1], dtype)";
        case SR_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case SR_ERR_DEVICE: return "HIP runtime error at launch";
        default: return "unknown status";
    }
}

int sr_hadamard_supported(int64_t K) { return sr::hadamard_supported(K) ? 1 : 0; }

int sr_tune_set(int knob, int64_t value)
{
    if (knob < 0 || knob >= sr::kTuneCount) return SR_ERR_ARG;
    sr::g_tune[knob].store(value, std::memory_order_relaxed);
    return SR_OK;
}

int64_t sr_tune_get(int knob)
{
    if (knob < 0 || knob >= sr::kTuneCount) return SR_TUNE_AUTO;
    return sr::tune(knob);
}

size_t sr_fold_workspace_bytes(int64_t K, int64_t N)
{
    if (!sr::hadamard_supported(K) || N <= 0 || N % 16 != 0) return 0;
    return fold_ws(K, N).total;
}

size_t sr_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    (void)M; (void)N; (void)K;
    return 0;                                        // both kernels keep their partial results on chip
}

int sr_calib_absmax(const void *X_f16, int64_t T, int64_t K, int64_t ldx, float *absmax_io, void *stream)
{
    if (T < 0 || K <= 0 || ldx < K) return SR_ERR_SHAPE;
    if (K % 8 != 0 || ldx % 8 != 0) return SR_ERR_ALIGN;
    if (!absmax_io) return SR_ERR_NULL;
    if (T == 0) return SR_OK;
    if (!X_f16) return SR_ERR_NULL;
    if (!aligned16(X_f16) || !aligned16(absmax_io)) return SR_ERR_ALIGN;
    return dev(sr::launch_calib_absmax(X_f16, T, K, ldx, absmax_io, static_cast<hipStream_t>(stream)));
}

// Index bits transformed by a head-wise Hadamard: K = n_heads * d seen as [n_heads, d].
static uint32_t head_mask(int64_t K, int64_t n_heads, int across)
{
    const uint32_t low = (uint32_t)(K / n_heads) - 1u;       // bits of the position inside a head
    return across ? ((uint32_t)K - 1u) & ~low : low;
}
static bool heads_ok(int64_t K, int64_t n_heads)
{
    return sr::is_pow2(K) && n_heads >= 1 && n_heads <= K && sr::is_pow2(n_heads);
}

static int fold_impl(const void *W_f16, int64_t K, int64_t N, int64_t ldw, const float *act_absmax, float alpha,
                     int64_t n_heads, int across, int clip_steps, float clip_lo, bool extended,
                     uint8_t *Wq, float *w_scale, float *inv_s, float *w_ratio,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    if (K <= 0 || N <= 0 || N % 16 != 0 || ldw < N) return SR_ERR_SHAPE;
    if (!sr::hadamard_supported(K)) return SR_ERR_UNSUPPORTED_K;
    if (!(alpha >= 0.f && alpha <= 1.f) || !(clip_lo > 0.f && clip_lo <= 1.f)) return SR_ERR_ARG;
    if (clip_steps < 1 || clip_steps > sr::kMaxClipGrid || n_heads < 0) return SR_ERR_ARG;
    if (n_heads > 0 && !heads_ok(K, n_heads)) return SR_ERR_ARG;
    if (!W_f16 || !Wq || !w_scale) return SR_ERR_NULL;
    if (ldw % 8 != 0 || !aligned16(W_f16) || !aligned16(Wq) || !aligned16(w_scale) ||
        (act_absmax && !aligned16(act_absmax)) || (inv_s && !aligned16(inv_s)))
        return SR_ERR_ALIGN;
    const FoldWs ws = fold_ws(K, N);
    if (!workspace || workspace_bytes < ws.total || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return SR_ERR_WORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    char *base = static_cast<char *>(workspace);
    void *Wt = base + ws.wt;
    float *s = reinterpret_cast<float *>(base + ws.s);
    float *wmax = reinterpret_cast<float *>(base + ws.wmax);

    // one pass over W gives the transposed copy and (where the factors need them) the row maxima
    hipError_t e = sr::launch_transpose_absmax_f16(W_f16, K, N, ldw, Wt, act_absmax ? wmax : nullptr, st);
    if (e == hipSuccess) e = sr::launch_smooth_factors(act_absmax, wmax, K, alpha, s, inv_s, st);
    if (e != hipSuccess) return dev(e);
    // rows of Wt are the columns of W: rotate (s * column) and quantise per output channel;
    // the 1/order of H H^T = order * I goes into the scale only (codes do not depend on it).
    if (!extended)
        return dev(sr::launch_fwht_quant(Wt, N, K, K, s, clip_lo, 1.0f / (float)K, Wq, w_scale, st));
    sr::RowExtras ex;
    float order = (float)K;
    if (n_heads > 0) {
        ex.had_mask = head_mask(K, n_heads, across);
        order = across ? (float)n_heads : (float)(K / n_heads);
    }
    if (clip_steps > 1) {
        ex.n_grid = clip_steps;
        for (int i = 0; i < clip_steps; ++i)
            ex.grid[i] = (float)(1.0 - (1.0 - (double)clip_lo) * (double)i / (double)(clip_steps - 1));
    }
    ex.ratio_out = w_ratio;
    return dev(sr::launch_fwht_quant_ex(Wt, N, K, K, s, clip_lo, 1.0f / order, Wq, w_scale, ex, st));
}

int sr_fold_smooth_rotate_quant(const void *W_f16, int64_t K, int64_t N, int64_t ldw,
                                const float *act_absmax, float alpha, float w_clip,
                                uint8_t *Wq, float *w_scale, float *inv_s,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    return fold_impl(W_f16, K, N, ldw, act_absmax, alpha, 0, 0, 1, w_clip, false, Wq, w_scale, inv_s, nullptr,
                     workspace, workspace_bytes, stream);
}

size_t sr_noalloc_scratch_bytes(void) { return kNoallocScratchBytes; }

int sr_fold_smooth_rotate_quant_noalloc(const void *W_f16, int64_t K, int64_t N, int64_t ldw,
                                        const float *act_absmax, float alpha, float w_clip,
                                        uint8_t *Wq, float *w_scale, float *inv_s, void *stream)
{
    // size first: a shape beyond the array is refused whatever else is wrong with the call
    if (K > 0 && N > 0 && N % 16 == 0 && sr::hadamard_supported(K) && fold_ws(K, N).total > kNoallocScratchBytes)
        return SR_ERR_WORKSPACE;
    // argument errors must not depend on the device: validate with a stand-in workspace address, launch nothing
    if (K <= 0 || N <= 0 || N % 16 != 0 || ldw < N) return SR_ERR_SHAPE;
    if (!sr::hadamard_supported(K)) return SR_ERR_UNSUPPORTED_K;
    if (!(alpha >= 0.f && alpha <= 1.f) || !(w_clip > 0.f && w_clip <= 1.f)) return SR_ERR_ARG;
    if (!W_f16 || !Wq || !w_scale) return SR_ERR_NULL;
    if (ldw % 8 != 0 || !aligned16(W_f16) || !aligned16(Wq) || !aligned16(w_scale) ||
        (act_absmax && !aligned16(act_absmax)) || (inv_s && !aligned16(inv_s)))
        return SR_ERR_ALIGN;
    hipError_t e = hipSuccess;
    void *ws = scratch_on_current_device(&e);
    if (!ws) return SR_ERR_DEVICE;
    return fold_impl(W_f16, K, N, ldw, act_absmax, alpha, 0, 0, 1, w_clip, false, Wq, w_scale, inv_s, nullptr,
                     ws, kNoallocScratchBytes, stream);
}

int sr_fold_smooth_rotate_quant_ex(const void *W_f16, int64_t K, int64_t N, int64_t ldw,
                                   const float *act_absmax, float alpha,
                                   int64_t n_heads, int across, int clip_steps, float clip_lo,
                                   uint8_t *Wq, float *w_scale, float *inv_s, float *w_ratio,
                                   void *workspace, size_t workspace_bytes, void *stream)
{
    return fold_impl(W_f16, K, N, ldw, act_absmax, alpha, n_heads, across, clip_steps, clip_lo, true, Wq, w_scale,
                     inv_s, w_ratio, workspace, workspace_bytes, stream);
}

int sr_fwht_quant_act(const void *X_f16, int64_t M, int64_t K, int64_t ldx, const float *inv_s, float clip,
                      uint8_t *Xq, float *x_scale, void *stream)
{
    if (M < 0 || K <= 0 || ldx < K) return SR_ERR_SHAPE;
    if (!sr::hadamard_supported(K)) return SR_ERR_UNSUPPORTED_K;
    if (!(clip > 0.f && clip <= 1.f)) return SR_ERR_ARG;
    if (M == 0) return SR_OK;
    if (!X_f16 || !Xq || !x_scale) return SR_ERR_NULL;
    if (ldx % 8 != 0 || !aligned16(X_f16) || !aligned16(Xq) || (inv_s && !aligned16(inv_s))) return SR_ERR_ALIGN;
    return dev(sr::launch_fwht_quant(X_f16, M, K, ldx, inv_s, clip, 1.0f, Xq, x_scale,
                                     static_cast<hipStream_t>(stream)));
}

int sr_fwht_quant_act_f6_warm(const void *X_f16, int64_t M, int64_t K, int64_t ldx, const float *inv_s, float clip,
                              uint8_t *X6, float *x_scale, const void *next_operand, size_t next_bytes, void *stream)
{
    if (M < 0 || K <= 0 || ldx < K) return SR_ERR_SHAPE;
    if (!sr::hadamard_supported(K) || K % 128 != 0) return SR_ERR_UNSUPPORTED_K;
    if (!(clip > 0.f && clip <= 1.f)) return SR_ERR_ARG;
    if (next_bytes && !next_operand) return SR_ERR_NULL;
    if (next_bytes && !aligned16(next_operand)) return SR_ERR_ALIGN;
    if (M == 0) return SR_OK;
    if (!X_f16 || !X6 || !x_scale) return SR_ERR_NULL;
    if (ldx % 8 != 0 || !aligned16(X_f16) || !aligned16(X6) || (inv_s && !aligned16(inv_s))) return SR_ERR_ALIGN;
    return dev(sr::launch_fwht_quant(X_f16, M, K, ldx, inv_s, clip, 1.0f, X6, x_scale,
                                     static_cast<hipStream_t>(stream), true, next_operand, next_bytes));
}

int sr_fwht_quant_act_f6(const void *X_f16, int64_t M, int64_t K, int64_t ldx, const float *inv_s, float clip,
                         uint8_t *X6, float *x_scale, void *stream)
{
    return sr_fwht_quant_act_f6_warm(X_f16, M, K, ldx, inv_s, clip, X6, x_scale, nullptr, 0, stream);
}

int sr_swiglu_fwht_quant_act(const void *G_f16, const void *U_f16, int64_t M, int64_t K, int64_t ldg, int64_t ldu,
                             const float *inv_s, float clip, uint8_t *Xq, float *x_scale, void *stream)
{
    if (M < 0 || K <= 0 || ldg < K || ldu < K) return SR_ERR_SHAPE;
    if (!sr::hadamard_supported(K)) return SR_ERR_UNSUPPORTED_K;
    if (!(clip > 0.f && clip <= 1.f)) return SR_ERR_ARG;
    if (M == 0) return SR_OK;
    if (!G_f16 || !U_f16 || !Xq || !x_scale) return SR_ERR_NULL;
    if (ldg % 8 != 0 || ldu % 8 != 0 || !aligned16(G_f16) || !aligned16(U_f16) || !aligned16(Xq) ||
        (inv_s && !aligned16(inv_s)))
        return SR_ERR_ALIGN;
    sr::RowExtras ex;
    ex.gate = static_cast<const __half *>(G_f16);
    ex.ldg = ldg;
    return dev(sr::launch_fwht_quant_ex(U_f16, M, K, ldu, inv_s, clip, 1.0f, Xq, x_scale, ex,
                                        static_cast<hipStream_t>(stream)));
}

int sr_swiglu_fwht_quant_act_f6(const void *G_f16, const void *U_f16, int64_t M, int64_t K, int64_t ldg, int64_t ldu,
                                const float *inv_s, float clip, uint8_t *X6, float *x_scale, void *stream)
{
    if (M < 0 || K <= 0 || ldg < K || ldu < K) return SR_ERR_SHAPE;
    if (!sr::hadamard_supported(K) || K % 128 != 0) return SR_ERR_UNSUPPORTED_K;
    if (!(clip > 0.f && clip <= 1.f)) return SR_ERR_ARG;
    if (M == 0) return SR_OK;
    if (!G_f16 || !U_f16 || !X6 || !x_scale) return SR_ERR_NULL;
    if (ldg % 8 != 0 || ldu % 8 != 0 || !aligned16(G_f16) || !aligned16(U_f16) || !aligned16(X6) ||
        (inv_s && !aligned16(inv_s)))
        return SR_ERR_ALIGN;
    sr::RowExtras ex;
    ex.gate = static_cast<const __half *>(G_f16);
    ex.ldg = ldg;
    return dev(sr::launch_fwht_quant_ex(U_f16, M, K, ldu, inv_s, clip, 1.0f, X6, x_scale, ex,
                                        static_cast<hipStream_t>(stream), true));
}

int sr_fwht_quant_act_heads(const void *X_f16, int64_t M, int64_t K, int64_t ldx, int64_t n_heads, int across,
                            const float *inv_s, float clip, uint8_t *Xq, float *x_scale, void *stream)
{
    if (M < 0 || K <= 0 || ldx < K) return SR_ERR_SHAPE;
    if (!sr::hadamard_supported(K) || !sr::is_pow2(K)) return SR_ERR_UNSUPPORTED_K;
    if (!(clip > 0.f && clip <= 1.f) || !heads_ok(K, n_heads)) return SR_ERR_ARG;
    if (M == 0) return SR_OK;
    if (!X_f16 || !Xq || !x_scale) return SR_ERR_NULL;
    if (ldx % 8 != 0 || !aligned16(X_f16) || !aligned16(Xq) || (inv_s && !aligned16(inv_s))) return SR_ERR_ALIGN;
    sr::RowExtras ex;
    ex.had_mask = head_mask(K, n_heads, across);
    return dev(sr::launch_fwht_quant_ex(X_f16, M, K, ldx, inv_s, clip, 1.0f, Xq, x_scale, ex,
                                        static_cast<hipStream_t>(stream)));
}

int sr_kv_quant_asym(const void *X_f16, int64_t rows, int64_t D, int64_t ldx, int64_t group, float clip,
                     uint8_t *Q, float *scale, float *zero, void *stream)
{
    if (rows < 0 || D <= 0 || ldx < D) return SR_ERR_SHAPE;
    if (group != 32 && group != 64 && group != 128 && group != 256 && group != 512) return SR_ERR_ARG;
    if (D % group != 0) return SR_ERR_SHAPE;
    if (!(clip > 0.f && clip <= 1.f)) return SR_ERR_ARG;
    if (rows == 0) return SR_OK;
    if (!X_f16 || !Q || !scale || !zero) return SR_ERR_NULL;
    if (ldx % 8 != 0 || !aligned16(X_f16) || !aligned16(Q)) return SR_ERR_ALIGN;
    return dev(sr::launch_kv_quant(X_f16, rows, D, ldx, group, clip, Q, scale, zero,
                                   static_cast<hipStream_t>(stream)));
}

size_t sr_linear_decode_workspace_bytes(int64_t M, int64_t K) { return sr::linear_decode_workspace_bytes(M, K); }

int sr_w4a4_linear_decode(const void *X_f16, int64_t M, int64_t K, int64_t ldx, const float *inv_s, float clip,
                          const uint8_t *Wq, const float *w_scale, int64_t N, void *Y_f16, int64_t ldy,
                          uint8_t *Xq_out, float *x_scale_out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (M < 0 || M > 16 || K <= 0 || N <= 0 || N % 16 != 0 || ldx < K || ldy < N) return SR_ERR_SHAPE;
    if ((double)N * (double)K >= 4294967296.0) return SR_ERR_SHAPE;
    if (!sr::linear_decode_supported(K)) return SR_ERR_UNSUPPORTED_K;
    if (!(clip > 0.f && clip <= 1.f)) return SR_ERR_ARG;
    if (M == 0) return SR_OK;
    const size_t need = sr::linear_decode_workspace_bytes(M, K);
    if (!X_f16 || !Wq || !w_scale || !Y_f16) return SR_ERR_NULL;
    if (ldx % 8 != 0 || (need && ldy % 8 != 0) || !aligned16(X_f16) || !aligned16(Wq) || !aligned16(Y_f16) ||
        !aligned16(w_scale) || (inv_s && !aligned16(inv_s)) || (Xq_out && !aligned16(Xq_out)))
        return SR_ERR_ALIGN;
    if (need && (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)))
        return SR_ERR_WORKSPACE;
    return dev(sr::launch_linear_decode(X_f16, M, K, ldx, inv_s, clip, Wq, w_scale, N, Y_f16, ldy, Xq_out,
                                        x_scale_out, workspace, static_cast<hipStream_t>(stream)));
}

int sr_w4a4_gemm(const uint8_t *Xq, const float *x_scale, const uint8_t *Wq, const float *w_scale,
                 int64_t M, int64_t N, int64_t K, void *Y, int64_t ldy, int out_dtype,
                 void *workspace, size_t workspace_bytes, void *stream)
{
    (void)workspace; (void)workspace_bytes;
    if (M < 0 || N <= 0 || K <= 0 || N % 16 != 0 || ldy < N) return SR_ERR_SHAPE;
    // kernels index rows with 32-bit byte offsets
    if ((double)M * (double)K >= 4294967296.0 || (double)N * (double)K >= 4294967296.0) return SR_ERR_SHAPE;
    if (K % 64 != 0 || K >= 131072) return SR_ERR_UNSUPPORTED_K;
    if (out_dtype != SR_F16 && out_dtype != SR_I32) return SR_ERR_ARG;
    if (M == 0) return SR_OK;
    if (!Xq || !Wq || !Y) return SR_ERR_NULL;
    if (out_dtype == SR_F16 && (!x_scale || !w_scale)) return SR_ERR_NULL;
    if (ldy % 8 != 0 || !aligned16(Xq) || !aligned16(Wq) || !aligned16(Y) ||
        (out_dtype == SR_F16 && !aligned16(w_scale)))
        return SR_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int i32 = out_dtype == SR_I32;
    if (M <= 16) return dev(sr::launch_gemm_decode(Xq, x_scale, Wq, w_scale, M, N, K, Y, ldy, i32, st));
    return dev(sr::launch_gemm_prefill(Xq, x_scale, Wq, w_scale, M, N, K, Y, ldy, i32, st));
}

size_t sr_f6_tiles_bytes(int64_t rows, int64_t K)
{
    if (rows <= 0 || K <= 0 || K % 128 != 0) return 0;
    return (size_t)((rows + 7) / 8) * (size_t)(K / 128) * 768;
}

int sr_pack_f6_tiles(const uint8_t *Q4, int64_t rows, int64_t K, uint8_t *T6, void *stream)
{
    if (rows < 0 || K <= 0) return SR_ERR_SHAPE;
    if ((double)rows * (double)K >= 4294967296.0) return SR_ERR_SHAPE;
    if (K % 128 != 0 || K >= 131072) return SR_ERR_UNSUPPORTED_K;
    if (rows == 0) return SR_OK;
    if (!Q4 || !T6) return SR_ERR_NULL;
    if (!aligned16(Q4) || !aligned16(T6)) return SR_ERR_ALIGN;
    return dev(sr::launch_pack_f6(Q4, rows, K, T6, static_cast<hipStream_t>(stream)));
}

int sr_w4a4_gemm_f6_warm(const uint8_t *X6, const float *x_scale, const uint8_t *W6, const float *w_scale,
                         int64_t M, int64_t N, int64_t K, void *Y, int64_t ldy, int out_dtype,
                         const void *next_operand, size_t next_bytes, void *workspace, size_t workspace_bytes, void *stream)
{
    (void)workspace; (void)workspace_bytes;
    if (M < 0 || N <= 0 || K <= 0 || N % 16 != 0 || ldy < N) return SR_ERR_SHAPE;
    // kernels index blocks with 32-bit byte offsets (0.75 bytes per code)
    if ((double)M * (double)K >= 4294967296.0 || (double)N * (double)K >= 4294967296.0) return SR_ERR_SHAPE;
    if (K % 128 != 0 || K >= 131072) return SR_ERR_UNSUPPORTED_K;
    if (out_dtype != SR_F16 && out_dtype != SR_I32) return SR_ERR_ARG;
    if (next_bytes && !next_operand) return SR_ERR_NULL;
    if (next_bytes && !aligned16(next_operand)) return SR_ERR_ALIGN;
    if (M == 0) return SR_OK;
    if (!X6 || !W6 || !Y) return SR_ERR_NULL;
    if (out_dtype == SR_F16 && (!x_scale || !w_scale)) return SR_ERR_NULL;
    if (ldy % 8 != 0 || !aligned16(X6) || !aligned16(W6) || !aligned16(Y)) return SR_ERR_ALIGN;
    return dev(sr::launch_gemm_f6(X6, x_scale, W6, w_scale, M, N, K, Y, ldy, out_dtype == SR_I32,
                                  static_cast<hipStream_t>(stream), next_operand, next_bytes));
}

int sr_w4a4_gemm_f6(const uint8_t *X6, const float *x_scale, const uint8_t *W6, const float *w_scale,
                    int64_t M, int64_t N, int64_t K, void *Y, int64_t ldy, int out_dtype,
                    void *workspace, size_t workspace_bytes, void *stream)
{
    return sr_w4a4_gemm_f6_warm(X6, x_scale, W6, w_scale, M, N, K, Y, ldy, out_dtype, nullptr, 0, workspace,
                                workspace_bytes, stream);
}

}  // extern "C"
