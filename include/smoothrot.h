/*
 * smoothrot.h -- C ABI of the MI355X (gfx950) SmoothRot W4A4 linear-layer library.
 *
 * SmoothRot (arXiv 2506.05413) smooths the input channels of a linear layer with
 * calibrated factors s, rotates them with a Hadamard matrix H, and runs the layer
 * with 4-bit weights and 4-bit activations:
 *
 *     Y = X W = (X diag(1/s) H) (H^T diag(s) W / n)          [paper, Eq. (2), A = (H Lambda)^-1]
 *
 * The calls below are the four operations of that layer.  Two are offline
 * (calibration, weight fold), two are the online hot path (rotate + quantise the
 * activations, INT4 x INT4 GEMM with dequantising epilogue).
 *
 * Conventions that hold for every call
 * ------------------------------------
 *  - Every data pointer is DEVICE memory owned by the caller.  The library never
 *    allocates, frees or keeps a pointer and is re-entrant.  Its only process-wide
 *    state: the tuning knobs of sr_tune_set (all "auto" unless a caller sets one), a
 *    cached compute-unit count per device, and the device-resident scratch array of
 *    sr_fold_smooth_rotate_quant_noalloc.  No environment variable is read.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *    only enqueue work and return; they never synchronise.
 *  - Arguments are validated on the host before anything is launched.  On error a
 *    status is returned, nothing is launched and outputs are untouched.
 *  - Input and output buffers must not overlap.  Non-finite inputs give
 *    unspecified values (never an out-of-bounds access).
 *  - X is [tokens, K] row-major fp16 (row = token, K = input channels);
 *    W is [K, N] row-major fp16 (N = output channels).
 *  - H is the unnormalised +-1 Hadamard matrix of order K: Sylvester
 *    (H[i][j] = (-1)^popcount(i&j)) for K = 2^p; H_28 (x) H_{2^p} for K = 28 * 2^p,
 *    with H_28 the Paley type-I matrix over GF(27) = GF(3)[x]/(x^3+2x+1) and the
 *    28-index the slow one.  The rotation is T(v)_j = sum_k v_k H[k][j].
 *  - INT4 codes are two's-complement values in [-8, 7], packed two per byte along
 *    K: byte b of a row holds code(2b) in bits 0-3 and code(2b+1) in bits 4-7.
 *  - Supported shapes: K = 2^p or 28 * 2^p with 64 <= K <= 32768 (28 * 2^p: <= 28672);
 *    N a multiple of 16; any M >= 1 (M = 0 or T = 0 is a no-op returning SR_OK).
 *    Base pointers must be 16-byte aligned and leading dimensions multiples of 8.
 */
#ifndef SMOOTHROT_H
#define SMOOTHROT_H

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__) || defined(__clang__)
#define SR_API __attribute__((visibility("default")))
#else
#define SR_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SR_OK = 0,
    SR_ERR_NULL = 1,          /* a required pointer is NULL                               */
    SR_ERR_SHAPE = 2,         /* negative size, N % 16 != 0, leading dimension too small  */
    SR_ERR_UNSUPPORTED_K = 3, /* K is not 2^p / 28*2^p in the supported range             */
    SR_ERR_ALIGN = 4,         /* pointer not 16-byte aligned / ld not a multiple of 8     */
    SR_ERR_ARG = 5,           /* alpha outside [0,1], clip outside (0,1], unknown dtype   */
    SR_ERR_WORKSPACE = 6,     /* workspace NULL or smaller than sr_*_workspace_bytes      */
    SR_ERR_DEVICE = 7         /* the HIP runtime refused a launch                          */
} sr_status;

/* Output type selector of sr_w4a4_gemm. */
enum { SR_F16 = 0, SR_I32 = 1 };

/* Static, NUL-terminated description of a status (never NULL). */
SR_API const char *sr_status_str(int status);

/*
 * Tuning knobs: process-wide overrides of the dispatch heuristics, for tests (every kernel on every
 * shape) and tuning runs (variants compared inside one process).  Results never depend on a knob --
 * only which kernel, tile or grid computes them.  SR_TUNE_AUTO restores the measured choice.  A knob
 * is read once per launch with a relaxed atomic load; setting one while another thread launches is
 * safe but that launch may see either value.
 *   SR_TUNE_GEMM_TILE      tile configuration of the prefill GEMMs by number (unknown numbers: auto)
 *   SR_TUNE_GEMM_GRID      persistent workgroups of the prefill GEMMs (rounded down to a multiple of 8)
 *   SR_TUNE_GEMM_XCDM      split of the tile grid over the 8 XCDs in m: 0 (none), 1, 2, 4, 8
 *   SR_TUNE_DECODE_KERNEL  M <= 16 GEMM: 1 dot product (M <= 2), 2 MFMA per 16 channels, 3 streaming MFMA
 *   SR_TUNE_FWHT4096       K = 4096 rotation: 1 wave per row (factors staged in LDS), 4 wave per row (factors
 *                          loaded per lane), 2 general workgroup-per-row kernel, 5 workgroup per row in two passes
 *   SR_TUNE_FWHT_STREAM    K = 14336 rotation: 1 workgroups walk over rows, 0 one workgroup per row
 *   SR_TUNE_GEMM_WARM      sr_w4a4_gemm_f6_warm: 0 = ignore the hint (the launch of sr_w4a4_gemm_f6)
 * sr_tune_set returns SR_ERR_ARG for an unknown knob; sr_tune_get returns SR_TUNE_AUTO for one.
 */
enum { SR_TUNE_GEMM_TILE = 0, SR_TUNE_GEMM_GRID = 1, SR_TUNE_GEMM_XCDM = 2, SR_TUNE_DECODE_KERNEL = 3,
       SR_TUNE_FWHT4096 = 4, SR_TUNE_FWHT_STREAM = 5, SR_TUNE_GEMM_WARM = 6 };
#define SR_TUNE_AUTO INT64_MIN
SR_API int sr_tune_set(int knob, int64_t value);
SR_API int64_t sr_tune_get(int knob);

/* 1 if a Hadamard matrix of order K is implemented (see "Supported shapes"), else 0. */
SR_API int sr_hadamard_supported(int64_t K);

/* Bytes of device scratch sr_fold_smooth_rotate_quant needs for a [K, N] weight
 * (0 if the shape is unsupported). */
SR_API size_t sr_fold_workspace_bytes(int64_t K, int64_t N);

/* Bytes of device scratch sr_w4a4_gemm needs (0 for every shape today: partial results stay
 * on chip; callers should still query it and pass what it asks for). */
SR_API size_t sr_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);

/*
 * Calibration: running per-channel activation maximum,
 *     absmax_io[j] <- max(absmax_io[j], max_t |X[t][j]|)
 * -- the max|X_j| of the smoothing-factor formula (paper, section "Methodology").
 *
 *   X_f16      fp16 [T, K], row stride ldx elements (ldx >= K)
 *   absmax_io  fp32 [K], in/out; the caller zero-initialises it before the first
 *              call and may call repeatedly over chunks of the calibration set
 *              (values must be >= 0).  The result is exact.
 */
SR_API int sr_calib_absmax(const void *X_f16, int64_t T, int64_t K, int64_t ldx,
                    float *absmax_io, void *stream);

/*
 * Weight fold (offline), paper section "Methodology" + "Quantization" settings:
 *     w_j   = max_n |W[j][n]|                         (input channel j, W as given)
 *     s_j   = max(a_j,1e-5)^alpha / max(w_j,1e-5)^(1-alpha)
 *     W^    = H^T diag(s) W / K                        (T applied to the columns of diag(s) W)
 *     dw_n  = w_clip * max_j |W^[j][n]| / 7            (per output channel; 1 if the column is 0)
 *     code  = clamp(rint(W^[j][n] / dw_n), -8, 7)      (round-to-nearest, ties to even)
 *
 *   W_f16       fp16 [K, N], row stride ldw (ldw >= N)
 *   act_absmax  fp32 [K] from sr_calib_absmax, or NULL for s = 1 (rotation only)
 *   alpha       migration strength in [0, 1];  w_clip in (0, 1] (1 = plain RTN)
 *   Wq          out, uint8 [N, K/2] packed codes, output channel major
 *   w_scale     out, fp32 [N]  (dw_n)
 *   inv_s       out, fp32 [K]  (1 / s_j), may be NULL
 *   workspace   at least sr_fold_workspace_bytes(K, N) bytes, 256-byte aligned
 */
SR_API int sr_fold_smooth_rotate_quant(const void *W_f16, int64_t K, int64_t N, int64_t ldw,
                                const float *act_absmax, float alpha, float w_clip,
                                uint8_t *Wq, float *w_scale, float *inv_s,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * sr_fold_smooth_rotate_quant for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments
 * without the workspace, same kernels, same results bit for bit.  The scratch (the fp16 transposed weight
 * and two fp32 [K] vectors) lives in a device-resident array of sr_noalloc_scratch_bytes() bytes
 * (32.25 MiB) that every GPU the library runs on holds until the process ends; the call itself allocates
 * and frees nothing.
 *   - Shapes whose sr_fold_workspace_bytes(K, N) exceeds that size (K * N > 16 Mi weights, e.g.
 *     4096 x 14336) return SR_ERR_WORKSPACE; use the call above with a workspace for those.
 *   - All calls on one GPU share the one array: two calls whose kernels overlap on the same GPU
 *     (different streams, different threads) race.  Nothing in it has to start at zero -- every word a
 *     kernel reads was written earlier in the same call -- so consecutive calls need no clearing.
 *   - The first call on a device asks the runtime for the array's address (no allocation); make that
 *     call outside a stream capture.
 */
SR_API size_t sr_noalloc_scratch_bytes(void);
SR_API int sr_fold_smooth_rotate_quant_noalloc(const void *W_f16, int64_t K, int64_t N, int64_t ldw,
                                        const float *act_absmax, float alpha, float w_clip,
                                        uint8_t *Wq, float *w_scale, float *inv_s, void *stream);

/*
 * Online rotation + per-token quantisation (paper: online Hadamard before the
 * projection, then per-token symmetric INT4 with a constant clipping ratio; Eq. (1)):
 *     y_m   = (x_m * inv_s) H                          (fp32, never written to memory)
 *     dx_m  = clip * max_j |y_mj| / 7                  (1 if the row is 0)
 *     code  = clamp(rint(y_mj / dx_m), -8, 7)
 *
 *   X_f16    fp16 [M, K], row stride ldx
 *   inv_s    fp32 [K] or NULL (activations already smoothed upstream, as when the
 *            factors are absorbed into the preceding projection)
 *   clip     clipping ratio in (0, 1] (paper: 0.9)
 *   Xq       out, uint8 [M, K/2] packed codes;  x_scale out, fp32 [M] (dx_m)
 */
SR_API int sr_fwht_quant_act(const void *X_f16, int64_t M, int64_t K, int64_t ldx,
                      const float *inv_s, float clip,
                      uint8_t *Xq, float *x_scale, void *stream);

/*
 * INT4 x INT4 GEMM with INT32 accumulation and dequantising epilogue
 * (paper: quantised forward pass; dequantisation Q(X) = X_int * Delta of Eq. (1)):
 *     acc[m][n] = sum_k codeX[m][k] * codeW[n][k]      (exact)
 *     Y[m][n]   = fp16( float(acc) * x_scale[m] * w_scale[n] )      out_dtype = SR_F16
 *     Y[m][n]   = acc[m][n] as int32 (scales ignored, may be NULL)  out_dtype = SR_I32
 *
 *   Xq [M, K/2], Wq [N, K/2] packed codes as produced by the two calls above
 *   Y   out, [M, N] with row stride ldy elements (fp16 or int32), ldy >= N
 *   workspace   at least sr_gemm_workspace_bytes(M, N, K) bytes, 256-byte aligned (may be NULL when
 *               that is 0)
 *   M * K and N * K must stay below 2^32 (rows are addressed with 32-bit byte offsets).
 *   K only needs to be a multiple of 64 here (no Hadamard involved), K < 131072.
 */
SR_API int sr_w4a4_gemm(const uint8_t *Xq, const float *x_scale,
                 const uint8_t *Wq, const float *w_scale,
                 int64_t M, int64_t N, int64_t K,
                 void *Y, int64_t ldy, int out_dtype,
                 void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * Rows around the core path.  Same conventions as above.
 * ------------------------------------------------------------------------------------------ */

/*
 * sr_fwht_quant_act with the gated-FFN product fused in front (paper, Fig. 2, FFN block: the
 * down-projection input sigma(gate) (.) up is smoothed, rotated and quantised):
 *     x_m = silu(G_m) * U_m     (fp32, silu(g) = g / (1 + exp(-g)); x is not rounded to fp16)
 *     then exactly sr_fwht_quant_act on x.
 *   G_f16, U_f16   fp16 [M, K], row strides ldg / ldu
 */
SR_API int sr_swiglu_fwht_quant_act(const void *G_f16, const void *U_f16, int64_t M, int64_t K,
                             int64_t ldg, int64_t ldu, const float *inv_s, float clip,
                             uint8_t *Xq, float *x_scale, void *stream);

/*
 * sr_fwht_quant_act with a head-wise Hadamard transform in place of the full one (paper,
 * section "Methodology": head-wise online Hadamard in the attention block).  The K axis is
 * seen as [n_heads, d], d = K / n_heads, both powers of two:
 *     across != 0:  H_{n_heads} (x) I_d   (mixes the heads, position inside the head kept)
 *     across == 0:  I_{n_heads} (x) H_d   (one transform of order d inside every head)
 * The two commute and compose to the full H_K.  K must be a power of two here;
 * 1 <= n_heads <= K (SR_ERR_ARG otherwise).
 */
SR_API int sr_fwht_quant_act_heads(const void *X_f16, int64_t M, int64_t K, int64_t ldx,
                            int64_t n_heads, int across, const float *inv_s, float clip,
                            uint8_t *Xq, float *x_scale, void *stream);

/*
 * sr_fold_smooth_rotate_quant with two options:
 *   n_heads, across   the transform folded into the weights: n_heads = 0 is the full Hadamard
 *                     (1/K folded into the scale); otherwise the head-wise transform of
 *                     sr_fwht_quant_act_heads (its order n_heads or K / n_heads folded instead).
 *   clip_steps, clip_lo   per-output-channel clipping ratio by linear search over the squared
 *                     quantisation error (paper, "Quantization" settings): candidates
 *                     r_i = 1 - (1 - clip_lo) * i / (clip_steps - 1), i = 0 .. clip_steps - 1;
 *                     err_i = sum_j (W^[j][n] - d_i * code_i(W^[j][n]))^2 with d_i = r_i * absmax / 7;
 *                     the smallest error wins, the larger ratio on ties.  clip_steps = 1 means
 *                     the fixed ratio clip_lo (plain RTN for 1.0).  1 <= clip_steps <= 32,
 *                     clip_lo in (0, 1].
 *   w_ratio           out, fp32 [N]: the ratio chosen per output channel; may be NULL.
 * Everything else as in sr_fold_smooth_rotate_quant (same workspace size).
 */
SR_API int sr_fold_smooth_rotate_quant_ex(const void *W_f16, int64_t K, int64_t N, int64_t ldw,
                                   const float *act_absmax, float alpha,
                                   int64_t n_heads, int across, int clip_steps, float clip_lo,
                                   uint8_t *Wq, float *w_scale, float *inv_s, float *w_ratio,
                                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * Asymmetric 4-bit group quantiser for keys and values (paper: Eq. (1), asymmetric case;
 * "Quantization" settings: group size 128, constant clipping ratio 0.95).  Per group of
 * `group` consecutive values of a row:
 *     hi = clip * max, lo = clip * min
 *     d  = (hi - lo) / 15        (1 when hi == lo)
 *     z  = -rint(lo / d)
 *     code = clamp(rint(v / d) + z, 0, 15),     dequantised value = (code - z) * d
 *
 *   X_f16   fp16 [rows, D], row stride ldx;  D a multiple of group;  group in {32, 64, 128, 256, 512}
 *   Q       out, uint8 [rows, D/2]: code(2b) in bits 0-3 of byte b, code(2b+1) in bits 4-7 (unsigned)
 *   scale   out, fp32 [rows, D/group]  (d);   zero  out, fp32 [rows, D/group]  (z, integer valued)
 */
SR_API int sr_kv_quant_asym(const void *X_f16, int64_t rows, int64_t D, int64_t ldx, int64_t group, float clip,
                     uint8_t *Q, float *scale, float *zero, void *stream);

/*
 * The whole online path of a decode step (up to 16 tokens) behind ONE call:
 *     exactly sr_fwht_quant_act(X, inv_s, clip) followed by sr_w4a4_gemm(..., SR_F16)
 * (paper: online Hadamard and per-token INT4 in front of the quantised projection, section
 * "Methodology", Eq. (1); Fig. 2 puts it in front of the down-projection, K = 14336 for an 8B model).
 * Codes and scales are the ones the two calls would produce, up to the rounding-order freedom of the
 * fp32 rotation (a code may sit on the other side of a rounding boundary).
 * One token with K = 2048 or 4096 runs as a SINGLE launch (rotation, quantiser and GEMM in one kernel, every
 * workgroup rotating the row while its weights travel): 8.0 us against 9.6 - 10.0 us for 4096 -> 14336.  Every
 * other shape runs the two kernels back to back inside the call -- measured, no single launch beats that pair
 * there (see csrc/linear_decode.hip) -- so the call is never slower than the two calls and saves their host side.
 *
 *   X_f16   fp16 [M, K], 1 <= M <= 16 (M = 0 is a no-op), row stride ldx
 *   K       2048, 4096, 8192 or 14336 (SR_ERR_UNSUPPORTED_K otherwise: use the two calls)
 *   Wq, w_scale   packed weights [N, K/2] and scales [N] from the fold; N a multiple of 16
 *   Y_f16   out, fp16 [M, N], row stride ldy
 *   Xq_out  out, optional (may be NULL): uint8 [M, K/2], the activation codes that were used
 *   x_scale_out  out, optional (may be NULL): fp32 [M]
 *   workspace    sr_linear_decode_workspace_bytes(M, K) bytes, 256-byte aligned: the codes and scales between the
 *                two kernels (may be NULL where that is 0: the single-launch shapes).  Contents need no
 *                initialisation; calls that share a workspace must not overlap.
 */
SR_API size_t sr_linear_decode_workspace_bytes(int64_t M, int64_t K);
SR_API int sr_w4a4_linear_decode(const void *X_f16, int64_t M, int64_t K, int64_t ldx,
                          const float *inv_s, float clip,
                          const uint8_t *Wq, const float *w_scale, int64_t N,
                          void *Y_f16, int64_t ldy,
                          uint8_t *Xq_out, float *x_scale_out,
                          void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * Fast prefill path: the same INT4 x INT4 product on the FP6 matrix pipe.
 *
 * gfx950 multiplies 6-bit floats at twice its int8 rate, and the 6-bit format E2M3 holds every
 * INT4 code exactly (value code / 8; pattern (code < 0 ? 32 : 0) | |code|), so the sums of the
 * paper's quantised forward pass come out bit for bit as from integer arithmetic (fp32
 * accumulation of integers / 64 below 2^24).  The operands are kept in "f6 tiles", a layout the
 * matrix instruction reads without any unpacking:
 *
 *   a code matrix [rows, K] (K % 128 == 0; rows padded to a multiple of 8 -- the padding rows may hold
 *   anything: sr_pack_f6_tiles writes zero codes there, sr_fwht_quant_act_f6 leaves them unwritten, and
 *   the GEMM multiplies them but never stores their outputs; every 6-bit pattern is a finite number) is
 *   cut into blocks of 8 rows x 128 codes; block (R, C) is 768 bytes at ((C * rows/8) + R) * 768
 *   (all row blocks of one 128-code chunk are contiguous);
 *   inside it, piece (r, t, g) = codes k = 128 C + 64 t + 32 g + j, j = 0..31, of row 8 R + r,
 *   code j in bits [6j, 6j+6) of a 24-byte little-endian string, whose first 16 bytes sit at
 *   256 t + 128 (g ^ (R & 1)) + 16 r and whose last 8 bytes at 512 + 128 (g ^ (R & 1)) + 16 r + 8 t.
 * ------------------------------------------------------------------------------------------ */

/* Bytes of the f6-tile form of a [rows, K] code matrix (0 if K % 128 != 0 or a size is <= 0). */
SR_API size_t sr_f6_tiles_bytes(int64_t rows, int64_t K);

/*
 * Repack canonical packed INT4 codes into f6 tiles (weights: once, offline; activations:
 * sr_fwht_quant_act_f6 writes the tiles directly).
 *   Q4   uint8 [rows, K/2] as written by the fold / the activation quantiser
 *   T6   out, sr_f6_tiles_bytes(rows, K) bytes, 16-byte aligned
 *   K a multiple of 128, rows * K < 2^32.
 */
SR_API int sr_pack_f6_tiles(const uint8_t *Q4, int64_t rows, int64_t K, uint8_t *T6, void *stream);

/*
 * sr_fwht_quant_act writing the activation codes as f6 tiles (same rotation, same scales, same
 * quantiser: clamp(rint(y / Delta), -8, 7), Eq. (1)).  The rounding is done by the hardware
 * FP6 conversion of the fp32 product y * (1 / Delta) instead of a fused multiply-add, so a code
 * may differ from the one sr_fwht_quant_act packs where y / Delta sits on a rounding boundary
 * (both are within the rounding freedom of the fp32 rotation).
 *   X6   out, sr_f6_tiles_bytes(M, K) bytes, 16-byte aligned; the rows that pad the last block of
 *        8 are left unwritten (the GEMM never stores their outputs)
 *   K    a supported Hadamard order that is a multiple of 128
 */
SR_API int sr_fwht_quant_act_f6(const void *X_f16, int64_t M, int64_t K, int64_t ldx,
                         const float *inv_s, float clip,
                         uint8_t *X6, float *x_scale, void *stream);

/*
 * sr_fwht_quant_act_f6 that, on the side, warms the memory-side cache (the 256 MB Infinity Cache in front of HBM)
 * for the call that follows: the launch reads one word of every 128-byte line of
 * [next_operand, next_operand + next_bytes) -- typically the f6-tile weights of the sr_w4a4_gemm_f6 that consumes
 * X6 -- so that the GEMM streams them from the cache instead of HBM (M = 2048, K = 4096: 2.5 us of 26 for
 * N = 4096, 4 us of 67 for N = 14336).  The outputs are exactly those of sr_fwht_quant_act_f6; the words read are
 * never used.  (The paper's deployment runs the online Hadamard + quantiser directly in front of each
 * projection; this pairs the two calls.)
 *   next_operand   device memory, readable for next_bytes bytes, 16-byte aligned; NULL with next_bytes = 0
 *                  gives sr_fwht_quant_act_f6
 *   next_bytes     the last next_bytes % 128 bytes are not touched
 * A hint: honoured where the launch is large enough to move megabytes on the side (K = 4096 with more than 1024
 * rows; K = 14336 and the other orders served by the default workgroup-per-row launch from 256 rows on), ignored
 * otherwise.  Errors as sr_fwht_quant_act_f6, plus SR_ERR_NULL / SR_ERR_ALIGN for the hint.
 */
SR_API int sr_fwht_quant_act_f6_warm(const void *X_f16, int64_t M, int64_t K, int64_t ldx,
                              const float *inv_s, float clip, uint8_t *X6, float *x_scale,
                              const void *next_operand, size_t next_bytes, void *stream);

/* sr_swiglu_fwht_quant_act writing f6 tiles (the down-projection input of a gated FFN on the fast path);
 * arguments as there, X6 / K as in sr_fwht_quant_act_f6. */
SR_API int sr_swiglu_fwht_quant_act_f6(const void *G_f16, const void *U_f16, int64_t M, int64_t K,
                                int64_t ldg, int64_t ldu, const float *inv_s, float clip,
                                uint8_t *X6, float *x_scale, void *stream);

/*
 * sr_w4a4_gemm on f6-tile operands: same sums (exact), same epilogue, same outputs.
 *   X6 = tiles of the activation codes [M, K], W6 = tiles of the weight codes [N, K].
 *   K a multiple of 128, K < 131072; N a multiple of 16; M * K and N * K below 2^32.
 *   workspace: none needed (pass NULL, 0).
 */
SR_API int sr_w4a4_gemm_f6(const uint8_t *X6, const float *x_scale,
                    const uint8_t *W6, const float *w_scale,
                    int64_t M, int64_t N, int64_t K,
                    void *Y, int64_t ldy, int out_dtype,
                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * sr_w4a4_gemm_f6 that, on the side, warms the memory-side cache for the call after it: where the launch has a
 * wave to spare -- the 256 x 128 tile configuration, which the dispatcher takes for shapes like M = 2048,
 * N = 4096, K = 4096: such a GEMM is short of L2 delivery and LDS bandwidth, HBM is mostly idle -- an extra wave
 * per workgroup reads one word of every 128-byte line of [next_operand, next_operand + next_bytes), spread over
 * the K loop; elsewhere the hint is ignored.  Typical use: the weights of the next linear layer (the paper's
 * deployment runs the projections of a block one after the other, Fig. 2), which a rotation + quantiser call
 * in between is too short to fetch without paying for it.  Outputs are exactly those of sr_w4a4_gemm_f6; the
 * words read are never used.
 *   next_operand   device memory, readable for next_bytes bytes, 16-byte aligned; NULL with next_bytes = 0
 *                  gives sr_w4a4_gemm_f6
 * Errors as sr_w4a4_gemm_f6; SR_ERR_NULL for next_bytes without next_operand, SR_ERR_ALIGN for a misaligned one.
 */
SR_API int sr_w4a4_gemm_f6_warm(const uint8_t *X6, const float *x_scale,
                         const uint8_t *W6, const float *w_scale,
                         int64_t M, int64_t N, int64_t K,
                         void *Y, int64_t ldy, int out_dtype,
                         const void *next_operand, size_t next_bytes,
                         void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * Measurement kernels (bench.py): what the chip sustains with nothing else in the way.  They compute
 * nothing of the method; their timings are the "measured ceilings" quoted beside the published peaks.
 * Each call enqueues ONE launch on `stream` and returns.  `sink` may be NULL (it is written only if a
 * checksum takes a value it cannot take; it exists so that the work cannot be optimised away).
 * ------------------------------------------------------------------------------------------ */

/* A pure read stream over [src, src + bytes): `grid` workgroups of `block` threads (a multiple of 64, at
 * most 1024), every thread keeping `in_flight` (1, 2, 4, 8 or 16) 16-byte loads in flight; nontemporal != 0
 * uses loads that do not allocate in the caches.  bytes a multiple of 16, src 16-byte aligned.
 * Algorithmic bytes per launch = bytes. */
SR_API int sr_ceiling_hbm_read(const void *src, size_t bytes, int grid, int block, int in_flight, int nontemporal,
                        uint32_t *sink, void *stream);

/* The memory traffic of a rotation + quantiser launch without the rotation: workgroup w (256 threads, lds_bytes of
 * LDS) reads row w of row_bytes from src with all loads issued up front, folds it, and writes out_bytes that depend
 * on every load to row w of dst; `grid` workgroups walk over `rows` rows.  src holds rows * row_bytes bytes, dst
 * rows * out_bytes; both 16-byte aligned, sizes multiples of 16.
 * Algorithmic bytes per launch = rows * (row_bytes + out_bytes). */
SR_API int sr_ceiling_row_stream(const void *src, void *dst, int64_t rows, int64_t row_bytes, int64_t out_bytes, int grid,
                          int lds_bytes, void *stream);

/* A bare issue loop of the FP6 matrix instruction of sr_w4a4_gemm_f6 (32 x 32 x 64 per instruction): `grid`
 * workgroups of 8 waves, each wave 8 independent accumulator tiles, `iters` rounds of 8 instructions, operands
 * taken once from `fields` (at least 9216 bytes of 6-bit patterns, e.g. the first bytes of an f6-tile buffer).
 * Operations per launch = grid * 8 waves * iters * 8 * 2 * 32 * 32 * 64. */
SR_API int sr_ceiling_mfma_f6(const void *fields, size_t bytes, int iters, int grid, float *sink, void *stream);

/* The same for the int8 matrix instruction of sr_w4a4_gemm (32 x 32 x 32 per instruction); `operands`: at least
 * 6144 bytes.  Operations per launch = grid * 8 * iters * 8 * 2 * 32 * 32 * 32. */
SR_API int sr_ceiling_mfma_i8(const void *operands, size_t bytes, int iters, int grid, int *sink, void *stream);

/* A bare loop of fp32 vector arithmetic in the mix of the rotation kernels' register passes: `grid` workgroups of
 * 4 waves, per iteration and wave 160 additions / subtractions and 32 multiplications.
 * Vector instructions per launch = grid * 4 * iters * 192 (each over 64 lanes). */
SR_API int sr_ceiling_valu_f32(int iters, int grid, float *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SMOOTHROT_H */
