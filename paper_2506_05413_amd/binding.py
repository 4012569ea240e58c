"""ctypes binding of libsmoothrot.so -- argument marshalling only.

Function names and argument order follow include/smoothrot.h.  torch supplies
device memory and the current stream; every step of the computation runs in the
library's HIP kernels.  There is no fallback: if the shared library is missing
or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

SR_OK, SR_ERR_NULL, SR_ERR_SHAPE, SR_ERR_UNSUPPORTED_K = 0, 1, 2, 3
SR_ERR_ALIGN, SR_ERR_ARG, SR_ERR_WORKSPACE, SR_ERR_DEVICE = 4, 5, 6, 7
SR_F16, SR_I32 = 0, 1
SR_TUNE_GEMM_TILE, SR_TUNE_GEMM_GRID, SR_TUNE_GEMM_XCDM, SR_TUNE_DECODE_KERNEL = 0, 1, 2, 3
SR_TUNE_FWHT4096, SR_TUNE_FWHT_STREAM, SR_TUNE_GEMM_WARM = 4, 5, 6
SR_TUNE_KNOBS = 7
SR_TUNE_AUTO = -(1 << 63)

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsmoothrot.so")

_c = ctypes
_vp, _i64, _f32, _sz, _int = _c.c_void_p, _c.c_int64, _c.c_float, _c.c_size_t, _c.c_int

_SIGNATURES = {
    "sr_status_str": (_c.c_char_p, [_int]),
    "sr_hadamard_supported": (_int, [_i64]),
    "sr_tune_set": (_int, [_int, _i64]),
    "sr_tune_get": (_i64, [_int]),
    "sr_fold_workspace_bytes": (_sz, [_i64, _i64]),
    "sr_gemm_workspace_bytes": (_sz, [_i64, _i64, _i64]),
    "sr_calib_absmax": (_int, [_vp, _i64, _i64, _i64, _vp, _vp]),
    "sr_fold_smooth_rotate_quant": (_int, [_vp, _i64, _i64, _i64, _vp, _f32, _f32, _vp, _vp, _vp, _vp, _sz, _vp]),
    "sr_noalloc_scratch_bytes": (_sz, []),
    "sr_fold_smooth_rotate_quant_noalloc": (_int, [_vp, _i64, _i64, _i64, _vp, _f32, _f32, _vp, _vp, _vp, _vp]),
    "sr_fwht_quant_act": (_int, [_vp, _i64, _i64, _i64, _vp, _f32, _vp, _vp, _vp]),
    "sr_w4a4_gemm": (_int, [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _i64, _int, _vp, _sz, _vp]),
    "sr_swiglu_fwht_quant_act": (_int, [_vp, _vp, _i64, _i64, _i64, _i64, _vp, _f32, _vp, _vp, _vp]),
    "sr_fwht_quant_act_heads": (_int, [_vp, _i64, _i64, _i64, _i64, _int, _vp, _f32, _vp, _vp, _vp]),
    "sr_fold_smooth_rotate_quant_ex": (_int, [_vp, _i64, _i64, _i64, _vp, _f32, _i64, _int, _int, _f32,
                                               _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "sr_kv_quant_asym": (_int, [_vp, _i64, _i64, _i64, _i64, _f32, _vp, _vp, _vp, _vp]),
    "sr_f6_tiles_bytes": (_sz, [_i64, _i64]),
    "sr_pack_f6_tiles": (_int, [_vp, _i64, _i64, _vp, _vp]),
    "sr_fwht_quant_act_f6": (_int, [_vp, _i64, _i64, _i64, _vp, _f32, _vp, _vp, _vp]),
    "sr_fwht_quant_act_f6_warm": (_int, [_vp, _i64, _i64, _i64, _vp, _f32, _vp, _vp, _vp, _sz, _vp]),
    "sr_swiglu_fwht_quant_act_f6": (_int, [_vp, _vp, _i64, _i64, _i64, _i64, _vp, _f32, _vp, _vp, _vp]),
    "sr_w4a4_gemm_f6": (_int, [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _i64, _int, _vp, _sz, _vp]),
    "sr_w4a4_gemm_f6_warm": (_int, [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _i64, _int, _vp, _sz, _vp, _sz, _vp]),
    "sr_ceiling_hbm_read": (_int, [_vp, _sz, _int, _int, _int, _int, _vp, _vp]),
    "sr_ceiling_row_stream": (_int, [_vp, _vp, _i64, _i64, _i64, _int, _int, _vp]),
    "sr_ceiling_mfma_f6": (_int, [_vp, _sz, _int, _int, _vp, _vp]),
    "sr_ceiling_mfma_i8": (_int, [_vp, _sz, _int, _int, _vp, _vp]),
    "sr_ceiling_valu_f32": (_int, [_int, _int, _vp, _vp]),
    "sr_linear_decode_workspace_bytes": (_sz, [_i64, _i64]),
    "sr_w4a4_linear_decode": (_int, [_vp, _i64, _i64, _i64, _vp, _f32, _vp, _vp, _i64, _vp, _i64, _vp, _vp, _vp, _sz, _vp]),
}

_lib = None


class SmoothRotError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = raw().sr_status_str(status).decode()
        super().__init__("%s: status %d (%s)" % (where, status, msg))


def raw() -> ctypes.CDLL:
    """The loaded C library with argtypes set (loads it on first use)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libsmoothrot.so is not built: run `python -m paper_2506_05413_amd.build` "
                              "(there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _check(status: int, where: str):
    if status != SR_OK:
        raise SmoothRotError(status, where)


def _dev(t: torch.Tensor, dtype, name: str):
    if not t.is_cuda:
        raise ValueError("%s must be a device tensor" % name)
    if t.dtype != dtype:
        raise ValueError("%s must have dtype %s" % (name, dtype))
    if t.dim() == 2 and t.stride(1) != 1 or t.dim() == 1 and t.numel() > 1 and t.stride(0) != 1:
        raise ValueError("%s must be contiguous along its last dimension" % name)


def sr_status_str(status: int) -> str:
    return raw().sr_status_str(status).decode()


def sr_hadamard_supported(K: int) -> bool:
    return bool(raw().sr_hadamard_supported(K))


def sr_tune_set(knob: int, value: int = SR_TUNE_AUTO) -> None:
    """Process-wide override of a dispatch heuristic (tests and tuning); SR_TUNE_AUTO restores the default."""
    _check(raw().sr_tune_set(knob, value), "sr_tune_set")


def sr_tune_get(knob: int) -> int:
    return int(raw().sr_tune_get(knob))


def sr_fold_workspace_bytes(K: int, N: int) -> int:
    return int(raw().sr_fold_workspace_bytes(K, N))


def sr_gemm_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(raw().sr_gemm_workspace_bytes(M, N, K))


def sr_calib_absmax(X: torch.Tensor, absmax_io: torch.Tensor) -> torch.Tensor:
    """absmax_io[j] <- max(absmax_io[j], max_t |X[t][j]|); X fp16 [T, K], absmax_io fp32 [K]."""
    _dev(X, torch.float16, "X"); _dev(absmax_io, torch.float32, "absmax_io")
    T, K = X.shape
    ldx = X.stride(0) if T > 1 else K
    _check(raw().sr_calib_absmax(_ptr(X), T, K, ldx, _ptr(absmax_io), _stream()), "sr_calib_absmax")
    return absmax_io


def sr_fold_smooth_rotate_quant(W, act_absmax, alpha: float, w_clip: float = 1.0,
                                Wq=None, w_scale=None, inv_s=None, workspace=None):
    """W fp16 [K, N] -> (Wq uint8 [N, K/2], w_scale fp32 [N], inv_s fp32 [K])."""
    _dev(W, torch.float16, "W")
    K, N = W.shape
    dev = W.device
    Wq = torch.empty((N, K // 2), dtype=torch.uint8, device=dev) if Wq is None else Wq
    w_scale = torch.empty(N, dtype=torch.float32, device=dev) if w_scale is None else w_scale
    inv_s = torch.empty(K, dtype=torch.float32, device=dev) if inv_s is None else inv_s
    if workspace is None:
        workspace = torch.empty(max(sr_fold_workspace_bytes(K, N), 256), dtype=torch.uint8, device=dev)
    _check(raw().sr_fold_smooth_rotate_quant(_ptr(W), K, N, W.stride(0), _ptr(act_absmax), alpha, w_clip,
                                             _ptr(Wq), _ptr(w_scale), _ptr(inv_s), _ptr(workspace),
                                             workspace.numel(), _stream()),
           "sr_fold_smooth_rotate_quant")
    return Wq, w_scale, inv_s


def sr_noalloc_scratch_bytes() -> int:
    return int(raw().sr_noalloc_scratch_bytes())


def sr_fold_smooth_rotate_quant_noalloc(W, act_absmax, alpha: float, w_clip, Wq, w_scale, inv_s):
    """sr_fold_smooth_rotate_quant on the library's device-resident scratch: the caller passes every output
    (nothing is allocated here either); returns (Wq, w_scale, inv_s)."""
    _dev(W, torch.float16, "W"); _dev(Wq, torch.uint8, "Wq"); _dev(w_scale, torch.float32, "w_scale")
    K, N = W.shape
    _check(raw().sr_fold_smooth_rotate_quant_noalloc(_ptr(W), K, N, W.stride(0), _ptr(act_absmax), alpha, w_clip,
                                                     _ptr(Wq), _ptr(w_scale), _ptr(inv_s), _stream()),
           "sr_fold_smooth_rotate_quant_noalloc")
    return Wq, w_scale, inv_s


def sr_fwht_quant_act(X, inv_s, clip: float = 0.9, Xq=None, x_scale=None):
    """X fp16 [M, K] -> (Xq uint8 [M, K/2], x_scale fp32 [M])."""
    _dev(X, torch.float16, "X")
    M, K = X.shape
    Xq = torch.empty((M, K // 2), dtype=torch.uint8, device=X.device) if Xq is None else Xq
    x_scale = torch.empty(M, dtype=torch.float32, device=X.device) if x_scale is None else x_scale
    ldx = X.stride(0) if M > 1 else K
    _check(raw().sr_fwht_quant_act(_ptr(X), M, K, ldx, _ptr(inv_s), clip, _ptr(Xq), _ptr(x_scale), _stream()),
           "sr_fwht_quant_act")
    return Xq, x_scale


def sr_w4a4_gemm(Xq, x_scale, Wq, w_scale, out_dtype: int = SR_F16, Y=None, workspace=None):
    """Xq uint8 [M, K/2], Wq uint8 [N, K/2] -> Y [M, N] fp16 (dequantised) or int32 (accumulators)."""
    _dev(Xq, torch.uint8, "Xq"); _dev(Wq, torch.uint8, "Wq")
    M, Kb = Xq.shape
    N = Wq.shape[0]
    if Wq.shape[1] != Kb:
        raise ValueError("Xq and Wq disagree on K")
    if Y is None:
        Y = torch.empty((M, N), dtype=torch.float16 if out_dtype == SR_F16 else torch.int32, device=Xq.device)
    ldy = Y.stride(0) if M > 1 else N
    if workspace is None:
        need = sr_gemm_workspace_bytes(M, N, 2 * Kb)
        if need:
            workspace = torch.empty(need, dtype=torch.uint8, device=Xq.device)
    _check(raw().sr_w4a4_gemm(_ptr(Xq), _ptr(x_scale), _ptr(Wq), _ptr(w_scale), M, N, 2 * Kb, _ptr(Y), ldy,
                              out_dtype, _ptr(workspace), 0 if workspace is None else workspace.numel(),
                              _stream()),
           "sr_w4a4_gemm")
    return Y


def sr_swiglu_fwht_quant_act(G, U, inv_s, clip: float = 0.9, Xq=None, x_scale=None):
    """G, U fp16 [M, K] -> codes and scales of silu(G) * U (smoothed, rotated, quantised)."""
    _dev(G, torch.float16, "G"); _dev(U, torch.float16, "U")
    M, K = U.shape
    if tuple(G.shape) != (M, K):
        raise ValueError("G and U must have the same shape")
    Xq = torch.empty((M, K // 2), dtype=torch.uint8, device=U.device) if Xq is None else Xq
    x_scale = torch.empty(M, dtype=torch.float32, device=U.device) if x_scale is None else x_scale
    ldg = G.stride(0) if M > 1 else K
    ldu = U.stride(0) if M > 1 else K
    _check(raw().sr_swiglu_fwht_quant_act(_ptr(G), _ptr(U), M, K, ldg, ldu, _ptr(inv_s), clip, _ptr(Xq),
                                          _ptr(x_scale), _stream()), "sr_swiglu_fwht_quant_act")
    return Xq, x_scale


def sr_fwht_quant_act_heads(X, n_heads: int, across: bool, inv_s, clip: float = 0.9, Xq=None, x_scale=None):
    """X fp16 [M, K] -> codes and scales after the head-wise Hadamard transform."""
    _dev(X, torch.float16, "X")
    M, K = X.shape
    Xq = torch.empty((M, K // 2), dtype=torch.uint8, device=X.device) if Xq is None else Xq
    x_scale = torch.empty(M, dtype=torch.float32, device=X.device) if x_scale is None else x_scale
    ldx = X.stride(0) if M > 1 else K
    _check(raw().sr_fwht_quant_act_heads(_ptr(X), M, K, ldx, n_heads, int(bool(across)), _ptr(inv_s), clip,
                                         _ptr(Xq), _ptr(x_scale), _stream()), "sr_fwht_quant_act_heads")
    return Xq, x_scale


def sr_fold_smooth_rotate_quant_ex(W, act_absmax, alpha: float, n_heads: int = 0, across: bool = False,
                                   clip_steps: int = 1, clip_lo: float = 1.0,
                                   Wq=None, w_scale=None, inv_s=None, w_ratio=None, workspace=None):
    """W fp16 [K, N] -> (Wq, w_scale, inv_s, w_ratio fp32 [N])."""
    _dev(W, torch.float16, "W")
    K, N = W.shape
    dev = W.device
    Wq = torch.empty((N, K // 2), dtype=torch.uint8, device=dev) if Wq is None else Wq
    w_scale = torch.empty(N, dtype=torch.float32, device=dev) if w_scale is None else w_scale
    inv_s = torch.empty(K, dtype=torch.float32, device=dev) if inv_s is None else inv_s
    w_ratio = torch.empty(N, dtype=torch.float32, device=dev) if w_ratio is None else w_ratio
    if workspace is None:
        workspace = torch.empty(max(sr_fold_workspace_bytes(K, N), 256), dtype=torch.uint8, device=dev)
    _check(raw().sr_fold_smooth_rotate_quant_ex(_ptr(W), K, N, W.stride(0), _ptr(act_absmax), alpha, n_heads,
                                                int(bool(across)), clip_steps, clip_lo, _ptr(Wq), _ptr(w_scale),
                                                _ptr(inv_s), _ptr(w_ratio), _ptr(workspace), workspace.numel(),
                                                _stream()),
           "sr_fold_smooth_rotate_quant_ex")
    return Wq, w_scale, inv_s, w_ratio


def sr_kv_quant_asym(X, group: int = 128, clip: float = 0.95, Q=None, scale=None, zero=None):
    """X fp16 [rows, D] -> (Q uint8 [rows, D/2], scale fp32 [rows, D/group], zero fp32 [rows, D/group])."""
    _dev(X, torch.float16, "X")
    rows, D = X.shape
    ng = max(D // group, 1)
    Q = torch.empty((rows, D // 2), dtype=torch.uint8, device=X.device) if Q is None else Q
    scale = torch.empty((rows, ng), dtype=torch.float32, device=X.device) if scale is None else scale
    zero = torch.empty((rows, ng), dtype=torch.float32, device=X.device) if zero is None else zero
    ldx = X.stride(0) if rows > 1 else D
    _check(raw().sr_kv_quant_asym(_ptr(X), rows, D, ldx, group, clip, _ptr(Q), _ptr(scale), _ptr(zero), _stream()),
           "sr_kv_quant_asym")
    return Q, scale, zero


def sr_linear_decode_workspace_bytes(M: int, K: int) -> int:
    return int(raw().sr_linear_decode_workspace_bytes(M, K))


def sr_w4a4_linear_decode(X, inv_s, Wq, w_scale, clip: float = 0.9, Y=None, Xq_out=None, x_scale_out=None,
                          workspace=None):
    """X fp16 [M <= 16, K], Wq uint8 [N, K/2] -> Y fp16 [M, N] in one launch (rotate, quantise, multiply).
    workspace: a uint8 device tensor of sr_linear_decode_workspace_bytes(M, K) bytes (reuse it from call to call);
    one is made per call if none is given."""
    _dev(X, torch.float16, "X"); _dev(Wq, torch.uint8, "Wq")
    M, K = X.shape
    N = Wq.shape[0]
    if Wq.shape[1] * 2 != K:
        raise ValueError("X and Wq disagree on K")
    Y = torch.empty((M, N), dtype=torch.float16, device=X.device) if Y is None else Y
    ldx = X.stride(0) if M > 1 else K
    ldy = Y.stride(0) if M > 1 else N
    need = sr_linear_decode_workspace_bytes(M, K)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    _check(raw().sr_w4a4_linear_decode(_ptr(X), M, K, ldx, _ptr(inv_s), clip, _ptr(Wq), _ptr(w_scale), N, _ptr(Y),
                                       ldy, _ptr(Xq_out), _ptr(x_scale_out), _ptr(workspace),
                                       0 if workspace is None else workspace.numel(), _stream()), "sr_w4a4_linear_decode")
    return Y


def sr_f6_tiles_bytes(rows: int, K: int) -> int:
    return int(raw().sr_f6_tiles_bytes(rows, K))


def sr_pack_f6_tiles(Q4, T6=None):
    """Q4 uint8 [rows, K/2] (canonical packed INT4 codes) -> T6 uint8 [sr_f6_tiles_bytes(rows, K)] (f6 tiles)."""
    _dev(Q4, torch.uint8, "Q4")
    if not Q4.is_contiguous():
        raise ValueError("Q4 must be contiguous")
    rows, Kb = Q4.shape
    if T6 is None:
        T6 = torch.empty(max(sr_f6_tiles_bytes(rows, 2 * Kb), 16), dtype=torch.uint8, device=Q4.device)
    _check(raw().sr_pack_f6_tiles(_ptr(Q4), rows, 2 * Kb, _ptr(T6), _stream()), "sr_pack_f6_tiles")
    return T6


def sr_w4a4_gemm_f6(X6, x_scale, W6, w_scale, M: int, N: int, K: int, out_dtype: int = SR_F16, Y=None, warm=None):
    """X6, W6 = f6 tiles of the codes [M, K] and [N, K] -> Y [M, N] fp16 (dequantised) or int32 (accumulators).
    warm: a contiguous device tensor (the weights of the next linear) to be pulled into the memory-side cache on
    the side where the launch has a wave to spare (sr_w4a4_gemm_f6_warm)."""
    _dev(X6, torch.uint8, "X6"); _dev(W6, torch.uint8, "W6")
    if X6.numel() < sr_f6_tiles_bytes(M, K) or W6.numel() < sr_f6_tiles_bytes(N, K):
        raise ValueError("tile buffers are smaller than sr_f6_tiles_bytes says")
    if Y is None:
        Y = torch.empty((M, N), dtype=torch.float16 if out_dtype == SR_F16 else torch.int32, device=X6.device)
    ldy = Y.stride(0) if M > 1 else N
    if warm is not None:
        if not (warm.is_cuda and warm.is_contiguous()):
            raise ValueError("warm must be a contiguous device tensor")
        _check(raw().sr_w4a4_gemm_f6_warm(_ptr(X6), _ptr(x_scale), _ptr(W6), _ptr(w_scale), M, N, K, _ptr(Y), ldy,
                                          out_dtype, _ptr(warm), warm.numel() * warm.element_size(), None, 0, _stream()),
               "sr_w4a4_gemm_f6_warm")
        return Y
    _check(raw().sr_w4a4_gemm_f6(_ptr(X6), _ptr(x_scale), _ptr(W6), _ptr(w_scale), M, N, K, _ptr(Y), ldy,
                                 out_dtype, None, 0, _stream()), "sr_w4a4_gemm_f6")
    return Y


def sr_w4a4_gemm_f6_warm(X6, x_scale, W6, w_scale, M: int, N: int, K: int, warm, out_dtype: int = SR_F16, Y=None):
    """sr_w4a4_gemm_f6 with the cache-warming hint (same outputs)."""
    return sr_w4a4_gemm_f6(X6, x_scale, W6, w_scale, M, N, K, out_dtype, Y, warm)


def sr_fwht_quant_act_f6(X, inv_s, clip: float = 0.9, X6=None, x_scale=None, warm=None):
    """X fp16 [M, K] -> (X6 uint8 [sr_f6_tiles_bytes(M, K)] f6 tiles of the codes, x_scale fp32 [M]).
    warm: a contiguous device tensor (the weights of the GEMM that follows) to be pulled into the memory-side
    cache on the side (sr_fwht_quant_act_f6_warm)."""
    _dev(X, torch.float16, "X")
    M, K = X.shape
    if X6 is None:
        X6 = torch.zeros(max(sr_f6_tiles_bytes(M, K), 16), dtype=torch.uint8, device=X.device)
    x_scale = torch.empty(M, dtype=torch.float32, device=X.device) if x_scale is None else x_scale
    ldx = X.stride(0) if M > 1 else K
    if warm is not None:
        if not (warm.is_cuda and warm.is_contiguous()):
            raise ValueError("warm must be a contiguous device tensor")
        _check(raw().sr_fwht_quant_act_f6_warm(_ptr(X), M, K, ldx, _ptr(inv_s), clip, _ptr(X6), _ptr(x_scale),
                                               _ptr(warm), warm.numel() * warm.element_size(), _stream()),
               "sr_fwht_quant_act_f6_warm")
        return X6, x_scale
    _check(raw().sr_fwht_quant_act_f6(_ptr(X), M, K, ldx, _ptr(inv_s), clip, _ptr(X6), _ptr(x_scale), _stream()),
           "sr_fwht_quant_act_f6")
    return X6, x_scale


def sr_fwht_quant_act_f6_warm(X, inv_s, clip: float, next_operand, X6=None, x_scale=None):
    """sr_fwht_quant_act_f6 that also pulls `next_operand` (a contiguous device tensor, typically the f6-tile
    weights of the GEMM that follows) into the memory-side cache; same outputs."""
    return sr_fwht_quant_act_f6(X, inv_s, clip, X6, x_scale, warm=next_operand)


def sr_swiglu_fwht_quant_act_f6(G, U, inv_s, clip: float = 0.9, X6=None, x_scale=None):
    """G, U fp16 [M, K] -> f6 tiles and scales of silu(G) * U (smoothed, rotated, quantised)."""
    _dev(G, torch.float16, "G"); _dev(U, torch.float16, "U")
    M, K = U.shape
    if tuple(G.shape) != (M, K):
        raise ValueError("G and U must have the same shape")
    if X6 is None:
        X6 = torch.zeros(max(sr_f6_tiles_bytes(M, K), 16), dtype=torch.uint8, device=U.device)
    x_scale = torch.empty(M, dtype=torch.float32, device=U.device) if x_scale is None else x_scale
    ldg = G.stride(0) if M > 1 else K
    ldu = U.stride(0) if M > 1 else K
    _check(raw().sr_swiglu_fwht_quant_act_f6(_ptr(G), _ptr(U), M, K, ldg, ldu, _ptr(inv_s), clip, _ptr(X6),
                                             _ptr(x_scale), _stream()), "sr_swiglu_fwht_quant_act_f6")
    return X6, x_scale


def sr_ceiling_hbm_read(src, grid: int, block: int = 256, in_flight: int = 8, nontemporal: bool = True):
    """Measurement kernel: reads every byte of `src` (a contiguous device tensor) once."""
    _check(raw().sr_ceiling_hbm_read(_ptr(src), src.numel() * src.element_size(), grid, block, in_flight,
                                     int(bool(nontemporal)), None, _stream()), "sr_ceiling_hbm_read")


def sr_ceiling_row_stream(src, dst, rows: int, row_bytes: int, out_bytes: int, grid: int, lds_bytes: int = 1024):
    """Measurement kernel: reads rows * row_bytes from src, writes rows * out_bytes to dst (a row's output depends
    on all of the row)."""
    if src.numel() * src.element_size() < rows * row_bytes or dst.numel() * dst.element_size() < rows * out_bytes:
        raise ValueError("buffers smaller than the rows say")
    _check(raw().sr_ceiling_row_stream(_ptr(src), _ptr(dst), rows, row_bytes, out_bytes, grid, lds_bytes, _stream()),
           "sr_ceiling_row_stream")


def sr_ceiling_mfma_f6(fields, iters: int, grid: int):
    """Measurement kernel: bare FP6 matrix-instruction loop; returns the operations of the launch."""
    _check(raw().sr_ceiling_mfma_f6(_ptr(fields), fields.numel() * fields.element_size(), iters, grid, None, _stream()),
           "sr_ceiling_mfma_f6")
    return grid * 8 * iters * 8 * 2.0 * 32 * 32 * 64


def sr_ceiling_mfma_i8(operands, iters: int, grid: int):
    """Measurement kernel: bare int8 matrix-instruction loop; returns the operations of the launch."""
    _check(raw().sr_ceiling_mfma_i8(_ptr(operands), operands.numel() * operands.element_size(), iters, grid, None,
                                    _stream()), "sr_ceiling_mfma_i8")
    return grid * 8 * iters * 8 * 2.0 * 32 * 32 * 32


def sr_ceiling_valu_f32(iters: int, grid: int):
    """Measurement kernel: bare fp32 vector-ALU loop; returns the wave-level vector instructions of the launch."""
    _check(raw().sr_ceiling_valu_f32(iters, grid, None, _stream()), "sr_ceiling_valu_f32")
    return grid * 4 * iters * 192.0
