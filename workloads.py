"""Seeded synthetic inputs for the W4A4 linear workloads.

This module only draws random tensors with the shapes, value distributions and
outlier structure of the benchmark configurations.  It contains none of the
method's arithmetic (no smoothing, rotation, quantisation or GEMM), so that it
can serve the CPU oracle and the HIP library alike.

Every draw comes from numpy's counter-based Philox generator keyed with
(seed, stream), is made in fp32 and is then cast to fp16 with saturation at
+-65504 (no infinities reach the kernels).

The structure mimics what the paper describes for LLM activations: a few
"massive outlier" channels whose magnitude is ~1000x the rest (section
"Massive Activation Outliers"), here applied to whole channels.
"""
from __future__ import annotations

import numpy as np

F16_MAX = 65504.0

# streams of the Philox key, so that tensors of one config are independent
_S_CHANNELS, _S_X, _S_W, _S_ROWSCALE, _S_CALIB, _S_B = 1, 2, 3, 4, 1000, 5


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def to_f16_sat(x: np.ndarray) -> np.ndarray:
    """fp32 -> fp16, clamping to the finite fp16 range first."""
    return np.clip(x, -F16_MAX, F16_MAX).astype(np.float16)


def outlier_channels(seed: int, K: int, n_out: int) -> np.ndarray:
    """Indices of the outlier channels of a config (drawn before anything else)."""
    return np.sort(_rng(seed, _S_CHANNELS).choice(K, size=n_out, replace=False))


def gauss_weights(seed: int, K: int, N: int, std: float) -> np.ndarray:
    """W fp16 [K, N] row-major, entries ~ N(0, std^2)."""
    w = _rng(seed, _S_W).standard_normal((K, N), dtype=np.float32) * np.float32(std)
    return to_f16_sat(w)


def gauss_acts(seed: int, M: int, K: int, n_out: int, out_scale: float,
               row_lognormal_sigma: float = 0.0, stream: int = _S_X) -> np.ndarray:
    """X fp16 [M, K] ~ N(0,1); n_out whole channels multiplied by out_scale;
    optionally each token row multiplied by exp(sigma * z_m), z_m ~ N(0,1)."""
    x = _rng(seed, stream).standard_normal((M, K), dtype=np.float32)
    if n_out:
        x[:, outlier_channels(seed, K, n_out)] *= np.float32(out_scale)
    if row_lognormal_sigma:
        z = _rng(seed, _S_ROWSCALE + 7919 * stream).standard_normal(M).astype(np.float32)
        x *= np.exp(np.float32(row_lognormal_sigma) * z)[:, None]
    return to_f16_sat(x)


def glu_acts(seed: int, M: int, K: int, n_out: int, out_scale: float,
             stream: int = _S_X) -> np.ndarray:
    """X fp16 [M, K] = SiLU(a) * b with a, b ~ N(0,1): the shape of a gated FFN's
    down-projection input; n_out whole channels multiplied by out_scale."""
    a = _rng(seed, stream).standard_normal((M, K), dtype=np.float32)
    b = _rng(seed, _S_B + 7919 * stream).standard_normal((M, K), dtype=np.float32)
    x = a / (1.0 + np.exp(-a)) * b
    if n_out:
        x[:, outlier_channels(seed, K, n_out)] *= np.float32(out_scale)
    return to_f16_sat(x)


def gate_up(seed: int, M: int, K: int, n_out: int, out_scale: float, stream: int = _S_X):
    """(G, U) fp16 [M, K], both ~ N(0,1): the two branches of a gated FFN before the
    non-linearity; n_out whole channels of U multiplied by out_scale (same draws as glu_acts)."""
    a = _rng(seed, stream).standard_normal((M, K), dtype=np.float32)
    b = _rng(seed, _S_B + 7919 * stream).standard_normal((M, K), dtype=np.float32)
    if n_out:
        b[:, outlier_channels(seed, K, n_out)] *= np.float32(out_scale)
    return to_f16_sat(a), to_f16_sat(b)


def kv_acts(seed: int, rows: int, D: int, stream: int = _S_X) -> np.ndarray:
    """Key / value rows fp16 [rows, D]: N(0,1) entries plus a fixed per-channel offset
    ~ N(0, 0.5^2) (keys carry channel biases, so groups are not centred on zero)."""
    x = _rng(seed, stream).standard_normal((rows, D), dtype=np.float32)
    x += np.float32(0.5) * _rng(seed, _S_CHANNELS + 50).standard_normal(D).astype(np.float32)[None, :]
    return to_f16_sat(x)


# --------------------------------------------------------------------------
# The configurations (numbered as in the benchmark description, 1-based).
# --------------------------------------------------------------------------

def cfg1():
    """Tiny single linear: X [16,512] with 4 outlier channels x500, W [512,512]
    ~ N(0, 0.02^2), calibration on the same X; seed 0."""
    seed, M, K, N = 0, 16, 512, 512
    X = gauss_acts(seed, M, K, 4, 500.0)
    W = gauss_weights(seed, K, N, 0.02)
    return dict(X=X, W=W, calib=[X], alpha=0.5, M=M, K=K, N=N)


def cfg2_X(M: int = 2048, K: int = 4096, seed: int = 1) -> np.ndarray:
    """Prefill activations: N(0,1), 6 outlier channels x1000, per-token
    LogNormal(0, 0.5) scale."""
    return gauss_acts(seed, M, K, 6, 1000.0, row_lognormal_sigma=0.5)


def cfg2_W(N: int, K: int = 4096, seed: int = 1) -> np.ndarray:
    """W [K, N] ~ N(0, 0.02^2); a different stream per N so the two shapes of the
    config do not share a prefix."""
    w = _rng(seed, _S_W + N).standard_normal((K, N), dtype=np.float32) * np.float32(0.02)
    return to_f16_sat(w)


def cfg2_calib_chunk(i: int, T: int = 2048, K: int = 4096, seed: int = 1) -> np.ndarray:
    """i-th calibration sequence ([T, K], fresh draw, same outlier channels and
    distribution as cfg2_X)."""
    return gauss_acts(seed, T, K, 6, 1000.0, row_lognormal_sigma=0.5, stream=_S_CALIB + i)


def cfg3_X(M: int = 2048, K: int = 14336, seed: int = 2) -> np.ndarray:
    """Down-projection input: SiLU(a)*b, 3 outlier channels x800."""
    return glu_acts(seed, M, K, 3, 800.0)


def cfg3_W(N: int = 4096, K: int = 14336, seed: int = 2) -> np.ndarray:
    """W [14336, N] ~ N(0, 0.015^2)."""
    return gauss_weights(seed, K, N, 0.015)


def cfg3_calib_chunk(i: int, T: int = 2048, K: int = 14336, seed: int = 2) -> np.ndarray:
    return glu_acts(seed, T, K, 3, 800.0, stream=_S_CALIB + i)


def cfg4_X(M: int, K: int) -> np.ndarray:
    """Decode activations: the first M token rows of the matching prefill generator
    (K=4096: cfg2, K=14336: cfg3), drawn with their own seed 3."""
    if K == 14336:
        return glu_acts(3, M, K, 3, 800.0)
    return gauss_acts(3, M, K, 6, 1000.0, row_lognormal_sigma=0.5)


def cfg4_W(K: int, N: int) -> np.ndarray:
    return gauss_weights(3 + (K == 14336), K, N, 0.015 if K == 14336 else 0.02)


# LLaMA-3.1-8B decoder-layer linears (name, K, N)
CFG5_LINEARS = (("q", 4096, 4096), ("k", 4096, 1024), ("v", 4096, 1024), ("o", 4096, 4096),
                ("gate", 4096, 14336), ("up", 4096, 14336), ("down", 14336, 4096))


def cfg5_W(name: str, seed: int = 4) -> np.ndarray:
    for i, (nm, K, N) in enumerate(CFG5_LINEARS):
        if nm == name:
            w = _rng(seed, _S_W + 100 + i).standard_normal((K, N), dtype=np.float32)
            return to_f16_sat(w * np.float32(0.015 if K == 14336 else 0.02))
    raise KeyError(name)


def cfg5_X(M: int, K: int = 4096, seed: int = 4, stream: int = _S_X) -> np.ndarray:
    """RMS-normalised N(0,1) rows with the cfg2 outlier channels (6 x1000)."""
    x = _rng(seed, stream).standard_normal((M, K), dtype=np.float32)
    x[:, outlier_channels(seed, K, 6)] *= np.float32(1000.0)
    x /= np.sqrt(np.mean(x.astype(np.float64) ** 2, axis=1, keepdims=True)).astype(np.float32)
    return to_f16_sat(x)


def random_codes(seed: int, rows: int, K: int) -> np.ndarray:
    """Uniform INT4 codes in [-8, 7], int8 [rows, K] (GEMM-only tests)."""
    return _rng(seed, 77).integers(-8, 8, size=(rows, K), dtype=np.int8)
