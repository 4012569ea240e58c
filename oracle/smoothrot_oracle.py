"""CPU oracle for the SmoothRot W4A4 linear layer.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 / exact-integer statement of what the hot path computes,
written from the paper (SmoothRot, arXiv 2506.05413).  It shares no code with
the HIP library and must never be imported by the product path: only tests,
the smoke check and the benchmark's cpu_baseline leg may call it.

Every function names the passage it follows.  Where the paper leaves a choice
open the reading taken is stated in the docstring (and collected in the design
notes of the repository).

Conventions
-----------
* X is [tokens, c_in] (row = token), W is [c_in, c_out]  ("Y = XW", Eq. (2)).
* T(v) = v @ H is THE rotation operator, applied to rows of X and to columns of
  diag(s) W, with H an unnormalised +-1 Hadamard matrix of order n = c_in;
  the 1/n of H H^T = n I is folded into the weights.
* INT4 codes are two's-complement integers in [-8, 7]; packed two per byte,
  even index in bits 0-3, odd index in bits 4-7.

All functions pinned by tests/test_oracle_pins.py; none is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

QMIN, QMAX = -8, 7          # signed 4-bit range
FLOOR = 1e-5                # lower clamp of calibration / weight absmax before the powers


# ---------------------------------------------------------------------------
# Hadamard matrices (section "Methodology": exact Hadamard transform online;
# the paper fixes neither size nor construction -- Sylvester for 2^p, Paley-I
# of order 28 Kronecker Sylvester for 28*2^p are this build's reading).
# ---------------------------------------------------------------------------

def sylvester(n: int) -> np.ndarray:
    """H[i][j] = (-1)^popcount(i & j), natural order, n a power of two."""
    assert n >= 1 and n & (n - 1) == 0
    i = np.arange(n)
    bits = i[:, None] & i[None, :]
    pop = np.zeros((n, n), dtype=np.int64)
    while bits.any():
        pop += bits & 1
        bits >>= 1
    return (1 - 2 * (pop & 1)).astype(np.int64)


def _gf27_mul(a: int, b: int) -> int:
    """Product in GF(27) = GF(3)[x]/(x^3 + 2x + 1); an element is the integer
    c0 + 3 c1 + 9 c2 for the polynomial c0 + c1 x + c2 x^2."""
    ca = [a % 3, a // 3 % 3, a // 9]
    cb = [b % 3, b // 3 % 3, b // 9]
    prod = [0] * 5
    for i in range(3):
        for j in range(3):
            prod[i + j] += ca[i] * cb[j]
    # x^3 = -2x - 1 = x + 2 (mod 3);  x^4 = x^2 + 2x
    for d in (4, 3):
        c = prod[d]
        prod[d] = 0
        prod[d - 3] += 2 * c
        prod[d - 2] += c
    c = [p % 3 for p in prod[:3]]
    return c[0] + 3 * c[1] + 9 * c[2]


def _gf27_sub(a: int, b: int) -> int:
    ca = [a % 3, a // 3 % 3, a // 9]
    cb = [b % 3, b // 3 % 3, b // 9]
    c = [(x - y) % 3 for x, y in zip(ca, cb)]
    return c[0] + 3 * c[1] + 9 * c[2]


def gf27_squares() -> set:
    """The 13 non-zero squares of GF(27)."""
    return {_gf27_mul(e, e) for e in range(1, 27)}


def paley28() -> np.ndarray:
    """Paley type-I Hadamard matrix of order 28 (q = 27 = 3 mod 4):
    Q[i][j] = chi(e_i - e_j) with chi the quadratic character of GF(27),
    H = [[1, 1^T], [-1, Q + I]]."""
    sq = gf27_squares()
    chi = [0] + [1 if e in sq else -1 for e in range(1, 27)]
    Q = np.array([[chi[_gf27_sub(i, j)] for j in range(27)] for i in range(27)], dtype=np.int64)
    H = np.empty((28, 28), dtype=np.int64)
    H[0, :] = 1
    H[1:, 0] = -1
    H[1:, 1:] = Q + np.eye(27, dtype=np.int64)
    return H


def hadamard_supported(n: int) -> bool:
    def pow2(v):
        return v >= 1 and v & (v - 1) == 0
    return pow2(n) or (n % 28 == 0 and pow2(n // 28))


def hadamard_dense(n: int) -> np.ndarray:
    """Explicit H of order n: Sylvester for 2^p; H28 (x) H_{2^p} for 28*2^p with
    (A(x)B)[i1*m + i2][j1*m + j2] = A[i1][j1] * B[i2][j2] (the 28-index is slow)."""
    if n & (n - 1) == 0:
        return sylvester(n)
    assert n % 28 == 0 and hadamard_supported(n)
    return np.kron(paley28(), sylvester(n // 28))


def fwht_pow2(x: np.ndarray) -> np.ndarray:
    """x @ sylvester(n) along the last axis by radix-2 butterflies (fp64).
    Verified against the explicit product in the pins before anything uses it."""
    n = x.shape[-1]
    assert n & (n - 1) == 0
    y = np.array(x, dtype=np.float64).reshape(-1, n)
    rows = y.shape[0]
    h = 1
    while h < n:
        y = y.reshape(rows, n // (2 * h), 2, h)
        lo = y[:, :, 0, :] + y[:, :, 1, :]
        hi = y[:, :, 0, :] - y[:, :, 1, :]
        y = np.stack((lo, hi), axis=2)
        h *= 2
    return y.reshape(x.shape)


def rotate(x: np.ndarray) -> np.ndarray:
    """T(x) = x @ H along the last axis, H = hadamard_dense(n) (never formed for
    large n).  For n = 28*m: y[j1, j2] = sum_{i1} H28[i1][j1] * (x[i1, :] @ H_m)[j2]."""
    n = x.shape[-1]
    assert hadamard_supported(n)
    if n & (n - 1) == 0:
        return fwht_pow2(x)
    m = n // 28
    z = fwht_pow2(np.asarray(x, dtype=np.float64).reshape(-1, 28, m))
    y = np.einsum("ij,rim->rjm", paley28().astype(np.float64), z)
    return y.reshape(x.shape)


# ---------------------------------------------------------------------------
# Quantiser (section "Background", Eq. (1); settings in "Experimental settings /
# Quantization": per-token symmetric activations with a constant clipping
# ratio, per-channel symmetric RTN weights).
# ---------------------------------------------------------------------------

def quant_sym_int4(v: np.ndarray, clip: float):
    """Row-wise symmetric 4-bit quantisation of v [rows, n] (fp64).

    Delta = clip * max_j |v_j| / (2^(b-1) - 1) = clip * absmax / 7, z = 0,
    code = clamp(rint(v / Delta), -8, 7).  Readings: 'max(X)' is the maximum of
    absolute values; the symmetric clamp range is the signed one; rounding is
    round-half-to-even; an all-zero row takes Delta = 1 (codes 0).
    Returns (codes int8 [rows, n], Delta fp64 [rows], t = v / Delta fp64)."""
    v = np.asarray(v, dtype=np.float64)
    absmax = np.max(np.abs(v), axis=1)
    delta = clip * absmax / float(QMAX)
    delta = np.where(absmax == 0.0, 1.0, delta)
    t = v / delta[:, None]
    codes = np.clip(np.rint(t), QMIN, QMAX).astype(np.int8)
    return codes, delta, t


def dequant(codes: np.ndarray, delta: np.ndarray) -> np.ndarray:
    """Q(X) = (X_int - z) * Delta with z = 0 (Eq. (1) ff.)."""
    return codes.astype(np.float64) * np.asarray(delta, dtype=np.float64)[:, None]


def pack_int4(codes: np.ndarray) -> np.ndarray:
    """[rows, n] int8 in [-8,7] -> [rows, n/2] uint8; byte b = code(2b) in bits 0-3,
    code(2b+1) in bits 4-7 (two's-complement nibbles)."""
    c = np.asarray(codes).astype(np.int16)
    assert c.shape[-1] % 2 == 0 and c.min(initial=0) >= QMIN and c.max(initial=0) <= QMAX
    lo = c[..., 0::2] & 0xF
    hi = c[..., 1::2] & 0xF
    return (lo | (hi << 4)).astype(np.uint8)


def unpack_int4(packed: np.ndarray) -> np.ndarray:
    p = np.asarray(packed, dtype=np.uint8).astype(np.int16)
    lo = p & 0xF
    hi = p >> 4
    lo = np.where(lo >= 8, lo - 16, lo)
    hi = np.where(hi >= 8, hi - 16, hi)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.int8)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    return out


# ---------------------------------------------------------------------------
# Offline: calibration and the weight fold (section "Methodology").
# ---------------------------------------------------------------------------

def calib_absmax(X: np.ndarray, absmax_io: np.ndarray) -> np.ndarray:
    """a_j <- max(a_j, max_t |X_tj|): the per-channel activation maximum that the
    smoothing factors are calibrated from.  Returns the updated vector (fp64)."""
    a = np.asarray(absmax_io, dtype=np.float64)
    if X.shape[0] == 0:
        return a.copy()
    return np.maximum(a, np.max(np.abs(np.asarray(X, dtype=np.float64)), axis=0))


def smoothing_factors(act_absmax: np.ndarray, W: np.ndarray, alpha: float) -> np.ndarray:
    """s_j = max|X_j|^alpha / max|W_j|^(1-alpha); W_j is row j of W [c_in, c_out]
    (input channel j), taken on the weight as given (before any transform).
    Both maxima are clamped below at 1e-5 (degenerate channels)."""
    a = np.maximum(np.asarray(act_absmax, dtype=np.float64), FLOOR)
    w = np.maximum(np.max(np.abs(np.asarray(W, dtype=np.float64)), axis=1), FLOOR)
    return a ** alpha / w ** (1.0 - alpha)


def fold_smooth_rotate_quant(W: np.ndarray, act_absmax, alpha: float, w_clip: float = 1.0):
    """Weights of the transformed layer, Eq. (2) with A^-1 = H^T diag(s) / n:

        W_hat[j][c] = (1/n) sum_k H[k][j] s_k W[k][c]      (= T applied to columns of diag(s) W)

    then per-output-channel symmetric RTN INT4.  act_absmax None means s = 1
    (rotation only).  Returns dict with
      codes  int8 [c_out, c_in]   (output channel major, c_in contiguous)
      packed uint8 [c_out, c_in/2]
      w_scale fp64 [c_out], s, inv_s fp64 [c_in], W_hat fp64 [c_in, c_out], t (pre-round) [c_out, c_in]."""
    Wd = np.asarray(W, dtype=np.float64)
    K, N = Wd.shape
    s = np.ones(K) if act_absmax is None else smoothing_factors(act_absmax, Wd, alpha)
    sw_t = (s[:, None] * Wd).T                   # [c_out, c_in]: columns of diag(s) W as rows
    what_t = rotate(np.ascontiguousarray(sw_t)) / float(K)
    codes, w_scale, t = quant_sym_int4(what_t, w_clip)
    return dict(codes=codes, packed=pack_int4(codes), w_scale=w_scale, s=s, inv_s=1.0 / s,
                W_hat=what_t.T, t=t)


# ---------------------------------------------------------------------------
# Online: rotate + quantise activations, integer GEMM, dequantise.
# ---------------------------------------------------------------------------

def fwht_quant_act(X: np.ndarray, inv_s, clip: float = 0.9):
    """x_hat = (x * inv_s) @ H per token row (smoothing then the online Hadamard),
    then per-token symmetric INT4 with clipping ratio `clip` (paper: 0.9).
    inv_s None = already smoothed upstream (the deployment of Fig. 2).
    Returns dict codes int8 [M,K], packed uint8 [M,K/2], x_scale fp64 [M], y fp64, t fp64."""
    Xd = np.asarray(X, dtype=np.float64)
    if inv_s is not None:
        Xd = Xd * np.asarray(inv_s, dtype=np.float64)[None, :]
    y = rotate(Xd)
    codes, x_scale, t = quant_sym_int4(y, clip)
    return dict(codes=codes, packed=pack_int4(codes), x_scale=x_scale, y=y, t=t)


def gemm_i32(cx: np.ndarray, cw: np.ndarray) -> np.ndarray:
    """acc[m][c] = sum_j cx[m][j] * cw[c][j] in int64, asserted to fit int32.
    cx [M, K], cw [N, K] integer codes."""
    acc = cx.astype(np.int64) @ cw.astype(np.int64).T
    assert np.abs(acc).max(initial=0) < 2 ** 31
    return acc


def dequant_out(acc: np.ndarray, x_scale: np.ndarray, w_scale: np.ndarray) -> np.ndarray:
    """Y[m][c] = acc[m][c] * Delta_x[m] * Delta_w[c]  (Q(X) Q(W) with both zero-points 0)."""
    return acc.astype(np.float64) * np.asarray(x_scale, np.float64)[:, None] * np.asarray(w_scale, np.float64)[None, :]


def w4a4_linear(X, W, act_absmax, alpha=0.5, clip=0.9, w_clip=1.0, use_c=False):
    """The whole layer: fold (offline) -> rotate+quantise activations -> integer GEMM
    -> dequantise.  Returns (Y fp64, parts)."""
    f = fold_smooth_rotate_quant(W, act_absmax, alpha, w_clip)
    a = fwht_quant_act(X, None if act_absmax is None else f["inv_s"], clip)
    acc = (gemm_i32_c if use_c else gemm_i32)(a["codes"], f["codes"])
    return dequant_out(acc, a["x_scale"], f["w_scale"]), dict(fold=f, act=a, acc=acc)


# ---------------------------------------------------------------------------
# Rows around the core path: the gated FFN input, head-wise Hadamard transforms,
# the weight clipping-ratio search and the KV-cache quantiser.
# ---------------------------------------------------------------------------

def swiglu(G: np.ndarray, U: np.ndarray) -> np.ndarray:
    """Input of the down-projection (Fig. 2, FFN block): sigma(gate) * up with
    sigma(g) = g / (1 + exp(-g)) (SiLU), elementwise, fp64."""
    g = np.asarray(G, dtype=np.float64)
    with np.errstate(over="ignore"):                 # exp(-g) = inf for very negative g: g / inf = -0
        return g / (1.0 + np.exp(-g)) * np.asarray(U, dtype=np.float64)


def fwht_quant_swiglu(G, U, inv_s, clip: float = 0.9):
    """fwht_quant_act applied to x = sigma(gate) * up without rounding x to fp16 in
    between (the smoothing, rotation and quantiser of Fig. 2's FFN branch)."""
    return fwht_quant_act(swiglu(G, U), inv_s, clip)


def rotate_heads(x: np.ndarray, n_heads: int, across: bool) -> np.ndarray:
    """Head-wise Hadamard transforms on a [.., n_heads * d] axis seen as [n_heads, d]
    (section "Methodology": the head-wise online Hadamard of the attention block).

    across=True : H_{n_heads} (x) I_d -- mixes the heads, position inside the head kept;
    across=False: I_{n_heads} (x) H_d -- one transform of order d inside every head.
    Both orders are powers of two (Sylvester).  Their composition is the full
    H_{n_heads * d}, which the pins check."""
    n = x.shape[-1]
    assert n % n_heads == 0
    d = n // n_heads
    v = np.asarray(x, dtype=np.float64).reshape(-1, n_heads, d)
    if across:
        y = np.einsum("ij,rid->rjd", sylvester(n_heads).astype(np.float64), v)
    else:
        y = fwht_pow2(v)
    return y.reshape(x.shape)


def fwht_quant_act_heads(X, n_heads: int, across: bool, inv_s, clip: float = 0.9):
    """fwht_quant_act with the head-wise transform in place of the full one."""
    Xd = np.asarray(X, dtype=np.float64)
    if inv_s is not None:
        Xd = Xd * np.asarray(inv_s, dtype=np.float64)[None, :]
    y = rotate_heads(Xd, n_heads, across)
    codes, x_scale, t = quant_sym_int4(y, clip)
    return dict(codes=codes, packed=pack_int4(codes), x_scale=x_scale, y=y, t=t)


def clip_grid(steps: int = 21, lo: float = 0.5) -> np.ndarray:
    """Candidate clipping ratios of the weight search, 1.0 down to `lo` in equal steps
    (the paper says 'linear search' and names no grid; 1.00, 0.975, .. 0.50 is this
    build's reading)."""
    return 1.0 - (1.0 - lo) * np.arange(steps) / float(steps - 1)


def weight_clip_search(v: np.ndarray, grid: np.ndarray):
    """Per-row clipping ratio by linear search over the squared error ("Quantization"
    settings: weights RTN per channel, clipping ratios by a linear search over the squared
    error).  For every ratio r of `grid` (descending): Delta = r * absmax / 7,
    c = clamp(rint(v / Delta), -8, 7), err_r = sum_j (v_j - Delta * c_j)^2; the row takes
    the ratio of smallest error, the first (largest) one on ties.
    Returns (best ratio [rows], err [rows, len(grid)], codes, Delta, t) for the chosen ratio."""
    v = np.asarray(v, dtype=np.float64)
    errs = np.empty((v.shape[0], len(grid)))
    for i, r in enumerate(grid):
        c, d, _ = quant_sym_int4(v, float(r))
        errs[:, i] = np.sum((v - dequant(c, d)) ** 2, axis=1)
    best = np.argmin(errs, axis=1)            # first minimum = largest ratio
    ratio = np.asarray(grid, dtype=np.float64)[best]
    absmax = np.max(np.abs(v), axis=1)
    delta = np.where(absmax == 0.0, 1.0, ratio * absmax / float(QMAX))
    t = v / delta[:, None]
    codes = np.clip(np.rint(t), QMIN, QMAX).astype(np.int8)
    return ratio, errs, codes, delta, t


def fold_clip_search(W, act_absmax, alpha: float, grid: np.ndarray):
    """fold_smooth_rotate_quant with the per-output-channel clipping ratio searched."""
    Wd = np.asarray(W, dtype=np.float64)
    K, N = Wd.shape
    s = np.ones(K) if act_absmax is None else smoothing_factors(act_absmax, Wd, alpha)
    what_t = rotate(np.ascontiguousarray((s[:, None] * Wd).T)) / float(K)
    ratio, errs, codes, w_scale, t = weight_clip_search(what_t, grid)
    return dict(codes=codes, packed=pack_int4(codes), w_scale=w_scale, s=s, inv_s=1.0 / s,
                ratio=ratio, errs=errs, t=t, W_hat_t=what_t)


def quant_asym_int4_groups(v: np.ndarray, group: int = 128, clip: float = 0.95):
    """Asymmetric 4-bit quantisation of consecutive groups of `group` values along the
    last axis (Eq. (1), asymmetric case; "Quantization" settings: keys and values,
    group size 128, constant clipping ratio 0.95):

        hi = clip * max, lo = clip * min over the group
        Delta = (hi - lo) / 15,  z = -rint(lo / Delta)
        code  = clamp(rint(v / Delta) + z, 0, 15),   Q(v) = (code - z) * Delta

    Readings: the clipping ratio shrinks both ends of the range; a group whose range is
    zero takes Delta = 1; z is kept as an integer of any size (a group that does not
    straddle zero has z outside 0..15).
    Returns (codes uint8 [rows, n], Delta [rows, n/group], z [rows, n/group] int64,
    u = v / Delta pre-round [rows, n], lo / Delta pre-round [rows, n/group])."""
    v = np.asarray(v, dtype=np.float64)
    rows, n = v.shape
    assert n % group == 0
    g = v.reshape(rows, n // group, group)
    hi = clip * g.max(axis=2)
    lo = clip * g.min(axis=2)
    delta = (hi - lo) / 15.0
    delta = np.where(hi == lo, 1.0, delta)
    zt = lo / delta
    z = -np.rint(zt).astype(np.int64)
    u = g / delta[:, :, None]
    codes = np.clip(np.rint(u) + z[:, :, None], 0, 15).astype(np.uint8)
    return codes.reshape(rows, n), delta, z, u.reshape(rows, n), zt


def dequant_asym(codes, delta, z, group: int = 128) -> np.ndarray:
    """Q(v) = (code - z) * Delta per group (Eq. (1) ff.)."""
    rows, n = codes.shape
    c = codes.reshape(rows, n // group, group).astype(np.float64)
    return ((c - np.asarray(z, np.float64)[:, :, None]) * np.asarray(delta, np.float64)[:, :, None]).reshape(rows, n)


def pack_uint4(codes: np.ndarray) -> np.ndarray:
    """[rows, n] codes in 0..15 -> [rows, n/2] bytes, even index in bits 0-3."""
    c = np.asarray(codes).astype(np.uint8)
    assert c.max(initial=0) <= 15
    return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)


# ---------------------------------------------------------------------------
# INT4 codes as 6-bit floats: the arithmetic claim behind running the quantised
# forward pass on a 6-bit float matrix pipe is that the element format E2M3 holds
# every code c exactly as c / 8, so the sums stay the integers of gemm_i32 (which
# remains the definition).  Only the format's value function lives here; the byte
# layout a library stores such operands in is that library's business and is
# decoded on the test side.
# ---------------------------------------------------------------------------

def e2m3_value(bits) -> np.ndarray:
    """Value of a 6-bit float with 1 sign, 2 exponent and 3 mantissa bits, bias 1, no
    infinities or NaNs (the OCP microscaling FP6 E2M3 element format): subnormal
    (-1)^s * 2^0 * (m/8) for e = 0, else (-1)^s * 2^(e-1) * (1 + m/8)."""
    b = np.asarray(bits).astype(np.int64)
    s, e, m = (b >> 5) & 1, (b >> 3) & 3, b & 7
    mag = np.where(e == 0, m / 8.0, (1.0 + m / 8.0) * np.exp2(e - 1.0))
    return np.where(s == 1, -mag, mag)


# ---------------------------------------------------------------------------
# The same integer GEMM as a plain C triple loop (oracle/gemm_i4.c), for sizes
# where numpy's int64 matmul is too slow.  Pinned to gemm_i32 in the tests.
# ---------------------------------------------------------------------------

_HERE = os.path.dirname(os.path.abspath(__file__))
_C_SRC = os.path.join(_HERE, "gemm_i4.c")
_C_LIB = os.path.join(_HERE, "liboracle_gemm.so")
_lib = None


def build_c(force: bool = False) -> str:
    if force or not os.path.exists(_C_LIB) or os.path.getmtime(_C_LIB) < os.path.getmtime(_C_SRC):
        subprocess.check_call(["gcc", "-O3", "-fopenmp", "-shared", "-fPIC", "-o", _C_LIB, _C_SRC])
    return _C_LIB


def _c_lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build_c())
        _lib.oracle_gemm_i4.restype = ctypes.c_int
        _lib.oracle_gemm_i4.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                        ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p]
        _lib.oracle_threads.restype = ctypes.c_int
    return _lib


def c_threads() -> int:
    return int(_c_lib().oracle_threads())


def gemm_i32_c(cx: np.ndarray, cw: np.ndarray) -> np.ndarray:
    cx = np.ascontiguousarray(cx, dtype=np.int8)
    cw = np.ascontiguousarray(cw, dtype=np.int8)
    M, K = cx.shape
    N, K2 = cw.shape
    assert K == K2
    acc = np.empty((M, N), dtype=np.int64)
    rc = _c_lib().oracle_gemm_i4(cx.ctypes.data, cw.ctypes.data, M, N, K, acc.ctypes.data)
    assert rc == 0, "accumulator left the int32 range"
    return acc
