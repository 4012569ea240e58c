"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests compares the oracle with itself or with the HIP path: each
checks a closed form, an invariant, a brute-force evaluation on tiny inputs, a
hand-worked fixture, or a special case that reduces to a textbook identity.
They are chosen so that a plausible mistake (a dropped term, a wrong sign or
index, a transposed operand, a wrong divisor) fails at least one of them.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import smoothrot_oracle as o
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------- Hadamard

@pytest.mark.parametrize("n", [1, 2, 4, 8, 64, 512, 1024])
def test_sylvester_orthogonal_symmetric_recursive(n):
    H = o.sylvester(n)
    assert set(np.unique(H)) <= {-1, 1}
    assert np.array_equal(H @ H.T, n * np.eye(n, dtype=np.int64))
    assert np.array_equal(H, H.T)
    if n >= 2:
        h = o.sylvester(n // 2)
        assert np.array_equal(H, np.block([[h, h], [h, -h]]))


def test_sylvester_4096_orthogonal():
    H = o.sylvester(4096).astype(np.float64)      # +-1 entries: the fp64 product is exact
    G = H @ H.T
    assert np.array_equal(G, 4096.0 * np.eye(4096))


def test_sylvester_popcount_entries():
    H = o.sylvester(16)
    for i, j in itertools.product(range(16), repeat=2):
        assert H[i, j] == (-1) ** bin(i & j).count("1")


def _gf27_pow(e, k):
    r = 1
    for _ in range(k):
        r = o._gf27_mul(r, e)
    return r


def test_gf27_is_a_field_and_euler_criterion():
    # multiplicative group of order 26: every non-zero element has e^26 = 1, no zero divisors
    for e in range(1, 27):
        assert _gf27_pow(e, 26) == 1
        assert all(o._gf27_mul(e, f) != 0 for f in range(1, 27))
    sq = o.gf27_squares()
    assert len(sq) == 13
    # Euler: e is a square iff e^((q-1)/2) = 1; otherwise it is -1 = 2
    for e in range(1, 27):
        assert _gf27_pow(e, 13) == (1 if e in sq else 2)
    assert 2 not in sq                           # -1 is a non-square because q = 3 mod 4
    # distributivity spot check of the reduction polynomial: x * x^2 = x^3 = x + 2
    assert o._gf27_mul(3, 9) == 2 + 3 * 1


def test_paley28_properties():
    H = o.paley28()
    assert set(np.unique(H)) == {-1, 1}
    I28 = np.eye(28, dtype=np.int64)
    assert np.array_equal(H @ H.T, 28 * I28)
    assert np.array_equal(H.T @ H, 28 * I28)
    Q = H[1:, 1:] - np.eye(27, dtype=np.int64)
    assert np.array_equal(Q, -Q.T)               # skew because q = 3 mod 4
    assert np.all(Q.sum(axis=1) == 0) and np.all(np.diag(Q) == 0)
    assert np.array_equal(Q @ Q.T, 27 * np.eye(27, dtype=np.int64) - np.ones((27, 27), dtype=np.int64))
    assert np.array_equal(H + H.T, 2 * I28)      # skew-type Hadamard
    assert not np.array_equal(H, H.T)            # so H versus H^T matters below


def test_kronecker_dense_small_and_index_order():
    H = o.hadamard_dense(28 * 4)
    assert np.array_equal(H @ H.T, 112 * np.eye(112, dtype=np.int64))
    A, B = o.paley28(), o.sylvester(4)
    for (i1, i2, j1, j2) in [(0, 0, 0, 0), (5, 3, 17, 2), (27, 1, 1, 3), (13, 2, 26, 1)]:
        assert H[i1 * 4 + i2, j1 * 4 + j2] == A[i1, j1] * B[i2, j2]


@pytest.mark.parametrize("n", [2, 8, 64, 512, 1024, 28, 56, 224, 896])
def test_rotate_equals_dense_product_exactly(n):
    rng = np.random.default_rng(n)
    x = rng.integers(-1000, 1000, size=(5, n)).astype(np.float64)
    assert np.array_equal(o.rotate(x), x @ o.hadamard_dense(n).astype(np.float64))


@pytest.mark.parametrize("n", [64, 896])
def test_rotate_unit_vectors_give_rows_of_H(n):
    H = o.hadamard_dense(n)
    for k in (0, 1, n // 2 + 3, n - 1):
        e = np.zeros((1, n))
        e[0, k] = 1.0
        assert np.array_equal(o.rotate(e)[0], H[k].astype(np.float64))


def _rotate_transposed(y):
    """y @ H^T written independently of oracle.rotate for n = 28*m (test-side helper)."""
    n = y.shape[-1]
    if n & (n - 1) == 0:
        return o.fwht_pow2(y)                    # Sylvester is symmetric
    m = n // 28
    z = o.fwht_pow2(y.reshape(-1, 28, m))
    return np.einsum("ji,rim->rjm", o.paley28().astype(np.float64), z).reshape(y.shape)


@pytest.mark.parametrize("n", [4096, 14336])
def test_rotate_full_size_inverse_and_parseval(n):
    rng = np.random.default_rng(7)
    x = rng.integers(-50, 50, size=(3, n)).astype(np.float64)
    y = o.rotate(x)
    assert np.array_equal(_rotate_transposed(y), n * x)          # H H^T = n I
    assert np.array_equal((y * y).sum(axis=1), n * (x * x).sum(axis=1))
    if n & (n - 1) == 0:
        assert np.array_equal(o.rotate(y), n * x)                # involution up to n


# ---------------------------------------------------------------- quantiser

def _load_hand_row():
    clip, xs, codes = None, [], []
    with open(os.path.join(GOLDEN, "hand_quant_row.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            p = line.split()
            if p[0] == "clip":
                clip = float(p[1])
            else:
                xs.append(float(p[0]))
                codes.append(int(p[1]))
    return clip, np.array([xs]), np.array(codes)


def test_quantiser_hand_worked_row():
    clip, x, want = _load_hand_row()
    codes, delta, _ = o.quant_sym_int4(x, clip)
    assert delta[0] == 1.0
    assert np.array_equal(codes[0], want)
    assert set(range(-8, 8)) <= set(codes[0].tolist())           # every one of the 16 codes occurs


def test_quantiser_properties():
    rng = np.random.default_rng(3)
    v = rng.standard_normal((64, 256)) * np.exp(rng.standard_normal((64, 1)))
    for clip in (1.0, 0.9):
        c, d, t = o.quant_sym_int4(v, clip)
        assert c.min() >= -8 and c.max() <= 7
        np.testing.assert_allclose(d * 7.0, clip * np.abs(v).max(axis=1), rtol=1e-15)
        unclipped = np.abs(t) <= 7.5
        assert np.all(np.abs(v - o.dequant(c, d))[unclipped] <= d[:, None].repeat(256, 1)[unclipped] / 2 * (1 + 1e-12))
        c2, d2, _ = o.quant_sym_int4(v * 2.0 ** -9, clip)     # power-of-two scaling: same codes
        assert np.array_equal(c, c2) and np.array_equal(d2, d * 2.0 ** -9)
    c, d, _ = o.quant_sym_int4(v, 1.0)
    am = np.abs(v).argmax(axis=1)
    assert np.all(np.abs(c[np.arange(64), am]) == 7) and c.min() >= -7
    c9, _, _ = o.quant_sym_int4(v, 0.9)
    assert c9.min() == -8                                     # with clip < 1 the code -8 is reachable
    cz, dz, _ = o.quant_sym_int4(np.zeros((2, 8)), 0.9)
    assert np.all(cz == 0) and np.all(dz == 1.0)


def test_pack_roundtrip_all_bytes_and_examples():
    allb = np.arange(256, dtype=np.uint8).reshape(1, 256)
    codes = o.unpack_int4(allb)
    assert codes.min() == -8 and codes.max() == 7
    assert np.array_equal(o.pack_int4(codes), allb)
    assert o.pack_int4(np.array([[-8, 7]]))[0, 0] == 0x78
    assert o.pack_int4(np.array([[1, -1]]))[0, 0] == 0xF1
    assert o.unpack_int4(np.array([[0x8F]], dtype=np.uint8)).tolist() == [[-1, -8]]


# ------------------------------------------------------- smoothing and fold

def test_smoothing_closed_forms():
    rng = np.random.default_rng(5)
    W = rng.standard_normal((32, 48)) * 0.02
    a = np.abs(rng.standard_normal(32)) * 10 + 0.1
    w = np.abs(W).max(axis=1)
    s = o.smoothing_factors(a, W, 0.5)
    np.testing.assert_allclose(a / s, np.sqrt(a * w), rtol=1e-13)      # balanced at alpha = 1/2
    np.testing.assert_allclose(s * w, np.sqrt(a * w), rtol=1e-13)
    np.testing.assert_allclose(a / o.smoothing_factors(a, W, 1.0), 1.0, rtol=1e-13)
    np.testing.assert_allclose(o.smoothing_factors(a, W, 0.0) * w, 1.0, rtol=1e-13)
    s3 = o.smoothing_factors(a, W, 0.3)
    np.testing.assert_allclose(np.log(s3), 0.3 * np.log(a) - 0.7 * np.log(w), rtol=1e-12)
    # degenerate channels are floored, never 0 or inf
    a0 = a.copy(); a0[3] = 0.0
    W0 = W.copy(); W0[4, :] = 0.0
    s0 = o.smoothing_factors(a0, W0, 0.5)
    assert np.all(np.isfinite(s0)) and np.all(s0 > 0)
    assert s0[3] == pytest.approx(np.sqrt(1e-5 / w[3])) and s0[4] == pytest.approx(np.sqrt(a[4] / 1e-5))


@pytest.mark.parametrize("K", [64, 112])
def test_fold_identity_eq2(K):
    """(X diag(1/s) H)(H^T diag(s) W)/n = X W in fp64 (Eq. (2)); K=112 uses the
    non-symmetric H28 so a transposed operand on either side fails."""
    rng = np.random.default_rng(K)
    X = rng.standard_normal((9, K)) * (1 + 50 * (rng.random(K) < 0.05))
    W = rng.standard_normal((K, 24)) * 0.02
    a = np.abs(X).max(axis=0)
    f = o.fold_smooth_rotate_quant(W, a, 0.5)
    act = o.fwht_quant_act(X, f["inv_s"], 0.9)
    Y = X @ W
    np.testing.assert_allclose(act["y"] @ f["W_hat"], Y, rtol=0, atol=1e-12 * np.abs(Y).max())
    # explicit matrices, written out
    H = o.hadamard_dense(K).astype(np.float64)
    np.testing.assert_allclose(f["W_hat"], H.T @ np.diag(f["s"]) @ W / K, rtol=0, atol=1e-15)
    np.testing.assert_allclose(act["y"], X @ np.diag(1 / f["s"]) @ H, rtol=0, atol=1e-10)
    if K == 112:   # sensitivity: the wrong transpose is not an equivalent transformation
        bad = (X @ np.diag(1 / f["s"]) @ H.T) @ f["W_hat"]
        assert np.abs(bad - Y).max() > 1e-3 * np.abs(Y).max()
    # rotation only
    f1 = o.fold_smooth_rotate_quant(W, None, 0.5)
    assert np.all(f1["s"] == 1.0)
    np.testing.assert_allclose(o.rotate(X) @ f1["W_hat"], Y, rtol=0, atol=1e-12 * np.abs(Y).max())


def test_fold_quantises_per_output_channel():
    rng = np.random.default_rng(11)
    W = rng.standard_normal((64, 16)) * 0.02
    W[:, 5] *= 40.0                                  # one loud output channel must not affect the others
    f = o.fold_smooth_rotate_quant(W, None, 0.5, 1.0)
    assert f["codes"].shape == (16, 64) and f["packed"].shape == (16, 32)
    np.testing.assert_allclose(f["w_scale"] * 7.0, np.abs(f["W_hat"]).max(axis=0), rtol=1e-14)
    assert np.all(np.abs(f["codes"]).max(axis=1) == 7)
    err = np.abs(f["codes"].T * f["w_scale"][None, :] - f["W_hat"])
    assert np.all(err <= f["w_scale"][None, :] / 2 * (1 + 1e-12))
    assert np.array_equal(o.unpack_int4(f["packed"]), f["codes"])


# --------------------------------------------------------------------- GEMM

def test_gemm_bruteforce_and_bounds():
    rng = np.random.default_rng(2)
    cx = rng.integers(-8, 8, size=(3, 10)).astype(np.int8)
    cw = rng.integers(-8, 8, size=(4, 10)).astype(np.int8)
    want = [[sum(int(cx[m, j]) * int(cw[c, j]) for j in range(10)) for c in range(4)] for m in range(3)]
    assert o.gemm_i32(cx, cw).tolist() == want
    assert o.gemm_i32_c(cx, cw).tolist() == want
    K = 512
    worst = o.gemm_i32(np.full((1, K), -8, np.int8), np.full((1, K), -8, np.int8))
    assert worst[0, 0] == 64 * K
    # one-hot weight codes select activation codes
    sel = np.zeros((K, K), np.int8)
    sel[np.arange(K), np.arange(K)[::-1]] = 1
    cx2 = rng.integers(-8, 8, size=(5, K)).astype(np.int8)
    assert np.array_equal(o.gemm_i32(cx2, sel), cx2[:, ::-1].astype(np.int64))
    # summation order is irrelevant
    perm = rng.permutation(K)
    cw2 = rng.integers(-8, 8, size=(7, K)).astype(np.int8)
    assert np.array_equal(o.gemm_i32(cx2, cw2), o.gemm_i32(cx2[:, perm], cw2[:, perm]))


def test_gemm_c_matches_numpy_ragged():
    cx = wl.random_codes(1, 37, 320)
    cw = wl.random_codes(2, 53, 320)
    assert np.array_equal(o.gemm_i32_c(cx, cw), o.gemm_i32(cx, cw))


# ------------------------------------------------------- end-to-end closed form

def test_one_hot_token_closed_form():
    """X row = c * e_k with clip = 1: every |y_j| = c, so all codes are +-7, Delta_x = c/7,
    the dequantised activation is exact and Y = c * Delta_w[n] * sum_j H[k][j] cW[n][j]."""
    K, N, k, c = 64, 8, 37, 3.25
    H = o.sylvester(K)
    X = np.zeros((1, K)); X[0, k] = c
    act = o.fwht_quant_act(X, None, 1.0)
    assert np.array_equal(act["codes"][0], 7 * H[k])
    assert act["x_scale"][0] == pytest.approx(c / 7, rel=1e-15)
    rng = np.random.default_rng(0)
    cw = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    dw = rng.random(N) + 0.5
    Y = o.dequant_out(o.gemm_i32(act["codes"], cw), act["x_scale"], dw)
    want = np.array([c * dw[n] * sum(int(H[k, j]) * int(cw[n, j]) for j in range(K)) for n in range(N)])
    np.testing.assert_allclose(Y[0], want, rtol=1e-14)


def test_absmax_definition_and_chunking():
    X = wl.cfg1()["X"]
    a = o.calib_absmax(X, np.zeros(512))
    assert np.array_equal(a, np.abs(X.astype(np.float64)).max(axis=0))
    b = np.zeros(512)
    for lo in range(0, 16, 5):
        b = o.calib_absmax(X[lo:lo + 5], b)
    assert np.array_equal(a, b)
    assert np.array_equal(o.calib_absmax(X[:0], a), a)
    assert np.array_equal(o.calib_absmax(X, a + 1e6), a + 1e6)     # running maximum


def test_qualitative_ordering_on_outlier_config():
    """Smoke test only: on massive-outlier inputs, 4-bit error without transform >
    rotation only > smoothing then rotation (paper: sections "Outlier Mitigation
    Techniques" and "Conclusion")."""
    c = wl.cfg1()
    X, W = c["X"].astype(np.float64), c["W"].astype(np.float64)
    Y = X @ W
    a = o.calib_absmax(c["X"], np.zeros(512))

    def rel(Yq):
        return np.linalg.norm(Yq - Y) / np.linalg.norm(Y)

    cx, dx, _ = o.quant_sym_int4(X, 0.9)
    cw, dw, _ = o.quant_sym_int4(W.T, 1.0)
    plain = rel(o.dequant_out(o.gemm_i32(cx, cw), dx, dw))
    rot = rel(o.w4a4_linear(c["X"], c["W"], None)[0])
    smoothrot = rel(o.w4a4_linear(c["X"], c["W"], a, alpha=0.5)[0])
    assert plain > rot > smoothrot
    # activation range after the (orthonormally scaled) transform shrinks in the same order
    r_rot = np.abs(o.rotate(X)).max() / np.sqrt(512)
    r_sr = np.abs(o.fwht_quant_act(c["X"], 1 / o.smoothing_factors(a, W, 0.5), 0.9)["y"]).max() / np.sqrt(512)
    assert np.abs(X).max() > r_rot > r_sr
