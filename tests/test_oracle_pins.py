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


# ----------------------------------------------------------------- rows around the core path

def test_swiglu_closed_forms_and_library_sigmoid():
    from scipy.special import expit          # an independent sigmoid
    rng = np.random.default_rng(5)
    g = rng.standard_normal(4000) * 4
    u = rng.standard_normal(4000)
    y = o.swiglu(g, u)
    assert np.allclose(y, g * expit(g) * u, rtol=1e-14, atol=0)
    # silu(g) - silu(-g) = g (sigma(g) + sigma(-g) = 1), silu(0) = 0, silu(g) -> g for large g
    one = np.ones_like(g)
    assert np.allclose(o.swiglu(g, one) - o.swiglu(-g, one), g, rtol=0, atol=1e-14)
    assert o.swiglu(np.zeros(1), np.ones(1))[0] == 0.0
    assert abs(o.swiglu(np.array([40.0]), np.array([1.0]))[0] - 40.0) < 1e-12
    # the gate, not the up branch, goes through the non-linearity
    assert o.swiglu(np.array([-30.0]), np.array([5.0]))[0] > -1e-10
    assert o.swiglu(np.array([5.0]), np.array([-30.0]))[0] < -100


@pytest.mark.parametrize("nh,d", [(4, 8), (8, 4), (32, 16), (1, 64), (64, 1)])
def test_rotate_heads_is_the_kronecker_product(nh, d):
    rng = np.random.default_rng(nh * 100 + d)
    x = rng.integers(-9, 10, size=(5, nh * d)).astype(np.float64)
    Hh, Hd = o.sylvester(nh), o.sylvester(d)
    across = np.kron(Hh, np.eye(d, dtype=np.int64))
    within = np.kron(np.eye(nh, dtype=np.int64), Hd)
    assert np.array_equal(o.rotate_heads(x, nh, True), x @ across)
    assert np.array_equal(o.rotate_heads(x, nh, False), x @ within)
    # the two commute and compose to the full transform of order nh * d
    full = x @ o.sylvester(nh * d)
    assert np.array_equal(o.rotate_heads(o.rotate_heads(x, nh, True), nh, False), full)
    assert np.array_equal(o.rotate_heads(o.rotate_heads(x, nh, False), nh, True), full)


def test_rotate_heads_full_size_involution():
    rng = np.random.default_rng(8)
    x = rng.integers(-50, 50, size=(3, 4096)).astype(np.float64)
    for across, order in ((True, 32), (False, 128)):
        y = o.rotate_heads(o.rotate_heads(x, 32, across), 32, across)
        assert np.array_equal(y, order * x)
    # a single non-zero entry stays inside its head (within) / inside its lane of the head (across)
    e = np.zeros((1, 4096)); e[0, 5 * 128 + 17] = 1.0
    yw = o.rotate_heads(e, 32, False).reshape(32, 128)
    assert np.all(yw[5] != 0) and np.count_nonzero(yw) == 128
    ya = o.rotate_heads(e, 32, True).reshape(32, 128)
    assert np.all(ya[:, 17] != 0) and np.count_nonzero(ya) == 32


def test_fwht_quant_act_heads_uses_the_head_transform():
    X = wl.cfg1()["X"][:4].astype(np.float64)
    r = o.fwht_quant_act_heads(X, 8, True, None, 0.9)
    y = X @ np.kron(o.sylvester(8), np.eye(64))
    assert np.allclose(r["y"], y, rtol=0, atol=1e-9)
    c, d, _ = o.quant_sym_int4(y, 0.9)
    assert np.array_equal(r["codes"], c) and np.allclose(r["x_scale"], d, rtol=1e-15)


def test_clip_grid():
    g = o.clip_grid()
    assert len(g) == 21 and g[0] == 1.0 and abs(g[-1] - 0.5) < 1e-15
    assert np.allclose(np.diff(g), -0.025, atol=1e-15)


def test_weight_clip_search_closed_form_row():
    # v = [8, 1 x m]: for a ratio r in (7/12, 1] the ones get code 1 and the 8 is clamped to 7, so
    # err(r) = m (1 - 8r/7)^2 + 64 (1 - r)^2; at r = 1 the 8 is exact: err = m / 49.
    m = 99
    v = np.array([[8.0] + [1.0] * m])
    grid = o.clip_grid()
    ratio, errs, codes, delta, _ = o.weight_clip_search(v, grid)
    for i, r in enumerate(grid):
        if r > 0.6:
            want = m * (1 - 8 * r / 7) ** 2 + 64 * (1 - r) ** 2
            assert abs(errs[0, i] - want) < 1e-9, (r, errs[0, i], want)
    # minimiser of the closed form over the grid
    cand = [(m * (1 - 8 * r / 7) ** 2 + 64 * (1 - r) ** 2, -r) for r in grid if r > 0.6]
    best_r = -min(cand)[1]
    assert abs(ratio[0] - best_r) < 1e-12 and best_r < 1.0
    assert abs(delta[0] - best_r * 8 / 7) < 1e-12
    assert codes[0, 0] == 7 and np.all(codes[0, 1:] == 1)


def test_weight_clip_search_brute_force_and_ties():
    rng = np.random.default_rng(21)
    v = rng.standard_normal((6, 24)) * rng.choice([0.1, 1.0, 5.0], size=(6, 24))
    grid = o.clip_grid()
    ratio, errs, codes, delta, _ = o.weight_clip_search(v, grid)
    for row in range(6):
        best, best_err = None, None
        amax = max(abs(float(x)) for x in v[row])
        for r in grid:                                  # descending: '<' keeps the larger ratio on ties
            d = float(r) * amax / 7.0
            e = 0.0
            for x in v[row]:
                c = min(7, max(-8, round(float(x) / d)))      # Python's round = half to even
                e += (float(x) - c * d) ** 2
            if best_err is None or e < best_err:
                best, best_err = float(r), e
        assert abs(ratio[row] - best) < 1e-12
        assert abs(errs[row].min() - best_err) <= 1e-12 * max(best_err, 1e-30)
    # a row already on the 15-level grid has zero error at ratio 1: the tie rule keeps 1.0
    exact = np.array([[7.0, -7.0, 3.0, 0.0, 1.0, -2.0, 5.0, -6.0]])
    r2, e2, c2, d2, _ = o.weight_clip_search(exact, grid)
    assert r2[0] == 1.0 and e2[0, 0] == 0.0 and d2[0] == 1.0
    assert np.array_equal(c2[0], exact[0].astype(np.int8))
    # never worse than plain RTN, zero row -> Delta 1
    assert np.all(errs.min(axis=1) <= errs[:, 0])
    assert o.weight_clip_search(np.zeros((1, 8)), grid)[3][0] == 1.0


def test_fold_clip_search_consistent_with_plain_fold():
    c1 = wl.cfg1()
    X, W = c1["X"], c1["W"]
    a = o.calib_absmax(X, np.zeros(512))
    f1 = o.fold_smooth_rotate_quant(W[:, :32], a, 0.5, 1.0)
    f = o.fold_clip_search(W[:, :32], a, 0.5, np.array([1.0]))      # one-point grid = plain RTN
    assert np.array_equal(f["codes"], f1["codes"]) and np.allclose(f["w_scale"], f1["w_scale"], rtol=1e-15)
    g = o.fold_clip_search(W[:, :32], a, 0.5, o.clip_grid())
    what = f1["W_hat"].T
    e_plain = np.sum((what - o.dequant(f1["codes"], f1["w_scale"])) ** 2, axis=1)
    e_srch = np.sum((what - o.dequant(g["codes"], g["w_scale"])) ** 2, axis=1)
    assert np.all(e_srch <= e_plain + 1e-18) and np.any(e_srch < e_plain)


def test_asym_quantiser_hand_worked_group():
    xs, want_c, want_q, clip = [], [], [], None
    for line in open(os.path.join(GOLDEN, "hand_asym_group.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        p = line.split()
        if p[0] == "clip":
            clip = float(p[1])
            continue
        xs.append(float(p[0])); want_c.append(int(p[1])); want_q.append(float(p[2]))
    v = np.array([xs])
    codes, delta, z, _, _ = o.quant_asym_int4_groups(v, group=8, clip=clip)
    assert delta[0, 0] == 0.25 and z[0, 0] == 5
    assert codes[0].tolist() == want_c
    assert o.dequant_asym(codes, delta, z, group=8)[0].tolist() == want_q


def test_asym_quantiser_properties():
    rng = np.random.default_rng(33)
    v = rng.standard_normal((16, 512)) * 3 + rng.standard_normal((16, 1))
    codes, delta, z, _, _ = o.quant_asym_int4_groups(v, 128, 1.0)
    assert codes.min() == 0 and codes.max() == 15
    g = v.reshape(16, 4, 128)
    cg = codes.reshape(16, 4, 128)
    # without clipping the minimum gets code 0, the maximum code 15, and no value moves by more than Delta / 2
    assert np.all(np.take_along_axis(cg, g.argmin(axis=2)[..., None], 2) == 0)
    assert np.all(np.take_along_axis(cg, g.argmax(axis=2)[..., None], 2) == 15)
    err = np.abs(o.dequant_asym(codes, delta, z) - v).reshape(16, 4, 128)
    assert np.all(err <= delta[:, :, None] / 2 * (1 + 1e-12))
    assert np.allclose(delta, (g.max(axis=2) - g.min(axis=2)) / 15, rtol=1e-15)
    # groups are independent: permuting groups permutes results
    perm = v.reshape(16, 4, 128)[:, ::-1, :].reshape(16, 512)
    c2, d2, z2, _, _ = o.quant_asym_int4_groups(perm, 128, 1.0)
    assert np.array_equal(c2.reshape(16, 4, 128)[:, ::-1], cg) and np.array_equal(d2[:, ::-1], delta)
    # power-of-two scaling leaves the codes alone; shifting by k * Delta moves only the zero-point
    c3, d3, z3, _, _ = o.quant_asym_int4_groups(v * 8.0, 128, 1.0)
    assert np.array_equal(c3, codes) and np.array_equal(z3, z) and np.allclose(d3, 8 * delta, rtol=1e-15)
    one = np.array([[-1.0, 0.0, 0.45, 2.0]])                # Delta = 0.2, no ties
    c4, d4, z4, _, _ = o.quant_asym_int4_groups(one, 4, 1.0)
    c5, d5, z5, _, _ = o.quant_asym_int4_groups(one + 3 * d4[0, 0], 4, 1.0)
    assert np.array_equal(c4, c5) and z5[0, 0] == z4[0, 0] - 3
    # all-positive group: zero-point is negative; constant group: Delta = 1
    c6, d6, z6, _, _ = o.quant_asym_int4_groups(np.array([[10.0, 25.0, 11.0, 12.0]]), 4, 1.0)
    assert d6[0, 0] == 1.0 and z6[0, 0] == -10 and c6[0].tolist() == [0, 15, 1, 2]
    c7, d7, z7, _, _ = o.quant_asym_int4_groups(np.full((1, 4), 3.0), 4, 0.95)
    assert d7[0, 0] == 1.0
    assert np.allclose(o.dequant_asym(c7, d7, z7, 4), 3.0)
    # clipping: range shrinks at both ends, clipped values saturate at 0 / 15
    c8, d8, z8, _, _ = o.quant_asym_int4_groups(v, 128, 0.95)
    assert np.allclose(d8, 0.95 * delta, rtol=1e-15)
    assert np.all(np.take_along_axis(c8.reshape(16, 4, 128), g.argmax(axis=2)[..., None], 2) == 15)
    assert np.all(np.take_along_axis(c8.reshape(16, 4, 128), g.argmin(axis=2)[..., None], 2) == 0)


def test_asym_quantiser_brute_force():
    rng = np.random.default_rng(34)
    v = rng.standard_normal((3, 16)) + 0.3
    codes, delta, z, _, _ = o.quant_asym_int4_groups(v, 8, 0.95)
    for r in range(3):
        for gi in range(2):
            xs = [float(x) for x in v[r, gi * 8:(gi + 1) * 8]]
            hi, lo = 0.95 * max(xs), 0.95 * min(xs)
            d = (hi - lo) / 15.0
            zz = -round(lo / d)
            assert abs(delta[r, gi] - d) < 1e-15 and z[r, gi] == zz
            for j, x in enumerate(xs):
                assert codes[r, gi * 8 + j] == min(15, max(0, round(x / d) + zz))


def test_pack_uint4_all_bytes():
    b = np.arange(256, dtype=np.uint8)
    codes = np.stack([b & 0xF, b >> 4], axis=1).reshape(1, 512)
    assert np.array_equal(o.pack_uint4(codes)[0], b)


# ----------------------------------------------------------------- INT4 codes as 6-bit floats

def test_e2m3_decoder_against_the_format_definition():
    """All 64 patterns against values written out from the format's definition: sign, exponent bias 1,
    three mantissa bits, subnormals at e = 0, no infinities or NaNs; largest magnitude 7.5."""
    pos = [m / 8 for m in range(8)] + [1 + m / 8 for m in range(8)] + [2 + m / 4 for m in range(8)] + \
          [4 + m / 2 for m in range(8)]
    want = np.array(pos + [-v for v in pos])
    got = o.e2m3_value(np.arange(64))
    assert np.array_equal(got, want) and got.max() == 7.5 and np.all(np.isfinite(got))
    assert np.array_equal(np.signbit(got), np.arange(64) >= 32)          # pattern 32 is -0


def test_every_int4_code_is_an_exact_e2m3_value():
    """code c is the pattern (c < 0 ? 32 : 0) | |c|, of value c / 8: sixteen distinct patterns, all exact."""
    codes = np.arange(-8, 8)
    f = np.where(codes < 0, 32, 0) | np.abs(codes)
    assert np.array_equal(8.0 * o.e2m3_value(f), codes.astype(np.float64))
    assert f.max() < 64 and len(set(f.tolist())) == 16


def test_fp32_accumulation_of_code_products_is_exact():
    """The argument behind running the integer GEMM on a float pipe: products of two values c/8 are
    integers / 64 and every partial sum stays below 2^24 / 64, so fp32 additions in ANY order are exact.
    Checked at the worst case (all codes -8, K = 131008) and on random codes with shuffled orders."""
    K = 131008
    worst = np.full(K, 1.0, np.float32)                                   # (-8/8) * (-8/8)
    assert float(np.cumsum(worst, dtype=np.float32)[-1]) * 64 == 64 * K
    assert 64 * K < 2 ** 24
    rng = np.random.default_rng(5)
    a, b = rng.integers(-8, 8, 14336), rng.integers(-8, 8, 14336)
    pattern = lambda c: np.where(c < 0, 32, 0) | np.abs(c)          # sign bit, then |c| in the low bits
    prod = (o.e2m3_value(pattern(a)) * o.e2m3_value(pattern(b))).astype(np.float32)
    assert np.array_equal(prod.astype(np.float64) * 64, (a * b).astype(np.float64))
    want = int(np.dot(a, b))
    for seed in range(4):
        perm = np.random.default_rng(seed).permutation(prod.size)
        acc = np.float32(0)
        for chunk in np.split(prod[perm], 112):                           # blocked like a matrix instruction
            acc = np.float32(acc + chunk.sum(dtype=np.float32))
        assert float(acc) * 64 == want
