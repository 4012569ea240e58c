"""GPU parity of the rows around the core path: gated-FFN prologue, head-wise Hadamard,
weight clipping-ratio search, asymmetric KV-cache quantiser -- each against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import smoothrot_oracle as o
import workloads as wl
from parity import CODE_TOL_REL, check_codes, check_scales

pytestmark = pytest.mark.gpu

# The search compares sums of squared errors.  The GPU forms each term in fp32 and adds in fp64, the oracle
# works in fp64 throughout; a ratio whose oracle error is within this relative margin of the oracle's minimum
# is an equally valid winner (several results are correct; what is unique is checked exactly).
SEARCH_ERR_RTOL = 1e-5


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


# ------------------------------------------------------------------ gated FFN prologue

def compare_swiglu(sr, G, U, inv_s, clip, what):
    print("case swiglu", what, G.shape, flush=True)
    Xq, xs = sr.sr_swiglu_fwht_quant_act(dev(G), dev(U), dev(inv_s), clip)
    torch.cuda.synchronize()
    ref = o.fwht_quant_swiglu(G, U, inv_s, clip)
    check_scales(xs.cpu().numpy(), ref["x_scale"], what + " x_scale")
    return check_codes(o.unpack_int4(Xq.cpu().numpy()), ref["codes"], ref["t"], what + " codes")


@pytest.mark.parametrize("K", [64, 512, 4096, 896, 14336])
def test_swiglu_orders(gpu, K):
    G, U = wl.gate_up(11, 6, K, 3, 800.0)
    rng = np.random.default_rng(K)
    inv_s = np.exp(rng.standard_normal(K) * 0.5).astype(np.float32)
    compare_swiglu(gpu, G, U, inv_s, 0.9, "K=%d" % K)
    compare_swiglu(gpu, G, U, None, 1.0, "K=%d no inv_s" % K)


@pytest.mark.parametrize("K,M", [(14336, 300), (14336, 100), (14336, 3), (7168, 600), (7168, 4), (8192, 5), (16384, 3), (28672, 2), (2048, 9), (1024, 3)])
def test_swiglu_thread_counts(gpu, K, M):
    """The gated prologue on the plain row kernel, with every number of threads per row its launcher picks
    (K = 14336 above 256 rows and K = 7168 above 512 rows: 256 threads; fewer rows, and the longer rows: 512 or 1024)."""
    G, U = wl.gate_up(21 + M, M, K, 3, 500.0)
    inv_s = np.exp(np.random.default_rng(K + M).standard_normal(K) * 0.5).astype(np.float32)
    compare_swiglu(gpu, G, U, inv_s, 0.9, "K=%d M=%d" % (K, M))


def test_swiglu_extreme_gates(gpu):
    K = 512
    G = np.zeros((4, K), np.float16)
    U = np.ones((4, K), np.float16)
    G[0, :] = np.linspace(-20, 20, K)
    G[1, :] = -65504.0            # exp(-g) overflows: silu -> -0
    G[1, 5] = 3.0
    G[2, :] = 65504.0
    U[2, :] = np.linspace(-1, 1, K) * 1e-3
    G[3, :] = 0.0                 # an all-zero row: Delta = 1, codes 0
    compare_swiglu(gpu, G, U, None, 0.9, "extreme")


def test_swiglu_cfg3_rows(gpu):
    G, U = wl.gate_up(2, 64, 14336, 3, 800.0)
    a = o.calib_absmax(o.swiglu(G, U), np.zeros(14336))
    inv_s = (1.0 / o.smoothing_factors(a, wl.cfg3_W()[:, :64], 0.5)).astype(np.float32)
    flips = compare_swiglu(gpu, G, U, inv_s, 0.9, "cfg3 gate/up")
    assert flips <= 64


def test_swiglu_padded_rows(gpu):
    G, U = wl.gate_up(12, 5, 1024, 2, 100.0)
    gb = torch.zeros((5, 1024 + 64), dtype=torch.float16, device="cuda")
    ub = torch.zeros((5, 1024 + 8), dtype=torch.float16, device="cuda")
    gb[:, :1024] = dev(G)
    ub[:, :1024] = dev(U)
    Xq, xs = gpu.sr_swiglu_fwht_quant_act(gb[:, :1024], ub[:, :1024], None, 0.9)
    torch.cuda.synchronize()
    ref = o.fwht_quant_swiglu(G, U, None, 0.9)
    check_scales(xs.cpu().numpy(), ref["x_scale"])
    check_codes(o.unpack_int4(Xq.cpu().numpy()), ref["codes"], ref["t"])


# ------------------------------------------------------------------ head-wise Hadamard

@pytest.mark.parametrize("K,nh", [(64, 4), (512, 8), (4096, 32), (4096, 1), (4096, 4096), (1024, 2), (32768, 64)])
@pytest.mark.parametrize("across", [True, False])
def test_heads(gpu, K, nh, across):
    rng = np.random.default_rng(K + nh)
    X = wl.to_f16_sat(rng.standard_normal((5, K)).astype(np.float32) * (1 + 300 * (rng.random(K) < 0.002)))
    inv_s = np.exp(rng.standard_normal(K) * 0.5).astype(np.float32)
    print("case heads", K, nh, across, flush=True)
    Xq, xs = gpu.sr_fwht_quant_act_heads(dev(X), nh, across, dev(inv_s), 0.9)
    torch.cuda.synchronize()
    ref = o.fwht_quant_act_heads(X, nh, across, inv_s, 0.9)
    check_scales(xs.cpu().numpy(), ref["x_scale"])
    check_codes(o.unpack_int4(Xq.cpu().numpy()), ref["codes"], ref["t"])


@pytest.mark.parametrize("nh", [32, 2, 512, 1])
@pytest.mark.parametrize("across", [True, False])
@pytest.mark.parametrize("smooth", [True, False])
def test_heads_many_rows_of_4096(gpu, nh, across, smooth):
    """More than 1024 rows of 4096: the head-wise transform runs in the wave-per-row kernel (a ragged row count,
    heads that split the register bits of both of its phases)."""
    M, K = 1029, 4096
    rng = np.random.default_rng(nh + 7 * across)
    X = wl.to_f16_sat(rng.standard_normal((M, K)).astype(np.float32) * (1 + 300 * (rng.random(K) < 0.002)))
    inv_s = np.exp(rng.standard_normal(K) * 0.5).astype(np.float32) if smooth else None
    Xq, xs = gpu.sr_fwht_quant_act_heads(dev(X), nh, across, None if inv_s is None else dev(inv_s), 0.9)
    torch.cuda.synchronize()
    ref = o.fwht_quant_act_heads(X, nh, across, inv_s, 0.9)
    check_scales(xs.cpu().numpy(), ref["x_scale"])
    check_codes(o.unpack_int4(Xq.cpu().numpy()), ref["codes"], ref["t"])


def test_heads_unit_vectors(gpu):
    """X = 3 e_k, clip 1: codes are 7 * (row k of the head-wise matrix), zero outside its support."""
    K, nh = 4096, 32
    ks = [0, 1, 127, 128, 129, 2047, 2048, 4095, 5 * 128 + 17]
    X = np.zeros((len(ks), K), np.float16)
    X[np.arange(len(ks)), ks] = 3.0
    for across in (True, False):
        Xq, xs = gpu.sr_fwht_quant_act_heads(dev(X), nh, across, None, 1.0)
        torch.cuda.synchronize()
        H = o.rotate_heads(np.eye(K)[ks], nh, across)
        assert np.array_equal(o.unpack_int4(Xq.cpu().numpy()).astype(np.int64), (7 * H).astype(np.int64))
        np.testing.assert_allclose(xs.cpu().numpy(), 3.0 / 7.0, rtol=1e-6)


def test_heads_cfg2_rows_and_fold_identity(gpu):
    """Across-heads transform on both sides: (X T)(T W / n_heads) = X W, checked through the quantised
    pipeline against the oracle's pipeline, stage by stage."""
    K, nh, N = 4096, 32, 64
    X = wl.cfg2_X(M=32)
    W = wl.cfg2_W(4096)[:, :N].copy()
    a = o.calib_absmax(X, np.zeros(K))
    Wq, ws, inv_s, ratio = gpu.sr_fold_smooth_rotate_quant_ex(dev(W), dev(a.astype(np.float32)), 0.5, nh, True, 1, 1.0)
    torch.cuda.synchronize()
    s = o.smoothing_factors(a, W, 0.5)
    what_t = o.rotate_heads(np.ascontiguousarray((s[:, None] * W.astype(np.float64)).T), nh, True) / nh
    c_ref, d_ref, t_ref = o.quant_sym_int4(what_t, 1.0)
    check_scales(ws.cpu().numpy(), d_ref, "heads fold scale")
    check_codes(o.unpack_int4(Wq.cpu().numpy()), c_ref, t_ref, "heads fold codes")
    assert np.all(ratio.cpu().numpy() == 1.0)
    Xq, xs = gpu.sr_fwht_quant_act_heads(dev(X), nh, True, inv_s, 0.9)
    torch.cuda.synchronize()
    ref = o.fwht_quant_act_heads(X, nh, True, inv_s.cpu().numpy().astype(np.float64), 0.9)
    check_scales(xs.cpu().numpy(), ref["x_scale"])
    check_codes(o.unpack_int4(Xq.cpu().numpy()), ref["codes"], ref["t"])
    # the transformed layer still computes X W (before quantisation): Eq. (2) with the head-wise matrix
    y = ref["y"] @ what_t.T
    exact = X.astype(np.float64) @ W.astype(np.float64)
    # (inv_s is the library's fp32 rounding of 1 / s, hence 1e-6 and not fp64 accuracy)
    assert np.abs(y - exact).max() <= 1e-6 * np.abs(exact).max()


@pytest.mark.parametrize("nh", [0, 32])
def test_fold_ex_reports_the_fixed_ratio_for_many_output_channels(gpu, nh):
    """More than 1024 output channels of K = 4096 without a search run in the wave-per-row kernel, which does not
    report a ratio itself: w_ratio must still come back as the fixed ratio for every channel (a buffer pre-filled
    with another value shows a missing write); codes and scales against the oracle as everywhere."""
    K, N = 4096, 1040
    W = wl.cfg2_W(4096)[:, :N].copy()
    a = np.abs(np.random.default_rng(3).standard_normal(K)).astype(np.float32) * 4 + 0.05
    ratio = torch.full((N,), -7.0, dtype=torch.float32, device="cuda")
    Wq, ws, inv_s, ratio = gpu.sr_fold_smooth_rotate_quant_ex(dev(W), dev(a), 0.5, nh, True, 1, 0.95, w_ratio=ratio)
    torch.cuda.synchronize()
    assert np.all(ratio.cpu().numpy() == np.float32(0.95))
    s = o.smoothing_factors(a.astype(np.float64), W, 0.5)
    sw_t = np.ascontiguousarray((s[:, None] * W.astype(np.float64)).T)
    what_t = o.rotate(sw_t) / K if nh == 0 else o.rotate_heads(sw_t, nh, True) / nh
    c_ref, d_ref, t_ref = o.quant_sym_int4(what_t, 0.95)
    check_scales(ws.cpu().numpy(), d_ref, "fold scale")
    check_codes(o.unpack_int4(Wq.cpu().numpy()), c_ref, t_ref, "fold codes")


# ------------------------------------------------------------------ weight clipping-ratio search

def compare_search(sr, W, a, alpha, steps, lo, what, n_heads=0, across=False):
    print("case clip search", what, W.shape, steps, lo, flush=True)
    Wq, ws, inv_s, ratio = sr.sr_fold_smooth_rotate_quant_ex(dev(W), None if a is None else dev(a.astype(np.float32)),
                                                             alpha, n_heads, across, steps, lo)
    torch.cuda.synchronize()
    grid = o.clip_grid(steps, lo) if steps > 1 else np.array([lo])
    ref = o.fold_clip_search(W, a, alpha, grid)
    ratio = ratio.cpu().numpy().astype(np.float64)
    idx = np.abs(ratio[:, None] - grid[None, :]).argmin(axis=1)
    np.testing.assert_allclose(ratio, grid[idx], rtol=1e-6)          # the ratio is one of the candidates
    errs = ref["errs"]
    chosen = errs[np.arange(len(idx)), idx]
    best = errs.min(axis=1)
    assert np.all(chosen <= best * (1 + SEARCH_ERR_RTOL) + 1e-300), "a chosen ratio is not a minimiser"
    same = idx == errs.argmin(axis=1)
    # quantise with the ratio the GPU chose (oracle arithmetic) and compare codes / scales exactly as elsewhere
    v = ref["W_hat_t"]
    absmax = np.abs(v).max(axis=1)
    delta = np.where(absmax == 0, 1.0, grid[idx] * absmax / 7.0)
    t = v / delta[:, None]
    codes = np.clip(np.rint(t), -8, 7).astype(np.int8)
    check_scales(ws.cpu().numpy(), delta, what + " w_scale")
    check_codes(o.unpack_int4(Wq.cpu().numpy()), codes, t, what + " codes")
    np.testing.assert_allclose(inv_s.cpu().numpy(), ref["inv_s"], rtol=2e-6)
    return float(same.mean()), idx


def test_clip_search_cfg1(gpu):
    c = wl.cfg1()
    a = o.calib_absmax(c["X"], np.zeros(512))
    agree, idx = compare_search(gpu, c["W"], a, 0.5, 21, 0.5, "cfg1")
    assert agree >= 0.98 and idx.max() > 0            # the search does move some channels off plain RTN
    compare_search(gpu, c["W"], None, 0.5, 21, 0.5, "cfg1 rotation only")
    compare_search(gpu, c["W"], a, 0.5, 1, 0.85, "cfg1 one fixed ratio")
    compare_search(gpu, c["W"], a, 0.5, 32, 0.25, "cfg1 32 steps")
    compare_search(gpu, c["W"], a, 0.5, 2, 0.9, "cfg1 2 steps")


@pytest.mark.parametrize("K,N", [(64, 16), (896, 32), (4096, 128), (14336, 32), (32768, 16)])
def test_clip_search_shapes(gpu, K, N):
    rng = np.random.default_rng(K + N)
    W = wl.to_f16_sat(rng.standard_normal((K, N)).astype(np.float32) * 0.02)
    W[:, 3] = 0                                        # a dead output channel: ratio = first candidate, Delta 1
    W[:: max(K // 50, 1), 5] *= 30                     # a heavy-tailed channel: wants a ratio well below 1
    a = (np.abs(rng.standard_normal(K)) * (1 + 800 * (rng.random(K) < 0.003))).astype(np.float32)
    agree, idx = compare_search(gpu, W, a, 0.5, 21, 0.5, "K=%d N=%d" % (K, N))
    assert idx[3] == 0


def test_clip_search_with_heads(gpu):
    rng = np.random.default_rng(77)
    W = wl.to_f16_sat(rng.standard_normal((1024, 48)).astype(np.float32) * 0.02)
    print("case clip search + heads", flush=True)
    Wq, ws, inv_s, ratio = gpu.sr_fold_smooth_rotate_quant_ex(dev(W), None, 0.5, 8, False, 21, 0.5)
    torch.cuda.synchronize()
    grid = o.clip_grid()
    v = o.rotate_heads(np.ascontiguousarray(W.astype(np.float64).T), 8, False) / 128.0
    r_ref, errs, _, _, _ = o.weight_clip_search(v, grid)
    idx = np.abs(ratio.cpu().numpy().astype(np.float64)[:, None] - grid[None, :]).argmin(axis=1)
    assert np.all(errs[np.arange(48), idx] <= errs.min(axis=1) * (1 + SEARCH_ERR_RTOL))
    delta = grid[idx] * np.abs(v).max(axis=1) / 7.0
    t = v / delta[:, None]
    check_scales(ws.cpu().numpy(), delta)
    check_codes(o.unpack_int4(Wq.cpu().numpy()), np.clip(np.rint(t), -8, 7).astype(np.int8), t)


# ------------------------------------------------------------------ KV-cache quantiser

def compare_kv(sr, X, group, clip, what, ldx=None):
    rows, D = X.shape
    print("case kv", what, X.shape, group, clip, flush=True)
    if ldx is None:
        Xd = dev(X)
    else:
        buf = torch.zeros((rows, ldx), dtype=torch.float16, device="cuda")
        buf[:, :D] = dev(X)
        Xd = buf[:, :D]
    Q, sc, ze = sr.sr_kv_quant_asym(Xd, group, clip)
    torch.cuda.synchronize()
    Q, sc, ze = Q.cpu().numpy(), sc.cpu().numpy().astype(np.float64), ze.cpu().numpy().astype(np.float64)
    codes, delta, z, u, zt = o.quant_asym_int4_groups(X, group, clip)
    np.testing.assert_allclose(sc, delta, rtol=1e-6, err_msg=what + " scale")
    assert np.all(ze == np.rint(ze))
    # zero-point: an integer decided in floating point -- may differ by one only where lo / Delta sits on a tie
    ng = D // group
    full = np.abs(u).reshape(rows, ng, group).max(axis=2)               # group full scale in code units
    dz = ze - z
    if np.any(dz != 0):
        assert np.all(np.abs(dz) <= 1)
        dist = np.abs(zt - (np.floor(zt) + 0.5))
        assert np.all(dist[dz != 0] <= CODE_TOL_REL * np.maximum(full, np.abs(zt))[dz != 0]), what + " zero-point"
    # codes, given the GPU's own zero-point
    gq = np.empty((rows, D), np.int16)
    gq[:, 0::2] = Q & 0xF
    gq[:, 1::2] = Q >> 4
    want = np.clip(np.rint(u).reshape(rows, ng, group) + ze[:, :, None], 0, 15).astype(np.int16).reshape(rows, D)
    diff = gq != want
    n = int(diff.sum())
    if n:
        r, c = np.nonzero(diff)
        assert np.all(np.abs(gq[r, c] - want[r, c]) == 1), what + ": codes differ by more than one"
        tt = u[r, c]
        dist = np.abs(tt - (np.floor(tt) + 0.5))
        tol = CODE_TOL_REL * np.maximum(full, np.abs(zt))[r, c // group]
        assert np.all(dist <= tol), "%s: %d mismatches away from a rounding boundary (worst %.3g)" % (what, n, dist.max())
    return n


def test_kv_paper_setting(gpu):
    X = wl.kv_acts(5, 257, 1024)                       # 8 KV heads of 128, a ragged row count
    flips = compare_kv(gpu, X, 128, 0.95, "kv 257 x 1024")
    assert flips <= 8
    compare_kv(gpu, X, 128, 1.0, "kv no clipping")


@pytest.mark.parametrize("group", [32, 64, 128, 256, 512])
def test_kv_group_sizes(gpu, group):
    X = wl.kv_acts(6, 33, 1024)
    compare_kv(gpu, X, group, 0.95, "group %d" % group)


def test_kv_edge_cases(gpu):
    X = wl.kv_acts(7, 4, 256).astype(np.float32)
    X[0, :128] = 3.0                                   # constant group: Delta = 1
    X[1, :128] = np.abs(X[1, :128]) + 10.0             # all-positive group: negative zero-point
    X[2, :128] = -np.abs(X[2, :128]) - 10.0            # all-negative group
    X[3, :] = 0.0
    X = X.astype(np.float16)
    compare_kv(gpu, X, 128, 0.95, "edge")
    compare_kv(gpu, X[:1], 128, 0.95, "single row")
    compare_kv(gpu, wl.kv_acts(8, 9, 128), 128, 0.95, "padded rows", ldx=136)
    Q, sc, ze = gpu.sr_kv_quant_asym(torch.empty((0, 128), dtype=torch.float16, device="cuda"))
    assert Q.shape[0] == 0


def test_kv_full_size_sampled(gpu):
    """32768 tokens x 1024 (8 KV heads x 128): every group's scale and zero-point, codes on sampled rows."""
    X = wl.kv_acts(9, 32768, 1024)
    Xd = dev(X)
    Q, sc, ze = gpu.sr_kv_quant_asym(Xd, 128, 0.95)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([np.arange(0, 32768, 997), [32767]]))
    codes, delta, z, u, zt = o.quant_asym_int4_groups(X[rows], 128, 0.95)
    np.testing.assert_allclose(sc.cpu().numpy()[rows], delta, rtol=1e-6)
    zg = ze.cpu().numpy()[rows]
    assert np.mean(zg == z) > 0.999 and np.all(np.abs(zg - z) <= 1)
    Qh = Q.cpu().numpy()[rows]
    gq = np.empty(codes.shape, np.int16)
    gq[:, 0::2] = Qh & 0xF
    gq[:, 1::2] = Qh >> 4
    ok = (zg == z).repeat(128, axis=1)
    assert np.mean(gq[ok] == codes[ok]) > 0.9999 and np.all(np.abs(gq[ok] - codes[ok].astype(np.int16)) <= 1)
    # property at full size: the dequantised value is within Delta/2 of the clipped input, every group
    g = X.astype(np.float32).reshape(32768, 8, 128)
    scn, zen = sc.cpu().numpy(), ze.cpu().numpy()
    Qa = Q.cpu().numpy()
    ca = np.empty((32768, 1024), np.float32)
    ca[:, 0::2] = Qa & 0xF
    ca[:, 1::2] = Qa >> 4
    deq = (ca.reshape(32768, 8, 128) - zen[:, :, None]) * scn[:, :, None]
    lo = 0.95 * g.min(axis=2, keepdims=True)
    hi = 0.95 * g.max(axis=2, keepdims=True)
    d3 = scn[:, :, None]
    inside = (g >= lo) & (g <= hi)
    assert np.all(np.abs(deq - g)[inside] <= (0.5001 * d3 + 1e-6).repeat(128, axis=2)[inside])
    assert np.all(deq >= lo - 0.5001 * d3 - 1e-6) and np.all(deq <= hi + 0.5001 * d3 + 1e-6)
