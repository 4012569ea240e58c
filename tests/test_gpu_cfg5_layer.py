"""GPU parity at the shapes of a LLaMA-3.1-8B decoder layer (benchmark config 5): seven random-init linears,
16384 tokens.  q/k/v share one quantised input, gate/up another; the down-projection input is a gated product
with outlier channels.  Calibration is the batch itself.  The oracle computes sampled token rows and sampled
output channels one by one; sums over all outputs are checked through identities that hold at any size."""
import numpy as np
import pytest
import torch

from oracle import smoothrot_oracle as o
import workloads as wl
import f6_codec as fc
from parity import check_codes, check_output, check_scales

pytestmark = pytest.mark.gpu

M = 16384
ROWS = np.unique(np.r_[0:6, 5000:5006, 12287:12293, M - 6:M])
GROUPS = (("qkv", 4096, ("q", "k", "v")), ("o", 4096, ("o",)), ("gateup", 4096, ("gate", "up")), ("down", 14336, ("down",)))


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("group", GROUPS, ids=[g[0] for g in GROUPS])
def test_layer_group(gpu, group):
    tag, K, names = group
    print("case cfg5", tag, flush=True)
    if K == 4096:
        X = wl.cfg5_X(M, K, stream=2 + len(tag))
    else:
        X = wl.cfg3_X(M=M, K=K, seed=4)
    Xd = dev(X)
    # calibration on the batch itself, in chunks
    absmax = torch.zeros(K, dtype=torch.float32, device="cuda")
    for c in range(0, M, 4096):
        gpu.sr_calib_absmax(Xd[c:c + 4096], absmax)
    torch.cuda.synchronize()
    a = absmax.cpu().numpy()
    assert np.array_equal(a, np.abs(X.astype(np.float32)).max(axis=0))            # exact
    Xs = X[ROWS]
    for name in names:
        W = wl.cfg5_W(name)
        N = W.shape[1]
        Wq, ws, inv_s = gpu.sr_fold_smooth_rotate_quant(dev(W), absmax, 0.5, 1.0)
        torch.cuda.synchronize()
        # fold: sampled output channels against the oracle
        cols = np.unique(np.r_[0:8, N // 2:N // 2 + 8, N - 8:N])
        # (smoothing factors use the row maxima of the whole W, not of the sampled columns)
        s_full = o.smoothing_factors(a.astype(np.float64), W, 0.5)
        what = o.rotate(np.ascontiguousarray((s_full[:, None] * W[:, cols].astype(np.float64)).T)) / K
        c_ref, d_ref, t_ref = o.quant_sym_int4(what, 1.0)
        check_scales(ws.cpu().numpy()[cols], d_ref, name + " w_scale")
        cw_all = o.unpack_int4(Wq.cpu().numpy())
        check_codes(cw_all[cols], c_ref, t_ref, name + " weight codes")
        np.testing.assert_allclose(inv_s.cpu().numpy(), 1.0 / s_full, rtol=2e-6)
        # activations (inv_s differs per linear: each has its own weight maxima)
        Xq, xs = gpu.sr_fwht_quant_act(Xd, inv_s, 0.9)
        torch.cuda.synchronize()
        act = o.fwht_quant_act(Xs, inv_s.cpu().numpy().astype(np.float64), 0.9)
        check_scales(xs.cpu().numpy()[ROWS], act["x_scale"], name + " x_scale")
        cx_all = o.unpack_int4(Xq.cpu().numpy())
        check_codes(cx_all[ROWS], act["codes"], act["t"], name + " activation codes")
        # GEMM: INT32 accumulators on the GPU's own codes
        acc = gpu.sr_w4a4_gemm(Xq, None, Wq, None, gpu.SR_I32).cpu().numpy().astype(np.int64)
        assert np.array_equal(acc[ROWS], o.gemm_i32_c(cx_all[ROWS], cw_all))
        assert np.array_equal(acc.sum(axis=1), cx_all.astype(np.int64) @ cw_all.astype(np.int64).sum(axis=0))
        assert np.array_equal(acc.sum(axis=0), cw_all.astype(np.int64) @ cx_all.astype(np.int64).sum(axis=0))
        # dequantised output
        Y = gpu.sr_w4a4_gemm(Xq, xs, Wq, ws, gpu.SR_F16).cpu().numpy()
        want = o.dequant_out(acc[ROWS], xs.cpu().numpy()[ROWS], ws.cpu().numpy())
        check_output(Y[ROWS], want, name + " Y")
        assert np.isfinite(Y).all()
        # the same linear through the FP6-pipe path (the one the benchmark times).  Its quantiser rounds with the
        # hardware FP6 conversion, so its codes are held to the boundary rule on their own, and its accumulators
        # are checked on ITS codes.
        W6 = gpu.sr_pack_f6_tiles(Wq)
        X6, xs6 = gpu.sr_fwht_quant_act_f6(Xd, inv_s, 0.9)
        acc6 = gpu.sr_w4a4_gemm_f6(X6, None, W6, None, M, N, K, gpu.SR_I32).cpu().numpy().astype(np.int64)
        Y6 = gpu.sr_w4a4_gemm_f6(X6, xs6, W6, ws, M, N, K, gpu.SR_F16)
        torch.cuda.synchronize()
        assert np.array_equal(xs6.cpu().numpy(), xs.cpu().numpy())
        cx6_all = fc.f6_codes(fc.f6_tiles_unpack(X6.cpu().numpy(), M, K))
        check_codes(cx6_all[ROWS], act["codes"], act["t"], name + " activation codes (f6 path)")
        assert np.count_nonzero(cx6_all != cx_all) <= 1e-5 * cx_all.size
        assert np.array_equal(acc6[ROWS], o.gemm_i32_c(cx6_all[ROWS], cw_all))
        assert np.array_equal(acc6.sum(axis=1), cx6_all.astype(np.int64) @ cw_all.astype(np.int64).sum(axis=0))
        assert np.array_equal(acc6.sum(axis=0), cw_all.astype(np.int64) @ cx6_all.astype(np.int64).sum(axis=0))
        want6 = o.dequant_out(acc6[ROWS], xs.cpu().numpy()[ROWS], ws.cpu().numpy())
        check_output(Y6.cpu().numpy()[ROWS], want6, name + " Y (f6 path)")
        del cx6_all
        del acc, Y, cx_all, cw_all, acc6, Y6, X6, W6


def test_chained_layer_as_the_benchmark_runs_it(gpu):
    """The chain bench.py times for config 5 (paper, Fig. 2): [q|k|v] folded and multiplied as ONE weight (N = 6144),
    [gate|up] as one (N = 28672) with the down-projection's 1/s absorbed into W_up, the gate/up outputs read in
    place by the fused silu(gate) * up rotation + quantiser (K = 14336 = 28 * 512, no factors), then down.  Stage by
    stage on sampled token rows: every stage's oracle runs on the GPU's own output of the stage before.  Last, the
    chain's output is compared with the unquantised fp64 FFN on those rows: only a consistent absorption (1/s in
    W_up's columns, s in W_down's rows) leaves a 4-bit-sized error."""
    K, KD, NQ, NG = 4096, 14336, 6144, 28672
    Xa, Xf = wl.cfg5_X(M, K, stream=40), wl.cfg5_X(M, K, stream=42)
    W = {n: wl.cfg5_W(n) for n in ("q", "k", "v", "gate", "up", "down")}
    Xa_d, Xf_d = dev(Xa), dev(Xf)

    def absmax_of(Xd, cols):
        a = torch.zeros(cols, dtype=torch.float32, device="cuda")
        gpu.sr_calib_absmax(Xd, a)
        return a
    a_a, a_f = absmax_of(Xa_d, K), absmax_of(Xf_d, K)
    # calibration of the down-projection input on the fp16 layer (plain fp16 matmuls, as calibration runs on the
    # unquantised model)
    Wg_d, Wu_d = dev(W["gate"]), dev(W["up"])
    D = torch.empty((M, KD), dtype=torch.float16, device="cuda")
    for r in range(0, M, 4096):
        D[r:r + 4096] = (torch.nn.functional.silu((Xf_d[r:r + 4096] @ Wg_d).float()) * (Xf_d[r:r + 4096] @ Wu_d).float()).half()
    a_d = absmax_of(D, KD)
    del D
    Wq_d, ws_d, inv_d = gpu.sr_fold_smooth_rotate_quant(dev(W["down"]), a_d, 0.5, 1.0)
    W_up_abs = (Wu_d.float() * inv_d[None, :]).half()
    Wqkv = np.concatenate([W["q"], W["k"], W["v"]], axis=1)
    Wgu_d = torch.cat([Wg_d, W_up_abs], 1).contiguous()
    Wq_q, ws_q, inv_q = gpu.sr_fold_smooth_rotate_quant(dev(Wqkv), a_a, 0.5, 1.0)
    Wq_g, ws_g, inv_g = gpu.sr_fold_smooth_rotate_quant(Wgu_d, a_f, 0.5, 1.0)
    torch.cuda.synchronize()

    def fold_cols_ok(Wh, a, Wq, ws, inv_s, what):
        Kw, Nw = Wh.shape
        cols = np.unique(np.r_[0:6, Nw // 2 - 3:Nw // 2 + 3, Nw - 6:Nw])
        s_full = o.smoothing_factors(a.cpu().numpy().astype(np.float64), Wh, 0.5)
        what_t = o.rotate(np.ascontiguousarray((s_full[:, None] * Wh[:, cols].astype(np.float64)).T)) / Kw
        c_ref, d_ref, t_ref = o.quant_sym_int4(what_t, 1.0)
        check_scales(ws.cpu().numpy()[cols], d_ref, what + " w_scale")
        check_codes(o.unpack_int4(Wq.cpu().numpy()[cols]), c_ref, t_ref, what + " weight codes")
        np.testing.assert_allclose(inv_s.cpu().numpy(), 1.0 / s_full, rtol=2e-6)
    fold_cols_ok(Wqkv, a_a, Wq_q, ws_q, inv_q, "qkv")
    fold_cols_ok(Wgu_d.cpu().numpy(), a_f, Wq_g, ws_g, inv_g, "gate|up")
    fold_cols_ok(W["down"], a_d, Wq_d, ws_d, inv_d, "down")

    W6_q, W6_g, W6_d = (gpu.sr_pack_f6_tiles(w) for w in (Wq_q, Wq_g, Wq_d))
    cw_q, cw_g, cw_d = (o.unpack_int4(w.cpu().numpy()) for w in (Wq_q, Wq_g, Wq_d))

    def stage(Xd, Xh, inv_s, W6, cw, ws, N, what):
        """rotate + quantise (tiles, warming hint as in the benchmark) and multiply; sampled rows against the oracle."""
        X6, xs = gpu.sr_fwht_quant_act_f6_warm(Xd, inv_s, 0.9, W6)
        Y = gpu.sr_w4a4_gemm_f6(X6, xs, W6, ws, M, N, K, gpu.SR_F16)
        acc = gpu.sr_w4a4_gemm_f6(X6, None, W6, None, M, N, K, gpu.SR_I32)
        torch.cuda.synchronize()
        act = o.fwht_quant_act(Xh[ROWS], inv_s.cpu().numpy().astype(np.float64), 0.9)
        cx = fc.f6_codes(fc.f6_tiles_unpack(X6.cpu().numpy(), M, K))[ROWS]
        check_scales(xs.cpu().numpy()[ROWS], act["x_scale"], what + " x_scale")
        check_codes(cx, act["codes"], act["t"], what + " activation codes")
        want = o.gemm_i32_c(cx, cw)
        assert np.array_equal(acc[torch.from_numpy(ROWS).cuda()].cpu().numpy().astype(np.int64), want), what
        check_output(Y[torch.from_numpy(ROWS).cuda()].cpu().numpy(), o.dequant_out(want, xs.cpu().numpy()[ROWS], ws.cpu().numpy()), what + " Y")
        del acc
        return Y

    print("case cfg5 chain qkv", flush=True)
    stage(Xa_d, Xa, inv_q, W6_q, cw_q, ws_q, NQ, "qkv")
    print("case cfg5 chain gate|up", flush=True)
    GU = stage(Xf_d, Xf, inv_g, W6_g, cw_g, ws_g, NG, "gate|up")
    print("case cfg5 chain down", flush=True)
    X6d, xsd = gpu.sr_swiglu_fwht_quant_act_f6(GU[:, :KD], GU[:, KD:], None, 0.9)
    Yd = gpu.sr_w4a4_gemm_f6(X6d, xsd, W6_d, ws_d, M, K, KD, gpu.SR_F16)
    accd = gpu.sr_w4a4_gemm_f6(X6d, None, W6_d, None, M, K, KD, gpu.SR_I32)
    torch.cuda.synchronize()
    ridx = torch.from_numpy(ROWS).cuda()
    gu = GU[ridx].cpu().numpy()
    act = o.fwht_quant_swiglu(gu[:, :KD], gu[:, KD:], None, 0.9)
    cxd = fc.f6_codes(fc.f6_tiles_unpack(X6d.cpu().numpy(), M, KD))[ROWS]
    check_scales(xsd.cpu().numpy()[ROWS], act["x_scale"], "down x_scale")
    check_codes(cxd, act["codes"], act["t"], "down activation codes")
    want = o.gemm_i32_c(cxd, cw_d)
    assert np.array_equal(accd[ridx].cpu().numpy().astype(np.int64), want)
    Yh = Yd[ridx].cpu().numpy()
    check_output(Yh, o.dequant_out(want, xsd.cpu().numpy()[ROWS], ws_d.cpu().numpy()), "down Y")
    # against the unquantised FFN in fp64 on the sampled rows
    xf = Xf[ROWS].astype(np.float64)
    exact = (o.swiglu(xf @ W["gate"].astype(np.float64), xf @ W["up"].astype(np.float64))) @ W["down"].astype(np.float64)
    q_err = np.linalg.norm(Yh - exact) / np.linalg.norm(exact)
    print("  chained FFN: 4-bit rel err vs fp64 %.3f" % q_err, flush=True)
    assert q_err < 0.6
