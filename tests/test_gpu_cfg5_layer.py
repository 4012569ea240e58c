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
