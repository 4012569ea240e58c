"""GPU parity of the whole layer (calibrate -> fold -> rotate+quantise -> GEMM), stage by stage.

Each stage is compared with the oracle run on the GPU's own output of the previous stage (already
checked against its tolerance), so a tolerated boundary flip upstream does not leak into the
comparison downstream: the last stage is compared with identical codes and scales on both sides."""
import numpy as np
import pytest
import torch

from oracle import smoothrot_oracle as o
import workloads as wl
from parity import check_codes, check_output, check_scales

pytestmark = pytest.mark.gpu


def run_layer(sr, X, W, calib, alpha=0.5, clip=0.9, w_clip=1.0, what=""):
    print("case", what, X.shape, W.shape, flush=True)
    K, N = W.shape
    a_d = torch.zeros(K, dtype=torch.float32, device="cuda")
    a_ref = np.zeros(K)
    for c in calib:
        sr.sr_calib_absmax(torch.from_numpy(c).cuda(), a_d)
        a_ref = o.calib_absmax(c, a_ref)
    assert np.array_equal(a_d.cpu().numpy().astype(np.float64), a_ref)

    Wq, ws, inv_s = sr.sr_fold_smooth_rotate_quant(torch.from_numpy(W).cuda(), a_d, alpha, w_clip)
    f = o.fold_smooth_rotate_quant(W, a_ref, alpha, w_clip)
    check_scales(inv_s.cpu().numpy(), f["inv_s"]); check_scales(ws.cpu().numpy(), f["w_scale"])
    cw_gpu = o.unpack_int4(Wq.cpu().numpy())
    wflips = check_codes(cw_gpu, f["codes"], f["t"], what + " W codes")

    Xq, xs = sr.sr_fwht_quant_act(torch.from_numpy(X).cuda(), inv_s, clip)
    act = o.fwht_quant_act(X, inv_s.cpu().numpy(), clip)            # oracle on the GPU's fp32 inv_s
    check_scales(xs.cpu().numpy(), act["x_scale"])
    cx_gpu = o.unpack_int4(Xq.cpu().numpy())
    xflips = check_codes(cx_gpu, act["codes"], act["t"], what + " X codes")

    acc = sr.sr_w4a4_gemm(Xq, None, Wq, None, sr.SR_I32)
    Y = sr.sr_w4a4_gemm(Xq, xs, Wq, ws, sr.SR_F16)
    torch.cuda.synchronize()
    rows = np.arange(X.shape[0])                                    # every token row, every output
    acc_ref = o.gemm_i32_c(cx_gpu[rows], cw_gpu)
    assert np.array_equal(acc.cpu().numpy()[rows].astype(np.int64), acc_ref)
    y_ref = o.dequant_out(acc_ref, xs.cpu().numpy()[rows], ws.cpu().numpy())
    rel = check_output(Y.cpu().numpy()[rows], y_ref, what + " Y")

    # sanity against the unquantised layer: 4-bit error, far from exact but far from garbage
    y_exact = X[rows].astype(np.float64) @ W.astype(np.float64)
    q_err = np.linalg.norm(Y.cpu().numpy()[rows] - y_exact) / np.linalg.norm(y_exact)
    print("  flips W/X: %d/%d, fp16 err/rms %.2e, 4-bit rel err vs fp64 XW %.3f" % (wflips, xflips, rel, q_err), flush=True)
    assert q_err < 0.5
    return q_err


def test_cfg1_layer(gpu):
    c = wl.cfg1()
    run_layer(gpu, c["X"], c["W"], c["calib"], what="cfg1")


def test_cfg2_layer_n4096(gpu):
    run_layer(gpu, wl.cfg2_X(), wl.cfg2_W(4096), [wl.cfg2_calib_chunk(i) for i in range(2)], what="cfg2/4096")


def test_cfg3_layer_small_m(gpu):
    run_layer(gpu, wl.cfg3_X(M=160), wl.cfg3_W(), [wl.cfg3_calib_chunk(0, T=256)], what="cfg3")


@pytest.mark.parametrize("M", [1, 4, 16])
def test_cfg4_decode_layer(gpu, M):
    K, N = 4096, 14336
    run_layer(gpu, wl.cfg4_X(M, K), wl.cfg4_W(K, N), [wl.cfg2_calib_chunk(0, T=256, seed=3)], what="cfg4 M=%d" % M)


def test_smoothing_helps_on_outliers(gpu):
    """Smoke: rotation-only (act_absmax = NULL) is worse than SmoothRot on the outlier config."""
    c = wl.cfg1()
    X, W = c["X"], c["W"]
    Y = X.astype(np.float64) @ W.astype(np.float64)

    def layer(absmax):
        Wd = torch.from_numpy(W).cuda()
        a = None if absmax is None else torch.from_numpy(absmax.astype(np.float32)).cuda()
        Wq, ws, inv_s = gpu.sr_fold_smooth_rotate_quant(Wd, a, 0.5, 1.0)
        Xq, xs = gpu.sr_fwht_quant_act(torch.from_numpy(X).cuda(), inv_s if a is not None else None, 0.9)
        out = gpu.sr_w4a4_gemm(Xq, xs, Wq, ws).cpu().numpy().astype(np.float64)
        return np.linalg.norm(out - Y) / np.linalg.norm(Y)

    assert layer(o.calib_absmax(X, np.zeros(512))) < layer(None)
