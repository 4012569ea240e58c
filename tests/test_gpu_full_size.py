"""The benchmarked launches at full size, every output compared.

configs[1] (M = 2048, K = 4096 -> N = 4096 and N = 14336) and configs[2] (K = 14336 -> N = 4096), in the launch
configuration bench.py times: activations rotated and quantised by sr_fwht_quant_act_f6_warm with the GEMM's
weights as the warming operand (N = 4096) or by sr_fwht_quant_act_f6 (N = 14336), then sr_w4a4_gemm_f6_warm with
44 MB to warm (N = 4096: the launch that carries the extra wave) or sr_w4a4_gemm_f6; and the same layer through the
canonical-nibble quantiser and the int8-MFMA GEMM.  ALL M x K activation codes are held to the rounding-boundary rule, ALL M x N INT32 accumulators
must equal the oracle's triple loop on the GPU's own codes, ALL fp16 outputs must lie within 1e-2 * rms and within
half an fp16 ulp (+ the two fp32 roundings of the epilogue) of the oracle's dequantised product."""
import numpy as np
import pytest
import torch

from oracle import smoothrot_oracle as o
import f6_codec as fc
import workloads as wl
from parity import check_codes, check_output, check_scales

pytestmark = pytest.mark.gpu


def every_output(Y, acc_ref, xs, ws, what):
    want = o.dequant_out(acc_ref, xs.astype(np.float64), ws.astype(np.float64))
    rel = check_output(Y, want, what)
    # fp16 rounding (2^-11 relative, 2^-25 absolute in the subnormal range) plus two fp32 roundings of the products
    assert np.all(np.abs(Y.astype(np.float64) - want) <= np.abs(want) * (2.0 ** -11 + 2.0 ** -22) + 2.0 ** -25), what
    return rel


@pytest.mark.parametrize("name,K,N", [("cfg2", 4096, 4096), ("cfg2", 4096, 14336), ("cfg3", 14336, 4096)])
def test_benchmarked_launches_every_output(gpu, name, K, N):
    M = 2048
    print("case", name, M, K, N, flush=True)
    if name == "cfg2":
        X, W = wl.cfg2_X(M, K), wl.cfg2_W(N, K)
        a = o.calib_absmax(wl.cfg2_calib_chunk(0, 512, K), np.zeros(K))
    else:
        X, W = wl.cfg3_X(M, K), wl.cfg3_W(N, K)
        a = o.calib_absmax(wl.cfg3_calib_chunk(0, 512, K), np.zeros(K))
    Xd = torch.from_numpy(X).cuda()
    Wq, ws, inv_s = gpu.sr_fold_smooth_rotate_quant(torch.from_numpy(W).cuda(), torch.from_numpy(a.astype(np.float32)).cuda(), 0.5, 1.0)
    W6 = gpu.sr_pack_f6_tiles(Wq)
    torch.cuda.synchronize()
    cw = o.unpack_int4(Wq.cpu().numpy())
    assert np.array_equal(fc.f6_codes(fc.f6_tiles_unpack(W6.cpu().numpy(), N, K)), cw)
    ws_h = ws.cpu().numpy()
    ref = o.fwht_quant_act(X, inv_s.cpu().numpy(), 0.9)                 # oracle on the GPU's fp32 factors

    # ---- tile path, as bench.py calls it
    if (K, N) == (4096, 14336):
        X6, xs6 = gpu.sr_fwht_quant_act_f6(Xd, inv_s, 0.9)
        nxt = None
    else:
        X6, xs6 = gpu.sr_fwht_quant_act_f6_warm(Xd, inv_s, 0.9, W6)
        nxt = torch.randint(0, 255, (gpu.sr_f6_tiles_bytes(14336, 4096),), dtype=torch.uint8, device="cuda")   # the next linear's weights
    acc6 = gpu.sr_w4a4_gemm_f6(X6, None, W6, None, M, N, K, gpu.SR_I32, warm=nxt)
    Y6 = gpu.sr_w4a4_gemm_f6(X6, xs6, W6, ws, M, N, K, gpu.SR_F16, warm=nxt)
    torch.cuda.synchronize()
    cx6 = fc.f6_codes(fc.f6_tiles_unpack(X6.cpu().numpy(), M, K))
    check_scales(xs6.cpu().numpy(), ref["x_scale"])
    flips6 = check_codes(cx6, ref["codes"], ref["t"], "X codes (tile path)")
    want6 = o.gemm_i32_c(cx6, cw)
    assert np.array_equal(acc6.cpu().numpy().astype(np.int64), want6)
    rel6 = every_output(Y6.cpu().numpy(), want6, xs6.cpu().numpy(), ws_h, "Y (FP6-pipe GEMM)")

    # ---- canonical nibbles + int8-MFMA GEMM
    Xq, xs = gpu.sr_fwht_quant_act(Xd, inv_s, 0.9)
    acc = gpu.sr_w4a4_gemm(Xq, None, Wq, None, gpu.SR_I32)
    Y = gpu.sr_w4a4_gemm(Xq, xs, Wq, ws, gpu.SR_F16)
    torch.cuda.synchronize()
    cx = o.unpack_int4(Xq.cpu().numpy())
    check_scales(xs.cpu().numpy(), ref["x_scale"])
    flips = check_codes(cx, ref["codes"], ref["t"], "X codes (nibble path)")
    want = want6 if np.array_equal(cx, cx6) else o.gemm_i32_c(cx, cw)
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), want)
    rel = every_output(Y.cpu().numpy(), want, xs.cpu().numpy(), ws_h, "Y (int8 GEMM)")
    print("  boundary flips tile/nibble path: %d/%d of %d codes; fp16 err/rms %.2e / %.2e" % (flips6, flips, cx.size, rel6, rel), flush=True)
