"""GPU parity: sr_w4a4_linear_decode (rotate + quantise + multiply in one launch, up to 16 tokens) against the
CPU oracle, stage by stage: the activation codes and scales it reports are checked like those of
sr_fwht_quant_act, and its output against the oracle's integer GEMM + dequantisation of those codes.
One token with K = 2048 / 4096 runs the single kernel in which every workgroup rotates the row itself; several
tokens, K = 8192 and K = 14336 run the rotation kernel and the GEMM back to back inside the call, codes and scales
going through the workspace."""
import numpy as np
import pytest
import torch

from oracle import smoothrot_oracle as o
import workloads as wl
from parity import check_codes, check_output, check_scales

pytestmark = pytest.mark.gpu


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_case(sr, X, inv_s, cw, ws, clip, what):
    M, K = X.shape
    N = cw.shape[0]
    print("case linear_decode", what, M, K, N, flush=True)
    Wq = dev(o.pack_int4(cw))
    Xq = torch.zeros((M, K // 2), dtype=torch.uint8, device="cuda")
    xs = torch.zeros(M, dtype=torch.float32, device="cuda")
    # ONE workspace for both calls below, pre-filled with a pattern: its contents need no initialisation
    wsp = torch.full((max(sr.sr_linear_decode_workspace_bytes(M, K), 256),), 0xA5, dtype=torch.uint8, device="cuda")
    Y = sr.sr_w4a4_linear_decode(dev(X), dev(inv_s), Wq, dev(ws), clip, Xq_out=Xq, x_scale_out=xs, workspace=wsp)
    torch.cuda.synchronize()
    ref = o.fwht_quant_act(X, inv_s, clip)
    check_scales(xs.cpu().numpy(), ref["x_scale"], what + " x_scale")
    codes = o.unpack_int4(Xq.cpu().numpy())
    flips = check_codes(codes, ref["codes"], ref["t"], what + " codes")
    # downstream of the (checked) codes everything is exact up to the fp16 rounding of the output
    want = o.dequant_out(o.gemm_i32_c(codes, cw), xs.cpu().numpy().astype(np.float64), ws)
    got = Y.cpu().numpy()
    check_output(got, want, what + " Y")
    assert np.all(np.abs(got.astype(np.float64) - want) <= np.abs(want) * 2.0 ** -10 + 1e-7)
    # without the optional outputs the result is the same, bit for bit (same workspace, second use)
    Y2 = sr.sr_w4a4_linear_decode(dev(X), dev(inv_s), Wq, dev(ws), clip, workspace=wsp)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2)
    return flips


@pytest.mark.parametrize("K,N", [(2048, 64), (2048, 6144), (4096, 14336), (4096, 4096), (4096, 2048), (8192, 1024),
                                 (8192, 8192), (4096, 1040), (4096, 16)])
def test_shapes(gpu, K, N):
    M = 1
    rng = np.random.default_rng(K + N + M)
    X = wl.cfg4_X(M, K) if K == 4096 else wl.to_f16_sat(
        rng.standard_normal((M, K)).astype(np.float32) * (1 + 300 * (rng.random(K) < 0.002)))
    inv_s = np.exp(rng.standard_normal(K) * 0.5).astype(np.float32)
    cw = wl.random_codes(N + K, N, K)
    ws = (np.exp(rng.standard_normal(N) * 0.3) * 1e-3).astype(np.float32)
    run_case(gpu, X, inv_s, cw, ws, 0.9, "K=%d N=%d" % (K, N))


def test_no_smoothing_zero_row_and_padded_output(gpu):
    K, N = 4096, 256
    rng = np.random.default_rng(3)
    X = wl.to_f16_sat(rng.standard_normal((1, K)).astype(np.float32))
    cw = wl.random_codes(9, N, K)
    ws = np.full(N, 1e-3, np.float32)
    run_case(gpu, X, None, cw, ws, 1.0, "no inv_s")
    run_case(gpu, np.zeros((1, K), np.float16), None, cw, ws, 0.9, "zero token")   # Delta = 1, codes 0, output 0
    yb = torch.full((1, N + 16), -7.0, dtype=torch.float16, device="cuda")
    gpu.sr_w4a4_linear_decode(dev(X), None, dev(o.pack_int4(cw)), dev(ws), 1.0, Y=yb[:, :N])
    torch.cuda.synchronize()
    assert bool((yb[:, N:] == -7).all())
    ref = gpu.sr_w4a4_linear_decode(dev(X), None, dev(o.pack_int4(cw)), dev(ws), 1.0)
    assert torch.equal(ref, yb[:, :N].contiguous())
    z = gpu.sr_w4a4_linear_decode(dev(np.zeros((1, K), np.float16)), None, dev(o.pack_int4(cw)), dev(ws), 0.9)
    assert bool((z == 0).all())


def test_matches_the_two_call_path(gpu):
    """Same fold outputs, same token: the one-launch path and sr_fwht_quant_act + sr_w4a4_gemm agree except
    where a code sits on a rounding boundary (different fp32 summation order in the two rotation kernels)."""
    X = wl.cfg4_X(1, 4096)
    W = wl.cfg4_W(4096, 14336)
    a = o.calib_absmax(wl.cfg2_calib_chunk(0, T=256), np.zeros(4096)).astype(np.float32)
    Wq, ws, inv_s = gpu.sr_fold_smooth_rotate_quant(dev(W), dev(a), 0.5, 1.0)
    Xq, xs = gpu.sr_fwht_quant_act(dev(X), inv_s, 0.9)
    Y2 = gpu.sr_w4a4_gemm(Xq, xs, Wq, ws, gpu.SR_F16)
    Xq1 = torch.zeros_like(Xq)
    xs1 = torch.zeros_like(xs)
    Y1 = gpu.sr_w4a4_linear_decode(dev(X), inv_s, Wq, ws, 0.9, Xq_out=Xq1, x_scale_out=xs1)
    torch.cuda.synchronize()
    np.testing.assert_allclose(xs1.cpu().numpy(), xs.cpu().numpy(), rtol=1e-6)
    c1, c2 = o.unpack_int4(Xq1.cpu().numpy()).astype(int), o.unpack_int4(Xq.cpu().numpy()).astype(int)
    assert np.abs(c1 - c2).max() <= 1 and (c1 != c2).sum() <= 4
    y1, y2 = Y1.cpu().numpy().astype(np.float64), Y2.cpu().numpy().astype(np.float64)
    assert np.abs(y1 - y2).max() <= 1e-2 * np.sqrt(np.mean(y2 ** 2))


# ---------------------------------------------------------------- several tokens, K = 8192, K = 14336

COOP = [(1, 8192, 8192), (1, 14336, 4096), (4, 14336, 4096), (16, 14336, 4096), (2, 4096, 14336), (16, 4096, 14336), (5, 4096, 4096),
        (3, 2048, 1040), (16, 8192, 2048), (9, 14336, 272), (16, 14336, 128), (7, 8192, 64)]


@pytest.mark.parametrize("M,K,N", COOP)
def test_general_shapes(gpu, M, K, N):
    rng = np.random.default_rng(K + N + M)
    if K == 4096:
        X = wl.cfg4_X(M, K)
    elif K == 14336:
        X = wl.cfg3_X(M=M, K=K, seed=3)
    else:
        X = wl.to_f16_sat(rng.standard_normal((M, K)).astype(np.float32) * (1 + 300 * (rng.random(K) < 0.002)))
    inv_s = np.exp(rng.standard_normal(K) * 0.5).astype(np.float32)
    cw = wl.random_codes(N + K, N, K)
    ws = (np.exp(rng.standard_normal(N) * 0.3) * 1e-3).astype(np.float32)
    run_case(gpu, X, inv_s if M % 2 else None, cw, ws, 0.9, "M=%d K=%d N=%d" % (M, K, N))


def test_padded_rows_and_zero_tokens(gpu):
    """Row strides larger than the rows on both sides, an all-zero token among others, nothing written outside Y."""
    M, K, N = 6, 14336, 528
    X = wl.cfg3_X(M=M, K=K, seed=5)
    X[2] = 0
    cw = wl.random_codes(3, N, K)
    ws = np.full(N, 2e-3, np.float32)
    Xp = torch.full((M, K + 64), 7.0, dtype=torch.float16, device="cuda")
    Xp[:, :K] = dev(X)
    Yp = torch.full((M + 1, N + 24), -7.0, dtype=torch.float16, device="cuda")
    Xq = torch.zeros((M, K // 2), dtype=torch.uint8, device="cuda")
    xs = torch.zeros(M, dtype=torch.float32, device="cuda")
    gpu.sr_w4a4_linear_decode(Xp[:, :K], None, dev(o.pack_int4(cw)), dev(ws), 0.9, Y=Yp[:M, :N], Xq_out=Xq, x_scale_out=xs)
    torch.cuda.synchronize()
    assert bool((Yp[:, N:] == -7).all()) and bool((Yp[M:] == -7).all())
    ref = o.fwht_quant_act(X, None, 0.9)
    check_scales(xs.cpu().numpy(), ref["x_scale"])
    codes = o.unpack_int4(Xq.cpu().numpy())
    check_codes(codes, ref["codes"], ref["t"])
    assert xs.cpu().numpy()[2] == 1.0 and not codes[2].any() and bool((Yp[2, :N] == 0).all())
    want = o.dequant_out(o.gemm_i32_c(codes, cw), xs.cpu().numpy().astype(np.float64), ws)
    check_output(Yp[:M, :N].cpu().numpy(), want)


def test_several_tokens_match_the_two_call_path(gpu):
    M, K, N = 16, 14336, 4096
    X = wl.cfg3_X(M=M, K=K, seed=3)
    W = wl.cfg4_W(K, N)
    a = o.calib_absmax(wl.cfg3_calib_chunk(0, T=256), np.zeros(K)).astype(np.float32)
    Wq, ws, inv_s = gpu.sr_fold_smooth_rotate_quant(dev(W), dev(a), 0.5, 1.0)
    Xq, xs = gpu.sr_fwht_quant_act(dev(X), inv_s, 0.9)
    Y2 = gpu.sr_w4a4_gemm(Xq, xs, Wq, ws, gpu.SR_F16)
    Xq1, xs1 = torch.zeros_like(Xq), torch.zeros_like(xs)
    Y1 = gpu.sr_w4a4_linear_decode(dev(X), inv_s, Wq, ws, 0.9, Xq_out=Xq1, x_scale_out=xs1)
    torch.cuda.synchronize()
    np.testing.assert_allclose(xs1.cpu().numpy(), xs.cpu().numpy(), rtol=1e-6)
    c1, c2 = o.unpack_int4(Xq1.cpu().numpy()).astype(int), o.unpack_int4(Xq.cpu().numpy()).astype(int)
    assert np.array_equal(c1, c2)                              # the same two kernels, inside the call
    assert torch.equal(Y1, Y2)
