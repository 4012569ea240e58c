"""GPU parity: sr_calib_absmax (exact) and sr_fold_smooth_rotate_quant against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import smoothrot_oracle as o
import workloads as wl
from parity import check_codes, check_scales

pytestmark = pytest.mark.gpu


def gpu_absmax(sr, chunks, K, ldx=None):
    a = torch.zeros(K, dtype=torch.float32, device="cuda")
    for X in chunks:
        if ldx is None:
            Xd = torch.from_numpy(X).cuda()
        else:
            buf = torch.full((X.shape[0], ldx), 60000.0, dtype=torch.float16, device="cuda")
            buf[:, :K] = torch.from_numpy(X).cuda()
            Xd = buf[:, :K]
        sr.sr_calib_absmax(Xd, a)
    torch.cuda.synchronize()
    return a.cpu().numpy()


# from 8192 rows on the kernel takes strips of 16 column groups instead of 8 (row counts around the switch, ragged
# strips, a last strip cut by K, and the 16384-token batch of config 5)
@pytest.mark.parametrize("T,K", [(1, 64), (3, 512), (16, 512), (63, 576), (64, 4096), (65, 4096), (1000, 1088),
                                 (2048, 4096), (777, 14336), (8191, 512), (8192, 576), (8209, 1088), (16384, 4096)])
def test_calib_absmax_exact(gpu, T, K):
    print("case", T, K, flush=True)
    rng = np.random.default_rng(T * K)
    X = wl.to_f16_sat(rng.standard_normal((T, K)).astype(np.float32) * (1 + 999 * (rng.random(K) < 0.01)))
    want = o.calib_absmax(X, np.zeros(K))
    assert np.array_equal(gpu_absmax(gpu, [X], K).astype(np.float64), want)
    # chunked accumulation and a padded leading dimension give the same running maximum
    assert np.array_equal(gpu_absmax(gpu, [X[: T // 3], X[T // 3:]], K, ldx=K + 8).astype(np.float64), want)


def test_calib_cfg2_chunks(gpu):
    chunks = [wl.cfg2_calib_chunk(i) for i in range(3)]
    want = np.zeros(4096)
    for c in chunks:
        want = o.calib_absmax(c, want)
    assert np.array_equal(gpu_absmax(gpu, chunks, 4096).astype(np.float64), want)


def gpu_fold(sr, W, a, alpha, w_clip):
    Wd = torch.from_numpy(W).cuda()
    ad = None if a is None else torch.from_numpy(a.astype(np.float32)).cuda()
    Wq, ws, inv_s = sr.sr_fold_smooth_rotate_quant(Wd, ad, alpha, w_clip)
    torch.cuda.synchronize()
    return Wq.cpu().numpy(), ws.cpu().numpy(), inv_s.cpu().numpy()


def compare_fold(sr, W, a, alpha, w_clip=1.0, what=""):
    print("case", what, W.shape, alpha, w_clip, flush=True)
    packed, ws, inv_s = gpu_fold(sr, W, a, alpha, w_clip)
    ref = o.fold_smooth_rotate_quant(W, None if a is None else a.astype(np.float32), float(np.float32(alpha)), w_clip)
    check_scales(inv_s, ref["inv_s"], what + " inv_s")
    check_scales(ws, ref["w_scale"], what + " w_scale")
    flips = check_codes(o.unpack_int4(packed), ref["codes"], ref["t"], what + " weight codes")
    return flips


def test_fold_cfg1(gpu):
    c = wl.cfg1()
    a = o.calib_absmax(c["X"], np.zeros(512))
    for alpha in (0.5, 0.0, 1.0, 0.45):
        compare_fold(gpu, c["W"], a, alpha, what="cfg1")
    compare_fold(gpu, c["W"], None, 0.5, what="cfg1 rotation only")
    compare_fold(gpu, c["W"], a, 0.5, 0.85, what="cfg1 clipped")


@pytest.mark.parametrize("K,N", [(64, 16), (448, 48), (1024, 80), (4096, 256), (14336, 64), (32768, 16)])
def test_fold_shapes(gpu, K, N):
    rng = np.random.default_rng(K + N)
    W = wl.to_f16_sat(rng.standard_normal((K, N)).astype(np.float32) * 0.02)
    a = (np.abs(rng.standard_normal(K)) * (1 + 800 * (rng.random(K) < 0.003))).astype(np.float32)
    a[1] = 0.0                                           # never-activated channel: floored
    W[2, :] = 0                                          # dead input channel: floored
    compare_fold(gpu, W, a, 0.5, what="K=%d N=%d" % (K, N))


def test_fold_zero_output_channel_and_padded_ld(gpu):
    K, N = 512, 32
    rng = np.random.default_rng(9)
    W = wl.to_f16_sat(rng.standard_normal((K, N)).astype(np.float32) * 0.02)
    W[:, 7] = 0
    buf = torch.zeros((K, N + 24), dtype=torch.float16, device="cuda")
    buf[:, :N] = torch.from_numpy(W).cuda()
    Wq, ws, inv_s = gpu.sr_fold_smooth_rotate_quant(buf[:, :N], None, 0.5, 1.0)
    torch.cuda.synchronize()
    ref = o.fold_smooth_rotate_quant(W, None, 0.5, 1.0)
    assert ws[7].item() == 1.0 and not Wq[7].any().item()
    check_scales(ws.cpu().numpy(), ref["w_scale"])
    check_codes(o.unpack_int4(Wq.cpu().numpy()), ref["codes"], ref["t"])
    assert np.all(inv_s.cpu().numpy() == 1.0)


def test_fold_cfg2_full_size(gpu):
    W = wl.cfg2_W(4096)
    a = o.calib_absmax(wl.cfg2_calib_chunk(0), np.zeros(4096))
    flips = compare_fold(gpu, W, a, 0.5, what="cfg2 N=4096")
    print("cfg2 weight boundary flips:", flips)
    assert flips <= 128


def test_fold_cfg3_full_size(gpu):
    W = wl.cfg3_W()
    a = o.calib_absmax(wl.cfg3_calib_chunk(0, T=512), np.zeros(14336))
    flips = compare_fold(gpu, W, a, 0.5, what="cfg3")
    print("cfg3 weight boundary flips:", flips)
    assert flips <= 512
