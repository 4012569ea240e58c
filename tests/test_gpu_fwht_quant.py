"""GPU parity: sr_fwht_quant_act (rotation + per-token INT4) against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import smoothrot_oracle as o
import workloads as wl
from parity import check_codes, check_scales

pytestmark = pytest.mark.gpu

POW2 = [64, 128, 256, 512, 1024, 2048, 4096, 8192, 16384, 32768]
KRON = [448, 896, 1792, 3584, 7168, 14336, 28672]


def run_gpu(sr, X, inv_s, clip, ldx=None):
    M, K = X.shape
    if ldx is None:
        Xd = torch.from_numpy(X).cuda()
    else:
        buf = torch.zeros((M, ldx), dtype=torch.float16, device="cuda")
        buf[:, :K] = torch.from_numpy(X).cuda()
        Xd = buf[:, :K]
    inv = None if inv_s is None else torch.from_numpy(inv_s).cuda()
    Xq, xs = sr.sr_fwht_quant_act(Xd, inv, clip)
    torch.cuda.synchronize()
    return Xq.cpu().numpy(), xs.cpu().numpy()


def compare(sr, X, inv_s, clip, ldx=None, what=""):
    print("case", what, X.shape, "inv_s" if inv_s is not None else "no-inv_s", clip, flush=True)
    packed, xs = run_gpu(sr, X, inv_s, clip, ldx)
    ref = o.fwht_quant_act(X, inv_s, clip)
    check_scales(xs, ref["x_scale"], what + " x_scale")
    codes = o.unpack_int4(packed)
    flips = check_codes(codes, ref["codes"], ref["t"], what + " codes")
    same = codes == ref["codes"]
    both = same[:, 0::2] & same[:, 1::2]
    assert np.array_equal(packed[both], ref["packed"][both])        # packed bytes bit-exact wherever codes agree
    return flips


def test_cfg1(gpu):
    c = wl.cfg1()
    a = o.calib_absmax(c["X"], np.zeros(512))
    inv_s = (1.0 / o.smoothing_factors(a, c["W"], 0.5)).astype(np.float32)
    for clip in (0.9, 1.0):
        compare(gpu, c["X"], inv_s, clip, what="cfg1")
        compare(gpu, c["X"], None, clip, what="cfg1-rot-only")


@pytest.mark.parametrize("K", POW2 + KRON)
def test_every_supported_order(gpu, K):
    rng = np.random.default_rng(K)
    X = wl.to_f16_sat(rng.standard_normal((5, K)).astype(np.float32) * (1 + 300 * (rng.random(K) < 0.002)))
    inv_s = np.exp(rng.standard_normal(K) * 0.5).astype(np.float32)
    compare(gpu, X, inv_s, 0.9, what="K=%d" % K)


@pytest.mark.parametrize("K,M", [(7168, 3), (7168, 520), (14336, 200), (14336, 300), (8192, 70), (16384, 40), (28672, 20), (32768, 20)])
def test_long_rows_both_workgroup_sizes(gpu, K, M):
    """Long rows run with 256, 512 or 1024 threads per row, for K = 7168 and 14336 depending on the row count
    (512 / 256 rows is where the launcher switches): every choice against the oracle."""
    rng = np.random.default_rng(K + M)
    X = wl.to_f16_sat(rng.standard_normal((M, K)).astype(np.float32) * (1 + 200 * (rng.random(K) < 0.002)))
    inv_s = np.exp(rng.standard_normal(K) * 0.5).astype(np.float32)
    compare(gpu, X, inv_s, 0.9, what="K=%d M=%d" % (K, M))


@pytest.mark.parametrize("K", [64, 512, 4096, 448, 14336])
def test_unit_vectors_reproduce_rows_of_H(gpu, K):
    """X = c * e_k with clip = 1: y = c * H[k], so every code is exactly 7 * H[k][j] and Delta = c / 7.
    This compares the GPU's Hadamard matrix (incl. its own Paley table) entry by entry with the oracle's."""
    ks = sorted(set([0, 1, 2, 3, K // 2 - 1, K // 2, K - 1] + list(range(5, K, max(1, K // 29)))))
    X = np.zeros((len(ks), K), np.float16)
    X[np.arange(len(ks)), ks] = 3.0
    packed, xs = run_gpu(gpu, X, None, 1.0)
    H = o.rotate(np.eye(K)[ks])                                   # rows k of H
    assert np.array_equal(o.unpack_int4(packed).astype(np.int64), (7 * H).astype(np.int64))
    np.testing.assert_allclose(xs, 3.0 / 7.0, rtol=1e-6)


def test_kron_all_28_blocks(gpu):
    """One unit vector in each of the 28 slow-index blocks of K = 28 * 16 hits every row of H_28."""
    K = 448
    ks = [i1 * 16 + (i1 % 16) for i1 in range(28)]
    X = np.zeros((28, K), np.float16)
    X[np.arange(28), ks] = 1.0
    packed, _ = run_gpu(gpu, X, None, 1.0)
    H = o.hadamard_dense(K)[ks]
    assert np.array_equal(o.unpack_int4(packed).astype(np.int64), 7 * H)


def test_edge_rows_and_strides(gpu):
    K = 4096
    rng = np.random.default_rng(1)
    X = wl.to_f16_sat(rng.standard_normal((7, K)).astype(np.float32))
    X[2] = 0                                            # all-zero row: Delta = 1, codes 0
    X[4] = 0; X[4, 17] = 65504.0                         # largest finite fp16
    X[5] = 6e-8                                          # fp16 subnormals
    packed, xs = run_gpu(gpu, X, None, 0.9)
    assert xs[2] == 1.0 and not packed[2].any()
    compare(gpu, X, None, 0.9, what="edge")
    compare(gpu, X, None, 0.9, ldx=K + 64, what="ragged-ld")
    compare(gpu, X[:1], None, 1.0, what="M=1")


@pytest.mark.parametrize("kernel", [5, 1, 4])
def test_k4096_many_row_kernels_edges(gpu, tune, kernel):
    """The K = 4096 kernels for many rows (5: a workgroup per row in two passes, the default up to 3072 rows;
    1 / 4: a wave per row, the default beyond): ragged row count (1027 = 4 * 256 + 3), degenerate rows, padded
    leading dimension, with and without smoothing factors."""
    tune(gpu.SR_TUNE_FWHT4096, kernel)
    K, M = 4096, 1027
    X = wl.cfg2_X(M=M).copy()
    X[2] = 0
    X[4] = 0; X[4, 17] = 65504.0
    X[5] = 6e-8
    X[M - 1] = 0; X[M - 1, K - 1] = -3.0
    rng = np.random.default_rng(2)
    inv_s = np.exp(rng.standard_normal(K) * 0.3).astype(np.float32)
    compare(gpu, X, inv_s, 0.9, what="wave edges")
    compare(gpu, X, None, 1.0, ldx=K + 8, what="wave edges ragged-ld")


def test_cfg2_full_size(gpu):
    X = wl.cfg2_X()
    rng = np.random.default_rng(0)
    inv_s = np.exp(rng.standard_normal(4096) * 0.3).astype(np.float32)
    inv_s[wl.outlier_channels(1, 4096, 6)] = 1.0 / 40.0
    flips = compare(gpu, X, inv_s, 0.9, what="cfg2")
    print("cfg2 boundary flips:", flips, "of", X.size)
    assert flips <= 64


def test_cfg3_full_size(gpu):
    X = wl.cfg3_X()
    inv_s = np.ones(14336, np.float32)
    inv_s[wl.outlier_channels(2, 14336, 3)] = 1.0 / 30.0
    flips = compare(gpu, X, inv_s, 0.9, what="cfg3")
    print("cfg3 boundary flips:", flips, "of", X.size)
    assert flips <= 256


def test_repeatable(gpu):
    X = wl.cfg2_X(M=256)
    a = run_gpu(gpu, X, None, 0.9)
    b = run_gpu(gpu, X, None, 0.9)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
