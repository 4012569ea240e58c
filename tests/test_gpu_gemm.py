"""GPU parity: sr_w4a4_gemm.  Given identical codes the INT32 accumulators must be bit-exact;
fp16 outputs within 1e-2 * rms of the oracle's dequantised product."""
import numpy as np
import pytest
import torch

from oracle import smoothrot_oracle as o
import workloads as wl
from parity import check_output

pytestmark = pytest.mark.gpu


def gpu_gemm(sr, cx, cw, xs=None, ws=None, dtype=None, ldy=None):
    dtype = sr.SR_I32 if dtype is None else dtype
    Xq = torch.from_numpy(o.pack_int4(cx)).cuda()
    Wq = torch.from_numpy(o.pack_int4(cw)).cuda()
    xs_d = None if xs is None else torch.from_numpy(xs.astype(np.float32)).cuda()
    ws_d = None if ws is None else torch.from_numpy(ws.astype(np.float32)).cuda()
    Y = None
    M, N = cx.shape[0], cw.shape[0]
    if ldy is not None:
        full = torch.full((M, ldy), -7, dtype=torch.int32 if dtype == sr.SR_I32 else torch.float16, device="cuda")
        Y = full[:, :N]
    out = sr.sr_w4a4_gemm(Xq, xs_d, Wq, ws_d, dtype, Y=Y)
    torch.cuda.synchronize()
    if ldy is not None:
        assert bool((full[:, N:] == -7).all())                      # nothing written past N
    return out.cpu().numpy()


SHAPES = [(1, 16, 64), (4, 48, 128), (2, 32, 448), (5, 80, 4096), (8, 4096, 4096), (7, 16, 14336), (9, 32, 576), (16, 512, 512), (16, 4096, 4096), (3, 64, 14336), (16, 256, 448),
          (3, 16, 64), (12, 48, 192), (9, 12816, 512), (16, 12816, 576), (6, 12816, 256),
          (17, 16, 64), (33, 48, 192), (100, 144, 448), (128, 128, 128), (129, 272, 576), (300, 1040, 512),
          (257, 400, 4096), (64, 128, 14336)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_int32_accumulators_bit_exact(gpu, M, N, K):
    print("case", M, N, K, flush=True)
    cx, cw = wl.random_codes(M + K, M, K), wl.random_codes(N + 3 * K, N, K)
    want = o.gemm_i32_c(cx, cw)
    got = gpu_gemm(gpu, cx, cw)
    assert got.dtype == np.int32 and np.array_equal(got.astype(np.int64), want)


@pytest.mark.parametrize("M", [1, 16, 40])
def test_extreme_codes_do_not_overflow(gpu, M):
    """All codes -8 at the largest K the call accepts: acc = 64 K, the worst case of the accumulator."""
    for K in (14336, 131008):
        cx = np.full((M, K), -8, np.int8)
        cw = np.full((32, K), -8, np.int8)
        cw[1::2] = 7
        got = gpu_gemm(gpu, cx, cw)
        assert np.all(got[:, 0::2] == 64 * K) and np.all(got[:, 1::2] == -56 * K)


@pytest.mark.parametrize("M,N,K", [(16, 512, 512), (4, 4096, 14336), (1, 14336, 4096), (200, 528, 1024), (2048, 1024, 4096)])
def test_fp16_epilogue(gpu, M, N, K):
    rng = np.random.default_rng(M * N)
    cx, cw = wl.random_codes(1, M, K), wl.random_codes(2, N, K)
    xs = np.exp(rng.standard_normal(M) * 0.5).astype(np.float32) * 0.05   # per-token spread of the prefill config
    ws = np.exp(rng.standard_normal(N) * 0.3).astype(np.float32) * 1e-3
    want = o.dequant_out(o.gemm_i32_c(cx, cw), xs, ws)
    got = gpu_gemm(gpu, cx, cw, xs, ws, gpu.SR_F16)
    rel = check_output(got, want, "Y %dx%dx%d" % (M, N, K))
    # fp16 rounding is the only error source: elementwise half-ulp bound as well
    assert np.all(np.abs(got.astype(np.float64) - want) <= np.abs(want) * 2.0 ** -10 + 1e-7), rel


def test_ragged_leading_dimension(gpu):
    cx, cw = wl.random_codes(5, 50, 256), wl.random_codes(6, 80, 256)
    want = o.gemm_i32(cx, cw)
    assert np.array_equal(gpu_gemm(gpu, cx, cw, ldy=96), want)
    assert np.array_equal(gpu_gemm(gpu, cx[:9], cw, ldy=96), want[:9])


@pytest.mark.parametrize("N", [4096, 14336])
def test_cfg2_full_size_every_accumulator(gpu, N):
    """Full prefill shape in the configuration the benchmark times: every INT32 accumulator against the oracle's
    triple loop; the two identities that hold at any size stay as a cross-check of the comparison:
    sum_n acc[m][n] = cx[m] . (sum_n cw[n])   and   sum_m acc[m][n] = (sum_m cx[m]) . cw[n]."""
    M, K = 2048, 4096
    cx, cw = wl.random_codes(11, M, K), wl.random_codes(12 + N, N, K)
    got = gpu_gemm(gpu, cx, cw).astype(np.int64)
    assert np.array_equal(got, o.gemm_i32_c(cx, cw))
    assert np.array_equal(got.sum(axis=1), cx.astype(np.int64) @ cw.astype(np.int64).sum(axis=0))
    assert np.array_equal(got.sum(axis=0), cw.astype(np.int64) @ cx.astype(np.int64).sum(axis=0))


def test_cfg3_full_size_every_accumulator(gpu):
    M, K, N = 2048, 14336, 4096
    cx, cw = wl.random_codes(21, M, K), wl.random_codes(22, N, K)
    got = gpu_gemm(gpu, cx, cw).astype(np.int64)
    assert np.array_equal(got, o.gemm_i32_c(cx, cw))
    assert np.array_equal(got.sum(axis=1), cx.astype(np.int64) @ cw.astype(np.int64).sum(axis=0))
    assert np.array_equal(got.sum(axis=0), cw.astype(np.int64) @ cx.astype(np.int64).sum(axis=0))


@pytest.mark.parametrize("M", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("K,N", [(4096, 14336), (14336, 4096)])
def test_cfg4_decode_shapes(gpu, M, K, N):
    cx, cw = wl.random_codes(31 + M, M, K), wl.random_codes(32 + K, N, K)
    assert np.array_equal(gpu_gemm(gpu, cx, cw).astype(np.int64), o.gemm_i32_c(cx, cw))


# The three decode kernels (forced through the library's tuning switch, so that each one is checked on
# every shape, not only where the dispatcher would pick it): 1 = dot product (at most 2 tokens), 2 = MFMA with a
# workgroup per 16 channels, 3 = streaming MFMA.  Shapes: K with a half-empty last 256-code slab (448, 576,
# 4160), a single 16-channel group, output lines that are not whole (N % 64 != 0), more channels than one pass
# of the streaming kernel takes (20000; 8208 at K = 4160), rows longer than one pass over K (14336, 16000).
DECODE_SHAPES = [(1, 16, 64), (2, 48, 448), (3, 16, 64), (5, 80, 4096), (8, 4096, 4096), (7, 16, 14336), (9, 32, 576),
                 (16, 512, 512), (16, 256, 448), (12, 48, 192), (16, 12816, 576), (6, 12816, 256), (16, 20000, 128),
                 (5, 8208, 4160), (13, 1040, 16000), (16, 4096, 8192), (4, 14336, 4096), (16, 4096, 14336), (2, 1024, 16000)]


def per_kernel(shapes):
    """(kernel, M, N, K) for every kernel that takes M tokens (the dot-product kernel: at most two)."""
    return [(k,) + tuple(sh) for sh in shapes for k in ("1", "2", "3") if k != "1" or sh[0] <= 2]


@pytest.mark.parametrize("kernel,M,N,K", per_kernel(DECODE_SHAPES))
def test_every_decode_kernel_bit_exact(gpu, tune, kernel, M, N, K):
    print("case", kernel, M, N, K, flush=True)
    tune(gpu.SR_TUNE_DECODE_KERNEL, kernel)
    cx, cw = wl.random_codes(7 * M + K, M, K), wl.random_codes(N + 5 * K, N, K)
    got = gpu_gemm(gpu, cx, cw)
    assert np.array_equal(got.astype(np.int64), o.gemm_i32_c(cx, cw))


@pytest.mark.parametrize("kernel,M", [(k, M) for (k, M) in per_kernel([(1,), (2,), (16,)])])
def test_every_decode_kernel_extreme_codes(gpu, tune, kernel, M):
    tune(gpu.SR_TUNE_DECODE_KERNEL, kernel)
    K = 131008
    cx = np.full((M, K), -8, np.int8)
    cw = np.full((48, K), -8, np.int8)
    cw[1::2] = 7
    got = gpu_gemm(gpu, cx, cw)
    assert np.all(got[:, 0::2] == 64 * K) and np.all(got[:, 1::2] == -56 * K)


@pytest.mark.parametrize("kernel,M,N,K", per_kernel([(2, 4096, 4096), (4, 14336, 4096), (11, 528, 1088), (16, 4096, 14336)]))
def test_every_decode_kernel_fp16_and_leading_dimension(gpu, tune, kernel, M, N, K):
    tune(gpu.SR_TUNE_DECODE_KERNEL, kernel)
    rng = np.random.default_rng(M * N + int(kernel))
    cx, cw = wl.random_codes(3, M, K), wl.random_codes(4, N, K)
    xs = np.exp(rng.standard_normal(M) * 0.5).astype(np.float32) * 0.05
    ws = np.exp(rng.standard_normal(N) * 0.3).astype(np.float32) * 1e-3
    acc = o.gemm_i32_c(cx, cw)
    want = o.dequant_out(acc, xs, ws)
    got = gpu_gemm(gpu, cx, cw, xs, ws, gpu.SR_F16, ldy=N + 24)
    check_output(got, want, "Y %dx%dx%d kernel %s" % (M, N, K, kernel))
    # fp16 rounding plus the two fp32 roundings of the dequantisation are the only error sources
    assert np.all(np.abs(got.astype(np.float64) - want) <= np.abs(want) * (2.0 ** -10 + 2.0 ** -21) + 1e-7)
    assert np.array_equal(gpu_gemm(gpu, cx, cw, ldy=N + 8).astype(np.int64), acc)


def test_decode_seeded_random_shapes(gpu, tune):
    """Thirty seeded shapes (M up to 16, N a multiple of 16 up to 9600, K a multiple of 64 up to 6144) through
    every decode kernel that takes them and through the dispatcher's own choice: accumulators bit-exact, nothing
    written past N."""
    rng = np.random.default_rng(20250606)
    for case in range(30):
        M = int(rng.integers(1, 17))
        N = 16 * int(rng.integers(1, 601))
        K = 64 * int(rng.integers(1, 97))
        cx, cw = wl.random_codes(3000 + case, M, K), wl.random_codes(4000 + case, N, K)
        want = o.gemm_i32_c(cx, cw)
        for kernel in ("0", "1", "2", "3"):
            if kernel == "1" and M > 2:
                continue
            print("case", case, M, N, K, "kernel", kernel, flush=True)
            tune(gpu.SR_TUNE_DECODE_KERNEL, kernel)
            assert np.array_equal(gpu_gemm(gpu, cx, cw, ldy=N + 8).astype(np.int64), want), (M, N, K, kernel)


def test_repeatable_bitwise(gpu):
    cx, cw = wl.random_codes(41, 300, 1024), wl.random_codes(42, 512, 1024)
    a = gpu_gemm(gpu, cx, cw)
    for _ in range(3):
        assert np.array_equal(a, gpu_gemm(gpu, cx, cw))
