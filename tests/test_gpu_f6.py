"""GPU parity of the FP6-matrix-pipe path: sr_pack_f6_tiles, sr_fwht_quant_act_f6, sr_w4a4_gemm_f6.

The sums are the integer sums of the quantised forward pass, so the bar is the same as for
sr_w4a4_gemm: INT32 accumulators bit-exact given identical codes, fp16 outputs within 1e-2 * rms,
tile images byte for byte what the format's definition (oracle) gives, activation codes under the
rounding-boundary rule."""
import numpy as np
import pytest
import torch

from oracle import smoothrot_oracle as o
import workloads as wl
import f6_codec as fc
from parity import check_codes, check_output, check_scales

pytestmark = pytest.mark.gpu


def tiles(sr, codes):
    return sr.sr_pack_f6_tiles(torch.from_numpy(o.pack_int4(codes)).cuda())


@pytest.mark.parametrize("rows,K", [(1, 128), (8, 128), (9, 256), (100, 896), (257, 4096), (2048, 1024), (33, 14336)])
def test_pack_matches_the_format_definition(gpu, rows, K):
    print("case", rows, K, flush=True)
    c = wl.random_codes(rows * 3 + K, rows, K)
    got = tiles(gpu, c).cpu().numpy()
    want = fc.f6_tiles_pack(c)
    assert got.size >= want.size and np.array_equal(got[:want.size], want)      # padding rows are zero codes here


def gemm_f6(sr, cx, cw, xs=None, ws=None, dtype=None, ldy=None):
    dtype = sr.SR_I32 if dtype is None else dtype
    M, K = cx.shape
    N = cw.shape[0]
    X6, W6 = tiles(sr, cx), tiles(sr, cw)
    xs_d = None if xs is None else torch.from_numpy(xs.astype(np.float32)).cuda()
    ws_d = None if ws is None else torch.from_numpy(ws.astype(np.float32)).cuda()
    Y = None
    if ldy is not None:
        full = torch.full((M, ldy), -7, dtype=torch.int32 if dtype == sr.SR_I32 else torch.float16, device="cuda")
        Y = full[:, :N]
    out = sr.sr_w4a4_gemm_f6(X6, xs_d, W6, ws_d, M, N, K, dtype, Y)
    torch.cuda.synchronize()
    if ldy is not None:
        assert bool((full[:, N:] == -7).all())                      # nothing written past N
    return out.cpu().numpy()


# single tile, ragged edges in M and N, several tiles per workgroup (persistent loop), K from one stage up
SHAPES = [(1, 16, 128), (5, 48, 256), (16, 512, 512), (17, 16, 128), (33, 48, 384), (100, 144, 896), (128, 128, 128),
          (129, 272, 640), (256, 256, 512), (300, 1040, 512), (257, 400, 4096), (64, 128, 14336), (520, 784, 1792),
          (1031, 528, 256)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_int32_accumulators_bit_exact(gpu, M, N, K):
    print("case", M, N, K, flush=True)
    cx, cw = wl.random_codes(M + K, M, K), wl.random_codes(N + 3 * K, N, K)
    want = o.gemm_i32_c(cx, cw)
    got = gemm_f6(gpu, cx, cw)
    assert got.dtype == np.int32 and np.array_equal(got.astype(np.int64), want)


def test_seeded_random_shapes(gpu):
    """Twenty seeded shapes (M up to 700, N a multiple of 16 up to 1200, K a multiple of 128 up to 1536) through
    whatever configuration the launch heuristic picks: accumulators bit-exact, nothing written past N."""
    rng = np.random.default_rng(20250605)
    for case in range(20):
        M = int(rng.integers(1, 701))
        N = 16 * int(rng.integers(1, 76))
        K = 128 * int(rng.integers(1, 13))
        print("case", case, M, N, K, flush=True)
        cx, cw = wl.random_codes(1000 + case, M, K), wl.random_codes(2000 + case, N, K)
        got = gemm_f6(gpu, cx, cw, ldy=N + 8)
        assert np.array_equal(got.astype(np.int64), o.gemm_i32_c(cx, cw)), (M, N, K)


@pytest.mark.parametrize("tile", ["61", "63", "64", "65", "66"])
def test_every_tile_configuration(gpu, tile, tune):
    """The launch heuristic picks one configuration per shape; each of them is checked on a shape with
    ragged edges and more tiles than workgroups can hold at once is covered by the full-size test below."""
    tune(gpu.SR_TUNE_GEMM_TILE, tile)
    M, N, K = 700, 1040, 640
    cx, cw = wl.random_codes(1, M, K), wl.random_codes(2, N, K)
    got = gemm_f6(gpu, cx, cw, ldy=1048)
    assert np.array_equal(got.astype(np.int64), o.gemm_i32_c(cx, cw))


@pytest.mark.parametrize("M", [1, 40])
def test_extreme_codes_stay_exact(gpu, M):
    """All codes -8 at the largest K the call accepts: |acc| = 64 K, the largest sum fp32 must hold."""
    for K in (14336, 130944):
        cx = np.full((M, K), -8, np.int8)
        cw = np.full((32, K), -8, np.int8)
        cw[1::2] = 7
        got = gemm_f6(gpu, cx, cw)
        assert np.all(got[:, 0::2] == 64 * K) and np.all(got[:, 1::2] == -56 * K)


@pytest.mark.parametrize("M,N,K", [(16, 512, 512), (200, 528, 1024), (2048, 1024, 4096)])
def test_fp16_epilogue(gpu, M, N, K):
    rng = np.random.default_rng(M * N)
    cx, cw = wl.random_codes(M, M, K), wl.random_codes(N, N, K)
    xs = rng.uniform(0.01, 2.0, M)
    ws = rng.uniform(1e-4, 1e-2, N)
    got = gemm_f6(gpu, cx, cw, xs, ws, gpu.SR_F16, ldy=N + 8)
    want = o.dequant_out(o.gemm_i32_c(cx, cw), xs.astype(np.float32).astype(np.float64),
                         ws.astype(np.float32).astype(np.float64))
    check_output(got, want)


@pytest.mark.parametrize("N", [4096, 14336])
def test_cfg2_full_size_every_accumulator(gpu, N):
    """M = 2048, K = 4096 in the launch configuration the benchmark times: every one of the M x N INT32
    accumulators against the oracle's triple loop, plus two sum identities (row sums against cx . colsum(cw),
    column sums against rowsum(cx) . cw) as an independent cross-check of the comparison itself."""
    M, K = 2048, 4096
    cx, cw = wl.random_codes(21, M, K), wl.random_codes(22 + N, N, K)
    got = gemm_f6(gpu, cx, cw).astype(np.int64)
    assert np.array_equal(got, o.gemm_i32_c(cx, cw))
    assert np.array_equal(got.sum(axis=1), cx.astype(np.int64) @ cw.astype(np.int64).sum(axis=0))
    assert np.array_equal(got.sum(axis=0), cx.astype(np.int64).sum(axis=0) @ cw.astype(np.int64).T)


def test_cfg3_full_size_every_accumulator(gpu):
    M, N, K = 2048, 4096, 14336
    cx, cw = wl.random_codes(31, M, K), wl.random_codes(32, N, K)
    got = gemm_f6(gpu, cx, cw).astype(np.int64)
    assert np.array_equal(got, o.gemm_i32_c(cx, cw))
    assert np.array_equal(got.sum(axis=1), cx.astype(np.int64) @ cw.astype(np.int64).sum(axis=0))


def test_repeatable_bitwise(gpu):
    cx, cw = wl.random_codes(5, 600, 1024), wl.random_codes(6, 784, 1024)
    a = gemm_f6(gpu, cx, cw)
    for _ in range(3):
        assert np.array_equal(gemm_f6(gpu, cx, cw), a)


# ---------------------------------------------------------------- activation quantiser writing tiles

def quant_f6(sr, X, inv_s, clip):
    M, K = X.shape
    inv = None if inv_s is None else torch.from_numpy(inv_s).cuda()
    X6, xs = sr.sr_fwht_quant_act_f6(torch.from_numpy(X).cuda(), inv, clip)
    torch.cuda.synchronize()
    return fc.f6_codes(fc.f6_tiles_unpack(X6.cpu().numpy(), M, K)), xs.cpu().numpy(), X6


@pytest.mark.parametrize("K", [128, 256, 512, 1024, 2048, 4096, 8192, 896, 1792, 3584, 14336])
@pytest.mark.parametrize("M", [1, 13])
def test_quantiser_tiles_every_order(gpu, M, K):
    print("case", M, K, flush=True)
    X = wl.gauss_acts(7, M, K, 3, 200.0)
    inv_s = np.random.default_rng(K).uniform(0.25, 4.0, K).astype(np.float32)
    for clip in (0.9, 1.0):
        codes, xs, _ = quant_f6(gpu, X, inv_s, clip)
        ref = o.fwht_quant_act(X, inv_s, clip)
        check_scales(xs, ref["x_scale"])
        check_codes(codes, ref["codes"], ref["t"])


def test_quantiser_tiles_agree_with_the_nibble_path(gpu):
    """Same rotation, two output formats.  The tile fields are rounded by the hardware FP6 conversion of the
    fp32 product y * (1 / Delta), the nibbles by a fused multiply-add with the rounding constant: each is held to
    the rounding-boundary rule against the oracle, the scales are identical, and the two sets of codes may differ
    only at such boundaries (a handful per million).  K = 4096 runs the two-pass workgroup-per-row kernel, K = 14336
    the general workgroup-per-row kernel."""
    for M, K in ((2048, 4096), (40, 4096), (24, 14336)):
        X = wl.cfg2_X(M, K) if K == 4096 else wl.cfg3_X(M, K)
        inv_s = np.random.default_rng(M).uniform(0.5, 2.0, K).astype(np.float32)
        codes, xs, _ = quant_f6(gpu, X, inv_s, 0.9)
        Xq, xs4 = gpu.sr_fwht_quant_act(torch.from_numpy(X).cuda(), torch.from_numpy(inv_s).cuda(), 0.9)
        torch.cuda.synchronize()
        codes4 = o.unpack_int4(Xq.cpu().numpy())
        assert np.array_equal(xs, xs4.cpu().numpy())
        ref = o.fwht_quant_act(X, inv_s, 0.9)
        check_codes(codes, ref["codes"], ref["t"])
        check_codes(codes4, ref["codes"], ref["t"])
        assert np.count_nonzero(codes != codes4) <= max(2, 1e-5 * codes.size)


@pytest.mark.parametrize("M", [1025, 1030, 1100])
@pytest.mark.parametrize("smooth", [True, False])
def test_quantiser_tiles_ragged_row_counts(gpu, M, smooth):
    """K = 4096 with row counts that leave the last 8-row block and the last 64-row group ragged (the dispatcher's
    own kernel: a workgroup per row in two passes; the other K = 4096 kernels are forced in
    test_every_k4096_kernel): tile fields from the hardware FP6 conversion against the oracle."""
    K = 4096
    X = wl.gauss_acts(11 + M, M, K, 5, 300.0)
    inv_s = np.random.default_rng(M).uniform(0.25, 4.0, K).astype(np.float32) if smooth else None
    for clip in (0.9, 1.0, 0.6):
        codes, xs, _ = quant_f6(gpu, X, inv_s, clip)
        ref = o.fwht_quant_act(X, inv_s, clip)
        check_scales(xs, ref["x_scale"])
        check_codes(codes, ref["codes"], ref["t"])
        assert codes.min() >= -8 and codes.max() <= 7


# K = 4096 has four kernels; the knob forces each one on row counts on both sides of the dispatcher's switch
# (1 = a wave per row with the factors staged in LDS, 4 = a wave per row with per-lane factor loads,
#  2 = the general workgroup-per-row kernel, 5 = a workgroup of four waves per row in two passes of six bits).
@pytest.mark.parametrize("kernel", [1, 4, 2, 5])
@pytest.mark.parametrize("M", [1, 7, 64, 300, 1030, 2048, 3080])
def test_every_k4096_kernel(gpu, tune, kernel, M):
    """Tiles and nibbles of every K = 4096 kernel against the oracle (scales to 1e-6, codes under the boundary rule),
    with and without factors, with a padded leading dimension, and with the cache-warming hint (outputs unchanged).
    The rotations differ in the order of their fp32 additions, so the kernels are held to the oracle, not to each
    other; only the two output formats of ONE kernel share a rotation: identical scales."""
    print("case", kernel, M, flush=True)
    K = 4096
    tune(gpu.SR_TUNE_FWHT4096, kernel)
    X = wl.gauss_acts(500 + M, M, K, 5, 300.0)
    rng = np.random.default_rng(M)
    for inv_s in (rng.uniform(0.25, 4.0, K).astype(np.float32), None):
        ref = o.fwht_quant_act(X, inv_s, 0.9)
        inv = None if inv_s is None else torch.from_numpy(inv_s).cuda()
        buf = torch.zeros((M, K + 24), dtype=torch.float16, device="cuda")
        buf[:, :K] = torch.from_numpy(X).cuda()
        for Xd in (torch.from_numpy(X).cuda(), buf[:, :K]):
            X6, xs6 = gpu.sr_fwht_quant_act_f6(Xd, inv, 0.9)
            Xq, xs4 = gpu.sr_fwht_quant_act(Xd, inv, 0.9)
            torch.cuda.synchronize()
            codes6 = fc.f6_codes(fc.f6_tiles_unpack(X6.cpu().numpy(), M, K))
            codes4 = o.unpack_int4(Xq.cpu().numpy())
            check_scales(xs6.cpu().numpy(), ref["x_scale"])
            assert torch.equal(xs6, xs4)
            check_codes(codes6, ref["codes"], ref["t"], "tiles, kernel %d" % kernel)
            check_codes(codes4, ref["codes"], ref["t"], "nibbles, kernel %d" % kernel)
        region = torch.randint(0, 255, (3 * 1024 * 1024 + 52,), dtype=torch.uint8, device="cuda")
        X6w, xsw = gpu.sr_fwht_quant_act_f6(torch.from_numpy(X).cuda(), inv, 0.9, warm=region)
        X6p, xsp = gpu.sr_fwht_quant_act_f6(torch.from_numpy(X).cuda(), inv, 0.9)
        torch.cuda.synchronize()
        assert torch.equal(X6w, X6p) and torch.equal(xsw, xsp)
    Z = np.zeros((M, K), np.float16)                                     # all-zero rows: Delta = 1, codes 0
    X6, xs = gpu.sr_fwht_quant_act_f6(torch.from_numpy(Z).cuda(), None, 0.9)
    torch.cuda.synchronize()
    assert bool((xs == 1.0).all()) and not fc.f6_codes(fc.f6_tiles_unpack(X6.cpu().numpy(), M, K)).any()


@pytest.mark.parametrize("M,K", [(13, 512), (1027, 4096), (33, 14336)])
def test_padding_rows_of_the_activation_tiles_cannot_leak(gpu, M, K):
    """The quantiser leaves the rows that pad the last block of 8 unwritten, so the GEMM multiplies whatever the
    buffer held there.  With the tile buffer pre-filled with 0xFF (the 6-bit pattern 63 = -7.5 in every field, the
    largest magnitude the format has) both outputs must be exactly what they are on a zero-filled buffer, and
    nothing beyond row M - 1 of a larger output may be written."""
    X = wl.gauss_acts(3 + M, M, K, 3, 200.0)
    inv_s = np.random.default_rng(K + M).uniform(0.25, 4.0, K).astype(np.float32)
    Xd, inv = torch.from_numpy(X).cuda(), torch.from_numpy(inv_s).cuda()
    N = 272
    W6 = tiles(gpu, wl.random_codes(5 + K, N, K))
    ws = torch.from_numpy(np.random.default_rng(1).uniform(1e-3, 2e-3, N).astype(np.float32)).cuda()
    outs = []
    for fill in (0x00, 0xFF):
        X6 = torch.full((gpu.sr_f6_tiles_bytes(M, K),), fill, dtype=torch.uint8, device="cuda")
        X6, xs = gpu.sr_fwht_quant_act_f6(Xd, inv, 0.9, X6=X6)
        acc = torch.full((M + 9, N), -7, dtype=torch.int32, device="cuda")
        Y = torch.full((M + 9, N), -7.0, dtype=torch.float16, device="cuda")
        gpu.sr_w4a4_gemm_f6(X6, None, W6, None, M, N, K, gpu.SR_I32, acc[:M])
        gpu.sr_w4a4_gemm_f6(X6, xs, W6, ws, M, N, K, gpu.SR_F16, Y[:M])
        torch.cuda.synchronize()
        assert bool((acc[M:] == -7).all()) and bool((Y[M:] == -7.0).all())
        assert bool(torch.isfinite(Y[:M]).all())
        outs.append((acc[:M].clone(), Y[:M].clone(), xs.clone()))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


@pytest.mark.parametrize("M,K", [(1100, 4096), (2048, 4096), (40, 4096), (64, 14336), (300, 14336), (1100, 14336), (600, 7168)])
def test_cache_warming_changes_nothing(gpu, M, K):
    """sr_fwht_quant_act_f6_warm reads, on the side, the lines of the operand that the next call will stream
    (here a weight matrix in f6 tiles; also a region shorter than one line and one with a ragged tail): tiles
    and scales must be exactly those of sr_fwht_quant_act_f6, the operand untouched, and the GEMM on it as
    before -- for the kernels that honour the hint (the wave-per-row kernel, the workgroup-per-row kernel from
    256 rows on, also where its workgroups walk over rows) and for the launches that ignore it."""
    X = wl.gauss_acts(41 + M, M, K, 4, 250.0)
    inv_s = np.random.default_rng(M).uniform(0.25, 4.0, K).astype(np.float32)
    Xd, inv = torch.from_numpy(X).cuda(), torch.from_numpy(inv_s).cuda()
    N = 272
    cw = wl.random_codes(7 + K, N, K)
    W6 = tiles(gpu, cw)
    W6_before = W6.clone()
    X6a, xsa = gpu.sr_fwht_quant_act_f6(Xd, inv, 0.9)
    for region in (W6, W6[:100], W6[: 128 * 37 + 52], W6[:0]):
        X6b, xsb = gpu.sr_fwht_quant_act_f6(Xd, inv, 0.9, warm=region if region.numel() else None)
        torch.cuda.synchronize()
        assert torch.equal(X6a, X6b) and torch.equal(xsa, xsb)
    assert torch.equal(W6, W6_before)
    ws = torch.full((N,), 1e-3, device="cuda")
    Ya = gpu.sr_w4a4_gemm_f6(X6a, xsa, W6, ws, M, N, K, gpu.SR_I32)
    X6b, xsb = gpu.sr_fwht_quant_act_f6(Xd, inv, 0.9, warm=W6)
    Yb = gpu.sr_w4a4_gemm_f6(X6b, xsb, W6, ws, M, N, K, gpu.SR_I32)
    torch.cuda.synchronize()
    assert torch.equal(Ya, Yb)


@pytest.mark.parametrize("M,N,K,grid", [(2048, 4096, 4096, None), (700, 1040, 640, None), (700, 1040, 640, 8), (300, 528, 1024, 16),
                                          (1, 16, 128, None), (2048, 14336, 4096, None)])
def test_gemm_cache_warming_changes_nothing(gpu, tune, M, N, K, grid):
    """sr_w4a4_gemm_f6_warm: where the 256 x 128 tile configuration runs (forced here except for the two full-size
    shapes, where the dispatcher's own choice is taken: N = 4096 honours the hint, N = 14336 ignores it) a ninth
    wave per workgroup reads the hinted region and joins every barrier of the tile loop -- one tile per workgroup,
    several tiles per workgroup (small forced grids: the barrier between tiles), regions shorter than a line, with a
    ragged tail, larger than the workgroups' first sweep.  Accumulators and fp16 outputs must be exactly those of
    sr_w4a4_gemm_f6, the region untouched, nothing written past the outputs; the knob that switches the hint off
    gives the same again."""
    print("case", M, N, K, grid, flush=True)
    if (M, N) != (2048, 4096) and (M, N) != (2048, 14336):
        tune(gpu.SR_TUNE_GEMM_TILE, 65)
    if grid:
        tune(gpu.SR_TUNE_GEMM_GRID, grid)
    cx, cw = wl.random_codes(51 + M, M, K), wl.random_codes(52 + N, N, K)
    X6, W6 = tiles(gpu, cx), tiles(gpu, cw)
    rng = np.random.default_rng(N)
    xs = torch.from_numpy((np.exp(rng.standard_normal(M) * 0.5) * 0.05).astype(np.float32)).cuda()
    ws = torch.from_numpy((np.exp(rng.standard_normal(N) * 0.3) * 1e-3).astype(np.float32)).cuda()
    acc0 = gpu.sr_w4a4_gemm_f6(X6, None, W6, None, M, N, K, gpu.SR_I32)
    Y0 = gpu.sr_w4a4_gemm_f6(X6, xs, W6, ws, M, N, K, gpu.SR_F16)
    torch.cuda.synchronize()
    assert np.array_equal(acc0.cpu().numpy().astype(np.int64), o.gemm_i32_c(cx, cw))
    big = torch.randint(0, 255, (5 * 1024 * 1024 + 52,), dtype=torch.uint8, device="cuda")
    big_before = big.clone()
    for region in (big, big[:100], big[: 128 * 37 + 52], big[: 64 * 128 * 300 + 128], W6):
        acc = torch.full((M + 3, N + 8), -7, dtype=torch.int32, device="cuda")
        Y = torch.full((M + 3, N + 8), -7.0, dtype=torch.float16, device="cuda")
        gpu.sr_w4a4_gemm_f6_warm(X6, None, W6, None, M, N, K, region, gpu.SR_I32, acc[:M, :N])
        gpu.sr_w4a4_gemm_f6_warm(X6, xs, W6, ws, M, N, K, region, gpu.SR_F16, Y[:M, :N])
        torch.cuda.synchronize()
        assert torch.equal(acc[:M, :N], acc0) and torch.equal(Y[:M, :N], Y0)
        assert bool((acc[M:] == -7).all()) and bool((acc[:, N:] == -7).all())
        assert bool((Y[M:] == -7.0).all()) and bool((Y[:, N:] == -7.0).all())
    assert torch.equal(big, big_before)
    tune(gpu.SR_TUNE_GEMM_WARM, 0)
    assert torch.equal(gpu.sr_w4a4_gemm_f6_warm(X6, xs, W6, ws, M, N, K, big), Y0)


@pytest.mark.parametrize("M", [700, 1100])
def test_row_kernel_walking_over_rows(gpu, tune, M):
    """K = 14336 with many rows: as many workgroups as the chip holds, each walking over several rows and
    fetching its next row while it works (forced here at a row count that leaves workgroups with one, two or
    three rows and a ragged last tile block).  Same arithmetic as one workgroup per row: every output must
    equal that launch's bit for bit, and the oracle's under the boundary rule."""
    K = 14336
    X = wl.gauss_acts(31 + M, M, K, 3, 300.0)
    inv_s = np.random.default_rng(M).uniform(0.5, 2.0, K).astype(np.float32)
    Xd, inv = torch.from_numpy(X).cuda(), torch.from_numpy(inv_s).cuda()

    def run_all():
        outs = []
        for pre in (inv, None):
            outs += list(gpu.sr_fwht_quant_act_f6(Xd, pre, 0.9))
            outs += list(gpu.sr_fwht_quant_act(Xd, pre, 0.9))
        torch.cuda.synchronize()
        return [t.cpu().numpy() for t in outs]

    tune(gpu.SR_TUNE_FWHT_STREAM, 0)
    one = run_all()
    tune(gpu.SR_TUNE_FWHT_STREAM, 1)
    walk = run_all()
    for a, b in zip(one, walk):
        assert np.array_equal(a, b)
    ref = o.fwht_quant_act(X, inv_s, 0.9)
    check_scales(walk[1], ref["x_scale"])
    check_codes(fc.f6_codes(fc.f6_tiles_unpack(walk[0], M, K)), ref["codes"], ref["t"])
    check_codes(o.unpack_int4(walk[2]), ref["codes"], ref["t"])
    ref = o.fwht_quant_act(X, None, 0.9)
    check_scales(walk[5], ref["x_scale"])
    check_codes(fc.f6_codes(fc.f6_tiles_unpack(walk[4], M, K)), ref["codes"], ref["t"])
    check_codes(o.unpack_int4(walk[6]), ref["codes"], ref["t"])


@pytest.mark.parametrize("M,K", [(5, 896), (24, 14336), (9, 4096)])
def test_gated_prologue_tiles(gpu, M, K):
    """silu(gate) * up fused in front of the rotation, tile output: codes under the boundary rule against the
    oracle; same scales as the nibble output of the same kernel, codes apart only at rounding boundaries."""
    G, U = wl.gate_up(3, M, K, 2, 300.0)
    inv_s = np.random.default_rng(K + M).uniform(0.5, 2.0, K).astype(np.float32)
    Gd, Ud, inv_d = torch.from_numpy(G).cuda(), torch.from_numpy(U).cuda(), torch.from_numpy(inv_s).cuda()
    X6, xs = gpu.sr_swiglu_fwht_quant_act_f6(Gd, Ud, inv_d, 0.9)
    Xq, xs4 = gpu.sr_swiglu_fwht_quant_act(Gd, Ud, inv_d, 0.9)
    torch.cuda.synchronize()
    codes = fc.f6_codes(fc.f6_tiles_unpack(X6.cpu().numpy(), M, K))
    ref = o.fwht_quant_swiglu(G, U, inv_s, 0.9)
    check_scales(xs.cpu().numpy(), ref["x_scale"])
    check_codes(codes, ref["codes"], ref["t"])
    codes4 = o.unpack_int4(Xq.cpu().numpy())
    check_codes(codes4, ref["codes"], ref["t"])
    assert np.count_nonzero(codes != codes4) <= max(2, 1e-5 * codes.size) and np.array_equal(xs.cpu().numpy(), xs4.cpu().numpy())


def test_cfg2_layer_through_the_f6_path(gpu):
    """Config 2 (M = 2048, K = 4096 -> N = 4096) end to end through the tile path, stage by stage: each
    stage's oracle runs on the GPU's own (already checked) output of the stage before."""
    M, K, N = 2048, 4096, 4096
    X, W = wl.cfg2_X(M, K), wl.cfg2_W(N, K)
    a = np.zeros(K)
    for i in range(2):
        a = o.calib_absmax(wl.cfg2_calib_chunk(i, 256, K), a)
    a_d = torch.from_numpy(a.astype(np.float32)).cuda()
    Wq, ws, inv_s = gpu.sr_fold_smooth_rotate_quant(torch.from_numpy(W).cuda(), a_d, 0.5, 1.0)
    W6 = gpu.sr_pack_f6_tiles(Wq)
    X6, xs = gpu.sr_fwht_quant_act_f6(torch.from_numpy(X).cuda(), inv_s, 0.9)
    Y = gpu.sr_w4a4_gemm_f6(X6, xs, W6, ws, M, N, K, gpu.SR_F16)
    acc = gpu.sr_w4a4_gemm_f6(X6, None, W6, None, M, N, K, gpu.SR_I32)
    torch.cuda.synchronize()
    cw = o.unpack_int4(Wq.cpu().numpy())
    assert np.array_equal(fc.f6_codes(fc.f6_tiles_unpack(W6.cpu().numpy(), N, K)), cw)
    ref = o.fwht_quant_act(X, inv_s.cpu().numpy(), 0.9)
    cx = fc.f6_codes(fc.f6_tiles_unpack(X6.cpu().numpy(), M, K))
    check_scales(xs.cpu().numpy(), ref["x_scale"])
    check_codes(cx, ref["codes"], ref["t"])
    rows = np.unique(np.r_[0:4, 1000:1003, M - 4:M])
    want = o.gemm_i32_c(cx[rows], cw)
    assert np.array_equal(acc.cpu().numpy().astype(np.int64)[rows], want)
    check_output(Y.cpu().numpy()[rows], o.dequant_out(want, xs.cpu().numpy().astype(np.float64)[rows],
                                                      ws.cpu().numpy().astype(np.float64)))
