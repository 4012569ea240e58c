"""The measurement kernels behind bench.py's "measured ceilings": they compute nothing that could be compared with
the oracle; what is checked is that every launch shape bench.py uses is accepted, runs to completion, leaves its
input untouched, and that bad arguments are refused on the host."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_ceiling_kernels_run_and_leave_their_inputs_alone(gpu):
    src = torch.randint(0, 256, (3 * 1024 * 1024 + 16 * 37,), dtype=torch.uint8, device="cuda")
    before = src.clone()
    for grid, block, fl, nt in ((2048, 256, 8, True), (1024, 512, 8, True), (2048, 256, 16, True), (4096, 256, 4, True),
                                (2048, 256, 8, False), (7168, 256, 4, True), (1, 64, 1, False), (3, 1024, 2, True)):
        gpu.sr_ceiling_hbm_read(src, grid, block, fl, nt)
    dst = torch.zeros(700 * 1536, dtype=torch.uint8, device="cuda")
    gpu.sr_ceiling_row_stream(src[:700 * 4096], dst, 700, 4096, 1536, 512, 70 * 1024)      # rows in, "codes" out
    gpu.sr_ceiling_row_stream(src[:100 * 28672], dst, 100, 28672, 10752, 37, 1024)
    assert gpu.sr_ceiling_mfma_f6(src, 5, 256) == 256 * 8 * 5 * 8 * 2.0 * 32 * 32 * 64
    assert gpu.sr_ceiling_mfma_i8(src, 5, 256) == 256 * 8 * 5 * 8 * 2.0 * 32 * 32 * 32
    assert gpu.sr_ceiling_valu_f32(4, 512) == 512 * 4 * 4 * 192.0
    torch.cuda.synchronize()
    assert torch.equal(src, before)


def test_ceiling_kernels_refuse_bad_arguments(gpu):
    r = gpu.raw()
    A = 0x1000
    assert r.sr_ceiling_hbm_read(None, 1024, 8, 256, 8, 1, None, None) == gpu.SR_ERR_NULL
    assert r.sr_ceiling_hbm_read(A, 1000, 8, 256, 8, 1, None, None) == gpu.SR_ERR_ALIGN
    assert r.sr_ceiling_hbm_read(A + 4, 1024, 8, 256, 8, 1, None, None) == gpu.SR_ERR_ALIGN
    for bad in ((0, 256, 8), (8, 100, 8), (8, 2048, 8), (8, 256, 3)):
        assert r.sr_ceiling_hbm_read(A, 1024, bad[0], bad[1], bad[2], 1, None, None) == gpu.SR_ERR_ARG
    assert r.sr_ceiling_mfma_f6(A, 100, 5, 256, None, None) == gpu.SR_ERR_ARG      # operand buffer too small
    assert r.sr_ceiling_mfma_i8(A, 100, 5, 256, None, None) == gpu.SR_ERR_ARG
    assert r.sr_ceiling_mfma_f6(None, 9216, 5, 256, None, None) == gpu.SR_ERR_NULL
    assert r.sr_ceiling_valu_f32(0, 512, None, None) == gpu.SR_ERR_ARG
