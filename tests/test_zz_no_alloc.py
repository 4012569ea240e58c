"""The fold entry point that allocates nothing (device-resident scratch) against the workspace one: identical
bytes on two calls in a row, the second on a smaller weight (the array keeps the first call's contents), and the
size limit."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


def fold_both(gpu, W, a, alpha, clip):
    Wd = torch.from_numpy(W).cuda()
    ad = None if a is None else torch.from_numpy(a.astype(np.float32)).cuda()
    K, N = W.shape
    ref = gpu.sr_fold_smooth_rotate_quant(Wd, ad, alpha, clip)
    # outputs pre-filled with a pattern, so that an entry point that launched nothing cannot pass
    Wq = torch.full((N, K // 2), 0xA5, dtype=torch.uint8, device="cuda")
    ws = torch.full((N,), -1.0, dtype=torch.float32, device="cuda")
    inv = torch.full((K,), -1.0, dtype=torch.float32, device="cuda")
    before = torch.cuda.memory_allocated()
    gpu.sr_fold_smooth_rotate_quant_noalloc(Wd, ad, alpha, clip, Wq, ws, inv)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    for got, want, what in zip((Wq, ws, inv), ref, ("codes", "scales", "inv_s")):
        assert torch.equal(got, want), what


def test_two_calls_in_a_row_second_smaller(gpu):
    rng = np.random.default_rng(5)
    W1 = wl.cfg2_W(4096)                                   # 4096 x 4096: the whole array is used
    a1 = np.abs(rng.standard_normal(4096)) * 3 + 0.1
    fold_both(gpu, W1, a1, 0.5, 1.0)
    W2 = wl.to_f16_sat(rng.standard_normal((896, 272)).astype(np.float32) * 0.02)   # smaller, Kronecker order, ragged N
    a2 = np.abs(rng.standard_normal(896)) + 0.1
    fold_both(gpu, W2, a2, 0.3, 0.9)
    fold_both(gpu, W2, None, 0.5, 1.0)                     # rotation only (s = 1): the maxima vector is not written


def test_size_limit_and_argument_errors(gpu):
    f = gpu.raw().sr_fold_smooth_rotate_quant_noalloc
    A = 0x1000
    assert gpu.sr_noalloc_scratch_bytes() >= gpu.sr_fold_workspace_bytes(4096, 4096)
    assert gpu.sr_fold_workspace_bytes(4096, 14336) > gpu.sr_noalloc_scratch_bytes()
    assert f(A, 4096, 14336, 14336, A, 0.5, 1.0, A, A, A, None) == gpu.SR_ERR_WORKSPACE
    assert f(A, 4096, 4160, 4160, A, 0.5, 1.0, A, A, A, None) == gpu.SR_ERR_WORKSPACE
    assert f(A, 500, 64, 64, A, 0.5, 1.0, A, A, A, None) == gpu.SR_ERR_UNSUPPORTED_K
    assert f(None, 512, 64, 64, A, 0.5, 1.0, A, A, A, None) == gpu.SR_ERR_NULL
