"""The library only enqueues kernels on the stream it is handed and keeps no state between calls.  So the
same calls issued on two streams at once, and the same calls replayed from a captured HIP graph, must give
what plain serial calls on the default stream give -- bit for bit (every kernel here is deterministic: integer
sums, order-free maxima, one rounding per output).

One "pass" below = the hot path on the FP6 pipe (rotate + quantise to tiles, GEMM), the canonical nibble
quantiser, a decode GEMM (M = 16: the streaming kernel with its dynamic LDS), the one-launch decode call,
the KV-cache quantiser and the calibration maximum (atomics)."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu

M, K, N = 300, 4096, 2048
KV_ROWS, KV_D = 512, 1024


def make_weights(sr):
    g = torch.Generator(device="cpu").manual_seed(5)
    Wq = torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, generator=g).cuda()     # any byte is two valid codes
    ws = (torch.rand(N, generator=g) * 0.01 + 0.001).cuda()
    inv_s = (torch.rand(K, generator=g) * 1.5 + 0.5).cuda()
    W6 = sr.sr_pack_f6_tiles(Wq)
    torch.cuda.synchronize()
    return {"Wq": Wq, "ws": ws, "inv_s": inv_s, "W6": W6}


def make_inputs(seed):
    X = torch.from_numpy(wl.gauss_acts(seed, M, K, 4, 200.0)).cuda()
    kv = torch.from_numpy(wl.kv_acts(seed, KV_ROWS, KV_D)).cuda()
    return {"X": X, "kv": kv}


def make_outputs(sr):
    dev = "cuda"
    return {
        "X6": torch.zeros(sr.sr_f6_tiles_bytes(M, K), dtype=torch.uint8, device=dev),
        "xs": torch.zeros(M, device=dev),
        "Y": torch.zeros((M, N), dtype=torch.float16, device=dev),
        "Xq": torch.zeros((M, K // 2), dtype=torch.uint8, device=dev),
        "xs4": torch.zeros(M, device=dev),
        "Yd": torch.zeros((16, N), dtype=torch.float16, device=dev),
        "Y1": torch.zeros((1, N), dtype=torch.float16, device=dev),
        "kq": torch.zeros((KV_ROWS, KV_D // 2), dtype=torch.uint8, device=dev),
        "ks": torch.zeros((KV_ROWS, KV_D // 128), device=dev),
        "kz": torch.zeros((KV_ROWS, KV_D // 128), device=dev),
        "amax": torch.zeros(K, device=dev),
    }


def one_pass(sr, w, inp, out):
    sr.sr_fwht_quant_act_f6(inp["X"], w["inv_s"], 0.9, out["X6"], out["xs"], warm=w["W6"])   # with the cache-warming hint
    # (256 x 128 tiles at this shape: the launch with the extra wave that reads the hinted region)
    sr.sr_w4a4_gemm_f6(out["X6"], out["xs"], w["W6"], w["ws"], M, N, K, sr.SR_F16, out["Y"], warm=w["Wq"])
    sr.sr_fwht_quant_act(inp["X"], w["inv_s"], 0.9, out["Xq"], out["xs4"])
    sr.sr_w4a4_gemm(out["Xq"][:16], out["xs4"][:16], w["Wq"], w["ws"], sr.SR_F16, out["Yd"])
    sr.sr_w4a4_linear_decode(inp["X"][:1], w["inv_s"], w["Wq"], w["ws"], 0.9, out["Y1"])
    sr.sr_kv_quant_asym(inp["kv"], 128, 0.95, out["kq"], out["ks"], out["kz"])
    out["amax"].zero_()                                   # a fill kernel
    sr.sr_calib_absmax(inp["X"], out["amax"])


def snapshot(out):
    torch.cuda.synchronize()
    return {k: v.clone() for k, v in out.items()}


def assert_same(got, want, what):
    for k in want:
        assert torch.equal(got[k], want[k]), (what, k)


def test_two_streams_at_once(gpu):
    assert gpu.sr_gemm_workspace_bytes(16, N, K) == 0        # the decode GEMM takes no workspace
    w = make_weights(gpu)
    inputs = [make_inputs(40), make_inputs(41)]
    want = []
    for inp in inputs:
        out = make_outputs(gpu)
        one_pass(gpu, w, inp, out)
        want.append(snapshot(out))
    assert not torch.equal(want[0]["Y"], want[1]["Y"])

    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [make_outputs(gpu), make_outputs(gpu)]
    torch.cuda.synchronize()
    for _ in range(3):                                       # alternate, so that the two queues really overlap
        for s, inp, out in zip(streams, inputs, outs):
            with torch.cuda.stream(s):
                one_pass(gpu, w, inp, out)
    for s in streams:
        s.synchronize()
    for i in range(2):
        assert_same(snapshot(outs[i]), want[i], "stream %d" % i)


def test_graph_replays(gpu):
    w = make_weights(gpu)
    inputs = [make_inputs(50 + r) for r in range(3)]
    want = []
    for inp in inputs:
        out = make_outputs(gpu)
        one_pass(gpu, w, inp, out)
        want.append(snapshot(out))

    static_in = {k: v.clone() for k, v in inputs[0].items()}
    static_out = make_outputs(gpu)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                            # warm-up outside the capture (function attributes, lazy loads)
        one_pass(gpu, w, static_in, static_out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        one_pass(gpu, w, static_in, static_out)
    torch.cuda.synchronize()

    scratch_out = make_outputs(gpu)
    for rnd in range(2):
        for r, inp in enumerate(inputs):
            for k in static_in:
                static_in[k].copy_(inp[k])
            one_pass(gpu, w, inputs[(r + 1) % 3], scratch_out)   # eager work of the same kernels between replays
            torch.cuda.synchronize()
            g.replay()
            assert_same(snapshot(static_out), want[r], "replay %d.%d" % (rnd, r))
