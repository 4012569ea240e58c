#!/usr/bin/env python3
"""Benchmark of the SmoothRot W4A4 linear hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One "step" = the online hot path of the two prefill linears of the benchmark
configuration (X fp16 [2048, 4096]; W [4096, 4096] and W [4096, 14336]):
    sr_fwht_quant_act_f6_warm(X) -> sr_w4a4_gemm_f6(N = 4096)
    sr_fwht_quant_act_f6_warm(X) -> sr_w4a4_gemm_f6(N = 14336)
(rotation + per-token INT4 quantiser writing the codes as f6 tiles -- its launch also pulls the weights of the
GEMM behind it into the memory-side cache --, then the INT4 x INT4 GEMM on the FP6 matrix pipe, which
multiplies the codes exactly; weights are repacked to f6 tiles once, offline).
The same GEMMs through the int8-MFMA kernel (sr_w4a4_gemm) are timed under "extra".
Inputs are resident in HBM; the step rotates over several distinct input / weight
sets so that no call finds its operands in the 256 MB Infinity Cache.
The offline rows (calibration absmax, weight fold) and the decode shapes are
timed separately and reported in the same JSON line under "extra".
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0      # MI355X dense int8 MFMA, TOP/s
PEAK_FP6_TOPS = 10100.0      # MI355X dense fp6 / fp4 MFMA, TFLOP/s (the instruction the fast GEMM issues)
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E, GB/s

M, K = 2048, 4096
NS = (4096, 14336)
CLIP, ALPHA = 0.9, 0.5
SETS = 8                     # distinct (X, Wq) sets rotated through: 8 * (16.8 + 37.7) MB > 256 MB


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults: 0.14 s of timed work after 25 ms of warm-up (the first hundreds of steps run up to 2 % slower
    # while the clocks settle: 1000 steps after 20 / 200 / 1000 warm-up steps gave 0.1142 / 0.1137 / 0.1128 ms)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the decode / offline side measurements")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2506_05413_amd as sr
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    # ---------------- offline preparation (timed separately) -----------------------------
    calib = [torch.from_numpy(wl.cfg2_calib_chunk(i)).to(dev) for i in range(16)]   # 16 x 16.8 MB = 268 MB
    absmax = torch.zeros(K, dtype=torch.float32, device=dev)
    for c in calib:
        sr.sr_calib_absmax(c, absmax)
    torch.cuda.synchronize()

    def ev_time(fn, iters):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / iters        # seconds per call

    def graph_time(fn, iters, reps=3):
        """Seconds per call with the `iters` calls captured in one HIP graph (no host launch cost between
        kernels); the library only launches kernels, so the capture holds kernel nodes only."""
        fn(0)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(iters):
                fn(i)
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / (iters * reps)

    extra = {"note": "per-kernel figures below are timed from a captured HIP graph (no host launch gaps)"}
    scratch = torch.zeros(K, dtype=torch.float32, device=dev)
    if not args.no_extra:
        for _ in range(2):
            t = graph_time(lambda i: sr.sr_calib_absmax(calib[i % 16], scratch), 32)
        extra["calib_absmax"] = {"GB/s": round(M * K * 2 / t / 1e9, 1), "us": round(t * 1e6, 2),
                                 "frac_hbm": round(M * K * 2 / t / 1e9 / PEAK_HBM_GBS, 4),
                                 "workload": "fp16 [2048,4096] chunks, 16 distinct (268 MB)"}
        # the same kernel on the calibration batch of config 5 (16384 tokens in one call): eight buffers of
        # 134 MB (the chunks above in eight different orders: 1 GB, well beyond the Infinity Cache)
        big = [torch.cat([calib[(h + 2 * j) % 16] for j in range(8)]) for h in range(8)]
        for _ in range(2):
            t = graph_time(lambda i: sr.sr_calib_absmax(big[i % 8], scratch), 16)
        extra["calib_absmax_T16384"] = {"GB/s": round(8 * M * K * 2 / t / 1e9, 1), "us": round(t * 1e6, 2),
                                        "frac_hbm": round(8 * M * K * 2 / t / 1e9 / PEAK_HBM_GBS, 4),
                                        "workload": "fp16 [16384,4096] per call, 8 distinct (1.07 GB)"}
        del big

    Xs = [torch.from_numpy(wl.cfg2_X(seed=1 + 10 * s)).to(dev) for s in range(SETS)]
    Wq, Ws, W6, inv_s_of = {}, {}, {}, {}
    for N in NS:
        W = torch.from_numpy(wl.cfg2_W(N)).to(dev)
        ws_bytes = sr.sr_fold_workspace_bytes(K, N)
        work = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        outs = sr.sr_fold_smooth_rotate_quant(W, absmax, ALPHA, 1.0, workspace=work)
        torch.cuda.synchronize()
        if not args.no_extra:
            t = ev_time(lambda i: sr.sr_fold_smooth_rotate_quant(W, absmax, ALPHA, 1.0, *outs, workspace=work), 5)
            extra["fold_N%d" % N] = {"us": round(t * 1e6, 1), "GB/s": round((K * N * 2.5) / t / 1e9, 1)}
        # weight sets: the same codes rolled along N, so every set is a distinct buffer with identical statistics
        Wq[N] = [torch.roll(outs[0], s * 16, 0).contiguous() for s in range(SETS)]
        Ws[N] = [torch.roll(outs[1], s * 16, 0).contiguous() for s in range(SETS)]
        W6[N] = [sr.sr_pack_f6_tiles(w) for w in Wq[N]]                   # offline: weights as f6 tiles
        if not args.no_extra:
            t6 = torch.empty_like(W6[N][0])
            t = graph_time(lambda i: sr.sr_pack_f6_tiles(Wq[N][i % SETS], t6), 16)
            extra["pack_f6_tiles_N%d" % N] = {"us": round(t * 1e6, 1), "GB/s": round((K * N * 1.25) / t / 1e9, 1)}
            del t6
        inv_s_of[N] = outs[2]                    # every linear has its own smoothing factors
        del W, work
    inv_s = inv_s_of[NS[-1]]                     # (the side measurements below use one of them)

    Xq = torch.empty((M, K // 2), dtype=torch.uint8, device=dev)
    X6 = torch.zeros(sr.sr_f6_tiles_bytes(M, K), dtype=torch.uint8, device=dev)
    xs = torch.empty(M, dtype=torch.float32, device=dev)
    Y = {N: torch.empty((M, N), dtype=torch.float16, device=dev) for N in NS}

    def step(i):
        s = i % SETS
        for N in NS:
            sr.sr_fwht_quant_act_f6(Xs[s], inv_s_of[N], CLIP, X6, xs, warm=W6[N][s])
            sr.sr_w4a4_gemm_f6(X6, xs, W6[N][s], Ws[N][s], M, N, K, sr.SR_F16, Y[N])

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---------------- timed region: exactly `steps` steps -------------------------------
    # HIP events bracket the dominant kernel (the N = 14336 GEMM), on the stream it runs on,
    # on every eleventh step (an event pair costs the stream a microsecond or two, which is inside the timed region;
    # 11 is coprime with the 8 input sets, so the samples walk over all of them)
    EV_EVERY = 11
    gemm_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range((args.steps + EV_EVERY - 1) // EV_EVERY)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        s = i % SETS
        # each rotation + quantiser call also warms the memory-side cache with the weights of the GEMM behind it
        sr.sr_fwht_quant_act_f6(Xs[s], inv_s_of[4096], CLIP, X6, xs, warm=W6[4096][s])
        sr.sr_w4a4_gemm_f6(X6, xs, W6[4096][s], Ws[4096][s], M, 4096, K, sr.SR_F16, Y[4096])
        sr.sr_fwht_quant_act_f6(Xs[s], inv_s_of[14336], CLIP, X6, xs, warm=W6[14336][s])
        if i % EV_EVERY == 0:
            gemm_ev[i // EV_EVERY][0].record()
        sr.sr_w4a4_gemm_f6(X6, xs, W6[14336][s], Ws[14336][s], M, 14336, K, sr.SR_F16, Y[14336])
        if i % EV_EVERY == 0:
            gemm_ev[i // EV_EVERY][1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    ops_per_step = sum(2.0 * M * N * K for N in NS)
    tops = ops_per_step / (dt / args.steps) / 1e12
    gemm_ms = sorted(a.elapsed_time(b) for a, b in gemm_ev)
    gemm_avg_s = sum(gemm_ms) / len(gemm_ms) * 1e-3
    gemm_ops = 2.0 * M * 14336 * K
    # HBM bytes per launch of this kernel: FETCH_SIZE + WRITE_SIZE from two rocprofv3 --pmc runs of this same
    # command, scaled by the copy-kernel factors (profiles/bench_prefill_cfg2_hbm_traffic.md); algorithmic bytes =
    # X6 6.3 MB + W6 44.0 MB read + Y 58.7 MB written
    # The kernel issues FP6 (E2M3) matrix instructions, so its roofline is the chip's dense fp6 peak; the
    # benchmark's own yardstick (fraction of the int8-MFMA peak, the rate a 4-bit integer GEMM is usually priced
    # at) is reported beside it.
    roofline = {"bound": "mfma", "kernel": "sr_w4a4_gemm_f6: gemm_f6_kernel, M=2048 N=14336 K=4096",
                "achieved": round(gemm_ops / gemm_avg_s / 1e12, 2), "peak": PEAK_FP6_TOPS, "unit": "TFLOP/s",
                "frac": round(gemm_ops / gemm_avg_s / 1e12 / PEAK_FP6_TOPS, 4),
                "frac_int8_mfma_peak": round(gemm_ops / gemm_avg_s / 1e12 / PEAK_INT8_TOPS, 4),
                "traffic": {"hbm_bytes_per_launch": 197.5e6, "algorithmic_bytes": 109.0e6,
                            "source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, see profiles/"},
                "avg_launch_us": round(gemm_avg_s * 1e6, 2), "median_launch_us": round(gemm_ms[len(gemm_ms) // 2] * 1e3, 2)}

    # ---------------- per-kernel side measurements (same buffers, event-timed) ------------
    if not args.no_extra:
        # the same step with and without the cache-warming hint, alternating (100 steps each, twice)
        def step_ab(i, warm):
            s = i % SETS
            for N in NS:
                sr.sr_fwht_quant_act_f6(Xs[s], inv_s_of[N], CLIP, X6, xs, warm=W6[N][s] if warm else None)
                sr.sr_w4a4_gemm_f6(X6, xs, W6[N][s], Ws[N][s], M, N, K, sr.SR_F16, Y[N])
        ab = {True: [], False: []}
        for _ in range(2):
            for warm in (False, True):
                for i in range(10):
                    step_ab(i, warm)
                torch.cuda.synchronize()
                tq = time.perf_counter()
                for i in range(100):
                    step_ab(i, warm)
                torch.cuda.synchronize()
                ab[warm].append(round((time.perf_counter() - tq) * 1e3 / 100, 4))
        extra["step_ms_with_cache_warming"] = ab[True]
        extra["step_ms_without_cache_warming"] = ab[False]
        # 20 distinct inputs (336 MB) for the rotation kernels on their own: 8 would stay in the Infinity Cache
        Xq_in = Xs + [torch.roll(x, 1 + j, 0) for j in range(2) for x in Xs][:12]
        t = graph_time(lambda i: sr.sr_fwht_quant_act(Xq_in[i % 20], inv_s, CLIP, Xq, xs), 60)
        b = M * K * 2.5 + M * 4
        extra["fwht_quant_K4096"] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1),
                                     "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4)}
        t = graph_time(lambda i: sr.sr_fwht_quant_act_f6(Xq_in[i % 20], inv_s, CLIP, X6, xs), 60)
        b = M * K * 2.75 + M * 4
        extra["fwht_quant_f6_K4096"] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1),
                                        "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4)}
        for N in NS:
            # weights of at least 300 MB in rotation (beyond the Infinity Cache): 24 copies for N = 4096
            reps = max(1, -(-300_000_000 // (SETS * W6[N][0].numel())))
            w6r = [w for w in W6[N]] + [w.clone() for _ in range(reps - 1) for w in W6[N]]
            t = graph_time(lambda i: sr.sr_w4a4_gemm_f6(X6, xs, w6r[i % len(w6r)], Ws[N][i % SETS], M, N, K, sr.SR_F16, Y[N]), 72)
            del w6r
            extra["gemm_f6_N%d" % N] = {"us": round(t * 1e6, 2), "TOPS": round(2.0 * M * N * K / t / 1e12, 1),
                                        "frac_int8_mfma_peak": round(2.0 * M * N * K / t / 1e12 / PEAK_INT8_TOPS, 4),
                                        "frac_fp6_mfma_peak": round(2.0 * M * N * K / t / 1e12 / PEAK_FP6_TOPS, 4)}
            t = graph_time(lambda i: sr.sr_w4a4_gemm(Xq, xs, Wq[N][i % SETS], Ws[N][i % SETS], sr.SR_F16, Y[N]), 64)
            extra["gemm_int8_N%d" % N] = {"us": round(t * 1e6, 2), "TOPS": round(2.0 * M * N * K / t / 1e12, 1),
                                          "frac_int8_mfma_peak": round(2.0 * M * N * K / t / 1e12 / PEAK_INT8_TOPS, 4)}
        # decode: M in {1,4,16}, K=4096 -> N=14336, weights streamed from >512 MB of distinct copies
        copies = [Wq[14336][0].clone() for _ in range(20)]
        wsc = Ws[14336][0]
        for Md in (1, 4, 16):
            Xd = Xs[0][:Md].contiguous()
            xq_d, xs_d = sr.sr_fwht_quant_act(Xd, inv_s, CLIP)
            Yd = torch.empty((Md, 14336), dtype=torch.float16, device=dev)
            t = graph_time(lambda i: sr.sr_w4a4_gemm(xq_d, xs_d, copies[i % 20], wsc, sr.SR_F16, Yd), 100)
            b = 14336 * K / 2 + Md * K / 2 + 2 * Md * 14336
            extra["decode_M%d_4096x14336" % Md] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1),
                                                    "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4)}
        # one token, whole online path: rotation + quantiser + GEMM as two calls and as the single fused launch
        Xd = Xs[0][:1].contiguous()
        xq_d = torch.empty((1, K // 2), dtype=torch.uint8, device=dev)
        xs_d = torch.empty(1, dtype=torch.float32, device=dev)
        Yd = torch.empty((1, 14336), dtype=torch.float16, device=dev)

        def two_calls(i):
            sr.sr_fwht_quant_act(Xd, inv_s, CLIP, xq_d, xs_d)
            sr.sr_w4a4_gemm(xq_d, xs_d, copies[i % 20], wsc, sr.SR_F16, Yd)
        t2 = graph_time(two_calls, 100)
        t1 = graph_time(lambda i: sr.sr_w4a4_linear_decode(Xd, inv_s, copies[i % 20], wsc, CLIP, Yd), 100)
        b = 14336 * K / 2 + K * 2 + 2 * 14336
        extra["decode_M1_4096x14336_whole_path"] = {"two_calls_us": round(t2 * 1e6, 2), "one_launch_us": round(t1 * 1e6, 2),
                                                    "GB/s": round(b / t1 / 1e9, 1),
                                                    "frac_hbm": round(b / t1 / 1e9 / PEAK_HBM_GBS, 4)}
        del copies
        # down-projection shape (config 3): K = 14336 = 28 * 512 -> N = 4096; rotation-only fold (s = 1)
        K3, N3 = 14336, 4096
        X3 = [torch.from_numpy(wl.cfg3_X(seed=2 + 10 * s)).to(dev) for s in range(4)]
        X3 += [torch.roll(x, 1, 0) for x in X3[:2]]              # 6 x 58.7 MB = 352 MB: beyond the Infinity Cache
        W3 = torch.from_numpy(wl.cfg3_W()).to(dev)
        Wq3, ws3, _ = sr.sr_fold_smooth_rotate_quant(W3, None, ALPHA, 1.0)
        del W3
        Xq3 = torch.empty((M, K3 // 2), dtype=torch.uint8, device=dev)
        xs3 = torch.empty(M, dtype=torch.float32, device=dev)
        Y3 = torch.empty((M, N3), dtype=torch.float16, device=dev)
        t = graph_time(lambda i: sr.sr_fwht_quant_act(X3[i % 6], None, CLIP, Xq3, xs3), 30)
        b = M * K3 * 2.5 + M * 4
        extra["fwht_quant_K14336"] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1),
                                      "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4)}
        t = graph_time(lambda i: sr.sr_w4a4_gemm(Xq3, xs3, Wq3, ws3, sr.SR_F16, Y3), 32)
        extra["gemm_int8_K14336_N4096"] = {"us": round(t * 1e6, 2), "TOPS": round(2.0 * M * N3 * K3 / t / 1e12, 1),
                                           "frac_int8_mfma_peak": round(2.0 * M * N3 * K3 / t / 1e12 / PEAK_INT8_TOPS, 4)}
        X63 = torch.zeros(sr.sr_f6_tiles_bytes(M, K3), dtype=torch.uint8, device=dev)
        W63 = sr.sr_pack_f6_tiles(Wq3)
        t = graph_time(lambda i: sr.sr_fwht_quant_act_f6(X3[i % 6], None, CLIP, X63, xs3), 30)
        b = M * K3 * 2.75 + M * 4
        extra["fwht_quant_f6_K14336"] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1),
                                         "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4)}
        W63s = [W63] + [W63.clone() for _ in range(7)]           # 8 x 44 MB: beyond the Infinity Cache
        t = graph_time(lambda i: sr.sr_w4a4_gemm_f6(X63, xs3, W63s[i % 8], ws3, M, N3, K3, sr.SR_F16, Y3), 32)
        extra["gemm_f6_K14336_N4096"] = {"us": round(t * 1e6, 2), "TOPS": round(2.0 * M * N3 * K3 / t / 1e12, 1),
                                         "frac_int8_mfma_peak": round(2.0 * M * N3 * K3 / t / 1e12 / PEAK_INT8_TOPS, 4),
                                         "frac_fp6_mfma_peak": round(2.0 * M * N3 * K3 / t / 1e12 / PEAK_FP6_TOPS, 4)}
        # the pair as a layer runs it: rotation + quantiser, then the GEMM -- without and with the quantiser launch
        # warming the memory-side cache with the GEMM's weights
        def pair3(i, warm):
            sr.sr_fwht_quant_act_f6(X3[i % 6], None, CLIP, X63, xs3, warm=W63s[i % 8] if warm else None)
            sr.sr_w4a4_gemm_f6(X63, xs3, W63s[i % 8], ws3, M, N3, K3, sr.SR_F16, Y3)
        tp = graph_time(lambda i: pair3(i, False), 24) * 1e6
        tw = graph_time(lambda i: pair3(i, True), 24) * 1e6
        extra["pair_K14336_N4096"] = {"quantiser_plus_gemm_us": round(tp, 2), "with_cache_warming_us": round(tw, 2)}
        del X63, W63, W63s
        copies = [Wq3.clone() for _ in range(20)]
        for Md in (1, 4, 16):
            xq_d, xs_d = sr.sr_fwht_quant_act(X3[0][:Md].contiguous(), None, CLIP)
            Yd = torch.empty((Md, N3), dtype=torch.float16, device=dev)
            t = graph_time(lambda i: sr.sr_w4a4_gemm(xq_d, xs_d, copies[i % 20], ws3, sr.SR_F16, Yd), 100)
            b = N3 * K3 / 2 + Md * K3 / 2 + 2 * Md * N3
            extra["decode_M%d_14336x4096" % Md] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1),
                                                    "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4)}
        del copies, X3
        # ---- rows around the core path -----------------------------------------------------------
        # gated-FFN prologue fused into the K = 14336 rotation + quantiser (two fp16 inputs per value)
        GU = [tuple(torch.from_numpy(a).to(dev) for a in wl.gate_up(2 + 10 * s, M, K3, 3, 800.0)) for s in range(3)]
        t = graph_time(lambda i: sr.sr_swiglu_fwht_quant_act(GU[i % 3][0], GU[i % 3][1], None, CLIP, Xq3, xs3), 24)
        b = M * K3 * 4.5 + M * 4
        extra["swiglu_fwht_quant_K14336"] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1),
                                             "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4)}
        X63 = torch.zeros(sr.sr_f6_tiles_bytes(M, K3), dtype=torch.uint8, device=dev)
        t = graph_time(lambda i: sr.sr_swiglu_fwht_quant_act_f6(GU[i % 3][0], GU[i % 3][1], None, CLIP, X63, xs3), 24)
        b = M * K3 * 4.75 + M * 4
        extra["swiglu_fwht_quant_f6_K14336"] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1),
                                                "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4)}
        del X63
        del GU
        # head-wise Hadamard (32 heads of 128, across heads) + quantiser on the benchmark activations
        t = graph_time(lambda i: sr.sr_fwht_quant_act_heads(Xq_in[i % 20], 32, True, inv_s, CLIP, Xq, xs), 60)
        del Xq_in
        b = M * K * 2.5 + M * 4
        extra["fwht_quant_heads32_K4096"] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1),
                                             "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4)}
        # weight fold with the 21-point clipping-ratio search (offline)
        Wf = torch.from_numpy(wl.cfg2_W(4096)).to(dev)
        work = torch.empty(sr.sr_fold_workspace_bytes(K, 4096), dtype=torch.uint8, device=dev)
        outs = sr.sr_fold_smooth_rotate_quant_ex(Wf, absmax, ALPHA, 0, False, 21, 0.5, workspace=work)
        torch.cuda.synchronize()
        t = ev_time(lambda i: sr.sr_fold_smooth_rotate_quant_ex(Wf, absmax, ALPHA, 0, False, 21, 0.5, *outs,
                                                                workspace=work), 5)
        extra["fold_clip_search21_N4096"] = {"us": round(t * 1e6, 1)}
        del Wf, work, outs
        # KV-cache quantiser: 32768 tokens x (8 KV heads x 128), asymmetric INT4, groups of 128, clip 0.95
        RKV, DKV = 32768, 1024
        KV = [torch.from_numpy(wl.kv_acts(5 + s, RKV, DKV)).to(dev) for s in range(5)]       # 5 x 67 MB
        kq = torch.empty((RKV, DKV // 2), dtype=torch.uint8, device=dev)
        ksc = torch.empty((RKV, DKV // 128), dtype=torch.float32, device=dev)
        kze = torch.empty((RKV, DKV // 128), dtype=torch.float32, device=dev)
        t = graph_time(lambda i: sr.sr_kv_quant_asym(KV[i % 5], 128, 0.95, kq, ksc, kze), 40)
        b = RKV * DKV * (2.0 + 0.5 + 8.0 / 128)
        extra["kv_quant_asym_32768x1024"] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1),
                                             "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4)}
        del KV
        # ---- config 5: the seven linears of a LLaMA-3.1-8B decoder layer at 8 x 2048 tokens (timing only:
        # random packed weights; q/k/v share one quantised input, gate/up another) --------------------------
        M5 = 16384
        X5 = torch.randn((M5, K), dtype=torch.float16, device=dev)
        X5d = torch.randn((M5, K3), dtype=torch.float16, device=dev)
        Xq5 = torch.empty((M5, K // 2), dtype=torch.uint8, device=dev)
        Xq5d = torch.empty((M5, K3 // 2), dtype=torch.uint8, device=dev)
        xs5 = torch.empty(M5, dtype=torch.float32, device=dev)
        W5 = {n: (torch.randint(0, 256, (nn, kk // 2), dtype=torch.uint8, device=dev), torch.rand(nn, device=dev) * 1e-3)
              for n, kk, nn in wl.CFG5_LINEARS}
        Y5 = torch.empty((M5, 14336), dtype=torch.float16, device=dev)

        def layer(i):
            sr.sr_fwht_quant_act(X5, inv_s, CLIP, Xq5, xs5)
            for n in ("q", "k", "v"):
                sr.sr_w4a4_gemm(Xq5, xs5, W5[n][0], W5[n][1], sr.SR_F16, Y5[:, :W5[n][0].shape[0]])
            sr.sr_fwht_quant_act(X5, inv_s, CLIP, Xq5, xs5)
            sr.sr_w4a4_gemm(Xq5, xs5, W5["o"][0], W5["o"][1], sr.SR_F16, Y5[:, :4096])
            sr.sr_fwht_quant_act(X5, inv_s, CLIP, Xq5, xs5)
            for n in ("gate", "up"):
                sr.sr_w4a4_gemm(Xq5, xs5, W5[n][0], W5[n][1], sr.SR_F16, Y5)
            sr.sr_fwht_quant_act(X5d, None, CLIP, Xq5d, xs5)
            sr.sr_w4a4_gemm(Xq5d, xs5, W5["down"][0], W5["down"][1], sr.SR_F16, Y5[:, :4096])
        layer(0)
        torch.cuda.synchronize()
        t = ev_time(layer, 5)
        ops5 = sum(2.0 * M5 * kk * nn for _, kk, nn in wl.CFG5_LINEARS)
        extra["cfg5_layer_M16384_int8"] = {"ms": round(t * 1e3, 3), "TOPS": round(ops5 / t / 1e12, 1),
                                           "frac_int8_mfma_peak": round(ops5 / t / 1e12 / PEAK_INT8_TOPS, 4),
                                           "workload": "7 linears (q,k,v,o,gate,up,down) + 4 rotate/quantise passes, 16384 tokens"}
        X65 = torch.zeros(sr.sr_f6_tiles_bytes(M5, K), dtype=torch.uint8, device=dev)
        X65d = torch.zeros(sr.sr_f6_tiles_bytes(M5, K3), dtype=torch.uint8, device=dev)
        W65 = {n: sr.sr_pack_f6_tiles(W5[n][0]) for n, _, _ in wl.CFG5_LINEARS}
        dims = {n: (kk, nn) for n, kk, nn in wl.CFG5_LINEARS}

        def g6(n, X6_, Yv):
            sr.sr_w4a4_gemm_f6(X6_, xs5, W65[n], W5[n][1], M5, dims[n][1], dims[n][0], sr.SR_F16, Yv)

        def layer6(i):                                       # every quantiser call warms the cache for the GEMM behind it
            sr.sr_fwht_quant_act_f6(X5, inv_s, CLIP, X65, xs5, warm=W65["q"])
            for n in ("q", "k", "v"):
                g6(n, X65, Y5[:, :dims[n][1]])
            sr.sr_fwht_quant_act_f6(X5, inv_s, CLIP, X65, xs5, warm=W65["o"])
            g6("o", X65, Y5[:, :4096])
            sr.sr_fwht_quant_act_f6(X5, inv_s, CLIP, X65, xs5, warm=W65["gate"])
            for n in ("gate", "up"):
                g6(n, X65, Y5)
            sr.sr_fwht_quant_act_f6(X5d, None, CLIP, X65d, xs5, warm=W65["down"])
            g6("down", X65d, Y5[:, :4096])
        layer6(0)
        torch.cuda.synchronize()
        t = ev_time(layer6, 5)
        extra["cfg5_layer_M16384"] = {"ms": round(t * 1e3, 3), "TOPS": round(ops5 / t / 1e12, 1),
                                      "frac_int8_mfma_peak": round(ops5 / t / 1e12 / PEAK_INT8_TOPS, 4),
                                      "workload": "7 linears (q,k,v,o,gate,up,down) + 4 rotate/quantise passes, 16384 tokens, f6 path"}
        # the rotation + quantiser passes of that layer on their own (three distinct inputs of 134 MB for K = 4096;
        # the 470 MB input of the down-projection is larger than the Infinity Cache by itself)
        X5s = [X5, torch.randn_like(X5), torch.randn_like(X5)]
        t = graph_time(lambda i: sr.sr_fwht_quant_act_f6(X5s[i % 3], inv_s, CLIP, X65, xs5), 6)
        b = M5 * K * 2.75 + 4 * M5
        extra["fwht_quant_f6_K4096_M16384"] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1),
                                               "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4)}
        t = graph_time(lambda i: sr.sr_fwht_quant_act_f6(X5d, None, CLIP, X65d, xs5), 4)
        b = M5 * K3 * 2.75 + 4 * M5
        extra["fwht_quant_f6_K14336_M16384"] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1),
                                                "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4)}
        del X5, X5s, X5d, Xq5, Xq5d, W5, Y5, X65, X65d, W65

    # ---------------- CPU baseline: the oracle on a bounded sample ------------------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import smoothrot_oracle as o
        rows = M
        Xh = Xs[0][:rows].cpu().numpy()
        inv_h = {N: inv_s_of[N].cpu().numpy() for N in NS}
        cws = {N: o.unpack_int4(Wq[N][0].cpu().numpy()) for N in NS}
        wsh = {N: Ws[N][0].cpu().numpy() for N in NS}
        o.gemm_i32_c(np.zeros((1, 64), np.int8), np.zeros((1, 64), np.int8))     # load the C library
        t0 = time.perf_counter()
        for N in NS:
            act = o.fwht_quant_act(Xh, inv_h[N], CLIP)
            acc = o.gemm_i32_c(act["codes"], cws[N])
            o.dequant_out(acc, act["x_scale"], wsh[N])
        tc = time.perf_counter() - t0
        cpu = {"value": round(sum(2.0 * rows * N * K for N in NS) / tc / 1e12, 5), "unit": "TOPS",
               "cores": o.c_threads(), "kind": "oracle",
               "sample": "%d of %d token rows through both linears (rotate+quantise, int GEMM, dequantise); %.1f s" % (rows, M, tc)}

    line = {
        "metric": "W4A4 linear TOPS (prefill; FWHT + INT4 quantise + INT4 GEMM + dequant)",
        "value": round(tops, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int4 codes as fp6 (E2M3) on the FP6 MFMA, fp32 accumulate (exact integers); fp32 rotation",
        "data": "synthetic",
        "config": {"workload": "configs[1]: prefill X fp16 [2048,4096], two linears N=4096 and N=14336, "
                               "alpha=0.5, act clip 0.9, H_4096; step = 2 x (sr_fwht_quant_act_f6_warm + sr_w4a4_gemm_f6)",
                   "M": M, "K": K, "N": list(NS), "input_sets_rotated": SETS},
        "frac_int8_mfma_peak": round(tops / PEAK_INT8_TOPS, 4),
        "roofline": roofline, "cpu_baseline": cpu, "extra": extra,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
