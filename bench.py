#!/usr/bin/env python3
"""Benchmark of the SmoothRot W4A4 linear hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One "step" = the online hot path of the two prefill linears of the benchmark
configuration (X fp16 [2048, 4096]; W [4096, 4096] and W [4096, 14336]):
    sr_fwht_quant_act_f6_warm(X) -> sr_w4a4_gemm_f6_warm(N = 4096)
    sr_fwht_quant_act_f6(X)      -> sr_w4a4_gemm_f6(N = 14336)
(rotation + per-token INT4 quantiser writing the codes as f6 tiles, then the INT4 x INT4 GEMM on the FP6 matrix
pipe, which multiplies the codes exactly; weights are repacked to f6 tiles once, offline.  The two `_warm` calls
also pull the weights of the next GEMM into the memory-side cache: the first quantiser launch those of the
N = 4096 GEMM, that GEMM those of the N = 14336 one; outputs are unchanged.)
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
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "bench_prefill_cfg2_hbm_traffic.json")


def measured_traffic(kernel_key):
    """HBM bytes per launch of a kernel of the timed step, as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    and committed under profiles/ (None if the file or the entry is missing: the counters cannot be read from
    inside this process)."""
    try:
        with open(TRAFFIC_JSON) as f:
            t = json.load(f)
        e = t["kernels"][kernel_key]
        return {"hbm_bytes_per_launch": e["read_bytes"] + e["written_bytes"], "read_bytes": e["read_bytes"],
                "written_bytes": e["written_bytes"], "algorithmic_bytes": e["algorithmic_bytes"],
                "source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by a copy kernel of known size; "
                          "profiles/bench_prefill_cfg2_hbm_traffic.json (tree %s)" % t.get("tree", "?")}
    except (OSError, KeyError, ValueError):
        return None

M, K = 2048, 4096
NS = (4096, 14336)
CLIP, ALPHA = 0.9, 0.5
SETS = 8                     # distinct (X, Wq) sets rotated through: 8 * (16.8 + 37.7) MB > 256 MB


def cfg5_chained(sr, wl, torch, dev, graph_time, ev_time, args):
    """Config 5: the seven linears of a LLaMA-3.1-8B-shaped decoder layer on 16384 tokens, W4A4 end to end on
    random-init weights, chained as the paper's Fig. 2 draws the blocks:
        Xa --rotate+quantise--> [q|k|v] one GEMM, N = 6144                  (folded as ONE weight: shared input, shared s)
        Xo --rotate+quantise--> o,      N = 4096                            (Xo: stand-in for the attention core's output)
        Xf --rotate+quantise--> [gate|up] one GEMM, N = 28672               (1/s of the down-projection absorbed into W_up)
        silu(gate) * up --rotate (H_28 x H_512)+quantise, no factors--> down, K = 14336 -> N = 4096
    The gate/up outputs ARE the down-projection's input (sr_swiglu_fwht_quant_act_f6 reads them in place).
    Left out and not timed: RMS-normalisation, residual additions, RoPE, softmax(QK^T)V, KV-cache quantisation --
    Xa, Xo, Xf are generated RMS-normalised tensors with the outlier channels of config 2.
    Offline, timed separately: calibration absmax of the four inputs (the down-projection's on the fp16 layer's own
    silu(gate) * up, as the paper calibrates on the fp16 model) and the four folds that cover the seven weights."""
    import numpy as np
    M5, K, KD, NQ, NG = 16384, 4096, 14336, 6144, 28672
    out = {}
    Xa, Xo, Xf = (torch.from_numpy(wl.cfg5_X(M5, K, stream=40 + j)).to(dev) for j in range(3))
    Wd = {n: torch.from_numpy(wl.cfg5_W(n)).to(dev) for n, _, _ in wl.CFG5_LINEARS}
    # ---- calibration (offline): one absmax pass per distinct input
    am = {k: torch.zeros(K, dtype=torch.float32, device=dev) for k in ("a", "o", "f")}
    calib_us = {}
    for k, X in (("a", Xa), ("o", Xo), ("f", Xf)):
        sr.sr_calib_absmax(X, am[k])
        scratch = torch.zeros(K, dtype=torch.float32, device=dev)
        calib_us[k] = ev_time(lambda i: sr.sr_calib_absmax(X, scratch), 3) * 1e6
    # the down-projection's input on the fp16 layer (plain fp16 matmuls: calibration runs on the unquantised model)
    D = torch.empty((M5, KD), dtype=torch.float16, device=dev)
    for r in range(0, M5, 4096):
        g = Xf[r:r + 4096] @ Wd["gate"]
        u = Xf[r:r + 4096] @ Wd["up"]
        D[r:r + 4096] = (torch.nn.functional.silu(g.float()) * u.float()).to(torch.float16)
    am_d = torch.zeros(KD, dtype=torch.float32, device=dev)
    sr.sr_calib_absmax(D, am_d)
    scratch = torch.zeros(KD, dtype=torch.float32, device=dev)
    calib_us["down"] = ev_time(lambda i: sr.sr_calib_absmax(D, scratch), 3) * 1e6
    del D, g, u
    # ---- folds (offline): down first (its 1/s goes into W_up), then the fused weights
    def fold(W, a, what):
        Kw, Nw = W.shape
        work = torch.empty(sr.sr_fold_workspace_bytes(Kw, Nw), dtype=torch.uint8, device=dev)
        outs = sr.sr_fold_smooth_rotate_quant(W, a, ALPHA, 1.0, workspace=work)
        torch.cuda.synchronize()
        t = ev_time(lambda i: sr.sr_fold_smooth_rotate_quant(W, a, ALPHA, 1.0, *outs, workspace=work), 3)
        t6 = sr.sr_pack_f6_tiles(outs[0])
        out.setdefault("offline_us", {})["fold_" + what] = round(t * 1e6, 1)
        return t6, outs[1], outs[2], outs[0]
    W6d, wsd, inv_d, Wqd = fold(Wd["down"], am_d, "down_14336x4096")
    W_up_abs = (Wd["up"].float() * inv_d[None, :]).to(torch.float16)          # Lambda^-1 of the down-projection, absorbed
    W6q, wsq, inv_q, Wqq = fold(torch.cat([Wd["q"], Wd["k"], Wd["v"]], 1).contiguous(), am["a"], "qkv_4096x6144")
    W6o, wso, inv_o, Wqo = fold(Wd["o"], am["o"], "o_4096x4096")
    W6g, wsg, inv_g, Wqg = fold(torch.cat([Wd["gate"], W_up_abs], 1).contiguous(), am["f"], "gateup_4096x28672")
    del Wd, W_up_abs
    for k, v in calib_us.items():
        out["offline_us"]["calib_absmax_" + k] = round(v, 1)
    # ---- the chained layer (timed)
    X6 = torch.zeros(sr.sr_f6_tiles_bytes(M5, K), dtype=torch.uint8, device=dev)
    X6d = torch.zeros(sr.sr_f6_tiles_bytes(M5, KD), dtype=torch.uint8, device=dev)
    xs = torch.empty(M5, dtype=torch.float32, device=dev)
    QKV = torch.empty((M5, NQ), dtype=torch.float16, device=dev)
    O = torch.empty((M5, K), dtype=torch.float16, device=dev)
    GU = torch.empty((M5, NG), dtype=torch.float16, device=dev)
    DN = torch.empty((M5, K), dtype=torch.float16, device=dev)

    def layer(i):
        sr.sr_fwht_quant_act_f6(Xa, inv_q, CLIP, X6, xs, warm=W6q)
        sr.sr_w4a4_gemm_f6(X6, xs, W6q, wsq, M5, NQ, K, sr.SR_F16, QKV)
        sr.sr_fwht_quant_act_f6(Xo, inv_o, CLIP, X6, xs, warm=W6o)
        sr.sr_w4a4_gemm_f6(X6, xs, W6o, wso, M5, K, K, sr.SR_F16, O)
        sr.sr_fwht_quant_act_f6(Xf, inv_g, CLIP, X6, xs, warm=W6g)
        sr.sr_w4a4_gemm_f6(X6, xs, W6g, wsg, M5, NG, K, sr.SR_F16, GU)
        sr.sr_swiglu_fwht_quant_act_f6(GU[:, :KD], GU[:, KD:], None, CLIP, X6d, xs)
        sr.sr_w4a4_gemm_f6(X6d, xs, W6d, wsd, M5, K, KD, sr.SR_F16, DN)
    layer(0)
    torch.cuda.synchronize()
    t = ev_time(layer, 5)
    ops5 = sum(2.0 * M5 * kk * nn for _, kk, nn in wl.CFG5_LINEARS)
    out["cfg5_layer_M16384"] = {
        "ms": round(t * 1e3, 3), "TOPS": round(ops5 / t / 1e12, 1),
        "frac_int8_mfma_peak": round(ops5 / t / 1e12 / PEAK_INT8_TOPS, 4),
        "workload": "chained layer, 16384 tokens, FP6-pipe path: [q|k|v] as one N=6144 GEMM, o, [gate|up] as one N=28672 GEMM "
                    "(1/s of down absorbed into W_up), silu(gate)*up read in place by the fused K=14336 rotate+quantise, down; "
                    "4 rotate/quantise launches + 4 GEMMs; left out: RMS-normalise, residual adds, RoPE, attention core, KV quantiser"}
    # the same chain through the canonical-nibble quantiser and the int8-MFMA GEMM
    Xq = torch.empty((M5, K // 2), dtype=torch.uint8, device=dev)
    Xqd = torch.empty((M5, KD // 2), dtype=torch.uint8, device=dev)

    def layer_i8(i):
        sr.sr_fwht_quant_act(Xa, inv_q, CLIP, Xq, xs)
        sr.sr_w4a4_gemm(Xq, xs, Wqq, wsq, sr.SR_F16, QKV)
        sr.sr_fwht_quant_act(Xo, inv_o, CLIP, Xq, xs)
        sr.sr_w4a4_gemm(Xq, xs, Wqo, wso, sr.SR_F16, O)
        sr.sr_fwht_quant_act(Xf, inv_g, CLIP, Xq, xs)
        sr.sr_w4a4_gemm(Xq, xs, Wqg, wsg, sr.SR_F16, GU)
        sr.sr_swiglu_fwht_quant_act(GU[:, :KD], GU[:, KD:], None, CLIP, Xqd, xs)
        sr.sr_w4a4_gemm(Xqd, xs, Wqd, wsd, sr.SR_F16, DN)
    layer_i8(0)
    torch.cuda.synchronize()
    t8 = ev_time(layer_i8, 3)
    out["cfg5_layer_M16384_int8"] = {"ms": round(t8 * 1e3, 3), "TOPS": round(ops5 / t8 / 1e12, 1),
                                     "frac_int8_mfma_peak": round(ops5 / t8 / 1e12 / PEAK_INT8_TOPS, 4),
                                     "workload": "the same chain through sr_fwht_quant_act / sr_swiglu_fwht_quant_act and sr_w4a4_gemm"}
    # the rotation + quantiser launches of the layer on their own
    t = graph_time(lambda i: sr.sr_fwht_quant_act_f6((Xa, Xo, Xf)[i % 3], inv_g, CLIP, X6, xs), 6)
    b = M5 * K * 2.75 + 4 * M5
    out["fwht_quant_f6_K4096_M16384"] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1),
                                         "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4)}
    t = graph_time(lambda i: sr.sr_swiglu_fwht_quant_act_f6(GU[:, :KD], GU[:, KD:], None, CLIP, X6d, xs), 4)
    b = M5 * KD * 4.75 + 4 * M5
    out["swiglu_fwht_quant_f6_K14336_M16384"] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1),
                                                 "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4)}
    # ---- the oracle on a seeded 256-row subsample of the same chain, extrapolated x 64 (all host cores)
    if not args.no_cpu_baseline:
        from oracle import smoothrot_oracle as o
        rows = np.sort(np.random.default_rng(5).choice(M5, 256, replace=False))
        ridx = torch.from_numpy(rows).to(dev)
        h = lambda tns: tns.cpu().numpy()
        xa, xo, xf = h(Xa[ridx]), h(Xo[ridx]), h(Xf[ridx])
        cw = {k: o.unpack_int4(h(v)) for k, v in (("q", Wqq), ("o", Wqo), ("g", Wqg), ("d", Wqd))}
        sc = {k: h(v).astype(np.float64) for k, v in (("q", wsq), ("o", wso), ("g", wsg), ("d", wsd))}
        iv = {k: h(v).astype(np.float64) for k, v in (("q", inv_q), ("o", inv_o), ("g", inv_g))}
        o.gemm_i32_c(np.zeros((1, 64), np.int8), np.zeros((1, 64), np.int8))
        t0 = time.perf_counter()
        for x, k in ((xa, "q"), (xo, "o")):
            act = o.fwht_quant_act(x, iv[k], CLIP)
            o.dequant_out(o.gemm_i32_c(act["codes"], cw[k]), act["x_scale"], sc[k])
        act = o.fwht_quant_act(xf, iv["g"], CLIP)
        gu = o.dequant_out(o.gemm_i32_c(act["codes"], cw["g"]), act["x_scale"], sc["g"]).astype(np.float16)
        act = o.fwht_quant_swiglu(gu[:, :KD], gu[:, KD:], None, CLIP)
        o.dequant_out(o.gemm_i32_c(act["codes"], cw["d"]), act["x_scale"], sc["d"])
        tc = time.perf_counter() - t0
        out["cfg5_layer_M16384"]["cpu_baseline_extrapolated"] = {
            "value": round(ops5 / (tc * 64) / 1e12, 5), "unit": "TOPS", "cores": o.c_threads(), "kind": "oracle",
            "sample": "256 seeded rows of 16384 through the whole chain against the full weights: %.1f s, x 64 = %.0f s (extrapolated)" % (tc, tc * 64)}
    return out


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
        sr.sr_fwht_quant_act_f6(Xs[s], inv_s_of[4096], CLIP, X6, xs, warm=W6[4096][s])
        sr.sr_w4a4_gemm_f6(X6, xs, W6[4096][s], Ws[4096][s], M, 4096, K, sr.SR_F16, Y[4096], warm=W6[14336][s])
        sr.sr_fwht_quant_act_f6(Xs[s], inv_s_of[14336], CLIP, X6, xs)
        sr.sr_w4a4_gemm_f6(X6, xs, W6[14336][s], Ws[14336][s], M, 14336, K, sr.SR_F16, Y[14336])

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
        # cache-warming hints: the first rotation + quantiser call reads the (12.6 MB of) weights of the GEMM behind it
        # on the side; the 44 MB of the second GEMM are read by the first GEMM, which has a wave and HBM bandwidth to
        # spare (256 x 128 tiles), so the second quantiser call carries no hint
        sr.sr_fwht_quant_act_f6(Xs[s], inv_s_of[4096], CLIP, X6, xs, warm=W6[4096][s])
        sr.sr_w4a4_gemm_f6(X6, xs, W6[4096][s], Ws[4096][s], M, 4096, K, sr.SR_F16, Y[4096], warm=W6[14336][s])
        sr.sr_fwht_quant_act_f6(Xs[s], inv_s_of[14336], CLIP, X6, xs)
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
                "traffic": measured_traffic("gemm_f6_N14336"),
                "avg_launch_us": round(gemm_avg_s * 1e6, 2), "median_launch_us": round(gemm_ms[len(gemm_ms) // 2] * 1e3, 2)}

    # ---------------- measured ceilings (committed measurement kernels of the library) ------
    # What this machine sustains with nothing else in the way, measured in this process: a bare issue loop of the
    # matrix instruction the GEMM uses on code-valued operands, a pure read of one packed weight (29.4 MB) over 20
    # rotating copies, a bare fp32 vector-ALU loop.  Every fraction of a published peak below is also given
    # against these.
    ceil = {}
    if not args.no_extra:
        CU = torch.cuda.get_device_properties(0).multi_processor_count
        f6_src = W6[4096][0]
        # ~60 us launches (the length of the N = 14336 GEMM), back to back in a graph
        ops = [0.0]
        def f6_loop(i):
            ops[0] = sr.sr_ceiling_mfma_f6(f6_src, 170, CU)
        t = graph_time(f6_loop, 40)
        ceil["mfma_f6_loop"] = {"us": round(t * 1e6, 2), "PFLOP/s": round(ops[0] / t / 1e15, 3),
                                "what": "v_mfma_scale_f32_32x32x64_f8f6f4 on 6-bit code fields, 8 waves per CU, 8 accumulator tiles per wave, no loads"}
        i8_src = Wq[4096][0]
        def i8_loop(i):
            ops[0] = sr.sr_ceiling_mfma_i8(i8_src, 170, CU)
        t = graph_time(i8_loop, 40)
        ceil["mfma_i8_loop"] = {"us": round(t * 1e6, 2), "POP/s": round(ops[0] / t / 1e15, 3),
                                "what": "v_mfma_i32_32x32x32_i8 on packed code bytes, same loop"}
        def valu_loop(i):
            ops[0] = sr.sr_ceiling_valu_f32(160, 2 * CU)
        t = graph_time(valu_loop, 20)
        ceil["valu_f32_loop"] = {"us": round(t * 1e6, 2), "T_wave_instr/s": round(ops[0] / t / 1e12, 3),
                                 "T_lane_instr/s": round(ops[0] * 64 / t / 1e12, 2),
                                 "frac_of_78.6_T_lane_instr/s": round(ops[0] * 64 / t / 78.6e12, 3),
                                 "SIMD_cycles_per_wave_instr_at_2.4GHz": round(2.4e9 * t * 4 * CU / ops[0], 2),
                                 "what": "fp32 add / sub / mul (no FMA, no packed forms) on 64 lanes, 2 waves per SIMD, 192 instructions per "
                                         "iteration; peak = 157.3 TFLOP/s FMA-counted = 78.6 T lane instructions/s"}
        rd = [Wq[14336][0].clone() for _ in range(20)]                         # 20 x 29.4 MB = 587 MB
        best = None
        for grid, block, fl, nt in ((8 * CU, 256, 8, True), (4 * CU, 512, 8, True), (8 * CU, 256, 16, True),
                                    (16 * CU, 256, 4, True), (8 * CU, 256, 8, False), (28 * CU, 256, 4, True)):
            t = graph_time(lambda i: sr.sr_ceiling_hbm_read(rd[i % 20], grid, block, fl, nt), 100)
            if best is None or t < best[0]:
                best = (t, grid, block, fl, nt)
        nbytes = rd[0].numel()
        ceil["hbm_read_29MB"] = {"us": round(best[0] * 1e6, 2), "GB/s": round(nbytes / best[0] / 1e9, 1),
                                 "frac_hbm": round(nbytes / best[0] / 1e9 / PEAK_HBM_GBS, 4),
                                 "config": {"workgroups": best[1], "threads": best[2], "loads_in_flight": best[3], "nontemporal": best[4]},
                                 "what": "pure read of one packed weight [14336, 2048] bytes per launch, 20 rotating copies, best of 6 launch shapes"}
        del rd
        # the traffic of the rotation + quantiser launches without the rotation: a row in, its codes out, same grid and
        # LDS footprint (K = 4096: 8 rows in flight per CU; K = 14336: 512 workgroups walking over the rows)
        xin = Xs + [torch.roll(x, 1 + j, 0) for j in range(2) for x in Xs][:12]              # 20 x 16.8 MB
        outb = torch.empty(M * 3072, dtype=torch.uint8, device=dev)
        t = graph_time(lambda i: sr.sr_ceiling_row_stream(xin[i % 20], outb, M, 2 * K, 3072, M, 19 * 1024), 60)
        b = M * (2 * K + 3072)
        ceil["row_stream_K4096"] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1), "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4),
                                    "what": "2048 rows of 8 KB read, 3 KB written per row (the bytes of sr_fwht_quant_act_f6 at K = 4096), 20 rotating inputs"}
        del xin, outb
        x3 = [torch.randint(0, 255, (M * 28672,), dtype=torch.uint8, device=dev) for _ in range(6)]       # 6 x 58.7 MB
        outb = torch.empty(M * 10752, dtype=torch.uint8, device=dev)
        t = graph_time(lambda i: sr.sr_ceiling_row_stream(x3[i % 6], outb, M, 28672, 10752, 2 * CU, 61 * 1024), 30)
        b = M * (28672 + 10752)
        ceil["row_stream_K14336"] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1), "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4),
                                     "what": "2048 rows of 28 KB read, 10.5 KB written per row (sr_fwht_quant_act_f6 at K = 14336), 6 rotating inputs"}
        del x3, outb
        extra["ceilings"] = ceil
        roofline["measured_ceiling"] = {"TFLOP/s": round(ceil["mfma_f6_loop"]["PFLOP/s"] * 1e3, 1),
                                        "frac": round(roofline["achieved"] / (ceil["mfma_f6_loop"]["PFLOP/s"] * 1e3), 4),
                                        "what": "bare FP6 MFMA issue loop, this box, this process"}

    # ---------------- per-kernel side measurements (same buffers, event-timed) ------------
    if not args.no_extra:
        # the same step under four cache-warming schemes, alternating (100 steps each, twice):
        #   none       no hint anywhere
        #   quantiser  each rotation + quantiser call reads the weights of the GEMM behind it
        #   gemm       the N = 4096 GEMM (256 x 128 tiles: a wave to spare) reads the weights of the N = 14336 GEMM;
        #              the first quantiser call still reads the N = 4096 weights, the second one nothing
        #   gemm_only  as before, and the first quantiser call reads nothing either
        def step_ab(i, scheme):
            s = i % SETS
            qa = W6[4096][s] if scheme in ("quantiser", "gemm") else None
            qb = W6[14336][s] if scheme == "quantiser" else None
            ga = W6[14336][s] if scheme in ("gemm", "gemm_only") else None
            sr.sr_fwht_quant_act_f6(Xs[s], inv_s_of[4096], CLIP, X6, xs, warm=qa)
            sr.sr_w4a4_gemm_f6(X6, xs, W6[4096][s], Ws[4096][s], M, 4096, K, sr.SR_F16, Y[4096], warm=ga)
            sr.sr_fwht_quant_act_f6(Xs[s], inv_s_of[14336], CLIP, X6, xs, warm=qb)
            sr.sr_w4a4_gemm_f6(X6, xs, W6[14336][s], Ws[14336][s], M, 14336, K, sr.SR_F16, Y[14336])
        schemes = ("none", "quantiser", "gemm", "gemm_only")
        ab = {k: [] for k in schemes}
        for _ in range(2):
            for scheme in schemes:
                for i in range(10):
                    step_ab(i, scheme)
                torch.cuda.synchronize()
                tq = time.perf_counter()
                for i in range(100):
                    step_ab(i, scheme)
                torch.cuda.synchronize()
                ab[scheme].append(round((time.perf_counter() - tq) * 1e3 / 100, 4))
        extra["step_ms_by_cache_warming_scheme"] = ab
        # 20 distinct inputs (336 MB) for the rotation kernels on their own: 8 would stay in the Infinity Cache
        Xq_in = Xs + [torch.roll(x, 1 + j, 0) for j in range(2) for x in Xs][:12]
        t = graph_time(lambda i: sr.sr_fwht_quant_act(Xq_in[i % 20], inv_s, CLIP, Xq, xs), 60)
        b = M * K * 2.5 + M * 4
        extra["fwht_quant_K4096"] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1),
                                     "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4)}
        t = graph_time(lambda i: sr.sr_fwht_quant_act_f6(Xq_in[i % 20], inv_s, CLIP, X6, xs), 60)
        b = M * K * 2.75 + M * 4
        extra["fwht_quant_f6_K4096"] = {"us": round(t * 1e6, 2), "GB/s": round(b / t / 1e9, 1),
                                        "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4),
                                        "frac_measured_row_stream": round(ceil["row_stream_K4096"]["us"] * 1e-6 / t, 4)}
        for N in NS:
            # weights of at least 300 MB in rotation (beyond the Infinity Cache): 24 copies for N = 4096
            reps = max(1, -(-300_000_000 // (SETS * W6[N][0].numel())))
            w6r = [w for w in W6[N]] + [w.clone() for _ in range(reps - 1) for w in W6[N]]
            t = graph_time(lambda i: sr.sr_w4a4_gemm_f6(X6, xs, w6r[i % len(w6r)], Ws[N][i % SETS], M, N, K, sr.SR_F16, Y[N]), 72)
            del w6r
            extra["gemm_f6_N%d" % N] = {"us": round(t * 1e6, 2), "TOPS": round(2.0 * M * N * K / t / 1e12, 1),
                                        "frac_int8_mfma_peak": round(2.0 * M * N * K / t / 1e12 / PEAK_INT8_TOPS, 4),
                                        "frac_fp6_mfma_peak": round(2.0 * M * N * K / t / 1e12 / PEAK_FP6_TOPS, 4),
                                        "frac_measured_f6_loop": round(2.0 * M * N * K / t / 1e15 / ceil["mfma_f6_loop"]["PFLOP/s"], 4)}
            t = graph_time(lambda i: sr.sr_w4a4_gemm(Xq, xs, Wq[N][i % SETS], Ws[N][i % SETS], sr.SR_F16, Y[N]), 64)
            extra["gemm_int8_N%d" % N] = {"us": round(t * 1e6, 2), "TOPS": round(2.0 * M * N * K / t / 1e12, 1),
                                          "frac_int8_mfma_peak": round(2.0 * M * N * K / t / 1e12 / PEAK_INT8_TOPS, 4),
                                          "frac_measured_i8_loop": round(2.0 * M * N * K / t / 1e15 / ceil["mfma_i8_loop"]["POP/s"], 4)}
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
                                                    "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4),
                                                    "frac_measured_read_29MB": round(b / t / 1e9 / ceil["hbm_read_29MB"]["GB/s"], 4)}
        # whole online path of a decode step: rotation + quantiser + GEMM as two calls and as the one call
        # sr_w4a4_linear_decode (one token, K = 4096: a single launch in which every workgroup rotates the row itself;
        # otherwise the two kernels back to back inside the call -- no single launch measured faster there)
        for Md in (1, 4, 16):
            Xd = Xs[0][:Md].contiguous()
            xq_d = torch.empty((Md, K // 2), dtype=torch.uint8, device=dev)
            xs_d = torch.empty(Md, dtype=torch.float32, device=dev)
            Yd = torch.empty((Md, 14336), dtype=torch.float16, device=dev)
            wsp = torch.zeros(max(sr.sr_linear_decode_workspace_bytes(Md, K), 256), dtype=torch.uint8, device=dev)

            def two_calls(i):
                sr.sr_fwht_quant_act(Xd, inv_s, CLIP, xq_d, xs_d)
                sr.sr_w4a4_gemm(xq_d, xs_d, copies[i % 20], wsc, sr.SR_F16, Yd)
            t2 = graph_time(two_calls, 100)
            t1 = graph_time(lambda i: sr.sr_w4a4_linear_decode(Xd, inv_s, copies[i % 20], wsc, CLIP, Yd, workspace=wsp), 100)
            b = 14336 * K / 2 + Md * K * 2 + 2 * Md * 14336
            extra["decode_M%d_4096x14336_whole_path" % Md] = {
                "two_calls_us": round(t2 * 1e6, 2), "one_call_us": round(t1 * 1e6, 2), "GB/s": round(b / t1 / 1e9, 1),
                "frac_hbm": round(b / t1 / 1e9 / PEAK_HBM_GBS, 4),
                "launches_in_the_one_call": 1 if Md == 1 else 2}
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
                                         "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4),
                                         "frac_measured_row_stream": round(ceil["row_stream_K14336"]["us"] * 1e-6 / t, 4)}
        W63s = [W63] + [W63.clone() for _ in range(7)]           # 8 x 44 MB: beyond the Infinity Cache
        t = graph_time(lambda i: sr.sr_w4a4_gemm_f6(X63, xs3, W63s[i % 8], ws3, M, N3, K3, sr.SR_F16, Y3), 32)
        extra["gemm_f6_K14336_N4096"] = {"us": round(t * 1e6, 2), "TOPS": round(2.0 * M * N3 * K3 / t / 1e12, 1),
                                         "frac_int8_mfma_peak": round(2.0 * M * N3 * K3 / t / 1e12 / PEAK_INT8_TOPS, 4),
                                         "frac_fp6_mfma_peak": round(2.0 * M * N3 * K3 / t / 1e12 / PEAK_FP6_TOPS, 4),
                                         "frac_measured_f6_loop": round(2.0 * M * N3 * K3 / t / 1e15 / ceil["mfma_f6_loop"]["PFLOP/s"], 4)}
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
                                                    "frac_hbm": round(b / t / 1e9 / PEAK_HBM_GBS, 4),
                                                    "frac_measured_read_29MB": round(b / t / 1e9 / ceil["hbm_read_29MB"]["GB/s"], 4)}
        # the down-projection's decode step (K = 14336 = 28 * 512: the place the paper puts the online Hadamard), whole path
        for Md in (1, 4, 16):
            Xd = X3[0][:Md].contiguous()
            xq_d = torch.empty((Md, K3 // 2), dtype=torch.uint8, device=dev)
            xs_d = torch.empty(Md, dtype=torch.float32, device=dev)
            Yd = torch.empty((Md, N3), dtype=torch.float16, device=dev)
            wsp = torch.zeros(sr.sr_linear_decode_workspace_bytes(Md, K3), dtype=torch.uint8, device=dev)

            def two_calls3(i):
                sr.sr_fwht_quant_act(Xd, None, CLIP, xq_d, xs_d)
                sr.sr_w4a4_gemm(xq_d, xs_d, copies[i % 20], ws3, sr.SR_F16, Yd)
            t2 = graph_time(two_calls3, 100)
            t1 = graph_time(lambda i: sr.sr_w4a4_linear_decode(Xd, None, copies[i % 20], ws3, CLIP, Yd, workspace=wsp), 100)
            b = N3 * K3 / 2 + Md * K3 * 2 + 2 * Md * N3
            extra["decode_M%d_14336x4096_whole_path" % Md] = {
                "two_calls_us": round(t2 * 1e6, 2), "one_call_us": round(t1 * 1e6, 2), "GB/s": round(b / t1 / 1e9, 1),
                "frac_hbm": round(b / t1 / 1e9 / PEAK_HBM_GBS, 4), "launches_in_the_one_call": 2,
                "note": "one-launch variants lose here (measured 11.9 - 13.4 us against this pair): the call runs the two kernels"}
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
        # ---- config 5: a LLaMA-3.1-8B-shaped decoder layer at 8 x 2048 tokens, chained (see cfg5_chained) ----
        extra.update(cfg5_chained(sr, wl, torch, dev, graph_time, ev_time, args))

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
                               "alpha=0.5, act clip 0.9, H_4096; step = sr_fwht_quant_act_f6_warm + sr_w4a4_gemm_f6_warm (N=4096) + sr_fwht_quant_act_f6 + sr_w4a4_gemm_f6 (N=14336)",
                   "M": M, "K": K, "N": list(NS), "input_sets_rotated": SETS},
        "frac_int8_mfma_peak": round(tops / PEAK_INT8_TOPS, 4),
        "roofline": roofline, "cpu_baseline": cpu, "extra": extra,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
