"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

import paper_2506_05413_amd as sr

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "smoothrot.h")

A = 0x1000          # a fake, 16-byte aligned, non-NULL "device pointer" (never dereferenced on the host)
WS = 0x10000        # 256-byte aligned fake workspace


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return re.findall(r"SR_API\s+[\w\s\*]+?\b(sr_\w+)\s*\(", text)


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) == 30 and "sr_w4a4_gemm" in names and "sr_calib_absmax" in names
    lib = ctypes.CDLL(sr.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(sr.binding._SIGNATURES)


def test_tuning_knobs_round_trip_and_reject_unknown_ones():
    for knob in range(sr.SR_TUNE_KNOBS):
        assert sr.sr_tune_get(knob) == sr.SR_TUNE_AUTO
        sr.sr_tune_set(knob, 3)
        assert sr.sr_tune_get(knob) == 3
        sr.sr_tune_set(knob, sr.SR_TUNE_AUTO)
        assert sr.sr_tune_get(knob) == sr.SR_TUNE_AUTO
    assert sr.raw().sr_tune_set(sr.SR_TUNE_KNOBS, 1) == sr.SR_ERR_ARG and sr.raw().sr_tune_set(-1, 1) == sr.SR_ERR_ARG
    assert sr.sr_tune_get(99) == sr.SR_TUNE_AUTO


def test_noalloc_fold_checks_size_and_arguments_before_any_device_call():
    f = sr.raw().sr_fold_smooth_rotate_quant_noalloc
    assert sr.sr_noalloc_scratch_bytes() >= sr.sr_fold_workspace_bytes(4096, 4096)
    assert f(A, 4096, 14336, 14336, A, 0.5, 1.0, A, A, A, None) == sr.SR_ERR_WORKSPACE
    assert f(A, 4096, 4160, 4160, A, 0.5, 1.0, A, A, A, None) == sr.SR_ERR_WORKSPACE
    assert f(A, 500, 64, 64, A, 0.5, 1.0, A, A, A, None) == sr.SR_ERR_UNSUPPORTED_K
    assert f(A, 512, 60, 64, A, 0.5, 1.0, A, A, A, None) == sr.SR_ERR_SHAPE
    assert f(None, 512, 64, 64, A, 0.5, 1.0, A, A, A, None) == sr.SR_ERR_NULL
    assert f(A, 512, 64, 64, A, 1.5, 1.0, A, A, A, None) == sr.SR_ERR_ARG
    assert f(A + 4, 512, 64, 64, A, 0.5, 1.0, A, A, A, None) == sr.SR_ERR_ALIGN


def test_status_strings():
    for code in range(0, 8):
        assert sr.sr_status_str(code) and sr.sr_status_str(code) != "unknown status"
    assert sr.sr_status_str(99) == "unknown status"


def test_hadamard_supported_orders():
    ok = [64, 128, 512, 4096, 8192, 32768, 448, 896, 14336, 28672]
    bad = [0, -4, 1, 16, 32, 65536, 100, 28, 56, 224, 57344, 12288, 4095, 3 * 4096]
    assert all(sr.sr_hadamard_supported(k) for k in ok)
    assert not any(sr.sr_hadamard_supported(k) for k in bad)


def test_workspace_sizes():
    assert sr.sr_fold_workspace_bytes(4096, 4096) >= 4096 * 4096 * 2 + 2 * 4096 * 4
    assert sr.sr_fold_workspace_bytes(4096, 4096) % 256 == 0
    assert sr.sr_fold_workspace_bytes(100, 64) == 0 and sr.sr_fold_workspace_bytes(4096, 10) == 0
    assert sr.sr_gemm_workspace_bytes(2048, 4096, 4096) == 0


def test_calib_absmax_rejects_bad_arguments():
    f = sr.raw().sr_calib_absmax
    assert f(A, -1, 512, 512, A, None) == sr.SR_ERR_SHAPE
    assert f(A, 4, 512, 256, A, None) == sr.SR_ERR_SHAPE          # ldx < K
    assert f(A, 4, 0, 0, A, None) == sr.SR_ERR_SHAPE
    assert f(A, 4, 516, 520, A, None) == sr.SR_ERR_ALIGN          # K % 8
    assert f(A, 4, 512, 516, A, None) == sr.SR_ERR_ALIGN          # ldx % 8
    assert f(None, 4, 512, 512, A, None) == sr.SR_ERR_NULL
    assert f(A, 4, 512, 512, None, None) == sr.SR_ERR_NULL
    assert f(A + 2, 4, 512, 512, A, None) == sr.SR_ERR_ALIGN
    assert f(None, 0, 512, 512, A, None) == sr.SR_OK               # T = 0: no-op


def test_fold_rejects_bad_arguments():
    f = sr.raw().sr_fold_smooth_rotate_quant
    need = sr.sr_fold_workspace_bytes(512, 64)

    def call(W=A, K=512, N=64, ldw=64, a=A, alpha=0.5, clip=1.0, Wq=A, ws=A, inv=A, wsp=WS, nbytes=need):
        return f(W, K, N, ldw, a, alpha, clip, Wq, ws, inv, wsp, nbytes, None)

    assert call(N=60) == sr.SR_ERR_SHAPE
    assert call(N=0) == sr.SR_ERR_SHAPE
    assert call(ldw=48) == sr.SR_ERR_SHAPE
    assert call(K=500) == sr.SR_ERR_UNSUPPORTED_K
    assert call(K=32) == sr.SR_ERR_UNSUPPORTED_K
    assert call(alpha=1.5) == sr.SR_ERR_ARG
    assert call(alpha=-0.1) == sr.SR_ERR_ARG
    assert call(alpha=float("nan")) == sr.SR_ERR_ARG
    assert call(clip=0.0) == sr.SR_ERR_ARG
    assert call(clip=1.01) == sr.SR_ERR_ARG
    assert call(W=None) == sr.SR_ERR_NULL
    assert call(Wq=None) == sr.SR_ERR_NULL
    assert call(ws=None) == sr.SR_ERR_NULL
    assert call(W=A + 8) == sr.SR_ERR_ALIGN
    assert call(ldw=68) == sr.SR_ERR_ALIGN
    assert call(wsp=None) == sr.SR_ERR_WORKSPACE
    assert call(nbytes=need - 1) == sr.SR_ERR_WORKSPACE
    assert call(wsp=WS + 16) == sr.SR_ERR_WORKSPACE


def test_fwht_quant_rejects_bad_arguments():
    f = sr.raw().sr_fwht_quant_act

    def call(X=A, M=4, K=4096, ldx=4096, inv=None, clip=0.9, Xq=A, xs=A):
        return f(X, M, K, ldx, inv, clip, Xq, xs, None)

    assert call(M=-1) == sr.SR_ERR_SHAPE
    assert call(ldx=2048) == sr.SR_ERR_SHAPE
    assert call(K=4000, ldx=4000) == sr.SR_ERR_UNSUPPORTED_K
    assert call(K=65536, ldx=65536) == sr.SR_ERR_UNSUPPORTED_K
    assert call(clip=0.0) == sr.SR_ERR_ARG
    assert call(clip=2.0) == sr.SR_ERR_ARG
    assert call(M=0, X=None, Xq=None, xs=None) == sr.SR_OK
    assert call(X=None) == sr.SR_ERR_NULL
    assert call(Xq=None) == sr.SR_ERR_NULL
    assert call(xs=None) == sr.SR_ERR_NULL
    assert call(ldx=4100) == sr.SR_ERR_ALIGN
    assert call(X=A + 4) == sr.SR_ERR_ALIGN
    assert call(inv=A + 4) == sr.SR_ERR_ALIGN


def test_gemm_rejects_bad_arguments():
    f = sr.raw().sr_w4a4_gemm

    def call(Xq=A, xs=A, Wq=A, ws=A, M=32, N=64, K=512, Y=A, ldy=64, dt=sr.SR_F16, wsp=WS, nbytes=32 * 512):
        return f(Xq, xs, Wq, ws, M, N, K, Y, ldy, dt, wsp, nbytes, None)

    assert call(M=-1) == sr.SR_ERR_SHAPE
    assert call(N=40) == sr.SR_ERR_SHAPE
    assert call(ldy=32) == sr.SR_ERR_SHAPE
    assert call(K=96) == sr.SR_ERR_UNSUPPORTED_K
    assert call(K=131072) == sr.SR_ERR_UNSUPPORTED_K
    assert call(dt=7) == sr.SR_ERR_ARG
    assert call(M=0) == sr.SR_OK
    assert call(Xq=None) == sr.SR_ERR_NULL
    assert call(Y=None) == sr.SR_ERR_NULL
    assert call(xs=None) == sr.SR_ERR_NULL
    assert call(ldy=68) == sr.SR_ERR_ALIGN
    assert call(Wq=A + 1) == sr.SR_ERR_ALIGN
    assert call(M=70000, N=16, K=65536, ldy=16) == sr.SR_ERR_SHAPE         # 32-bit row offsets


def test_binding_refuses_host_tensors():
    import torch
    with pytest.raises(ValueError):
        sr.sr_fwht_quant_act(torch.zeros(2, 64, dtype=torch.float16), None)


def test_swiglu_rejects_bad_arguments():
    f = sr.raw().sr_swiglu_fwht_quant_act
    assert f(A, A, -1, 512, 512, 512, None, 0.9, A, A, None) == sr.SR_ERR_SHAPE
    assert f(A, A, 4, 512, 256, 512, None, 0.9, A, A, None) == sr.SR_ERR_SHAPE      # ldg < K
    assert f(A, A, 4, 512, 512, 256, None, 0.9, A, A, None) == sr.SR_ERR_SHAPE      # ldu < K
    assert f(A, A, 4, 100, 104, 104, None, 0.9, A, A, None) == sr.SR_ERR_UNSUPPORTED_K
    assert f(A, A, 4, 512, 512, 512, None, 0.0, A, A, None) == sr.SR_ERR_ARG
    assert f(None, A, 4, 512, 512, 512, None, 0.9, A, A, None) == sr.SR_ERR_NULL
    assert f(A, None, 4, 512, 512, 512, None, 0.9, A, A, None) == sr.SR_ERR_NULL
    assert f(A + 2, A, 4, 512, 512, 512, None, 0.9, A, A, None) == sr.SR_ERR_ALIGN
    assert f(A, A, 4, 512, 516, 512, None, 0.9, A, A, None) == sr.SR_ERR_ALIGN
    assert f(None, None, 0, 512, 512, 512, None, 0.9, None, None, None) == sr.SR_OK


def test_heads_rejects_bad_arguments():
    f = sr.raw().sr_fwht_quant_act_heads
    assert f(A, 4, 14336, 14336, 32, 1, None, 0.9, A, A, None) == sr.SR_ERR_UNSUPPORTED_K   # not a power of two
    assert f(A, 4, 4096, 4096, 0, 1, None, 0.9, A, A, None) == sr.SR_ERR_ARG
    assert f(A, 4, 4096, 4096, 24, 1, None, 0.9, A, A, None) == sr.SR_ERR_ARG
    assert f(A, 4, 4096, 4096, 8192, 0, None, 0.9, A, A, None) == sr.SR_ERR_ARG
    assert f(A, 4, 4096, 4096, 32, 1, None, 1.5, A, A, None) == sr.SR_ERR_ARG
    assert f(A, 4, 4096, 2048, 32, 1, None, 0.9, A, A, None) == sr.SR_ERR_SHAPE
    assert f(None, 4, 4096, 4096, 32, 1, None, 0.9, A, A, None) == sr.SR_ERR_NULL
    assert f(None, 0, 4096, 4096, 32, 1, None, 0.9, None, None, None) == sr.SR_OK


def test_fold_ex_rejects_bad_arguments():
    f = sr.raw().sr_fold_smooth_rotate_quant_ex
    need = sr.sr_fold_workspace_bytes(512, 64)
    ok = (A, 512, 64, 64, A, 0.5)
    out = (A, A, A, A, WS, need, None)
    assert f(*ok, 0, 0, 0, 1.0, *out) == sr.SR_ERR_ARG            # clip_steps < 1
    assert f(*ok, 0, 0, 33, 0.5, *out) == sr.SR_ERR_ARG           # clip_steps > 32
    assert f(*ok, 0, 0, 21, 0.0, *out) == sr.SR_ERR_ARG           # clip_lo out of range
    assert f(*ok, 24, 1, 1, 1.0, *out) == sr.SR_ERR_ARG           # n_heads not a power of two
    assert f(*ok, -1, 1, 1, 1.0, *out) == sr.SR_ERR_ARG
    assert f(A, 896, 64, 64, A, 0.5, 8, 1, 1, 1.0, A, A, A, A, WS, 1 << 30, None) == sr.SR_ERR_ARG   # heads need 2^p
    assert f(*ok, 0, 0, 21, 0.5, A, A, A, A, WS, need - 1, None) == sr.SR_ERR_WORKSPACE
    assert f(A, 512, 60, 64, A, 0.5, 0, 0, 1, 1.0, *out) == sr.SR_ERR_SHAPE
    assert f(None, 512, 64, 64, A, 0.5, 0, 0, 1, 1.0, *out) == sr.SR_ERR_NULL


def test_kv_quant_rejects_bad_arguments():
    f = sr.raw().sr_kv_quant_asym
    assert f(A, -1, 1024, 1024, 128, 0.95, A, A, A, None) == sr.SR_ERR_SHAPE
    assert f(A, 4, 1024, 512, 128, 0.95, A, A, A, None) == sr.SR_ERR_SHAPE
    assert f(A, 4, 1000, 1000, 128, 0.95, A, A, A, None) == sr.SR_ERR_SHAPE          # D % group
    assert f(A, 4, 1024, 1024, 100, 0.95, A, A, A, None) == sr.SR_ERR_ARG
    assert f(A, 4, 1024, 1024, 128, 0.0, A, A, A, None) == sr.SR_ERR_ARG
    assert f(None, 4, 1024, 1024, 128, 0.95, A, A, A, None) == sr.SR_ERR_NULL
    assert f(A, 4, 1024, 1024, 128, 0.95, A, None, A, None) == sr.SR_ERR_NULL
    assert f(A + 4, 4, 1024, 1024, 128, 0.95, A, A, A, None) == sr.SR_ERR_ALIGN
    assert f(A, 4, 1024, 1028, 128, 0.95, A, A, A, None) == sr.SR_ERR_ALIGN
    assert f(None, 0, 1024, 1024, 128, 0.95, None, None, None, None) == sr.SR_OK


def test_linear_decode_rejects_bad_arguments():
    f = sr.raw().sr_w4a4_linear_decode
    ok = dict(X=A, M=1, K=4096, ldx=4096, inv=None, clip=0.9, Wq=A, ws=A, N=64, Y=A, ldy=64, xq=None, xs=None,
              wsp=None, wsb=0, st=None)
    def call(**kw):
        a = dict(ok); a.update(kw)
        return f(a["X"], a["M"], a["K"], a["ldx"], a["inv"], a["clip"], a["Wq"], a["ws"], a["N"], a["Y"], a["ldy"],
                 a["xq"], a["xs"], a["wsp"], a["wsb"], a["st"])
    assert call(M=17) == sr.SR_ERR_SHAPE                        # more than sixteen tokens: use the two calls
    assert call(M=-1) == sr.SR_ERR_SHAPE
    assert call(N=40) == sr.SR_ERR_SHAPE
    assert call(ldx=2048) == sr.SR_ERR_SHAPE
    assert call(ldy=32) == sr.SR_ERR_SHAPE
    assert call(K=512, ldx=512) == sr.SR_ERR_UNSUPPORTED_K      # a valid Hadamard order, but not built for this call
    assert call(K=28672, ldx=28672) == sr.SR_ERR_UNSUPPORTED_K
    assert call(K=4000, ldx=4000) == sr.SR_ERR_UNSUPPORTED_K
    assert call(clip=0.0) == sr.SR_ERR_ARG
    assert call(X=None) == sr.SR_ERR_NULL
    assert call(Y=None) == sr.SR_ERR_NULL
    assert call(ws=None) == sr.SR_ERR_NULL
    assert call(X=A + 2) == sr.SR_ERR_ALIGN
    assert call(ldx=4100) == sr.SR_ERR_ALIGN
    assert call(M=0, X=None, Y=None) == sr.SR_OK
    # beyond one token with K = 2048 / 4096 the call runs two kernels and needs its workspace
    assert sr.sr_linear_decode_workspace_bytes(1, 4096) == 0 and sr.sr_linear_decode_workspace_bytes(1, 2048) == 0
    assert sr.sr_linear_decode_workspace_bytes(1, 8192) == 512 + 4096
    assert sr.sr_linear_decode_workspace_bytes(1, 14336) == 512 + 7168
    assert sr.sr_linear_decode_workspace_bytes(16, 4096) == 512 + 16 * 2048
    assert sr.sr_linear_decode_workspace_bytes(17, 4096) == 0 and sr.sr_linear_decode_workspace_bytes(2, 512) == 0
    assert call(M=2, N=4096, ldy=4096) == sr.SR_ERR_WORKSPACE
    assert call(M=2, N=4096, ldy=4096, wsp=WS, wsb=100) == sr.SR_ERR_WORKSPACE
    assert call(M=2, N=4096, ldy=4096, wsp=WS + 16, wsb=1 << 20) == sr.SR_ERR_WORKSPACE
    assert call(K=14336, ldx=14336) == sr.SR_ERR_WORKSPACE
    assert call(M=2, N=4096, ldy=4100, wsp=WS, wsb=1 << 20) == sr.SR_ERR_ALIGN


def test_f6_calls_reject_bad_arguments():
    raw = sr.raw()
    assert raw.sr_f6_tiles_bytes(2048, 4096) == 256 * 32 * 768
    assert raw.sr_f6_tiles_bytes(9, 128) == 2 * 768
    assert raw.sr_f6_tiles_bytes(8, 192) == 0 and raw.sr_f6_tiles_bytes(0, 128) == 0

    def pack(Q4=A, rows=8, K=256, T6=A):
        return raw.sr_pack_f6_tiles(Q4, rows, K, T6, None)
    assert pack(rows=-1) == sr.SR_ERR_SHAPE
    assert pack(K=192) == sr.SR_ERR_UNSUPPORTED_K
    assert pack(rows=0, Q4=None, T6=None) == sr.SR_OK
    assert pack(Q4=None) == sr.SR_ERR_NULL
    assert pack(T6=A + 8) == sr.SR_ERR_ALIGN
    assert pack(rows=70000, K=65536) == sr.SR_ERR_SHAPE

    def quant(X=A, M=4, K=4096, ldx=4096, inv=None, clip=0.9, X6=A, xs=A):
        return raw.sr_fwht_quant_act_f6(X, M, K, ldx, inv, clip, X6, xs, None)
    assert quant(M=-1) == sr.SR_ERR_SHAPE
    assert quant(K=64, ldx=64) == sr.SR_ERR_UNSUPPORTED_K              # a Hadamard order, but not a multiple of 128
    assert quant(K=448, ldx=448) == sr.SR_ERR_UNSUPPORTED_K
    assert quant(K=4000, ldx=4000) == sr.SR_ERR_UNSUPPORTED_K
    assert quant(clip=0.0) == sr.SR_ERR_ARG
    assert quant(M=0, X=None, X6=None, xs=None) == sr.SR_OK
    assert quant(X6=None) == sr.SR_ERR_NULL
    assert quant(X6=A + 4) == sr.SR_ERR_ALIGN

    def swiglu(G=A, U=A, M=4, K=14336, ldg=14336, ldu=14336, inv=None, clip=0.9, X6=A, xs=A):
        return raw.sr_swiglu_fwht_quant_act_f6(G, U, M, K, ldg, ldu, inv, clip, X6, xs, None)
    assert swiglu(ldg=4096) == sr.SR_ERR_SHAPE
    assert swiglu(K=448, ldg=448, ldu=448) == sr.SR_ERR_UNSUPPORTED_K
    assert swiglu(clip=1.5) == sr.SR_ERR_ARG
    assert swiglu(G=None) == sr.SR_ERR_NULL
    assert swiglu(X6=A + 2) == sr.SR_ERR_ALIGN
    assert swiglu(M=0) == sr.SR_OK

    def gemm(X6=A, xs=A, W6=A, ws=A, M=32, N=64, K=512, Y=A, ldy=64, dt=sr.SR_F16):
        return raw.sr_w4a4_gemm_f6(X6, xs, W6, ws, M, N, K, Y, ldy, dt, None, 0, None)
    assert gemm(M=-1) == sr.SR_ERR_SHAPE
    assert gemm(N=40) == sr.SR_ERR_SHAPE
    assert gemm(ldy=32) == sr.SR_ERR_SHAPE
    assert gemm(K=192) == sr.SR_ERR_UNSUPPORTED_K
    assert gemm(K=131072) == sr.SR_ERR_UNSUPPORTED_K
    assert gemm(dt=7) == sr.SR_ERR_ARG
    assert gemm(M=0) == sr.SR_OK
    assert gemm(X6=None) == sr.SR_ERR_NULL
    assert gemm(xs=None) == sr.SR_ERR_NULL
    assert gemm(ldy=68) == sr.SR_ERR_ALIGN
    assert gemm(W6=A + 1) == sr.SR_ERR_ALIGN


def test_generated_h28_program_is_the_oracles_paley_matrix():
    """The kernels multiply by H28 with a generated list of additions (csrc/h28_program.h).  Read as
    text and evaluated in integers on the 28 unit vectors, it must give the oracle's Paley matrix
    (paper: online Hadamard of the down-projection input, 14336 = 28 * 512), entry by entry."""
    import numpy as np
    from oracle import smoothrot_oracle as orc

    text = open(os.path.join(ROOT, "paper_2506_05413_amd", "csrc", "h28_program.h")).read()
    shared = re.findall(r"const T (w\d+) = (\S+) ([+-]) (\S+);", text)
    outs = re.findall(r"o\[(\d+)\] = (.+);", text)
    assert len(outs) == 28 and sorted(int(j) for j, _ in outs) == list(range(28))

    H = np.zeros((28, 28), dtype=np.int64)
    n_ops = len(shared)
    for i in range(28):
        val = {"v[%d]" % k: int(k == i) for k in range(28)}
        for name, a, op, b in shared:
            val[name] = val[a] + val[b] if op == "+" else val[a] - val[b]
        for j, expr in outs:
            terms = re.findall(r"([+-]?)\s*(v\[\d+\]|w\d+)", expr)
            H[i, int(j)] = sum(-val[t] if sg == "-" else val[t] for sg, t in terms)
            if i == 0:
                n_ops += len(terms) - 1
    assert np.array_equal(H, orc.paley28())
    assert n_ops < 28 * 14                     # fewer additions than "row sum minus twice the negative terms"


def test_bench_refuses_more_than_one_gpu():
    """Nothing here spans GPUs: bench.py --gpus N with N > 1 (or under a multi-rank launcher) must say so and
    exit with an error before it touches a device."""
    import subprocess
    import sys

    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in (r.stdout + r.stderr)
    env = dict(os.environ, WORLD_SIZE="2")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, timeout=120,
                       env=env)
    assert r.returncode != 0 and "ONE GPU" in (r.stdout + r.stderr)


def test_binding_fails_loudly_without_the_library():
    """There is no fallback path: with the shared library out of reach the first call raises, and neither the
    package nor the binding imports anything of the oracle."""
    import subprocess
    import sys

    code = (
        "import sys; sys.path.insert(0, %r)\n"
        "import paper_2506_05413_amd as sr, paper_2506_05413_amd.binding as b\n"
        "assert not any(m == 'oracle' or m.startswith('oracle.') for m in sys.modules)\n"
        "b.LIB_PATH = b.LIB_PATH + '.absent'\n"
        "try:\n"
        "    sr.sr_hadamard_supported(4096)\n"
        "except ImportError as e:\n"
        "    assert 'no fallback' in str(e); print('RAISED')\n"
    ) % ROOT
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "RAISED" in r.stdout, r.stderr


def test_cache_warming_quantiser_rejects_bad_hints():
    raw = sr.raw()

    def call(X=A, M=32, K=4096, ldx=4096, inv=A, clip=0.9, X6=A, xs=A, nxt=A, nbytes=4096):
        return raw.sr_fwht_quant_act_f6_warm(X, M, K, ldx, inv, clip, X6, xs, nxt, nbytes, None)
    assert call(nxt=None) == sr.SR_ERR_NULL
    assert call(nxt=A + 4) == sr.SR_ERR_ALIGN
    assert call(K=192) == sr.SR_ERR_UNSUPPORTED_K
    assert call(clip=0.0) == sr.SR_ERR_ARG
    assert call(ldx=100) == sr.SR_ERR_SHAPE
    assert call(X=None) == sr.SR_ERR_NULL
    assert call(M=0) == sr.SR_OK
    assert call(M=0, nxt=None, nbytes=0) == sr.SR_OK



def test_cache_warming_gemm_rejects_bad_hints():
    raw = sr.raw()

    def call(X6=A, xs=A, W6=A, ws=A, M=32, N=64, K=256, Y=A, ldy=64, dt=None, nxt=A, nbytes=4096):
        return raw.sr_w4a4_gemm_f6_warm(X6, xs, W6, ws, M, N, K, Y, ldy, sr.SR_F16 if dt is None else dt, nxt, nbytes,
                                        None, 0, None)
    assert call(nxt=None) == sr.SR_ERR_NULL
    assert call(nxt=A + 4) == sr.SR_ERR_ALIGN
    assert call(K=192) == sr.SR_ERR_UNSUPPORTED_K
    assert call(N=60) == sr.SR_ERR_SHAPE
    assert call(ldy=32) == sr.SR_ERR_SHAPE
    assert call(dt=7) == sr.SR_ERR_ARG
    assert call(X6=None) == sr.SR_ERR_NULL
    assert call(xs=None) == sr.SR_ERR_NULL
    assert call(ldy=68) == sr.SR_ERR_ALIGN
    assert call(M=0) == sr.SR_OK
    assert call(M=0, nxt=None, nbytes=0) == sr.SR_OK


def test_header_is_plain_c_and_cpp():
    """include/smoothrot.h is the boundary: it must compile on its own as C99 and as C++ (no HIP, no torch types),
    and a C program must be able to link a call against the library."""
    import subprocess, tempfile
    inc = os.path.join(ROOT, "include")
    with tempfile.TemporaryDirectory() as d:
        c = os.path.join(d, "t.c")
        with open(c, "w") as f:
            f.write('#include "smoothrot.h"\nint main(void) { return sr_hadamard_supported(14336) == 1 && '
                    'sr_hadamard_supported(100) == 0 && sr_f6_tiles_bytes(8, 128) == 768 ? 0 : 1; }\n')
        r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", inc, "-fsyntax-only", c], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
        r = subprocess.run(["g++", "-std=c++11", "-Wall", "-Werror", "-I", inc, "-x", "c++", "-fsyntax-only", c], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
        exe = os.path.join(d, "t")
        lib_dir = os.path.dirname(sr.LIB_PATH)
        r = subprocess.run(["gcc", "-std=c99", "-I", inc, c, "-o", exe, "-L", lib_dir, "-lsmoothrot", "-Wl,-rpath," + lib_dir],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
        r = subprocess.run([exe], capture_output=True, text=True)
        assert r.returncode == 0, (r.returncode, r.stderr)
