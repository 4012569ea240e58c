"""The oracle's C file under AddressSanitizer + UndefinedBehaviorSanitizer on the CPU: a small driver (heap buffers
of exactly the operand sizes, so that any access past an end is caught) runs the ragged-shape pin and the result
must still equal the numpy triple-sum.  Host code only; nothing here touches a GPU."""
import os
import shutil
import subprocess

import numpy as np
import pytest

import workloads as wl
from oracle import smoothrot_oracle as o

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
C_SRC = os.path.join(ROOT, "oracle", "gemm_i4.c")

DRIVER = r'''
#include <stdio.h>
#include <stdlib.h>
#include <stdint.h>
int oracle_gemm_i4(const int8_t *cx, const int8_t *cw, int64_t M, int64_t N, int64_t K, int64_t *acc);
int main(int argc, char **argv)
{
    if (argc != 6) return 2;
    const int64_t M = atoll(argv[1]), N = atoll(argv[2]), K = atoll(argv[3]);
    int8_t *cx = malloc((size_t)(M * K)), *cw = malloc((size_t)(N * K));
    int64_t *acc = malloc((size_t)(M * N) * sizeof(int64_t));
    FILE *f = fopen(argv[4], "rb");
    if (!f || fread(cx, 1, (size_t)(M * K), f) != (size_t)(M * K) || fread(cw, 1, (size_t)(N * K), f) != (size_t)(N * K)) return 3;
    fclose(f);
    const int rc = oracle_gemm_i4(cx, cw, M, N, K, acc);
    f = fopen(argv[5], "wb");
    if (!f || fwrite(acc, sizeof(int64_t), (size_t)(M * N), f) != (size_t)(M * N)) return 4;
    fclose(f);
    free(cx); free(cw); free(acc);
    return rc ? 10 : 0;
}
'''


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no gcc")
def test_gemm_c_under_address_and_ub_sanitizers(tmp_path):
    drv = tmp_path / "driver.c"
    drv.write_text(DRIVER)
    exe = tmp_path / "gemm_asan"
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-o", str(exe), str(drv), C_SRC])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0", OMP_NUM_THREADS="4")
    for seed, (M, N, K) in enumerate([(37, 53, 320), (1, 16, 64), (5, 3, 7)]):
        cx, cw = wl.random_codes(10 + seed, M, K), wl.random_codes(20 + seed, N, K)
        fin, fout = tmp_path / "in.bin", tmp_path / "out.bin"
        fin.write_bytes(cx.astype(np.int8).tobytes() + cw.astype(np.int8).tobytes())
        r = subprocess.run([str(exe), str(M), str(N), str(K), str(fin), str(fout)], env=env, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        acc = np.frombuffer(fout.read_bytes(), dtype=np.int64).reshape(M, N)
        assert np.array_equal(acc, o.gemm_i32(cx, cw))
    # the overflow report (an accumulator outside int32) under the sanitizers as well: all -8 against all -8
    cx = np.full((1, 2 ** 25 + 64), -8, np.int8)           # 64 K > 2^31
    fin.write_bytes(cx.tobytes() + cx.tobytes())
    r = subprocess.run([str(exe), "1", "1", str(cx.shape[1]), str(fin), str(fout)], env=env, capture_output=True, text=True)
    assert r.returncode == 10, r.stderr[-2000:]
