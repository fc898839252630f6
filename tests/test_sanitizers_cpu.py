"""The plain-C oracle and the host side of the C ABI under AddressSanitizer and
UndefinedBehaviorSanitizer (host code only; no GPU is touched).  Each is built into a small
executable of its own and run as a child process: a sanitizer report ends it with a
non-zero status."""
import os
import shutil
import struct
import subprocess
import sys

import numpy as np
import pytest

from oracle import c_oracle
from paper_2502_06766_amd import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="4")
ENV.pop("LD_PRELOAD", None)      # the sanitizer runtime must come first among the loaded libraries


def _cases():
    g = np.random.default_rng(77)
    shapes = [  # dtype, M, Hq, Hkv, d, N, causal, k, window
        (wl.F32, 1, 1, 1, 64, 1, 0, 1, 0),          # one token
        (wl.F16, 1, 8, 2, 128, 333, 0, 40, 0),
        (wl.BF16, 1, 4, 4, 32, 65, 0, 90, 0),       # k > N
        (wl.F16, 1, 6, 2, 64, 200, 0, 10, 57),      # window
        (wl.BF16, 1, 4, 1, 32, 50, 0, 7, 50),       # window covers everything: nothing searched
        (wl.F32, 1, 2, 1, 16, 50, 0, 7, 80),        # window beyond the cache
        (wl.F16, 3, 4, 2, 64, 120, 1, 16, 0),       # causal chunk
        (wl.BF16, 4, 2, 2, 32, 4, 1, 3, 2),         # causal chunk as long as the cache, with a window
        (wl.F32, 2, 4, 2, 32, 90, 0, 200, 5),       # non-causal chunk, k > N
    ]
    out = []
    for dtype, M, Hq, Hkv, d, N, causal, k, window in shapes:
        q = wl.quantize(g.standard_normal((M, Hq, d)).astype(np.float32), dtype)
        K = wl.quantize(g.standard_normal((Hkv, N, d)).astype(np.float32), dtype)
        V = wl.quantize(g.standard_normal((Hkv, N, d)).astype(np.float32), dtype)
        K[:, N // 2] = K[:, 0]                      # a duplicate key: the tie rule runs too
        out.append(((dtype, M, Hq, Hkv, d, N, causal, k, window), q, K, V))
    return out


def test_c_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.check_call(["gcc", *SAN, "-fopenmp", "-Wall", "-Wextra", "-o", exe,
                           os.path.join(HERE, "sanitize_oracle_driver.c"),
                           os.path.join(ROOT, "oracle", "topk_attn_oracle.c"), "-lm"])
    cases = _cases()
    fin, fout = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(fin, "wb") as f:
        f.write(struct.pack("<q", len(cases)))
        for hd, q, K, V in cases:
            f.write(struct.pack("<9q", *hd))
            for a in (q, K, V):
                f.write(np.ascontiguousarray(a).tobytes())
    r = subprocess.run([exe, fin, fout], env=ENV, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, f"sanitizer run failed ({r.returncode}):\n{r.stderr[-4000:]}"
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    raw = open(fout, "rb").read()
    off = 0

    def take(n, dt):
        nonlocal off
        a = np.frombuffer(raw, dtype=dt, count=n, offset=off)
        off += a.nbytes
        return a

    for (dtype, M, Hq, Hkv, d, N, causal, k, window), q, K, V in cases:
        assert take(1, np.int64)[0] == 0
        out, idx = take(M * Hq * d, np.float64).reshape(M, Hq, d), take(M * Hq * k, np.int64).reshape(M, Hq, k)
        vals, lse = take(M * Hq * k, np.float64).reshape(M, Hq, k), take(M * Hq, np.float64).reshape(M, Hq)
        S = take(Hq * N, np.float64).reshape(Hq, N)
        ref = c_oracle.topk_attention_multi(q, K, V, dtype, k, bool(causal), window)
        for got, want in zip((out, idx, vals, lse), ref):
            np.testing.assert_array_equal(got, want)      # same code, same thread-independent arithmetic
        np.testing.assert_array_equal(S, c_oracle.scores(q[0], K, dtype))
    assert off == len(raw)


HIPCC = "/opt/rocm/bin/hipcc"


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_host_side_of_the_abi_under_asan_and_ubsan(tmp_path):
    """api.hip (handle, argument checks, workspace layout, k schedule) with sanitized host code, linked
    with stand-ins for the kernel launchers of the other translation units; the driver walks the
    calls that need no device and the error paths of those that do."""
    obj, exe = str(tmp_path / "api_san.o"), str(tmp_path / "abi_san")
    host_san = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"):
        host_san += ["-Xarch_host", f]
    common = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", *host_san,
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    subprocess.check_call([*common, "-c", os.path.join(ROOT, "paper_2502_06766_amd", "csrc", "api.hip"), "-o", obj],
                          stderr=subprocess.DEVNULL)
    drv = str(tmp_path / "driver_san.o")
    subprocess.check_call([*common, "-c", os.path.join(HERE, "sanitize_abi_driver.hip"), "-o", drv],
                          stderr=subprocess.DEVNULL)
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-fno-gpu-sanitize", "-fsanitize=address",
                           "-fsanitize=undefined", drv, obj, "-o", exe], stderr=subprocess.DEVNULL)
    env = dict(ENV, ASAN_OPTIONS=ENV["ASAN_OPTIONS"] + ":protect_shadow_gap=0",
               LSAN_OPTIONS="suppressions=" + os.path.join(HERE, "sanitize_lsan.supp") + ":print_suppressions=0",
               HIP_VISIBLE_DEVICES="", ROCR_VISIBLE_DEVICES="")   # host paths only, also on a GPU machine
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, f"sanitizer run failed ({r.returncode}):\n{r.stdout[-2000:]}\n{r.stderr[-4000:]}"
    assert "runtime error" not in r.stderr and "ERROR: AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    assert "abi driver: all checks passed" in r.stdout
