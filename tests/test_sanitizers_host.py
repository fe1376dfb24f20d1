"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

Two small programs are compiled here and run once each:

* the CPU oracle (``oracle/conv_ref.c``, ``oracle/bn_ref.c``) over odd shapes in all three input
  types, with buffers exactly as large as the tensors; its checksums must equal
  those of the ordinary (unsanitized) oracle library;
* the C ABI's host side (``csrc/api.cpp``: validation, dispatch, workspace
  rules) with the kernel families replaced by stubs, over the rejection table
  and shape arithmetic at the integer limits.

Device code is not sanitized (not available for this GPU); only host code is.
"""
import os
import shutil
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="2")
ENV.pop("LD_PRELOAD", None)     # the sanitizer runtime has to be the first library of the process


def run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert res.returncode == 0, f"{' '.join(cmd)}\n{res.stdout}\n{res.stderr}"
    return res.stdout


def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    run(["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-o", exe,
         os.path.join(SAN, "oracle_driver.c"), os.path.join(ROOT, "oracle", "conv_ref.c"),
         os.path.join(ROOT, "oracle", "bn_ref.c"), "-lm"])
    lines = run([exe], env=ENV).split("\n")
    assert lines[-2] == "ok"
    got = {(int(a), int(b)): (float(c), float(d), float(e)) for a, b, c, d, e in (l.split() for l in lines[:-2])}
    assert len(got) == 27

    # the same problems through the ordinary oracle library
    from oracle import convref as ref
    cases = [(2, 3, 7, 6, 4, 3, 3, 1, 1, 1, 1, 1), (1, 4, 9, 8, 6, 3, 2, 2, 1, 0, 1, 2), (2, 6, 8, 11, 6, 1, 3, 1, 3, 0, 2, 3),
             (1, 2, 12, 12, 2, 5, 5, 2, 2, 2, 2, 2), (2, 3, 13, 9, 5, 4, 3, 3, 2, 1, 0, 1), (1, 8, 6, 6, 8, 3, 3, 1, 1, 1, 1, 8),
             (2, 5, 8, 8, 7, 3, 3, 3, 3, 0, 0, 1), (1, 2, 10, 7, 4, 3, 3, 1, 1, 3, 2, 1), (5, 1, 1, 1, 3, 1, 1, 1, 1, 0, 0, 1)]

    def tensor(n, seed):
        s, out = seed, np.empty(n, dtype=np.float64)
        for i in range(n):
            s = (s * 1664525 + 1013904223) & 0xFFFFFFFF
            out[i] = float(np.fmod(s >> 24, 17)) - 8.0      # C's % on a non-negative int
        return out

    def checksum(a):
        a = a.reshape(-1)
        return float(np.sum(a * (np.arange(a.size) % 13 + 1)))

    for ci, (N, C, H, W, K, R, S, sh, sw, ph, pw, g) in enumerate(cases):
        P, Q = (H + 2 * ph - R) // sh + 1, (W + 2 * pw - S) // sw + 1
        x = tensor(N * C * H * W, 11 + ci).reshape(N, C, H, W)
        w = tensor(K * (C // g) * R * S, 23 + ci).reshape(K, C // g, R, S)
        dy = tensor(N * K * P * Q, 37 + ci).reshape(N, K, P, Q)
        want = (checksum(ref.conv2d_fwd(x, w, (sh, sw), (ph, pw), g)),
                checksum(ref.conv2d_bwd_data(dy, w, x.shape, (sh, sw), (ph, pw), g)),
                checksum(ref.conv2d_bwd_weight(x, dy, w.shape, (sh, sw), (ph, pw), g)))
        for dtype in range(3):     # small integers are exact in bf16, fp32 and fp64 alike
            assert got[(ci, dtype)] == want, (ci, dtype, got[(ci, dtype)], want)


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not installed")
def test_abi_validation_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "abi_san")
    host = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
            "-Xarch_host", "-fno-sanitize-recover=all"]
    run(["hipcc", "-x", "hip", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fno-gpu-sanitize"] + host +
        ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"),
         os.path.join(SAN, "abi_driver.cpp"), os.path.join(ROOT, "paper_1912_01703_amd", "csrc", "api.cpp"),
         "-o", exe])
    out = run([exe], env=ENV)
    assert out.strip().split("\n")[-1] == "ok", out
