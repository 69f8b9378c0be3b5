"""Sanitizer builds of the host-side code (no GPU): the C oracle and the library's host logic (argument checks,
quick returns, selection model, workspace sizing, convolution geometry) compiled with AddressSanitizer and
UndefinedBehaviorSanitizer and run on edge inputs - the largest legal sizes, leading dimensions beyond 32-bit
byte offsets, geometries whose products overflow 32 bits.  The kernels are stand-ins that record launches."""
import os
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _run(cmd, **kw):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=ENV, **kw)
    assert p.returncode == 0, "%s\n%s" % (" ".join(cmd), p.stdout[-4000:])
    return p.stdout


def test_host_logic_under_sanitizers(tmp_path):
    exe = str(tmp_path / "host_driver")
    _run(["g++", "-std=c++17", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include"] + SAN +
         [os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"),
          os.path.join(ROOT, "paper_2310_17408_amd", "csrc", "gemm_api.cpp"), "-o", exe])
    out = _run([exe])
    assert out.strip().splitlines()[-1].startswith("ok"), out


def test_oracle_under_sanitizers(tmp_path):
    """The oracle's C code on ragged shapes with padded leading dimensions, in a child process that loads the
    sanitized build (the sanitizer runtime must be loaded before anything else)."""
    lib = str(tmp_path / "libref_san.so")
    _run(["gcc", "-std=c99", "-shared", "-fPIC", "-fopenmp"] + SAN +
         [os.path.join(ROOT, "oracle", "ref_gemm.c"), os.path.join(ROOT, "oracle", "ref_conv.c"), "-lm", "-o", lib])
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    if not os.path.isabs(asan):
        pytest.skip("no shared AddressSanitizer runtime in this toolchain")
    code = r'''
import ctypes, sys
import numpy as np
sys.path.insert(0, %r)
import oracle.ref as ref
ref._LIB = %r                 # newer than the sources, so the loader takes it as it is
import oracle, workloads as wl
for layout in ("col", "row"):
    M, N, K = 37, 29, 53
    lda, ldb, ldc = wl.tight_ld(layout, M, K) + 3, wl.tight_ld(layout, K, N) + 1, wl.tight_ld(layout, M, N) + 2
    A, B, C = wl.uniform_f32(1, layout, M, K, lda), wl.uniform_f32(2, layout, K, N, ldb), wl.uniform_f32(3, layout, M, N, ldc)
    r = oracle.gemm_f32(layout, M, N, K, np.float32(1.5), A, lda, B, ldb, np.float32(0.5), C, ldc)
    assert r.shape == (M, N)
    Ah, Bh = wl.normal_f16_bits(4, layout, M, K, lda), wl.normal_f16_bits(5, layout, K, N, ldb)
    oracle.gemm_f16(layout, M, N, K, np.float32(1), Ah, lda, Bh, ldb, np.float32(0), None, ldc)
    oracle.gemm_bf16(layout, M, N, K, np.float32(1), wl.normal_bf16_bits(6, layout, M, K, lda), lda,
                     wl.normal_bf16_bits(7, layout, K, N, ldb), ldb, np.float32(0), None, ldc)
    Ai, Bi = wl.uniform_i8(8, layout, M, K, lda), wl.uniform_i8(9, layout, K, N, ldb)
    oracle.gemm_i8(layout, M, N, K, 2, Ai, lda, Bi, ldb, -1, wl.uniform_i32(10, layout, M, N, ldc), ldc)
    for ta in (0, 1):
        for tb in (0, 1):
            ar, ac = (K, M) if ta else (M, K)
            br, bc = (N, K) if tb else (K, N)
            oracle.gemm_ex("f32", layout, ta, tb, M, N, K, 1.0, wl.uniform_f32(11, layout, ar, ac), wl.tight_ld(layout, ar, ac),
                           wl.uniform_f32(12, layout, br, bc), wl.tight_ld(layout, br, bc), 0.0, None, wl.tight_ld(layout, M, N))
    rows, cols = np.array([0, M - 1, 5]), np.array([N - 1, 0, 7])
    oracle.gemm_sample("f32", layout, K, np.float32(1.5), A, lda, B, ldb, np.float32(0.5), C, ldc, rows, cols)
image, filt, _ = wl.conv_tensors_f32(13, 2, 9, 7, 5, 6, 3, 3, 5, 4)
oracle.conv2d_nhwc_f32(image, filt, (2, 2), (1, 1))
oracle.im2row_f32(image, 3, 3, (2, 2), (1, 1))
print("ok")
''' % (ROOT, lib)
    env = dict(ENV, LD_PRELOAD=asan, ASAN_OPTIONS="detect_leaks=0")      # CPython itself is not leak-clean
    p = subprocess.run([sys.executable, "-c", code], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env)
    assert p.returncode == 0 and p.stdout.strip().endswith("ok"), p.stdout[-4000:]
