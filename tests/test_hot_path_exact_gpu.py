"""Exact-arithmetic parity on the hot loop of every tile configuration.

Inputs are integers in [-8, 8] and K = 4096, so every partial sum is an integer below 2^24 and exact in fp32
in any summation order: the GPU result must equal the oracle bit for bit.  The sizes are chosen so that even
the 256 x 256 tiles run their unguarded path: 768 x 512 is whole tiles of every configuration (direct
global -> LDS transfers only), 784 x 528 adds edge tiles that are moved back inside the matrix.  A dropped or
doubled K step, a tile read from the wrong place or a fragment fed to the wrong MFMA block changes integers
and cannot hide below a floating-point tolerance.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2310_17408_amd as mg
from gpu_case import DT, LAYOUT, to_device

pytestmark = pytest.mark.gpu

K = 4096
SHAPES = [(768, 512), (784, 528)]
GEN = {"f32": wl.small_int_f32, "f16": wl.small_int_f16_bits, "bf16": wl.small_int_bf16_bits, "i8": wl.uniform_i8}


def _problem(dtype, layout, ta, tb, M, N, seed):
    ar, ac = (K, M) if ta else (M, K)
    br, bc = (N, K) if tb else (K, N)
    lda, ldb, ldc = wl.tight_ld(layout, ar, ac), wl.tight_ld(layout, br, bc), wl.tight_ld(layout, M, N)
    A, B = GEN[dtype](seed, layout, ar, ac, lda), GEN[dtype](seed + 1, layout, br, bc, ldb)
    C = wl.uniform_i32(seed + 2, layout, M, N, ldc) if dtype == "i8" else wl.small_int_f32(seed + 2, layout, M, N, ldc)
    return A, lda, B, ldb, C, ldc


def _every_kernel_exact(dtype, layout, ta, tb, M, N, alpha, beta, seed, want_all):
    """The oracle once, then every configuration forced in turn on the same operands."""
    A, lda, B, ldb, C, ldc = _problem(dtype, layout, ta, tb, M, N, seed)
    ref = oracle.gemm_ex(dtype, layout, ta, tb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc)
    ref = oracle.wrap_int32(ref) if dtype == "i8" else ref
    _, dA = to_device(A)
    _, dB = to_device(B)
    ws = torch.empty(max(mg.gemm_workspace_bytes(DT[dtype], M, N, K), 16), dtype=torch.uint8, device="cuda")
    ran = set()
    for kid in [-1] + list(range(mg.gemm_kernel_count(DT[dtype]))):
        _, dC = to_device(C)
        mg.gemm_force_kernel(DT[dtype], kid, 1 if kid >= 0 else 0)
        try:
            mg.gemm_ex(DT[dtype], LAYOUT[layout], ta, tb, M, N, K, alpha, dA, lda, dB, ldb, beta, dC, ldc, ws)
            k, s = mg.gemm_last_kernel_id(), mg.gemm_last_split()
        finally:
            mg.gemm_force_kernel(DT[dtype], -1, 0)
        torch.cuda.synchronize()
        got = wl.logical(layout, dC.cpu().numpy().reshape(C.shape), M, N)
        what = "%s %s ta=%d tb=%d %dx%dx%d kernel %s split %d" % (dtype, layout, ta, tb, M, N, K,
                                                                mg.gemm_kernel_name(DT[dtype], k), s)
        assert np.array_equal(got.astype(ref.dtype), ref), what
        if kid >= 0:
            if want_all:
                assert k == kid, what          # canonical operands: a forced configuration is the one that runs
            ran.add(k)
    return ran


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i8"])
@pytest.mark.parametrize("layout", ["col", "row"])
@pytest.mark.parametrize("M,N", SHAPES)
def test_every_kernel_hot_loop_exact(dtype, layout, M, N):
    a, b = (2, -1) if dtype == "i8" else (2.0, -1.0)
    ran = _every_kernel_exact(dtype, layout, 0, 0, M, N, a, b, 9500, want_all=True)
    assert len(ran) == mg.gemm_kernel_count(DT[dtype])


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i8"])
@pytest.mark.parametrize("ta,tb", [(1, 0), (0, 1), (1, 1)])
def test_transposed_operands_hot_loop_exact(dtype, ta, tb):
    """The same through gemm_ex: the configurations that take the orientation run it, the others are
    replaced by one that does; all results exact.  The direct 16- and 8-bit kernels must be among those
    that ran."""
    for (M, N) in SHAPES:
        a, b = (1, 1) if dtype == "i8" else (0.5, 2.0)
        ran = _every_kernel_exact(dtype, "col", ta, tb, M, N, a, b, 9600, want_all=False)
        names = {mg.gemm_kernel_name(DT[dtype], k) for k in ran}
        if dtype != "f32":
            assert any(n.endswith("256x256_w128x64_dma16") for n in names), names
            assert any(n.endswith("256x256_w128x64_ring") for n in names), names
