"""GPU parity tests: the HIP library, called through its C-ABI binding, against
the CPU oracle, element by element, on seeded inputs.

Bars: int8 bit-exact; floating point max|C - C_ref| / (K max|A| max|B|) <= 1e-6
(fp32) and <= 2e-3 (binary16 inputs, fp32 accumulation); inputs made of small
integers must match exactly in every data type.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2310_17408_amd as mg
from gpu_case import DT, LAYOUT, check_case, gpu_gemm, make_inputs, oracle_gemm, to_device

pytestmark = pytest.mark.gpu

DTYPES = ["f32", "f16", "i8", "bf16"]
LAYOUTS = ["col", "row"]


def _kernels(dtype):
    return list(range(mg.gemm_kernel_count(DT[dtype])))


# ------------------------------------------------------------ configuration 1
def test_f32_256_cube_col_major():
    check_case("f32", "col", 256, 256, 256, 1.0, 0.0, seed=1000)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("layout", LAYOUTS)
def test_7x5x3(dtype, layout):
    check_case(dtype, layout, 7, 5, 3, 1, 0, seed=1001)
    check_case(dtype, layout, 7, 5, 3, 2, -1, seed=1002, pad=(1, 2, 3))


# ------------------------------------------------------------ every tile configuration
@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("layout", LAYOUTS)
def test_every_kernel_aligned_multi_tile(dtype, layout):
    """Sizes that span several tiles of every configuration, multiples of 16 bytes (vector loaders)."""
    for kid in _kernels(dtype):
        got, _ = check_case(dtype, layout, 512, 768, 384, 1.5 if dtype != "i8" else 3, 0.5 if dtype != "i8" else -2,
                            seed=2000 + kid, kernel_id=kid)
        assert got == kid


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("layout", LAYOUTS)
def test_every_kernel_ragged(dtype, layout):
    """Ragged M, N, K (edge tiles, K tail) with aligned and with odd leading dimensions."""
    for kid in _kernels(dtype):
        check_case(dtype, layout, 300, 270, 200, 1, 0, seed=2100 + kid, kernel_id=kid, pad=(4, 8, 12) if dtype == "f32" else (16, 32, 4))
        check_case(dtype, layout, 333, 259, 131, 1, 1, seed=2200 + kid, kernel_id=kid, pad=(1, 2, 3))
        check_case(dtype, layout, 257, 129, 65, 2, -1, seed=2300 + kid, kernel_id=kid, offsets=(1, 3, 1))


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("layout", LAYOUTS)
def test_every_kernel_edge_tiles_with_aligned_rows(dtype, layout):
    """M and N that are multiples of 16 elements but of no tile size: the edge tiles of the direct
    kernels overlap their neighbours and must store only their own part (beta != 0, also with K split)."""
    for kid in _kernels(dtype):
        a, b = (1.5, 0.5) if dtype != "i8" else (3, -2)
        check_case(dtype, layout, 304, 272, 256, a, b, seed=2500 + kid, kernel_id=kid)
        check_case(dtype, layout, 336, 80, 1280, a, b, seed=2600 + kid, kernel_id=kid, split=3)


@pytest.mark.parametrize("dtype", DTYPES)
def test_tile_minus_plus_one(dtype):
    for kid in _kernels(dtype):
        for d in (-1, 1):
            check_case(dtype, "col", 256 + d, 256 - d, 128 + d, 1, 0, seed=2400 + kid, kernel_id=kid)


# ------------------------------------------------------------ split K
@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("layout", LAYOUTS)
def test_split_k(dtype, layout):
    for kid in _kernels(dtype):
        for split in (2, 5):
            k, s = check_case(dtype, layout, 200, 136, 2100, 1, 1, seed=3000 + kid, kernel_id=kid, split=split)
            assert s > 1
    # automatic selection on a skinny problem splits K, over workgroups or over the waves that share
    # a tile in a register-direct kernel; no workspace falls back to no split over workgroups
    k, s = check_case(dtype, layout, 49, 512, 4608, 1, 0, seed=3100)
    assert s > 1 or "_k" in mg.gemm_kernel_name(DT[dtype], k)
    k, s = check_case(dtype, layout, 49, 512, 4608, 1, 0, seed=3100, workspace_bytes=0)
    assert s == 1


def test_split_k_invariance_int8_and_determinism():
    A, lda, B, ldb, C, ldc = make_inputs("i8", "col", 130, 70, 3000, 3200)
    outs = [gpu_gemm("i8", "col", 130, 70, 3000, 1, A, lda, B, ldb, 0, C, ldc, kernel_id=k, split=s)[0]
            for k in _kernels("i8") for s in (1, 3)]
    for o in outs[1:]:
        assert np.array_equal(o, outs[0])
    A, lda, B, ldb, C, ldc = make_inputs("f32", "col", 130, 70, 3000, 3300)
    a = gpu_gemm("f32", "col", 130, 70, 3000, np.float32(1), A, lda, B, ldb, np.float32(0), C, ldc, split=4)[0]
    b = gpu_gemm("f32", "col", 130, 70, 3000, np.float32(1), A, lda, B, ldb, np.float32(0), C, ldc, split=4)[0]
    assert np.array_equal(a, b)


# ------------------------------------------------------------ exact regimes
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("alpha,beta", [(1, 0), (2, -1), (0.5, 1), (-1, 2)])
def test_small_integer_inputs_exact(dtype, layout, alpha, beta):
    for kid in _kernels(dtype):
        check_case(dtype, layout, 150, 140, 4096, alpha, beta, seed=4000 + kid, kernel_id=kid, values="smallint",
                   exact=True)


@pytest.mark.parametrize("layout", LAYOUTS)
def test_identity_and_permutation(layout):
    n, N = 200, 150
    rng = np.random.default_rng(7)
    perm = rng.permutation(n)
    P = np.zeros((n, n), dtype=np.float32)
    P[np.arange(n), perm] = 1.0
    Bl = rng.standard_normal((n, N)).astype(np.float32)

    def buf(x, dt=np.float32):
        return np.ascontiguousarray((x.T if layout == "col" else x).astype(dt))

    ldp, ldb = wl.tight_ld(layout, n, n), wl.tight_ld(layout, n, N)
    C0 = np.zeros_like(buf(Bl))
    out, _, _ = gpu_gemm("f32", layout, n, N, n, np.float32(1), buf(P), ldp, buf(Bl), ldb, np.float32(0), C0, ldb)
    assert np.array_equal(wl.logical(layout, out, n, N), Bl[perm])
    Bh = Bl.astype(np.float16)
    out, _, _ = gpu_gemm("f16", layout, n, N, n, np.float32(1), buf(P, np.float16).view(np.uint16), ldp,
                         buf(Bh, np.float16).view(np.uint16), ldb, np.float32(0), C0, ldb)
    assert np.array_equal(wl.logical(layout, out, n, N), Bh[perm].astype(np.float32))
    Bi = rng.integers(-128, 128, size=(n, N)).astype(np.int8)
    out, _, _ = gpu_gemm("i8", layout, n, N, n, 1, buf(P, np.int8), ldp, buf(Bi, np.int8), ldb, 0,
                         C0.astype(np.int32), ldb)
    assert np.array_equal(wl.logical(layout, out, n, N), Bi[perm].astype(np.int32))


@pytest.mark.parametrize("layout", LAYOUTS)
def test_i8_extremes(layout):
    M, N, K = 70, 40, 1000
    for va, vb, want in ((-128, -128, 16384), (-128, 127, -16256), (127, -128, -16256)):
        A = np.full(wl._shape(layout, M, K, wl.tight_ld(layout, M, K)), va, dtype=np.int8)
        B = np.full(wl._shape(layout, K, N, wl.tight_ld(layout, K, N)), vb, dtype=np.int8)
        C = np.zeros(wl._shape(layout, M, N, wl.tight_ld(layout, M, N)), dtype=np.int32)
        out, _, _ = gpu_gemm("i8", layout, M, N, K, 1, A, wl.tight_ld(layout, M, K), B, wl.tight_ld(layout, K, N), 0,
                             C, wl.tight_ld(layout, M, N))
        assert np.all(out == want * K)


# ------------------------------------------------------------ quick returns and special scalars
@pytest.mark.parametrize("dtype", DTYPES)
def test_beta_zero_does_not_read_c(dtype):
    M, N, K = 100, 90, 600
    A, lda, B, ldb, C, ldc = make_inputs(dtype, "col", M, N, K, 5000)
    if dtype == "i8":
        poisoned = np.full_like(C, 2 ** 31 - 1)
        one, zero = 1, 0
    else:
        poisoned = np.full_like(C, np.nan)
        one, zero = np.float32(1), np.float32(0)
    out, _, _ = gpu_gemm(dtype, "col", M, N, K, one, A, lda, B, ldb, zero, poisoned, ldc)
    ref = oracle_gemm(dtype, "col", M, N, K, one, A, lda, B, ldb, zero, None, ldc)
    got = wl.logical("col", out, M, N)
    if dtype == "i8":
        assert np.array_equal(got, oracle.wrap_int32(ref))
    else:
        assert np.all(np.isfinite(got))
        assert oracle.normalised_error(got, ref, K, 4.0, 4.0) < 1e-3
    # the split-K path and the K == 0 / alpha == 0 paths must not read it either
    out, _, s = gpu_gemm(dtype, "col", M, N, K, one, A, lda, B, ldb, zero, poisoned, ldc, split=2)
    assert s == 2
    got = wl.logical("col", out, M, N)
    assert np.all(np.isfinite(got.astype(np.float64)))
    out, _, _ = gpu_gemm(dtype, "col", M, N, 0, one, A, lda, B, max(ldb, 1), zero, poisoned, ldc)
    assert np.all(wl.logical("col", out, M, N) == 0)
    out, _, _ = gpu_gemm(dtype, "col", M, N, K, zero, A, lda, B, ldb, zero, poisoned, ldc)
    assert np.all(wl.logical("col", out, M, N) == 0)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("layout", LAYOUTS)
def test_quick_returns(dtype, layout):
    M, N, K = 37, 41, 29
    A, lda, B, ldb, C, ldc = make_inputs(dtype, layout, M, N, K, 5100, pad=(0, 0, 2))
    two = 2 if dtype == "i8" else np.float32(2)
    one = 1 if dtype == "i8" else np.float32(1)
    zero = 0 if dtype == "i8" else np.float32(0)
    # alpha == 0: C <- beta*C
    out, _, _ = gpu_gemm(dtype, layout, M, N, K, zero, A, lda, B, ldb, two, C, ldc)
    assert np.array_equal(wl.logical(layout, out, M, N), 2 * wl.logical(layout, C, M, N))
    mask = np.ones(out.shape, dtype=bool)
    wl.logical(layout, mask, M, N)[...] = False
    assert np.array_equal(out[mask], C[mask])
    # K == 0 likewise; alpha == 0 and beta == 1 leaves C alone; M == 0 or N == 0 touches nothing
    out, _, _ = gpu_gemm(dtype, layout, M, N, 0, one, A, max(lda, 1), B, max(ldb, 1), two, C, ldc)
    assert np.array_equal(wl.logical(layout, out, M, N), 2 * wl.logical(layout, C, M, N))
    out, _, _ = gpu_gemm(dtype, layout, M, N, K, zero, A, lda, B, ldb, one, C, ldc)
    assert np.array_equal(out, C)
    out, _, _ = gpu_gemm(dtype, layout, 0, N, K, one, A, lda, B, ldb, zero, C, ldc)
    assert np.array_equal(out, C)
    out, _, _ = gpu_gemm(dtype, layout, M, 0, K, one, A, lda, B, ldb, zero, C, ldc)
    assert np.array_equal(out, C)


def test_row_major_equals_swapped_col_major_bitwise():
    M, N, K = 190, 210, 333
    A, lda, B, ldb, C, ldc = make_inputs("f32", "row", M, N, K, 5200)
    a = gpu_gemm("f32", "row", M, N, K, np.float32(1.5), A, lda, B, ldb, np.float32(0.5), C, ldc)[0]
    b = gpu_gemm("f32", "col", N, M, K, np.float32(1.5), B, ldb, A, lda, np.float32(0.5), C, ldc)[0]
    assert np.array_equal(a, b)


def test_error_codes_leave_c_alone():
    M, N, K = 16, 16, 16
    A, lda, B, ldb, C, ldc = make_inputs("f32", "col", M, N, K, 5300)
    _, dA = to_device(A)
    _, dB = to_device(B)
    _, dC = to_device(C)
    for args, want in (((7, M, N, K, 1.0, dA, lda, dB, ldb, 0.0, dC, ldc), -1),
                       ((0, -1, N, K, 1.0, dA, lda, dB, ldb, 0.0, dC, ldc), -2),
                       ((0, M, N, K, 1.0, dA, M - 1, dB, ldb, 0.0, dC, ldc), -7),
                       ((0, M, N, K, 1.0, dA, lda, dB, K - 1, 0.0, dC, ldc), -9),
                       ((0, M, N, K, 1.0, dA, lda, dB, ldb, 0.0, dC, M - 1), -12),
                       ((0, M, N, K, 1.0, None, lda, dB, ldb, 0.0, dC, ldc), -6),
                       ((0, M, N, K, 1.0, dA, lda, dB, ldb, 0.0, None, ldc), -11)):
        assert mg.gemm_f32(*args, check=False) == want
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy().reshape(C.shape), C)


# ------------------------------------------------------------ the paper's shapes
@pytest.mark.parametrize("layout", LAYOUTS)
def test_im2row_headline_shapes_f32(layout):
    for idx, (M, N, K) in enumerate(wl.IM2ROW_HEADLINE):
        check_case("f32", layout, M, N, K, 1.0, 0.0, seed=4000 + idx)


@pytest.mark.parametrize("layout", LAYOUTS)
def test_int8_ragged_shapes(layout):
    for idx, (M, N, K) in enumerate(wl.INT8_SHAPES[1:]):
        check_case("i8", layout, M, N, K, 1, 0, seed=5000 + idx)
    check_case("i8", layout, 1000, 999, 1001, 2, -1, seed=5010)


@pytest.mark.parametrize("layout", LAYOUTS)
def test_every_im2row_table_shape_f32(layout):
    """All 20 ResNet50 v1.5 and 9 VGG16 GEMMs of the paper's two tables, automatic selection."""
    for idx, (M, N, K) in enumerate(wl.RESNET50_IM2ROW + wl.VGG16_IM2ROW):
        check_case("f32", layout, M, N, K, 1.0, 0.0, seed=4200 + idx)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_resnet50_table_shapes_in_16_and_8_bit(dtype):
    """The 20 ResNet50 v1.5 GEMMs in the other data types, automatic selection (register-direct and
    direct-to-LDS kernels of those types), alternating layouts."""
    for idx, (M, N, K) in enumerate(wl.RESNET50_IM2ROW):
        check_case(dtype, LAYOUTS[idx % 2], M, N, K, 1, 0, seed=4300 + idx)


@pytest.mark.parametrize("dtype", DTYPES)
def test_random_shapes_automatic_selection(dtype):
    """Seeded random small problems with padded leading dimensions and operands off 16-byte alignment:
    whatever the selector picks must agree with the oracle."""
    rng = np.random.default_rng(4400)
    for idx in range(24):
        M, N = int(rng.integers(1, 400)), int(rng.integers(1, 400))
        K = int(rng.integers(1, 700)) if idx % 3 else int(rng.integers(700, 5000))
        pad = tuple(int(x) for x in rng.integers(0, 5, 3))
        offsets = tuple(int(x) for x in rng.integers(0, 4, 3)) if idx % 2 else (0, 0, 0)
        a, b = ((1, 0), (2, -1), (1, 1))[idx % 3]
        check_case(dtype, LAYOUTS[idx % 2], M, N, K, a, b, seed=4400 + idx, pad=pad, offsets=offsets)


def test_other_table_shapes_f32():
    """A few of the remaining rows of the two im2row tables (tiny K, skinny M, wide N)."""
    for idx, (M, N, K) in enumerate([wl.VGG16_IM2ROW[0], wl.RESNET50_IM2ROW[1], wl.RESNET50_IM2ROW[12],
                                     wl.RESNET50_IM2ROW[17]]):
        check_case("f32", "col", M, N, K, 1.0, 0.0, seed=4100 + idx)


# ------------------------------------------------------------ solo mode
@pytest.mark.parametrize("dtype", DTYPES)
def test_solo_mode_runs_every_kernel(dtype):
    """The micro-kernel benchmark launches and completes for every tile configuration."""
    for kid in _kernels(dtype):
        bm, bn, bk, wpc = mg.gemm_kernel_tile(DT[dtype], kid)
        assert bm % 16 == 0 and bn % 16 == 0 and bk > 0 and wpc >= 1
        for fill in (0, 1):
            assert mg.gemm_solo(DT[dtype], kid, 64, 50, fill) == 0
    torch.cuda.synchronize()
    assert mg.gemm_solo(DT[dtype], 0, 0, 10, 1, check=False) == -3
    assert mg.gemm_solo(DT[dtype], 99, 8, 10, 1, check=False) == -2
    assert mg.gemm_solo(DT[dtype], 0, 8, 10, 2, check=False) == -5


# ------------------------------------------------------------ leading dimensions beyond 32-bit byte offsets
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_huge_leading_dimension(dtype):
    """lda of 2^26 + 8 elements: a k-row of A starts more than 2^28 bytes after the previous one, so the
    kernels that address a tile with 32-bit lane offsets must step aside (selection) or take their
    guarded path (when forced), and the result must still be right."""
    M, N, K = 300, 40, 24
    lda, ldb, ldc = (1 << 26) + 8, K, M
    rng = np.random.default_rng(77)
    if dtype == "f32":
        A = np.zeros(K * lda, dtype=np.float32)
        B = (rng.random(N * ldb, dtype=np.float32) * 2 - 1).astype(np.float32)
        for k in range(K):
            A[k * lda:k * lda + M] = rng.random(M, dtype=np.float32) * 2 - 1
        ref_fn, amax = oracle.gemm_f32, 1.0
    else:
        A = np.zeros(K * lda, dtype=np.uint16)
        B = wl.normal_f16_bits(78, "col", K, N).reshape(-1)
        for k in range(K):
            A[k * lda:k * lda + M] = wl.normal_f16_bits(79 + k, "col", M, 1).reshape(-1)
        ref_fn, amax = oracle.gemm_f16, 6.0
    C = np.zeros(N * ldc, dtype=np.float32)
    ref = ref_fn("col", M, N, K, np.float32(1), A.reshape(K, lda), lda, B.reshape(N, ldb), ldb, np.float32(0), None, ldc)
    kernels = [-1] + _kernels(dtype)
    dA = torch.from_numpy(A.view(np.int16) if dtype == "f16" else A).cuda()
    dB = torch.from_numpy(B.view(np.int16) if dtype == "f16" else B).cuda()
    for kid in kernels:
        dC = torch.from_numpy(C).cuda()
        mg.gemm_force_kernel(DT[dtype], kid, 0)
        try:
            {"f32": mg.gemm_f32, "f16": mg.gemm_f16}[dtype](mg.COL_MAJOR, M, N, K, 1.0, dA, lda, dB, ldb, 0.0, dC, ldc)
        finally:
            mg.gemm_force_kernel(DT[dtype], -1, 0)
        torch.cuda.synchronize()
        got = dC.cpu().numpy().reshape(N, ldc)[:, :M].T
        err = oracle.normalised_error(got, ref, K, amax, amax)
        assert err <= (1e-6 if dtype == "f32" else 2e-3), (kid, err)
