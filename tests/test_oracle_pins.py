"""Pins for the CPU oracle: each test fixes it to something other than itself.

The product has a closed definition (paper Sec. II-A, and the alpha/beta form
of its reference micro-kernel), so the pins are: exact rational brute force on
a tiny case, identity / permutation operands, closed forms (all-ones, rank-1),
exact small-integer arithmetic in Python ints, int8 extremes, numpy's float16
for every binary16 pattern, torch.matmul in float64 / int64, and algebraic
invariants (K-split, zero padding, linearity in alpha, layout transposition).
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
import workloads as wl

LAYOUTS = ["col", "row"]


def _get(layout, buf, i, j, ld):
    flat = buf.reshape(-1)
    return flat[i + j * ld] if layout == "col" else flat[i * ld + j]


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("layout", LAYOUTS)
def test_f32_7x5x3_exact_rational(layout):
    """7x5x3 with padded leading dimensions against a sum written out in exact rationals."""
    M, N, K = 7, 5, 3
    pad = 2
    lda = wl.tight_ld(layout, M, K) + pad
    ldb = wl.tight_ld(layout, K, N) + pad + 1
    ldc = wl.tight_ld(layout, M, N) + pad + 2
    A = wl.uniform_f32(11, layout, M, K, lda)
    B = wl.uniform_f32(12, layout, K, N, ldb)
    C = wl.uniform_f32(13, layout, M, N, ldc)
    alpha, beta = np.float32(1.5), np.float32(-0.75)
    D = oracle.gemm_f32(layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc)
    assert D.shape == (M, N)
    for i in range(M):
        for j in range(N):
            s = Fraction(0)
            for p in range(K):
                s += Fraction(float(_get(layout, A, i, p, lda))) * Fraction(float(_get(layout, B, p, j, ldb)))
            want = Fraction(float(alpha)) * s + Fraction(float(beta)) * Fraction(float(_get(layout, C, i, j, ldc)))
            # fp64 evaluation of a 3-term sum of exact products: a few ulps of the magnitude
            assert abs(Fraction(float(D[i, j])) - want) <= Fraction(1, 2 ** 48)


@pytest.mark.parametrize("layout", LAYOUTS)
def test_i8_small_exact_python_ints(layout):
    M, N, K = 6, 4, 9
    lda = wl.tight_ld(layout, M, K) + 3
    ldb = wl.tight_ld(layout, K, N) + 1
    ldc = wl.tight_ld(layout, M, N) + 2
    A = wl.uniform_i8(21, layout, M, K, lda)
    B = wl.uniform_i8(22, layout, K, N, ldb)
    C = wl.uniform_i32(23, layout, M, N, ldc)
    alpha, beta = 3, -2
    D = oracle.gemm_i8(layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc)
    for i in range(M):
        for j in range(N):
            s = sum(int(_get(layout, A, i, p, lda)) * int(_get(layout, B, p, j, ldb)) for p in range(K))
            assert int(D[i, j]) == alpha * s + beta * int(_get(layout, C, i, j, ldc))


@pytest.mark.parametrize("layout", LAYOUTS)
def test_f16_small_exact_rational(layout):
    M, N, K = 5, 6, 4
    lda = wl.tight_ld(layout, M, K) + 1
    ldb = wl.tight_ld(layout, K, N) + 2
    A = wl.normal_f16_bits(31, layout, M, K, lda)
    B = wl.normal_f16_bits(32, layout, K, N, ldb)
    D = oracle.gemm_f16(layout, M, N, K, 1.0, A, lda, B, ldb, 0.0, None, 0)
    Af, Bf = A.view(np.float16), B.view(np.float16)
    for i in range(M):
        for j in range(N):
            s = Fraction(0)
            for p in range(K):
                s += Fraction(float(_get(layout, Af, i, p, lda))) * Fraction(float(_get(layout, Bf, p, j, ldb)))
            # binary16 products have 22-bit significands; a 4-term sum of them is exact in fp64
            assert Fraction(float(D[i, j])) == s


# ---------------------------------------------------------------- binary16 decode
def test_half_decode_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(b) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


# ---------------------------------------------------------------- identity / permutation
@pytest.mark.parametrize("layout", LAYOUTS)
def test_identity_and_permutation_f32(layout):
    n, N = 13, 9
    rng = np.random.default_rng(5)
    perm = rng.permutation(n)
    P = np.zeros((n, n), dtype=np.float32)
    P[np.arange(n), perm] = 1.0                      # (P @ B)[i] = B[perm[i]]
    Bl = rng.standard_normal((n, N)).astype(np.float32)
    Cl = rng.standard_normal((n, N)).astype(np.float32)

    def buf(x):
        return np.ascontiguousarray(x.T if layout == "col" else x)

    lda, ldb, ldc = wl.tight_ld(layout, n, n), wl.tight_ld(layout, n, N), wl.tight_ld(layout, n, N)
    eye = np.eye(n, dtype=np.float32)
    D = oracle.gemm_f32(layout, n, N, n, 2.0, buf(eye), lda, buf(Bl), ldb, 0.5, buf(Cl), ldc)
    assert np.array_equal(D, 2.0 * Bl.astype(np.float64) + 0.5 * Cl.astype(np.float64))
    D = oracle.gemm_f32(layout, n, N, n, 1.0, buf(P), lda, buf(Bl), ldb, 0.0, None, 0)
    assert np.array_equal(D, Bl[perm].astype(np.float64))
    # identity on the right: C = A * I
    Al = rng.standard_normal((N, n)).astype(np.float32)
    D = oracle.gemm_f32(layout, N, n, n, 1.0, buf(Al), wl.tight_ld(layout, N, n), buf(eye), lda, 0.0, None, 0)
    assert np.array_equal(D, Al.astype(np.float64))
    # a column permutation from the right: (A @ P)[:, perm[i]] = A[:, i]
    D = oracle.gemm_f32(layout, N, n, n, 1.0, buf(Al), wl.tight_ld(layout, N, n), buf(P), lda, 0.0, None, 0)
    want = np.zeros((N, n))
    want[:, perm] = Al
    assert np.array_equal(D, want)


@pytest.mark.parametrize("layout", LAYOUTS)
def test_permutation_i8_and_f16(layout):
    n, N = 11, 7
    rng = np.random.default_rng(6)
    perm = rng.permutation(n)
    P = np.zeros((n, n))
    P[np.arange(n), perm] = 1

    def buf(x, dt):
        return np.ascontiguousarray((x.T if layout == "col" else x).astype(dt))

    Bl = rng.integers(-128, 128, size=(n, N))
    D = oracle.gemm_i8(layout, n, N, n, 1, buf(P, np.int8), wl.tight_ld(layout, n, n), buf(Bl, np.int8),
                       wl.tight_ld(layout, n, N), 0, None, 0)
    assert np.array_equal(D, Bl[perm])
    Bh = rng.standard_normal((n, N)).astype(np.float16)
    D = oracle.gemm_f16(layout, n, N, n, 1.0, buf(P, np.float16).view(np.uint16), wl.tight_ld(layout, n, n),
                        buf(Bh, np.float16).view(np.uint16), wl.tight_ld(layout, n, N), 0.0, None, 0)
    assert np.array_equal(D, Bh[perm].astype(np.float64))


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("K", [1, 2, 63, 1000])
def test_all_ones_and_rank1(layout, K):
    M, N = 10, 12
    ones_a = np.ones(wl._shape(layout, M, K, wl.tight_ld(layout, M, K)), dtype=np.float32)
    ones_b = np.ones(wl._shape(layout, K, N, wl.tight_ld(layout, K, N)), dtype=np.float32)
    D = oracle.gemm_f32(layout, M, N, K, 1.0, ones_a, wl.tight_ld(layout, M, K), ones_b,
                        wl.tight_ld(layout, K, N), 0.0, None, 0)
    assert np.all(D == K)
    D = oracle.gemm_i8(layout, M, N, K, 1, ones_a.astype(np.int8), wl.tight_ld(layout, M, K),
                       ones_b.astype(np.int8), wl.tight_ld(layout, K, N), 0, None, 0)
    assert np.all(D == K)
    D = oracle.gemm_f16(layout, M, N, K, 1.0, ones_a.astype(np.float16).view(np.uint16),
                        wl.tight_ld(layout, M, K), ones_b.astype(np.float16).view(np.uint16),
                        wl.tight_ld(layout, K, N), 0.0, None, 0)
    assert np.all(D == K)
    # rank-1: A(i,p) = i%7-3, B(p,j) = j%5-2  =>  C(i,j) = K * a_i * b_j
    a = (np.arange(M) % 7 - 3).astype(np.float32)
    b = (np.arange(N) % 5 - 2).astype(np.float32)
    Al = np.repeat(a[:, None], K, axis=1)
    Bl = np.repeat(b[None, :], K, axis=0)

    def buf(x):
        return np.ascontiguousarray(x.T if layout == "col" else x)

    D = oracle.gemm_f32(layout, M, N, K, 1.0, buf(Al), wl.tight_ld(layout, M, K), buf(Bl),
                        wl.tight_ld(layout, K, N), 0.0, None, 0)
    assert np.array_equal(D, K * np.outer(a, b).astype(np.float64))


@pytest.mark.parametrize("layout", LAYOUTS)
def test_i8_extremes(layout):
    M, N, K = 5, 4, 300

    def full(rows, cols, v):
        return np.full(wl._shape(layout, rows, cols, wl.tight_ld(layout, rows, cols)), v, dtype=np.int8)

    lda, ldb = wl.tight_ld(layout, M, K), wl.tight_ld(layout, K, N)
    D = oracle.gemm_i8(layout, M, N, K, 1, full(M, K, -128), lda, full(K, N, -128), ldb, 0, None, 0)
    assert np.all(D == 16384 * K)
    D = oracle.gemm_i8(layout, M, N, K, 1, full(M, K, -128), lda, full(K, N, 127), ldb, 0, None, 0)
    assert np.all(D == -16256 * K)
    D = oracle.gemm_i8(layout, M, N, K, 1, full(M, K, 127), lda, full(K, N, -128), ldb, 0, None, 0)
    assert np.all(D == -16256 * K)


def test_wrap_int32():
    v = np.array([0, 1, -1, 2 ** 31 - 1, 2 ** 31, -2 ** 31, -2 ** 31 - 1, 2 ** 32 + 5, -2 ** 32 - 7], dtype=np.int64)
    want = [((int(x) + 2 ** 31) % 2 ** 32) - 2 ** 31 for x in v]
    assert oracle.wrap_int32(v).tolist() == want


# ---------------------------------------------------------------- small integers: exact in any order
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("alpha,beta", [(1.0, 0.0), (2.0, -1.0), (0.5, 1.0), (-1.0, 2.0)])
def test_small_integer_inputs_exact(layout, alpha, beta):
    M, N, K = 17, 9, 130
    lda, ldb, ldc = wl.tight_ld(layout, M, K), wl.tight_ld(layout, K, N), wl.tight_ld(layout, M, N)
    A = wl.small_int_f32(41, layout, M, K)
    B = wl.small_int_f32(42, layout, K, N)
    C = wl.small_int_f32(43, layout, M, N)
    D = oracle.gemm_f32(layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc)
    Ai = wl.logical(layout, A, M, K).astype(np.int64)
    Bi = wl.logical(layout, B, K, N).astype(np.int64)
    Ci = wl.logical(layout, C, M, N).astype(np.int64)
    want2 = int(2 * alpha) * (Ai @ Bi) + int(2 * beta) * Ci       # doubled, to keep 0.5 integral
    assert np.array_equal(2 * D, want2.astype(np.float64))
    Dh = oracle.gemm_f16(layout, M, N, K, alpha, A.astype(np.float16).view(np.uint16), lda,
                         B.astype(np.float16).view(np.uint16), ldb, beta, C, ldc)
    assert np.array_equal(Dh, D)


# ---------------------------------------------------------------- library second opinion
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("shape", [(64, 48, 200), (1, 1, 1), (33, 17, 129), (128, 3, 7)])
def test_against_torch_matmul(layout, shape):
    M, N, K = shape
    lda = wl.tight_ld(layout, M, K) + 3
    ldb = wl.tight_ld(layout, K, N) + 5
    ldc = wl.tight_ld(layout, M, N) + 1
    A = wl.uniform_f32(51, layout, M, K, lda)
    B = wl.uniform_f32(52, layout, K, N, ldb)
    C = wl.uniform_f32(53, layout, M, N, ldc)
    alpha, beta = np.float32(1.5), np.float32(0.5)
    D = oracle.gemm_f32(layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc)
    tA = torch.from_numpy(wl.logical(layout, A, M, K).astype(np.float64))
    tB = torch.from_numpy(wl.logical(layout, B, K, N).astype(np.float64))
    tC = torch.from_numpy(wl.logical(layout, C, M, N).astype(np.float64))
    want = (float(alpha) * (tA @ tB) + float(beta) * tC).numpy()
    assert np.max(np.abs(D - want)) <= (K + 2) * 2.0 ** -52 * K      # |terms| <= 1
    # binary16
    Ah = wl.normal_f16_bits(54, layout, M, K, lda)
    Bh = wl.normal_f16_bits(55, layout, K, N, ldb)
    D = oracle.gemm_f16(layout, M, N, K, alpha, Ah, lda, Bh, ldb, beta, C, ldc)
    tA = torch.from_numpy(wl.logical(layout, Ah.view(np.float16), M, K).astype(np.float64))
    tB = torch.from_numpy(wl.logical(layout, Bh.view(np.float16), K, N).astype(np.float64))
    want = (float(alpha) * (tA @ tB) + float(beta) * tC).numpy()
    scale = float(tA.abs().max() * tB.abs().max()) if K else 0.0
    assert np.max(np.abs(D - want)) <= (K + 2) * 2.0 ** -52 * K * max(scale, 1.0) * 2
    # int8
    Ai = wl.uniform_i8(56, layout, M, K, lda)
    Bi = wl.uniform_i8(57, layout, K, N, ldb)
    Ci = wl.uniform_i32(58, layout, M, N, ldc)
    D = oracle.gemm_i8(layout, M, N, K, 2, Ai, lda, Bi, ldb, -1, Ci, ldc)
    tA = torch.from_numpy(wl.logical(layout, Ai, M, K).astype(np.int64))
    tB = torch.from_numpy(wl.logical(layout, Bi, K, N).astype(np.int64))
    tC = torch.from_numpy(wl.logical(layout, Ci, M, N).astype(np.int64))
    assert np.array_equal(D, (2 * (tA @ tB) - tC).numpy())


# ---------------------------------------------------------------- invariants
@pytest.mark.parametrize("layout", LAYOUTS)
def test_layout_transposition_identity(layout):
    """A row-major call equals the column-major call on the same buffers with operands swapped."""
    M, N, K = 9, 14, 21
    other = "row" if layout == "col" else "col"
    A = wl.uniform_f32(61, layout, M, K)
    B = wl.uniform_f32(62, layout, K, N)
    C = wl.uniform_f32(63, layout, M, N)
    D = oracle.gemm_f32(layout, M, N, K, 1.25, A, wl.tight_ld(layout, M, K), B, wl.tight_ld(layout, K, N),
                        -0.5, C, wl.tight_ld(layout, M, N))
    # the same bytes read in the other layout hold A^T (K x M), B^T (N x K), C^T (N x M)
    Dt = oracle.gemm_f32(other, N, M, K, 1.25, B, wl.tight_ld(other, N, K), A, wl.tight_ld(other, K, M),
                         -0.5, C, wl.tight_ld(other, N, M))
    assert np.array_equal(D, Dt.T)


def test_k_split_zero_padding_and_linearity():
    layout = "col"
    M, N, K = 12, 10, 40
    A = wl.small_int_f32(71, layout, M, K)
    B = wl.small_int_f32(72, layout, K, N)
    full = oracle.gemm_f32(layout, M, N, K, 1.0, A, M, B, K, 0.0, None, 0)
    # K split: first 25 columns of A with first 25 rows of B, then the rest accumulated with beta = 1
    K1 = 25
    part = oracle.gemm_f32(layout, M, N, K1, 1.0, A, M, B, K, 0.0, None, 0)
    part32 = np.ascontiguousarray(part.T.astype(np.float32))
    rest = oracle.gemm_f32(layout, M, N, K - K1, 1.0, A.reshape(-1)[K1 * M:], M, B.reshape(-1)[K1:], K,
                           1.0, part32, M)
    assert np.array_equal(rest, full)
    # zero padding of K changes nothing
    Ap = np.zeros((K + 5, M), dtype=np.float32)
    Ap[:K] = A
    Bp = np.zeros((N, K + 5), dtype=np.float32)
    Bp[:, :K] = B
    padded = oracle.gemm_f32(layout, M, N, K + 5, 1.0, Ap, M, Bp, K + 5, 0.0, None, 0)
    assert np.array_equal(padded, full)
    # linearity in alpha (exact for powers of two)
    assert np.array_equal(oracle.gemm_f32(layout, M, N, K, 4.0, A, M, B, K, 0.0, None, 0), 4.0 * full)


def test_beta_zero_ignores_old_c_and_k_zero():
    layout = "col"
    M, N, K = 4, 3, 5
    A = wl.uniform_f32(81, layout, M, K)
    B = wl.uniform_f32(82, layout, K, N)
    C = np.full((N, M), np.nan, dtype=np.float32)
    D = oracle.gemm_f32(layout, M, N, K, 1.0, A, M, B, K, 0.0, C, M)
    assert np.all(np.isfinite(D))
    C = wl.uniform_f32(83, layout, M, N)
    D = oracle.gemm_f32(layout, M, N, 0, 1.0, A, M, B, 1, 2.0, C, M)
    assert np.array_equal(D, 2.0 * wl.logical(layout, C, M, N).astype(np.float64))


# ---------------------------------------------------------------- sampled evaluation agrees with the full one
@pytest.mark.parametrize("layout", LAYOUTS)
def test_sampled_oracle_matches_full(layout):
    M, N, K = 40, 30, 77
    lda, ldb, ldc = wl.tight_ld(layout, M, K) + 1, wl.tight_ld(layout, K, N) + 2, wl.tight_ld(layout, M, N) + 3
    rng = np.random.default_rng(9)
    rows, cols = rng.integers(0, M, 50), rng.integers(0, N, 50)
    A, B, C = wl.uniform_f32(91, layout, M, K, lda), wl.uniform_f32(92, layout, K, N, ldb), wl.uniform_f32(93, layout, M, N, ldc)
    D = oracle.gemm_f32(layout, M, N, K, 1.5, A, lda, B, ldb, 0.5, C, ldc)
    s = oracle.gemm_sample("f32", layout, K, 1.5, A, lda, B, ldb, 0.5, C, ldc, rows, cols)
    assert np.array_equal(s, D[rows, cols])
    Ah, Bh = wl.normal_f16_bits(94, layout, M, K, lda), wl.normal_f16_bits(95, layout, K, N, ldb)
    D = oracle.gemm_f16(layout, M, N, K, 1.0, Ah, lda, Bh, ldb, 0.0, None, 0)
    s = oracle.gemm_sample("f16", layout, K, 1.0, Ah, lda, Bh, ldb, 0.0, None, 0, rows, cols)
    assert np.array_equal(s, D[rows, cols])
    Ai, Bi, Ci = wl.uniform_i8(96, layout, M, K, lda), wl.uniform_i8(97, layout, K, N, ldb), wl.uniform_i32(98, layout, M, N, ldc)
    D = oracle.gemm_i8(layout, M, N, K, 2, Ai, lda, Bi, ldb, -1, Ci, ldc)
    s = oracle.gemm_sample("i8", layout, K, 2, Ai, lda, Bi, ldb, -1, Ci, ldc, rows, cols)
    assert np.array_equal(s, D[rows, cols].astype(np.float64))


# ---------------------------------------------------------------- the metric tells fp16 accumulation apart
def test_metric_distinguishes_fp16_accumulation():
    """A result accumulated in binary16 must fail a bound that fp32 accumulation passes easily."""
    layout = "row"
    M, N, K = 16, 16, 8192
    A = wl.normal_f16_bits(101, layout, M, K)
    B = wl.normal_f16_bits(102, layout, K, N)
    D = oracle.gemm_f16(layout, M, N, K, 1.0, A, K, B, N, 0.0, None, 0)
    Af, Bf = A.view(np.float16), B.view(np.float16)
    max_a, max_b = float(np.abs(Af.astype(np.float64)).max()), float(np.abs(Bf.astype(np.float64)).max())
    acc16 = np.zeros((M, N), dtype=np.float16)
    acc32 = np.zeros((M, N), dtype=np.float32)
    for p in range(K):
        prod = np.outer(Af[:, p].astype(np.float32), Bf[p, :].astype(np.float32))     # exact in fp32
        acc16 = (acc16.astype(np.float32) + prod).astype(np.float16)
        acc32 = acc32 + prod
    assert oracle.normalised_error(acc32, D, K, max_a, max_b) < 1e-7
    assert oracle.normalised_error(acc16, D, K, max_a, max_b) > 1e-5


# ---------------------------------------------------------------- bfloat16
def test_bfloat16_decode_all_patterns():
    """A bfloat16 is the upper half of an IEEE binary32: every pattern against numpy's float32."""
    bits = np.arange(65536, dtype=np.uint16)
    with np.errstate(invalid="ignore"):      # signalling NaN patterns are among the 65536
        want = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    got = np.array([oracle.bfloat16_to_double(b) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_bfloat16_generator_rounds_to_nearest_even():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -7, -2.5, 3.0e38, 1.0 + 2.0 ** -8 + 2.0 ** -20],
                 dtype=np.float32)
    got = wl.bf16_bits_to_f32(wl._to_bf16_bits(x))
    # ties go to the even significand: 1 + 2^-8 -> 1, 1 + 3*2^-8 -> 1 + 2^-6; above a tie rounds up
    assert got.tolist() == [1.0, 1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -2.5, 226 * 2.0 ** 120,
                            1.0 + 2.0 ** -7]


@pytest.mark.parametrize("layout", LAYOUTS)
def test_bf16_small_exact_rational_and_library(layout):
    M, N, K = 5, 6, 4
    lda = wl.tight_ld(layout, M, K) + 1
    ldb = wl.tight_ld(layout, K, N) + 2
    ldc = wl.tight_ld(layout, M, N) + 3
    A = wl.normal_bf16_bits(61, layout, M, K, lda)
    B = wl.normal_bf16_bits(62, layout, K, N, ldb)
    C = wl.uniform_f32(63, layout, M, N, ldc)
    D = oracle.gemm_bf16(layout, M, N, K, 1.0, A, lda, B, ldb, 0.0, None, 0)
    Af, Bf = wl.bf16_bits_to_f32(A), wl.bf16_bits_to_f32(B)
    for i in range(M):
        for j in range(N):
            s = Fraction(0)
            for p in range(K):
                s += Fraction(float(_get(layout, Af, i, p, lda))) * Fraction(float(_get(layout, Bf, p, j, ldb)))
            # bfloat16 products have 16-bit significands; a 4-term sum of N(0,1)-sized ones is exact in fp64
            assert Fraction(float(D[i, j])) == s
    # alpha, beta and a library second opinion in float64
    M, N, K = 33, 17, 129
    lda, ldb, ldc = wl.tight_ld(layout, M, K) + 3, wl.tight_ld(layout, K, N) + 5, wl.tight_ld(layout, M, N) + 1
    A, B = wl.normal_bf16_bits(64, layout, M, K, lda), wl.normal_bf16_bits(65, layout, K, N, ldb)
    C = wl.uniform_f32(66, layout, M, N, ldc)
    D = oracle.gemm_bf16(layout, M, N, K, np.float32(1.5), A, lda, B, ldb, np.float32(0.5), C, ldc)
    tA = torch.from_numpy(wl.logical(layout, wl.bf16_bits_to_f32(A), M, K).astype(np.float64))
    tB = torch.from_numpy(wl.logical(layout, wl.bf16_bits_to_f32(B), K, N).astype(np.float64))
    tC = torch.from_numpy(wl.logical(layout, C, M, N).astype(np.float64))
    want = (1.5 * (tA @ tB) + 0.5 * tC).numpy()
    scale = float(tA.abs().max() * tB.abs().max())
    assert np.max(np.abs(D - want)) <= (K + 2) * 2.0 ** -52 * K * max(scale, 1.0) * 2
    # sampled evaluation agrees with the full one
    rows, cols = np.array([0, 5, 32, 7]), np.array([0, 16, 3, 9])
    samp = oracle.gemm_sample("bf16", layout, K, 1.5, A, lda, B, ldb, 0.5, C, ldc, rows, cols)
    assert np.array_equal(samp, D[rows, cols])


@pytest.mark.parametrize("layout", LAYOUTS)
def test_bf16_small_integers_match_fp32_oracle(layout):
    M, N, K = 17, 9, 130
    lda, ldb, ldc = wl.tight_ld(layout, M, K), wl.tight_ld(layout, K, N), wl.tight_ld(layout, M, N)
    A, B, C = wl.small_int_f32(41, layout, M, K), wl.small_int_f32(42, layout, K, N), wl.small_int_f32(43, layout, M, N)
    D = oracle.gemm_f32(layout, M, N, K, 2.0, A, lda, B, ldb, -1.0, C, ldc)
    Db = oracle.gemm_bf16(layout, M, N, K, 2.0, wl._to_bf16_bits(A), lda, wl._to_bf16_bits(B), ldb, -1.0, C, ldc)
    assert np.array_equal(Db, D)


# ---------------------------------------------------------------- transposed operands
def _stored(layout, logical_matrix, ld_pad):
    """Buffer holding `logical_matrix` (rows x cols) in `layout` with a padded leading dimension."""
    rows, cols = logical_matrix.shape
    ld = wl.tight_ld(layout, rows, cols) + ld_pad
    buf = np.zeros(wl._shape(layout, rows, cols, ld), dtype=logical_matrix.dtype)
    wl.logical(layout, buf, rows, cols)[...] = logical_matrix
    return buf, ld


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("ta,tb", [(0, 0), (1, 0), (0, 1), (1, 1)])
def test_transposed_operands_exact_rational_and_against_plain(layout, ta, tb):
    """op(A) = A^T / op(B) = B^T: exact rational brute force on 7x5x3 from the stored matrices, and
    identity with the plain oracle on explicitly transposed copies (every data type)."""
    M, N, K = 7, 5, 3
    rng = np.random.default_rng(900 + 2 * ta + tb)
    opA = (rng.random((M, K), dtype=np.float32) * 2 - 1).astype(np.float32)
    opB = (rng.random((K, N), dtype=np.float32) * 2 - 1).astype(np.float32)
    Cm = (rng.random((M, N), dtype=np.float32) * 2 - 1).astype(np.float32)
    A, lda = _stored(layout, opA.T.copy() if ta else opA, 2)
    B, ldb = _stored(layout, opB.T.copy() if tb else opB, 1)
    C, ldc = _stored(layout, Cm, 3)
    D = oracle.gemm_ex("f32", layout, ta, tb, M, N, K, 1.5, A, lda, B, ldb, 0.5, C, ldc)
    for i in range(M):
        for j in range(N):
            s = sum(Fraction(float(opA[i, p])) * Fraction(float(opB[p, j])) for p in range(K))
            want = Fraction(3, 2) * s + Fraction(1, 2) * Fraction(float(Cm[i, j]))
            assert abs(Fraction(float(D[i, j])) - want) <= Fraction(1, 2 ** 50)
    # the plain oracle on untransposed copies computes the same sums in the same order
    A0, lda0 = _stored(layout, opA, 0)
    B0, ldb0 = _stored(layout, opB, 0)
    assert np.array_equal(D, oracle.gemm_f32(layout, M, N, K, np.float32(1.5), A0, lda0, B0, ldb0, np.float32(0.5), C, ldc))
    # 16-bit and 8-bit inputs
    M, N, K = 33, 17, 40
    for dtype, gen, plain in (("f16", wl.normal_f16_bits, oracle.gemm_f16), ("bf16", wl.normal_bf16_bits, oracle.gemm_bf16),
                              ("i8", wl.uniform_i8, oracle.gemm_i8)):
        opA = wl.logical("row", gen(910, "row", M, K), M, K)
        opB = wl.logical("row", gen(911, "row", K, N), K, N)
        A, lda = _stored(layout, opA.T.copy() if ta else opA.copy(), 1)
        B, ldb = _stored(layout, opB.T.copy() if tb else opB.copy(), 2)
        A0, lda0 = _stored(layout, opA.copy(), 0)
        B0, ldb0 = _stored(layout, opB.copy(), 0)
        one = 1 if dtype == "i8" else np.float32(1)
        zero = 0 if dtype == "i8" else np.float32(0)
        got = oracle.gemm_ex(dtype, layout, ta, tb, M, N, K, 1, A, lda, B, ldb, 0, None, 0)
        assert np.array_equal(got, plain(layout, M, N, K, one, A0, lda0, B0, ldb0, zero, None, 0))


# ------------------------------------------------------------ convolution / im2row (oracle/ref_conv.c)
def test_conv_worked_examples_by_hand():
    """3 x 3 image 0..8, one channel.  2 x 2 filter [[1,2],[3,4]], no flip:
    stride 1, no padding: out[0,0] = 0*1 + 1*2 + 3*3 + 4*4 = 27, out[0,1] = 1+4+12+20 = 37,
    out[1,0] = 3+8+18+28 = 57, out[1,1] = 4+10+21+32 = 67;
    stride 2, padding 1 (taps outside the image are zero): out[0,0] = x[0,0]*4 = 0,
    out[0,1] = x[0,1]*3 + x[0,2]*4 = 11, out[1,0] = x[1,0]*2 + x[2,0]*4 = 30, out[1,1] = 4+10+21+32 = 67."""
    x = np.arange(9, dtype=np.float32).reshape(1, 3, 3, 1)
    w = np.array([[1, 2], [3, 4]], dtype=np.float32).reshape(2, 2, 1, 1)
    assert np.array_equal(oracle.conv2d_nhwc_f32(x, w, (1, 1), (0, 0))[0, :, :, 0], [[27, 37], [57, 67]])
    assert np.array_equal(oracle.conv2d_nhwc_f32(x, w, (2, 2), (1, 1))[0, :, :, 0], [[0, 11], [30, 67]])
    # the im2row matrix of the first case, row (oh, ow), column (r, s)
    assert np.array_equal(oracle.im2row_f32(x, 2, 2, (1, 1), (0, 0)),
                          [[0, 1, 3, 4], [1, 2, 4, 5], [3, 4, 6, 7], [4, 5, 7, 8]])
    # alpha and beta: 2 * conv - 1 * old
    old = np.full((1, 2, 2, 1), 10, dtype=np.float32)
    assert np.array_equal(oracle.conv2d_nhwc_f32(x, w, (1, 1), (0, 0), 2.0, -1.0, old)[0, :, :, 0], [[44, 64], [104, 124]])
    # beta == 0 does not read the old output
    bad = np.full((1, 2, 2, 1), np.nan, dtype=np.float32)
    assert np.array_equal(oracle.conv2d_nhwc_f32(x, w, (1, 1), (0, 0), 1.0, 0.0, bad)[0, :, :, 0], [[27, 37], [57, 67]])


def test_conv_shapes_of_the_papers_table():
    """The layer geometries give the (m, n, k) the paper prints (Table "resnet50")."""
    path = os.path.join(os.path.dirname(__file__), "golden", "resnet50_v1.5_conv_geometry.txt")
    rows = [[int(t) for t in line.split()] for line in open(path) if line.strip() and not line.startswith("#")]
    assert len(rows) == 6
    for H, W, Cin, Cout, kh, kw, stride, pad, m, n, k in rows:
        Hout, Wout = oracle.conv_output_shape(H, W, kh, kw, (stride, stride), (pad, pad))
        assert (Hout * Wout, Cout, kh * kw * Cin) == (m, n, k)
    assert [(r[8], r[9], r[10]) for r in rows] == list(wl.IM2ROW_HEADLINE)
    # and the transform produces a matrix of that shape (a small-channel instance of the first row)
    x = np.zeros((1, 224, 224, 3), dtype=np.float32)
    assert oracle.im2row_f32(x, 7, 7, (2, 2), (3, 3)).shape == (12544, 147)


@pytest.mark.parametrize("stride,pad", [((1, 1), (0, 0)), ((2, 1), (1, 2)), ((3, 2), (2, 0))])
def test_conv_single_one_input_returns_the_filter(stride, pad):
    """An image that is zero except for one element equal to 1 at (i0, j0, c0): the output at (oh, ow, co)
    is filter[i0 - oh*sh + ph][j0 - ow*sw + pw][c0][co] where those indices exist, else 0."""
    H, W, Cin, Cout, kh, kw = 7, 6, 3, 4, 3, 2
    rng = np.random.default_rng(77)
    w = rng.standard_normal((kh, kw, Cin, Cout)).astype(np.float32)
    Hout, Wout = oracle.conv_output_shape(H, W, kh, kw, stride, pad)
    for (i0, j0, c0) in ((0, 0, 0), (3, 2, 1), (6, 5, 2)):
        x = np.zeros((1, H, W, Cin), dtype=np.float32)
        x[0, i0, j0, c0] = 1
        got = oracle.conv2d_nhwc_f32(x, w, stride, pad)
        want = np.zeros((1, Hout, Wout, Cout))
        for oh in range(Hout):
            for ow in range(Wout):
                r, s = i0 - oh * stride[0] + pad[0], j0 - ow * stride[1] + pad[1]
                if 0 <= r < kh and 0 <= s < kw:
                    want[0, oh, ow] = w[r, s, c0]
        assert np.array_equal(got, want)


def test_conv_all_ones_counts_the_taps_inside_the_image():
    H, W, Cin, Cout, kh, kw, stride, pad = 6, 5, 4, 2, 3, 3, (1, 2), (1, 1)
    x = np.ones((2, H, W, Cin), dtype=np.float32)
    w = np.ones((kh, kw, Cin, Cout), dtype=np.float32)
    got = oracle.conv2d_nhwc_f32(x, w, stride, pad)
    Hout, Wout = oracle.conv_output_shape(H, W, kh, kw, stride, pad)
    for oh in range(Hout):
        for ow in range(Wout):
            rows = sum(1 for r in range(kh) if 0 <= oh * stride[0] - pad[0] + r < H)
            cols = sum(1 for s in range(kw) if 0 <= ow * stride[1] - pad[1] + s < W)
            assert np.all(got[:, oh, ow, :] == rows * cols * Cin)


def test_conv_is_the_gemm_of_the_im2row_matrix_and_matches_torch():
    """The paper's premise: the convolution is a GEMM of the im2row matrix with the filter matrix.  Also
    against torch's convolution in float64 (an independent implementation, channels-first)."""
    rng = np.random.default_rng(78)
    for (batch, H, W, Cin, Cout, kh, kw, stride, pad) in ((2, 9, 8, 5, 7, 3, 3, (1, 1), (1, 1)), (1, 11, 13, 16, 6, 5, 2, (2, 3), (2, 1)),
                                                          (3, 6, 6, 8, 8, 1, 1, (1, 1), (0, 0)), (1, 8, 8, 4, 3, 3, 3, (2, 2), (0, 0))):
        x = rng.standard_normal((batch, H, W, Cin)).astype(np.float32)
        w = rng.standard_normal((kh, kw, Cin, Cout)).astype(np.float32)
        old = rng.standard_normal((batch,) + oracle.conv_output_shape(H, W, kh, kw, stride, pad) + (Cout,)).astype(np.float32)
        got = oracle.conv2d_nhwc_f32(x, w, stride, pad, 1.5, 0.5, old)
        A = oracle.im2row_f32(x, kh, kw, stride, pad)
        M, K = A.shape
        via_gemm = oracle.gemm_f32("row", M, Cout, K, np.float32(1.5), A, K, w.reshape(K, Cout), Cout, np.float32(0.5),
                                   old.reshape(M, Cout), Cout)
        assert np.allclose(got.reshape(M, Cout), via_gemm, rtol=0, atol=1e-12)
        t = torch.nn.functional.conv2d(torch.from_numpy(x).double().permute(0, 3, 1, 2),
                                       torch.from_numpy(w).double().permute(3, 2, 0, 1), stride=stride, padding=pad)
        want = 1.5 * t.permute(0, 2, 3, 1).numpy() + 0.5 * old.astype(np.float64)
        assert np.allclose(got, want, rtol=0, atol=1e-12)
        if kh == 1 and kw == 1:
            # a 1 x 1 filter at stride 1 is the plain GEMM of the image with the filter
            assert np.array_equal(A, x.reshape(M, K))


# ------------------------------------------------------------ the same for binary16, bfloat16 and int8 inputs
def _to_type(dtype, x):
    """Small-integer or otherwise exactly representable float values as arrays of the oracle's input type."""
    x = np.asarray(x, dtype=np.float64)
    if dtype == "f32":
        return x.astype(np.float32)
    if dtype == "f16":
        return x.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        return (x.astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)     # exact for these values
    return x.astype(np.int8)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i8"])
def test_typed_conv_worked_examples_by_hand(dtype):
    """The 3 x 3 example worked out in test_conv_worked_examples_by_hand, in every input type (its values
    are small integers, which all of them hold exactly)."""
    x = _to_type(dtype, np.arange(9).reshape(1, 3, 3, 1))
    w = _to_type(dtype, np.array([[1, 2], [3, 4]]).reshape(2, 2, 1, 1))
    assert np.array_equal(oracle.conv2d_nhwc(dtype, x, w, (1, 1), (0, 0))[0, :, :, 0], [[27, 37], [57, 67]])
    assert np.array_equal(oracle.conv2d_nhwc(dtype, x, w, (2, 2), (1, 1))[0, :, :, 0], [[0, 11], [30, 67]])
    assert np.array_equal(oracle.im2row(dtype, x, 2, 2, (1, 1), (0, 0)),
                          _to_type(dtype, [[0, 1, 3, 4], [1, 2, 4, 5], [3, 4, 6, 7], [4, 5, 7, 8]]))
    old = np.full((1, 2, 2, 1), 10, dtype=np.int32 if dtype == "i8" else np.float32)
    assert np.array_equal(oracle.conv2d_nhwc(dtype, x, w, (1, 1), (0, 0), 2, -1, old)[0, :, :, 0], [[44, 64], [104, 124]])
    if dtype != "i8":
        bad = np.full((1, 2, 2, 1), np.nan, dtype=np.float32)       # beta == 0 does not read the old output
        assert np.array_equal(oracle.conv2d_nhwc(dtype, x, w, (1, 1), (0, 0), 1, 0, bad)[0, :, :, 0], [[27, 37], [57, 67]])


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
@pytest.mark.parametrize("stride,pad", [((1, 1), (0, 0)), ((2, 1), (1, 2)), ((3, 2), (2, 0))])
def test_typed_conv_single_one_input_returns_the_filter(dtype, stride, pad):
    H, W, Cin, Cout, kh, kw = 7, 6, 3, 4, 3, 2
    rng = np.random.default_rng(79)
    wv = rng.integers(-100, 101, size=(kh, kw, Cin, Cout)).astype(np.float64)      # exact in all three types
    w = _to_type(dtype, wv)
    Hout, Wout = oracle.conv_output_shape(H, W, kh, kw, stride, pad)
    for (i0, j0, c0) in ((0, 0, 0), (3, 2, 1), (6, 5, 2)):
        xv = np.zeros((1, H, W, Cin))
        xv[0, i0, j0, c0] = 1
        got = oracle.conv2d_nhwc(dtype, _to_type(dtype, xv), w, stride, pad)
        want = np.zeros((1, Hout, Wout, Cout))
        for oh in range(Hout):
            for ow in range(Wout):
                r, s = i0 - oh * stride[0] + pad[0], j0 - ow * stride[1] + pad[1]
                if 0 <= r < kh and 0 <= s < kw:
                    want[0, oh, ow] = wv[r, s, c0]
        assert np.array_equal(got, want)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_typed_conv_all_ones_counts_the_taps_inside_the_image(dtype):
    H, W, Cin, Cout, kh, kw, stride, pad = 6, 5, 4, 2, 3, 3, (1, 2), (1, 1)
    got = oracle.conv2d_nhwc(dtype, _to_type(dtype, np.ones((2, H, W, Cin))), _to_type(dtype, np.ones((kh, kw, Cin, Cout))), stride, pad)
    Hout, Wout = oracle.conv_output_shape(H, W, kh, kw, stride, pad)
    for oh in range(Hout):
        for ow in range(Wout):
            rows = sum(1 for r in range(kh) if 0 <= oh * stride[0] - pad[0] + r < H)
            cols = sum(1 for s in range(kw) if 0 <= ow * stride[1] - pad[1] + s < W)
            assert np.all(got[:, oh, ow, :] == rows * cols * Cin)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i8"])
def test_typed_conv_is_the_gemm_of_the_im2row_matrix_and_matches_torch(dtype):
    """conv == the (pinned) GEMM oracle of the same type on the im2row matrix, the typed transform == the fp32
    transform on the decoded values, and torch's convolution in float64 on the decoded values."""
    gen = {"f32": wl.uniform_f32, "f16": wl.normal_f16_bits, "bf16": wl.normal_bf16_bits, "i8": wl.uniform_i8}[dtype]
    gemm = {"f32": oracle.gemm_f32, "f16": oracle.gemm_f16, "bf16": oracle.gemm_bf16, "i8": oracle.gemm_i8}[dtype]
    decode = {"f32": lambda b: b.astype(np.float64), "f16": oracle.half_bits_to_double, "bf16": oracle.bfloat16_bits_to_double,
              "i8": lambda b: b.astype(np.float64)}[dtype]
    rng = np.random.default_rng(80)
    for idx, (batch, H, W, Cin, Cout, kh, kw, stride, pad) in enumerate(((2, 9, 8, 5, 7, 3, 3, (1, 1), (1, 1)), (1, 11, 13, 16, 6, 5, 2, (2, 3), (2, 1)),
                                                                         (3, 6, 6, 8, 8, 1, 1, (1, 1), (0, 0)), (1, 8, 8, 4, 3, 3, 3, (2, 2), (0, 0)))):
        x = gen(8100 + idx, "row", batch * H * W, Cin).reshape(batch, H, W, Cin)
        w = gen(8200 + idx, "row", kh * kw * Cin, Cout).reshape(kh, kw, Cin, Cout)
        Hout, Wout = oracle.conv_output_shape(H, W, kh, kw, stride, pad)
        if dtype == "i8":
            old = rng.integers(-1000, 1000, size=(batch, Hout, Wout, Cout)).astype(np.int32)
            alpha, beta = 2, -1
        else:
            old = rng.standard_normal((batch, Hout, Wout, Cout)).astype(np.float32)
            alpha, beta = np.float32(1.5), np.float32(0.5)
        got = oracle.conv2d_nhwc(dtype, x, w, stride, pad, alpha, beta, old)
        A = oracle.im2row(dtype, x, kh, kw, stride, pad)
        M, K = A.shape
        assert np.array_equal(decode(A), oracle.im2row_f32(decode(x).astype(np.float32), kh, kw, stride, pad).astype(np.float64))
        via_gemm = gemm("row", M, Cout, K, alpha, A, K, w.reshape(K, Cout), Cout, beta, old.reshape(M, Cout), Cout)
        t = torch.nn.functional.conv2d(torch.from_numpy(decode(x)).permute(0, 3, 1, 2), torch.from_numpy(decode(w)).permute(3, 2, 0, 1),
                                       stride=stride, padding=pad)
        want = float(alpha) * t.permute(0, 2, 3, 1).numpy() + float(beta) * old.astype(np.float64)
        if dtype == "i8":
            assert np.array_equal(got.reshape(M, Cout), via_gemm)
            assert np.array_equal(got, want.astype(np.int64))
        else:
            assert np.allclose(got.reshape(M, Cout), via_gemm, rtol=0, atol=1e-11)
            assert np.allclose(got, want, rtol=0, atol=1e-11)


# ------------------------------------------------------------ narrowing to 16-bit storage
def test_narrowing_to_binary16_against_numpy_and_by_hand():
    # every pattern survives the round trip (NaNs stay NaN)
    bits = np.arange(65536, dtype=np.uint16)
    vals = oracle.half_bits_to_double(bits)
    back = oracle.narrow_f16(vals)
    finite = ~np.isnan(vals)
    assert np.array_equal(back[finite], bits[finite])
    assert np.all(np.isnan(oracle.half_bits_to_double(back[~finite])))
    for b in (0x0001, 0x03FF, 0x0400, 0x3C00, 0x7BFF, 0xFBFF, 0x8000):
        assert oracle.half_to_double(b) == vals[b]
    # ties go to the even neighbour; just above a tie goes up (ulp(1) = 2^-10)
    cases = {1 + 2.0 ** -11: 0x3C00, 1 + 2.0 ** -11 + 2.0 ** -30: 0x3C01, 1 + 3 * 2.0 ** -11: 0x3C02,
             65504.0: 0x7BFF, 65519.999: 0x7BFF, 65520.0: 0x7C00, -65520.0: 0xFC00, 1e9: 0x7C00,
             2.0 ** -24: 0x0001, 2.0 ** -25: 0x0000, 2.0 ** -25 * 1.0001: 0x0001, 3 * 2.0 ** -25: 0x0002,
             2.0 ** -14 - 2.0 ** -25: 0x0400, -0.0: 0x8000, float("inf"): 0x7C00}
    for x, want in cases.items():
        assert int(oracle.narrow_f16(np.array([x]))[0]) == want, (x, hex(want))
    # against numpy's conversion on values of every magnitude, and on every midpoint between neighbours
    rng = np.random.default_rng(5)
    x = rng.standard_normal(200000) * np.exp(rng.uniform(-20, 12, 200000))
    with np.errstate(over="ignore"):
        assert np.array_equal(oracle.narrow_f16(x), x.astype(np.float16).view(np.uint16))
        pos = oracle.half_bits_to_double(np.arange(0, 0x7BFF, dtype=np.uint16))
        mid = (pos[:-1] + pos[1:]) / 2
        assert np.array_equal(oracle.narrow_f16(mid), mid.astype(np.float16).view(np.uint16))
        assert np.array_equal(oracle.narrow_f16(mid) & 1, np.zeros(mid.size, dtype=np.uint16))


def test_narrowing_to_bfloat16():
    bits = np.arange(65536, dtype=np.uint16)
    vals = oracle.bfloat16_bits_to_double(bits)
    back = oracle.narrow_bf16(vals)
    finite = ~np.isnan(vals)
    assert np.array_equal(back[finite], bits[finite])
    for b in (0x0001, 0x007F, 0x0080, 0x3F80, 0x7F7F, 0xFF7F):
        assert oracle.bfloat16_to_double(b) == vals[b]
    # ulp(1) = 2^-7: ties to even, just above goes up, overflow, smallest subnormal 2^-133
    cases = {1 + 2.0 ** -8: 0x3F80, 1 + 2.0 ** -8 + 2.0 ** -40: 0x3F81, 1 + 3 * 2.0 ** -8: 0x3F82,
             (2 - 2.0 ** -7) * 2.0 ** 127: 0x7F7F, (2 - 2.0 ** -8) * 2.0 ** 127: 0x7F80, 2.0 ** -133: 0x0001,
             2.0 ** -134: 0x0000, -1.0: 0xBF80}
    for x, want in cases.items():
        assert int(oracle.narrow_bf16(np.array([x]))[0]) == want, (x, hex(want))
    # on fp32 values the integer rule "add 0x7FFF plus the lowest kept bit, cut" is the same rounding
    rng = np.random.default_rng(6)
    f = (rng.standard_normal(200000) * np.exp(rng.uniform(-60, 60, 200000))).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    want = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
    assert np.array_equal(oracle.narrow_bf16(f.astype(np.float64)), want)
