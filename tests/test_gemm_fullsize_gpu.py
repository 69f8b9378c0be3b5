"""GPU parity at the benchmark's full sizes, in the launch configuration the
benchmark times (automatic kernel selection, tight leading dimensions).

The full triple loop would take hours at 8192^3, so each case is checked twice:
  * sampled outputs: the oracle's definition evaluated one element at a time at
    rows / columns next to every tile boundary and at random positions;
  * all outputs at once through a Freivalds product: C x against
    alpha * A (B x) + beta * C_old x for random +-1 vectors x, in fp64 (exact
    integers for int8), which any wrong tile or element would upset.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2310_17408_amd as mg
from gpu_case import DT, TIGHT, TOL, gpu_gemm, make_inputs, max_abs

pytestmark = pytest.mark.gpu


def _sample_positions(M, N, rng, n_random=6000, per_edge=48):
    edges = set()
    for t in (32, 64, 128, 256):
        for base in range(0, max(M, N) + 1, t):
            for d in (-1, 0):
                edges.add(base + d)
    rows_e = np.array(sorted(e for e in edges if 0 <= e < M))
    cols_e = np.array(sorted(e for e in edges if 0 <= e < N))
    # thin the boundary lists to keep the sample bounded, always keeping the first and last tiles
    if rows_e.size > 200:
        rows_e = np.concatenate([rows_e[:60], rng.choice(rows_e[60:-60], 80, replace=False), rows_e[-60:]])
    if cols_e.size > 200:
        cols_e = np.concatenate([cols_e[:60], rng.choice(cols_e[60:-60], 80, replace=False), cols_e[-60:]])
    r = [rng.integers(0, M, n_random)]
    c = [rng.integers(0, N, n_random)]
    for e in rows_e:
        r.append(np.full(per_edge, e))
        c.append(rng.integers(0, N, per_edge))
    for e in cols_e:
        r.append(rng.integers(0, M, per_edge))
        c.append(np.full(per_edge, e))
    return np.concatenate(r).astype(np.int64), np.concatenate(c).astype(np.int64)


def _as_f64_blocks(dtype, view):
    """Row blocks of a logical matrix view as float64 (binary16 bit patterns are decoded by numpy)."""
    step = 512
    for i in range(0, view.shape[0], step):
        blk = view[i:i + step]
        if dtype == "f16":
            blk = np.ascontiguousarray(blk).view(np.float16)
        yield i, np.asarray(blk, dtype=np.float64)


def _matvec(dtype, view, x):
    out = np.zeros(view.shape[0])
    for i, blk in _as_f64_blocks(dtype, view):
        out[i:i + blk.shape[0]] = blk @ x
    return out


def _full_size_case(dtype, layout, M, N, K, alpha, beta, seed):
    A, lda, B, ldb, C, ldc = make_inputs(dtype, layout, M, N, K, seed)
    if dtype != "i8":
        alpha, beta = np.float32(alpha), np.float32(beta)
    out, kid, split = gpu_gemm(dtype, layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc)
    got = wl.logical(layout, out, M, N)
    max_a, max_b = max_abs(dtype, layout, A, M, K), max_abs(dtype, layout, B, K, N)
    rng = np.random.default_rng(seed + 77)

    # 1. sampled elements against the oracle's definition
    rows, cols = _sample_positions(M, N, rng)
    ref = oracle.gemm_sample(dtype, layout, K, alpha, A, lda, B, ldb, beta, C if beta != 0 else None, ldc, rows, cols)
    g = got[rows, cols]
    if dtype == "i8":
        assert np.array_equal(g, oracle.wrap_int32(ref.astype(np.int64))), "sampled int8 outputs differ (kernel %d)" % kid
    else:
        err = oracle.normalised_error(g, ref, K, max_a, max_b)
        assert err <= TOL[dtype], "sampled error %.3e (kernel %d split %d)" % (err, kid, split)
        assert err <= TIGHT[dtype], "sampled error %.3e above the internal bound (kernel %d split %d)" % (err, kid, split)

    # 2. every element through random +-1 vectors
    a_view = wl.logical(layout, A if dtype != "f16" else A, M, K)
    b_view = wl.logical(layout, B, K, N)
    c_view = wl.logical(layout, C, M, N)
    for _ in range(2):
        x = rng.choice([-1.0, 1.0], N)
        want = float(alpha) * _matvec(dtype, a_view, _matvec(dtype, b_view, x))
        if beta != 0:
            want = want + float(beta) * _matvec("f32", c_view, x)
        have = _matvec("f32", got, x)
        if dtype == "i8":
            assert np.array_equal(have, want), "Freivalds product differs for int8 (kernel %d)" % kid
        else:
            # fp32 accumulation for every input type (16-bit products are exact in fp32): one bound
            bound = 1e-7 * K * max_a * max_b * np.sqrt(N)
            assert np.max(np.abs(have - want)) <= bound, "Freivalds residual %.3e > %.3e (kernel %d)" % (
                np.max(np.abs(have - want)), bound, kid)
    return kid, split


@pytest.mark.parametrize("n", wl.FP32_SQUARES)
def test_fp32_squares_full_size(n):
    _full_size_case("f32", "col", n, n, n, 1.5, 0.5, 2000 + n)


@pytest.mark.parametrize("n", wl.FP16_SQUARES)
def test_fp16_squares_full_size(n):
    _full_size_case("f16", "row", n, n, n, 1.0, 0.0, 3000 + n)


@pytest.mark.parametrize("layout", ["col", "row"])
def test_int8_4096_full_size(layout):
    _full_size_case("i8", layout, 4096, 4096, 4096, 1, 0, 5000)


def test_fp32_1024_every_element():
    """The smallest square of the sweep is cheap enough for the full oracle."""
    from gpu_case import check_case
    check_case("f32", "col", 1024, 1024, 1024, 1.5, 0.5, seed=2999)
