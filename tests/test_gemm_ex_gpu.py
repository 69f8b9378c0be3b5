"""GPU parity of the general entry point gemm_ex (transposed operands, every data type) against the
oracle's gemm_ex, element by element, on seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2310_17408_amd as mg
from gpu_case import DT, LAYOUT, TIGHT, TOL, max_abs, to_device

pytestmark = pytest.mark.gpu

GEN = {"f32": wl.uniform_f32, "f16": wl.normal_f16_bits, "bf16": wl.normal_bf16_bits, "i8": wl.uniform_i8}
DIRECT = ("_dma16", "_ring")       # the direct-to-LDS kernels with 16 x 16 MFMA blocks: two stages, or a ring of four
SMALL = {"f32": wl.small_int_f32, "f16": wl.small_int_f16_bits, "bf16": wl.small_int_bf16_bits}


def _case(dtype, layout, ta, tb, M, N, K, alpha, beta, seed, pad=(0, 0, 0), kernel_id=-1, split=0, exact=False):
    ar, ac = (K, M) if ta else (M, K)          # the stored matrices
    br, bc = (N, K) if tb else (K, N)
    lda = wl.tight_ld(layout, ar, ac) + pad[0]
    ldb = wl.tight_ld(layout, br, bc) + pad[1]
    ldc = wl.tight_ld(layout, M, N) + pad[2]
    gen = SMALL[dtype] if exact else GEN[dtype]
    A, B = gen(seed, layout, ar, ac, lda), gen(seed + 1, layout, br, bc, ldb)
    if dtype == "i8":
        C = wl.uniform_i32(seed + 2, layout, M, N, ldc)
    else:
        C = (wl.small_int_f32 if exact else wl.uniform_f32)(seed + 2, layout, M, N, ldc)
    _, dA = to_device(A)
    _, dB = to_device(B)
    _, dC = to_device(C)
    nbytes = max(mg.gemm_workspace_bytes(DT[dtype], M, N, K), max(split, 1) * M * N * 4, 16)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    mg.gemm_force_kernel(DT[dtype], kernel_id, split)
    try:
        mg.gemm_ex(DT[dtype], LAYOUT[layout], ta, tb, M, N, K, alpha, dA, lda, dB, ldb, beta, dC, ldc, ws)
        kid, ks = mg.gemm_last_kernel_id(), mg.gemm_last_split()
    finally:
        mg.gemm_force_kernel(DT[dtype], -1, 0)
    torch.cuda.synchronize()
    out = dC.cpu().numpy().reshape(C.shape)
    ref = oracle.gemm_ex(dtype, layout, ta, tb, M, N, K, alpha, A, lda, B, ldb, beta, C if beta != 0 else None, ldc)
    got = wl.logical(layout, out, M, N)
    what = "%s %s ta=%d tb=%d %dx%dx%d kernel %s split %d" % (dtype, layout, ta, tb, M, N, K,
                                                            mg.gemm_kernel_name(DT[dtype], kid), ks)
    if dtype == "i8":
        assert np.array_equal(got, oracle.wrap_int32(ref)), what
    elif exact:
        assert np.array_equal(got.astype(np.float64), ref), what
    else:
        err = oracle.normalised_error(got, ref, K, max_abs(dtype, layout, A, ar, ac) or 1.0,
                                      max_abs(dtype, layout, B, br, bc) or 1.0)
        assert err <= TOL[dtype], "%s: normalised error %.3e" % (what, err)
        assert err <= TIGHT[dtype], "%s: normalised error %.3e above the internal bound" % (what, err)
    mask = np.ones(out.shape, dtype=bool)
    wl.logical(layout, mask, M, N)[...] = False
    assert np.array_equal(out[mask], np.asarray(C)[mask]), what + ": padding of C was overwritten"
    return kid, ks


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i8"])
@pytest.mark.parametrize("layout", ["col", "row"])
@pytest.mark.parametrize("ta,tb", [(0, 0), (1, 0), (0, 1), (1, 1)])
def test_gemm_ex_all_orientations(dtype, layout, ta, tb):
    a, b = (3, -2) if dtype == "i8" else (1.5, 0.5)
    # several tiles of every staged configuration, 16-byte aligned rows
    _case(dtype, layout, ta, tb, 320, 272, 192, a, b, seed=7000)
    # ragged everywhere, odd leading dimensions, a K tail
    _case(dtype, layout, ta, tb, 133, 77, 91, a, b, seed=7100, pad=(1, 2, 3))
    # tiny
    _case(dtype, layout, ta, tb, 7, 5, 3, 1, 0, seed=7200)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i8"])
@pytest.mark.parametrize("ta,tb", [(1, 0), (0, 1), (1, 1)])
def test_gemm_ex_transposed_every_staged_kernel_and_split(dtype, ta, tb):
    """Every configuration that takes transposed operands, unsplit and with K split over workgroups;
    a forced configuration that does not take them must be replaced, not run."""
    n = mg.gemm_kernel_count(DT[dtype])
    ran = set()
    for kid in range(n):
        a, b = (1, 1) if dtype == "i8" else (1.0, 1.0)
        k, s = _case(dtype, "col", ta, tb, 200, 136, 700, a, b, seed=7300 + kid, kernel_id=kid)
        ran.add(k)
        k2, s2 = _case(dtype, "row", ta, tb, 200, 136, 2100, a, b, seed=7400 + kid, kernel_id=kid, split=3)
        assert s2 == 3 or k2 != kid
    assert len(ran) >= 2          # at least the 64x64 and one larger staged tile ran


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("ta,tb", [(1, 0), (0, 1), (1, 1)])
def test_gemm_ex_small_integers_exact(dtype, ta, tb):
    for layout in ("col", "row"):
        _case(dtype, layout, ta, tb, 150, 140, 1024, 2, -1, seed=7500, exact=True)


def test_gemm_ex_untransposed_is_the_plain_entry_point():
    """transa = transb = 0 selects and computes exactly what gemm_f32 does."""
    M, N, K = 300, 200, 150
    A, B, C = wl.uniform_f32(1, "col", M, K), wl.uniform_f32(2, "col", K, N), wl.uniform_f32(3, "col", M, N)
    _, dA = to_device(A)
    _, dB = to_device(B)
    _, c1 = to_device(C)
    _, c2 = to_device(C)
    mg.gemm_f32(mg.COL_MAJOR, M, N, K, 1.5, dA, M, dB, K, 0.5, c1, M)
    k1 = mg.gemm_last_kernel_id()
    mg.gemm_ex(mg.F32, mg.COL_MAJOR, 0, 0, M, N, K, 1.5, dA, M, dB, K, 0.5, c2, M)
    assert mg.gemm_last_kernel_id() == k1
    torch.cuda.synchronize()
    assert torch.equal(c1, c2)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_k_contiguous_a_on_the_direct_kernels(dtype):
    """op(A) = A^T in column-major terms, or x W^T in row-major terms (both operands with K contiguous): the
    direct-to-LDS kernels stage A like B.  Aligned multi-tile shapes (transfers only), shapes whose last tile
    is moved back, odd leading dimensions (guarded staging) and a K split, on every such kernel; and the
    automatic choice must be one of them for a large problem."""
    direct = [i for i in range(mg.gemm_kernel_count(DT[dtype])) if mg.gemm_kernel_name(DT[dtype], i).endswith(DIRECT)]
    assert len(direct) >= 3
    a, b = (3, -2) if dtype == "i8" else (1.5, 0.5)
    for kid in direct:
        k, _ = _case(dtype, "col", 1, 0, 512, 384, 256, a, b, seed=7600 + kid, kernel_id=kid)
        assert k == kid
        k, _ = _case(dtype, "row", 0, 1, 640, 512, 320, a, b, seed=7610 + kid, kernel_id=kid)
        assert k == kid
        _case(dtype, "col", 1, 0, 400, 336, 448, a, b, seed=7620 + kid, kernel_id=kid)            # edge tiles moved back
        _case(dtype, "col", 1, 0, 300, 270, 200, a, b, seed=7630 + kid, kernel_id=kid, pad=(3, 5, 1))
        k, s = _case(dtype, "row", 0, 1, 256, 256, 2048, a, b, seed=7640 + kid, kernel_id=kid, split=4)
        assert (k, s) == (kid, 4)
    k, _ = _case(dtype, "row", 0, 1, 2048, 2048, 1024, 1, 0, seed=7650)
    assert mg.gemm_kernel_name(DT[dtype], k).endswith(DIRECT)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_n_contiguous_b_on_the_square_direct_kernels(dtype):
    """op(B) = B^T in column-major terms (B with N contiguous), alone and together with a K-contiguous A: the
    direct kernels with square tiles stage B like the canonical A (transposing LDS reads)."""
    square = [i for i in range(mg.gemm_kernel_count(DT[dtype]))
              if mg.gemm_kernel_name(DT[dtype], i).endswith(DIRECT) and mg.gemm_kernel_tile(DT[dtype], i)[0] == mg.gemm_kernel_tile(DT[dtype], i)[1]]
    assert len(square) >= 2
    a, b = (3, -2) if dtype == "i8" else (1.5, 0.5)
    for kid in square:
        for ta in (0, 1):
            k, _ = _case(dtype, "col", ta, 1, 512, 768, 256, a, b, seed=7700 + 2 * kid + ta, kernel_id=kid)
            assert k == kid
            _case(dtype, "col", ta, 1, 400, 336, 448, a, b, seed=7720 + 2 * kid + ta, kernel_id=kid)         # edge tiles moved back
            _case(dtype, "col", ta, 1, 300, 270, 200, a, b, seed=7740 + 2 * kid + ta, kernel_id=kid, pad=(3, 5, 1))
        k, _ = _case(dtype, "row", 1, 0, 640, 512, 320, a, b, seed=7760 + kid, kernel_id=kid)               # row-major: transa is the N-contiguous B
        assert k == kid
        k, s = _case(dtype, "col", 1, 1, 256, 256, 2048, a, b, seed=7770 + kid, kernel_id=kid, split=4)
        assert (k, s) == (kid, 4)
    # a tile that is not square cannot take it: the selector must replace it
    odd = [i for i in range(mg.gemm_kernel_count(DT[dtype])) if mg.gemm_kernel_name(DT[dtype], i).endswith("128x64_w64x32_dma16")]
    k, _ = _case(dtype, "col", 0, 1, 300, 270, 200, a, b, seed=7780, kernel_id=odd[0])
    assert k != odd[0]
    for ta in (0, 1):
        k, _ = _case(dtype, "col", ta, 1, 2048, 2048, 1024, 1, 0, seed=7790 + ta)
        assert mg.gemm_kernel_name(DT[dtype], k).endswith(DIRECT)


@pytest.mark.parametrize("ta,tb", [(1, 0), (0, 1), (1, 1)])
def test_fp32_transposed_operands_on_the_direct_kernels(ta, tb):
    """The fp32 direct-to-LDS configurations that take transposed operands (each operand is staged as it lies in
    memory; only the fragment index maps change): aligned multi-tile shapes (transfers only), last tiles moved
    back (at rows that are and are not 16-byte aligned), matrices smaller than a tile, odd leading dimensions
    (guarded staging), a partial last K step, a K split; the automatic choice for a large aligned problem must be
    one of them."""
    names = [mg.gemm_kernel_name(mg.F32, i) for i in range(mg.gemm_kernel_count(mg.F32))]
    direct = [i for i, nm in enumerate(names) if nm in ("f32_64x64_w32x32_dma", "f32_128x64_w64x32_dma", "f32_128x128_w64x64_dma")]
    assert len(direct) == 3
    for kid in direct:
        for layout in ("col", "row"):
            k, _ = _case("f32", layout, ta, tb, 512, 384, 256, 1.5, 0.5, seed=7800 + kid, kernel_id=kid)
            assert k == kid
            _case("f32", layout, ta, tb, 400, 336, 448, 1.5, 0.5, seed=7810 + kid, kernel_id=kid)        # moved back, aligned rows
            _case("f32", layout, ta, tb, 402, 331, 203, 1.5, 0.5, seed=7820 + kid, kernel_id=kid)        # moved back, unaligned
        _case("f32", "col", ta, tb, 300, 270, 200, 1.5, 0.5, seed=7830 + kid, kernel_id=kid, pad=(3, 5, 1))
        _case("f32", "col", ta, tb, 40, 50, 100, 1.5, 0.0, seed=7840 + kid, kernel_id=kid)
        k, s = _case("f32", "row", ta, tb, 256, 256, 2048, 1.5, 0.5, seed=7850 + kid, kernel_id=kid, split=4)
        assert (k, s) == (kid, 4)
        _case("f32", "col", ta, tb, 150, 140, 1024, 2, -1, seed=7860 + kid, kernel_id=kid, exact=True)
    k, _ = _case("f32", "col", ta, tb, 2048, 2048, 512, 1.0, 0.0, seed=7870)
    assert k in direct
    _case("f32", "col", ta, tb, 1026, 1026, 514, 1.0, 0.0, seed=7880)          # rows of 1026 or 514 floats: no transfers
