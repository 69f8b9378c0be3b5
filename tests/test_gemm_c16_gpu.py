"""gemm_f16_c16 / gemm_bf16_c16 (C kept in the 16-bit format of the inputs) against the CPU oracle, element by
element through the C-ABI: every kernel of both data types, both layouts, ragged and padded shapes, K split
(reduce kernel), the beta-only path, and the rounding itself bit for bit on cases whose exact value is known."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2310_17408_amd as mg
from gpu_case import DT, LAYOUT, to_device

pytestmark = pytest.mark.gpu
FN = {"f16": mg.gemm_f16_c16, "bf16": mg.gemm_bf16_c16}
GEN = {"f16": wl.normal_f16_bits, "bf16": wl.normal_bf16_bits}
SMALL = {"f16": wl.small_int_f16_bits, "bf16": wl.small_int_bf16_bits}
WIDE = {"f16": oracle.half_bits_to_double, "bf16": oracle.bfloat16_bits_to_double}
NARROW = {"f16": oracle.narrow_f16, "bf16": oracle.narrow_bf16}
ORACLE = {"f16": oracle.gemm_f16, "bf16": oracle.gemm_bf16}
ULP = {"f16": 2.0 ** -10, "bf16": 2.0 ** -7}


def run(dtype, layout, M, N, K, alpha, beta, seed, pad=(0, 0, 0), kernel_id=-1, split=0, gen=None):
    gen = gen or GEN[dtype]
    lda, ldb, ldc = (wl.tight_ld(layout, M, K) + pad[0], wl.tight_ld(layout, K, N) + pad[1], wl.tight_ld(layout, M, N) + pad[2])
    A, B, C = gen(seed, layout, M, K, lda), gen(seed + 1, layout, K, N, ldb), gen(seed + 2, layout, M, N, ldc)
    _, dA = to_device(A)
    _, dB = to_device(B)
    _, dC = to_device(C)
    nbytes = max(mg.gemm_workspace_bytes(DT[dtype], M, N, K), split * M * N * 4, 16)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    mg.gemm_force_kernel(DT[dtype], kernel_id, split)
    try:
        FN[dtype](LAYOUT[layout], M, N, K, alpha, dA, lda, dB, ldb, beta, dC, ldc, ws)
        kid, ks = mg.gemm_last_kernel_id(), mg.gemm_last_split()
    finally:
        mg.gemm_force_kernel(DT[dtype], -1, 0)
    torch.cuda.synchronize()
    out = dC.cpu().numpy().view(np.uint16).reshape(C.shape)
    c_old = WIDE[dtype](C).astype(np.float32)           # exact: 16-bit values are fp32 values
    ref = ORACLE[dtype](layout, M, N, K, np.float32(alpha), A, lda, B, ldb, np.float32(beta), c_old if beta != 0 else None, ldc)
    got_bits = wl.logical(layout, out, M, N)
    # padding of C untouched
    mask = np.ones(out.shape, dtype=bool)
    wl.logical(layout, mask, M, N)[...] = False
    assert np.array_equal(out[mask], C[mask])
    return got_bits, ref, (wl.logical(layout, A, M, K), wl.logical(layout, B, K, N)), kid, ks


def check(dtype, layout, M, N, K, alpha, beta, seed, **kw):
    got_bits, ref, (A, B), kid, ks = run(dtype, layout, M, N, K, alpha, beta, seed, **kw)
    got = WIDE[dtype](got_bits)
    assert np.isfinite(got).all()
    ma, mb = float(np.abs(WIDE[dtype](A)).max()), float(np.abs(WIDE[dtype](B)).max())
    err = oracle.normalised_error(got, ref, max(K, 1), ma or 1.0, mb or 1.0)
    assert err <= 2e-3, (dtype, layout, M, N, K, kid, ks, err)
    # and the stored value is the oracle's value rounded to the format, up to the fp32 accumulation error:
    # within one unit in the last place of the larger of the result and the accumulation bound
    want = WIDE[dtype](NARROW[dtype](ref))
    slack = ULP[dtype] * np.maximum(np.abs(want), 1e-3 * K * ma * mb)
    assert np.all(np.abs(got - want) <= slack), (dtype, kid, ks)
    return kid, ks


def _kernels(dtype):
    return range(mg.gemm_kernel_count(DT[dtype]))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("layout", ["col", "row"])
def test_every_kernel(dtype, layout):
    for kid in _kernels(dtype):
        got, _ = check(dtype, layout, 304, 272, 256, 1.5, 0.5, 9000 + kid, kernel_id=kid)
        assert got == kid
        check(dtype, layout, 333, 259, 131, 1.0, 0.0, 9100 + kid, kernel_id=kid, pad=(1, 2, 3))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_k_split_goes_through_the_reduce_kernel(dtype):
    for kid in _kernels(dtype):
        _, ks = check(dtype, "col", 96, 80, 2048, 1.0, -0.5, 9200 + kid, kernel_id=kid, split=4)
        assert ks == 4 or "_k" in mg.gemm_kernel_name(DT[dtype], kid)
    check(dtype, "row", 49, 512, 4608, 1.0, 0.0, 9250)         # automatic choice on a headline shape


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_small_integers_are_bit_exact(dtype):
    """Inputs in {-8..8}: every product sum and the update are exact, so the stored bits are the oracle's."""
    for kid in _kernels(dtype):
        bits, ref, _, _, _ = run(dtype, "col", 130, 70, 24, 1.0, 2.0, 9300 + kid, kernel_id=kid, gen=SMALL[dtype])
        assert np.abs(ref).max() <= 2048 if dtype == "f16" else True
        if dtype == "bf16":
            ok = np.abs(ref) <= 256          # integers beyond 2^8 are not all bfloat16 values
            assert np.array_equal(bits[ok], NARROW[dtype](ref)[ok])
        else:
            assert np.array_equal(bits, NARROW[dtype](ref))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_rounding_is_to_nearest_even_once(dtype):
    """K = 1: alpha*a*b is exact in fp32, so the stored pattern must be the one rounding of the exact product,
    for magnitudes from the subnormal range to overflow."""
    M, N = 256, 192
    rng = np.random.default_rng(9400)
    a = rng.standard_normal(M) * np.exp(rng.uniform(-9, 6, M))
    b = rng.standard_normal(N) * np.exp(rng.uniform(-9, 6, N))
    A, B = NARROW[dtype](a).reshape(1, M), NARROW[dtype](b).reshape(N, 1)       # column-major M x 1 and 1 x N
    C = np.zeros((N, M), dtype=np.uint16)
    _, dA = to_device(A)
    _, dB = to_device(B)
    _, dC = to_device(C)
    FN[dtype](mg.COL_MAJOR, M, N, 1, 1.0, dA, M, dB, 1, 0.0, dC, M)
    torch.cuda.synchronize()
    got = dC.cpu().numpy().view(np.uint16).reshape(N, M)
    exact = np.outer(WIDE[dtype](B.reshape(-1)), WIDE[dtype](A.reshape(-1)))
    want = NARROW[dtype](exact)
    if dtype == "bf16":
        # fp32 flushes nothing here, but products below the fp32 normal range are not exact in fp32
        keep = np.abs(exact) >= 2.0 ** -126
        assert np.array_equal(got[keep], want[keep])
    else:
        assert np.array_equal(got, want)
    wide = WIDE[dtype](want)
    assert np.isinf(wide).any() if dtype == "f16" else True
    assert ((wide != 0) & (np.abs(wide) < (2.0 ** -14 if dtype == "f16" else 0))).any() if dtype == "f16" else True


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_beta_only_paths(dtype):
    """alpha == 0 (scale kernel) and beta == 0 over a NaN-filled C."""
    M, N, K = 70, 50, 40
    C = GEN[dtype](9500, "col", M, N, M)
    _, dC = to_device(C)
    FN[dtype](mg.COL_MAJOR, M, N, K, 0.0, None, M, None, K, 0.5, dC, M)
    torch.cuda.synchronize()
    got = dC.cpu().numpy().view(np.uint16).reshape(C.shape)
    assert np.array_equal(got, NARROW[dtype](0.5 * WIDE[dtype](C)))
    nan = np.full((N, M), 0x7E00 if dtype == "f16" else 0x7FC0, dtype=np.uint16)
    A, B = GEN[dtype](9501, "col", M, K, M), GEN[dtype](9502, "col", K, N, K)
    _, dA = to_device(A)
    _, dB = to_device(B)
    _, dN = to_device(nan)
    FN[dtype](mg.COL_MAJOR, M, N, K, 1.0, dA, M, dB, K, 0.0, dN, M)
    torch.cuda.synchronize()
    assert np.isfinite(WIDE[dtype](dN.cpu().numpy().view(np.uint16))).all()
