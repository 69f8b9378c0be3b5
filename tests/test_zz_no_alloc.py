"""gemm_ex_static_ws (the entry point that allocates nothing: the K-split scratch is the library's own
fixed array) against gemm_ex with a caller's workspace of gemm_workspace_bytes, bit for bit, and against
the CPU oracle at the usual bar; two calls in a row on one stream, the second on a smaller problem, so
that what the first call left in the shared array must not leak into the second."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2310_17408_amd as mg
from gpu_case import DT, LAYOUT, TOL, make_inputs, max_abs, oracle_gemm, to_device

pytestmark = pytest.mark.gpu


def _run_pair(dtype, layout, M, N, K, alpha, beta, seed):
    """Returns (C from gemm_ex_static_ws, C from gemm_ex with a workspace, split of each, host inputs)."""
    A, lda, B, ldb, C, ldc = make_inputs(dtype, layout, M, N, K, seed)
    _, dA = to_device(A)
    _, dB = to_device(B)
    _, dC1 = to_device(C)
    _, dC2 = to_device(C)
    need = mg.gemm_workspace_bytes(DT[dtype], M, N, K)
    assert need <= mg.STATIC_WS_BYTES
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda") if need else None
    # raw call through the C ABI: device addresses, host pointers to alpha / beta, the stream handle
    lib = mg.load()
    scal = ctypes.c_int32 if dtype == "i8" else ctypes.c_float
    a, b = scal(alpha), scal(beta)
    stream = torch.cuda.current_stream().cuda_stream
    rc = lib.gemm_ex_static_ws(DT[dtype], LAYOUT[layout], 0, 0, M, N, K, ctypes.byref(a), dA.data_ptr(), lda,
                               dB.data_ptr(), ldb, ctypes.byref(b), dC1.data_ptr(), ldc, stream)
    assert rc == 0, mg.load().gemm_ex_status_string(rc).decode()
    kid1, split1 = mg.gemm_last_kernel_id(), mg.gemm_last_split()
    mg.gemm_ex(DT[dtype], LAYOUT[layout], 0, 0, M, N, K, alpha, dA, lda, dB, ldb, beta, dC2, ldc, ws)
    kid2, split2 = mg.gemm_last_kernel_id(), mg.gemm_last_split()
    torch.cuda.synchronize()
    assert (kid1, split1) == (kid2, split2)
    out1 = dC1.cpu().numpy().reshape(np.shape(C))
    out2 = dC2.cpu().numpy().reshape(np.shape(C))
    return out1, out2, split1, (A, lda, B, ldb, C, ldc)


def _check(dtype, layout, M, N, K, alpha, beta, seed, want_split):
    out1, out2, split, (A, lda, B, ldb, C, ldc) = _run_pair(dtype, layout, M, N, K, alpha, beta, seed)
    if want_split:
        assert split > 1, "the case is meant to use the scratch array (split %d)" % split
    assert np.array_equal(out1.view(np.uint32), out2.view(np.uint32)), "differs from gemm_ex with a workspace"
    if dtype != "i8":
        alpha, beta = np.float32(alpha), np.float32(beta)
    ref = oracle_gemm(dtype, layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc)
    got = wl.logical(layout, out1, M, N)
    if dtype == "i8":
        assert np.array_equal(got, oracle.wrap_int32(ref))
    else:
        err = oracle.normalised_error(got, ref, K, max_abs(dtype, layout, A, M, K), max_abs(dtype, layout, B, K, N))
        assert err <= TOL[dtype], "normalised error %.3e" % err


@pytest.mark.parametrize("dtype,alpha,beta", [("f32", 1.5, 0.5), ("f16", 1.0, 0.0), ("i8", 2, -1)])
def test_two_calls_in_a_row_second_smaller(dtype, alpha, beta):
    # deep K, few output tiles: the selector splits K over workgroups and the partial tiles go to the array
    _check(dtype, "col", 49, 512, 4608, alpha, beta, 9100, want_split=True)
    _check(dtype, "col", 33, 64, 4608, alpha, beta, 9200, want_split=True)
    # and a problem that does not split at all (no scratch used) after those
    _check(dtype, "row", 200, 300, 150, alpha, beta, 9300, want_split=False)


def test_problem_beyond_the_array_is_rejected_before_any_launch():
    M = N = 2048
    K = 65536
    assert mg.gemm_workspace_bytes(mg.F16, M, N, K) > mg.STATIC_WS_BYTES
    one, zero = ctypes.c_float(1.0), ctypes.c_float(0.0)
    P = 0x1000      # never dereferenced
    rc = mg.load().gemm_ex_static_ws(mg.F16, mg.COL_MAJOR, 0, 0, M, N, K, ctypes.byref(one), P, M, P, K, ctypes.byref(zero),
                                     P, M, None)
    assert rc == mg.STATUS_STATIC_WS_TOO_SMALL
    assert "workspace" in mg.load().gemm_ex_status_string(rc).decode()
