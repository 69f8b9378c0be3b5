"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and its host logic (argument checks, quick returns, workspace
sizing, kernel table) behaves as include/mi_gemm.h says.  Nothing here launches
a kernel: every call returns before the first HIP call."""
import ctypes
import os
import re

import pytest

import paper_2310_17408_amd as mg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "mi_gemm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    # every identifier that is followed by an argument list at the start of a declaration
    return sorted(set(re.findall(r"^(?:const\s+)?[a-z_0-9]+\s*\*?\s*([a-z][a-z0-9_]*)\s*\(", text, flags=re.M)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(mg.lib_path())
    names = _declared_functions()
    assert {"gemm_f32", "gemm_f16", "gemm_bf16", "gemm_i8", "gemm_f16_c16", "gemm_bf16_c16", "gemm_ex", "gemm_workspace_bytes",
            "gemm_status_string", "gemm_solo", "gemm_select", "gemm_predict_us", "conv2d_im2row_f32", "im2row_f32",
            "conv2d_im2row_workspace_bytes", "conv2d_im2row_shape", "conv2d_im2row_status_string",
            "gemm_ex_status_string"} <= set(names)
    for n in names:
        assert hasattr(lib, n), "symbol %s is declared but not exported" % n


def test_header_is_plain_c():
    """The boundary is a C header: it must compile as C99 and as C++ without anything else included first."""
    import subprocess
    header = os.path.join(ROOT, "include", "mi_gemm.h")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", header])
    subprocess.check_call(["g++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", header])


def test_kernel_table():
    for dtype in (mg.F32, mg.F16, mg.I8, mg.BF16):
        n = mg.gemm_kernel_count(dtype)
        assert n >= 3
        names = [mg.gemm_kernel_name(dtype, i) for i in range(n)]
        assert len(set(names)) == n and all(names)
        assert mg.gemm_kernel_name(dtype, n) == ""
        assert mg.gemm_force_kernel(dtype, n, 0) == -1
        assert mg.gemm_force_kernel(dtype, 0, 3) == 0
        assert mg.gemm_force_kernel(dtype, -1, 0) == 0
    assert mg.gemm_kernel_count(7) == 0
    assert mg.gemm_force_kernel(5, 0, 0) == -1


@pytest.mark.parametrize("fn", [mg.gemm_f32, mg.gemm_f16, mg.gemm_i8, mg.gemm_bf16, mg.gemm_f16_c16, mg.gemm_bf16_c16])
def test_argument_errors_return_before_any_launch(fn):
    P = 0x1000            # never dereferenced: every call below fails validation or returns early
    ok = dict(layout=mg.COL_MAJOR, M=8, N=9, K=10, alpha=1, A=P, lda=8, B=P, ldb=10, beta=0, C=P, ldc=8)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return fn(a["layout"], a["M"], a["N"], a["K"], a["alpha"], a["A"], a["lda"], a["B"], a["ldb"], a["beta"],
                  a["C"], a["ldc"], None, 0, check=False)

    assert call(layout=2) == -1
    assert call(M=-1) == -2
    assert call(N=-5) == -3
    assert call(K=-1) == -4
    assert call(M=2 ** 31) == -2
    assert call(lda=7) == -7
    assert call(ldb=9) == -9
    assert call(ldc=7) == -12
    assert call(layout=mg.ROW_MAJOR, lda=9, ldb=9, ldc=9) == -7       # row-major: lda >= K
    assert call(layout=mg.ROW_MAJOR, lda=10, ldb=8, ldc=9) == -9      # ldb >= N
    assert call(layout=mg.ROW_MAJOR, lda=10, ldb=9, ldc=8) == -12     # ldc >= N
    assert call(A=None) == -6
    assert call(B=None) == -8
    assert call(C=None) == -11
    # quick returns that touch nothing
    assert call(M=0, lda=1, ldc=1) == 0
    assert call(N=0) == 0
    assert call(M=0, C=None, lda=1, ldc=1) == 0
    assert call(alpha=0, beta=1, A=None, B=None) == 0
    for status in range(0, -16, -1):
        assert mg.gemm_status_string(status)
    with pytest.raises(mg.GemmError):
        fn(mg.COL_MAJOR, 8, 9, 10, 1, P, 7, P, 10, 0, P, 8)


def test_misaligned_workspace_is_rejected():
    lib = mg.load()
    rc = lib.gemm_f32(0, 8, 8, 8, 1.0, 0x1000, 8, 0x1000, 8, 0.0, 0x1000, 8, 0x1004, 1 << 20, None)
    assert rc == -13


def test_workspace_bytes():
    # big squares never split K; skinny long-K problems do, and the bound covers split * M * N * 4
    assert mg.gemm_workspace_bytes(mg.F32, 8192, 8192, 8192) == 0
    assert mg.gemm_workspace_bytes(mg.F32, 0, 10, 10) == 0
    assert mg.gemm_workspace_bytes(9, 10, 10, 10) == 0
    w = mg.gemm_workspace_bytes(mg.F32, 49, 512, 4608)
    assert w >= 2 * 49 * 512 * 4 and w % (49 * 512 * 4) == 0
    assert mg.gemm_workspace_bytes(mg.F32, 49, 512, 4608) == mg.gemm_workspace_bytes(mg.F32, 512, 49, 4608)


def _auto_selectable(dtype, kid):
    # a configuration is open to automatic selection if some problem selects it; the table marks
    # the others as explicit-only, which shows in their never being returned unforced
    probes = [(12544, 64, 147), (3136, 64, 64), (3136, 64, 576), (784, 128, 1152), (196, 256, 2304), (49, 512, 4608),
              (3136, 128, 256), (784, 512, 128), (1024, 1024, 1024), (2048, 2048, 2048), (8192, 8192, 8192),
              (64, 64, 64), (4096, 64, 4096), (50176, 64, 576), (33, 17, 2049), (256, 256, 256)]
    return any(mg.gemm_select(dtype, 0, m, n, k, 32 * m * n * 4)[0] == kid for (m, n, k) in probes)


def test_timing_model_and_selection_agree():
    """gemm_select returns the (configuration, split) with the smallest predicted time among the
    configurations open to automatic selection, and the model behaves sanely: more work never
    takes less time, bad arguments are refused."""
    for dtype in (mg.F32, mg.F16, mg.I8, mg.BF16):
        for (M, N, K) in [(12544, 64, 147), (49, 512, 4608), (1024, 1024, 1024), (4096, 4096, 4096), (33, 17, 2049)]:
            kid, split = mg.gemm_select(dtype, 0, M, N, K, 32 * M * N * 4)
            t = mg.gemm_predict_us(dtype, kid, M, N, K, split)
            assert t > 0
            # forcing another configuration is never predicted to be clearly faster than the pick (a split
            # configuration must beat an unsplit one by 3 %)
            t_eff = t * (1.03 if split > 1 else 1.0)
            for other in range(mg.gemm_kernel_count(dtype)):
                mg.gemm_force_kernel(dtype, other, 0)
                k2, s2 = mg.gemm_select(dtype, 0, M, N, K, 32 * M * N * 4)
                mg.gemm_force_kernel(dtype, -1, 0)
                if k2 != other:
                    continue                       # not addressable for this problem
                name = mg.gemm_kernel_name(dtype, other)
                assert name
                if _auto_selectable(dtype, other):
                    t2 = mg.gemm_predict_us(dtype, other, M, N, K, s2) * (1.03 if s2 > 1 else 1.0)
                    assert t2 >= t_eff * 0.999, (name, M, N, K)
        big = mg.gemm_predict_us(dtype, 0, 4096, 4096, 4096, 1)
        assert big > mg.gemm_predict_us(dtype, 0, 2048, 2048, 2048, 1) > mg.gemm_predict_us(dtype, 0, 512, 512, 512, 1)
    with pytest.raises(mg.GemmError):
        mg.gemm_predict_us(mg.F32, 99, 10, 10, 10, 1)
    with pytest.raises(mg.GemmError):
        mg.gemm_predict_us(mg.F32, 0, 10, 10, 10, 0)


def test_gemm_ex_argument_errors():
    """Status -k names the k-th argument of gemm_ex's own list; nothing is launched."""
    P = 0x1000
    ok = dict(dtype=mg.F32, layout=0, ta=0, tb=0, M=8, N=6, K=4, lda=8, ldb=4, ldc=8)

    def call(**kw):
        a = dict(ok, **kw)
        return mg.gemm_ex(a["dtype"], a["layout"], a["ta"], a["tb"], a["M"], a["N"], a["K"], 1.0, P, a["lda"], P, a["ldb"],
                          0.0, P, a["ldc"], None, check=False)

    assert call(dtype=9) == -1
    assert call(layout=2) == -2
    assert call(ta=2) == -3
    assert call(tb=-1) == -4
    assert call(M=-1) == -5 and call(N=-1) == -6 and call(K=-1) == -7
    # leading dimensions follow the stored matrix: a transposed A is K x M
    assert call(lda=7) == -10 and call(ta=1, lda=3) == -10 and call(ta=1, lda=4, M=0) == 0
    assert call(ldb=3) == -12 and call(tb=1, ldb=5) == -12
    assert call(layout=1, lda=3) == -10 and call(layout=1, ta=1, lda=7) == -10
    assert call(ldc=7) == -15
    assert "argument 10 (lda)" in mg.load().gemm_ex_status_string(-10).decode()
    assert "transa" in mg.load().gemm_ex_status_string(-3).decode()
    lib = mg.load()
    import ctypes
    one = ctypes.c_float(1.0)
    assert lib.gemm_ex(0, 0, 0, 0, 8, 6, 4, None, P, 8, P, 4, ctypes.byref(one), P, 8, None, 0, None) == -8
    assert lib.gemm_ex(0, 0, 0, 0, 8, 6, 4, ctypes.byref(one), P, 8, P, 4, None, P, 8, None, 0, None) == -13


def test_conv_geometry_and_argument_errors():
    """conv2d_im2row_f32 / im2row_f32: shapes and argument checks run on the host before anything is launched."""
    assert mg.conv2d_im2row_shape(1, 224, 224, 3, 64, 7, 7, 2, 2, 3, 3) == (112, 112, 12544, 64, 147)
    assert mg.conv2d_im2row_shape(4, 56, 56, 64, 256, 1, 1, 1, 1, 0, 0) == (56, 56, 4 * 3136, 256, 64)
    assert mg.conv2d_im2row_shape(1, 5, 7, 2, 3, 3, 2, 2, 3, 1, 0) == (3, 2, 6, 3, 12)
    good = [1, 8, 8, 16, 4, 3, 3, 1, 1, 1, 1]
    bad = {1: 0, 2: 0, 3: -1, 4: 0, 5: 0, 6: 0, 7: 0, 8: 0, 9: -2, 10: -1, 11: 1 << 21}
    for pos, value in bad.items():
        args = list(good)
        args[pos - 1] = value
        assert mg.conv2d_im2row_f32(*args, 1.0, 1 << 20, 1 << 20, 0.0, 1 << 20, check=False) == -pos
        assert str(pos) in mg.conv2d_im2row_status_string(-pos)
    # a filter larger than the padded image
    assert mg.conv2d_im2row_f32(1, 4, 8, 16, 4, 7, 3, 1, 1, 1, 1, 1.0, 1 << 20, 1 << 20, 0.0, 1 << 20, check=False) == -10
    assert mg.conv2d_im2row_f32(*good, 1.0, None, 1 << 20, 0.0, 1 << 20, check=False) == -13
    assert mg.conv2d_im2row_f32(*good, 1.0, 1 << 20, None, 0.0, 1 << 20, check=False) == -14
    assert mg.conv2d_im2row_f32(*good, 1.0, 1 << 20, 1 << 20, 0.0, None, check=False) == -16
    assert mg.conv2d_im2row_workspace_bytes(*good) >= 64 * 144 * 4
    assert mg.conv2d_im2row_workspace_bytes(0, *good[1:]) == 0
    assert mg.im2row_f32(1, 8, 8, 16, 3, 3, 1, 1, 1, 1, None, 1 << 20, check=False) == -11
    assert mg.im2row_f32(1, 8, 8, 16, 3, 3, 1, 1, 1, 1, 1 << 20, None, check=False) == -12
    assert mg.im2row_f32(1, 8, 8, 16, 0, 3, 1, 1, 1, 1, 1 << 20, 1 << 20, check=False) == -5
    with pytest.raises(mg.GemmError):
        mg.conv2d_im2row_force_path(3)


def test_repeated_selection_is_a_table_lookup():
    """The timing model runs once per distinct problem and thread: 10^4 repeats of gemm_select on a shape whose
    selection weighs a dozen configurations and splits must cost about a microsecond each at most beyond what the
    foreign-function call itself costs (measured on a call of the same arity that returns at its first check),
    and a fraction of what the same number of distinct problems costs."""
    import time
    lib = mg.load()
    kid, split = ctypes.c_int(-1), ctypes.c_int(0)
    pk, ps = ctypes.byref(kid), ctypes.byref(split)
    ws = mg.gemm_workspace_bytes(mg.F32, 49, 512, 4608)

    def mean_us(dtype, reps=10000, distinct=False):
        t0 = time.perf_counter()
        for i in range(reps):
            lib.gemm_select(dtype, mg.COL_MAJOR, 49, 512, 4608 + (i if distinct else 0), ws, pk, ps)
        return (time.perf_counter() - t0) / reps * 1e6

    for dtype in (mg.F32, mg.F16, mg.I8):
        assert lib.gemm_select(dtype, mg.COL_MAJOR, 49, 512, 4608, ws, pk, ps) == 0      # the first call fills the table
        first = (kid.value, split.value)
        floor = min(mean_us(99) for _ in range(3))             # unknown dtype: returns -1 at once
        cached = min(mean_us(dtype) for _ in range(3))
        assert (kid.value, split.value) == first
        modelled = min(mean_us(dtype, distinct=True) for _ in range(3))   # 10^4 keys through 256 slots: all misses
        what = "selection costs %.2f us per repeat, %.2f us per new problem, the call itself %.2f" % (cached, modelled, floor)
        assert cached - floor < 1.5 and cached - floor < 0.5 * (modelled - floor), what
    # the table is keyed on everything the choice depends on: another workspace size, a forced configuration
    # and a forced split each get their own answer, and the first answer comes back afterwards
    base = mg.gemm_select(mg.F32, mg.COL_MAJOR, 49, 512, 4608, ws)
    assert mg.gemm_select(mg.F32, mg.COL_MAJOR, 49, 512, 4608, 0)[1] == 1
    mg.gemm_force_kernel(mg.F32, 0, 3)
    try:
        assert mg.gemm_select(mg.F32, mg.COL_MAJOR, 49, 512, 4608, ws) == (0, 3)
    finally:
        mg.gemm_force_kernel(mg.F32, -1, 0)
    assert mg.gemm_select(mg.F32, mg.COL_MAJOR, 49, 512, 4608, ws) == base
    assert mg.gemm_select(mg.F32, mg.ROW_MAJOR, 512, 49, 4608, ws) == base           # the same canonical problem


def test_force_kernel_is_per_thread():
    import threading
    seen = {}
    mg.gemm_force_kernel(mg.F32, 0, 2)
    try:
        t = threading.Thread(target=lambda: seen.setdefault("other", mg.gemm_select(mg.F32, mg.COL_MAJOR, 49, 512, 4608, 1 << 22)))
        t.start()
        t.join()
        seen["mine"] = mg.gemm_select(mg.F32, mg.COL_MAJOR, 49, 512, 4608, 1 << 22)
    finally:
        mg.gemm_force_kernel(mg.F32, -1, 0)
    assert seen["mine"] == (0, 2)
    assert seen["other"] == mg.gemm_select(mg.F32, mg.COL_MAJOR, 49, 512, 4608, 1 << 22) != (0, 2)


def test_static_workspace_entry_point_rejects_what_does_not_fit():
    lib = mg.load()
    M = N = 2048
    K = 65536
    assert mg.gemm_workspace_bytes(mg.F16, M, N, K) > mg.STATIC_WS_BYTES
    one, zero = ctypes.c_float(1.0), ctypes.c_float(0.0)
    P = 0x1000      # never dereferenced: the call returns before any HIP call
    rc = lib.gemm_ex_static_ws(mg.F16, mg.COL_MAJOR, 0, 0, M, N, K, ctypes.byref(one), P, M, P, K, ctypes.byref(zero), P, M, None)
    assert rc == mg.STATUS_STATIC_WS_TOO_SMALL
    # argument errors are those of gemm_ex, in the same positions
    assert lib.gemm_ex_static_ws(9, mg.COL_MAJOR, 0, 0, 8, 8, 8, ctypes.byref(one), P, 8, P, 8, ctypes.byref(zero), P, 8, None) == -1
    assert lib.gemm_ex_static_ws(mg.F32, mg.COL_MAJOR, 0, 0, 8, 8, 8, ctypes.byref(one), P, 7, P, 8, ctypes.byref(zero), P, 8, None) == -10
