"""ctypes loader for the CPU oracle (``ref_gemm.c``).  TEST INFRASTRUCTURE ONLY.

Nothing here does arithmetic of the method except ``wrap_int32`` (reduction of
the exact int64 result modulo 2^32, the int8 contract) and
``normalised_error`` (the acceptance metric max|C - C_ref| / (K max|A| max|B|)).
Arrays are numpy, host memory.  ``layout`` is "col" or "row"; a matrix is passed
as the 1-D or 2-D numpy buffer that holds it plus its leading dimension.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ref_gemm.c")
_SRC_CONV = os.path.join(_HERE, "ref_conv.c")
_LIB = os.path.join(_HERE, "libref_gemm.so")
_lib = None

_LAYOUT = {"col": 0, "row": 1}


def build(force=False):
    """Compile ref_gemm.c and ref_conv.c into libref_gemm.so next to them (gcc -O2 -fopenmp)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_CONV)):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-o", tmp, _SRC, _SRC_CONV, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, f32, i32, vp, dbl = (ctypes.c_int64, ctypes.c_float, ctypes.c_int32,
                                  ctypes.c_void_p, ctypes.c_double)
        for name, scal in (("ref_gemm_f32", f32), ("ref_gemm_f16", f32), ("ref_gemm_bf16", f32), ("ref_gemm_i8", i32)):
            fn = getattr(lib, name)
            fn.restype = ctypes.c_int
            fn.argtypes = [ctypes.c_int, i64, i64, i64, scal, vp, i64, vp, i64, scal, vp, i64, vp, i64]
        lib.ref_gemm_ex.restype = ctypes.c_int
        lib.ref_gemm_ex.argtypes = [ctypes.c_int] * 4 + [i64, i64, i64, dbl, vp, i64, vp, i64, dbl, vp, i64, vp, i64]
        lib.ref_gemm_sample.restype = ctypes.c_int
        lib.ref_gemm_sample.argtypes = [ctypes.c_int, ctypes.c_int, i64, dbl, vp, i64, vp, i64,
                                        dbl, vp, i64, i64, vp, vp, vp]
        lib.ref_half_to_double.restype = dbl
        lib.ref_half_to_double.argtypes = [ctypes.c_uint16]
        lib.ref_bfloat16_to_double.restype = dbl
        lib.ref_bfloat16_to_double.argtypes = [ctypes.c_uint16]
        lib.ref_num_threads.restype = ctypes.c_int
        for name in ("ref_narrow_f16", "ref_narrow_bf16"):
            getattr(lib, name).restype = None
            getattr(lib, name).argtypes = [vp, vp, i64]
        lib.ref_im2row_f32.restype = ctypes.c_int
        lib.ref_im2row_f32.argtypes = [i64] * 10 + [vp, vp]
        lib.ref_im2row_ex.restype = ctypes.c_int
        lib.ref_im2row_ex.argtypes = [ctypes.c_int] + [i64] * 10 + [vp, vp]
        lib.ref_conv2d_nhwc_ex.restype = ctypes.c_int
        lib.ref_conv2d_nhwc_ex.argtypes = [ctypes.c_int] + [i64] * 11 + [dbl, vp, vp, dbl, vp, vp]
        lib.ref_conv2d_nhwc_f32.restype = ctypes.c_int
        lib.ref_conv2d_nhwc_f32.argtypes = [i64] * 11 + [f32, vp, vp, f32, vp, vp]
        _lib = lib
    return _lib


def num_threads():
    """Threads the oracle's OpenMP loops use (OMP_NUM_THREADS or the core count)."""
    return int(_load().ref_num_threads())


def half_to_double(bits):
    return float(_load().ref_half_to_double(int(bits) & 0xFFFF))


def bfloat16_to_double(bits):
    return float(_load().ref_bfloat16_to_double(int(bits) & 0xFFFF))


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _extent(layout, rows, cols, ld):
    """Elements the buffer of a rows x cols matrix with leading dimension ld must hold."""
    if rows == 0 or cols == 0:
        return 0
    return (cols - 1) * ld + rows if layout == "col" else (rows - 1) * ld + cols


def _check(name, a, dtype, layout, rows, cols, ld):
    if a is None:
        return
    if a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise ValueError("%s must be a C-contiguous %s buffer" % (name, np.dtype(dtype)))
    if a.size < _extent(layout, rows, cols, ld):
        raise ValueError("%s buffer too small for %dx%d with ld=%d" % (name, rows, cols, ld))


def _run(fn, in_dtype, c_dtype, d_dtype, layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc):
    _check("A", A, in_dtype, layout, M, K, lda)
    _check("B", B, in_dtype, layout, K, N, ldb)
    _check("C", C, c_dtype, layout, M, N, ldc)
    ldd = max(1, M if layout == "col" else N)
    D = np.zeros((N, M) if layout == "col" else (M, N), dtype=d_dtype)
    if C is None:
        if beta != 0:
            raise ValueError("beta != 0 needs C")
        ldc = ldd
    rc = fn(_LAYOUT[layout], M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc, _ptr(D), ldd)
    if rc != 0:
        raise RuntimeError("oracle returned %d" % rc)
    # D is returned as an M x N array (logical indexing), whatever the layout
    return D.T if layout == "col" else D


def gemm_f32(layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc):
    """float32 inputs; returns the un-narrowed double result as an (M, N) array."""
    return _run(_load().ref_gemm_f32, np.float32, np.float32, np.float64,
                layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc)


def gemm_f16(layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc):
    """binary16 bit patterns (uint16) in, float32 C in; returns double (M, N)."""
    return _run(_load().ref_gemm_f16, np.uint16, np.float32, np.float64,
                layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc)


def gemm_bf16(layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc):
    """bfloat16 bit patterns (uint16) in, float32 C in; returns double (M, N)."""
    return _run(_load().ref_gemm_bf16, np.uint16, np.float32, np.float64,
                layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc)


def gemm_i8(layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc):
    """int8 inputs, int32 C in; returns the exact int64 result (M, N)."""
    return _run(_load().ref_gemm_i8, np.int8, np.int32, np.int64,
                layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc)


def gemm_ex(dtype, layout, transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc):
    """C = alpha*op(A)*op(B) + beta*C with op(X) = X^T where the flag is set; dtype is "f32", "f16",
    "bf16" or "i8".  Returns the wide result (double, or int64 for int8) as an (M, N) array."""
    code = {"f32": 0, "f16": 1, "i8": 2, "bf16": 3}[dtype]
    in_dtype = {"f32": np.float32, "f16": np.uint16, "bf16": np.uint16, "i8": np.int8}[dtype]
    ar, ac = (K, M) if transa else (M, K)
    br, bc = (N, K) if transb else (K, N)
    _check("A", A, in_dtype, layout, ar, ac, lda)
    _check("B", B, in_dtype, layout, br, bc, ldb)
    _check("C", C, np.int32 if dtype == "i8" else np.float32, layout, M, N, ldc)
    if C is None and beta != 0:
        raise ValueError("beta != 0 needs C")
    ldd = max(1, M if layout == "col" else N)
    D = np.zeros((N, M) if layout == "col" else (M, N), dtype=np.int64 if dtype == "i8" else np.float64)
    rc = _load().ref_gemm_ex(code, _LAYOUT[layout], int(bool(transa)), int(bool(transb)), M, N, K, float(alpha),
                             _ptr(A), lda, _ptr(B), ldb, float(beta), _ptr(C), ldc if C is not None else ldd,
                             _ptr(D), ldd)
    if rc != 0:
        raise RuntimeError("oracle returned %d" % rc)
    return D.T if layout == "col" else D


def gemm_sample(dtype, layout, K, alpha, A, lda, B, ldb, beta, C, ldc, rows, cols):
    """The definition evaluated at positions (rows[s], cols[s]) only; returns double[nsamp]."""
    code = {"f32": 0, "f16": 1, "i8": 2, "bf16": 3}[dtype]
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    out = np.zeros(rows.size, dtype=np.float64)
    if C is None and beta != 0:
        raise ValueError("beta != 0 needs C")
    rc = _load().ref_gemm_sample(code, _LAYOUT[layout], K, float(alpha), _ptr(A), lda, _ptr(B), ldb,
                                 float(beta), _ptr(C), ldc, rows.size, _ptr(rows), _ptr(cols), _ptr(out))
    if rc != 0:
        raise RuntimeError("oracle returned %d" % rc)
    return out


def conv_output_shape(H, W, kh, kw, stride, pad):
    """(Hout, Wout) of a convolution; stride and pad are (vertical, horizontal) pairs."""
    return (H + 2 * pad[0] - kh) // stride[0] + 1, (W + 2 * pad[1] - kw) // stride[1] + 1


def im2row_f32(x, kh, kw, stride, pad):
    """The im2row matrix (batch*Hout*Wout, kh*kw*Cin) of a float32 channels-last tensor x[batch, H, W, Cin]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    batch, H, W, Cin = x.shape
    Hout, Wout = conv_output_shape(H, W, kh, kw, stride, pad)
    out = np.zeros((batch * Hout * Wout, kh * kw * Cin), dtype=np.float32)
    rc = _load().ref_im2row_f32(batch, H, W, Cin, kh, kw, stride[0], stride[1], pad[0], pad[1], _ptr(x), _ptr(out))
    if rc != 0:
        raise RuntimeError("oracle returned %d" % rc)
    return out


def conv2d_nhwc_f32(x, w, stride, pad, alpha=1.0, beta=0.0, y_old=None):
    """alpha * conv(x[batch,H,W,Cin], w[kh,kw,Cin,Cout]) + beta * y_old as float64 [batch,Hout,Wout,Cout]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    batch, H, W, Cin = x.shape
    kh, kw, cin2, Cout = w.shape
    if cin2 != Cin:
        raise ValueError("filter and input disagree on Cin")
    Hout, Wout = conv_output_shape(H, W, kh, kw, stride, pad)
    if y_old is None:
        if beta != 0:
            raise ValueError("beta != 0 needs y_old")
    else:
        y_old = np.ascontiguousarray(y_old, dtype=np.float32)
        if y_old.shape != (batch, Hout, Wout, Cout):
            raise ValueError("y_old has the wrong shape")
    out = np.zeros((batch, Hout, Wout, Cout), dtype=np.float64)
    rc = _load().ref_conv2d_nhwc_f32(batch, H, W, Cin, Cout, kh, kw, stride[0], stride[1], pad[0], pad[1],
                                     alpha, _ptr(x), _ptr(w), beta, _ptr(y_old), _ptr(out))
    if rc != 0:
        raise RuntimeError("oracle returned %d" % rc)
    return out


_CODE = {"f32": 0, "f16": 1, "i8": 2, "bf16": 3}
_IN_DTYPE = {"f32": np.float32, "f16": np.uint16, "bf16": np.uint16, "i8": np.int8}


def im2row(dtype, x, kh, kw, stride, pad):
    """The im2row matrix of a channels-last tensor x[batch, H, W, Cin] of any of the data types ("f32", "f16" and
    "bf16" as uint16 bit patterns, "i8"), in the same type."""
    x = np.ascontiguousarray(x, dtype=_IN_DTYPE[dtype])
    batch, H, W, Cin = x.shape
    Hout, Wout = conv_output_shape(H, W, kh, kw, stride, pad)
    out = np.zeros((batch * Hout * Wout, kh * kw * Cin), dtype=_IN_DTYPE[dtype])
    rc = _load().ref_im2row_ex(_CODE[dtype], batch, H, W, Cin, kh, kw, stride[0], stride[1], pad[0], pad[1], _ptr(x), _ptr(out))
    if rc != 0:
        raise RuntimeError("oracle returned %d" % rc)
    return out


def conv2d_nhwc(dtype, x, w, stride, pad, alpha=1, beta=0, y_old=None):
    """alpha * conv(x[batch,H,W,Cin], w[kh,kw,Cin,Cout]) + beta * y_old for inputs of any data type; y_old is float32
    (int32 for "i8"); returns float64 (int64 for "i8") [batch,Hout,Wout,Cout]."""
    x = np.ascontiguousarray(x, dtype=_IN_DTYPE[dtype])
    w = np.ascontiguousarray(w, dtype=_IN_DTYPE[dtype])
    batch, H, W, Cin = x.shape
    kh, kw, cin2, Cout = w.shape
    if cin2 != Cin:
        raise ValueError("filter and input disagree on Cin")
    Hout, Wout = conv_output_shape(H, W, kh, kw, stride, pad)
    if y_old is None:
        if beta != 0:
            raise ValueError("beta != 0 needs y_old")
    else:
        y_old = np.ascontiguousarray(y_old, dtype=np.int32 if dtype == "i8" else np.float32)
        if y_old.shape != (batch, Hout, Wout, Cout):
            raise ValueError("y_old has the wrong shape")
    out = np.zeros((batch, Hout, Wout, Cout), dtype=np.int64 if dtype == "i8" else np.float64)
    rc = _load().ref_conv2d_nhwc_ex(_CODE[dtype], batch, H, W, Cin, Cout, kh, kw, stride[0], stride[1], pad[0], pad[1],
                                    float(alpha), _ptr(x), _ptr(w), float(beta), _ptr(y_old), _ptr(out))
    if rc != 0:
        raise RuntimeError("oracle returned %d" % rc)
    return out


def narrow_f16(d):
    """float64 array -> IEEE binary16 bit patterns (uint16), one rounding to nearest even."""
    d = np.ascontiguousarray(d, dtype=np.float64)
    out = np.zeros(d.shape, dtype=np.uint16)
    _load().ref_narrow_f16(_ptr(d), _ptr(out), d.size)
    return out


def narrow_bf16(d):
    """float64 array -> bfloat16 bit patterns (uint16), one rounding to nearest even."""
    d = np.ascontiguousarray(d, dtype=np.float64)
    out = np.zeros(d.shape, dtype=np.uint16)
    _load().ref_narrow_bf16(_ptr(d), _ptr(out), d.size)
    return out


def half_bits_to_double(bits):
    """uint16 array of binary16 patterns -> float64 (numpy's float16 is IEEE binary16; pinned against ref_half_to_double)."""
    return np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def bfloat16_bits_to_double(bits):
    """uint16 array of bfloat16 patterns -> float64: the pattern is the upper half of an fp32."""
    with np.errstate(invalid="ignore"):      # signalling NaN patterns
        return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def wrap_int32(d):
    """Reduce exact int64 values modulo 2^32 into int32 (two's complement)."""
    return np.asarray(d, dtype=np.int64).astype(np.uint64).astype(np.uint32).view(np.int32).reshape(np.shape(d))


def normalised_error(c, c_ref, K, max_a, max_b):
    """max |c - c_ref| / (K * max|A| * max|B|), the acceptance metric for floating point."""
    c = np.asarray(c, dtype=np.float64)
    c_ref = np.asarray(c_ref, dtype=np.float64)
    if c.size == 0:
        return 0.0
    denom = float(K) * float(max_a) * float(max_b)
    diff = float(np.max(np.abs(c - c_ref)))
    if not np.all(np.isfinite(c)):
        return float("inf")
    return diff / denom if denom > 0 else (0.0 if diff == 0 else float("inf"))
