"""ctypes binding of libmi_gemm.so: argument marshalling only.

Every function has the name and the argument order of its C entry point
(include/mi_gemm.h).  Matrix arguments are torch tensors on the GPU (any shape;
only data_ptr() is used) or raw integer device addresses; `stream` is a
torch.cuda.Stream, a raw hipStream_t value or None for torch's current stream.
`workspace` is a torch tensor (its byte size is taken from it) or None.
Nothing here computes: if the library is missing, loading raises.
"""
import ctypes
import os

COL_MAJOR, ROW_MAJOR = 0, 1
F32, F16, I8, BF16 = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmi_gemm.so")
_lib = None


class GemmError(RuntimeError):
    def __init__(self, status, text):
        RuntimeError.__init__(self, "mi_gemm status %d: %s" % (status, text))
        self.status = status


def lib_path():
    return _LIB_PATH


def load():
    """Load the built library; build it first if it was never built (needs hipcc)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build(force=True)
    lib = ctypes.CDLL(_LIB_PATH)
    i64, vp, sz, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    for name, scal in (("gemm_f32", ctypes.c_float), ("gemm_f16", ctypes.c_float), ("gemm_bf16", ctypes.c_float),
                       ("gemm_f16_c16", ctypes.c_float), ("gemm_bf16_c16", ctypes.c_float), ("gemm_i8", ctypes.c_int32)):
        fn = getattr(lib, name)
        fn.restype = ci
        fn.argtypes = [ci, i64, i64, i64, scal, vp, i64, vp, i64, scal, vp, i64, vp, sz, vp]
    lib.gemm_workspace_bytes.restype = sz
    lib.gemm_workspace_bytes.argtypes = [ci, i64, i64, i64]
    lib.gemm_status_string.restype = ctypes.c_char_p
    lib.gemm_status_string.argtypes = [ci]
    lib.gemm_kernel_count.restype = ci
    lib.gemm_kernel_count.argtypes = [ci]
    lib.gemm_kernel_name.restype = ctypes.c_char_p
    lib.gemm_kernel_name.argtypes = [ci, ci]
    lib.gemm_force_kernel.restype = ci
    lib.gemm_force_kernel.argtypes = [ci, ci, ci]
    lib.gemm_kernel_tile.restype = ci
    lib.gemm_kernel_tile.argtypes = [ci, ci] + [ctypes.POINTER(ci)] * 4
    lib.gemm_ex.restype = ci
    lib.gemm_ex.argtypes = [ci, ci, ci, ci, i64, i64, i64, vp, vp, i64, vp, i64, vp, vp, i64, vp, sz, vp]
    lib.gemm_ex_static_ws.restype = ci
    lib.gemm_ex_static_ws.argtypes = [ci, ci, ci, ci, i64, i64, i64, vp, vp, i64, vp, i64, vp, vp, i64, vp]
    lib.gemm_ex_status_string.restype = ctypes.c_char_p
    lib.gemm_ex_status_string.argtypes = [ci]
    lib.gemm_predict_us.restype = ctypes.c_double
    lib.gemm_predict_us.argtypes = [ci, ci, i64, i64, i64, ci]
    lib.gemm_select.restype = ci
    lib.gemm_select.argtypes = [ci, ci, i64, i64, i64, sz, ctypes.POINTER(ci), ctypes.POINTER(ci)]
    lib.gemm_solo.restype = ci
    lib.gemm_solo.argtypes = [ci, ci, ci, ci, ci, vp]
    lib.conv2d_im2row_f32.restype = ci
    lib.conv2d_im2row_f32.argtypes = [i64] * 11 + [ctypes.c_float, vp, vp, ctypes.c_float, vp, vp, sz, vp]
    lib.conv2d_im2row_ex.restype = ci
    lib.conv2d_im2row_ex.argtypes = [ci] + [i64] * 11 + [vp, vp, vp, vp, vp, vp, sz, vp]
    lib.conv2d_im2row_ex_workspace_bytes.restype = sz
    lib.conv2d_im2row_ex_workspace_bytes.argtypes = [ci] + [i64] * 11
    lib.conv2d_im2row_ex_status_string.restype = ctypes.c_char_p
    lib.conv2d_im2row_ex_status_string.argtypes = [ci]
    lib.conv2d_im2row_workspace_bytes.restype = sz
    lib.conv2d_im2row_workspace_bytes.argtypes = [i64] * 11
    lib.conv2d_im2row_status_string.restype = ctypes.c_char_p
    lib.conv2d_im2row_status_string.argtypes = [ci]
    lib.conv2d_im2row_shape.restype = ci
    lib.conv2d_im2row_shape.argtypes = [i64] * 11 + [ctypes.POINTER(i64)] * 5
    lib.im2row_f32.restype = ci
    lib.im2row_f32.argtypes = [i64] * 10 + [vp, vp, vp]
    lib.conv2d_im2row_force_path.restype = ci
    lib.conv2d_im2row_force_path.argtypes = [ci]
    lib.conv2d_im2row_last_path.restype = ci
    lib.gemm_last_kernel_id.restype = ci
    lib.gemm_last_split.restype = ci
    _lib = lib
    return lib


def _addr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _ws(workspace):
    if workspace is None:
        return None, 0
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def _call(name, layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace, stream, check):
    lib = load()
    ws, ws_bytes = _ws(workspace)
    status = getattr(lib, name)(layout, M, N, K, alpha, _addr(A), lda, _addr(B), ldb, beta, _addr(C), ldc,
                                ws, ws_bytes, _stream(stream))
    if check and status != 0:
        raise GemmError(status, gemm_status_string(status))
    return status


def gemm_f32(layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace=None, stream=None, check=True):
    return _call("gemm_f32", layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace, stream, check)


def gemm_f16(layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace=None, stream=None, check=True):
    return _call("gemm_f16", layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace, stream, check)


def gemm_bf16(layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace=None, stream=None, check=True):
    return _call("gemm_bf16", layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace, stream, check)


def gemm_i8(layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace=None, stream=None, check=True):
    return _call("gemm_i8", layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace, stream, check)


def gemm_ex(dtype, layout, transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace=None, stream=None,
            check=True):
    """C = alpha*op(A)*op(B) + beta*C for any data type; alpha and beta are Python numbers."""
    lib = load()
    ws, ws_bytes = _ws(workspace)
    scal = ctypes.c_int32 if dtype == I8 else ctypes.c_float
    a, b = scal(alpha), scal(beta)
    status = lib.gemm_ex(dtype, layout, int(transa), int(transb), M, N, K, ctypes.byref(a), _addr(A), lda, _addr(B), ldb,
                         ctypes.byref(b), _addr(C), ldc, ws, ws_bytes, _stream(stream))
    if check and status != 0:
        raise GemmError(status, lib.gemm_ex_status_string(status).decode())
    return status


STATIC_WS_BYTES = 16 << 20
STATUS_STATIC_WS_TOO_SMALL = -100


def gemm_ex_static_ws(dtype, layout, transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream=None, check=True):
    """gemm_ex with the K-split scratch in the library's own fixed array (no workspace, nothing allocated)."""
    lib = load()
    scal = ctypes.c_int32 if dtype == I8 else ctypes.c_float
    a, b = scal(alpha), scal(beta)
    status = lib.gemm_ex_static_ws(dtype, layout, int(transa), int(transb), M, N, K, ctypes.byref(a), _addr(A), lda, _addr(B),
                                   ldb, ctypes.byref(b), _addr(C), ldc, _stream(stream))
    if check and status != 0:
        raise GemmError(status, lib.gemm_ex_status_string(status).decode())
    return status


def gemm_workspace_bytes(dtype, M, N, K):
    return int(load().gemm_workspace_bytes(dtype, M, N, K))


def gemm_status_string(status):
    return load().gemm_status_string(status).decode()


def gemm_kernel_count(dtype):
    return int(load().gemm_kernel_count(dtype))


def gemm_kernel_name(dtype, kernel_id):
    return load().gemm_kernel_name(dtype, kernel_id).decode()


def gemm_force_kernel(dtype, kernel_id=-1, split=0):
    return int(load().gemm_force_kernel(dtype, kernel_id, split))


def gemm_kernel_tile(dtype, kernel_id):
    """(BM, BN, BK, workgroups per CU) of a tile configuration."""
    out = [ctypes.c_int(0) for _ in range(4)]
    status = load().gemm_kernel_tile(dtype, kernel_id, *[ctypes.byref(o) for o in out])
    if status != 0:
        raise GemmError(status, "unknown dtype or kernel id")
    return tuple(o.value for o in out)


def gemm_predict_us(dtype, kernel_id, M, N, K, split=1):
    """Time in microseconds the selector's model predicts for this configuration and split."""
    t = load().gemm_predict_us(dtype, kernel_id, M, N, K, split)
    if t < 0:
        raise GemmError(-1, "gemm_predict_us: bad argument")
    return t


def gemm_select(dtype, layout, M, N, K, workspace_bytes):
    """(kernel id, split) a call with these arguments would launch; nothing runs."""
    kid, split = ctypes.c_int(-1), ctypes.c_int(0)
    status = load().gemm_select(dtype, layout, M, N, K, workspace_bytes, ctypes.byref(kid), ctypes.byref(split))
    if status != 0:
        raise GemmError(status, "gemm_select: bad argument")
    return kid.value, split.value


def gemm_solo(dtype, kernel_id, workgroups, ksteps, fill=1, stream=None, check=True):
    status = load().gemm_solo(dtype, kernel_id, workgroups, ksteps, fill, _stream(stream))
    if check and status != 0:
        raise GemmError(status, "gemm_solo: bad argument" if status < 0 else gemm_status_string(status))
    return status


def gemm_last_kernel_id():
    return int(load().gemm_last_kernel_id())


def gemm_last_split():
    return int(load().gemm_last_split())


def gemm_f16_c16(layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace=None, stream=None, check=True):
    return _call("gemm_f16_c16", layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace, stream, check)


def gemm_bf16_c16(layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace=None, stream=None, check=True):
    return _call("gemm_bf16_c16", layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace, stream, check)


def conv2d_im2row_f32(batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w, alpha, image, filter, beta, output,
                      workspace=None, stream=None, check=True):
    ws, ws_bytes = _ws(workspace)
    status = load().conv2d_im2row_f32(batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w, alpha, _addr(image),
                                      _addr(filter), beta, _addr(output), ws, ws_bytes, _stream(stream))
    if check and status != 0:
        raise GemmError(status, conv2d_im2row_status_string(status))
    return status


def conv2d_im2row_ex(dtype, batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w, alpha, image, filter, beta, output,
                     workspace=None, stream=None, check=True):
    """The convolution for any data type; alpha and beta are Python numbers."""
    lib = load()
    ws, ws_bytes = _ws(workspace)
    scal = ctypes.c_int32 if dtype == I8 else ctypes.c_float
    a, b = scal(alpha), scal(beta)
    status = lib.conv2d_im2row_ex(dtype, batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w, ctypes.byref(a),
                                  _addr(image), _addr(filter), ctypes.byref(b), _addr(output), ws, ws_bytes, _stream(stream))
    if check and status != 0:
        raise GemmError(status, lib.conv2d_im2row_ex_status_string(status).decode())
    return status


def conv2d_im2row_ex_workspace_bytes(dtype, batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w):
    return int(load().conv2d_im2row_ex_workspace_bytes(dtype, batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w))


def conv2d_im2row_workspace_bytes(batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w):
    return int(load().conv2d_im2row_workspace_bytes(batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w))


def conv2d_im2row_status_string(status):
    return load().conv2d_im2row_status_string(status).decode()


def conv2d_im2row_shape(batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w):
    """(Hout, Wout, M, N, K) of the convolution and of its GEMM."""
    out = [ctypes.c_int64(0) for _ in range(5)]
    status = load().conv2d_im2row_shape(batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w,
                                        *[ctypes.byref(o) for o in out])
    if status != 0:
        raise GemmError(status, conv2d_im2row_status_string(status))
    return tuple(int(o.value) for o in out)


def im2row_f32(batch, H, W, Cin, kh, kw, stride_h, stride_w, pad_h, pad_w, image, matrix, stream=None, check=True):
    status = load().im2row_f32(batch, H, W, Cin, kh, kw, stride_h, stride_w, pad_h, pad_w, _addr(image), _addr(matrix),
                               _stream(stream))
    if check and status != 0:
        raise GemmError(status, "im2row_f32: argument %d is illegal" % -status if status < 0 else "HIP error")
    return status


def conv2d_im2row_force_path(path):
    if load().conv2d_im2row_force_path(path) != 0:
        raise GemmError(-1, "conv2d_im2row_force_path: path must be 0, 1 or 2")


def conv2d_im2row_last_path():
    return int(load().conv2d_im2row_last_path())
