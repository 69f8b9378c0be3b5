"""Parity of conv2d_im2row_ex (the convolution for binary16, bfloat16 and int8 inputs; fp32 goes the way of
conv2d_im2row_f32) with the CPU oracle's convolution of the same type, element by element through the C-ABI:
the in-place path on every register-direct configuration of each type, the path through the im2row matrix,
the automatic choice on the layers behind the paper's headline GEMM sizes, alpha/beta, K split, error codes.
Bars as for the GEMMs: int8 bit-exact; 16-bit inputs 2e-3 officially and 1e-5 internally (fp32 accumulation of
exact products)."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2310_17408_amd as mg
from gpu_case import DT, TIGHT, TOL

pytestmark = pytest.mark.gpu

GEN = {"f32": wl.uniform_f32, "f16": wl.normal_f16_bits, "bf16": wl.normal_bf16_bits, "i8": wl.uniform_i8}
DECODE = {"f32": lambda b: b.astype(np.float64), "f16": oracle.half_bits_to_double, "bf16": oracle.bfloat16_bits_to_double}


def _dev(x):
    t = torch.from_numpy(np.ascontiguousarray(x).reshape(-1))
    if t.dtype == torch.uint16:
        t = t.view(torch.int16)
    return t.cuda()


def run_conv(dtype, geom, seed, alpha=1, beta=0, path=0, kernel_id=-1, split=0, workspace="full", expect_path=None):
    batch, H, W, Cin, Cout, kh, kw, sh, sw, ph, pw = geom
    Hout, Wout, M, N, K = mg.conv2d_im2row_shape(*geom)
    image = GEN[dtype](seed, "row", batch * H * W, Cin).reshape(batch, H, W, Cin)
    filt = GEN[dtype](seed + 1, "row", kh * kw * Cin, Cout).reshape(kh, kw, Cin, Cout)
    if dtype == "i8":
        old = wl.uniform_i32(seed + 2, "row", M, N).reshape(batch, Hout, Wout, Cout)
        poison = np.full_like(old, 2 ** 31 - 1)
    else:
        old = wl.uniform_f32(seed + 2, "row", M, N).reshape(batch, Hout, Wout, Cout)
        poison = np.full_like(old, np.nan)
    ref = oracle.conv2d_nhwc(dtype, image, filt, (sh, sw), (ph, pw), alpha, beta, old if beta != 0 else None)
    d_image, d_filt = _dev(image), _dev(filt)
    d_out = _dev(old if beta != 0 else poison)
    ws = None
    if workspace == "full":
        ws = torch.empty(mg.conv2d_im2row_ex_workspace_bytes(DT[dtype], *geom) + 32 * M * N * 4 + 16, dtype=torch.uint8, device="cuda")
    elif workspace == "split":
        ws = torch.empty(32 * M * N * 4 + 16, dtype=torch.uint8, device="cuda")
    mg.conv2d_im2row_force_path(path)
    mg.gemm_force_kernel(DT[dtype], kernel_id, split)
    try:
        mg.conv2d_im2row_ex(DT[dtype], batch, H, W, Cin, Cout, kh, kw, sh, sw, ph, pw, alpha, d_image, d_filt, beta, d_out, ws)
        torch.cuda.synchronize()
        took, kid, sp = mg.conv2d_im2row_last_path(), mg.gemm_last_kernel_id(), mg.gemm_last_split()
    finally:
        mg.conv2d_im2row_force_path(0)
        mg.gemm_force_kernel(DT[dtype], -1, 0)
    got = d_out.cpu().numpy().reshape(M, N)
    what = (dtype, geom, took, mg.gemm_kernel_name(DT[dtype], kid) if kid >= 0 else kid, sp)
    if dtype == "i8":
        assert np.array_equal(got, oracle.wrap_int32(ref).reshape(M, N)), what
    else:
        assert np.isfinite(got).all(), what
        err = oracle.normalised_error(got.astype(np.float64), ref.reshape(M, N), K, float(np.abs(DECODE[dtype](image)).max()),
                                      float(np.abs(DECODE[dtype](filt)).max()))
        assert err <= TOL[dtype] and err <= TIGHT[dtype], what + (err,)
    if expect_path is not None:
        assert took == expect_path, what
    return took, kid, sp


def _fused_kernels(dtype):
    return [i for i in range(mg.gemm_kernel_count(DT[dtype])) if mg.gemm_kernel_name(DT[dtype], i).endswith("_reg")]


# Cin a multiple of 64, so that a K step of every type's register-direct kernels (32 elements of 16 bits, 64 of
# 8 bits) lies inside one filter tap
GEOMS = [
    (2, 9, 8, 64, 24, 3, 3, 1, 1, 1, 1),       # padding on every side, ragged pixel and channel counts
    (1, 14, 14, 64, 40, 3, 3, 2, 2, 1, 1),     # stride 2
    (3, 6, 7, 128, 16, 1, 1, 1, 1, 0, 0),      # 1 x 1 filter: a plain GEMM
    (1, 12, 10, 64, 33, 5, 5, 2, 2, 2, 2),     # larger filter, taps outside the image on all sides, odd Cout
    (1, 11, 13, 64, 70, 5, 2, 2, 3, 2, 1),     # anisotropic filter, stride and padding
]


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_in_place_path_on_every_register_direct_kernel(dtype):
    kernels = _fused_kernels(dtype)
    assert len(kernels) >= 3
    a, b = (2, -1) if dtype == "i8" else (1.5, 0.5)
    for kid in kernels:
        for i, geom in enumerate(GEOMS):
            took, got, _ = run_conv(dtype, geom, 7000 + 10 * kid + i, a, b, path=1, kernel_id=kid, expect_path=1)
            assert got == kid
        # K split over workgroups, beta == 0 on an output full of NaN (int8: of the largest int)
        _, got, sp = run_conv(dtype, GEOMS[3], 7200 + kid, 1, 0, path=1, kernel_id=kid, split=3, workspace="split", expect_path=1)
        assert got == kid and (sp == 3 or "_k" in mg.gemm_kernel_name(DT[dtype], kid))
    # no workspace at all: in place, no split over workgroups
    _, _, sp = run_conv(dtype, GEOMS[0], 7300, workspace=None, expect_path=1)
    assert sp == 1


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_path_through_the_matrix(dtype):
    a, b = (3, 1) if dtype == "i8" else (-1.0, 2.0)
    for i, geom in enumerate(GEOMS):
        run_conv(dtype, geom, 7400 + i, a, b, path=2, expect_path=2)
    # geometries the in-place kernels do not take go there by themselves: Cin that is no multiple of the K step,
    # fewer output channels than a word of the filter holds
    run_conv(dtype, (1, 10, 9, 24, 20, 3, 3, 1, 1, 1, 1), 7450, a, b, expect_path=2)
    run_conv(dtype, (2, 8, 8, 3, 16, 3, 3, 2, 2, 1, 1), 7460, a, b, expect_path=2)
    run_conv(dtype, (1, 8, 8, 64, 1, 3, 3, 1, 1, 1, 1), 7470, a, b, expect_path=2)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_layers_behind_the_headline_shapes(dtype):
    """The ResNet50 v1.5 layers of the paper's headline GEMM sizes, automatic choice of path and kernel; those
    with Cin a multiple of 64 must run in place."""
    for i, (H, W, Cin, Cout, kh, kw, stride, pad) in enumerate(wl.RESNET50_HEADLINE_CONVS):
        geom = (1, H, W, Cin, Cout, kh, kw, stride, stride, pad, pad)
        took, _, _ = run_conv(dtype, geom, 7500 + i)
        if Cin % 64 == 0:
            assert took == 1
    run_conv(dtype, (4, 28, 28, 128, 128, 3, 3, 2, 2, 1, 1), 7590)       # a batch of 4


def test_fp32_through_the_general_entry_point_is_the_fp32_entry_point():
    geom = (1, 14, 14, 32, 40, 3, 3, 2, 2, 1, 1)
    Hout, Wout, M, N, K = mg.conv2d_im2row_shape(*geom)
    image, filt, _ = wl.conv_tensors_f32(7600, 1, 14, 14, 32, 40, 3, 3, Hout, Wout)
    a, b = torch.zeros(M * N, device="cuda"), torch.zeros(M * N, device="cuda")
    mg.conv2d_im2row_f32(*geom, 1.5, _dev(image), _dev(filt), 0.0, a)
    k1 = (mg.conv2d_im2row_last_path(), mg.gemm_last_kernel_id())
    mg.conv2d_im2row_ex(mg.F32, *geom, 1.5, _dev(image), _dev(filt), 0.0, b)
    assert k1 == (mg.conv2d_im2row_last_path(), mg.gemm_last_kernel_id())
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_errors_and_quick_returns():
    geom = (1, 8, 8, 64, 16, 3, 3, 1, 1, 1, 1)
    Hout, Wout, M, N, K = mg.conv2d_im2row_shape(*geom)
    image, filt = _dev(wl.normal_f16_bits(1, "row", 64, 64)), _dev(wl.normal_f16_bits(2, "row", K, N))
    out = torch.full((M * N,), 3.0, device="cuda")
    assert mg.conv2d_im2row_ex(9, *geom, 1.0, image, filt, 0.0, out, check=False) == -1
    assert mg.conv2d_im2row_ex(mg.F16, 1, 8, 8, 64, 16, 3, 3, 0, 1, 1, 1, 1.0, image, filt, 0.0, out, check=False) == -9
    assert mg.conv2d_im2row_ex(mg.F16, *geom, 1.0, None, filt, 0.0, out, check=False) == -14
    assert mg.conv2d_im2row_ex(mg.F16, *geom, 1.0, image, filt, 0.0, None, check=False) == -17
    # a geometry that needs the matrix with no workspace for it
    assert mg.conv2d_im2row_ex(mg.F16, 1, 8, 8, 24, 16, 3, 3, 1, 1, 1, 1, 1.0, image, filt, 0.0, out, check=False) == -19
    with pytest.raises(mg.GemmError):
        mg.conv2d_im2row_ex(mg.F16, 1, 8, 8, 24, 16, 3, 3, 1, 1, 1, 1, 1.0, image, filt, 0.0, out)
    torch.cuda.synchronize()
    assert torch.all(out == 3.0)
    # alpha == 0: output <- beta * output, neither operand is read
    assert mg.conv2d_im2row_ex(mg.F16, *geom, 0.0, None, None, 2.0, out) == 0
    torch.cuda.synchronize()
    assert torch.all(out == 6.0)
    one, zero = ctypes.c_float(1.0), ctypes.c_float(0.0)
    assert mg.load().conv2d_im2row_ex(mg.F16, *geom, None, image.data_ptr(), filt.data_ptr(), ctypes.byref(zero), out.data_ptr(),
                                      None, 0, None) == -13
