"""Parity of the convolution entry points (conv2d_im2row_f32, im2row_f32) with the CPU oracle, element by
element through the C-ABI: the in-place (fused im2row) path on every register-direct fp32 configuration,
the path through the im2row matrix, the automatic choice on the layer geometries behind the paper's six
headline GEMM sizes, alpha/beta, K split, and the error codes."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2310_17408_amd as mg

pytestmark = pytest.mark.gpu
TOL = 1e-6      # max|C - C_ref| / (K max|A| max|B|), the fp32 bar of the GEMM tests


def run_conv(geom, seed, alpha=1.0, beta=0.0, path=0, kernel_id=-1, split=0, workspace="full", expect_path=None):
    batch, H, W, Cin, Cout, kh, kw, sh, sw, ph, pw = geom
    Hout, Wout, M, N, K = mg.conv2d_im2row_shape(*geom)
    image, filt, old = wl.conv_tensors_f32(seed, batch, H, W, Cin, Cout, kh, kw, Hout, Wout)
    ref = oracle.conv2d_nhwc_f32(image, filt, (sh, sw), (ph, pw), alpha, beta, old if beta != 0 else None)
    d_image, d_filt = torch.from_numpy(image).cuda(), torch.from_numpy(filt).cuda()
    d_out = torch.from_numpy(old).cuda() if beta != 0 else torch.full((batch, Hout, Wout, Cout), float("nan"), device="cuda")
    ws = None
    if workspace == "full":
        ws = torch.empty(mg.conv2d_im2row_workspace_bytes(*geom) + 32 * M * N * 4 + 16, dtype=torch.uint8, device="cuda")
    elif workspace == "split":
        ws = torch.empty(32 * M * N * 4 + 16, dtype=torch.uint8, device="cuda")
    mg.conv2d_im2row_force_path(path)
    mg.gemm_force_kernel(mg.F32, kernel_id, split)
    try:
        mg.conv2d_im2row_f32(batch, H, W, Cin, Cout, kh, kw, sh, sw, ph, pw, alpha, d_image, d_filt, beta, d_out, ws)
        torch.cuda.synchronize()
        took, kid, sp = mg.conv2d_im2row_last_path(), mg.gemm_last_kernel_id(), mg.gemm_last_split()
    finally:
        mg.conv2d_im2row_force_path(0)
        mg.gemm_force_kernel(mg.F32, -1, 0)
    got = d_out.cpu().numpy().astype(np.float64)
    err = oracle.normalised_error(got.reshape(M, N), ref.reshape(M, N), K, float(np.abs(image).max()), float(np.abs(filt).max()))
    assert np.isfinite(got).all()
    assert err <= TOL, (geom, took, kid, sp, err)
    if expect_path is not None:
        assert took == expect_path
    return took, kid, sp


def _fused_kernels():
    return [i for i in range(mg.gemm_kernel_count(mg.F32)) if mg.gemm_kernel_name(mg.F32, i).endswith(("_reg", "_reg16"))]


GEOMS = [
    (2, 9, 8, 16, 24, 3, 3, 1, 1, 1, 1),       # padding on every side, ragged pixel and channel counts
    (1, 14, 14, 32, 40, 3, 3, 2, 2, 1, 1),     # stride 2
    (3, 6, 7, 48, 16, 1, 1, 1, 1, 0, 0),       # 1 x 1 filter: a plain GEMM
    (1, 20, 18, 16, 33, 7, 7, 2, 2, 3, 3),     # large filter, taps outside the image on all sides
    (1, 11, 13, 16, 70, 5, 2, 2, 3, 2, 1),     # anisotropic filter, stride and padding
]


def test_fused_path_on_every_register_direct_kernel():
    kernels = _fused_kernels()
    assert len(kernels) >= 4
    for kid in kernels:
        for i, geom in enumerate(GEOMS):
            took, got, _ = run_conv(geom, 7000 + 10 * kid + i, 1.5, 0.5, path=1, kernel_id=kid, expect_path=1)
            assert got == kid


DMA_GEOMS = [
    (2, 12, 10, 32, 70, 3, 3, 1, 1, 1, 1),     # padding on every side; 240 pixels and 70 channels: ragged tiles
    (1, 20, 18, 64, 130, 5, 5, 2, 2, 2, 2),    # stride 2, two K steps per tap
    (1, 9, 9, 32, 64, 1, 1, 1, 1, 0, 0),       # 1 x 1 filter
    (3, 7, 5, 96, 40, 3, 2, 1, 2, 1, 0),       # fewer pixels (fewer than a 64-row tile in one case) than tile rows
]


def test_fused_path_on_the_direct_to_lds_kernels():
    """Cin a multiple of 32: the direct-to-LDS fp32 kernels stage the image in place (taps outside the image
    are read from the nearest pixel inside and zeroed in LDS)."""
    kernels = [i for i in range(mg.gemm_kernel_count(mg.F32)) if "_dma" in mg.gemm_kernel_name(mg.F32, i)]
    assert len(kernels) >= 3
    for kid in kernels:
        for i, geom in enumerate(DMA_GEOMS):
            took, got, _ = run_conv(geom, 7800 + 10 * kid + i, 1.5, 0.5, path=1, kernel_id=kid, expect_path=1)
            assert got == kid
        _, _, sp = run_conv(DMA_GEOMS[1], 7900 + kid, 1.0, 0.0, path=1, kernel_id=kid, split=3, workspace="split", expect_path=1)
        assert sp == 3
    # an image that is only 4-byte aligned goes to the register-direct kernels
    geom = DMA_GEOMS[0]
    Hout, Wout, M, N, K = mg.conv2d_im2row_shape(*geom)
    image, filt, _ = wl.conv_tensors_f32(7950, geom[0], geom[1], geom[2], geom[3], geom[4], geom[5], geom[6], Hout, Wout)
    buf = torch.zeros(image.size + 8, device="cuda")
    d_image = buf[1:1 + image.size]
    d_image.copy_(torch.from_numpy(image.reshape(-1)))
    d_out = torch.zeros(M * N, device="cuda")
    mg.conv2d_im2row_f32(*geom, 1.0, d_image, torch.from_numpy(filt).cuda(), 0.0, d_out)
    torch.cuda.synchronize()
    assert mg.conv2d_im2row_last_path() == 1 and "_reg" in mg.gemm_kernel_name(mg.F32, mg.gemm_last_kernel_id())
    ref = oracle.conv2d_nhwc_f32(image, filt, (geom[7], geom[8]), (geom[9], geom[10]))
    assert oracle.normalised_error(d_out.cpu().numpy().reshape(M, N).astype(np.float64), ref.reshape(M, N), K, 1.0, 1.0) <= TOL


def test_fused_path_with_k_split_and_without_workspace():
    for kid in _fused_kernels():
        _, _, sp = run_conv(GEOMS[3], 7200 + kid, 1.0, -0.5, path=1, kernel_id=kid, split=3, workspace="split", expect_path=1)
        assert sp == 3 or "_k" in mg.gemm_kernel_name(mg.F32, kid)
    # no workspace at all: the in-place path without a split over workgroups
    _, _, sp = run_conv(GEOMS[0], 7300, workspace=None, expect_path=1)
    assert sp == 1


RUN_GEOMS = [
    (2, 32, 30, 3, 20, 7, 7, 2, 2, 3, 3),      # Cin = 3: the first layer of both networks
    (1, 17, 19, 5, 9, 3, 3, 1, 1, 1, 1),       # K = 45: less than three K steps
    (1, 9, 9, 1, 17, 3, 3, 1, 1, 1, 1),        # one channel: runs shorter than a lane's share of a step
    (1, 10, 12, 20, 33, 3, 2, 2, 1, 0, 1),     # Cin a multiple of 4 but not of 16
]


def test_fused_path_for_any_channel_count_on_every_register_direct_kernel():
    """Cin that is no multiple of the K step: the run-wise reader (elements one by one, partial last step)."""
    for kid in _fused_kernels():
        for i, geom in enumerate(RUN_GEOMS):
            took, got, _ = run_conv(geom, 7350 + 10 * kid + i, 1.5, 0.5, path=1, kernel_id=kid, expect_path=1)
            assert got == kid
        run_conv(RUN_GEOMS[0], 7390 + kid, 1.0, 0.0, path=1, kernel_id=kid, split=2, workspace="split", expect_path=1)


def test_path_through_the_im2row_matrix():
    run_conv(RUN_GEOMS[0], 7400, 1.0, 0.0, path=2, expect_path=2)
    run_conv(RUN_GEOMS[1], 7401, 2.0, 1.0, path=2, expect_path=2)
    run_conv(GEOMS[1], 7402, 1.5, 0.5, path=2, expect_path=2)


def test_alpha_zero_and_beta_cases():
    geom = GEOMS[0]
    Hout, Wout, M, N, K = mg.conv2d_im2row_shape(*geom)
    out = torch.ones((geom[0], Hout, Wout, geom[4]), device="cuda")
    mg.conv2d_im2row_f32(*geom, 0.0, None, None, 3.0, out)
    torch.cuda.synchronize()
    assert torch.all(out == 3.0)
    run_conv(geom, 7500, 1.0, 1.0, path=1)
    run_conv(geom, 7501, -2.0, 0.0, path=1)


@pytest.mark.parametrize("i", range(len(wl.RESNET50_HEADLINE_CONVS)))
def test_resnet50_headline_layers_at_full_size(i):
    """The layers behind the paper's six headline GEMM sizes, batch 1, automatic path and kernel."""
    H, W, Cin, Cout, kh, kw, stride, pad = wl.RESNET50_HEADLINE_CONVS[i]
    geom = (1, H, W, Cin, Cout, kh, kw, stride, stride, pad, pad)
    assert mg.conv2d_im2row_shape(*geom)[2:] == wl.IM2ROW_HEADLINE[i]
    took, _, _ = run_conv(geom, 7600 + i)
    assert took == 1


def test_im2row_matrix_is_bit_exact():
    for (batch, H, W, Cin, kh, kw, sh, sw, ph, pw) in ((2, 9, 8, 5, 3, 3, 1, 1, 1, 1), (1, 16, 12, 3, 7, 7, 2, 2, 3, 3),
                                                       (1, 7, 7, 16, 1, 1, 1, 1, 0, 0), (3, 5, 6, 4, 2, 3, 2, 1, 0, 2)):
        Hout, Wout, M, _, K = mg.conv2d_im2row_shape(batch, H, W, Cin, 1, kh, kw, sh, sw, ph, pw)
        image = wl.uniform_f32(7700, "row", batch * H * W, Cin).reshape(batch, H, W, Cin)
        want = oracle.im2row_f32(image, kh, kw, (sh, sw), (ph, pw))
        d = torch.full((M, K), float("nan"), device="cuda")
        mg.im2row_f32(batch, H, W, Cin, kh, kw, sh, sw, ph, pw, torch.from_numpy(image).cuda(), d)
        torch.cuda.synchronize()
        assert np.array_equal(d.cpu().numpy(), want)


def test_workspace_too_small_for_the_matrix_is_an_error():
    geom = (1, 16, 16, 3, 8, 3, 3, 1, 1, 1, 1)
    Hout, Wout, M, N, K = mg.conv2d_im2row_shape(*geom)
    image = torch.zeros((1, 16, 16, 3), device="cuda")
    filt = torch.zeros((3, 3, 3, 8), device="cuda")
    out = torch.full((1, Hout, Wout, 8), 5.0, device="cuda")
    mg.conv2d_im2row_force_path(2)
    try:
        assert mg.conv2d_im2row_f32(*geom, 1.0, image, filt, 0.0, out, None, check=False) == -18
        small = torch.empty(M * K * 4 - 16, dtype=torch.uint8, device="cuda")
        assert mg.conv2d_im2row_f32(*geom, 1.0, image, filt, 0.0, out, small, check=False) == -18
    finally:
        mg.conv2d_im2row_force_path(0)
    torch.cuda.synchronize()
    assert torch.all(out == 5.0)      # nothing was launched
