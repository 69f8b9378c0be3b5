"""The entry points are captured into a HIP graph (through torch's capture stream) and replayed: every replay
must reproduce the eager result bit for bit, with eager launches and synchronisations between the replays.
Covers a K split with its reduce kernel, a register-direct kernel, the 16-bit-C update and a convolution."""
import numpy as np
import pytest
import torch

import workloads as wl
import paper_2310_17408_amd as mg

pytestmark = pytest.mark.gpu


def _dev(x):
    t = torch.from_numpy(np.ascontiguousarray(x).reshape(-1))
    return (t.view(torch.int16) if t.dtype == torch.uint16 else t).cuda()


def _replays_match(make_call, out, fresh):
    """make_call(stream) launches the work; `fresh()` restores the output buffer's initial contents."""
    fresh()
    make_call(None)
    torch.cuda.synchronize()
    want = out.clone()
    fresh()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        make_call(None)
    for _ in range(3):
        fresh()
        make_call(None)                     # eager work of the same kind between the replays
        torch.cuda.synchronize()
        fresh()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want)


def test_gemm_with_k_split_in_a_graph():
    M, N, K = 96, 80, 4096
    A, B, C = wl.uniform_f32(1, "col", M, K), wl.uniform_f32(2, "col", K, N), wl.uniform_f32(3, "col", M, N)
    dA, dB, dC0 = _dev(A), _dev(B), _dev(C)
    dC = dC0.clone()
    ws = torch.empty(8 * M * N * 4, dtype=torch.uint8, device="cuda")
    mg.gemm_force_kernel(mg.F32, 4, 4)       # a direct-to-LDS configuration, K split over 4 workgroups + reduce kernel
    try:
        _replays_match(lambda s: mg.gemm_f32(mg.COL_MAJOR, M, N, K, 1.5, dA, M, dB, K, 0.5, dC, M, ws, s), dC,
                       lambda: dC.copy_(dC0))
        assert mg.gemm_last_split() == 4
    finally:
        mg.gemm_force_kernel(mg.F32, -1, 0)


def test_int8_register_direct_and_16_bit_c_in_a_graph():
    M, N, K = 200, 136, 700
    A, B = wl.uniform_i8(4, "row", M, K), wl.uniform_i8(5, "row", K, N)
    dA, dB = _dev(A), _dev(B)
    dC = torch.zeros(M * N, dtype=torch.int32, device="cuda")
    _replays_match(lambda s: mg.gemm_i8(mg.ROW_MAJOR, M, N, K, 1, dA, K, dB, N, 0, dC, N, None, s), dC, lambda: dC.zero_())
    assert "_reg" in mg.gemm_kernel_name(mg.I8, mg.gemm_last_kernel_id())
    Ah, Bh = wl.normal_f16_bits(6, "row", M, K), wl.normal_f16_bits(7, "row", K, N)
    C0 = _dev(wl.normal_f16_bits(8, "row", M, N))
    dAh, dBh, dCh = _dev(Ah), _dev(Bh), C0.clone()
    _replays_match(lambda s: mg.gemm_f16_c16(mg.ROW_MAJOR, M, N, K, 1.0, dAh, K, dBh, N, 0.5, dCh, N, None, s), dCh,
                   lambda: dCh.copy_(C0))


def test_convolution_in_a_graph():
    for geom in ((2, 12, 10, 32, 70, 3, 3, 1, 1, 1, 1), (1, 16, 16, 3, 24, 7, 7, 2, 2, 3, 3)):
        Hout, Wout, M, N, K = mg.conv2d_im2row_shape(*geom)
        image, filt, old = wl.conv_tensors_f32(9, geom[0], geom[1], geom[2], geom[3], geom[4], geom[5], geom[6], Hout, Wout)
        d_image, d_filt, d_old = _dev(image), _dev(filt), _dev(old)
        d_out = d_old.clone()
        ws = torch.empty(mg.conv2d_im2row_workspace_bytes(*geom) + 16, dtype=torch.uint8, device="cuda")
        for path in (1, 2):
            mg.conv2d_im2row_force_path(path)
            try:
                _replays_match(lambda s: mg.conv2d_im2row_f32(*geom, 1.0, d_image, d_filt, 0.5, d_out, ws, s), d_out,
                               lambda: d_out.copy_(d_old))
                assert mg.conv2d_im2row_last_path() == path
            finally:
                mg.conv2d_im2row_force_path(0)
