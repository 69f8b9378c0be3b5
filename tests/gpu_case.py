"""Shared driver for the GPU parity tests: build seeded inputs, run the HIP
library through its C-ABI binding, run the CPU oracle on the same bits, and
hand both results back.  Holds no arithmetic of the method."""
import numpy as np
import torch

import oracle
import workloads as wl
import paper_2310_17408_amd as mg

DT = {"f32": mg.F32, "f16": mg.F16, "i8": mg.I8, "bf16": mg.BF16}
LAYOUT = {"col": mg.COL_MAJOR, "row": mg.ROW_MAJOR}
# max|C - C_ref| / (K max|A| max|B|); bfloat16 inputs take the bar of the other 16-bit format: their
# products are exact in fp32 as well, so the error is that of the fp32 accumulation alone
TOL = {"f32": 1e-6, "f16": 2e-3, "bf16": 2e-3}
# What the arithmetic itself allows for the 16-bit inputs: their products are exact in fp32, so only the fp32
# accumulation and the epilogue round (as for fp32 inputs, whose bar is 1e-6 on values of magnitude 1; the
# 16-bit normal inputs reach magnitudes of 4 to 6, which enters the denominator squared).  The official
# bar of 2e-3 would let a dropped K step of 64 in 384 pass (8e-4); this one does not.
TIGHT = {"f32": 1e-6, "f16": 1e-5, "bf16": 1e-5}


def make_inputs(dtype, layout, M, N, K, seed, pad=(0, 0, 0), values="random"):
    lda = wl.tight_ld(layout, M, K) + pad[0]
    ldb = wl.tight_ld(layout, K, N) + pad[1]
    ldc = wl.tight_ld(layout, M, N) + pad[2]
    if dtype == "f32":
        gen = wl.small_int_f32 if values == "smallint" else wl.uniform_f32
        A, B = gen(seed, layout, M, K, lda), gen(seed + 1, layout, K, N, ldb)
        C = gen(seed + 2, layout, M, N, ldc)
    elif dtype == "f16":
        gen = wl.small_int_f16_bits if values == "smallint" else wl.normal_f16_bits
        A, B = gen(seed, layout, M, K, lda), gen(seed + 1, layout, K, N, ldb)
        C = (wl.small_int_f32 if values == "smallint" else wl.uniform_f32)(seed + 2, layout, M, N, ldc)
    elif dtype == "bf16":
        gen = wl.small_int_bf16_bits if values == "smallint" else wl.normal_bf16_bits
        A, B = gen(seed, layout, M, K, lda), gen(seed + 1, layout, K, N, ldb)
        C = (wl.small_int_f32 if values == "smallint" else wl.uniform_f32)(seed + 2, layout, M, N, ldc)
    else:
        A, B = wl.uniform_i8(seed, layout, M, K, lda), wl.uniform_i8(seed + 1, layout, K, N, ldb)
        C = wl.uniform_i32(seed + 2, layout, M, N, ldc)
    return A, lda, B, ldb, C, ldc


def to_device(host, offset_elems=0):
    """Copy a host buffer to the GPU, optionally shifted by some elements to break 16-byte alignment."""
    flat = torch.from_numpy(np.ascontiguousarray(host).reshape(-1))
    if flat.dtype == torch.uint16:
        flat = flat.view(torch.int16)
    buf = torch.empty(flat.numel() + offset_elems + 16, dtype=flat.dtype, device="cuda")
    view = buf[offset_elems:offset_elems + flat.numel()]
    view.copy_(flat)
    return buf, view


def max_abs(dtype, layout, buf, rows, cols):
    if dtype == "f16":
        buf = buf.view(np.float16)
    elif dtype == "bf16":
        buf = wl.bf16_bits_to_f32(buf)
    x = wl.logical(layout, buf, rows, cols)
    return float(np.max(np.abs(x.astype(np.float64)))) if x.size else 0.0


def gpu_gemm(dtype, layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, kernel_id=-1, split=0,
             workspace_bytes=None, offsets=(0, 0, 0)):
    """Run the library on host arrays; returns (C buffer after the call as numpy, kernel id, split)."""
    fn = {"f32": mg.gemm_f32, "f16": mg.gemm_f16, "i8": mg.gemm_i8, "bf16": mg.gemm_bf16}[dtype]
    _, dA = to_device(A, offsets[0])
    _, dB = to_device(B, offsets[1])
    _, dC = to_device(C, offsets[2])
    if workspace_bytes is None:
        workspace_bytes = mg.gemm_workspace_bytes(DT[dtype], M, N, K)
        if split > 1:
            workspace_bytes = max(workspace_bytes, split * M * N * 4)
    ws = torch.empty(max(workspace_bytes, 16), dtype=torch.uint8, device="cuda") if workspace_bytes > 0 else None
    mg.gemm_force_kernel(DT[dtype], kernel_id, split)
    try:
        fn(LAYOUT[layout], M, N, K, alpha, dA, lda, dB, ldb, beta, dC, ldc, ws)
        kid, ks = mg.gemm_last_kernel_id(), mg.gemm_last_split()
    finally:
        mg.gemm_force_kernel(DT[dtype], -1, 0)
    torch.cuda.synchronize()
    out = dC.cpu().numpy().reshape(np.shape(C))
    return out, kid, ks


def oracle_gemm(dtype, layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc):
    fn = {"f32": oracle.gemm_f32, "f16": oracle.gemm_f16, "i8": oracle.gemm_i8, "bf16": oracle.gemm_bf16}[dtype]
    return fn(layout, M, N, K, alpha, A, lda, B, ldb, beta, C if beta != 0 else None, ldc)


def check_case(dtype, layout, M, N, K, alpha=1, beta=0, seed=1, pad=(0, 0, 0), kernel_id=-1, split=0,
               values="random", offsets=(0, 0, 0), workspace_bytes=None, exact=False):
    """One parity case: every element against the oracle, and the padding of C untouched."""
    A, lda, B, ldb, C, ldc = make_inputs(dtype, layout, M, N, K, seed, pad, values)
    if dtype != "i8":
        alpha, beta = np.float32(alpha), np.float32(beta)
    out, kid, ks = gpu_gemm(dtype, layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, kernel_id, split,
                            workspace_bytes, offsets)
    ref = oracle_gemm(dtype, layout, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc)
    got = wl.logical(layout, out, M, N)
    if dtype == "i8":
        assert np.array_equal(got, oracle.wrap_int32(ref)), "int8 result is not bit-exact (kernel %d split %d)" % (kid, ks)
    elif exact:
        assert np.array_equal(got.astype(np.float64), ref), "exact-arithmetic case differs (kernel %d split %d)" % (kid, ks)
    else:
        err = oracle.normalised_error(got, ref, max(K, 1), max_abs(dtype, layout, A, M, K) or 1.0,
                                      max_abs(dtype, layout, B, K, N) or 1.0)
        assert err <= TOL[dtype], "normalised error %.3e > %.1e (kernel %d split %d)" % (err, TOL[dtype], kid, ks)
        assert err <= TIGHT[dtype], "normalised error %.3e > internal bound %.1e (kernel %d split %d)" % (err, TIGHT[dtype], kid, ks)
    # elements of the C buffer outside the M x N matrix must be untouched
    mask = np.ones(out.shape, dtype=bool)
    wl.logical(layout, mask, M, N)[...] = False
    assert np.array_equal(out[mask], np.asarray(C)[mask]), "padding of C was overwritten"
    return kid, ks
