"""CPU oracle for C = alpha*A*B + beta*C.  TEST INFRASTRUCTURE ONLY.

This package is the checker that the GPU library is compared against; it is
never part of the product path.  Only the tests, the smoke check and the
benchmark's CPU-baseline leg may import it, and it imports nothing from the
GPU package.

The arithmetic lives in ``ref_gemm.c`` (a triple loop in fp64 / int64 that
follows the definition of the product in the paper's Sec. II-A and the
alpha/beta form of its reference micro-kernel).  This module only compiles
that file with gcc and marshals numpy arrays into it.  ``ref_conv.c`` holds the
im2row transform and the convolution the paper's rectangular GEMMs come from
(Sec. "Rectangular Matrices"), written out directly over the image.
"""
from .ref import (  # noqa: F401
    build,
    num_threads,
    half_to_double,
    bfloat16_to_double,
    gemm_f32,
    gemm_f16,
    gemm_bf16,
    gemm_i8,
    gemm_ex,
    gemm_sample,
    conv_output_shape,
    im2row_f32,
    conv2d_nhwc_f32,
    im2row,
    conv2d_nhwc,
    narrow_f16,
    narrow_bf16,
    half_bits_to_double,
    bfloat16_bits_to_double,
    wrap_int32,
    normalised_error,
)
