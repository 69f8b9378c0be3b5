"""Seeded synthetic inputs and the shape lists of the benchmark configurations.

This module holds no arithmetic of the method: it only draws matrices (numpy,
host memory) and lists shapes.  Both the CPU oracle's tests and the GPU tests /
benchmark take their inputs from here, so that both sides see identical bits.

Value recipes (one per configuration family):
  * fp32: i.i.d. uniform on [-1, 1), float32.
  * fp16: i.i.d. standard normal, rounded to nearest-even to binary16, handed
    over as uint16 bit patterns.
  * int8: i.i.d. uniform integers on [-128, 127].
The matrices stand in for the paper's workloads: a square GEMM (Sec. "Squared
Matrices") and the GEMMs that the im2row transform produces from the
convolution layers of ResNet50 v1.5 and VGG16 at batch 1 (Tables "resnet50" and "vgg16"),
where the
lowered activation matrix is replaced by an i.i.d. matrix of the same shape.
"""
import numpy as np

# (m, n, k) of the 20 distinct ResNet50 v1.5 layers, batch 1 (paper, Table "resnet50").
RESNET50_IM2ROW = [
    (12544, 64, 147), (3136, 64, 64), (3136, 64, 576), (3136, 256, 64), (3136, 64, 256),
    (3136, 128, 256), (784, 128, 1152), (784, 512, 128), (784, 512, 256), (784, 128, 512),
    (784, 256, 512), (196, 256, 2304), (196, 1024, 256), (196, 1024, 512), (196, 256, 1024),
    (196, 512, 1024), (49, 512, 4608), (49, 2048, 512), (49, 2048, 1024), (49, 512, 2048),
]
# How many layers of the network share each of those shapes (same table, "Layer numbers").
RESNET50_MULTIPLICITY = [1, 1, 3, 4, 2, 1, 4, 4, 1, 3, 1, 6, 6, 1, 5, 1, 3, 3, 1, 2]

# (m, n, k) of the 9 distinct VGG16 layers, batch 1 (paper, Table "vgg16").
VGG16_IM2ROW = [
    (50176, 64, 27), (50176, 64, 576), (12544, 128, 576), (12544, 128, 1152), (3136, 256, 1152),
    (3136, 256, 2304), (784, 256, 2304), (784, 512, 4608), (196, 512, 4608),
]
VGG16_MULTIPLICITY = [1, 1, 1, 1, 1, 2, 1, 2, 3]

# The six headline im2row shapes: rows 1, 3, 7, 12, 17, 5 of the ResNet50 table.
IM2ROW_HEADLINE = [RESNET50_IM2ROW[r - 1] for r in (1, 3, 7, 12, 17, 5)]

FP32_SQUARES = [1024, 2048, 4096, 8192]
FP16_SQUARES = [2048, 4096, 8192]
INT8_SHAPES = [(4096, 4096, 4096), (1000, 999, 1001), (4096, 64, 4096), (64, 4096, 4096), (33, 17, 2049)]


def tight_ld(layout, rows, cols):
    """Leading dimension of a rows x cols matrix stored without padding."""
    return max(1, rows if layout == "col" else cols)


def _shape(layout, rows, cols, ld):
    # buffer as a 2-D array whose second axis is the contiguous one
    return (cols, ld) if layout == "col" else (rows, ld)


def _rng(seed):
    return np.random.default_rng(int(seed))


def uniform_f32(seed, layout, rows, cols, ld=None):
    """rows x cols float32 matrix, entries U[-1,1); padding entries (ld > extent) are drawn too."""
    ld = tight_ld(layout, rows, cols) if ld is None else ld
    return (_rng(seed).random(_shape(layout, rows, cols, ld), dtype=np.float32) * 2.0 - 1.0).astype(np.float32)


def normal_f16_bits(seed, layout, rows, cols, ld=None):
    """rows x cols matrix of N(0,1) draws rounded to binary16, returned as uint16 bit patterns."""
    ld = tight_ld(layout, rows, cols) if ld is None else ld
    x = _rng(seed).standard_normal(_shape(layout, rows, cols, ld), dtype=np.float32)
    return np.ascontiguousarray(x.astype(np.float16).view(np.uint16))


def _to_bf16_bits(x):
    """float32 array -> bfloat16 bit patterns (the upper 16 bits), rounded to nearest, ties to even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def normal_bf16_bits(seed, layout, rows, cols, ld=None):
    """rows x cols matrix of N(0,1) draws rounded to bfloat16, returned as uint16 bit patterns."""
    ld = tight_ld(layout, rows, cols) if ld is None else ld
    return _to_bf16_bits(_rng(seed).standard_normal(_shape(layout, rows, cols, ld), dtype=np.float32))


def uniform_i8(seed, layout, rows, cols, ld=None):
    """rows x cols int8 matrix, entries uniform on [-128, 127]."""
    ld = tight_ld(layout, rows, cols) if ld is None else ld
    return _rng(seed).integers(-128, 128, size=_shape(layout, rows, cols, ld), dtype=np.int8)


def uniform_i32(seed, layout, rows, cols, ld=None, lo=-1000, hi=1000):
    ld = tight_ld(layout, rows, cols) if ld is None else ld
    return _rng(seed).integers(lo, hi + 1, size=_shape(layout, rows, cols, ld), dtype=np.int32)


def small_int_f32(seed, layout, rows, cols, ld=None, bound=8):
    """float32 matrix of integers in [-bound, bound]: every partial sum stays exact in fp32."""
    ld = tight_ld(layout, rows, cols) if ld is None else ld
    return _rng(seed).integers(-bound, bound + 1, size=_shape(layout, rows, cols, ld)).astype(np.float32)


def small_int_f16_bits(seed, layout, rows, cols, ld=None, bound=8):
    ld = tight_ld(layout, rows, cols) if ld is None else ld
    x = _rng(seed).integers(-bound, bound + 1, size=_shape(layout, rows, cols, ld)).astype(np.float16)
    return np.ascontiguousarray(x.view(np.uint16))


def small_int_bf16_bits(seed, layout, rows, cols, ld=None, bound=8):
    ld = tight_ld(layout, rows, cols) if ld is None else ld
    x = _rng(seed).integers(-bound, bound + 1, size=_shape(layout, rows, cols, ld)).astype(np.float32)
    return _to_bf16_bits(x)          # small integers are bfloat16 values already


def bf16_bits_to_f32(bits):
    """bfloat16 bit patterns -> the float32 values they denote."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def logical(layout, buf, rows, cols):
    """View the rows x cols matrix held in a buffer made by the generators above as (rows, cols)."""
    return buf[:cols, :rows].T if layout == "col" else buf[:rows, :cols]


def conv_tensors_f32(seed, batch, H, W, Cin, Cout, kh, kw, Hout, Wout):
    """Seeded U[-1,1) channels-last image [batch,H,W,Cin], filter [kh,kw,Cin,Cout] and old output
    [batch,Hout,Wout,Cout] of a convolution layer (float32)."""
    image = uniform_f32(seed, "row", batch * H * W, Cin).reshape(batch, H, W, Cin)
    filt = uniform_f32(seed + 1, "row", kh * kw * Cin, Cout).reshape(kh, kw, Cin, Cout)
    old = uniform_f32(seed + 2, "row", batch * Hout * Wout, Cout).reshape(batch, Hout, Wout, Cout)
    return image, filt, old


# Convolution geometries (H, W, Cin, Cout, kh, kw, stride, pad) of ResNet50 v1.5 layers whose im2row
# GEMMs are the paper's six headline shapes, in the order of IM2ROW_HEADLINE.
RESNET50_HEADLINE_CONVS = [
    (224, 224, 3, 64, 7, 7, 2, 3),
    (56, 56, 64, 64, 3, 3, 1, 1),
    (56, 56, 128, 128, 3, 3, 2, 1),
    (28, 28, 256, 256, 3, 3, 2, 1),
    (14, 14, 512, 512, 3, 3, 2, 1),
    (56, 56, 256, 64, 1, 1, 1, 0),
]

# The 13 convolution layers of VGG16 (all 3 x 3, stride 1, padding 1) grouped as in the paper's Table
# "vgg16" (H, W, Cin, Cout, kh, kw, stride, pad), in the order of VGG16_IM2ROW.  Row 7 of the table prints
# n = 256 where the network's layer has 512 output channels; the geometry keeps the network's value.
VGG16_CONVS = [
    (224, 224, 3, 64, 3, 3, 1, 1), (224, 224, 64, 64, 3, 3, 1, 1), (112, 112, 64, 128, 3, 3, 1, 1),
    (112, 112, 128, 128, 3, 3, 1, 1), (56, 56, 128, 256, 3, 3, 1, 1), (56, 56, 256, 256, 3, 3, 1, 1),
    (28, 28, 256, 512, 3, 3, 1, 1), (28, 28, 512, 512, 3, 3, 1, 1), (14, 14, 512, 512, 3, 3, 1, 1),
]
