"""The synthetic workload's shape tables against the values the paper prints (tests/golden/), and
against the convolution arithmetic that produces them: m = Hout*Wout, n = Cout, k = kh*kw*Cin."""
import os

import workloads as wl

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _table(name):
    rows = []
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        idx, layers, m, n, k = line.split()
        rows.append((int(idx), layers.split("/"), int(m), int(n), int(k)))
    return rows


def test_resnet50_table_matches_the_paper():
    rows = _table("resnet50_v1.5_im2row_gemm_dims.txt")
    assert [r[0] for r in rows] == list(range(1, 21))
    assert [(m, n, k) for _, _, m, n, k in rows] == list(wl.RESNET50_IM2ROW)
    assert [len(layers) for _, layers, _, _, _ in rows] == list(wl.RESNET50_MULTIPLICITY)
    assert sum(wl.RESNET50_MULTIPLICITY) == 53          # the 53 convolutions of ResNet50
    # the six shapes the benchmark's im2row configuration names are rows 1, 3, 7, 12, 17, 5
    assert wl.IM2ROW_HEADLINE == [(12544, 64, 147), (3136, 64, 576), (784, 128, 1152), (196, 256, 2304),
                                  (49, 512, 4608), (3136, 64, 256)]


def test_vgg16_table_matches_the_paper():
    rows = _table("vgg16_im2row_gemm_dims.txt")
    assert [(m, n, k) for _, _, m, n, k in rows] == list(wl.VGG16_IM2ROW)
    assert [len(layers) for _, layers, _, _, _ in rows] == list(wl.VGG16_MULTIPLICITY)
    assert sum(wl.VGG16_MULTIPLICITY) == 13             # the 13 convolutions of VGG16


def test_tables_follow_from_the_convolution_shapes():
    """m = output pixels, n = output channels, k = kernel height * width * input channels, batch 1."""
    # VGG16: 3x3 convolutions, stride 1, 'same' padding, on 224, 112, 56, 28, 14 pixel squares
    vgg = [(224, 3, 64), (224, 64, 64), (112, 64, 128), (112, 128, 128), (56, 128, 256), (56, 256, 256),
           (28, 256, 512), (28, 512, 512), (14, 512, 512)]
    derived = [(hw * hw, cout, 9 * cin) for hw, cin, cout in vgg]
    # row 7 (the first 28x28 layer, 256 -> 512 channels): the paper prints n = 256 where the network
    # has 512 output channels; the workload keeps the printed value, every other row agrees
    assert derived[6] == (784, 512, 2304) and wl.VGG16_IM2ROW[6] == (784, 256, 2304)
    assert derived[:6] + derived[7:] == list(wl.VGG16_IM2ROW[:6]) + list(wl.VGG16_IM2ROW[7:])
    # ResNet50 v1.5: the 7x7 stride-2 stem on 224x224x3, then bottleneck blocks (1x1, 3x3, 1x1 and the
    # 1x1 projection) on 56, 28, 14 and 7 pixel squares
    resnet = [(112, 7, 3, 64), (56, 1, 64, 64), (56, 3, 64, 64), (56, 1, 64, 256), (56, 1, 256, 64),
              (56, 1, 256, 128), (28, 3, 128, 128), (28, 1, 128, 512), (28, 1, 256, 512), (28, 1, 512, 128),
              (28, 1, 512, 256), (14, 3, 256, 256), (14, 1, 256, 1024), (14, 1, 512, 1024), (14, 1, 1024, 256),
              (14, 1, 1024, 512), (7, 3, 512, 512), (7, 1, 512, 2048), (7, 1, 1024, 2048), (7, 1, 2048, 512)]
    assert [(hw * hw, cout, kk * kk * cin) for hw, kk, cin, cout in resnet] == list(wl.RESNET50_IM2ROW)


def test_vgg16_layer_geometries_give_the_tables_gemm_sizes():
    """m = Hout*Wout, n = Cout, k = kh*kw*Cin for every row (row 7: the table's n is a misprint, m and k agree)."""
    assert len(wl.VGG16_CONVS) == len(wl.VGG16_IM2ROW)
    for i, ((H, W, Cin, Cout, kh, kw, stride, pad), (m, n, k)) in enumerate(zip(wl.VGG16_CONVS, wl.VGG16_IM2ROW)):
        Hout, Wout = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
        assert (Hout * Wout, kh * kw * Cin) == (m, k)
        assert Cout == n or (i == 6 and (Cout, n) == (512, 256))
