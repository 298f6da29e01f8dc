"""Descriptor pins: Table I's teacher columns (tests/golden/table1_teachers.txt) and textbook totals."""
import os

import numpy as np

from paper_2301_12443_amd import workloads as W


def _totals(blocks, in_shape):
    r = W.macs_and_params(blocks, in_shape)
    return sum(d + w for d, w, _ in r), sum(p for *_, p in r)


def _table1(model, dataset):
    """(params in millions, flops, unit multiplier, operations per multiply-accumulate) of one printed row."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "table1_teachers.txt")
    for line in open(path):
        f = line.split()
        if f and not line.startswith("#") and f[0] == model and f[1] == dataset:
            return float(f[2]), float(f[3]), {"M": 1e6, "B": 1e9}[f[4]], int(f[5])
    raise KeyError((model, dataset))


def test_vgg16_cifar_matches_table1():
    wl = W.vgg16_dsconv()
    macs, params = _totals(wl.teacher, wl.in_shape)
    p_m, flops, unit, per_mac = _table1("VGG-16", "Cifar-10")
    assert round(per_mac * macs / unit, 2) == flops            # 0.63 B
    assert round((params + 512 * 10 + 10) / 1e6, 2) == p_m     # + FC-10 head: 14.72 M
    assert W.activation_shapes(wl) == [(3, 32, 32), (64, 16, 16), (128, 8, 8), (256, 4, 4), (512, 1, 1)]


def test_mobilenetv2_imagenet_matches_table1():
    wl = W.mbv2_mbconv()
    macs, params = _totals(wl.teacher, wl.in_shape)
    head_macs = 320 * 1280 * 49 + 1280 * 1000                # 1x1 -> 1280 head at 7x7, FC-1000
    head_params = 320 * 1280 + 2 * 1280 + 1280 * 1000 + 1000
    p_m, flops, unit, per_mac = _table1("MobileNetV2", "ImageNet")
    assert abs(per_mac * (macs + head_macs) / unit - flops) < 0.05    # 300.77 M
    assert round((params + head_params) / 1e6, 2) == p_m              # 3.50 M
    macs_b = [d + w for d, w, _ in W.macs_and_params(wl.student, wl.in_shape)]
    assert macs_b[0] == max(macs_b)                          # Sec. VII-A: block 0 is the heaviest at 224^2
    sizes = [int(np.prod(s)) for s in W.activation_shapes(wl)[1:]]
    assert sizes[0] == max(sizes)                            # Sec. VII-C: early feature maps are the largest


def test_resnet50_textbook_totals():
    wl = W.resnet50_wide()
    macs, params = _totals(wl.teacher, wl.in_shape)
    assert abs((macs + 2048 * 1000) / 1e9 - 4.09) < 0.01
    assert abs((params + 2048 * 1000 + 1000) / 1e6 - 25.56) < 0.01
    assert W.activation_shapes(wl)[1:] == [(256, 56, 56), (512, 28, 28), (1024, 14, 14), (2048, 7, 7)]


def test_supernet_has_six_candidates_in_24_layers():
    wl = W.mbv2_supernet()
    mixes = [op for b in wl.student for op in b.ops if op.type == W.OP_MIX]
    assert len(mixes) == 24 and all(len(m.inputs) == 6 for m in mixes)
    assert all(abs(sum(m.p) - 1.0) < 1e-12 for m in mixes)


def test_pack_roundtrip_header_and_seeded_params_are_reproducible():
    for name, make in W.CONFIGS.items():
        wl = make()
        words, pool = W.pack(wl)
        assert words[0] == W.MAGIC and words[2] == wl.B and tuple(words[3:6]) == wl.in_shape
        nops = sum(len(b.ops) for b in wl.teacher + wl.student)
        assert len(words) == 6 + 2 * wl.B + nops * W.REC
    wl = W.tiny_cnn()
    a = W.make_param(wl, 1, 2, 0, W.P_WEIGHT, (32, 32, 3, 3))
    b = W.make_param(wl, 1, 2, 0, W.P_WEIGHT, (32, 32, 3, 3))
    np.testing.assert_array_equal(a, b)
    assert abs(a.std() - np.sqrt(2.0 / (32 * 9))) < 0.01
