"""Pins for arithmetic intensity, CMR and the selector against values the paper prints."""
import os

import pytest

import oracle
from paper_2104_09455_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [float(l) for l in f if l.strip() and not l.startswith("#")]


def test_square_intensities_fig11_axis_labels():
    """FP16 AI of M=N=K=n is n/3; the paper prints 10.7 ... 682.7 under Fig. 11 (Sec. 6.4)."""
    printed = [10.7, 21.3, 42.7, 85.3, 170.7, 341.3, 682.7]
    for n, p in zip(wl.square_sizes_paper(), printed):
        assert round(oracle.arithmetic_intensity(n, n, n, "f16"), 1) == p
    assert oracle.flops(2, 3, 5) == 60 and oracle.bytes_moved(2, 3, 5, "f16") == 2 * (10 + 15 + 6)
    assert oracle.bytes_moved(2, 3, 5, "i8") == 10 + 15 + 4 * 6


def test_resnet50_hd_per_layer_intensity_fig5():
    """All 54 bar heights of Fig. 5 (ResNet-50, 1080x1920, batch 1), unpadded dimensions."""
    want = _golden("resnet50_hd_layer_ai.txt")
    layers = wl.resnet50_layers(1, 1080, 1920, with_fc=True)
    assert len(want) == len(layers) == 54
    for l, w in zip(layers, want):
        assert oracle.arithmetic_intensity(l.M, l.N, l.K, "f16") == pytest.approx(w, rel=1e-12), l.name
    assert min(want) == pytest.approx(0.9985139304394631) and round(max(want)) == 511  # "1--511", Sec. 3.2


def test_aggregate_intensities_printed_in_the_paper():
    """Aggregate AI = sum FLOPs / sum bytes (Sec. 3.2), dimensions padded to multiples of 8
    (Sec. 6.2): ResNet-50 122.0 at 1080x1920 and 72 at 224x224; DLRM MLP-Bottom 7.4 at batch 1
    and 92.0 at batch 2048 (labels of Fig. 4 / Fig. 10)."""
    shp = lambda ls: [(l.M, l.N, l.K) for l in ls]
    hd = oracle.aggregate_intensity(shp(wl.resnet50_layers(1, 1080, 1920, with_fc=True)), pad_to=8)
    assert round(hd, 1) == 122.0
    lo = oracle.aggregate_intensity(shp(wl.resnet50_layers(1, 224, 224, with_fc=True)), pad_to=8)
    assert round(lo) == 72
    bottom = lambda b: shp(wl.dlrm_layers(b)[:3])
    assert round(oracle.aggregate_intensity(bottom(1), pad_to=8), 1) == 7.4
    assert round(oracle.aggregate_intensity(bottom(2048), pad_to=8), 1) == 92.0
    # "70--109 at batch size 256" (Sec. 3.2): the bottom MLP is the 70
    assert round(oracle.aggregate_intensity(bottom(256), pad_to=8)) == 70


def test_cmr_values_printed_in_the_paper():
    """T4: 65 FP16 TFLOP/s over 320 GB/s = 203; P4: 11 TFLOP/s, T4 has 1.7x its bandwidth -> 58
    (Sec. 3.3, Sec. 6.2)."""
    assert round(oracle.cmr(65e12, 320e9)) == 203
    assert round(oracle.cmr(11e12, 320e9 / 1.7)) == 58


def test_selector_rule_and_t4_crossover():
    """Eq. 1 is a strict inequality; on the T4 the square sizes up to 512 are bandwidth bound
    and 1024, 2048 compute bound (dashed line of Fig. 11)."""
    t4 = oracle.cmr(65e12, 320e9)
    picks = [oracle.select(n, n, n, "f16", t4) for n in wl.square_sizes_paper()]
    assert picks == [oracle.THREAD] * 5 + [oracle.GLOBAL] * 2
    ai = oracle.arithmetic_intensity(600, 600, 600, "f16")  # exactly 200
    assert ai == 200.0
    assert oracle.select(600, 600, 600, "f16", 200.0) == oracle.THREAD      # tie -> not compute bound
    assert oracle.select(600, 600, 600, "f16", 199.999) == oracle.GLOBAL


def test_mi355x_selection_of_benchmark_shapes():
    """With the spec-sheet ratio 2.5166 PFLOP/s / 8 TB/s = 314.6 (fp16/bf16) and 629 (int8)."""
    c16 = oracle.cmr(2516.6e12, 8e12)
    c8 = oracle.cmr(5033.2e12, 8e12)
    assert round(c16, 1) == 314.6 and round(c8) == 629
    for n in (4096, 8192):
        assert oracle.select(n, n, n, "f16", c16) == oracle.GLOBAL
    assert oracle.select(8192, 8192, 8192, "i8", c8) == oracle.GLOBAL
    for b in (1, 16, 256):
        assert all(oracle.select(l.M, l.N, l.K, "f16", c16) == oracle.THREAD for l in wl.dlrm_layers(b))
    # sweep N = K = 4096: crossover between M = 256 and M = 512
    picks = {m: oracle.select(m, 4096, 4096, "f16", c16) for m in wl.sweep_m()}
    assert picks[256] == oracle.THREAD and picks[512] == oracle.GLOBAL


def test_resnet50_224_has_53_convs_with_expected_shapes():
    ls = wl.resnet50_layers(1)
    assert len(ls) == 53
    assert (ls[0].M, ls[0].N, ls[0].K) == (112 * 112, 64, 147)
    by = {l.name: l for l in ls}
    l = by["layer3.1.conv2"]   # 3x3 256->256 on 14x14
    assert (l.M, l.N, l.K) == (196, 256, 2304)
    l = by["layer3.1.conv1"]   # 1x1 1024->256 on 14x14
    assert (l.M, l.N, l.K) == (196, 256, 1024)
    l = wl.resnet50_layers(64)[-1]
    assert (l.M, l.N, l.K) == (64 * 49, 2048, 512)
