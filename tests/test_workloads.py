"""Layer tables and generators: counts, shapes and totals (CPU only)."""
import numpy as np

from paper_2507_17301_amd import workloads as wl


def test_stack_sizes_and_unique_shapes():
    r18, r50, r101 = wl.resnet18_stack(), wl.resnet50_stack(), wl.resnet101_stack()
    assert (len(r18), len(wl.unique_shapes(r18))) == (20, 11)
    assert (len(r50), len(wl.unique_shapes(r50))) == (53, 23)
    assert (len(r101), len(wl.unique_shapes(r101))) == (104, 23)
    for stack in (r18, r50, r101):
        assert stack[0].n == stack[0].m == 1 and stack[0].Cin == 3      # dense stem
        assert all(l.K % l.m == 0 and l.Cin % l.m == 0 for l in stack[1:])
    assert {(l.n, l.m) for l in r101 if l.stage == 3} == {(2, 8)}


def test_flop_totals():
    # 2*P*K*Cout summed over ResNet-50 at batch 64: 8.17 dense GFLOP per image
    r50 = wl.resnet50_stack()
    assert abs(sum(l.dense_flops(64) for l in r50) / 64e9 - 8.174) < 0.01
    assert abs(sum(l.effective_flops(64) for l in r50) / 1e9 - 269.1) < 0.1
    # chained shapes: each 3x3 s2 halves the resolution
    assert [l.Ho for l in r50 if l.name.endswith("b0_conv2_3x3")] == [56, 28, 14, 7]


def test_generators_are_seeded_and_shaped():
    l = wl.single_conv_config1()
    x, w, b = wl.make_tensors(l, 1, 0, weight_sigma=0.05)
    x2, w2, b2 = wl.make_tensors(l, 1, 0, weight_sigma=0.05)
    assert x.shape == (1, 56, 56, 64) and w.shape == (64, 3, 3, 64) and b.shape == (64,)
    assert np.array_equal(x, x2) and np.array_equal(w, w2) and np.array_equal(b, b2)
    assert x.min() >= 0 and x.max() < 1 and abs(w.std() - 0.05) < 0.002
    pts = wl.sample_points(l, 1, 10, 0)
    assert pts.shape == (26, 4) and pts[:, 3].max() < 64
