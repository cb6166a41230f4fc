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


def test_network_graphs_are_consistent_with_the_layer_tables():
    """The whole-network graphs hold the same convolutions as the layer stacks (plus the
    classifier), every residual tensor is shaped like the output it is added to, and every
    operator reads a tensor that an earlier operator (or the input) produced."""
    from paper_2507_17301_amd import workloads as wl
    for graph, stack, batch in ((wl.resnet50_graph(), wl.resnet50_stack(), 2), (wl.resnet18_graph(), wl.resnet18_stack(), 2),
                                (wl.resnet101_graph(), wl.resnet101_stack(), 1)):
        convs = [op.layer for op in graph if op.kind == "conv"]
        key = lambda l: (l.H, l.W, l.Cin, l.Cout, l.Kh, l.Kw, l.stride, l.pad, l.n, l.m, l.tile)
        assert sorted(map(key, convs[:-1])) == sorted(map(key, stack))
        assert convs[-1].name == "fc" and convs[-1].n == convs[-1].m
        shapes = wl.net_tensor_shapes(graph, batch, 224)
        made = {0}
        for op in graph:
            assert op.src in made and op.dst not in made
            if op.kind == "conv":
                assert shapes[op.src] == (batch, op.layer.H, op.layer.W, op.layer.Cin)
                if op.residual >= 0:
                    assert op.residual in made and shapes[op.residual] == shapes[op.dst]
            made.add(op.dst)
        assert shapes[graph[-1].dst] == (batch, 1, 1, 1000)
        assert sum(op.residual >= 0 for op in graph) == sum(1 for op in graph if op.kind == "conv" and "conv1" in op.layer.name)
    ids = [i for i, w, b in wl.net_parameters(wl.resnet18_graph(), 7)]
    assert len(ids) == 21
