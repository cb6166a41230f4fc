"""nm_conv2d_static -- the entry point that allocates nothing -- against nm_conv2d_res:
K-split variants forced, so that the static scratch buffer is what carries the partial
sums; two calls in a row, the second on a smaller input; then a size it must refuse."""
import numpy as np
import pytest

from paper_2507_17301_amd import binding as nm
from paper_2507_17301_amd import workloads as wl
from gpu_util import say

pytestmark = pytest.mark.gpu

L = wl.ConvLayer


def _split_variant(wp, splits):
    for v in range(nm.nm_variant_count()):
        name = nm.nm_variant_name(v)
        if name.endswith(f"_S{splits}") and nm.nm_variant_legal(v, wp):
            return v
    raise AssertionError("no K-split variant is legal for this layer")


def test_static_entry_point_matches_the_allocating_one():
    import torch
    big = L("static_big", 14, 14, 256, 64, 3, 3, 1, 1, 1, 2, 4, 16)
    small = L("static_small", 7, 7, 256, 64, 3, 3, 1, 1, 1, 2, 4, 16)
    _, w, bias = wl.make_tensors(big, 1, 80, with_input=False)
    wp = nm.nm_prune(w, 2, 4, 16)
    bd = torch.from_numpy(bias).cuda()
    try:
        for layer, batch, splits in ((big, 4, 8), (small, 2, 4)):      # the second call is the smaller one
            x, _, _ = wl.make_tensors(layer, batch, 81)
            xd = torch.from_numpy(x).cuda()
            rng = np.random.default_rng(3)
            rd = torch.from_numpy(rng.standard_normal((batch, layer.Ho, layer.Wo, 64)).astype(np.float32)).cuda()
            v = _split_variant(wp, splits)
            nm.nm_force_variant(v)
            say(f"static entry point: {layer.name} batch {batch} {nm.nm_variant_name(v)}")
            y_ref = nm.nm_conv2d_res(xd, wp, rd, bd, 1, 1, 1, True)
            y = torch.full_like(y_ref, float("nan"))
            nm.nm_conv2d_static(xd, wp, rd, bd, 1, 1, 1, True, y)
            torch.cuda.synchronize()
            assert nm.nm_last_variant() == v
            assert torch.equal(y, y_ref)        # same kernels, same order of additions: bit for bit
        # 8 splits x 64 x 112 x 112 pixels x 64 channels x 4 bytes = 1.6 GB of partial sums: refused, nothing launched
        huge = L("static_huge", 112, 112, 256, 64, 3, 3, 1, 1, 1, 2, 4, 16)
        xh = torch.zeros((64, 112, 112, 256), device="cuda")
        yh = torch.zeros((64, 112, 112, 64), device="cuda")
        nm.nm_force_variant(_split_variant(wp, 8))
        with pytest.raises(nm.NMError) as e:
            nm.nm_conv2d_static(xh, wp, None, bd, 1, 1, 1, True, yh)
        assert e.value.code == nm.NM_ERR_SHAPE and "static buffer" in str(e.value)
    finally:
        nm.nm_force_variant(-1)
