"""K-split variants of the fp32 MFMA kernel (several workgroups share the K axis of one
output tile; a second kernel adds their partial sums and applies bias, residual and
activation) against the CPU oracle, through the C ABI."""
import re

import numpy as np
import pytest

import oracle
from paper_2507_17301_amd import binding as nm
from paper_2507_17301_amd import workloads as wl
from gpu_util import FP32_TOL, BF16_TOL, say, norm_err

pytestmark = pytest.mark.gpu

L = wl.ConvLayer

CASES = [
    # name, H, W, Cin, Cout, Kh, Kw, stride, pad, dil, n, m, tile | batch, bf16
    (L("sk_3x3", 9, 7, 64, 48, 3, 3, 1, 1, 1, 2, 4, 16), 2, False),
    (L("sk_7x7_deep", 7, 7, 512, 64, 3, 3, 1, 1, 1, 2, 4, 16), 1, False),        # the case it is for: 49 pixels, K' = 2304
    (L("sk_1x1_s2_cout37", 9, 9, 128, 37, 1, 1, 2, 0, 1, 2, 4, 5), 2, False),     # element-wise stores
    (L("sk_stem_like", 20, 20, 3, 32, 7, 7, 2, 3, 1, 1, 1, 16), 2, False),        # element-wise staging
    (L("sk_T8_dil2", 10, 9, 32, 24, 3, 3, 1, 2, 2, 1, 4, 8), 1, False),
    (L("sk_group_per_tap", 8, 8, 128, 32, 3, 3, 1, 1, 1, 16, 128, 16), 2, False), # variable-step form
    (L("sk_bf16_io", 9, 7, 64, 48, 3, 3, 1, 1, 1, 2, 4, 16), 2, True),            # fp32 MFMA kernel on bf16 tensors
]


@pytest.mark.parametrize("layer,batch,bf16", CASES, ids=[c[0].name for c in CASES])
@pytest.mark.parametrize("with_res", [False, True])
def test_k_split_variants(layer, batch, bf16, with_res):
    import torch
    x, w, bias = wl.make_tensors(layer, batch, 71, weight_sigma=0.1)
    _, _, wz = oracle.prune(w, layer.n, layer.m, layer.tile)
    rng = np.random.default_rng(9)
    res = rng.standard_normal((batch, layer.Ho, layer.Wo, layer.Cout)).astype(np.float32) if with_res else None
    rnd = oracle.round_bf16 if bf16 else (lambda a: a)
    relu, use_bias = (not with_res), (with_res or layer.Cout != 48)
    b = bias if use_bias else None
    if with_res:
        ref = oracle.conv2d_res(rnd(x), rnd(wz), rnd(res), b, layer.stride, layer.pad, layer.dil, relu, out_bf16=bf16)
    else:
        ref = oracle.conv2d(rnd(x), rnd(wz), b, layer.stride, layer.pad, layer.dil, relu, out_bf16=bf16)
    tdt = torch.bfloat16 if bf16 else torch.float32
    ndt = nm.NM_BF16 if bf16 else nm.NM_F32
    wp = nm.nm_prune(w, layer.n, layer.m, layer.tile, ndt)
    xd = torch.from_numpy(x).cuda().to(tdt)
    rd = torch.from_numpy(res).cuda().to(tdt) if with_res else None
    bd = torch.from_numpy(bias).cuda() if use_bias else None
    ran = {}
    try:
        for v in range(nm.nm_variant_count()):
            name = nm.nm_variant_name(v)
            m = re.search(r"_S(\d+)$", name)
            if not m or not nm.nm_variant_legal(v, wp, ndt, ndt):
                continue
            split = int(m.group(1))
            if ran.get(split, 0) >= 12:       # a dozen tile shapes per split count is plenty here
                continue
            say(f"forced {name} on {layer.name} residual={with_res}")
            nm.nm_force_variant(v)
            y = nm.nm_conv2d_res(xd, wp, rd, bd, layer.stride, layer.pad, layer.dil, relu)
            torch.cuda.synchronize()
            assert nm.nm_last_variant() == v
            assert norm_err(y.float().cpu().numpy(), ref) <= (BF16_TOL if bf16 else FP32_TOL), name
            ran[split] = ran.get(split, 0) + 1
    finally:
        nm.nm_force_variant(-1)
    assert ran.get(2, 0) >= 3, ran            # every case has at least two chunks
    if layer.K >= 4096:
        assert ran.get(16, 0) >= 3, ran


def test_tuner_takes_a_split_where_the_tiles_cannot_fill_the_chip():
    """7x7x512 -> 512, 3x3, batch 1: 49 pixels and 32 row blocks are at most 32 output tiles
    for 256 CUs; the tuner times the K-split forms too, and whatever it picks matches the oracle."""
    import torch
    layer = L("deep_b1", 7, 7, 512, 512, 3, 3, 1, 1, 1, 2, 4, 16)
    x, w, bias = wl.make_tensors(layer, 1, 72)
    _, _, wz = oracle.prune(w, 2, 4, 16)
    ref = oracle.conv2d(x, wz, bias, 1, 1, 1, True)
    wp = nm.nm_prune(w, 2, 4, 16)
    v, ms = nm.nm_autotune(nm.NM_F32, 1, 7, 7, 512, wp, True, 1, 1, 1, True)
    name = nm.nm_variant_name(v)
    say(f"tuned pick for {layer.name}: {name} {ms * 1e3:.1f} us")
    y = nm.nm_conv2d(torch.from_numpy(x).cuda(), wp, torch.from_numpy(bias).cuda(), 1, 1, 1, True)
    torch.cuda.synchronize()
    assert nm.nm_last_variant() == v
    assert norm_err(y.cpu().numpy(), ref) <= FP32_TOL
    assert re.search(r"_S\d+$", name), name   # with 9 x 8 = 72 chunks to share, a split wins here
    nm.nm_workspace_free()
    y2 = nm.nm_conv2d(torch.from_numpy(x).cuda(), wp, torch.from_numpy(bias).cuda(), 1, 1, 1, True)   # grows it again
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
