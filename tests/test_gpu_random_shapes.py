"""Seeded random layer geometries through the C ABI against the CPU oracle: the
default variant and one randomly forced legal variant per case, with and without
a residual input, fp32 and bf16.  The draw covers what the fixed grids do not
combine: odd image sizes with strides and dilations, channel counts that are not
multiples of the tile, groups wider than a chunk, ragged last pixel tiles."""
import numpy as np
import pytest

import oracle
from paper_2507_17301_amd import binding as nm
from paper_2507_17301_amd import workloads as wl
from gpu_util import FP32_TOL, BF16_TOL, say, norm_err

pytestmark = pytest.mark.gpu


def _draw(rng):
    k = int(rng.choice([1, 1, 3, 3, 5]))
    kw = k if rng.random() < 0.8 else int(rng.choice([1, 3]))
    dil = int(rng.choice([1, 1, 1, 2]))
    stride = int(rng.choice([1, 1, 2]))
    pad = int(rng.integers(0, (k // 2) * dil + 2))
    cin = int(rng.choice([8, 16, 24, 32, 48, 64, 96, 128]))
    tile = int(rng.choice([8, 16, 16, 16, 32]))
    cout = int(rng.choice([tile, 2 * tile, 3 * tile, 2 * tile + 4, 5 * tile - 8, 72]))
    K = k * kw * cin
    n, m = [(2, 4), (1, 4), (2, 8), (4, 8), (1, 8), (1, 1), (cin // 2, cin), (K // 4, K)][int(rng.integers(0, 8))]
    lo = (max(k, kw) - 1) * dil + 1
    h = int(rng.integers(max(lo - 2 * pad, 1), 24))
    w = int(rng.integers(max(lo - 2 * pad, 1), 24))
    return wl.ConvLayer("rand", h, w, cin, max(cout, 4), k, kw, stride, pad, dil, n, m, tile), int(rng.integers(1, 5))


CASES = []
_rng = np.random.default_rng(20250717)
while len(CASES) < 48:
    layer, batch = _draw(_rng)
    if layer.K % layer.m == 0 and layer.m <= 16384 and layer.Ho >= 1 and layer.Wo >= 1:
        CASES.append((layer, batch, len(CASES)))


@pytest.mark.parametrize("layer,batch,idx", CASES, ids=[f"case{c[2]}" for c in CASES])
def test_random_geometry(layer, batch, idx):
    import torch
    bf16 = idx % 3 == 2
    with_res = idx % 4 == 1
    say(f"random {idx} {layer} batch={batch} bf16={bf16} residual={with_res}")
    rng = np.random.default_rng(9000 + idx)
    x, w, bias = wl.make_tensors(layer, batch, 9000 + idx, weight_sigma=0.1)
    res = rng.standard_normal((batch, layer.Ho, layer.Wo, layer.Cout), dtype=np.float32) if with_res else None
    _, _, wz = oracle.prune(w, layer.n, layer.m, layer.tile)
    if bf16:
        wz, xr = oracle.round_bf16(wz), oracle.round_bf16(x)
        rr = oracle.round_bf16(res) if with_res else None
    else:
        xr, rr = x, res
    if with_res:
        ref = oracle.conv2d_res(xr, wz, rr, bias, layer.stride, layer.pad, layer.dil, True, out_bf16=bf16)
    else:
        ref = oracle.conv2d(xr, wz, bias, layer.stride, layer.pad, layer.dil, True, out_bf16=bf16)
    ndt = nm.NM_BF16 if bf16 else nm.NM_F32
    tdt = torch.bfloat16 if bf16 else torch.float32
    wp = nm.nm_prune(w, layer.n, layer.m, layer.tile, ndt)
    xd = torch.from_numpy(x).cuda().to(tdt)
    bd = torch.from_numpy(bias).cuda()
    rd = torch.from_numpy(res).cuda().to(tdt) if with_res else None
    legal = [v for v in range(nm.nm_variant_count()) if nm.nm_variant_legal(v, wp, ndt, ndt)]
    assert legal
    forced = legal[int(rng.integers(0, len(legal)))]
    tol = BF16_TOL if bf16 else FP32_TOL
    try:
        for v in (-1, forced):
            nm.nm_force_variant(v)
            if with_res:
                y = nm.nm_conv2d_res(xd, wp, rd, bd, layer.stride, layer.pad, layer.dil, True)
            else:
                y = nm.nm_conv2d(xd, wp, bd, layer.stride, layer.pad, layer.dil, True)
            torch.cuda.synchronize()
            assert y.shape == ref.shape
            name = "default" if v < 0 else nm.nm_variant_name(v)
            assert norm_err(y.float().cpu().numpy(), ref) <= tol, name
    finally:
        nm.nm_force_variant(-1)
