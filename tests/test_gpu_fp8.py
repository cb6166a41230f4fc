"""The fp8 (E4M3) workload against the CPU oracle, through the C ABI: kept sets and the
stored E4M3 values bit for bit, the convolution within the bf16 tolerance (exact products,
fp32 accumulation, one bf16 rounding) with the oracle fed the E4M3 operands as exact floats."""
import re

import numpy as np
import pytest

import oracle
from paper_2507_17301_amd import binding as nm
from paper_2507_17301_amd import workloads as wl
from gpu_util import BF16_TOL, say, norm_err

pytestmark = pytest.mark.gpu

L = wl.ConvLayer
R50 = wl.resnet50_stack()


def _fp8_input(shape, seed):
    """(device E4M3 tensor, the same values as fp32 numpy): uniform [0, 1) rounded to E4M3."""
    import torch
    g = torch.Generator().manual_seed(seed)
    x8 = torch.rand(shape, generator=g, dtype=torch.float32).to(torch.float8_e4m3fn)
    return x8.cuda(), x8.float().numpy()


def _oracle_weights(layer, w):
    """Zero-filled weights as the fp8 path stores them: kept set from the fp32 weights, then
    one power-of-two scale per layer and E4M3 rounding."""
    _, idx, wz = oracle.prune(w, layer.n, layer.m, layer.tile)
    wq, s = oracle.quantize_e4m3(wz)
    return idx, wq, s


@pytest.mark.parametrize("cout,cin,k,n,m,tile,sigma", [
    (48, 64, 3, 2, 4, 16, 0.05), (40, 128, 1, 1, 4, 16, 1.0), (72, 64, 3, 2, 8, 32, 3e-4), (16, 64, 1, 4, 8, 16, 200.0)])
def test_fp8_prune_matches_the_oracle_bit_for_bit(cout, cin, k, n, m, tile, sigma):
    rng = np.random.default_rng(cout + cin)
    w = (rng.standard_normal((cout, k, k, cin)) * sigma).astype(np.float32)
    say(f"fp8 prune {cout}x{k}x{k}x{cin} {n}:{m} T={tile} sigma={sigma}")
    wp = nm.nm_prune(w, n, m, tile, nm.NM_F8E4M3)
    mask, idx, wz = oracle.prune(w, n, m, tile)
    assert np.array_equal(nm.nm_packed_indices(wp), idx)
    assert np.array_equal(nm.nm_packed_mask(wp), mask)
    s = oracle.fp8_weight_scale(wz)
    assert nm.nm_packed_scale(wp) == s
    vals = oracle.pack(w, idx, n, m, tile)
    want = (oracle.round_e4m3(vals * np.float32(s)) / np.float32(s)).astype(np.float32)
    got = nm.nm_packed_values(wp)
    assert np.array_equal(got, want) and np.array_equal(np.signbit(got), np.signbit(want))
    assert np.all(np.abs(want) * s <= 448.0) and np.max(np.abs(want)) * s > 224.0   # the scale uses the top binade


CASES = [
    # name, H, W, Cin, Cout, Kh, Kw, stride, pad, dil, n, m, tile | batch
    (L("f8_3x3", 11, 9, 64, 80, 3, 3, 1, 1, 1, 2, 4, 16), 3),
    (L("f8_3x3_s2_cout40", 13, 11, 64, 40, 3, 3, 2, 1, 1, 2, 4, 16), 3),       # last row block half empty
    (L("f8_3x3_dil2", 12, 10, 128, 48, 3, 3, 1, 2, 2, 1, 4, 16), 2),
    (L("f8_1x1_s2_T32_cout72", 9, 9, 192, 72, 1, 1, 2, 0, 1, 2, 8, 32), 3),    # T = 32, third tile a quarter full
    (L("f8_1x3_pad0", 7, 9, 64, 64, 1, 3, 1, 0, 1, 2, 4, 16), 2),
    (L("f8_dense", 10, 10, 64, 96, 3, 3, 1, 1, 1, 1, 1, 16), 2),
    (L("f8_one_pixel", 3, 3, 64, 24, 3, 3, 1, 0, 1, 2, 4, 16), 1),
    (L("f8_group_per_tap", 8, 8, 128, 32, 3, 3, 1, 1, 1, 32, 128, 16), 2),
    (L("f8_3x3_cin256", 9, 7, 256, 56, 3, 3, 1, 1, 1, 2, 4, 16), 3),           # 256-channel chunks, ring of stages wraps
    (L("f8_1x1_cin512_s2", 15, 15, 512, 144, 1, 1, 2, 0, 1, 1, 4, 16), 2),     # 1, 2 or 4 ... 8 chunks by chunk size
]


@pytest.mark.parametrize("layer,batch", CASES, ids=[c[0].name for c in CASES])
@pytest.mark.parametrize("with_res", [False, True])
def test_fp8_conv_every_variant(layer, batch, with_res):
    import torch
    _, w, bias = wl.make_tensors(layer, batch, 91, weight_sigma=0.1, with_input=False)
    xd, x = _fp8_input((batch, layer.H, layer.W, layer.Cin), 92)
    _, wq, s = _oracle_weights(layer, w)
    rng = np.random.default_rng(7)
    res = rng.standard_normal((batch, layer.Ho, layer.Wo, layer.Cout)).astype(np.float32) if with_res else None
    relu, use_bias = (not with_res), (with_res or layer.Cout != 64)
    b = bias if use_bias else None
    if with_res:
        ref = oracle.conv2d_res(x, wq, oracle.round_bf16(res), b, layer.stride, layer.pad, layer.dil, relu, out_bf16=True)
    else:
        ref = oracle.conv2d(x, wq, b, layer.stride, layer.pad, layer.dil, relu, out_bf16=True)
    wp = nm.nm_prune(w, layer.n, layer.m, layer.tile, nm.NM_F8E4M3)
    rd = torch.from_numpy(res).cuda().to(torch.bfloat16) if with_res else None
    bd = torch.from_numpy(bias).cuda() if use_bias else None
    ran, families = 0, set()
    try:
        for v in range(nm.nm_variant_count()):
            if not nm.nm_variant_legal(v, wp, nm.NM_F8E4M3, nm.NM_BF16):
                continue
            name = nm.nm_variant_name(v)
            # F8: register-streaming kernel; F8S / F8W / F8R: the LDS-staged one, plain, with producer
            # wavefronts, with producer wavefronts and register-held weights
            assert re.match(r"F8[SWR]?_NB", name)
            families.add(name.split("_")[0])
            say(f"forced {name} on {layer.name} residual={with_res}")
            nm.nm_force_variant(v)
            y = nm.nm_conv2d_res(xd, wp, rd, bd, layer.stride, layer.pad, layer.dil, relu)
            torch.cuda.synchronize()
            assert y.dtype == torch.bfloat16
            assert norm_err(y.float().cpu().numpy(), ref) <= BF16_TOL, name
            ran += 1
    finally:
        nm.nm_force_variant(-1)
    assert ran >= 10 and families == {"F8", "F8S", "F8W", "F8R"}
    y = nm.nm_conv2d_res(xd, wp, rd, bd, layer.stride, layer.pad, layer.dil, relu)    # the untuned default
    torch.cuda.synchronize()
    assert norm_err(y.float().cpu().numpy(), ref) <= BF16_TOL


def _ids():
    return [f"{R50.index(l):03d}_{l.name}" for l in wl.unique_shapes(R50) if l.Cin % 64 == 0]


@pytest.mark.parametrize("layer", [l for l in wl.unique_shapes(R50) if l.Cin % 64 == 0], ids=_ids())
def test_fp8_resnet50_batch64(layer):
    """Every pruned shape of the ResNet-50 stack at batch 64 through the tuned fp8 variant (the
    first layer, 3 input channels, is not an fp8 layer); every output of images 0, 1, 32, 63."""
    import torch
    i = R50.index(layer)
    _, w, bias = wl.make_tensors(layer, 64, 4000 + i, with_input=False)
    xd, x = _fp8_input((64, layer.H, layer.W, layer.Cin), 4000 + i)
    _, wq, s = _oracle_weights(layer, w)
    wp = nm.nm_prune(w, layer.n, layer.m, layer.tile, nm.NM_F8E4M3)
    v, ms = nm.nm_autotune(nm.NM_F8E4M3, 64, layer.H, layer.W, layer.Cin, wp, True, layer.stride, layer.pad,
                           layer.dil, True)
    say(f"fp8 batch 64 layer {i} {layer.name}: {nm.nm_variant_name(v)} {ms * 1e3:.1f} us, scale 2^{int(np.log2(s))}")
    y = nm.nm_conv2d(xd, wp, torch.from_numpy(bias).cuda(), layer.stride, layer.pad, layer.dil, True)
    torch.cuda.synchronize()
    assert nm.nm_last_variant() == v
    images = [0, 1, 32, 63]
    ref = oracle.conv2d(x[images], wq, bias, layer.stride, layer.pad, layer.dil, True, out_bf16=True)
    got = y[torch.tensor(images, device=y.device)].float().cpu().numpy()
    for n_, b in enumerate(images):
        assert norm_err(got[n_], ref[n_]) <= BF16_TOL, f"image {b}"


def test_fp8_argument_errors():
    import torch
    layer = L("f8_err", 6, 6, 64, 16, 3, 3, 1, 1, 1, 2, 4, 16)
    _, w, _ = wl.make_tensors(layer, 1, 3, with_input=False)
    with pytest.raises(nm.NMError) as e:                         # 48 channels: no 64-channel k-steps
        nm.nm_prune(np.ones((16, 1, 1, 48), dtype=np.float32), 2, 4, 16, nm.NM_F8E4M3)
    assert e.value.code == nm.NM_ERR_UNSUPPORTED
    wp8 = nm.nm_prune(w, 2, 4, 16, nm.NM_F8E4M3)
    wp16 = nm.nm_prune(w, 2, 4, 16, nm.NM_BF16)
    x8, _ = _fp8_input((1, 6, 6, 64), 1)
    with pytest.raises(nm.NMError) as e:                         # E4M3 tensors need E4M3 weights
        nm.nm_conv2d(x8, wp16)
    assert e.value.code == nm.NM_ERR_UNSUPPORTED
    with pytest.raises(nm.NMError) as e:                         # and E4M3 weights need E4M3 tensors
        nm.nm_conv2d(x8.float().to(torch.bfloat16), wp8)
    assert e.value.code == nm.NM_ERR_UNSUPPORTED
    with pytest.raises(nm.NMError) as e:                         # the output of the fp8 path is bf16
        nm.nm_conv2d(x8, wp8, None, 1, 1, 1, False, y=torch.empty((1, 6, 6, 16), device="cuda", dtype=torch.float32))
    assert e.value.code == nm.NM_ERR_UNSUPPORTED
