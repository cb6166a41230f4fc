"""The benchmark configurations at their full sizes, in the launch configuration
bench.py times (per-layer tuned variant), against the CPU oracle.

Every unique layer shape of every configuration runs at its full batch through
the tuned variant.  Configurations 3 and 4 (both dtypes) are compared on the
whole batch, every output; configuration 5 (batch 256) on every output of the
images {0, 1, B/2, B-1} -- images are independent, but pixel tiles cross image
boundaries, hence the first, the last and the middle of the batch.
"""
import dataclasses
import re

import numpy as np
import pytest

import oracle

from paper_2507_17301_amd import binding as nm
from paper_2507_17301_amd import workloads as wl
from gpu_util import FP32_TOL, BF16_TOL, say, norm_err, oracle_conv

pytestmark = pytest.mark.gpu

R18 = wl.resnet18_stack()
R50 = wl.resnet50_stack()
R101 = wl.resnet101_stack()


def _ids(stack):
    return [f"{stack.index(l):03d}_{l.name}" for l in wl.unique_shapes(stack)]


def _run_tuned(layer, batch, x, w, bias, bf16):
    import torch
    ndt = nm.NM_BF16 if bf16 else nm.NM_F32
    wp = nm.nm_prune(w, layer.n, layer.m, layer.tile, ndt)
    v, ms = nm.nm_autotune(ndt, batch, layer.H, layer.W, layer.Cin, wp, True,
                           layer.stride, layer.pad, layer.dil, True)
    xd = torch.from_numpy(x).cuda()
    if bf16:
        xd = xd.to(torch.bfloat16)
    y = nm.nm_conv2d(xd, wp, torch.from_numpy(bias).cuda(), layer.stride, layer.pad, layer.dil, True)
    torch.cuda.synchronize()
    return y, nm.nm_variant_name(v)


def _check_images(layer, batch, seed, bf16, images=None):
    """The layer at its full batch through the tuned variant; every output of the
    listed images (None = the whole batch) against the oracle."""
    x, w, bias = wl.make_tensors(layer, batch, seed)
    y, vname = _run_tuned(layer, batch, x, w, bias, bf16)
    tol = BF16_TOL if bf16 else FP32_TOL
    if images is None:
        images = list(range(batch))
    images = sorted(set(images))
    ref = oracle_conv(layer, x[images], w, bias, relu=True, bf16=bf16)
    import torch
    got = y[torch.tensor(images, device=y.device)].float().cpu().numpy()
    assert got.shape == ref.shape
    for n, b in enumerate(images):
        err = norm_err(got[n], ref[n])
        assert err <= tol, f"{layer.name} {vname} image {b}: {err}"
    return x, w, bias, y


def _check_sampled(layer, batch, seed, bf16, npts=2000):
    x, w, bias = wl.make_tensors(layer, batch, seed)
    y, vname = _run_tuned(layer, batch, x, w, bias, bf16)
    pts = wl.sample_points(layer, batch, npts, seed)
    import torch
    idx = torch.from_numpy(pts.astype(np.int64)).cuda()
    got = y[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].float().cpu().numpy()
    ref = oracle_conv(layer, x, w, bias, relu=True, bf16=bf16, pts=pts)
    err = norm_err(got, ref)
    assert err <= (BF16_TOL if bf16 else FP32_TOL), f"{layer.name} {vname}: {err}"
    return x, w, bias, y


def test_config3_resnet18_batch1_full():
    for i, layer in enumerate(R18):
        say(f"config 3 batch 1 layer {i} {layer.name}")
        x, w, bias = wl.make_tensors(layer, 1, 3000 + i)
        y, vname = _run_tuned(layer, 1, x, w, bias, False)
        ref = oracle_conv(layer, x, w, bias, relu=True)
        assert norm_err(y.cpu().numpy(), ref) <= FP32_TOL, f"{layer.name} {vname}"


@pytest.mark.parametrize("layer", wl.unique_shapes(R18), ids=_ids(R18))
def test_config3_resnet18_batch32_whole_batch(layer):
    i = R18.index(layer)
    say(f"config 3 fp32 batch 32 layer {i} {layer.name}, every output")
    _check_images(layer, 32, 3000 + i, False)


@pytest.mark.parametrize("layer", wl.unique_shapes(R50), ids=_ids(R50))
def test_config4_resnet50_batch64_fp32_whole_batch(layer):
    i = R50.index(layer)
    say(f"config 4 fp32 batch 64 layer {i} {layer.name}, every output")
    _check_images(layer, 64, 4000 + i, False)


@pytest.mark.parametrize("layer", wl.unique_shapes(R50), ids=_ids(R50))
def test_config4_resnet50_batch64_bf16_whole_batch(layer):
    i = R50.index(layer)
    say(f"config 4 bf16 batch 64 layer {i} {layer.name}, every output")
    _check_images(layer, 64, 4000 + i, True)


@pytest.mark.parametrize("bf16", [False, True], ids=["fp32", "bf16"])
def test_config4_resnet50_batch64_untuned_default(bf16):
    """What a caller gets without tuning: with the cache empty, every unique shape of the stack runs
    the library's default variant at the full batch; every output of images 0 and 63."""
    import torch
    nm.nm_cache_clear()
    tol = BF16_TOL if bf16 else FP32_TOL
    ndt = nm.NM_BF16 if bf16 else nm.NM_F32
    picks = set()
    for layer in wl.unique_shapes(R50):
        i = R50.index(layer)
        x, w, bias = wl.make_tensors(layer, 64, 4000 + i)
        wp = nm.nm_prune(w, layer.n, layer.m, layer.tile, ndt)
        xd = torch.from_numpy(x).cuda()
        if bf16:
            xd = xd.to(torch.bfloat16)
        say(f"config 4 {'bf16' if bf16 else 'fp32'} batch 64 layer {i} {layer.name}, untuned default")
        y = nm.nm_conv2d(xd, wp, torch.from_numpy(bias).cuda(), layer.stride, layer.pad, layer.dil, True)
        torch.cuda.synchronize()
        vname = nm.nm_variant_name(nm.nm_last_variant())
        assert not re.search(r"_S\d+$", vname)   # the default never needs the K-split workspace
        picks.add(vname.split("_")[0])
        ref = oracle_conv(layer, x[[0, 63]], w, bias, relu=True, bf16=bf16)
        got = y[torch.tensor([0, 63], device=y.device)].float().cpu().numpy()
        for n_, b in enumerate((0, 63)):
            assert norm_err(got[n_], ref[n_]) <= tol, f"{layer.name} {vname} image {b}"
    if bf16:   # the gather-free kernels (and the kernel-row-run kernel for the first layer), not the fp32 path on bf16 data
        assert picks <= {"SP1", "SPW1", "SPR1", "RUN"}, picks


def test_config4_resnet50_batch64_large_groups():
    """Section 3.1's adaptive setting at full size: one group per kernel tap (M = Cin, half
    kept) and one group per row of the weight matrix (M = K), tuned launch configuration,
    both tensor types; every output of the first two, the middle and the last image."""
    names = ("s2b1_conv2_3x3", "s3b1_conv1_1x1", "s4b1_conv3_1x1")
    picked = [l for l in R50 if l.name in names]
    assert len(picked) == len(names)
    for mode in ("cin", "row"):
        for layer in wl.with_large_groups(picked, mode):
            if mode == "row" and layer.K > 16384:
                continue   # beyond the group size the library accepts
            i = [l.name for l in R50].index(layer.name)
            for bf16 in (False, True):
                say(f"config 4 {'bf16' if bf16 else 'fp32'} batch 64 groups per {mode} layer {i} "
                    f"{layer.name} {layer.n}:{layer.m}")
                _check_images(layer, 64, 4100 + i, bf16, images=(0, 1, 32, 63))


@pytest.mark.parametrize("layer", wl.unique_shapes(R101), ids=_ids(R101))
def test_config5_resnet101_batch256_bf16_mixed_sparsity(layer):
    """T = 32, stage 1 1:4, stage 2 2:4, stage 3 2:8, stage 4 4:8, bf16 in/out, fp32
    accumulation, full batch of 256; every output of images 0, 1, 128 and 255."""
    i = R101.index(layer)
    say(f"config 5 bf16 batch 256 layer {i} {layer.name} {layer.n}:{layer.m} T={layer.tile}")
    _check_images(layer, 256, 5000 + i, True, images=(0, 1, 128, 255))


def test_tuning_cache_round_trip(tmp_path):
    layer = wl.ConvLayer("cache", 14, 14, 64, 64, 3, 3, 1, 1, 1, 2, 4, 16)
    x, w, bias = wl.make_tensors(layer, 4, 1)
    wp = nm.nm_prune(w, 2, 4, 16)
    nm.nm_cache_clear()
    v, ms = nm.nm_autotune(nm.NM_F32, 4, 14, 14, 64, wp, True, 1, 1, 1, True)
    assert nm.nm_cache_size() == 1 and ms > 0
    path = str(tmp_path / "tune.txt")
    nm.nm_cache_save(path)
    nm.nm_cache_clear()
    assert nm.nm_cache_size() == 0
    nm.nm_cache_load(path)
    assert nm.nm_cache_size() == 1
    v2, ms2 = nm.nm_autotune(nm.NM_F32, 4, 14, 14, 64, wp, True, 1, 1, 1, True)   # served from the cache
    assert v2 == v and abs(ms2 - ms) < 1e-6
    # the first line of the file names the device the timings were taken on
    head = open(path).readline().split()
    assert head[:2] == ["nmconv-cache", "2"] and len(head) == 5 and "CU" in head[4]
    # what nm_conv2d launches for the tuned shape is the cached variant
    import torch
    y = nm.nm_conv2d(torch.from_numpy(x).cuda(), wp, torch.from_numpy(bias).cuda(), 1, 1, 1, True)
    torch.cuda.synchronize()
    assert nm.nm_last_variant() == v
    # bias and activation flags are part of the key: the same shape without them is a new entry
    nm.nm_autotune(nm.NM_F32, 4, 14, 14, 64, wp, False, 1, 1, 1, False)
    assert nm.nm_cache_size() == 2
    # and so are the operand tables of the handle: with one group per tap (M = Cin = 64, a
    # quarter kept), kept columns crowded into the first 16 channels need twice the k-steps
    # per 32-channel chunk that kept columns spread evenly (every fourth channel) need
    crowded, spread = w.copy(), w.copy()
    crowded[:, :, :, :16] *= 1000.0
    spread[:, :, :, ::4] *= 1000.0
    wp_c, wp_s = nm.nm_prune(crowded, 16, 64, 16), nm.nm_prune(spread, 16, 64, 16)
    nm.nm_autotune(nm.NM_F32, 4, 14, 14, 64, wp_c, True, 1, 1, 1, True)
    n_before = nm.nm_cache_size()
    vs, _ = nm.nm_autotune(nm.NM_F32, 4, 14, 14, 64, wp_s, True, 1, 1, 1, True)
    assert nm.nm_cache_size() == n_before + 1
    assert nm.nm_variant_legal(vs, wp_s)
    with pytest.raises(nm.NMError):
        nm.nm_cache_load(str(tmp_path / "missing.txt"))


def test_tuner_chooses_the_tile_size():
    """nm_autotune_tile: every candidate T is pruned and tuned, the fastest handle
    comes back, its masks are the oracle's at that T and it convolves like the oracle."""
    import torch
    layer = wl.ConvLayer("tile_choice", 14, 14, 64, 96, 3, 3, 1, 1, 1, 2, 4, 16)
    x, w, bias = wl.make_tensors(layer, 4, 77, weight_sigma=0.1)
    tiles = [8, 16, 32]
    say(f"autotune over tiles {tiles} {layer}")
    wp, best, ms = nm.nm_autotune_tile(w, layer.n, layer.m, tiles, nm.NM_F32, 4, layer.H, layer.W,
                                       True, layer.stride, layer.pad, layer.dil, True)
    assert best in tiles and wp.tile == best
    assert len(ms) == 3 and all(t > 0 for t in ms)
    assert ms[tiles.index(best)] == min(ms)
    mask_ref, _, _ = oracle.prune(w, layer.n, layer.m, best)
    assert np.array_equal(nm.nm_packed_mask(wp), mask_ref)
    y = nm.nm_conv2d(torch.from_numpy(x).cuda(), wp, torch.from_numpy(bias).cuda(),
                     layer.stride, layer.pad, layer.dil, True)
    torch.cuda.synchronize()
    chosen = dataclasses.replace(layer, tile=best)
    ref = oracle_conv(chosen, x, w, bias, relu=True)
    assert norm_err(y.cpu().numpy(), ref) <= FP32_TOL
    # errors of a candidate fail the whole call: tile 0 is not a tile
    with pytest.raises(nm.NMError):
        nm.nm_autotune_tile(w, layer.n, layer.m, [16, 0], nm.NM_F32, 4, layer.H, layer.W)
