"""nm_conv2d on the GPU against the CPU oracle, element by element, through the
C ABI.  fp32: |err| <= 1e-4 * (1 + |ref|).  bf16: 2e-2 * (1 + |ref|)."""
import numpy as np
import pytest

from paper_2507_17301_amd import binding as nm
from paper_2507_17301_amd import workloads as wl
from gpu_util import FP32_TOL, BF16_TOL, say, norm_err, gpu_conv, oracle_conv

pytestmark = pytest.mark.gpu

L = wl.ConvLayer

# name, H, W, Cin, Cout, Kh, Kw, stride, pad, dil, n, m, tile   (+ batch)
GRID = [
    (L("3x3_s1", 14, 14, 32, 64, 3, 3, 1, 1, 1, 2, 4, 16), 3),
    (L("3x3_s2_odd", 15, 13, 32, 48, 3, 3, 2, 1, 1, 2, 4, 16), 2),
    (L("1x1", 9, 11, 64, 96, 1, 1, 1, 0, 1, 2, 4, 16), 2),
    (L("1x1_s2", 10, 10, 32, 32, 1, 1, 2, 0, 1, 1, 4, 16), 3),
    (L("3x3_dil2", 12, 12, 16, 32, 3, 3, 1, 2, 2, 2, 4, 16), 1),
    (L("3x3_pad0", 12, 10, 16, 16, 3, 3, 1, 0, 1, 4, 8, 16), 2),
    (L("5x3_pad3", 9, 9, 8, 24, 5, 3, 1, 3, 1, 2, 8, 16), 1),
    (L("T8", 10, 10, 32, 40, 3, 3, 1, 1, 1, 2, 4, 8), 2),
    (L("T32", 10, 10, 32, 96, 3, 3, 1, 1, 1, 1, 8, 32), 2),
    (L("T32_ragged", 7, 7, 64, 80, 1, 1, 1, 0, 1, 2, 8, 32), 5),
    (L("T5_cout37", 8, 8, 16, 37, 3, 3, 1, 1, 1, 2, 4, 5), 2),
    (L("T1_rowwise", 6, 6, 16, 20, 3, 3, 1, 1, 1, 2, 4, 1), 1),
    (L("cin48_partial_chunk", 8, 8, 48, 32, 3, 3, 1, 1, 1, 2, 4, 16), 2),
    (L("cin6_flat", 9, 9, 6, 16, 3, 3, 1, 1, 1, 1, 2, 16), 2),
    (L("stem_small", 30, 30, 3, 64, 7, 7, 2, 3, 1, 1, 1, 16), 2),
    (L("dense_cin32", 8, 8, 32, 32, 3, 3, 1, 1, 1, 1, 1, 16), 2),
    (L("M_is_cin", 8, 8, 64, 32, 3, 3, 1, 1, 1, 16, 64, 16), 2),
    (L("one_pixel", 3, 3, 16, 16, 3, 3, 1, 0, 1, 2, 4, 16), 1),
    # output tiles with a ragged last column tile: 4 and 8 live channels of 16, and a channel count
    # whose bf16 pixel rows are not 16-byte aligned (direct stores instead of the LDS output tile)
    (L("cout20_T16", 11, 9, 32, 20, 3, 3, 1, 1, 1, 2, 4, 16), 3),
    (L("cout24_T16", 11, 9, 64, 24, 1, 1, 1, 0, 1, 2, 4, 16), 3),
    (L("cout36_T16", 9, 11, 64, 36, 3, 3, 1, 1, 1, 2, 4, 16), 2),
]


@pytest.mark.parametrize("layer,batch", GRID, ids=[g[0].name for g in GRID])
def test_shape_grid_fp32(layer, batch):
    say(f"grid fp32 {layer} batch={batch}")
    x, w, bias = wl.make_tensors(layer, batch, 100 + batch, weight_sigma=0.1)
    _, got = gpu_conv(layer, x, w, bias, relu=True)
    ref = oracle_conv(layer, x, w, bias, relu=True)
    assert got.shape == ref.shape
    assert norm_err(got, ref) <= FP32_TOL
    _, got = gpu_conv(layer, x, w, bias, relu=False, use_bias=False)
    ref = oracle_conv(layer, x, w, bias, relu=False, use_bias=False)
    assert norm_err(got, ref) <= FP32_TOL


@pytest.mark.parametrize("layer,batch", GRID[:4] + GRID[7:10] + GRID[14:15] + GRID[18:],
                         ids=[g[0].name for g in GRID[:4] + GRID[7:10] + GRID[14:15] + GRID[18:]])
def test_shape_grid_bf16(layer, batch):
    say(f"grid bf16 {layer} batch={batch}")
    x, w, bias = wl.make_tensors(layer, batch, 200 + batch, weight_sigma=0.1)
    _, got = gpu_conv(layer, x, w, bias, relu=True, bf16=True)
    ref = oracle_conv(layer, x, w, bias, relu=True, bf16=True)
    assert norm_err(got, ref) <= BF16_TOL


def test_every_variant_in_turn():
    """Each kernel variant that is legal for the layer, forced, on a layer that
    spans several pixel tiles with a ragged tail (P = 2*19*17 = 646) and more
    row blocks than one workgroup covers (Cout = 272 = 17 row blocks)."""
    layer = L("variants", 19, 17, 64, 272, 3, 3, 1, 1, 1, 2, 4, 16)
    x, w, bias = wl.make_tensors(layer, 2, 7, weight_sigma=0.1)
    ref = oracle_conv(layer, x, w, bias, relu=True)
    import torch
    wp = nm.nm_prune(w, layer.n, layer.m, layer.tile)
    xd = torch.from_numpy(x).cuda()
    bd = torch.from_numpy(bias).cuda()
    ran = 0
    try:
        for v in range(nm.nm_variant_count()):
            if not nm.nm_variant_legal(v, wp):
                continue
            say(f"forced variant {v} {nm.nm_variant_name(v)}")
            nm.nm_force_variant(v)
            y = nm.nm_conv2d(xd, wp, bd, 1, 1, 1, True)
            torch.cuda.synchronize()
            assert norm_err(y.cpu().numpy(), ref) <= FP32_TOL, nm.nm_variant_name(v)
            ran += 1
    finally:
        nm.nm_force_variant(-1)
    assert ran >= 9


# the last four have groups wider than a chunk (M = Cin, M = the whole row, few kept columns so
# that some chunks of a tile hold none): the kept columns are spread unevenly over the chunks
@pytest.mark.parametrize("n,m,tile", [(1, 8, 32), (1, 4, 8), (4, 8, 16), (1, 1, 16),
                                      (64, 128, 16), (32, 128, 32), (576, 1152, 16), (8, 128, 16)])
def test_every_variant_other_sparsities(n, m, tile):
    layer = L("variants2", 9, 9, 128, 64, 3, 3, 2, 1, 1, n, m, tile)
    x, w, bias = wl.make_tensors(layer, 6, 8, weight_sigma=0.1)
    ref = oracle_conv(layer, x, w, bias, relu=False)
    import torch
    wp = nm.nm_prune(w, n, m, tile)
    xd = torch.from_numpy(x).cuda()
    bd = torch.from_numpy(bias).cuda()
    ran = var_ran = 0
    try:
        for v in range(nm.nm_variant_count()):
            if not nm.nm_variant_legal(v, wp):
                continue
            say(f"forced variant {v} {nm.nm_variant_name(v)} {n}:{m} T={tile}")
            nm.nm_force_variant(v)
            y = nm.nm_conv2d(xd, wp, bd, 2, 1, 1, False)
            torch.cuda.synchronize()
            assert norm_err(y.cpu().numpy(), ref) <= FP32_TOL, nm.nm_variant_name(v)
            ran += 1
            var_ran += nm.nm_variant_name(v).startswith("VAR_")
    finally:
        nm.nm_force_variant(-1)
    assert ran >= 9
    assert (var_ran > 0) == (m >= 128)   # the variable-step form exists exactly where it pays


@pytest.mark.parametrize("n,m,tile,cin,ksize", [
    (2, 4, 16, 64, 3), (2, 8, 32, 128, 3), (1, 4, 32, 64, 3), (4, 8, 8, 64, 3), (1, 1, 16, 32, 3),
    (2, 4, 16, 40, 3), (2, 4, 16, 256, 3), (1, 8, 16, 128, 3), (1, 1, 16, 64, 3), (6, 8, 32, 64, 3),
    (2, 4, 16, 256, 1), (1, 4, 32, 512, 1)])   # 1x1: K loops of one or two chunks, which need less LDS
def test_every_variant_bf16(n, m, tile, cin, ksize):
    """bf16 tensors: every legal variant, i.e. the fp32-MFMA kernels on bf16 data, the
    bf16 matrix-core gather kernels (T = 32 also with the shared operand) and, where
    the channel count is a multiple of 64, the gather-free kernels (sparse matrix
    instruction for N <= 2 of M % 4 == 0, dense instruction on zero-filled weights
    for everything), forced in turn."""
    layer = L("variants_bf16", 11, 9, cin, 80, ksize, ksize, 1, ksize // 2, 1, n, m, tile)
    x, w, bias = wl.make_tensors(layer, 3, 9, weight_sigma=0.1)
    ref = oracle_conv(layer, x, w, bias, relu=True, bf16=True)
    import torch
    wp = nm.nm_prune(w, n, m, tile, nm.NM_BF16)
    xd = torch.from_numpy(x).cuda().to(torch.bfloat16)
    bd = torch.from_numpy(bias).cuda()
    ran = ran16 = ran_sp = ran_dn = ran_pw = ran_pr = 0
    try:
        for v in range(nm.nm_variant_count()):
            if not nm.nm_variant_legal(v, wp, nm.NM_BF16, nm.NM_BF16):
                continue
            say(f"forced bf16 variant {v} {nm.nm_variant_name(v)} {n}:{m} T={tile} cin={cin} k={ksize}")
            nm.nm_force_variant(v)
            y = nm.nm_conv2d(xd, wp, bd, layer.stride, layer.pad, layer.dil, True)
            torch.cuda.synchronize()
            assert norm_err(y.float().cpu().numpy(), ref) <= BF16_TOL, nm.nm_variant_name(v)
            ran += 1
            ran16 += nm.nm_variant_name(v).startswith("B16")
            ran_sp += nm.nm_variant_name(v).startswith("SP1")
            ran_dn += nm.nm_variant_name(v).startswith("SP0")
            ran_pw += nm.nm_variant_name(v).startswith("SPW")   # the same kernels with producer wavefronts
            ran_pr += nm.nm_variant_name(v).startswith("SPR")   # ... and the weights loaded straight into registers
    finally:
        nm.nm_force_variant(-1)
    assert ran >= 9 and ran16 >= 5
    if cin % 64 == 0:
        assert ran_dn >= 14 and ran_pw >= 8 and ran_pr >= 6
        assert (ran_sp >= 14) == (n <= 2 and m % 4 == 0)
    else:
        assert ran_sp == 0 and ran_dn == 0 and ran_pw == 0 and ran_pr == 0


# name, H, W, Cin, Cout, Kh, Kw, stride, pad, dil, n, m, tile  | batch | the kernel-row-run kernel applies
FEW_CHANNELS = [
    (L("stem_7x7_s2", 30, 30, 3, 64, 7, 7, 2, 3, 1, 1, 1, 16), 3, True),      # runs start one element early
    (L("c3_3x3_s2", 17, 18, 3, 40, 3, 3, 2, 1, 1, 1, 1, 16), 2, True),
    (L("c3_5x5_s2_p2", 16, 16, 3, 32, 5, 5, 2, 2, 1, 1, 1, 16), 3, True),     # even padding: no lead-in
    (L("c4_3x3_s1_2of4", 9, 10, 4, 48, 3, 3, 1, 1, 1, 2, 4, 16), 2, True),    # pruned, stride 1
    (L("c2_7x7_s1", 12, 12, 2, 16, 7, 7, 1, 3, 1, 1, 1, 16), 2, True),
    (L("c1_3x3_s2", 10, 12, 1, 20, 3, 3, 2, 1, 1, 1, 1, 16), 2, True),
    (L("c4_7x7_s1_four_ksteps", 10, 10, 4, 16, 7, 7, 1, 3, 1, 1, 1, 16), 2, True),
    (L("c3_3x3_pad0_T32", 11, 12, 3, 70, 3, 3, 2, 0, 1, 1, 1, 32), 2, True),
    (L("c3_odd_width", 15, 15, 3, 32, 3, 3, 2, 1, 1, 1, 1, 16), 2, False),    # W*Cin odd: rows not 4-byte aligned
    (L("c3_s1", 12, 12, 3, 32, 3, 3, 1, 1, 1, 1, 1, 16), 2, False),           # stride*Cin odd
    (L("c4_dil2", 12, 12, 4, 32, 3, 3, 1, 2, 2, 1, 1, 16), 2, False),         # dilated columns are not one run
]


@pytest.mark.parametrize("layer,batch,applies", FEW_CHANNELS, ids=[g[0].name for g in FEW_CHANNELS])
def test_few_input_channels_bf16(layer, batch, applies):
    """Layers with very few input channels in bf16: the kernel that fetches whole kernel
    rows as contiguous runs, every shape of it forced in turn, where the geometry allows
    it; an error (never a wrong answer) where it does not; and the default choice."""
    import torch
    x, w, bias = wl.make_tensors(layer, batch, 31, weight_sigma=0.2)
    ref = oracle_conv(layer, x, w, bias, relu=True, bf16=True)
    wp = nm.nm_prune(w, layer.n, layer.m, layer.tile, nm.NM_BF16)
    xd = torch.from_numpy(x).cuda().to(torch.bfloat16)
    bd = torch.from_numpy(bias).cuda()
    ran = refused = 0
    try:
        for v in range(nm.nm_variant_count()):
            name = nm.nm_variant_name(v)
            if not name.startswith("RUN") or not nm.nm_variant_legal(v, wp, nm.NM_BF16, nm.NM_BF16):
                continue
            say(f"forced {name} on {layer.name}")
            nm.nm_force_variant(v)
            try:
                y = nm.nm_conv2d(xd, wp, bd, layer.stride, layer.pad, layer.dil, True)
            except nm.NMError as e:
                assert e.code == nm.NM_ERR_UNSUPPORTED
                refused += 1
                continue
            torch.cuda.synchronize()
            assert norm_err(y.float().cpu().numpy(), ref) <= BF16_TOL, name
            ran += 1
    finally:
        nm.nm_force_variant(-1)
    if applies:
        assert ran >= 5 and refused == 0
    else:
        assert ran == 0
    y = nm.nm_conv2d(xd, wp, bd, layer.stride, layer.pad, layer.dil, True)
    torch.cuda.synchronize()
    assert norm_err(y.float().cpu().numpy(), ref) <= BF16_TOL


def test_illegal_forced_variant_is_an_error_not_a_fallback():
    layer = L("flat_only", 6, 6, 6, 16, 3, 3, 1, 1, 1, 1, 2, 16)
    x, w, bias = wl.make_tensors(layer, 1, 3)
    import torch
    wp = nm.nm_prune(w, 1, 2, 16)
    illegal = [v for v in range(nm.nm_variant_count()) if not nm.nm_variant_legal(v, wp)]
    assert illegal
    nm.nm_force_variant(illegal[0])
    try:
        with pytest.raises(nm.NMError) as e:
            nm.nm_conv2d(torch.from_numpy(x).cuda(), wp, None, 1, 1, 1, False)
        assert e.value.code == -3
    finally:
        nm.nm_force_variant(-1)


def test_argument_errors():
    import torch
    layer = L("err", 6, 6, 8, 16, 3, 3, 1, 1, 1, 2, 4, 16)
    x, w, bias = wl.make_tensors(layer, 1, 3)
    wp = nm.nm_prune(w, 2, 4, 16)
    xd = torch.from_numpy(x).cuda()
    with pytest.raises(nm.NMError) as e:      # kernel larger than padded input
        nm.nm_conv2d(torch.zeros(1, 1, 1, 8, device="cuda"), wp, None, 1, 0, 1, False,
                     y=torch.zeros(1, 1, 1, 16, device="cuda"))
    assert e.value.code == -2
    with pytest.raises(nm.NMError) as e:      # channel mismatch
        nm.nm_conv2d(torch.zeros(1, 6, 6, 4, device="cuda"), wp, None, 1, 1, 1, False)
    assert e.value.code == -1
    with pytest.raises(nm.NMError) as e:      # mixed dtypes are not provided
        nm.nm_conv2d(xd, wp, None, 1, 1, 1, False,
                     y=torch.zeros(1, 6, 6, 16, device="cuda", dtype=torch.bfloat16))
    assert e.value.code == -3
    with pytest.raises(nm.NMError):           # stride 0
        nm.nm_conv2d(xd, wp, None, 0, 1, 1, False, y=torch.zeros(1, 6, 6, 16, device="cuda"))
    with pytest.raises(ValueError):           # an output tensor of the wrong shape never reaches the kernel
        nm.nm_conv2d(xd, wp, None, 1, 1, 1, False, y=torch.zeros(1, 6, 6, 8, device="cuda"))
    with pytest.raises(ValueError):
        nm.nm_conv2d(xd, wp, None, 1, 1, 1, False, y=torch.zeros(1, 6, 12, 16, device="cuda")[:, :, ::2])


def test_config1_single_layer():
    """56x56x64 -> 64, 3x3, 2:4, T = 16, batch 1, weights N(0, 0.05), seed 0."""
    layer = wl.single_conv_config1()
    say(f"config 1 {layer}")
    x, w, bias = wl.make_tensors(layer, 1, 0, weight_sigma=0.05)
    wp, got = gpu_conv(layer, x, w, bias, relu=True)
    ref = oracle_conv(layer, x, w, bias, relu=True)
    assert norm_err(got, ref) <= FP32_TOL
    # the packed format holds exactly N of every M columns per tile
    mask = nm.nm_packed_mask(wp)
    assert np.all(mask.reshape(64, -1, 4).sum(axis=2) == 2)


@pytest.mark.parametrize("cell", list(range(15)))
def test_config2_sweep_cell(cell):
    """14x14x256 -> 256, batch 32, N:M x T sweep; full output against the oracle
    for a 4-image slice, sampled outputs over the whole batch."""
    layer = wl.sweep_config2()[cell]
    say(f"config 2 cell {cell} {layer.name}")
    x, w, bias = wl.make_tensors(layer, 32, cell, weight_sigma=0.05)
    _, got = gpu_conv(layer, x, w, bias, relu=True)
    pts = wl.sample_points(layer, 32, 3000, cell)
    ref = oracle_conv(layer, x, w, bias, relu=True, pts=pts)
    assert norm_err(got[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]], ref) <= FP32_TOL
    sl = [0, 13, 31]
    ref_full = oracle_conv(layer, x[sl], w, bias, relu=True)
    assert norm_err(got[sl], ref_full) <= FP32_TOL
