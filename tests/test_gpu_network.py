"""Residual convolution and pooling on the GPU against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

import oracle
from paper_2507_17301_amd import binding as nm
from paper_2507_17301_amd import workloads as wl
from gpu_util import FP32_TOL, BF16_TOL, say, norm_err

pytestmark = pytest.mark.gpu

L = wl.ConvLayer


def _residual_case(layer, batch, bf16, seed, forced_prefixes=None):
    import torch
    x, w, bias = wl.make_tensors(layer, batch, seed, weight_sigma=0.1)
    _, _, wz = oracle.prune(w, layer.n, layer.m, layer.tile)
    rng = np.random.default_rng(seed + 1)
    shape = (batch, layer.Ho, layer.Wo, layer.Cout)
    res = rng.standard_normal(shape).astype(np.float32)
    xo, ro = x, res
    if bf16:
        wz, xo, ro = oracle.round_bf16(wz), oracle.round_bf16(x), oracle.round_bf16(res)
    ref = oracle.conv2d_res(xo, wz, ro, bias, layer.stride, layer.pad, layer.dil, True, out_bf16=bf16)
    tdt = torch.bfloat16 if bf16 else torch.float32
    ndt = nm.NM_BF16 if bf16 else nm.NM_F32
    wp = nm.nm_prune(w, layer.n, layer.m, layer.tile, ndt)
    xd = torch.from_numpy(x).cuda().to(tdt)
    rd = torch.from_numpy(res).cuda().to(tdt)
    bd = torch.from_numpy(bias).cuda()
    tol = BF16_TOL if bf16 else FP32_TOL
    y = nm.nm_conv2d_res(xd, wp, rd, bd, layer.stride, layer.pad, layer.dil, True)
    torch.cuda.synchronize()
    assert norm_err(y.float().cpu().numpy(), ref) <= tol
    # residual = None is plain nm_conv2d
    y0 = nm.nm_conv2d_res(xd, wp, None, bd, layer.stride, layer.pad, layer.dil, True)
    y1 = nm.nm_conv2d(xd, wp, bd, layer.stride, layer.pad, layer.dil, True)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    if forced_prefixes:
        seen = set()
        try:
            for v in range(nm.nm_variant_count()):
                name = nm.nm_variant_name(v)
                fam = name.split("_")[0]
                if fam not in forced_prefixes or fam in seen or not nm.nm_variant_legal(v, wp, ndt, ndt):
                    continue
                say(f"residual, forced {name} on {layer.name}")
                nm.nm_force_variant(v)
                y = nm.nm_conv2d_res(xd, wp, rd, bd, layer.stride, layer.pad, layer.dil, True)
                torch.cuda.synchronize()
                assert norm_err(y.float().cpu().numpy(), ref) <= tol, name
                seen.add(fam)
        finally:
            nm.nm_force_variant(-1)
        assert seen == set(forced_prefixes)


def test_residual_fp32():
    _residual_case(L("res_3x3", 13, 11, 32, 48, 3, 3, 1, 1, 1, 2, 4, 16), 2, False, 50, {"NB4", "NB8"})
    _residual_case(L("res_1x1_cout37", 9, 9, 16, 37, 1, 1, 1, 0, 1, 2, 4, 5), 2, False, 51)   # element-wise tail


def test_residual_bf16_every_kernel_family():
    # 64 channels, 2:4: fp32-MFMA kernel on bf16 data, gather kernel, sparse and dense instruction, both also with producer wavefronts
    _residual_case(L("res16_3x3", 12, 10, 64, 80, 3, 3, 1, 1, 1, 2, 4, 16), 3, True, 52, {"NB4", "B16", "SP1", "SP0", "SPW1", "SPW0", "SPR1", "SPR0"})
    _residual_case(L("res16_stem", 20, 20, 3, 32, 7, 7, 2, 3, 1, 1, 1, 16), 2, True, 53, {"RUN"})
    _residual_case(L("res16_cout37", 9, 9, 64, 37, 1, 1, 1, 0, 1, 2, 4, 16), 2, True, 54)


def test_residual_argument_errors():
    import torch
    layer = L("res_err", 6, 6, 16, 16, 3, 3, 1, 1, 1, 2, 4, 16)
    x, w, bias = wl.make_tensors(layer, 1, 3)
    wp = nm.nm_prune(w, 2, 4, 16)
    xd = torch.from_numpy(x).cuda()
    y = torch.empty((1, 6, 6, 16), device="cuda")
    with pytest.raises(ValueError):
        nm.nm_conv2d_res(xd, wp, torch.empty((1, 6, 6, 8), device="cuda"))
    with pytest.raises(nm.NMError) as e:                       # residual overlapping the output
        nm.nm_conv2d_res(xd, wp, y, None, 1, 1, 1, True, y=y)
    assert e.value.code == nm.NM_ERR_ARG


@pytest.mark.parametrize("k,stride,pad,H,W,C", [(3, 2, 1, 112, 112, 64), (3, 2, 1, 11, 9, 5), (2, 2, 0, 8, 8, 4),
                                                 (3, 1, 1, 7, 6, 3), (5, 3, 2, 13, 12, 66)])
@pytest.mark.parametrize("bf16", [False, True])
def test_maxpool(k, stride, pad, H, W, C, bf16):
    import torch
    rng = np.random.default_rng(H + C)
    x = rng.standard_normal((2, H, W, C)).astype(np.float32)
    if bf16:
        x = oracle.round_bf16(x)
    ref = oracle.maxpool2d(x, k, stride, pad)
    xd = torch.from_numpy(x).cuda().to(torch.bfloat16 if bf16 else torch.float32)
    y = nm.nm_maxpool2d(xd, k, stride, pad)
    torch.cuda.synchronize()
    assert np.array_equal(y.float().cpu().numpy(), ref)        # a selection: bit-exact


@pytest.mark.parametrize("H,W,C,B", [(7, 7, 2048, 3), (1, 1, 5, 2), (5, 9, 100, 4)])
@pytest.mark.parametrize("bf16", [False, True])
def test_avgpool_global(H, W, C, B, bf16):
    import torch
    rng = np.random.default_rng(H * C)
    x = (rng.standard_normal((B, H, W, C)) + 0.5).astype(np.float32)
    if bf16:
        x = oracle.round_bf16(x)
    ref = oracle.avgpool_global(x, out_bf16=bf16)
    xd = torch.from_numpy(x).cuda().to(torch.bfloat16 if bf16 else torch.float32)
    y = nm.nm_avgpool_global(xd)
    torch.cuda.synchronize()
    assert norm_err(y.float().cpu().numpy(), ref) <= (BF16_TOL if bf16 else FP32_TOL)


def test_pool_argument_errors():
    import torch
    x = torch.zeros((1, 4, 4, 4), device="cuda")
    with pytest.raises(nm.NMError) as e:
        nm.nm_maxpool2d(x, 3, 2, 3)
    assert e.value.code == nm.NM_ERR_ARG
    with pytest.raises(nm.NMError) as e:
        nm.nm_maxpool2d(x, 7, 1, 1, y=torch.zeros((1, 1, 1, 4), device="cuda"))
    assert e.value.code == nm.NM_ERR_SHAPE


def _oracle_op(op, params, i, src, residual, bf16):
    """One operator of the network through the oracle, on the given input tensors."""
    rnd = oracle.round_bf16 if bf16 else (lambda a: a)
    if op.kind == "conv":
        l = op.layer
        w, b = params[i]
        _, _, wz = oracle.prune(w, l.n, l.m, l.tile)
        wz = rnd(wz)
        if residual is not None:
            return oracle.conv2d_res(src, wz, residual, b, l.stride, l.pad, l.dil, op.relu, out_bf16=bf16)
        return oracle.conv2d(src, wz, b, l.stride, l.pad, l.dil, op.relu, out_bf16=bf16)
    if op.kind == "maxpool":
        return oracle.maxpool2d(src, op.k, op.stride, op.pad)
    a = oracle.avgpool_global(src, out_bf16=bf16)
    return a.reshape(a.shape[0], 1, 1, a.shape[1])


@pytest.mark.parametrize("bottleneck", [True, False])
@pytest.mark.parametrize("bf16", [False, True])
def test_small_residual_network_end_to_end(bottleneck, bf16):
    """A two-stage ResNet of either block type on a 40x40 input, run end to end on the GPU;
    then every operator is checked on its own: the oracle is given the tensors the GPU
    operator actually read (its input and residual, exact as floats) and must reproduce
    the tensor the GPU wrote within the per-layer tolerance.  Errors of earlier layers
    therefore do not accumulate into the bound, and every tensor of the network is covered."""
    import torch
    from paper_2507_17301_amd.network import Network
    ops = wl.resnet_graph((1, 2), (16, 32), bottleneck, 40, [(2, 4), (1, 4)], 16, stem_width=16, num_classes=10)
    batch, seed0 = 2, 900
    rng = np.random.default_rng(77)
    x = rng.random((batch, 40, 40, 3), dtype=np.float32)
    net = Network(ops, batch, 40, nm.NM_BF16 if bf16 else nm.NM_F32, seed0)
    xd = torch.from_numpy(x).cuda().to(net.tdt)
    out = net.forward(xd)
    torch.cuda.synchronize()
    assert out.shape == (batch, 1, 1, 10)
    got = {k: t.float().cpu().numpy() for k, t in net.t.items()}
    params = {i: (w, b) for i, w, b in wl.net_parameters(ops, seed0)}
    tol = BF16_TOL if bf16 else FP32_TOL
    written = {0}
    for i, op in enumerate(ops):
        assert op.src in written and (op.residual < 0 or op.residual in written)
        res = got[op.residual] if op.residual >= 0 else None
        ref = _oracle_op(op, params, i, got[op.src], res, bf16)
        assert got[op.dst].shape == ref.shape
        if op.kind == "maxpool":
            assert np.array_equal(got[op.dst], ref), f"operator {i} (max pooling is a selection)"
        else:
            assert norm_err(got[op.dst], ref) <= tol, f"operator {i} {op.kind}"
        written.add(op.dst)
    assert written == set(net.t.keys())


@pytest.mark.parametrize("layer,batch", [(L("i2c_3x3", 13, 11, 32, 48, 3, 3, 1, 1, 1, 2, 4, 16), 2),
                                         (L("i2c_3x3_s2", 14, 14, 16, 32, 3, 3, 2, 1, 1, 2, 4, 16), 2),
                                         (L("i2c_7x7_c3", 20, 20, 3, 16, 7, 7, 2, 3, 1, 1, 1, 16), 2),
                                         (L("i2c_dil2", 10, 9, 8, 16, 3, 3, 1, 2, 2, 2, 4, 16), 1)])
@pytest.mark.parametrize("bf16", [False, True])
def test_im2col_and_the_unfused_pipeline(layer, batch, bf16):
    """nm_im2col is a copy (bit-exact against the oracle's); the unfused pipeline of the
    paper's ablation -- im2col to memory, then the same kept-column contraction as a 1x1
    convolution over it -- gives the fused kernel's result."""
    import torch
    x, w, bias = wl.make_tensors(layer, batch, 60, weight_sigma=0.1)
    rnd = oracle.round_bf16 if bf16 else (lambda a: a)
    tdt = torch.bfloat16 if bf16 else torch.float32
    ndt = nm.NM_BF16 if bf16 else nm.NM_F32
    xd = torch.from_numpy(x).cuda().to(tdt)
    a = nm.nm_im2col(xd, layer.Kh, layer.Kw, layer.stride, layer.pad, layer.dil)
    torch.cuda.synchronize()
    ref_a = oracle.im2col(rnd(x), layer.Kh, layer.Kw, layer.stride, layer.pad, layer.dil)
    assert np.array_equal(a.float().cpu().numpy(), ref_a)
    _, _, wz = oracle.prune(w, layer.n, layer.m, layer.tile)
    ref = oracle.conv2d(rnd(x), rnd(wz), bias, layer.stride, layer.pad, layer.dil, True, out_bf16=bf16)
    bd = torch.from_numpy(bias).cuda()
    wp1 = nm.nm_prune(np.ascontiguousarray(w.reshape(layer.Cout, 1, 1, -1)), layer.n, layer.m, layer.tile, ndt)
    y_unfused = nm.nm_conv2d(a, wp1, bd, 1, 0, 1, True)
    wp = nm.nm_prune(w, layer.n, layer.m, layer.tile, ndt)
    y_fused = nm.nm_conv2d(xd, wp, bd, layer.stride, layer.pad, layer.dil, True)
    torch.cuda.synchronize()
    tol = BF16_TOL if bf16 else FP32_TOL
    assert norm_err(y_unfused.float().cpu().numpy(), ref) <= tol
    assert norm_err(y_fused.float().cpu().numpy(), ref) <= tol
    assert np.array_equal(nm.nm_packed_indices(wp1), nm.nm_packed_indices(wp))   # same kept columns either way


def test_stream_floor_touches_exactly_its_ranges():
    """The measuring kernel: every 16-byte unit of y is overwritten, nothing beyond y's
    whole units is, x is left alone; sizes that are not multiples of the grid or of 16."""
    import torch
    for nx, ny in ((1 << 20, 3 << 18), (1000, 17), (16, 16 * 5000 + 8), (32, 4096), (4096 * 33, 16)):
        x = torch.full((nx + 16,), 7, dtype=torch.uint8, device="cuda")
        y = torch.zeros((ny + 64,), dtype=torch.uint8, device="cuda")
        nm.nm_stream_floor(x[:nx], y[:ny])
        torch.cuda.synchronize()
        whole = ny // 16 * 16
        assert bool((y[:whole].view(torch.int32).view(-1, 4) != 0).all()) if whole else True
        assert int(y[whole:].sum()) == 0
        assert int((x != 7).sum()) == 0
