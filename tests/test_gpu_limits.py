"""The largest tensors the library accepts, and the first sizes it refuses.

The kernels address the input through a 2 GiB buffer window with 32-bit byte
offsets and the output with 32-bit element offsets; the limits are therefore
x < 2^31 bytes and P * Cout < 2^31 elements.  Each case sits within one image
row of a limit, runs the default variant of its kernel family, and is checked
by the oracle on sampled outputs that include the corners of the last image and
the last channel, i.e. the highest addresses.
"""
import numpy as np
import pytest

from paper_2507_17301_amd import binding as nm
from paper_2507_17301_amd import workloads as wl
from gpu_util import FP32_TOL, BF16_TOL, say, norm_err, oracle_conv

pytestmark = pytest.mark.gpu

L = wl.ConvLayer

#            name                    H     W    Cin Cout kh kw s  p  d  n  m  T   batch bf16
CASES = [
    (L("in_f32_vec_3x3",          4095, 4096,  32,  16, 3, 3, 1, 1, 1, 2, 4, 16), 1, False),
    (L("in_f32_scalar_1x1",       2048, 2048,  63,  16, 1, 1, 1, 0, 1, 2, 3, 16), 2, False),
    (L("out_f32_tile_path_1x1",   4095, 4096,   4, 128, 1, 1, 1, 0, 1, 2, 4, 16), 1, False),
    (L("out_f32_direct_path_1x1", 4095, 4096,   4, 127, 1, 1, 1, 0, 1, 2, 4, 16), 1, False),
    (L("in_out_bf16_sparse_1x1",  4095, 4096,  64, 128, 1, 1, 1, 0, 1, 2, 4, 16), 1, True),
    (L("in_bf16_sparse_3x3",      4095, 4096,  64,  16, 3, 3, 1, 1, 1, 2, 4, 16), 1, True),
    (L("in_bf16_dense_form_3x3",  4095, 4096,  64,  16, 3, 3, 1, 1, 1, 4, 8, 16), 1, True),
]


@pytest.mark.parametrize("layer,batch,bf16", CASES, ids=[c[0].name for c in CASES])
def test_largest_accepted(layer, batch, bf16):
    import torch
    es = 2 if bf16 else 4
    xin = batch * layer.H * layer.W * layer.Cin
    yout = layer.P(batch) * layer.Cout
    assert xin * es < 2 ** 31 and yout < 2 ** 31
    say(f"limits {layer.name}: x {xin * es} bytes, y {yout} elements")
    x, w, bias = wl.make_tensors(layer, batch, 7000)
    wp = nm.nm_prune(w, layer.n, layer.m, layer.tile, nm.NM_BF16 if bf16 else nm.NM_F32)
    xd = torch.from_numpy(x).cuda()
    if bf16:
        xd = xd.to(torch.bfloat16)
    y = nm.nm_conv2d(xd, wp, torch.from_numpy(bias).cuda(), layer.stride, layer.pad, layer.dil, True)
    torch.cuda.synchronize()
    del xd
    pts = wl.sample_points(layer, batch, 1500, 7000)
    idx = torch.from_numpy(pts.astype(np.int64)).cuda()
    got = y[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].float().cpu().numpy()
    # the last pixel's channels, through the flat view: the highest output addresses
    tail = y.reshape(-1)[-layer.Cout:].float().cpu().numpy()
    del y
    last = np.array([(batch - 1, layer.Ho - 1, layer.Wo - 1, co) for co in range(layer.Cout)], dtype=np.int32)
    ref = oracle_conv(layer, x, w, bias, relu=True, bf16=bf16, pts=np.concatenate([pts, last]))
    tol = BF16_TOL if bf16 else FP32_TOL
    assert norm_err(got, ref[:len(pts)]) <= tol
    assert norm_err(tail, ref[len(pts):]) <= tol


def test_first_sizes_refused():
    """One image row more than the cases above: refused on the host, before any launch."""
    import torch
    for cin, cout, dt, what in ((32, 16, torch.float32, "x of 2 GiB, fp32"),
                                (64, 16, torch.bfloat16, "x of 2 GiB, bf16"),
                                (4, 128, torch.float32, "2^31 output elements")):
        say("limits refused: " + what)
        w = np.ones((cout, 1, 1, cin), dtype=np.float32)
        wp = nm.nm_prune(w, 2, 4, 16, nm.NM_BF16 if dt == torch.bfloat16 else nm.NM_F32)
        x = torch.empty((1, 4096, 4096, cin), dtype=dt, device="cuda")
        y = torch.empty((1, 4096, 4096, cout), dtype=dt, device="cuda")   # never written
        with pytest.raises(nm.NMError) as e:
            nm.nm_conv2d(x, wp, None, 1, 0, 1, False, y=y)
        assert e.value.code == nm.NM_ERR_SHAPE
        del x, y
