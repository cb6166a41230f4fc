"""Pins for the oracle's convolution (CPU only).

The oracle's seven-loop sum is checked against: PyTorch's CPU conv2d in fp64
(a library routine for the same definition), a scatter-form brute force written
independently here, closed forms (delta input, all-ones input), linearity, and
the property the paper's Alg. 1 rests on: contracting only the kept columns of
the compressed weights equals the dense result with pruned weights zeroed.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2507_17301_amd import workloads as wl

TOL = 2e-6   # fp64 accumulate, one rounding to fp32


def _torch_conv(x, w, bias, stride, pad, dil, relu):
    xt = torch.from_numpy(x).double().permute(0, 3, 1, 2)          # NHWC -> NCHW
    wt = torch.from_numpy(w).double().permute(0, 3, 1, 2)          # OHWI -> OIHW
    bt = None if bias is None else torch.from_numpy(bias).double()
    y = torch.nn.functional.conv2d(xt, wt, bt, stride=stride, padding=pad, dilation=dil)
    if relu:
        y = torch.relu(y)
    return y.permute(0, 2, 3, 1).contiguous().numpy()


def _scatter_conv(x, w, stride, pad, dil):
    """Input-stationary form: every input element adds its contribution to all
    outputs it reaches.  Deliberately a different loop nest from the oracle."""
    B, H, W, Cin = x.shape
    Cout, Kh, Kw, _ = w.shape
    sh, sw = stride
    ph, pw = pad
    dh, dw = dil
    Ho = (H + 2 * ph - dh * (Kh - 1) - 1) // sh + 1
    Wo = (W + 2 * pw - dw * (Kw - 1) - 1) // sw + 1
    y = np.zeros((B, Ho, Wo, Cout), dtype=np.float64)
    for b in range(B):
        for hi in range(H):
            for wi in range(W):
                for kh in range(Kh):
                    th = hi + ph - kh * dh
                    if th < 0 or th % sh:
                        continue
                    ho = th // sh
                    if ho >= Ho:
                        continue
                    for kw in range(Kw):
                        tw = wi + pw - kw * dw
                        if tw < 0 or tw % sw:
                            continue
                        wo = tw // sw
                        if wo >= Wo:
                            continue
                        y[b, ho, wo, :] += w[:, kh, kw, :].astype(np.float64) @ x[b, hi, wi, :].astype(np.float64)
    return y


GRID = [
    # B, H, W, Cin, Cout, Kh, Kw, stride, pad, dil
    (1, 8, 8, 4, 8, 3, 3, (1, 1), (1, 1), (1, 1)),
    (2, 9, 7, 8, 5, 3, 3, (2, 2), (1, 1), (1, 1)),
    (1, 11, 10, 3, 6, 7, 7, (2, 2), (3, 3), (1, 1)),
    (2, 7, 9, 8, 16, 1, 1, (1, 1), (0, 0), (1, 1)),
    (1, 9, 9, 4, 4, 1, 1, (2, 2), (0, 0), (1, 1)),
    (1, 10, 12, 4, 7, 3, 3, (1, 1), (2, 2), (2, 2)),
    (1, 12, 9, 4, 3, 3, 2, (2, 1), (0, 1), (1, 2)),
    (3, 5, 6, 12, 9, 2, 3, (1, 2), (1, 0), (2, 1)),
]


@pytest.mark.parametrize("B,H,W,Cin,Cout,Kh,Kw,stride,pad,dil", GRID)
@pytest.mark.parametrize("relu", [False, True])
def test_against_torch_cpu_fp64(B, H, W, Cin, Cout, Kh, Kw, stride, pad, dil, relu):
    rng = np.random.default_rng(B * 100 + H + Cin)
    x = rng.random((B, H, W, Cin), dtype=np.float32)
    w = rng.standard_normal((Cout, Kh, Kw, Cin)).astype(np.float32) * 0.2
    bias = rng.standard_normal(Cout).astype(np.float32) * 0.1
    ref = _torch_conv(x, w, bias, stride, pad, dil, relu)
    got = oracle.conv2d(x, w, bias, stride, pad, dil, relu, nthreads=3)
    assert got.shape == ref.shape
    assert np.max(np.abs(got - ref) / (1 + np.abs(ref))) < TOL
    nob = oracle.conv2d(x, w, None, stride, pad, dil, relu, nthreads=1)
    refnb = _torch_conv(x, w, None, stride, pad, dil, relu)
    assert np.max(np.abs(nob - refnb) / (1 + np.abs(refnb))) < TOL


@pytest.mark.parametrize("B,H,W,Cin,Cout,Kh,Kw,stride,pad,dil", GRID[:3] + GRID[5:])
def test_against_scatter_brute_force(B, H, W, Cin, Cout, Kh, Kw, stride, pad, dil):
    rng = np.random.default_rng(99)
    x = rng.random((B, H, W, Cin), dtype=np.float32)
    w = rng.standard_normal((Cout, Kh, Kw, Cin)).astype(np.float32)
    ref = _scatter_conv(x, w, stride, pad, dil)
    got = oracle.conv2d(x, w, None, stride, pad, dil, False)
    assert np.max(np.abs(got - ref) / (1 + np.abs(ref))) < TOL


def test_delta_input_reproduces_the_taps():
    """x = unit impulse at (h0, w0, c0): y[ho, wo, co] = w[co, kh, kw, c0] where
    the tap (kh, kw) of output (ho, wo) lands on the impulse."""
    H = W = 7
    Cin, Cout, Kh, Kw = 3, 4, 3, 3
    rng = np.random.default_rng(1)
    w = rng.standard_normal((Cout, Kh, Kw, Cin)).astype(np.float32)
    x = np.zeros((1, H, W, Cin), dtype=np.float32)
    h0, w0, c0 = 3, 4, 2
    x[0, h0, w0, c0] = 1.0
    y = oracle.conv2d(x, w, None, 1, 1, 1, False)
    want = np.zeros_like(y)
    for kh in range(Kh):
        for kw in range(Kw):
            ho, wo = h0 + 1 - kh, w0 + 1 - kw
            want[0, ho, wo, :] = w[:, kh, kw, c0]
    assert np.array_equal(y, want)


def test_all_ones_counts_in_bounds_kept_taps():
    """x = 1, kept weights = 1: each output equals the number of kept weights
    whose tap falls inside the image, plus the bias."""
    H, W, Cin, Cout, Kh, Kw = 6, 5, 4, 8, 3, 3
    rng = np.random.default_rng(2)
    w = rng.standard_normal((Cout, Kh, Kw, Cin)).astype(np.float32)
    mask, idx, _ = oracle.prune(w, 2, 4, 4)
    ones_w = mask.reshape(Cout, Kh, Kw, Cin).astype(np.float32)
    bias = np.arange(Cout, dtype=np.float32)
    x = np.ones((2, H, W, Cin), dtype=np.float32)
    y = oracle.conv2d(x, ones_w, bias, 1, 1, 1, False)
    for ho in range(H):
        for wo in range(W):
            inb = np.zeros((Kh, Kw), dtype=bool)
            for kh in range(Kh):
                for kw in range(Kw):
                    inb[kh, kw] = (0 <= ho - 1 + kh < H) and (0 <= wo - 1 + kw < W)
            cnt = (ones_w * inb[None, :, :, None]).sum(axis=(1, 2, 3))
            assert np.array_equal(y[0, ho, wo], cnt + bias)
            assert np.array_equal(y[1, ho, wo], cnt + bias)
    # interior pixels: every tap in bounds -> exactly K' = K/M*N kept weights
    assert np.all(y[:, 1:-1, 1:-1, :] - bias == Kh * Kw * Cin // 4 * 2)


def test_linearity_in_the_input():
    rng = np.random.default_rng(4)
    x1 = rng.integers(-4, 5, size=(1, 6, 6, 4)).astype(np.float32)
    x2 = rng.integers(-4, 5, size=(1, 6, 6, 4)).astype(np.float32)
    w = (rng.integers(-8, 9, size=(5, 3, 3, 4)) / 8.0).astype(np.float32)
    y1 = oracle.conv2d(x1, w, None, 1, 1, 1, False)
    y2 = oracle.conv2d(x2, w, None, 1, 1, 1, False)
    y12 = oracle.conv2d(2 * x1 - x2, w, None, 1, 1, 1, False)
    assert np.array_equal(y12, 2 * y1 - y2)   # all values exact in fp32


@pytest.mark.parametrize("n,m,tile", [(2, 4, 4), (1, 4, 8), (4, 8, 3), (2, 8, 16)])
def test_compressed_contraction_equals_zero_filled_dense(n, m, tile):
    """Alg. 1 read as a definition: out[p, jT+t] = sum over kept kk of
    A[Idx[j][kk], p] * W'[j][kk][t], with A the im2col matrix (section 2.2).
    It must equal the direct convolution with zero-filled weights."""
    B, H, W, Cin, Cout, Kh, Kw = 2, 6, 5, 8, 10, 3, 3
    rng = np.random.default_rng(n * 10 + m)
    x = rng.random((B, H, W, Cin), dtype=np.float32)
    w = rng.standard_normal((Cout, Kh, Kw, Cin)).astype(np.float32)
    mask, idx, wz = oracle.prune(w, n, m, tile)
    vals = oracle.pack(w, idx, n, m, tile)
    y = oracle.conv2d(x, wz, None, 1, 1, 1, False)
    # im2col matrix A[K, P] built with plain indexing
    K = Kh * Kw * Cin
    xp = np.pad(x.astype(np.float64), ((0, 0), (1, 1), (1, 1), (0, 0)))
    A = np.zeros((K, B * H * W))
    for kh in range(Kh):
        for kw in range(Kw):
            patch = xp[:, kh:kh + H, kw:kw + W, :].reshape(B * H * W, Cin)
            A[(kh * Kw + kw) * Cin:(kh * Kw + kw + 1) * Cin] = patch.T
    out = np.zeros((B * H * W, Cout))
    for j in range(idx.shape[0]):
        kept = idx[j].reshape(-1)
        cols = vals[j].astype(np.float64)                      # [K', T]
        res = A[kept].T @ cols                                 # [P, T]
        hi = min(tile, Cout - j * tile)
        out[:, j * tile:j * tile + hi] = res[:, :hi]
    ref = out.reshape(B, H, W, Cout)
    assert np.max(np.abs(y - ref) / (1 + np.abs(ref))) < TOL


def test_points_and_thread_count_do_not_change_values():
    layer = wl.ConvLayer("t", 9, 8, 8, 12, 3, 3, 2, 1, 1, 2, 4, 4)
    x, w, bias = wl.make_tensors(layer, 3, 5)
    full1 = oracle.conv2d(x, w, bias, 2, 1, 1, True, nthreads=1)
    full8 = oracle.conv2d(x, w, bias, 2, 1, 1, True, nthreads=8)
    assert np.array_equal(full1, full8)
    pts = wl.sample_points(layer, 3, 50, 1)
    got = oracle.conv2d_points(x, w, pts, bias, 2, 1, 1, True)
    assert np.array_equal(got, full1[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]])


def test_bf16_rounding_matches_library_conversion():
    rng = np.random.default_rng(8)
    a = np.concatenate([
        rng.standard_normal(4096).astype(np.float32),
        rng.random(4096, dtype=np.float32) * 1e-3,
        # exact ties between two bf16 neighbours, both parities
        np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(2.0 + 2.0 ** -7), 0.0, -0.0,
                  3.3895313892515355e38], dtype=np.float32),
    ])
    got = oracle.round_bf16(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    assert got[8192] == 1.0 and got[8193] == np.float32(1.0 + 2.0 ** -6)   # ties to even


def test_bf16_output_is_one_extra_rounding():
    layer = wl.ConvLayer("t", 6, 6, 8, 8, 3, 3, 1, 1, 1, 2, 4, 4)
    x, w, bias = wl.make_tensors(layer, 1, 6)
    y32 = oracle.conv2d(x, w, bias, 1, 1, 1, True)
    y16 = oracle.conv2d(x, w, bias, 1, 1, 1, True, out_bf16=True)
    assert np.array_equal(y16, oracle.round_bf16(y32))


def test_output_geometry():
    assert oracle.out_size(224, 224, 7, 7, 2, 3, 1) == (112, 112)
    assert oracle.out_size(56, 56, 3, 3, 1, 1, 1) == (56, 56)
    assert oracle.out_size(56, 56, 1, 1, 2, 0, 1) == (28, 28)
    assert oracle.out_size(10, 12, 3, 3, 1, 2, 2) == (10, 12)
    with pytest.raises(ValueError):
        oracle.out_size(2, 2, 5, 5, 1, 0, 1)


def test_e4m3_rounding_matches_the_reference_conversion():
    """oracle.round_e4m3 against torch's float8_e4m3fn conversion: every representable value,
    every midpoint between neighbours (ties to even), values just off the midpoints, the
    subnormal range, the overflow boundary (464 is the last value that rounds to 448; beyond
    that the format has nothing to round to and the result is NaN), random values."""
    import torch
    codes = torch.arange(256, dtype=torch.uint8)
    vals = codes.view(torch.float8_e4m3fn).float().numpy()
    finite = np.sort(vals[np.isfinite(vals)])
    assert finite.size == 254 and finite[-1] == 448.0 and finite[0] == -448.0
    assert np.array_equal(oracle.round_e4m3(finite), finite)                     # fixed points
    mids = ((finite[:-1].astype(np.float64) + finite[1:].astype(np.float64)) / 2).astype(np.float32)
    rng = np.random.default_rng(0)
    probe = np.concatenate([
        mids, np.nextafter(mids, np.float32(np.inf)), np.nextafter(mids, np.float32(-np.inf)),
        np.float32([2.0 ** -9, 2.0 ** -10, 1.5 * 2.0 ** -10, 0.75 * 2.0 ** -9, 2.0 ** -6, 2.0 ** -7 * 1.0625]),
        np.float32([448.0, 455.9, 463.99, 464.0, -464.0]),
        rng.standard_normal(20000).astype(np.float32) * 3, rng.random(20000, dtype=np.float32),
        (rng.standard_normal(5000) * 0.02).astype(np.float32), rng.uniform(-448, 448, 5000).astype(np.float32)])
    want = torch.from_numpy(probe).to(torch.float8_e4m3fn).float().numpy()
    got = oracle.round_e4m3(probe)
    assert np.array_equal(got, want) and np.array_equal(np.signbit(got), np.signbit(want))
    beyond = np.float32([464.0000305, 480.0, 1e6, -1e6])
    assert np.all(np.isnan(oracle.round_e4m3(beyond)))
    assert np.all(np.isnan(torch.from_numpy(beyond).to(torch.float8_e4m3fn).float().numpy()))


def test_fp8_weight_scale_is_the_largest_power_of_two_that_fits():
    for m in (1.0, 0.3, 447.9, 448.0, 448.1, 3.5e-4, 7.0, 224.0, 0.02734375):
        s = oracle.fp8_weight_scale(np.float32([0.0, -m, m / 3]))
        assert s == 2.0 ** round(np.log2(s))
        assert np.float32(m) * s <= 448.0 < np.float32(m) * s * 2
    assert oracle.fp8_weight_scale(np.zeros(4, dtype=np.float32)) == 1.0
    w = (np.random.default_rng(1).standard_normal((8, 3, 3, 16)) * 0.05).astype(np.float32)
    wq, s = oracle.quantize_e4m3(w)
    assert np.array_equal(oracle.round_e4m3(wq * np.float32(s)), wq * np.float32(s))   # representable under the scale
    assert np.max(np.abs(wq - w)) <= np.max(np.abs(w)) / 16 + 2.0 ** -9 / s            # within half a step of the top binade
