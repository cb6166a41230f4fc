"""Helpers for the GPU parity tests: run one layer through the C-ABI library
and through the CPU oracle on identical seeded buffers."""
import sys

import numpy as np

import oracle
from paper_2507_17301_amd import binding as nm
from paper_2507_17301_amd import workloads as wl

FP32_TOL = 1e-4    # |err| <= tol * (1 + |ref|)
BF16_TOL = 2e-2


def say(msg):
    """Name the case before it runs, flushed, so that a GPU fault is attributable."""
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def norm_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref) / (1.0 + np.abs(ref)))) if ref.size else 0.0


def gpu_conv(layer, x_np, w_np, bias_np, relu, bf16=False, use_bias=True):
    """Prune + convolve on the GPU.  Returns (packed handle, y as fp32 numpy)."""
    import torch
    dev = torch.device("cuda:0")
    wp = nm.nm_prune(w_np, layer.n, layer.m, layer.tile, nm.NM_BF16 if bf16 else nm.NM_F32)
    x = torch.from_numpy(x_np).to(dev)
    if bf16:
        x = x.to(torch.bfloat16)
    b = torch.from_numpy(bias_np).to(dev) if use_bias else None
    y = nm.nm_conv2d(x, wp, b, layer.stride, layer.pad, layer.dil, relu)
    torch.cuda.synchronize()
    return wp, y.float().cpu().numpy()


def oracle_conv(layer, x_np, w_np, bias_np, relu, bf16=False, use_bias=True, pts=None):
    """Oracle result for the same layer.  For bf16 the oracle is fed the
    bf16-rounded input and bf16-rounded kept weights as exact floats."""
    _, _, wz = oracle.prune(w_np, layer.n, layer.m, layer.tile)
    if bf16:
        wz = oracle.round_bf16(wz)
        x_np = oracle.round_bf16(x_np)
    b = bias_np if use_bias else None
    if pts is None:
        return oracle.conv2d(x_np, wz, b, layer.stride, layer.pad, layer.dil, relu, out_bf16=bf16)
    return oracle.conv2d_points(x_np, wz, pts, b, layer.stride, layer.pad, layer.dil, relu,
                                out_bf16=bf16)
