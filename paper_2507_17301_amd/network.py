"""Runs a whole network (a list of workloads.NetOp) on device tensors through the
C ABI: every convolution is nm_conv2d / nm_conv2d_res on pruned, packed weights,
pooling is nm_maxpool2d / nm_avgpool_global.  This file only allocates tensors
and sequences calls; all arithmetic is in the library's kernels."""
from __future__ import annotations

from typing import List, Optional

from . import binding as nm
from . import workloads as wl


class Network:
    def __init__(self, ops: List[wl.NetOp], batch: int, in_hw: int, dtype: int = nm.NM_F32, seed0: int = 0,
                 device: str = "cuda:0"):
        import torch
        self.ops, self.batch, self.dtype = ops, batch, dtype
        self.tdt = torch.bfloat16 if dtype == nm.NM_BF16 else torch.float32
        self.dev = torch.device(device)
        self.shapes = wl.net_tensor_shapes(ops, batch, in_hw)
        self.packed, self.bias = {}, {}
        for i, w, bias in wl.net_parameters(ops, seed0):
            l = ops[i].layer
            self.packed[i] = nm.nm_prune(w, l.n, l.m, l.tile, dtype)
            self.bias[i] = torch.from_numpy(bias).to(self.dev)
        self.t = {k: torch.empty(v, dtype=self.tdt, device=self.dev) for k, v in self.shapes.items()}
        self.out = ops[-1].dst

    def autotune(self):
        """Profile every legal kernel variant for every convolution shape (cached by shape)."""
        for i, op in enumerate(self.ops):
            if op.kind == "conv":
                b, h, w, c = self.shapes[op.src]
                l = op.layer
                nm.nm_autotune(self.dtype, b, h, w, c, self.packed[i], True, l.stride, l.pad, l.dil, op.relu)

    def forward(self, x=None, stream=None):
        """Enqueue the whole network; x (optional) is copied into the input tensor first.
        Returns the output tensor [B,1,1,classes] (owned by the network, overwritten per call)."""
        if x is not None:
            self.t[0].copy_(x)
        for i, op in enumerate(self.ops):
            src, dst = self.t[op.src], self.t[op.dst]
            if op.kind == "conv":
                l = op.layer
                res = self.t[op.residual] if op.residual >= 0 else None
                nm.nm_conv2d_res(src, self.packed[i], res, self.bias[i], l.stride, l.pad, l.dil, op.relu,
                                 y=dst, stream=stream)
            elif op.kind == "maxpool":
                nm.nm_maxpool2d(src, op.k, op.stride, op.pad, y=dst, stream=stream)
            else:
                nm.nm_avgpool_global(src, y=dst.view(dst.shape[0], dst.shape[3]), stream=stream)
        return self.t[self.out]
