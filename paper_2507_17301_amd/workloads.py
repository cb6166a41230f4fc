"""Synthetic workloads: layer tables and seeded input generators.

This module holds shapes and random-number recipes only -- none of the
method's arithmetic (no pruning, no packing, no convolution).  It is the one
piece shared by the tests of the CPU oracle, the GPU parity tests and the
benchmark, so that both sides see identical buffers.

The shapes stand in for the Torchvision ResNets the paper evaluates
(section 4.1.2); the first convolution is left dense (section 4.1.2, last
paragraph), all others are pruned column-wise.  Values are synthetic: the
paper's ImageNet-trained weights are not needed for timing or parity.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class ConvLayer:
    name: str
    H: int
    W: int
    Cin: int
    Cout: int
    Kh: int
    Kw: int
    stride: int = 1
    pad: int = 0
    dil: int = 1
    n: int = 2          # kept columns per group
    m: int = 4          # group size along K
    tile: int = 16      # column-tile width T (output channels per tile)
    stage: int = 0      # 0 = stem, 1..4 = residual stage

    @property
    def K(self) -> int:
        return self.Kh * self.Kw * self.Cin

    @property
    def Kprime(self) -> int:
        return self.K // self.m * self.n

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.dil * (self.Kh - 1) - 1) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.dil * (self.Kw - 1) - 1) // self.stride + 1

    def P(self, batch: int) -> int:
        return batch * self.Ho * self.Wo

    def dense_flops(self, batch: int) -> int:
        return 2 * self.P(batch) * self.K * self.Cout

    def effective_flops(self, batch: int) -> int:
        return 2 * self.P(batch) * self.Kprime * self.Cout

    def algorithmic_bytes(self, batch: int, in_bytes: int = 4, out_bytes: int = 4) -> int:
        """Bytes the method has to move: input once, output once, packed
        values, 16-bit kept indices, bias.  Never the im2col matrix."""
        n_tiles = -(-self.Cout // self.tile)
        return (batch * self.H * self.W * self.Cin * in_bytes
                + self.P(batch) * self.Cout * out_bytes
                + self.Cout * self.Kprime * in_bytes
                + n_tiles * self.Kprime * 2
                + 4 * self.Cout)

    def shape_key(self) -> Tuple:
        return (self.H, self.W, self.Cin, self.Cout, self.Kh, self.Kw, self.stride,
                self.pad, self.dil, self.n, self.m, self.tile)


def _dense(layer: ConvLayer) -> ConvLayer:
    return replace(layer, n=1, m=1)


def dense_form(layer: ConvLayer, name: str = "dense") -> ConvLayer:
    """The same convolution with nothing pruned (N = M = 1): the reference of the
    sparse-over-dense speedup."""
    return replace(layer, name=name, n=1, m=1)


# --------------------------------------------------------------------------
# layer tables
# --------------------------------------------------------------------------

def single_conv_config1() -> ConvLayer:
    """One 3x3 conv, 56x56x64 -> 64, stride 1, pad 1, 2:4, T = 16 (batch 1)."""
    return ConvLayer("cfg1_3x3_56x56x64", 56, 56, 64, 64, 3, 3, 1, 1, 1, 2, 4, 16, 1)


def sweep_config2() -> List[ConvLayer]:
    """ResNet-50 stage-3 3x3 conv (14x14x256 -> 256) over N:M x T (batch 32).
    Cell order: ratio-major, T-minor; the cell index is the seed."""
    cells = []
    for (n, m) in [(1, 4), (2, 4), (1, 8), (2, 8), (4, 8)]:
        for t in (8, 16, 32):
            cells.append(ConvLayer(f"cfg2_{n}of{m}_T{t}", 14, 14, 256, 256, 3, 3, 1, 1, 1,
                                   n, m, t, 3))
    return cells


def _stem(n: int, m: int, tile: int) -> ConvLayer:
    return _dense(ConvLayer("stem_7x7", 224, 224, 3, 64, 7, 7, 2, 3, 1, n, m, tile, 0))


def resnet18_stack(n: int = 2, m: int = 4, tile: int = 16) -> List[ConvLayer]:
    """All 20 convolutions of ResNet-18 (Torchvision form)."""
    L = [_stem(n, m, tile)]
    res, cin = 56, 64
    for stage, width in enumerate((64, 128, 256, 512), start=1):
        for block in range(2):
            s = 2 if (stage > 1 and block == 0) else 1
            pre = f"s{stage}b{block}"
            L.append(ConvLayer(pre + "_conv1_3x3", res, res, cin, width, 3, 3, s, 1, 1,
                               n, m, tile, stage))
            res_out = res // s
            L.append(ConvLayer(pre + "_conv2_3x3", res_out, res_out, width, width, 3, 3, 1, 1, 1,
                               n, m, tile, stage))
            if s == 2:
                L.append(ConvLayer(pre + "_proj_1x1", res, res, cin, width, 1, 1, 2, 0, 1,
                                   n, m, tile, stage))
            res, cin = res_out, width
    return L


def _bottleneck_stack(blocks: Tuple[int, int, int, int], per_stage_nm, tile: int) -> List[ConvLayer]:
    n0, m0 = per_stage_nm[0]
    L = [_stem(n0, m0, tile)]
    res, cin = 56, 64
    for stage, (width, nblk) in enumerate(zip((64, 128, 256, 512), blocks), start=1):
        n, m = per_stage_nm[stage - 1]
        for block in range(nblk):
            s = 2 if (stage > 1 and block == 0) else 1
            pre = f"s{stage}b{block}"
            L.append(ConvLayer(pre + "_conv1_1x1", res, res, cin, width, 1, 1, 1, 0, 1,
                               n, m, tile, stage))
            L.append(ConvLayer(pre + "_conv2_3x3", res, res, width, width, 3, 3, s, 1, 1,
                               n, m, tile, stage))
            res_out = res // s
            L.append(ConvLayer(pre + "_conv3_1x1", res_out, res_out, width, 4 * width, 1, 1, 1, 0, 1,
                               n, m, tile, stage))
            if block == 0:
                L.append(ConvLayer(pre + "_proj_1x1", res, res, cin, 4 * width, 1, 1, s, 0, 1,
                                   n, m, tile, stage))
            res, cin = res_out, 4 * width
    return L


def resnet50_stack(n: int = 2, m: int = 4, tile: int = 16) -> List[ConvLayer]:
    """All 53 convolutions of ResNet-50 (stride on the 3x3 and the projection)."""
    return _bottleneck_stack((3, 4, 6, 3), [(n, m)] * 4, tile)


def resnet101_stack(tile: int = 32) -> List[ConvLayer]:
    """All 104 convolutions of ResNet-101, sparsity mixed per stage:
    stage 1 1:4, stage 2 2:4, stage 3 2:8, stage 4 4:8."""
    return _bottleneck_stack((3, 4, 23, 3), [(1, 4), (2, 4), (2, 8), (4, 8)], tile)


def with_large_groups(layers: List[ConvLayer], mode: str, keep: float = 0.5) -> List[ConvLayer]:
    """The paper's adaptive setting (section 3.1): one group spans all input channels of a
    kernel tap (mode "cin": M = Cin) or the whole row of the weight matrix (mode "row":
    M = K), and N = keep * M columns survive.  Dense layers (N = M) stay dense."""
    out = []
    for l in layers:
        if l.n == l.m:
            out.append(l)
            continue
        m = l.Cin if mode == "cin" else l.K
        out.append(replace(l, n=max(1, int(round(keep * m))), m=m))
    return out


# --------------------------------------------------------------------------
# whole networks: which tensor feeds which operator (structure only)
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class NetOp:
    """One operator of a network.  Tensors are named by small integers; tensor 0 is
    the network input.  kind: "conv" (layer, relu, optional residual tensor added
    before the activation), "maxpool" (k, stride, pad), "avgpool" (global)."""
    kind: str
    src: int
    dst: int
    layer: Optional[ConvLayer] = None
    relu: bool = False
    residual: int = -1
    k: int = 0
    stride: int = 0
    pad: int = 0


def resnet_graph(blocks: Tuple[int, ...], widths: Tuple[int, ...], bottleneck: bool, in_hw: int,
                 per_stage_nm, tile: int, stem_width: int = 64, num_classes: int = 1000) -> List[NetOp]:
    """A Torchvision-form ResNet with batch norm folded into the convolutions' biases:
    7x7/2 stem (dense), 3x3/2 max pooling, residual stages (the skip connection is
    the `residual` of the block's last convolution), global average pooling and the
    classifier as a dense 1x1 convolution on the pooled 1x1 map."""
    ops: List[NetOp] = []
    nxt = [1]

    def new():
        nxt[0] += 1
        return nxt[0] - 1

    n0, m0 = per_stage_nm[0]
    stem = _dense(ConvLayer("stem_7x7", in_hw, in_hw, 3, stem_width, 7, 7, 2, 3, 1, n0, m0, tile, 0))
    t = new()
    ops.append(NetOp("conv", 0, t, stem, relu=True))
    res = stem.Ho
    t2 = new()
    ops.append(NetOp("maxpool", t, t2, k=3, stride=2, pad=1))
    res = (res + 2 - 3) // 2 + 1
    cur, cin = t2, stem_width
    exp = 4 if bottleneck else 1
    for stage, (width, nblk) in enumerate(zip(widths, blocks), start=1):
        n, m = per_stage_nm[stage - 1]
        for block in range(nblk):
            s = 2 if (stage > 1 and block == 0) else 1
            pre = f"s{stage}b{block}"
            res_out = res // s
            ident = cur
            if s == 2 or cin != width * exp:
                ident = new()
                ops.append(NetOp("conv", cur, ident, ConvLayer(pre + "_proj_1x1", res, res, cin, width * exp,
                                                               1, 1, s, 0, 1, n, m, tile, stage)))
            if bottleneck:
                a, b_, c = new(), new(), new()
                ops.append(NetOp("conv", cur, a, ConvLayer(pre + "_conv1_1x1", res, res, cin, width, 1, 1, 1, 0, 1,
                                                           n, m, tile, stage), relu=True))
                ops.append(NetOp("conv", a, b_, ConvLayer(pre + "_conv2_3x3", res, res, width, width, 3, 3, s, 1, 1,
                                                          n, m, tile, stage), relu=True))
                ops.append(NetOp("conv", b_, c, ConvLayer(pre + "_conv3_1x1", res_out, res_out, width, width * 4,
                                                          1, 1, 1, 0, 1, n, m, tile, stage),
                                 relu=True, residual=ident))
            else:
                a, c = new(), new()
                ops.append(NetOp("conv", cur, a, ConvLayer(pre + "_conv1_3x3", res, res, cin, width, 3, 3, s, 1, 1,
                                                           n, m, tile, stage), relu=True))
                ops.append(NetOp("conv", a, c, ConvLayer(pre + "_conv2_3x3", res_out, res_out, width, width,
                                                         3, 3, 1, 1, 1, n, m, tile, stage),
                                 relu=True, residual=ident))
            cur, cin, res = c, width * exp, res_out
    t = new()
    ops.append(NetOp("avgpool", cur, t))
    t2 = new()
    ops.append(NetOp("conv", t, t2, _dense(ConvLayer("fc", 1, 1, cin, num_classes, 1, 1, 1, 0, 1, 1, 1, tile, 5))))
    return ops


def net_parameters(ops: List[NetOp], seed0: int):
    """Seeded weights and biases of a network's convolutions, in operator order:
    yields (operator index, w [Cout,Kh,Kw,Cin] fp32, bias [Cout] fp32)."""
    for i, op in enumerate(ops):
        if op.kind == "conv":
            _, w, bias = make_tensors(op.layer, 1, seed0 + i, with_input=False)
            yield i, w, bias


def net_tensor_shapes(ops: List[NetOp], batch: int, in_hw: int) -> dict:
    """Shape of every tensor of the network (NHWC; the pooled map is [B,1,1,C])."""
    shapes = {0: (batch, in_hw, in_hw, 3)}
    for op in ops:
        b, h, w, c = shapes[op.src]
        if op.kind == "conv":
            l = op.layer
            shapes[op.dst] = (b, l.Ho, l.Wo, l.Cout)
        elif op.kind == "maxpool":
            shapes[op.dst] = (b, (h + 2 * op.pad - op.k) // op.stride + 1, (w + 2 * op.pad - op.k) // op.stride + 1, c)
        else:
            shapes[op.dst] = (b, 1, 1, c)
    return shapes


def resnet50_graph(n: int = 2, m: int = 4, tile: int = 16) -> List[NetOp]:
    return resnet_graph((3, 4, 6, 3), (64, 128, 256, 512), True, 224, [(n, m)] * 4, tile)


def resnet18_graph(n: int = 2, m: int = 4, tile: int = 16) -> List[NetOp]:
    return resnet_graph((2, 2, 2, 2), (64, 128, 256, 512), False, 224, [(n, m)] * 4, tile)


def resnet101_graph(tile: int = 32) -> List[NetOp]:
    return resnet_graph((3, 4, 23, 3), (64, 128, 256, 512), True, 224, [(1, 4), (2, 4), (2, 8), (4, 8)], tile)


def unique_shapes(layers: List[ConvLayer]) -> List[ConvLayer]:
    seen, out = set(), []
    for l in layers:
        k = l.shape_key()
        if k not in seen:
            seen.add(k)
            out.append(l)
    return out


# --------------------------------------------------------------------------
# seeded generators (numpy; handed to oracle and GPU library alike)
# --------------------------------------------------------------------------

def he_sigma(layer: ConvLayer) -> float:
    return float(np.sqrt(2.0 / (layer.Kh * layer.Kw * layer.Cin)))


def make_tensors(layer: ConvLayer, batch: int, seed: int, weight_sigma: Optional[float] = None,
                 with_input: bool = True):
    """x ~ U[0,1) NHWC, w ~ N(0, sigma) OHWI (He-normal if sigma is None),
    bias ~ N(0, 0.01).  All fp32, drawn in the order w, bias, x."""
    rng = np.random.default_rng(seed)
    sigma = he_sigma(layer) if weight_sigma is None else weight_sigma
    w = (rng.standard_normal((layer.Cout, layer.Kh, layer.Kw, layer.Cin), dtype=np.float32)
         * np.float32(sigma))
    bias = rng.standard_normal(layer.Cout, dtype=np.float32) * np.float32(0.01)
    x = None
    if with_input:
        x = rng.random((batch, layer.H, layer.W, layer.Cin), dtype=np.float32)
    return x, w, bias


def sample_points(layer: ConvLayer, batch: int, count: int, seed: int) -> np.ndarray:
    """Random output positions (b, ho, wo, co), always including the four
    corners of the first and last image and the last channel."""
    rng = np.random.default_rng(seed)
    pts = np.stack([rng.integers(0, batch, count), rng.integers(0, layer.Ho, count),
                    rng.integers(0, layer.Wo, count), rng.integers(0, layer.Cout, count)], axis=1)
    fixed = []
    for b in (0, batch - 1):
        for ho in (0, layer.Ho - 1):
            for wo in (0, layer.Wo - 1):
                for co in (0, layer.Cout - 1):
                    fixed.append((b, ho, wo, co))
    return np.concatenate([np.array(fixed, dtype=np.int64), pts]).astype(np.int32)
