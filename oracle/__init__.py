"""CPU oracle (test infrastructure only).

Thin ctypes wrapper over ``nm_oracle.c``: argument marshalling between numpy
arrays and the C functions, nothing else.  Only ``tests/``, the smoke check and
the benchmark's ``cpu_baseline`` leg may import this package; the GPU library
never does and shares nothing with it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nm_oracle.c")
_LIB = os.path.join(_HERE, "libnm_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile nm_oracle.c with gcc into libnm_oracle.so next to it."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared", "-pthread",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        fp = ctypes.POINTER(ctypes.c_float)
        i32p = ctypes.POINTER(ctypes.c_int32)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        ci = ctypes.c_int
        L.oracle_prune.argtypes = [fp, ci, ci, ci, ci, ci, u8p, i32p, fp]
        L.oracle_prune.restype = ci
        L.oracle_pack.argtypes = [fp, ci, ci, ci, ci, ci, i32p, fp]
        L.oracle_pack.restype = ci
        L.oracle_round_bf16.argtypes = [fp, fp, ctypes.c_long]
        L.oracle_round_bf16.restype = None
        L.oracle_round_e4m3.argtypes = [fp, fp, ctypes.c_long]
        L.oracle_round_e4m3.restype = None
        conv_common = [fp, ci, ci, ci, ci, fp, ci, ci, ci, fp,
                       ci, ci, ci, ci, ci, ci, ci, ci]
        L.oracle_conv2d.argtypes = conv_common + [fp, ci]
        L.oracle_conv2d.restype = ci
        L.oracle_conv2d_points.argtypes = conv_common + [i32p, ctypes.c_long, fp]
        L.oracle_conv2d_points.restype = ci
        L.oracle_conv2d_res.argtypes = (conv_common[:10] + [fp] + conv_common[10:] + [fp])
        L.oracle_conv2d_res.restype = ci
        L.oracle_maxpool2d.argtypes = [fp, ci, ci, ci, ci, ci, ci, ci, fp]
        L.oracle_maxpool2d.restype = ci
        L.oracle_avgpool_global.argtypes = [fp, ci, ci, ci, ci, ci, fp]
        L.oracle_avgpool_global.restype = ci
        L.oracle_im2col.argtypes = [fp] + [ci] * 12 + [fp]
        L.oracle_im2col.restype = ci
        L.oracle_out_size.argtypes = [ci] * 10 + [ctypes.POINTER(ci), ctypes.POINTER(ci)]
        L.oracle_out_size.restype = ci
        _lib = L
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _pair(v):
    if isinstance(v, (tuple, list)):
        return int(v[0]), int(v[1])
    return int(v), int(v)


def out_size(H, W, Kh, Kw, stride=1, pad=0, dil=1):
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dil)
    ho, wo = ctypes.c_int(), ctypes.c_int()
    rc = _load().oracle_out_size(H, W, Kh, Kw, sh, sw, ph, pw, dh, dw,
                                 ctypes.byref(ho), ctypes.byref(wo))
    if rc != 0:
        raise ValueError("oracle_out_size: bad geometry")
    return ho.value, wo.value


def prune(w_ohwi, n, m, tile):
    """w_ohwi [Cout,Kh,Kw,Cin] fp32 -> (mask [Cout,K] u8, idx [n_tiles,G,N] i32,
    w_zero_filled [Cout,Kh,Kw,Cin] fp32)."""
    w, wp = _f32(w_ohwi)
    cout = w.shape[0]
    K = int(np.prod(w.shape[1:]))
    if K % m != 0:
        raise ValueError("K %% M != 0")
    G = K // m
    n_tiles = (cout + tile - 1) // tile
    mask = np.zeros((cout, K), dtype=np.uint8)
    idx = np.zeros((n_tiles, G, n), dtype=np.int32)
    wz = np.zeros_like(w)
    rc = _load().oracle_prune(
        wp, cout, K, n, m, tile,
        mask.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
        idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
        wz.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if rc != 0:
        raise ValueError("oracle_prune rejected its arguments")
    return mask, idx, wz


def pack(w_ohwi, idx, n, m, tile):
    """Compressed values vals[n_tiles, K', T] for kept positions idx."""
    w, wp = _f32(w_ohwi)
    cout = w.shape[0]
    K = int(np.prod(w.shape[1:]))
    G = K // m
    n_tiles = (cout + tile - 1) // tile
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    vals = np.zeros((n_tiles, G * n, tile), dtype=np.float32)
    rc = _load().oracle_pack(
        wp, cout, K, n, m, tile,
        idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
        vals.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if rc != 0:
        raise ValueError("oracle_pack rejected its arguments")
    return vals


def round_bf16(a):
    """Round fp32 values to the nearest bf16 (ties to even), returned as fp32."""
    a, ap = _f32(a)
    out = np.empty_like(a)
    _load().oracle_round_bf16(ap, out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), a.size)
    return out


def round_e4m3(a):
    """Round fp32 values to the nearest fp8 E4M3 value (OCP e4m3fn; ties to even, NaN beyond
    the largest finite value 448), returned as fp32."""
    a, ap = _f32(a)
    out = np.empty_like(a)
    _load().oracle_round_e4m3(ap, out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), a.size)
    return out


def fp8_weight_scale(w_kept):
    """The power-of-two scale under which a layer's kept weights are stored as E4M3: the
    largest 2^e with max|w| * 2^e <= 448 (1 for an all-zero layer).  Scaling by a power of
    two is exact, so the stored value times 2^-e is the weight the convolution uses."""
    m = float(np.max(np.abs(w_kept))) if np.size(w_kept) else 0.0
    if m == 0.0:
        return 1.0
    f, e = np.frexp(448.0 / m)          # 448 / m = f * 2^e with 0.5 <= f < 1: floor(log2) = e - 1
    s = float(np.ldexp(1.0, int(e) - 1))
    while m * s > 448.0:                # the division above is rounded: step back if it rounded up across a power of two
        s /= 2.0
    return s


def quantize_e4m3(w_kept):
    """(dequantized weights, scale): w -> round_e4m3(w * s) / s with s = fp8_weight_scale(w)."""
    s = fp8_weight_scale(w_kept)
    w = np.ascontiguousarray(w_kept, dtype=np.float32)
    return (round_e4m3(w * np.float32(s)) / np.float32(s)).astype(np.float32), s


def _conv_args(x, w, bias, stride, pad, dil, relu, out_bf16):
    x, xp = _f32(x)
    w, wp = _f32(w)
    B, H, W, Cin = x.shape
    Cout, Kh, Kw, Cin2 = w.shape
    if Cin2 != Cin:
        raise ValueError("channel mismatch")
    if bias is None:
        b, bp = None, ctypes.POINTER(ctypes.c_float)()
    else:
        b, bp = _f32(bias)
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dil)
    keep = (x, w, b)
    args = [xp, B, H, W, Cin, wp, Cout, Kh, Kw, bp, sh, sw, ph, pw, dh, dw,
            int(bool(relu)), int(bool(out_bf16))]
    Ho, Wo = out_size(H, W, Kh, Kw, (sh, sw), (ph, pw), (dh, dw))
    return args, keep, (B, Ho, Wo, Cout)


def conv2d(x, w, bias=None, stride=1, pad=0, dil=1, relu=False, out_bf16=False,
           nthreads=None):
    """Direct convolution.  x [B,H,W,Cin], w [Cout,Kh,Kw,Cin] -> y [B,Ho,Wo,Cout]."""
    args, keep, oshape = _conv_args(x, w, bias, stride, pad, dil, relu, out_bf16)
    y = np.empty(oshape, dtype=np.float32)
    if nthreads is None:
        nthreads = os.cpu_count() or 1
    rc = _load().oracle_conv2d(*args, y.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                               int(nthreads))
    if rc != 0:
        raise ValueError("oracle_conv2d rejected its arguments")
    return y


def conv2d_res(x, w, residual, bias=None, stride=1, pad=0, dil=1, relu=False, out_bf16=False):
    """relu?(conv(x, w) + bias + residual); residual is shaped like the output."""
    args, keep, oshape = _conv_args(x, w, bias, stride, pad, dil, relu, out_bf16)
    res = np.ascontiguousarray(residual, dtype=np.float32)
    if res.shape != tuple(oshape):
        raise ValueError("residual must be shaped like the output")
    y = np.empty(oshape, dtype=np.float32)
    fp = ctypes.POINTER(ctypes.c_float)
    # argument order of the C function: ..., bias, residual, strides ...
    head, tail = args[:10], args[10:]
    rc = _load().oracle_conv2d_res(*head, res.ctypes.data_as(fp), *tail, y.ctypes.data_as(fp))
    if rc != 0:
        raise ValueError("oracle_conv2d_res rejected its arguments")
    return y


def maxpool2d(x, k, stride, pad):
    """Max pooling of x [B,H,W,C] with a k x k window; padding never wins."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    B, H, W, C = x.shape
    if H + 2 * pad < k or W + 2 * pad < k:
        raise ValueError("empty output")
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    y = np.empty((B, Ho, Wo, C), dtype=np.float32)
    fp = ctypes.POINTER(ctypes.c_float)
    rc = _load().oracle_maxpool2d(x.ctypes.data_as(fp), B, H, W, C, int(k), int(stride), int(pad),
                                  y.ctypes.data_as(fp))
    if rc != 0:
        raise ValueError("oracle_maxpool2d rejected its arguments")
    return y


def avgpool_global(x, out_bf16=False):
    """Mean over all positions: x [B,H,W,C] -> [B,C]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    B, H, W, C = x.shape
    y = np.empty((B, C), dtype=np.float32)
    fp = ctypes.POINTER(ctypes.c_float)
    rc = _load().oracle_avgpool_global(x.ctypes.data_as(fp), B, H, W, C, int(bool(out_bf16)),
                                       y.ctypes.data_as(fp))
    if rc != 0:
        raise ValueError("oracle_avgpool_global rejected its arguments")
    return y


def im2col(x, kh, kw, stride=1, pad=0, dil=1):
    """The im2col matrix as [B,Ho,Wo,kh*kw*Cin], k order (kh, kw, ci), zero outside the image."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    B, H, W, C = x.shape
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dil)
    Ho, Wo = out_size(H, W, kh, kw, (sh, sw), (ph, pw), (dh, dw))
    a = np.empty((B, Ho, Wo, kh * kw * C), dtype=np.float32)
    fp = ctypes.POINTER(ctypes.c_float)
    rc = _load().oracle_im2col(x.ctypes.data_as(fp), B, H, W, C, int(kh), int(kw), sh, sw, ph, pw, dh, dw,
                               a.ctypes.data_as(fp))
    if rc != 0:
        raise ValueError("oracle_im2col rejected its arguments")
    return a


def conv2d_points(x, w, pts, bias=None, stride=1, pad=0, dil=1, relu=False,
                  out_bf16=False):
    """The same convolution evaluated at pts [n,4] = (b, ho, wo, co) only."""
    args, keep, _ = _conv_args(x, w, bias, stride, pad, dil, relu, out_bf16)
    pts = np.ascontiguousarray(pts, dtype=np.int32).reshape(-1, 4)
    out = np.empty(pts.shape[0], dtype=np.float32)
    rc = _load().oracle_conv2d_points(
        *args, pts.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), pts.shape[0],
        out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if rc != 0:
        raise ValueError("oracle_conv2d_points rejected its arguments")
    return out
