"""ctypes binding of libnmconv.so -- argument marshalling only.

Same names as the C ABI in ``include/nm_conv.h``.  Tensors are torch tensors
used purely as device buffers (``data_ptr()``) and for the current stream; all
arithmetic happens inside the library's kernels.  There is no fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np

NM_F32, NM_BF16, NM_F8E4M3 = 0, 1, 2
NM_OK = 0
NM_ERR_ARG, NM_ERR_SHAPE, NM_ERR_UNSUPPORTED, NM_ERR_ALLOC, NM_ERR_HIP, NM_ERR_IO = -1, -2, -3, -4, -5, -6
_STATUS = {0: "NM_OK", -1: "NM_ERR_ARG", -2: "NM_ERR_SHAPE", -3: "NM_ERR_UNSUPPORTED",
           -4: "NM_ERR_ALLOC", -5: "NM_ERR_HIP", -6: "NM_ERR_IO"}

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libnmconv.so")
_lib = None


class NMError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{_STATUS.get(code, code)}: {msg}")
        self.code = code


def lib():
    """Open libnmconv.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2507_17301_amd.build` "
                "(there is no fallback path)")
        # PyTorch ships its own copy of the HIP runtime; a process must not end up with two.
        # Importing torch first makes its copy the one libnmconv.so binds to as well (loaded
        # the other way round, torch finds no GPU).
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        ci, cf, vp = ctypes.c_int, ctypes.c_float, ctypes.c_void_p
        pi = ctypes.POINTER(ctypes.c_int)
        L.nm_last_error.restype = ctypes.c_char_p
        L.nm_variant_count.restype = ci
        L.nm_last_variant.restype = ci
        L.nm_variant_name.argtypes = [ci]
        L.nm_variant_name.restype = ctypes.c_char_p
        L.nm_prune.argtypes = [vp, ci, ci, ci, ci, ci, ci, ci, ci, ctypes.POINTER(vp)]
        L.nm_packed_free.argtypes = [vp]
        L.nm_packed_dims.argtypes = [vp, pi, pi, pi, pi]
        L.nm_packed_indices.argtypes = [vp, vp]
        L.nm_packed_values.argtypes = [vp, vp]
        L.nm_packed_mask.argtypes = [vp, vp]
        L.nm_packed_scale.argtypes = [vp, ctypes.POINTER(cf)]
        L.nm_conv2d.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp, ci, vp]
        L.nm_conv2d_res.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp, ci, vp]
        L.nm_conv2d_static.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp, ci, vp]
        L.nm_maxpool2d.argtypes = [vp, ci, ci, ci, ci, ci, ci, ci, ci, vp, vp]
        L.nm_avgpool_global.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp]
        L.nm_im2col.argtypes = [vp] + [ci] * 13 + [vp, vp]
        L.nm_stream_floor.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp]
        L.nm_autotune.argtypes = [ci, ci, ci, ci, ci, vp, ci, ci, ci, ci, ci, ci, ci, ci, ci, vp,
                                  pi, ctypes.POINTER(cf)]
        L.nm_autotune_tile.argtypes = ([vp] + [ci] * 6 + [pi, ci, ci] + [ci] * 13 +
                                       [vp, ctypes.POINTER(vp), pi, ctypes.POINTER(ctypes.c_float)])
        L.nm_cache_save.argtypes = [ctypes.c_char_p]
        L.nm_cache_load.argtypes = [ctypes.c_char_p]
        L.nm_force_variant.argtypes = [ci]
        L.nm_variant_legal.argtypes = [ci, vp, ci, ci]
        for name in ("nm_prune", "nm_packed_free", "nm_packed_dims", "nm_packed_indices",
                     "nm_packed_values", "nm_packed_mask", "nm_packed_scale", "nm_conv2d", "nm_conv2d_res", "nm_conv2d_static",
                     "nm_maxpool2d",
                     "nm_avgpool_global", "nm_im2col", "nm_stream_floor", "nm_autotune",
                     "nm_cache_save", "nm_cache_load", "nm_cache_clear", "nm_cache_size", "nm_workspace_free",
                     "nm_force_variant", "nm_variant_legal"):
            getattr(L, name).restype = ci
        _lib = L
    return _lib


def _check(rc: int) -> int:
    if rc < 0:
        raise NMError(rc, lib().nm_last_error().decode())
    return rc


def _pair(v) -> Tuple[int, int]:
    if isinstance(v, (tuple, list)):
        return int(v[0]), int(v[1])
    return int(v), int(v)


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return NM_F32
    if t.dtype == torch.bfloat16:
        return NM_BF16
    if t.dtype == torch.float8_e4m3fn:
        return NM_F8E4M3
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


class Packed:
    """Owner of an nm_packed_t handle."""

    def __init__(self, handle, cout, kh, kw, cin, n, m, tile, value_dtype):
        self.handle = handle
        self.cout, self.kh, self.kw, self.cin = cout, kh, kw, cin
        self.n, self.m, self.tile, self.value_dtype = n, m, tile, value_dtype
        self.K = kh * kw * cin

    def free(self):
        """Release the handle now (idempotent)."""
        h, self.handle = getattr(self, "handle", None), None
        if h and _lib is not None:
            _lib.nm_packed_free(h)

    def __del__(self):
        # at interpreter shutdown the module globals may already be gone; the
        # process is ending then and the driver reclaims the device memory
        try:
            self.free()
        except Exception:
            pass


def nm_variant_count() -> int:
    return lib().nm_variant_count()


def nm_last_variant() -> int:
    """Variant id launched by this thread's last successful nm_conv2d / nm_conv2d_res."""
    return lib().nm_last_variant()


def nm_variant_name(v: int) -> Optional[str]:
    s = lib().nm_variant_name(v)
    return s.decode() if s else None


def nm_prune(w_ohwi: np.ndarray, n: int, m: int, tile: int, value_dtype: int = NM_F32) -> Packed:
    """w_ohwi: host numpy array [Cout,Kh,Kw,Cin] fp32."""
    w = np.ascontiguousarray(w_ohwi, dtype=np.float32)
    cout, kh, kw, cin = w.shape
    h = ctypes.c_void_p()
    _check(lib().nm_prune(w.ctypes.data, cout, kh, kw, cin, n, m, tile, value_dtype,
                          ctypes.byref(h)))
    return Packed(h, cout, kh, kw, cin, n, m, tile, value_dtype)


def nm_packed_dims(wp: Packed):
    a, b, c, d = (ctypes.c_int() for _ in range(4))
    _check(lib().nm_packed_dims(wp.handle, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c),
                                ctypes.byref(d)))
    return a.value, b.value, c.value, d.value


def nm_packed_indices(wp: Packed) -> np.ndarray:
    n_tiles, groups, n, _ = nm_packed_dims(wp)
    out = np.empty((n_tiles, groups, n), dtype=np.int32)
    _check(lib().nm_packed_indices(wp.handle, out.ctypes.data))
    return out


def nm_packed_values(wp: Packed) -> np.ndarray:
    n_tiles, _, _, kprime = nm_packed_dims(wp)
    out = np.empty((n_tiles, kprime, wp.tile), dtype=np.float32)
    _check(lib().nm_packed_values(wp.handle, out.ctypes.data))
    return out


def nm_packed_mask(wp: Packed) -> np.ndarray:
    out = np.empty((wp.cout, wp.K), dtype=np.uint8)
    _check(lib().nm_packed_mask(wp.handle, out.ctypes.data))
    return out


def nm_packed_scale(wp: Packed) -> float:
    """The power-of-two scale of an fp8 handle (stored value = weight * scale); 1 otherwise."""
    v = ctypes.c_float(0)
    _check(lib().nm_packed_scale(wp.handle, ctypes.byref(v)))
    return v.value


def _out_dtype(x):
    """fp32 -> fp32, bf16 -> bf16, E4M3 -> bf16."""
    import torch
    return torch.bfloat16 if x.dtype == torch.float8_e4m3fn else x.dtype


def _stream_ptr(stream) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def out_shape(x_shape, wp: Packed, stride, pad, dil):
    b, h, w, _ = x_shape
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dil)
    if sh < 1 or sw < 1:
        raise NMError(NM_ERR_ARG, "stride must be >= 1")
    ho = (h + 2 * ph - dh * (wp.kh - 1) - 1) // sh + 1
    wo = (w + 2 * pw - dw * (wp.kw - 1) - 1) // sw + 1
    return (b, ho, wo, wp.cout)


def _check_out(y, shp, x):
    """A caller-supplied output must cover exactly what the kernel will write (the
    library itself checks the dtype pair)."""
    if tuple(y.shape) != tuple(shp) or not y.is_cuda or y.device != x.device or not y.is_contiguous():
        raise ValueError(f"y must be a contiguous device tensor of shape {tuple(shp)} on {x.device}")


def nm_conv2d(x, wp: Packed, bias=None, stride=1, pad=0, dil=1, relu=False, y=None, stream=None):
    """x: device tensor NHWC [B,H,W,Cin] (fp32 or bf16, contiguous); bias: device
    fp32 [Cout] or None; y: optional preallocated output.  Enqueues on `stream`
    (default: torch's current stream) and returns y."""
    import torch
    if not x.is_cuda or not x.is_contiguous():
        raise ValueError("x must be a contiguous device tensor")
    b, h, w, cin = x.shape
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dil)
    shp = out_shape(x.shape, wp, stride, pad, dil)
    if min(shp) < 1:
        raise NMError(-2, "output would be empty")
    if y is None:
        y = torch.empty(shp, dtype=_out_dtype(x), device=x.device)
    else:
        _check_out(y, shp, x)
    bptr = None
    if bias is not None:
        if bias.dtype != torch.float32 or not bias.is_cuda or not bias.is_contiguous():
            raise ValueError("bias must be a contiguous fp32 device tensor")
        bptr = bias.data_ptr()
    _check(lib().nm_conv2d(x.data_ptr(), _dtype_code(x), b, h, w, cin, wp.handle, bptr,
                           sh, sw, ph, pw, dh, dw, int(bool(relu)), y.data_ptr(), _dtype_code(y),
                           _stream_ptr(stream)))
    return y


def nm_conv2d_static(x, wp: Packed, residual, bias, stride, pad, dil, relu, y, stream=None):
    """nm_conv2d_res through the entry point that allocates nothing; y must be given."""
    return nm_conv2d_res(x, wp, residual, bias, stride, pad, dil, relu, y=y, stream=stream, _entry="nm_conv2d_static")


def nm_conv2d_res(x, wp: Packed, residual, bias=None, stride=1, pad=0, dil=1, relu=False, y=None,
                  stream=None, _entry="nm_conv2d_res"):
    """nm_conv2d with a residual (device tensor shaped and typed like the output, or None)
    added before the activation."""
    import torch
    if not x.is_cuda or not x.is_contiguous():
        raise ValueError("x must be a contiguous device tensor")
    b, h, w, cin = x.shape
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dil)
    shp = out_shape(x.shape, wp, stride, pad, dil)
    if min(shp) < 1:
        raise NMError(-2, "output would be empty")
    if y is None:
        y = torch.empty(shp, dtype=_out_dtype(x), device=x.device)
    else:
        _check_out(y, shp, x)
    rptr = None
    if residual is not None:
        if (tuple(residual.shape) != tuple(shp) or residual.dtype != y.dtype or not residual.is_cuda
                or not residual.is_contiguous()):
            raise ValueError("residual must be a contiguous device tensor shaped and typed like the output")
        rptr = residual.data_ptr()
    bptr = None
    if bias is not None:
        if bias.dtype != torch.float32 or not bias.is_cuda or not bias.is_contiguous():
            raise ValueError("bias must be a contiguous fp32 device tensor")
        bptr = bias.data_ptr()
    _check(getattr(lib(), _entry)(x.data_ptr(), _dtype_code(x), b, h, w, cin, wp.handle, bptr, rptr,
                               sh, sw, ph, pw, dh, dw, int(bool(relu)), y.data_ptr(), _dtype_code(y),
                               _stream_ptr(stream)))
    return y


def nm_maxpool2d(x, k: int, stride: int, pad: int, y=None, stream=None):
    """Max pooling of a contiguous NHWC device tensor (fp32 or bf16)."""
    import torch
    if not x.is_cuda or not x.is_contiguous():
        raise ValueError("x must be a contiguous device tensor")
    b, h, w, c = x.shape
    ho, wo = (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1
    if y is None:
        if min(ho, wo) < 1:
            raise NMError(-2, "output would be empty")
        y = torch.empty((b, ho, wo, c), dtype=x.dtype, device=x.device)
    _check(lib().nm_maxpool2d(x.data_ptr(), _dtype_code(x), b, h, w, c, k, stride, pad, y.data_ptr(),
                              _stream_ptr(stream)))
    return y


def nm_avgpool_global(x, y=None, stream=None):
    """Mean over all positions of a contiguous NHWC device tensor: [B,H,W,C] -> [B,C]."""
    import torch
    if not x.is_cuda or not x.is_contiguous():
        raise ValueError("x must be a contiguous device tensor")
    b, h, w, c = x.shape
    if y is None:
        y = torch.empty((b, c), dtype=x.dtype, device=x.device)
    _check(lib().nm_avgpool_global(x.data_ptr(), _dtype_code(x), b, h, w, c, y.data_ptr(),
                                   _stream_ptr(stream)))
    return y


def nm_im2col(x, kh: int, kw: int, stride=1, pad=0, dil=1, a=None, stream=None):
    """The im2col matrix of a contiguous NHWC device tensor, as the NHWC tensor
    [B,Hout,Wout,kh*kw*Cin] (k order (kh, kw, ci))."""
    import torch
    if not x.is_cuda or not x.is_contiguous():
        raise ValueError("x must be a contiguous device tensor")
    b, h, w, c = x.shape
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dil)
    ho = (h + 2 * ph - dh * (kh - 1) - 1) // sh + 1
    wo = (w + 2 * pw - dw * (kw - 1) - 1) // sw + 1
    if a is None:
        if min(ho, wo) < 1:
            raise NMError(-2, "output would be empty")
        a = torch.empty((b, ho, wo, kh * kw * c), dtype=x.dtype, device=x.device)
    _check(lib().nm_im2col(x.data_ptr(), _dtype_code(x), b, h, w, c, kh, kw, sh, sw, ph, pw, dh, dw,
                           a.data_ptr(), _stream_ptr(stream)))
    return a


def nm_stream_floor(x, y, stream=None):
    """Reads all of x and overwrites all of y (contents unspecified) with one plain
    streaming kernel: the cost of a layer's traffic alone."""
    if not (x.is_cuda and y.is_cuda and x.is_contiguous() and y.is_contiguous()):
        raise ValueError("x and y must be contiguous device tensors")
    _check(lib().nm_stream_floor(x.data_ptr(), x.numel() * x.element_size(), y.data_ptr(),
                                 y.numel() * y.element_size(), _stream_ptr(stream)))


def nm_autotune(x_dtype: int, b: int, h: int, w: int, cin: int, wp: Packed, has_bias=True,
                stride=1, pad=0, dil=1, relu=True, y_dtype: Optional[int] = None, stream=None):
    """Returns (chosen variant id, its time in ms)."""
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dil)
    v, ms = ctypes.c_int(-1), ctypes.c_float(0)
    _check(lib().nm_autotune(x_dtype, b, h, w, cin, wp.handle, int(bool(has_bias)), sh, sw, ph, pw,
                             dh, dw, int(bool(relu)),
                             (NM_BF16 if x_dtype == NM_F8E4M3 else x_dtype) if y_dtype is None else y_dtype,
                             _stream_ptr(stream), ctypes.byref(v), ctypes.byref(ms)))
    return v.value, ms.value


def nm_autotune_tile(w_ohwi: np.ndarray, n: int, m: int, tiles, x_dtype: int, b: int, h: int, w: int,
                     has_bias=True, stride=1, pad=0, dil=1, relu=True, value_dtype: Optional[int] = None,
                     stream=None):
    """Prunes at every candidate tile size, tunes each and returns
    (handle of the fastest, its tile size, [ms per candidate])."""
    wt = np.ascontiguousarray(w_ohwi, dtype=np.float32)
    cout, kh, kw, cin = wt.shape
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dil)
    vd = x_dtype if value_dtype is None else value_dtype
    cand = (ctypes.c_int * len(tiles))(*[int(t) for t in tiles])
    ms = (ctypes.c_float * len(tiles))()
    hnd, best = ctypes.c_void_p(), ctypes.c_int(0)
    _check(lib().nm_autotune_tile(wt.ctypes.data, cout, kh, kw, cin, n, m, cand, len(tiles), vd,
                                  x_dtype, b, h, w, int(bool(has_bias)), sh, sw, ph, pw, dh, dw,
                                  int(bool(relu)), x_dtype, _stream_ptr(stream),
                                  ctypes.byref(hnd), ctypes.byref(best), ms))
    return Packed(hnd, cout, kh, kw, cin, n, m, best.value, vd), best.value, list(ms)


def nm_cache_save(path: str):
    _check(lib().nm_cache_save(path.encode()))


def nm_cache_load(path: str):
    _check(lib().nm_cache_load(path.encode()))


def nm_workspace_free():
    _check(lib().nm_workspace_free())


def nm_cache_clear():
    _check(lib().nm_cache_clear())


def nm_cache_size() -> int:
    return _check(lib().nm_cache_size())


def nm_force_variant(v: int):
    _check(lib().nm_force_variant(v))


def nm_variant_legal(v: int, wp: Packed, x_dtype: int = NM_F32, y_dtype: int = NM_F32) -> bool:
    return _check(lib().nm_variant_legal(v, wp.handle, x_dtype, y_dtype)) == 1
