"""ctypes front end of the CPU oracle (focused_conv_oracle.c).

Test infrastructure only: the tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this; the product package never does.  It takes
and returns numpy arrays and does argument marshalling only - every number comes
from the C file, which follows Sec. III-A / III-B of the paper.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "focused_conv_oracle.c")
_LIB = os.path.join(_HERE, "libfc_oracle.so")

F32, BF16, F16, FP8 = 0, 1, 2, 3
RULE_CENTRE, RULE_ANY, RULE_ALL = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over the image rows)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
             "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


class _Conv(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in (
        "n", "h", "w", "c_in", "c_out", "kh", "kw", "stride_h", "stride_w",
        "pad_h", "pad_w", "dil_h", "dil_w", "dtype", "relu")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.fco_out_dim.restype = ctypes.c_int32
        L.fco_out_dim.argtypes = [ctypes.c_int32] * 5
        L.fco_num_threads.restype = ctypes.c_int32
        L.fco_mask_downsample.restype = ctypes.c_int32
        L.fco_mask_downsample.argtypes = [ctypes.c_void_p] + [ctypes.c_int32] * 11 + [ctypes.c_void_p]
        L.fco_active_index_compact.restype = ctypes.c_int64
        L.fco_active_index_compact.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
        L.fco_focused_gconv2d.restype = ctypes.c_int32
        L.fco_focused_gconv2d.argtypes = [ctypes.POINTER(_Conv), ctypes.c_int32] + [ctypes.c_void_p] * 5
        L.fco_active_index_compact_tiled.restype = ctypes.c_int64
        L.fco_active_index_compact_tiled.argtypes = [ctypes.c_void_p] + [ctypes.c_int32] * 5 + [ctypes.c_void_p]
        L.fco_widen.restype = ctypes.c_int32
        L.fco_widen.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
        L.fco_narrow_fp8.restype = ctypes.c_int32
        L.fco_narrow_fp8.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
        L.fco_focused_conv2d.restype = ctypes.c_int32
        L.fco_focused_conv2d.argtypes = [ctypes.POINTER(_Conv)] + [ctypes.c_void_p] * 5
        L.fco_focused_conv2d_at.restype = ctypes.c_int32
        L.fco_focused_conv2d_at.argtypes = ([ctypes.POINTER(_Conv)] + [ctypes.c_void_p] * 5
                                            + [ctypes.c_int64, ctypes.c_void_p])
        L.fco_mask_downsample_rule.restype = ctypes.c_int32
        L.fco_mask_downsample_rule.argtypes = [ctypes.c_void_p] + [ctypes.c_int32] * 12 + [ctypes.c_void_p]
        L.fco_focused_conv2d_labelled.restype = ctypes.c_int32
        L.fco_focused_conv2d_labelled.argtypes = [ctypes.POINTER(_Conv)] + [ctypes.c_void_p] * 6
        L.fco_focused_dwconv2d.restype = ctypes.c_int32
        L.fco_focused_dwconv2d.argtypes = [ctypes.POINTER(_Conv)] + [ctypes.c_void_p] * 5
        L.fco_focused_dwconv2d_at.restype = ctypes.c_int32
        L.fco_focused_dwconv2d_at.argtypes = ([ctypes.POINTER(_Conv)] + [ctypes.c_void_p] * 5
                                              + [ctypes.c_int64, ctypes.c_void_p])
        _lib = L
    return _lib


@dataclass
class ConvShape:
    n: int
    h: int
    w: int
    c_in: int
    c_out: int
    kh: int = 3
    kw: int = 3
    stride: tuple = (1, 1)
    pad: tuple = (1, 1)
    dil: tuple = (1, 1)
    relu: bool = False


def out_dim(size: int, k: int, stride: int, pad: int, dil: int = 1) -> int:
    return int(lib().fco_out_dim(size, k, stride, pad, dil))


def out_dims(s: ConvShape):
    return (out_dim(s.h, s.kh, s.stride[0], s.pad[0], s.dil[0]),
            out_dim(s.w, s.kw, s.stride[1], s.pad[1], s.dil[1]))


def num_threads() -> int:
    return int(lib().fco_num_threads())


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _storage(a: np.ndarray, dtype: int) -> np.ndarray:
    """x / w arrive as float32 (dtype F32), as raw uint16 bit patterns, or as raw bytes (FP8)."""
    want = np.float32 if dtype == F32 else np.uint8 if dtype == FP8 else np.uint16
    if a.dtype != want:
        raise TypeError("storage dtype %s does not match code %d" % (a.dtype, dtype))
    return np.ascontiguousarray(a)


def widen(stored: np.ndarray, dtype: int) -> np.ndarray:
    """The values a storage array holds, as float64 (exact)."""
    a = _storage(stored, dtype)
    out = np.empty(a.shape, dtype=np.float64)
    if lib().fco_widen(dtype, _ptr(a), a.size, _ptr(out)) != 0:
        raise ValueError("dtype %r" % (dtype,))
    return out


def narrow_fp8(values: np.ndarray) -> np.ndarray:
    """The 8-bit (E4M3) codes a layer with 8-bit output stores for these values: nearest value,
    ties to the even code, saturating at 448."""
    v = np.ascontiguousarray(values, dtype=np.float64)
    out = np.empty(v.shape, dtype=np.uint8)
    if lib().fco_narrow_fp8(_ptr(v), v.size, _ptr(out)) != 0:
        raise ValueError("narrow_fp8")
    return out


def _mask(m, shape):
    if m is None:
        return None
    m = np.ascontiguousarray(m, dtype=np.uint8)
    if m.shape != tuple(shape):
        raise ValueError("mask shape %s, expected %s" % (m.shape, tuple(shape)))
    return m


def mask_downsample(mask_in: np.ndarray, kh, kw, stride, pad, dil=(1, 1)) -> np.ndarray:
    n, h, w = mask_in.shape
    m = _mask(mask_in, (n, h, w))
    ho = out_dim(h, kh, stride[0], pad[0], dil[0])
    wo = out_dim(w, kw, stride[1], pad[1], dil[1])
    out = np.empty((n, ho, wo), dtype=np.uint8)
    rc = lib().fco_mask_downsample(_ptr(m), n, h, w, kh, kw, stride[0], stride[1],
                                   pad[0], pad[1], dil[0], dil[1], _ptr(out))
    if rc != 0:
        raise ValueError("fco_mask_downsample rc=%d" % rc)
    return out


def mask_downsample_rule(mask_in: np.ndarray, kh, kw, stride, pad, dil=(1, 1), rule: int = RULE_CENTRE) -> np.ndarray:
    """Labels of a layer's patches under the centre-tap, any-pixel or all-pixels rule."""
    n, h, w = mask_in.shape
    m = _mask(mask_in, (n, h, w))
    ho = out_dim(h, kh, stride[0], pad[0], dil[0])
    wo = out_dim(w, kw, stride[1], pad[1], dil[1])
    out = np.empty((n, ho, wo), dtype=np.uint8)
    rc = lib().fco_mask_downsample_rule(_ptr(m), n, h, w, kh, kw, stride[0], stride[1],
                                        pad[0], pad[1], dil[0], dil[1], rule, _ptr(out))
    if rc != 0:
        raise ValueError("fco_mask_downsample_rule rc=%d" % rc)
    return out


def active_index_compact(mask: np.ndarray):
    m = np.ascontiguousarray(mask, dtype=np.uint8).reshape(-1)
    idx = np.empty(m.size, dtype=np.int32)
    cnt = int(lib().fco_active_index_compact(_ptr(m), m.size, _ptr(idx)))
    return idx[:cnt].copy(), cnt


def active_index_compact_tiled(mask, tile_h: int, tile_w: int):
    """(idx, count): the kept positions of a [n, ho, wo] mask in tile order (tiles row-major,
    positions row-major inside a tile)."""
    m = np.ascontiguousarray(mask, dtype=np.uint8)
    n, ho, wo = m.shape
    idx = np.empty(m.size, dtype=np.int32)
    cnt = int(lib().fco_active_index_compact_tiled(_ptr(m), n, ho, wo, tile_h, tile_w, _ptr(idx)))
    if cnt < 0:
        raise ValueError("bad sizes")
    return idx[:cnt].copy(), cnt


def _conv_struct(s: ConvShape, dtype: int) -> _Conv:
    return _Conv(s.n, s.h, s.w, s.c_in, s.c_out, s.kh, s.kw, s.stride[0], s.stride[1],
                 s.pad[0], s.pad[1], s.dil[0], s.dil[1], dtype, 1 if s.relu else 0)


def _check_operands(s: ConvShape, x, w, bias, mask_in, dtype):
    x = _storage(x, dtype)
    w = _storage(w, dtype)
    if x.shape != (s.n, s.h, s.w, s.c_in):
        raise ValueError("x shape %s" % (x.shape,))
    if w.shape != (s.c_out, s.kh, s.kw, s.c_in):
        raise ValueError("w shape %s" % (w.shape,))
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        if bias.shape != (s.c_out,):
            raise ValueError("bias shape %s" % (bias.shape,))
    return x, w, bias, _mask(mask_in, (s.n, s.h, s.w))


def focused_conv2d(s: ConvShape, x, w, bias=None, mask_in=None, dtype: int = F32) -> np.ndarray:
    """Whole layer; returns float64 [N, Ho, Wo, C_out]."""
    x, w, bias, m = _check_operands(s, x, w, bias, mask_in, dtype)
    ho, wo = out_dims(s)
    out = np.empty((s.n, ho, wo, s.c_out), dtype=np.float64)
    c = _conv_struct(s, dtype)
    rc = lib().fco_focused_conv2d(ctypes.byref(c), _ptr(x), _ptr(m), _ptr(w), _ptr(bias), _ptr(out))
    if rc != 0:
        raise ValueError("fco_focused_conv2d rc=%d" % rc)
    return out


def focused_conv2d_labelled(s: ConvShape, x, w, labels, bias=None, mask_in=None, dtype: int = F32) -> np.ndarray:
    """Whole layer with the kept positions given as labels [N, Ho, Wo]; float64 [N, Ho, Wo, C_out]."""
    x, w, bias, m = _check_operands(s, x, w, bias, mask_in, dtype)
    ho, wo = out_dims(s)
    lab = _mask(labels, (s.n, ho, wo))
    out = np.empty((s.n, ho, wo, s.c_out), dtype=np.float64)
    c = _conv_struct(s, dtype)
    rc = lib().fco_focused_conv2d_labelled(ctypes.byref(c), _ptr(x), _ptr(m), _ptr(lab), _ptr(w), _ptr(bias),
                                           _ptr(out))
    if rc != 0:
        raise ValueError("fco_focused_conv2d_labelled rc=%d" % rc)
    return out


def focused_conv2d_at(s: ConvShape, x, w, positions, bias=None, mask_in=None,
                      dtype: int = F32) -> np.ndarray:
    """Rows of the layer's output at the given flat positions; float64 [len, C_out]."""
    x, w, bias, m = _check_operands(s, x, w, bias, mask_in, dtype)
    pos = np.ascontiguousarray(positions, dtype=np.int64).reshape(-1)
    out = np.empty((pos.size, s.c_out), dtype=np.float64)
    c = _conv_struct(s, dtype)
    rc = lib().fco_focused_conv2d_at(ctypes.byref(c), _ptr(x), _ptr(m), _ptr(w), _ptr(bias),
                                     _ptr(pos), pos.size, _ptr(out))
    if rc != 0:
        raise ValueError("fco_focused_conv2d_at rc=%d" % rc)
    return out


def focused_gconv2d(s: ConvShape, groups: int, x, w, bias=None, mask_in=None, dtype: int = F32) -> np.ndarray:
    """The grouped layer: w is [C_out, KH, KW, C_in / groups]; out float64 NHWC."""
    x = _storage(x, dtype)
    w = _storage(w, dtype)
    if groups <= 0 or s.c_in % groups or s.c_out % groups:
        raise ValueError("channel counts are not multiples of groups")
    if x.shape != (s.n, s.h, s.w, s.c_in) or w.shape != (s.c_out, s.kh, s.kw, s.c_in // groups):
        raise ValueError("operand shapes")
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    m = _mask(mask_in, (s.n, s.h, s.w))
    ho, wo = out_dims(s)
    out = np.empty((s.n, ho, wo, s.c_out), dtype=np.float64)
    c = _conv_struct(s, dtype)
    rc = lib().fco_focused_gconv2d(ctypes.byref(c), groups, _ptr(x), _ptr(m), _ptr(w), _ptr(bias), _ptr(out))
    if rc != 0:
        raise ValueError("fco_focused_gconv2d failed: %d" % rc)
    return out


def _check_dw_operands(s: ConvShape, x, w, bias, mask_in, dtype):
    if s.c_in != s.c_out:
        raise ValueError("depthwise layer: c_in %d != c_out %d" % (s.c_in, s.c_out))
    x = _storage(x, dtype)
    w = _storage(w, dtype)
    if x.shape != (s.n, s.h, s.w, s.c_in):
        raise ValueError("x shape %s" % (x.shape,))
    if w.shape != (s.c_out, s.kh, s.kw):
        raise ValueError("w shape %s" % (w.shape,))
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        if bias.shape != (s.c_out,):
            raise ValueError("bias shape %s" % (bias.shape,))
    return x, w, bias, _mask(mask_in, (s.n, s.h, s.w))


def focused_dwconv2d(s: ConvShape, x, w, bias=None, mask_in=None, dtype: int = F32) -> np.ndarray:
    """Depthwise layer (w is [C, KH, KW]); returns float64 [N, Ho, Wo, C]."""
    x, w, bias, m = _check_dw_operands(s, x, w, bias, mask_in, dtype)
    ho, wo = out_dims(s)
    out = np.empty((s.n, ho, wo, s.c_out), dtype=np.float64)
    c = _conv_struct(s, dtype)
    rc = lib().fco_focused_dwconv2d(ctypes.byref(c), _ptr(x), _ptr(m), _ptr(w), _ptr(bias), _ptr(out))
    if rc != 0:
        raise ValueError("fco_focused_dwconv2d rc=%d" % rc)
    return out


def focused_dwconv2d_at(s: ConvShape, x, w, positions, bias=None, mask_in=None,
                        dtype: int = F32) -> np.ndarray:
    """Rows of the depthwise layer's output at the given flat positions; float64 [len, C]."""
    x, w, bias, m = _check_dw_operands(s, x, w, bias, mask_in, dtype)
    pos = np.ascontiguousarray(positions, dtype=np.int64).reshape(-1)
    out = np.empty((pos.size, s.c_out), dtype=np.float64)
    c = _conv_struct(s, dtype)
    rc = lib().fco_focused_dwconv2d_at(ctypes.byref(c), _ptr(x), _ptr(m), _ptr(w), _ptr(bias),
                                       _ptr(pos), pos.size, _ptr(out))
    if rc != 0:
        raise ValueError("fco_focused_dwconv2d_at rc=%d" % rc)
    return out
