"""Python binding of the C ABI in include/focused_conv.h.

Argument marshalling only: every step of the path runs in the HIP kernels of
libfocused_conv.so.  PyTorch supplies device memory and the stream.  There is
no fallback - if the library is not built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfocused_conv.so")

F32, BF16, F16, FP8 = 0, 1, 2, 3
RELU, SKIP_ZERO_FILL, WORKSPACE_READY, COMPACT_OUT, COMPACT_IN, PACKED_MASKS, RESIDENT_WEIGHTS = 1, 2, 4, 8, 16, 32, 64
RULE_CENTRE, RULE_ANY, RULE_ALL = 0, 1, 2
WORKSPACE_COUNTER_BYTES = 2048
NOALLOC_SCRATCH_BYTES = 40 << 20

FUNCTIONS = ("fc_status_string", "fc_out_dims", "fc_workspace_bytes", "fc_compact_workspace_bytes",
             "fc_mask_downsample", "fc_mask_downsample_rule", "fc_active_index_compact",
             "fc_compact_tiled_workspace_bytes", "fc_active_index_compact_tiled", "fc_mask_pyramid_dims",
             "fc_mask_pyramid_workspace_bytes", "fc_mask_pyramid", "fc_focused_conv2d", "fc_focused_gconv2d",
             "fc_noalloc_init", "fc_focused_conv2d_noalloc", "fc_calibrate_mfma", "fc_calibrate_copy", "fc_calibrate_issue",
             "fc_packed_mask_bytes", "fc_mask_pack", "fc_mask_downsample_packed", "fc_active_index_compact_packed",
             "fc_mask_pyramid_packed",
             "fc_expand_group_weights",
             "fc_focused_dwconv2d",
             "fc_maxpool2d", "fc_maxpool2d_masked")
MAX_PYRAMID_LEVELS = 8


class FcError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__("%s failed: %s" % (what, status_string(status)))


class ConvDesc(ctypes.Structure):
    """Mirror of fc_conv_desc."""
    _fields_ = [(k, ctypes.c_int32) for k in (
        "n", "h", "w", "c_in", "c_out", "kh", "kw", "stride_h", "stride_w",
        "pad_h", "pad_w", "dil_h", "dil_w", "in_dtype", "out_dtype")] + [("flags", ctypes.c_uint32)]


class MaskStep(ctypes.Structure):
    """Mirror of fc_mask_step: the window that takes one pyramid level to the next."""
    _fields_ = [(k, ctypes.c_int32) for k in ("kh", "kw", "stride_h", "stride_w", "pad_h", "pad_w", "dil_h", "dil_w")]


def conv_desc(n, h, w, c_in, c_out, k=(3, 3), stride=(1, 1), pad=(1, 1), dil=(1, 1),
              in_dtype=BF16, out_dtype=None, flags=0) -> ConvDesc:
    return ConvDesc(n, h, w, c_in, c_out, k[0], k[1], stride[0], stride[1], pad[0], pad[1],
                    dil[0], dil[1], in_dtype,
                    (BF16 if in_dtype == FP8 else in_dtype) if out_dtype is None else out_dtype, flags)


_lib = None


def lib():
    """The loaded C library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "%s is missing: build it with `python -m paper_2207_10741_amd.build` "
                "(hipcc --offload-arch=gfx950); there is no CPU fallback" % LIB_PATH)
        # PyTorch ships its own HIP runtime; load it first so that this library binds to the same
        # one (two runtimes in one process do not share the device)
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        L.fc_status_string.restype = ctypes.c_char_p
        L.fc_status_string.argtypes = [i32]
        L.fc_out_dims.restype = i32
        L.fc_out_dims.argtypes = [ctypes.POINTER(ConvDesc), ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.fc_workspace_bytes.restype = i32
        L.fc_workspace_bytes.argtypes = [ctypes.POINTER(ConvDesc), ctypes.POINTER(ctypes.c_size_t)]
        L.fc_compact_workspace_bytes.restype = i32
        L.fc_compact_workspace_bytes.argtypes = [i64, ctypes.POINTER(ctypes.c_size_t)]
        L.fc_mask_downsample.restype = i32
        L.fc_mask_downsample.argtypes = [vp] + [i32] * 11 + [vp, vp]
        L.fc_mask_downsample_rule.restype = i32
        L.fc_mask_downsample_rule.argtypes = [vp] + [i32] * 12 + [vp, vp]
        L.fc_active_index_compact.restype = i32
        L.fc_active_index_compact.argtypes = [vp, i64, vp, vp, vp, ctypes.c_size_t, vp]
        L.fc_compact_tiled_workspace_bytes.restype = i32
        L.fc_compact_tiled_workspace_bytes.argtypes = [i32] * 5 + [ctypes.POINTER(ctypes.c_size_t)]
        L.fc_active_index_compact_tiled.restype = i32
        L.fc_active_index_compact_tiled.argtypes = [vp] + [i32] * 5 + [vp, vp, vp, ctypes.c_size_t, vp]
        L.fc_mask_pyramid_dims.restype = i32
        L.fc_mask_pyramid_dims.argtypes = [i32, i32, i32, ctypes.POINTER(MaskStep), ctypes.POINTER(i32),
                                           ctypes.POINTER(i32)]
        L.fc_mask_pyramid_workspace_bytes.restype = i32
        L.fc_mask_pyramid_workspace_bytes.argtypes = [i32, i32, i32, i32, ctypes.POINTER(MaskStep),
                                                      ctypes.POINTER(ctypes.c_size_t)]
        L.fc_mask_pyramid.restype = i32
        L.fc_mask_pyramid.argtypes = [vp, i32, i32, i32, i32, ctypes.POINTER(MaskStep), ctypes.POINTER(vp),
                                      ctypes.POINTER(vp), ctypes.POINTER(vp), vp, ctypes.c_size_t, vp]
        L.fc_packed_mask_bytes.restype = ctypes.c_size_t
        L.fc_packed_mask_bytes.argtypes = [i64]
        L.fc_mask_pack.restype = i32
        L.fc_mask_pack.argtypes = [vp, i64, vp, vp]
        L.fc_mask_downsample_packed.restype = i32
        L.fc_mask_downsample_packed.argtypes = [vp] + [i32] * 11 + [vp, vp]
        L.fc_active_index_compact_packed.restype = i32
        L.fc_active_index_compact_packed.argtypes = [vp, i64, vp, vp, vp, ctypes.c_size_t, vp]
        L.fc_mask_pyramid_packed.restype = i32
        L.fc_mask_pyramid_packed.argtypes = [vp, i32, i32, i32, i32, i32, ctypes.POINTER(MaskStep), ctypes.POINTER(vp),
                                             ctypes.POINTER(vp), ctypes.POINTER(vp), vp, ctypes.c_size_t, vp]
        L.fc_focused_conv2d.restype = i32
        L.fc_focused_conv2d.argtypes = [ctypes.POINTER(ConvDesc)] + [vp] * 9 + [ctypes.c_size_t, vp]
        L.fc_noalloc_init.restype = i32
        L.fc_noalloc_init.argtypes = []
        L.fc_focused_conv2d_noalloc.restype = i32
        L.fc_focused_conv2d_noalloc.argtypes = [ctypes.POINTER(ConvDesc)] + [vp] * 6
        L.fc_calibrate_mfma.restype = i32
        L.fc_calibrate_mfma.argtypes = [i32, i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.fc_calibrate_copy.restype = i32
        L.fc_calibrate_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.fc_calibrate_issue.restype = i32
        L.fc_calibrate_issue.argtypes = [i32, i32, i32, i32, vp, ctypes.c_size_t, vp, vp, vp]
        L.fc_focused_gconv2d.restype = i32
        L.fc_focused_gconv2d.argtypes = [ctypes.POINTER(ConvDesc), i32] + [vp] * 9 + [ctypes.c_size_t, vp]
        L.fc_expand_group_weights.restype = i32
        L.fc_expand_group_weights.argtypes = [i32] * 6 + [vp, vp, vp]
        L.fc_focused_dwconv2d.restype = i32
        L.fc_focused_dwconv2d.argtypes = [ctypes.POINTER(ConvDesc)] + [vp] * 6
        L.fc_maxpool2d.restype = i32
        L.fc_maxpool2d.argtypes = [vp] + [i32] * 8 + [vp, vp]
        L.fc_maxpool2d_masked.restype = i32
        L.fc_maxpool2d_masked.argtypes = [vp] + [i32] * 8 + [vp, vp, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().fc_status_string(int(status)).decode()


def _check(status: int, what: str):
    if status != 0:
        raise FcError(status, what)


def out_dims(desc: ConvDesc):
    ho, wo = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().fc_out_dims(ctypes.byref(desc), ctypes.byref(ho), ctypes.byref(wo)), "fc_out_dims")
    return ho.value, wo.value


def workspace_bytes(desc: ConvDesc) -> int:
    b = ctypes.c_size_t()
    _check(lib().fc_workspace_bytes(ctypes.byref(desc), ctypes.byref(b)), "fc_workspace_bytes")
    return b.value


def compact_workspace_bytes(m: int) -> int:
    b = ctypes.c_size_t()
    _check(lib().fc_compact_workspace_bytes(int(m), ctypes.byref(b)), "fc_compact_workspace_bytes")
    return b.value


# ---- device-side calls (torch tensors in, torch tensors out) ----------------

def _torch():
    import torch
    return torch


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = _torch().cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def torch_dtype(code: int):
    torch = _torch()
    return {F32: torch.float32, BF16: torch.bfloat16, F16: torch.float16, FP8: torch.float8_e4m3fn}[code]


def _require_cuda(*tensors):
    for t in tensors:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError("tensors must be contiguous device tensors")


def mask_downsample(mask_in, k=(3, 3), stride=(1, 1), pad=(1, 1), dil=(1, 1), out=None, stream=None):
    """fc_mask_downsample: uint8 [N,H,W] -> uint8 [N,Ho,Wo] (0/1)."""
    torch = _torch()
    _require_cuda(mask_in, out)
    n, h, w = mask_in.shape
    d = conv_desc(n, h, w, 1, 1, k, stride, pad, dil, F32)
    ho, wo = out_dims(d)
    if out is None:
        out = torch.empty((n, ho, wo), dtype=torch.uint8, device=mask_in.device)
    _check(lib().fc_mask_downsample(_ptr(mask_in), n, h, w, k[0], k[1], stride[0], stride[1], pad[0], pad[1],
                                    dil[0], dil[1], _ptr(out), _stream(stream)), "fc_mask_downsample")
    return out


def mask_downsample_rule(mask_in, k=(3, 3), stride=(1, 1), pad=(1, 1), dil=(1, 1), rule=RULE_CENTRE, out=None,
                         stream=None):
    """fc_mask_downsample_rule: patch labels by the centre tap, any pixel or all pixels of the window."""
    torch = _torch()
    _require_cuda(mask_in, out)
    n, h, w = mask_in.shape
    d = conv_desc(n, h, w, 1, 1, k, stride, pad, dil, F32)
    ho, wo = out_dims(d)
    if out is None:
        out = torch.empty((n, ho, wo), dtype=torch.uint8, device=mask_in.device)
    _check(lib().fc_mask_downsample_rule(_ptr(mask_in), n, h, w, k[0], k[1], stride[0], stride[1], pad[0], pad[1],
                                         dil[0], dil[1], rule, _ptr(out), _stream(stream)),
           "fc_mask_downsample_rule")
    return out


def _steps_array(steps):
    arr = (MaskStep * len(steps))()
    for i, (k, stride, pad, dil) in enumerate(steps):
        arr[i] = MaskStep(k[0], k[1], stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])
    return arr


def mask_pyramid_dims(h: int, w: int, steps):
    """fc_mask_pyramid_dims: [(h_l, w_l)] for steps = [(k, stride, pad, dil), ...] (pairs each)."""
    arr = _steps_array(steps)
    hs, ws = (ctypes.c_int32 * len(steps))(), (ctypes.c_int32 * len(steps))()
    _check(lib().fc_mask_pyramid_dims(h, w, len(steps), arr, hs, ws), "fc_mask_pyramid_dims")
    return [(int(a), int(b)) for a, b in zip(hs, ws)]


def packed_mask_words(m: int) -> int:
    """64-bit words of a packed mask of m pixels."""
    return lib().fc_packed_mask_bytes(int(m)) // 8


def _packed_tensor(m: int, device):
    torch = _torch()
    return torch.empty((max(packed_mask_words(m), 2),), dtype=torch.int64, device=device)   # (at least 16 bytes)


def mask_pack(mask, out=None, stream=None):
    """fc_mask_pack: uint8 [...] -> int64 words, one bit per pixel (bit p % 64 of word p // 64)."""
    _require_cuda(mask, out)
    m = mask.numel()
    if out is None:
        out = _packed_tensor(m, mask.device)
    _check(lib().fc_mask_pack(_ptr(mask), m, _ptr(out), _stream(stream)), "fc_mask_pack")
    return out


def mask_downsample_packed(bits_in, shape, k=(3, 3), stride=(1, 1), pad=(1, 1), dil=(1, 1), out=None, stream=None):
    """fc_mask_downsample_packed: packed [N,H,W] (shape = (N, H, W)) -> packed [N,Ho,Wo]; returns (bits, (N, Ho, Wo))."""
    _require_cuda(bits_in, out)
    n, h, w = shape
    d = conv_desc(n, h, w, 1, 1, k, stride, pad, dil, F32)
    ho, wo = out_dims(d)
    if out is None:
        out = _packed_tensor(n * ho * wo, bits_in.device)
    _check(lib().fc_mask_downsample_packed(_ptr(bits_in), n, h, w, k[0], k[1], stride[0], stride[1], pad[0], pad[1],
                                           dil[0], dil[1], _ptr(out), _stream(stream)), "fc_mask_downsample_packed")
    return out, (n, ho, wo)


def active_index_compact_packed(bits, m: int, idx=None, count=None, workspace=None, stream=None):
    """fc_active_index_compact_packed: packed mask of m pixels -> (idx, count)."""
    torch = _torch()
    _require_cuda(bits, idx, count, workspace)
    if idx is None:
        idx = torch.empty((m,), dtype=torch.int32, device=bits.device)
    if count is None:
        count = torch.empty((1,), dtype=torch.int32, device=bits.device)
    if workspace is None:
        workspace = torch.empty((compact_workspace_bytes(m),), dtype=torch.uint8, device=bits.device)
    _check(lib().fc_active_index_compact_packed(_ptr(bits), m, _ptr(idx), _ptr(count), _ptr(workspace),
                                                workspace.numel(), _stream(stream)), "fc_active_index_compact_packed")
    return idx, count


class PreparedPyramid:
    """fc_mask_pyramid (or, with packed=True, fc_mask_pyramid_packed) with its arguments marshalled
    once: all levels' masks and kept lists from one input mask.  `levels` holds (mask_out, idx, count)
    per level; with packed=True mask_out is the packed mask (int64 words) and `dims` its (N, H, W).
    packed_in: the input mask is packed too (then `shape` = its (N, H, W))."""

    def __init__(self, mask_in, steps, packed: bool = False, packed_in: bool = False, shape=None):
        torch = _torch()
        _require_cuda(mask_in)
        n, h, w = shape if packed_in else mask_in.shape
        self._steps = _steps_array(steps)
        dims = mask_pyramid_dims(h, w, steps)
        self.dims = [(n, hl, wl) for hl, wl in dims]
        dev = mask_in.device
        self.levels = [((_packed_tensor(n * hl * wl, dev) if packed else
                         torch.empty((n, hl, wl), dtype=torch.uint8, device=dev)),
                        torch.empty((n * hl * wl,), dtype=torch.int32, device=dev),
                        torch.empty((1,), dtype=torch.int32, device=dev)) for hl, wl in dims]
        b = ctypes.c_size_t()
        _check(lib().fc_mask_pyramid_workspace_bytes(n, h, w, len(steps), self._steps, ctypes.byref(b)),
               "fc_mask_pyramid_workspace_bytes")
        self._ws = torch.empty((max(int(b.value), 16),), dtype=torch.uint8, device=dev)
        vp = ctypes.c_void_p
        nl = len(steps)
        self._ptrs = tuple((vp * nl)(*[_ptr(lv[i]) for lv in self.levels]) for i in range(3))
        if packed:
            self._args = (_ptr(mask_in), 1 if packed_in else 0, n, h, w, nl, self._steps, *self._ptrs,
                          _ptr(self._ws), self._ws.numel())
            self._fn = lib().fc_mask_pyramid_packed
        else:
            if packed_in:
                raise ValueError("a packed input mask gives packed levels: pass packed=True")
            self._args = (_ptr(mask_in), n, h, w, nl, self._steps, *self._ptrs, _ptr(self._ws), self._ws.numel())
            self._fn = lib().fc_mask_pyramid
        self.mask_in = mask_in   # (kept alive: the call reads it)
        self._current_stream = torch.cuda.current_stream

    def __call__(self, stream=None):
        hnd = (self._current_stream() if stream is None else stream).cuda_stream
        rc = self._fn(*self._args, ctypes.c_void_p(hnd))
        if rc != 0:
            raise FcError(rc, "fc_mask_pyramid")
        return self.levels


def active_index_compact(mask, idx=None, count=None, workspace=None, stream=None):
    """fc_active_index_compact: uint8 [...] -> (idx int32 [m] (first `count` valid), count int32 [1])."""
    torch = _torch()
    _require_cuda(mask, idx, count, workspace)
    m = mask.numel()
    if idx is None:
        idx = torch.empty((m,), dtype=torch.int32, device=mask.device)
    if count is None:
        count = torch.empty((1,), dtype=torch.int32, device=mask.device)
    if workspace is None:
        workspace = torch.empty((compact_workspace_bytes(m),), dtype=torch.uint8, device=mask.device)
    _check(lib().fc_active_index_compact(_ptr(mask), m, _ptr(idx), _ptr(count), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream)),
           "fc_active_index_compact")
    return idx, count


def active_index_compact_tiled(mask, tile_h: int = 8, tile_w: int = 16, idx=None, count=None, stream=None):
    """fc_active_index_compact_tiled: (idx, count) of a [n, ho, wo] mask in tile order."""
    torch = _torch()
    _require_cuda(mask, idx, count)
    n, ho, wo = mask.shape
    if idx is None:
        idx = torch.empty((n * ho * wo,), dtype=torch.int32, device=mask.device)
    if count is None:
        count = torch.empty((1,), dtype=torch.int32, device=mask.device)
    b = ctypes.c_size_t()
    _check(lib().fc_compact_tiled_workspace_bytes(n, ho, wo, tile_h, tile_w, ctypes.byref(b)),
           "fc_compact_tiled_workspace_bytes")
    ws = torch.empty((max(int(b.value), 16),), dtype=torch.uint8, device=mask.device)
    _check(lib().fc_active_index_compact_tiled(_ptr(mask), n, ho, wo, tile_h, tile_w, _ptr(idx), _ptr(count),
                                               _ptr(ws), ws.numel(), _stream(stream)),
           "fc_active_index_compact_tiled")
    return idx, count


def focused_conv2d(desc: ConvDesc, x, w, bias=None, mask_in=None, mask_out=None, idx=None, count=None,
                   out=None, workspace=None, stream=None):
    """fc_focused_conv2d.  x NHWC, w [C_out,KH,KW,C_in]; returns out NHWC."""
    torch = _torch()
    _require_cuda(x, w, bias, mask_in, mask_out, idx, count, out, workspace)
    ho, wo = out_dims(desc)
    if out is None:
        out = torch.empty((desc.n, ho, wo, desc.c_out), dtype=torch_dtype(desc.out_dtype), device=x.device)
    if workspace is None and mask_in is not None and idx is None:
        workspace = torch.empty((workspace_bytes(desc),), dtype=torch.uint8, device=x.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().fc_focused_conv2d(ctypes.byref(desc), _ptr(x), _ptr(mask_in), _ptr(w), _ptr(bias),
                                   _ptr(mask_out), _ptr(idx), _ptr(count), _ptr(out), _ptr(workspace),
                                   ws_bytes, _stream(stream)), "fc_focused_conv2d")
    return out


def focused_conv2d_noalloc(desc: ConvDesc, x, w, bias, mask_in, out, stream=None):
    """fc_focused_conv2d_noalloc: the caller passes inputs and the output tensor, nothing is allocated."""
    _require_cuda(x, w, bias, mask_in, out)
    _check(lib().fc_focused_conv2d_noalloc(ctypes.byref(desc), _ptr(x), _ptr(mask_in), _ptr(w), _ptr(bias),
                                           _ptr(out), _stream(stream)), "fc_focused_conv2d_noalloc")
    return out


class PreparedConv:
    """fc_focused_conv2d with its arguments marshalled once: calling it costs one
    foreign call, which matters when layers take a few microseconds.  The tensors
    must stay alive and in place; `stream=None` means the stream current at call
    time (so the same object works eagerly and under graph capture)."""

    def __init__(self, desc: ConvDesc, x, w, bias=None, mask_in=None, mask_out=None, idx=None, count=None,
                 out=None, workspace=None, workspace_ready: bool = False):
        """workspace_ready: the caller has cleared the workspace's leading counters once
        (`ready_workspace`) and only this library writes to it since: every call is then made
        with FC_WORKSPACE_READY and skips the launch that clears them."""
        torch = _torch()
        if workspace_ready:
            desc = ConvDesc.from_buffer_copy(desc)
            desc.flags |= WORKSPACE_READY
        _require_cuda(x, w, bias, mask_in, mask_out, idx, count, out, workspace)
        ho, wo = out_dims(desc)
        if out is None:
            out = torch.empty((desc.n, ho, wo, desc.c_out), dtype=torch_dtype(desc.out_dtype), device=x.device)
        if workspace is None and mask_in is not None and idx is None:
            workspace = torch.empty((workspace_bytes(desc),), dtype=torch.uint8, device=x.device)
        self.out = out
        self._keep = (desc, x, w, bias, mask_in, mask_out, idx, count, out, workspace)
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        self._args = (ctypes.byref(desc), _ptr(x), _ptr(mask_in), _ptr(w), _ptr(bias), _ptr(mask_out), _ptr(idx),
                      _ptr(count), _ptr(out), _ptr(workspace), ws_bytes)
        self._fn = lib().fc_focused_conv2d
        self._current_stream = torch.cuda.current_stream

    def __call__(self, stream=None):
        h = (self._current_stream() if stream is None else stream).cuda_stream
        rc = self._fn(*self._args, ctypes.c_void_p(h))
        if rc != 0:
            raise FcError(rc, "fc_focused_conv2d")
        return self.out


def focused_gconv2d(desc: ConvDesc, groups: int, x, w, bias=None, mask_in=None, mask_out=None, idx=None,
                    count=None, out=None, workspace=None, stream=None):
    """fc_focused_gconv2d.  x NHWC, w [C_out,KH,KW,C_in/groups]; returns out NHWC."""
    torch = _torch()
    _require_cuda(x, w, bias, mask_in, mask_out, idx, count, out, workspace)
    ho, wo = out_dims(desc)
    if out is None:
        out = torch.empty((desc.n, ho, wo, desc.c_out), dtype=torch_dtype(desc.out_dtype), device=x.device)
    if workspace is None and mask_in is not None and idx is None:
        workspace = torch.empty((workspace_bytes(desc),), dtype=torch.uint8, device=x.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().fc_focused_gconv2d(ctypes.byref(desc), groups, _ptr(x), _ptr(mask_in), _ptr(w), _ptr(bias),
                                    _ptr(mask_out), _ptr(idx), _ptr(count), _ptr(out), _ptr(workspace),
                                    ws_bytes, _stream(stream)), "fc_focused_gconv2d")
    return out


def expand_group_weights(w, groups: int, dtype: int, stream=None):
    """fc_expand_group_weights: [C_out,KH,KW,C_in/groups] -> block-diagonal [C_out,KH,KW,C_in]."""
    torch = _torch()
    _require_cuda(w)
    c_out, kh, kw, cig = w.shape
    full = torch.empty((c_out, kh, kw, cig * groups), dtype=w.dtype, device=w.device)
    _check(lib().fc_expand_group_weights(cig * groups, c_out, kh, kw, groups, dtype, _ptr(w), _ptr(full),
                                         _stream(stream)), "fc_expand_group_weights")
    return full


def focused_dwconv2d(desc: ConvDesc, x, w, bias=None, mask_in=None, out=None, stream=None):
    """fc_focused_dwconv2d.  x NHWC, w [C,KH,KW] (one filter per channel); returns out NHWC."""
    torch = _torch()
    _require_cuda(x, w, bias, mask_in, out)
    ho, wo = out_dims(desc)
    if out is None:
        out = torch.empty((desc.n, ho, wo, desc.c_out), dtype=torch_dtype(desc.out_dtype), device=x.device)
    _check(lib().fc_focused_dwconv2d(ctypes.byref(desc), _ptr(x), _ptr(mask_in), _ptr(w), _ptr(bias), _ptr(out),
                                     _stream(stream)), "fc_focused_dwconv2d")
    return out


class PreparedDwConv:
    """fc_focused_dwconv2d with its arguments marshalled once (see PreparedConv)."""

    def __init__(self, desc: ConvDesc, x, w, bias=None, mask_in=None, out=None):
        torch = _torch()
        _require_cuda(x, w, bias, mask_in, out)
        ho, wo = out_dims(desc)
        if out is None:
            out = torch.empty((desc.n, ho, wo, desc.c_out), dtype=torch_dtype(desc.out_dtype), device=x.device)
        self.out = out
        self._keep = (desc, x, w, bias, mask_in, out)
        self._args = (ctypes.byref(desc), _ptr(x), _ptr(mask_in), _ptr(w), _ptr(bias), _ptr(out))
        self._fn = lib().fc_focused_dwconv2d
        self._current_stream = torch.cuda.current_stream

    def __call__(self, stream=None):
        h = (self._current_stream() if stream is None else stream).cuda_stream
        rc = self._fn(*self._args, ctypes.c_void_p(h))
        if rc != 0:
            raise FcError(rc, "fc_focused_dwconv2d")
        return self.out


def calibrate_mfma(dtype: int, iters: int, blocks: int, sink, stream=None) -> float:
    """fc_calibrate_mfma: enqueues the register-only matrix-instruction loop; returns the FLOP of the launch."""
    _require_cuda(sink)
    flop = ctypes.c_double()
    _check(lib().fc_calibrate_mfma(dtype, iters, blocks, _ptr(sink), ctypes.byref(flop), _stream(stream)),
           "fc_calibrate_mfma")
    return flop.value


def calibrate_copy(src, dst, stream=None) -> int:
    """fc_calibrate_copy: enqueues one streaming copy src -> dst; returns the bytes copied (each way)."""
    _require_cuda(src, dst)
    nbytes = src.numel() * src.element_size()
    _check(lib().fc_calibrate_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)), "fc_calibrate_copy")
    return nbytes


def calibrate_issue(mode: int, waves_per_simd: int, steps: int, blocks: int, src, stream=None):
    """fc_calibrate_issue: enqueues the issue probe; returns the device tensor of per-workgroup
    shader cycles (int64, `blocks` entries) of the whole loop."""
    torch = _torch()
    _require_cuda(src)
    cycles = torch.zeros((blocks,), dtype=torch.int64, device=src.device)
    sink = torch.zeros((blocks,), dtype=torch.float32, device=src.device)
    _check(lib().fc_calibrate_issue(mode, waves_per_simd, steps, blocks, _ptr(src), src.numel() * src.element_size(),
                                    _ptr(cycles), _ptr(sink), _stream(stream)), "fc_calibrate_issue")
    return cycles


def ready_workspace(workspace):
    """Clears the arrival counters at the start of a workspace (a fill kernel on the current
    stream), after which calls may carry FC_WORKSPACE_READY."""
    workspace.view(_torch().uint8)[:WORKSPACE_COUNTER_BYTES].zero_()
    return workspace


def maxpool2d(x, k: int, stride: int, pad: int, dtype: int, out=None, stream=None, keep=None):
    """fc_maxpool2d / fc_maxpool2d_masked helper: NHWC max-pool; with `keep` ([N,Ho,Wo] bytes) only
    the kept output positions are computed, the others are zero."""
    torch = _torch()
    _require_cuda(x, out, keep)
    n, h, w, c = x.shape
    d = conv_desc(n, h, w, 1, 1, (k, k), (stride, stride), (pad, pad), (1, 1), F32)
    ho, wo = out_dims(d)
    if out is None:
        out = torch.empty((n, ho, wo, c), dtype=x.dtype, device=x.device)
    if keep is None:
        _check(lib().fc_maxpool2d(_ptr(x), n, h, w, c, dtype, k, stride, pad, _ptr(out), _stream(stream)),
               "fc_maxpool2d")
    else:
        if tuple(keep.shape) != (n, ho, wo):
            raise ValueError("keep shape %s, expected %s" % (tuple(keep.shape), (n, ho, wo)))
        _check(lib().fc_maxpool2d_masked(_ptr(x), n, h, w, c, dtype, k, stride, pad, _ptr(keep), _ptr(out),
                                         _stream(stream)), "fc_maxpool2d_masked")
    return out
