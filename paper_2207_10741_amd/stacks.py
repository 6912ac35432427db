"""Runs a conv stack (workloads.Op list) through the library: mask propagation and
kept-position lists are built once per (mask, window geometry) and shared by every
layer that sees the same mask through the same geometry (Sec. III-B: one mask,
rescaled per layer) - by one fc_mask_pyramid call per pass when the mask levels form
a chain, as they do in a feed-forward network; each conv is one fc_focused_conv2d
call, each depthwise conv one fc_focused_dwconv2d call.

Plumbing only: the order of library calls and which tensor feeds which.  Max-pools
(not part of the paper's method) go through the library's helper, which with a mask
computes only the pooled positions the mask keeps.
"""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np

from . import binding as B
from . import synth


class ConvStack:
    def __init__(self, ops, n: int, h: int, w: int, dtype: int = B.BF16, seed: int = 0, relu: bool = True):
        import torch
        self.torch = torch
        self.ops = list(ops)
        self.n, self.h, self.w, self.dtype = n, h, w, dtype
        self.dev = torch.device("cuda:0")
        self.relu = relu
        if dtype == B.FP8 and not all(op.kind == "conv" and op.c_in % 16 == 0 and op.c_out % 16 == 0 for op in self.ops):
            raise ValueError("an 8-bit stack takes convolutions with multiples of 16 channels only")
        self.weights: Dict[int, object] = {}
        self.biases: Dict[int, object] = {}
        self.host_weights: Dict[int, np.ndarray] = {}
        self.host_biases: Dict[int, np.ndarray] = {}
        for i, op in enumerate(self.ops):
            if op.kind not in ("conv", "dwconv"):
                continue
            if op.kind == "dwconv":
                wt = np.ascontiguousarray(synth.he_weights(op.c_out, op.k, op.k, 1, dtype, seed, i, 2)[..., 0])
            else:
                wt = synth.he_weights(op.c_out, op.k, op.k, op.c_in, dtype, seed, i, 2)
            bs = synth.bias(op.c_out, seed, i, 3)
            self.host_weights[i], self.host_biases[i] = wt, bs
            self.weights[i] = self._to_dev(wt)
            self.biases[i] = torch.from_numpy(bs).to(self.dev)
        # spatial size of every op's output
        self.sizes = {-1: (h, w)}
        for i, op in enumerate(self.ops):
            hi, wi = self.sizes[op.src]
            d = B.conv_desc(n, hi, wi, 1, 1, (op.k, op.k), (op.stride, op.stride), (op.pad, op.pad), (1, 1), B.F32)
            self.sizes[i] = B.out_dims(d)
        # one workspace for all layers (calls are ordered on one stream): lets small layers
        # split their reduction over more workgroups
        need = max(B.workspace_bytes(self.desc(i)) for i, op in enumerate(self.ops) if op.kind == "conv")
        self.workspace = torch.empty((need,), dtype=torch.uint8, device=self.dev)
        # its arrival counters are cleared once here; every library call leaves them at zero,
        # so the calls carry FC_WORKSPACE_READY and none of them launches a clear
        B.ready_workspace(self.workspace)
        # the mask levels the ops need, when they form one chain (input -> level 0 -> level 1 ...):
        # then one fc_mask_pyramid call per pass builds all of them
        self.pyramid_steps = self._pyramid_steps()
        self._pyramids: Dict[int, object] = {}

    def _same_view(self, i: int) -> bool:
        op = self.ops[i]
        return op.stride == 1 and self.sizes[i] == self.sizes[op.src] and op.pad == (op.k - 1) // 2

    def _pyramid_steps(self):
        """The windows that take each mask level to the next, in the order the ops first need them,
        or None when the levels do not form a single chain (then every level is built by its own
        fc_mask_downsample + fc_active_index_compact calls)."""
        level_of = {-1: -1}       # op -> level its output mask is (-1: the input mask)
        plans: Dict[tuple, int] = {}
        steps = []
        for i, op in enumerate(self.ops):
            src_level = level_of[op.src]
            key = (src_level, op.stride, (op.k - 1) // 2 - op.pad, self.sizes[i])
            if self._same_view(i) and src_level >= 0:
                level = src_level
            elif key in plans:
                level = plans[key]
            else:
                if src_level != len(steps) - 1:
                    return None
                steps.append(((op.k, op.k), (op.stride, op.stride), (op.pad, op.pad), (1, 1)))
                level = plans[key] = len(steps) - 1
            level_of[i] = level
        return steps if 0 < len(steps) <= B.MAX_PYRAMID_LEVELS else None

    def _to_dev(self, storage: np.ndarray):
        torch = self.torch
        if self.dtype == B.F32:
            return torch.from_numpy(np.ascontiguousarray(storage, dtype=np.float32)).to(self.dev)
        if self.dtype == B.FP8:
            return torch.from_numpy(np.ascontiguousarray(storage, dtype=np.uint8)).to(self.dev).view(torch.float8_e4m3fn)
        t = torch.from_numpy(np.ascontiguousarray(storage).view(np.int16)).to(self.dev)
        return t.view(torch.bfloat16 if self.dtype == B.BF16 else torch.float16)

    def desc(self, i: int, out_dtype: Optional[int] = None, flags_extra: int = 0) -> B.ConvDesc:
        op = self.ops[i]
        hi, wi = self.sizes[op.src]
        flags = (B.RELU if (self.relu and op.relu) else 0) | flags_extra
        if out_dtype is None and self.dtype == B.FP8:
            out_dtype = B.FP8       # an 8-bit stack hands on 8-bit activations
        return B.conv_desc(self.n, hi, wi, op.c_in, op.c_out, (op.k, op.k), (op.stride, op.stride),
                           (op.pad, op.pad), (1, 1), self.dtype, out_dtype, flags)

    def _pointwise(self, i: int) -> bool:
        op = self.ops[i]
        return op.kind == "conv" and op.k == 1 and op.stride == 1 and op.pad == 0

    def _matrix_core_shape(self, i: int) -> bool:
        op = self.ops[i]
        if self.dtype == B.FP8:
            return op.kind == "conv" and op.c_in % 16 == 0 and op.c_out % 16 == 0 and op.k * op.k <= 32
        return (op.kind == "conv" and self.dtype in (B.BF16, B.F16) and op.c_in % 8 == 0 and op.c_out % 8 == 0
                and op.k * op.k <= 32)

    def run(self, x, mask=None, keep_outputs: bool = True, chain: bool = False, canary=None, compact: bool = False):
        """x: device NHWC tensor; mask: device uint8 [N,H,W] or None (dense).
        Returns (outputs, masks): per-op output tensors and per-op output masks
        (index -1 = the stack's input).

        chain: a conv whose output is read only by other convs leaves its irrelevant rows
        unwritten (FC_SKIP_ZERO_FILL): every reader gates its taps by the same mask, so those
        rows are never looked at (Sec. III-A: irrelevant pixels are excluded from the
        product; Sec. III-B: the mask is the same all the way).  Outputs that a pooling
        layer or nobody reads are still zero-filled.
        compact (with chain): a conv read only by 1x1 convs of unit stride writes its kept rows
        compacted, in list order (FC_COMPACT_OUT), and those readers read them that way
        (FC_COMPACT_IN): they see the same mask through the same geometry, hence the same list.
        canary: value every conv output buffer is pre-filled with (tests)."""
        readers: Dict[int, List[str]] = {}
        reader_ops: Dict[int, List[int]] = {}
        for j, op in enumerate(self.ops):
            readers.setdefault(op.src, []).append(op.kind)
            reader_ops.setdefault(op.src, []).append(j)
        compacted: Dict[int, bool] = {}   # op -> its output is stored compacted
        outs: Dict[int, object] = {-1: x}
        masks: Dict[int, object] = {-1: mask}
        plans: Dict[tuple, tuple] = {}
        produced: Dict[int, tuple] = {}   # 0/1 masks this run wrote, with their kept lists
        levels = None                     # all mask levels from one call, taken in order
        if mask is not None and self.pyramid_steps is not None:
            pyr = self._pyramids.get(mask.data_ptr())
            if pyr is None or pyr.mask_in is not mask:
                pyr = self._pyramids[mask.data_ptr()] = B.PreparedPyramid(mask, self.pyramid_steps)
            levels = list(pyr())
        last_use = {}
        for i, op in enumerate(self.ops):
            last_use[op.src] = i
        for i, op in enumerate(self.ops):
            src, m_in = outs[op.src], masks[op.src]
            geo = ((op.k, op.k), (op.stride, op.stride), (op.pad, op.pad), (1, 1))
            plan = None
            if m_in is not None:
                hi, wi = self.sizes[op.src]
                same_view = self._same_view(i)
                # two windows with the same stride, the same centre-tap offset and the same output
                # size keep the same positions (a 3x3/2 pad 1 conv and the 1x1/2 projection beside it)
                key = (id(m_in), op.stride, (op.k - 1) // 2 - op.pad, self.sizes[i])
                if same_view and id(m_in) in produced:
                    # the window is centred and does not change the resolution: the mask this op
                    # keeps is the (already 0/1) mask it reads, and so is the kept list
                    plan = produced[id(m_in)]
                elif key in plans:
                    plan = plans[key]
                elif levels is not None:
                    m_out, idx, count = levels.pop(0)
                    plan = plans[key] = produced[id(m_out)] = (m_out, idx, count)
                else:
                    m_out = B.mask_downsample(m_in, *geo)
                    idx, count = B.active_index_compact(m_out)
                    plan = plans[key] = produced[id(m_out)] = (m_out, idx, count)
            if op.kind in ("conv", "dwconv"):
                gated_readers_only = bool(readers.get(i)) and all(k in ("conv", "dwconv") for k in readers[i])
                skip = chain and plan is not None and gated_readers_only
                extra = B.WORKSPACE_READY | (B.SKIP_ZERO_FILL if skip else 0)
                out = None
                ho, wo = self.sizes[i]
                if compacted.get(op.src, False):
                    extra |= B.COMPACT_IN
                if (compact and skip and op.kind == "conv" and self._matrix_core_shape(i)
                        and all(self._pointwise(j) and self._matrix_core_shape(j) for j in reader_ops[i])):
                    extra |= B.COMPACT_OUT
                    compacted[i] = True
                    out = (self.torch.empty if canary is None else
                           (lambda *a, **k: self.torch.full(*a, canary, **k)))(
                        (self.n * ho * wo, op.c_out), dtype=B.torch_dtype(self.dtype), device=self.dev)
                elif canary is not None:
                    out = self.torch.full((self.n, ho, wo, op.c_out), canary, dtype=B.torch_dtype(self.dtype),
                                          device=self.dev)
                d = self.desc(i, flags_extra=extra)
                if op.kind == "dwconv":
                    # labels come from the input mask inside the call: no list, no workspace
                    d.flags &= ~B.WORKSPACE_READY
                    outs[i] = B.focused_dwconv2d(d, src, self.weights[i], self.biases[i],
                                                 mask_in=m_in if plan is not None else None, out=out)
                elif plan is None:
                    outs[i] = B.focused_conv2d(d, src, self.weights[i], self.biases[i], out=out,
                                               workspace=self.workspace)
                else:
                    outs[i] = B.focused_conv2d(d, src, self.weights[i], self.biases[i], mask_in=m_in,
                                               mask_out=plan[0], idx=plan[1], count=plan[2], out=out,
                                               workspace=self.workspace)
            else:
                # with a mask, only the pooled positions it keeps are computed; the rest is zero
                outs[i] = B.maxpool2d(src, op.k, op.stride, op.pad, self.dtype,
                                      keep=None if plan is None else plan[0])
            masks[i] = None if plan is None else plan[0]
            if not keep_outputs:
                for j in [j for j in outs if j != i and last_use.get(j, -2) <= i and j != -1]:
                    del outs[j]
        return outs, masks

    def conv_flops(self, masks_host: Optional[Dict[int, np.ndarray]] = None):
        """(dense FLOPs, kept FLOPs) of the stack; kept needs the host copies of the masks."""
        dense = kept = 0.0
        for i, op in enumerate(self.ops):
            if op.kind not in ("conv", "dwconv"):
                continue
            ho, wo = self.sizes[i]
            per_pos = 2.0 * op.k * op.k * op.c_in * (op.c_out if op.kind == "conv" else 1)
            dense += self.n * ho * wo * per_pos
            if masks_host is not None:
                kept += float(np.count_nonzero(masks_host[i])) * per_pos
        return dense, kept
