"""The entry point that allocates nothing (fc_focused_conv2d_noalloc: its workspace is a
device array inside the library) against fc_focused_conv2d with a caller's workspace: same
kernels, so the outputs must be equal bit for bit, call after call on the shared array, and
both within the fp32-output bar of the oracle."""
import ctypes

import numpy as np
import pytest

from oracle import fc_oracle as O
from paper_2207_10741_amd import binding as B, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

TOL_F32_OUT = 1e-4


def _layer(seed, n, h, w, ci, co, k, s, irrelevant, out_dtype):
    torch = G.torch_mod()
    dtype = synth.BF16
    p = k // 2
    x = synth.activations((n, h, w, ci), dtype, seed, 1)
    wt = synth.he_weights(co, k, k, ci, dtype, seed, 2)
    bias = synth.bias(co, seed, 3)
    mask = synth.mask_objects(n, h, w, irrelevant, seed, 4)
    desc = B.conv_desc(n, h, w, ci, co, (k, k), (s, s), (p, p), (1, 1), dtype, out_dtype, B.RELU)
    ho, wo = B.out_dims(desc)
    xd, wd, bd, md = G.to_dev(x, dtype), G.to_dev(wt, dtype), torch.from_numpy(bias).to(G.dev()), G.mask_dev(mask)
    canary = lambda: torch.full((n, ho, wo, co), 7.0, dtype=B.torch_dtype(out_dtype), device=G.dev())
    got = B.focused_conv2d_noalloc(desc, xd, wd, bd, md, canary())
    want = B.focused_conv2d(desc, xd, wd, bd, mask_in=md, out=canary())
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), "differs from fc_focused_conv2d"
    if out_dtype == B.F32:
        ref = O.focused_conv2d(O.ConvShape(n, h, w, ci, co, k, k, (s, s), (p, p), (1, 1), relu=True), x, wt,
                               bias=bias, mask_in=mask, dtype=dtype)
        keep = O.mask_downsample(mask, k, k, (s, s), (p, p), (1, 1)) != 0
        g64 = G.to_f64(got)
        assert G.rel_err(g64, ref, keep) <= TOL_F32_OUT
        assert not g64[~keep].any()
    return desc


def test_two_calls_in_a_row_the_second_smaller():
    assert B.lib().fc_noalloc_init() == 0
    # a 3x3 layer with a few hundred tiles, then a smaller layer whose list, labels and
    # split-K partial tiles land on what the first call left in the array
    _layer(701, 3, 60, 72, 64, 128, 3, 1, 0.48, B.F32)
    _layer(702, 1, 20, 24, 256, 256, 3, 1, 0.48, B.F32)
    # ... a strided layer with 16-bit outputs, and the dense layer (no mask) through the same array
    _layer(703, 2, 33, 47, 64, 64, 3, 2, 0.3, B.BF16)
    torch = G.torch_mod()
    dtype = synth.BF16
    x = synth.activations((1, 24, 24, 128), dtype, 704, 1)
    wt = synth.he_weights(128, 3, 3, 128, dtype, 704, 2)
    desc = B.conv_desc(1, 24, 24, 128, 128, in_dtype=dtype, out_dtype=B.F32)
    xd, wd = G.to_dev(x, dtype), G.to_dev(wt, dtype)
    out = torch.empty((1, 24, 24, 128), dtype=torch.float32, device=G.dev())
    rc = B.lib().fc_focused_conv2d_noalloc(ctypes.byref(desc), xd.data_ptr(), None, wd.data_ptr(), None,
                                           out.data_ptr(), None)
    assert rc == 0
    ws = torch.zeros((B.workspace_bytes(desc),), dtype=torch.uint8, device=G.dev())
    want = B.focused_conv2d(desc, xd, wd, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(out, want)


def test_layers_beyond_the_array_are_refused_before_any_launch():
    torch = G.torch_mod()
    # 4 x 2048 x 1100 positions (labels + list: 5 bytes each) need more than the 40 MiB array
    desc = B.conv_desc(4, 2048, 1100, 8, 8, (1, 1), (1, 1), (0, 0), (1, 1), B.BF16, B.BF16)
    assert B.workspace_bytes(desc) > B.NOALLOC_SCRATCH_BYTES
    t = torch.zeros((16,), dtype=torch.uint8, device=G.dev())       # never dereferenced
    rc = B.lib().fc_focused_conv2d_noalloc(ctypes.byref(desc), t.data_ptr(), t.data_ptr(), t.data_ptr(), None,
                                           t.data_ptr() + 0, None)
    assert rc == -6
