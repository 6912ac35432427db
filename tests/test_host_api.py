"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2207_10741_amd import binding as B
from oracle import fc_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER_TEXT = open(os.path.join(ROOT, "include", "focused_conv.h")).read()


def _declared():
    text = open(os.path.join(ROOT, "include", "focused_conv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fc_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert set(names) == set(B.FUNCTIONS)
    L = B.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings():
    assert B.status_string(0) == "FC_OK"
    for code in range(-7, 0):
        assert B.status_string(code).startswith("FC_ERR_")
    assert "unknown" in B.status_string(5)


@pytest.mark.parametrize("h,w,k,s,p,d", [(224, 224, 7, 2, 3, 1), (56, 56, 3, 1, 1, 1), (135, 240, 2, 2, 0, 1),
                                          (17, 9, 3, 2, 1, 2), (4, 6, 3, 1, 0, 1), (1080, 1920, 3, 1, 1, 1)])
def test_out_dims_match_oracle(h, w, k, s, p, d):
    desc = B.conv_desc(1, h, w, 8, 8, (k, k), (s, s), (p, p), (d, d))
    assert B.out_dims(desc) == (O.out_dim(h, k, s, p, d), O.out_dim(w, k, s, p, d))


def test_descriptor_errors():
    def rc(**kw):
        base = dict(n=1, h=8, w=8, c_in=8, c_out=8)
        base.update(kw)
        d = B.conv_desc(**base)
        ho, wo = ctypes.c_int32(), ctypes.c_int32()
        return B.lib().fc_out_dims(ctypes.byref(d), ctypes.byref(ho), ctypes.byref(wo))
    assert rc() == 0
    assert rc(n=0) == -2 and rc(c_in=-1) == -2 and rc(stride=(0, 1)) == -2 and rc(pad=(-1, 0)) == -2
    assert rc(h=2, pad=(0, 0)) == -2                      # empty output
    assert rc(in_dtype=7) == -3
    assert rc(in_dtype=B.F32, out_dtype=B.BF16) == -3     # output narrower than the input type
    assert rc(in_dtype=B.FP8, out_dtype=B.BF16) == 0 and rc(in_dtype=B.FP8, out_dtype=B.F32) == 0
    assert rc(in_dtype=B.FP8, out_dtype=B.FP8) == 0 and rc(in_dtype=B.FP8, out_dtype=B.F16) == -3
    assert rc(in_dtype=B.BF16, out_dtype=B.FP8) == 0 and rc(in_dtype=B.F32, out_dtype=B.FP8) == -3
    assert rc(flags=128) == -3
    assert rc(flags=B.RESIDENT_WEIGHTS) == 0
    assert rc(flags=B.RELU | B.SKIP_ZERO_FILL | B.WORKSPACE_READY) == 0
    assert B.WORKSPACE_COUNTER_BYTES == int(re.search(r"FC_WORKSPACE_COUNTER_BYTES\s*=\s*(\d+)", HEADER_TEXT).group(1))
    assert rc(n=40000, h=1000, w=1000, k=(1, 1), pad=(0, 0)) == -6
    assert B.lib().fc_out_dims(None, None, None) == -1


def test_workspace_sizes():
    d = B.conv_desc(2, 30, 40, 16, 16)
    m = 2 * 30 * 40
    ws = B.workspace_bytes(d)
    assert ws >= m + 4 * m + 4 + B.compact_workspace_bytes(m)
    assert B.compact_workspace_bytes(1) >= 4
    assert B.compact_workspace_bytes(4097) >= 8
    with pytest.raises(B.FcError):
        B.compact_workspace_bytes(0)
    with pytest.raises(B.FcError) as e:
        B.compact_workspace_bytes(2 ** 31)
    assert e.value.status == -6


def test_null_pointers_rejected_before_any_launch():
    L = B.lib()
    d = B.conv_desc(1, 8, 8, 8, 8)
    assert L.fc_focused_conv2d(ctypes.byref(d), None, None, None, None, None, None, None, None, None, 0, None) == -1
    assert L.fc_mask_downsample(None, 1, 8, 8, 3, 3, 1, 1, 1, 1, 1, 1, None, None) == -1
    assert L.fc_active_index_compact(None, 10, None, None, None, 0, None) == -1
    assert L.fc_mask_downsample_rule(None, 1, 8, 8, 3, 3, 1, 1, 1, 1, 1, 1, 1, None, None) == -1
    assert L.fc_mask_downsample_rule(ctypes.c_void_p(0x1000), 1, 8, 8, 3, 3, 1, 1, 1, 1, 1, 1, 7,
                                     ctypes.c_void_p(0x2000), None) == -3     # unknown rule
    assert L.fc_mask_downsample_rule(ctypes.c_void_p(0x1000), 1, 8, 8, 3, 3, 0, 1, 1, 1, 1, 1, 2,
                                     ctypes.c_void_p(0x2000), None) == -2
    assert L.fc_maxpool2d(None, 1, 8, 8, 8, 0, 2, 2, 0, None, None) == -1
    # fake but well-formed addresses: the checks below fail before anything touches them
    a = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1008)
    assert L.fc_active_index_compact(a, 10, a, a, None, 0, None) == -5
    assert L.fc_active_index_compact(a, 10, a, a, a, 1, None) == -5
    assert L.fc_active_index_compact(odd, 10, a, a, a, 4096, None) == -4
    assert L.fc_active_index_compact(a, 0, a, a, a, 4096, None) == -2
    nb = ctypes.c_size_t()
    assert L.fc_compact_tiled_workspace_bytes(2, 64, 64, 8, 16, ctypes.byref(nb)) == 0 and nb.value >= 4 * 2
    assert L.fc_compact_tiled_workspace_bytes(2, 64, 64, 8, 33, ctypes.byref(nb)) == -2       # tile wider than 32
    assert L.fc_compact_tiled_workspace_bytes(2, 64, 64, 0, 16, ctypes.byref(nb)) == -2
    assert L.fc_compact_tiled_workspace_bytes(2, 64, 64, 8, 16, None) == -1
    assert L.fc_active_index_compact_tiled(None, 2, 64, 64, 8, 16, a, a, a, 4096, None) == -1
    assert L.fc_active_index_compact_tiled(a, 2, 64, 64, 8, 16, a, a, None, 0, None) == -5
    assert L.fc_active_index_compact_tiled(a, 2, 64, 64, 8, 16, odd, a, a, 4096, None) == -4
    assert L.fc_active_index_compact_tiled(a, 40000, 1000, 1000, 8, 16, a, a, a, 4096, None) == -6
    o = ctypes.c_void_p(0x2000)
    conv = lambda *args: L.fc_focused_conv2d(ctypes.byref(d), *args)
    #            x    mask_in w  bias  mask_out idx  count out ws    ws_bytes stream
    assert conv(odd, None, a, None, None, None, None, o, None, 0, None) == -4
    assert conv(a, None, a, None, None, a, None, o, None, 0, None) == -1      # idx without count
    assert conv(a, None, a, None, None, a, a, o, None, 0, None) == -1         # idx without the input mask
    assert conv(a, None, a, odd, None, None, None, o, None, 0, None) == -4    # misaligned bias
    assert conv(a, a, a, None, None, None, None, o, None, 0, None) == -5      # needs a workspace
    assert conv(a, a, a, None, None, None, None, o, a, 16, None) == -5        # workspace too small
    assert conv(a, None, a, None, None, None, None, a, None, 0, None) == -1   # out aliases x
    part = ctypes.c_void_p(0x1000 + 16 * 8)                                    # out starts inside x
    assert conv(a, None, a, None, None, None, None, part, None, 0, None) == -1
    before = ctypes.c_void_p(0x1000 - 16)                                      # out ends inside x
    assert conv(a, None, a, None, None, None, None, before, None, 0, None) == -1
    assert L.fc_focused_conv2d_noalloc(None, a, None, a, None, o, None) == -1
    big = B.conv_desc(4, 2048, 1100, 8, 8, (1, 1), (1, 1), (0, 0), (1, 1), B.BF16, B.BF16)
    assert L.fc_focused_conv2d_noalloc(ctypes.byref(big), a, a, a, None, o, None) == -6   # beyond the static scratch
    # 8-bit layers: only what the matrix-core path takes (16 | c_in, 8 | c_out, at most 32 taps)
    fp8 = lambda ci, co, k=(3, 3): L.fc_focused_conv2d(
        ctypes.byref(B.conv_desc(1, 8, 8, ci, co, k, pad=(k[0] // 2, k[1] // 2), in_dtype=B.FP8, out_dtype=B.F32)),
        a, None, a, None, None, None, None, o, None, 0, None)
    assert fp8(24, 64) == -3 and fp8(64, 20) == -3 and fp8(3, 64, (7, 7)) == -3 and fp8(16, 16, (7, 7)) == -3
    assert L.fc_expand_group_weights(64, 64, 3, 3, 4, B.BF16, None, a, None) == -1
    assert L.fc_expand_group_weights(64, 64, 3, 3, 5, B.BF16, a, a, None) == -2       # channels not multiples of groups
    assert L.fc_expand_group_weights(64, 64, 3, 3, 4, 9, a, a, None) == -3
    gc = lambda groups, *args: L.fc_focused_gconv2d(ctypes.byref(B.conv_desc(1, 8, 8, 24, 36)), groups, *args)
    assert gc(5, a, None, a, None, None, None, None, o, None, 0, None) == -2
    assert gc(3, None, None, a, None, None, None, None, o, None, 0, None) == -1
    assert gc(3, a, a, a, None, None, None, None, o, None, 0, None) == -5              # mask without a list needs a workspace
    dw = lambda desc, *args: L.fc_focused_dwconv2d(ctypes.byref(desc), *args)
    assert dw(B.conv_desc(1, 8, 8, 16, 16, in_dtype=B.FP8), a, None, a, None, o, None) == -3
    #              x  mask_in w  bias out stream
    assert dw(d, None, None, a, None, o, None) == -1
    assert dw(d, odd, None, a, None, o, None) == -4
    assert dw(d, a, None, a, odd, o, None) == -4
    assert dw(d, a, None, a, None, a, None) == -1                             # out aliases x
    assert dw(B.conv_desc(1, 8, 8, 8, 16), a, None, a, None, o, None) == -2   # not one filter per channel
    far = ctypes.c_void_p(1 << 45)                                            # (beyond the 25 GB such an x would span)
    assert dw(B.conv_desc(1, 40000, 40000, 8, 8, in_dtype=B.BF16), a, None, a, None, far, None) == -6
    assert L.fc_maxpool2d(a, 1, 8, 8, 8, 0, 2, 2, 2, a, None) == -2
    assert L.fc_maxpool2d_masked(a, 1, 8, 8, 8, 0, 2, 2, 2, a, a, None) == -2
    assert L.fc_maxpool2d_masked(None, 1, 8, 8, 8, 0, 2, 2, 0, a, a, None) == -1
    assert L.fc_maxpool2d(a, 1, 8, 8, 8, 9, 2, 2, 0, a, None) == -3


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libfocused_conv.so"))
    with pytest.raises(ImportError):
        B.lib()


def test_product_package_does_not_use_the_oracle():
    pkg = os.path.join(ROOT, "paper_2207_10741_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "fc_oracle" not in src and "fco_" not in src and "import oracle" not in src, f


def test_mask_pyramid_dims_and_argument_checks():
    steps = [((3, 3), (1, 1), (1, 1), (1, 1)), ((3, 3), (2, 2), (1, 1), (1, 1)), ((1, 1), (2, 2), (0, 0), (1, 1)),
             ((2, 2), (2, 2), (0, 0), (1, 1)), ((7, 5), (2, 1), (3, 2), (1, 1))]
    h, w = 135, 241
    want = []
    for k, s_, p, d in steps:
        h, w = O.out_dim(h, k[0], s_[0], p[0], d[0]), O.out_dim(w, k[1], s_[1], p[1], d[1])
        want.append((h, w))
    assert B.mask_pyramid_dims(135, 241, steps) == want
    L = B.lib()
    arr = B._steps_array(steps[:2])
    hs, ws = (ctypes.c_int32 * 2)(), (ctypes.c_int32 * 2)()
    assert L.fc_mask_pyramid_dims(8, 8, 0, arr, hs, ws) == -2                      # no levels
    assert L.fc_mask_pyramid_dims(8, 8, B.MAX_PYRAMID_LEVELS + 1, arr, hs, ws) == -2
    assert L.fc_mask_pyramid_dims(8, 8, 2, None, hs, ws) == -1
    bad = B._steps_array([((3, 3), (0, 1), (1, 1), (1, 1))])
    assert L.fc_mask_pyramid_dims(8, 8, 1, bad, hs, ws) == -2                      # zero stride
    tiny = B._steps_array([((3, 3), (1, 1), (0, 0), (1, 1))])
    assert L.fc_mask_pyramid_dims(2, 2, 1, tiny, hs, ws) == -2                     # empty level
    nbytes = ctypes.c_size_t()
    assert L.fc_mask_pyramid_workspace_bytes(2, 64, 64, 2, arr, ctypes.byref(nbytes)) == 0 and nbytes.value >= 4 * 3
    a = ctypes.c_void_p(0x1000)
    ptrs = (ctypes.c_void_p * 2)(a, a)
    none = (ctypes.c_void_p * 2)(a, None)
    assert L.fc_mask_pyramid(None, 2, 64, 64, 2, arr, ptrs, ptrs, ptrs, a, 4096, None) == -1
    assert L.fc_mask_pyramid(a, 2, 64, 64, 2, arr, none, ptrs, ptrs, a, 4096, None) == -1
    assert L.fc_mask_pyramid(a, 2, 64, 64, 2, arr, ptrs, ptrs, ptrs, None, 0, None) == -5
    assert L.fc_mask_pyramid(a, 2, 64, 64, 2, arr, ptrs, ptrs, ptrs, a, 4, None) == -5


def test_bench_refuses_more_than_one_gpu_with_a_message():
    """bench.py --gpus N > 1 exits with a message before touching a GPU (this build is one GPU)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr and not res.stdout.strip()
