"""Packed masks (one bit per pixel): packing, rescaling, compaction and the mask pyramid against
the oracle's byte masks after unpacking (bit-exact), and layers that take packed masks against
the same layers with byte masks (same kernels, same order: bit-identical outputs) and the oracle."""
import ctypes

import numpy as np
import pytest

from oracle import fc_oracle as O
from paper_2207_10741_amd import binding as B, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

TOL_F32_OUT = 1e-4


def pack_np(mask: np.ndarray) -> np.ndarray:
    """The layout written out: bit p % 64 of word p // 64, zero bits past the end."""
    flat = (mask.reshape(-1) != 0).astype(np.uint8)
    words = (flat.size + 63) // 64
    padded = np.zeros(words * 64, np.uint8)
    padded[:flat.size] = flat
    weights = (np.uint64(1) << np.arange(64, dtype=np.uint64))
    return (padded.reshape(words, 64).astype(np.uint64) * weights).sum(axis=1, dtype=np.uint64)


def unpack_dev(bits, m: int) -> np.ndarray:
    raw = bits.cpu().numpy().view(np.uint8)
    return np.unpackbits(raw, bitorder="little")[:m]


def bits_dev(mask: np.ndarray):
    torch = G.torch_mod()
    w = pack_np(mask)
    if w.size < 2:
        w = np.concatenate([w, np.zeros(2 - w.size, np.uint64)])
    return torch.from_numpy(w.view(np.int64)).to(G.dev())


@pytest.mark.parametrize("m", [1, 63, 64, 65, 1000, 4096, 4097, 100003, 3000017])
def test_pack_is_the_stated_layout(m):
    mask = synth.mask_bernoulli(1, 1, m, 0.45, 601, m) * np.uint8(5)     # nonzero, not just 1
    got = B.mask_pack(G.mask_dev(mask.reshape(-1)))
    want = pack_np(mask)
    np.testing.assert_array_equal(got.cpu().numpy().view(np.uint64)[:want.size], want)
    # and numpy's own little-endian bit packing agrees with the stated layout
    np.testing.assert_array_equal(np.packbits(mask.reshape(-1) != 0, bitorder="little"),
                                  want.view(np.uint8)[:(m + 7) // 8])


@pytest.mark.parametrize("n,h,w,k,s,p,d", [
    (1, 56, 56, 3, 1, 1, 1), (2, 57, 43, 3, 2, 1, 1), (3, 224, 224, 7, 2, 3, 1), (2, 135, 241, 2, 2, 0, 1),
    (1, 9, 300, 1, 2, 0, 1), (2, 33, 35, 3, 1, 2, 2), (1, 5, 5, 1, 1, 1, 1), (1, 1, 1, 1, 1, 0, 1),
])
def test_rescaling_and_compaction_of_packed_masks_bit_exact(n, h, w, k, s, p, d):
    mask = synth.mask_bernoulli(n, h, w, 0.45, 602, h, w)
    bits, shape = B.mask_downsample_packed(bits_dev(mask), (n, h, w), (k, k), (s, s), (p, p), (d, d))
    want = O.mask_downsample(mask, k, k, (s, s), (p, p), (d, d))
    assert shape == want.shape
    m = want.size
    np.testing.assert_array_equal(unpack_dev(bits, m), want.reshape(-1))
    assert not unpack_dev(bits, ((m + 63) // 64) * 64)[m:].any()          # zero bits past the end
    idx, count = B.active_index_compact_packed(bits, m)
    want_idx, want_cnt = O.active_index_compact(want)
    assert int(count.item()) == want_cnt
    np.testing.assert_array_equal(idx[:want_cnt].cpu().numpy(), want_idx)


@pytest.mark.parametrize("packed_in", [False, True])
@pytest.mark.parametrize("n,h,w,irr", [(2, 96, 128, 0.48), (1, 135, 241, 0.3), (16, 128, 128, 0.48), (3, 57, 43, 0.9)])
def test_packed_pyramid_matches_the_chain_of_rescalings(n, h, w, irr, packed_in):
    steps = [((3, 3), (1, 1), (1, 1), (1, 1)), ((3, 3), (2, 2), (1, 1), (1, 1)), ((1, 1), (2, 2), (0, 0), (1, 1)),
             ((2, 2), (2, 2), (0, 0), (1, 1))]
    mask = synth.mask_objects(n, h, w, irr, 603, h)
    src = bits_dev(mask) if packed_in else G.mask_dev(mask)
    pyr = B.PreparedPyramid(src, steps, packed=True, packed_in=packed_in, shape=(n, h, w))
    levels = pyr()
    G.torch_mod().cuda.synchronize()
    cur = mask
    for (bits, idx, count), dims, (k, s_, p, d) in zip(levels, pyr.dims, steps):
        cur = O.mask_downsample(cur, k[0], k[1], s_, p, d)
        assert dims == cur.shape
        np.testing.assert_array_equal(unpack_dev(bits, cur.size), cur.reshape(-1))
        want_idx, want_cnt = O.active_index_compact(cur)
        assert int(count.item()) == want_cnt
        np.testing.assert_array_equal(idx[:want_cnt].cpu().numpy(), want_idx)


LAYERS = [
    # n, h, w, ci, co, k, s, p, d
    (2, 40, 56, 64, 128, 3, 1, 1, 1),       # tiled matrix-core kernel, shared pixel lines (4480 positions)
    (1, 19, 23, 64, 128, 3, 2, 1, 1),       # small layer: ranks its rows inside the kernel
    (6, 64, 64, 64, 128, 3, 1, 1, 1),       # one-workgroup-per-CU kernel (24576 positions)
    (2, 20, 24, 64, 256, 1, 1, 0, 1),       # 1x1
    (1, 17, 13, 24, 40, 3, 1, 1, 1),        # channel tails
    (1, 12, 12, 5, 7, 3, 1, 1, 1),          # direct kernel
]


@pytest.mark.parametrize("with_list", [False, True])
@pytest.mark.parametrize("layer", LAYERS)
def test_layer_with_packed_masks_equals_the_layer_with_byte_masks(layer, with_list):
    torch = G.torch_mod()
    n, h, w, ci, co, k, s, p, d = layer
    dtype = synth.BF16
    x = synth.activations((n, h, w, ci), dtype, 604, 1)
    wt = synth.he_weights(co, k, k, ci, dtype, 604, 2)
    bias = synth.bias(co, 604, 3)
    mask = synth.mask_objects(n, h, w, 0.48, 604, 4)
    xd, wd, bd = G.to_dev(x, dtype), G.to_dev(wt, dtype), torch.from_numpy(bias).to(G.dev())
    md, mbits = G.mask_dev(mask), bits_dev(mask)
    geom = ((k, k), (s, s), (p, p), (d, d))
    outs = []
    for packed in (False, True):
        desc = B.conv_desc(n, h, w, ci, co, *geom, dtype, B.F32, B.RELU | (B.PACKED_MASKS if packed else 0))
        ho, wo = B.out_dims(desc)
        out = torch.full((n, ho, wo, co), 7.0, dtype=torch.float32, device=G.dev())
        kw = {}
        if with_list:
            if packed:
                labels, shape = B.mask_downsample_packed(mbits, (n, h, w), *geom)
                idx, count = B.active_index_compact_packed(labels, shape[0] * shape[1] * shape[2])
            else:
                labels = B.mask_downsample(md, *geom)
                idx, count = B.active_index_compact(labels)
            kw = dict(mask_out=labels, idx=idx, count=count)
        ws = torch.empty((B.workspace_bytes(desc),), dtype=torch.uint8, device=G.dev())
        B.focused_conv2d(desc, xd, wd, bd, mask_in=mbits if packed else md, out=out, workspace=ws, **kw)
        torch.cuda.synchronize()
        outs.append(out)
    assert torch.equal(outs[0], outs[1])
    want = O.focused_conv2d(O.ConvShape(n, h, w, ci, co, k, k, (s, s), (p, p), (d, d), relu=True), x, wt, bias=bias,
                            mask_in=mask, dtype=dtype)
    keep = O.mask_downsample(mask, k, k, (s, s), (p, p), (d, d)) != 0
    assert G.rel_err(G.to_f64(outs[1]), want, keep) <= TOL_F32_OUT
    assert not outs[1].cpu().numpy()[~keep].view(np.uint32).any()


def test_grouped_layer_with_packed_masks():
    torch = G.torch_mod()
    n, h, w, c, groups = 2, 30, 41, 32, 4
    dtype = synth.BF16
    x = synth.activations((n, h, w, c), dtype, 605, 1)
    wt = synth.he_weights(c, 3, 3, c // groups, dtype, 605, 2)
    mask = synth.mask_objects(n, h, w, 0.48, 605, 4)
    xd, wd = G.to_dev(x, dtype), G.to_dev(wt, dtype)
    outs = []
    for packed in (False, True):
        desc = B.conv_desc(n, h, w, c, c, in_dtype=dtype, out_dtype=B.F32, flags=B.PACKED_MASKS if packed else 0)
        outs.append(B.focused_gconv2d(desc, groups, xd, wd, mask_in=bits_dev(mask) if packed else G.mask_dev(mask)))
    torch.cuda.synchronize()
    assert torch.equal(outs[0], outs[1])
    want = O.focused_gconv2d(O.ConvShape(n, h, w, c, c), groups, x, wt, mask_in=mask, dtype=dtype)
    assert G.rel_err(G.to_f64(outs[1]), want, mask != 0) <= TOL_F32_OUT


def test_layers_that_read_byte_masks_refuse_packed_ones():
    torch = G.torch_mod()
    t = torch.zeros((4096,), dtype=torch.uint8, device=G.dev())
    o = torch.zeros((1 << 20,), dtype=torch.uint8, device=G.dev())
    stem = B.conv_desc(1, 16, 16, 3, 64, in_dtype=B.BF16, out_dtype=B.BF16, flags=B.PACKED_MASKS)
    rc = B.lib().fc_focused_conv2d(ctypes.byref(stem), t.data_ptr(), t.data_ptr(), t.data_ptr(), None, None, None,
                                   None, o.data_ptr(), None, 0, None)
    assert rc == -3
    dw = B.conv_desc(1, 16, 16, 16, 16, in_dtype=B.BF16, out_dtype=B.BF16, flags=B.PACKED_MASKS)
    assert B.lib().fc_focused_dwconv2d(ctypes.byref(dw), t.data_ptr(), t.data_ptr(), t.data_ptr(), None, o.data_ptr(),
                                       None) == -3
