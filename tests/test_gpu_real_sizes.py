"""GPU parity at the sizes the workloads name, where the tensors are gigabytes: VGG-16 layers on
full-HD frames at batch 8, tensors whose byte offsets pass 2^31, and a tensor too large for
the 32-bit buffer offsets of the matrix-core kernels (the layer must then take the direct
kernel).  The oracle computes a boundary-stratified sample of output positions one by one;
that every irrelevant row is all-zero bytes is checked in full on the device.  Also the
single-layer workload exactly as stated: fp32 storage, a top band plus three boxes, 48 %."""
import numpy as np
import pytest

from oracle import fc_oracle as O
from paper_2207_10741_amd import binding as B, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

TOL_F32_OUT = 1e-4


def _positions(m_out, count, seed, images=None):
    """Flat output positions: half of them kept positions next to a mask edge or the image border."""
    n, h, w = m_out.shape
    g = synth.rng(seed, 78)
    imgs = np.arange(n) if images is None else np.asarray(images)
    pos = []
    for b in imgs:
        m = m_out[b] != 0
        edge = np.zeros_like(m)
        edge[:2, :] = edge[-2:, :] = True
        edge[:, :2] = edge[:, -2:] = True
        edge[1:, :] |= m[1:, :] != m[:-1, :]
        edge[:-1, :] |= m[1:, :] != m[:-1, :]
        edge[:, 1:] |= m[:, 1:] != m[:, :-1]
        edge[:, :-1] |= m[:, 1:] != m[:, :-1]
        near = np.flatnonzero(edge & m)
        per = max(2, count // len(imgs))
        a = g.choice(near, size=min(per // 2, near.size), replace=False) if near.size else np.empty(0, np.int64)
        c = g.integers(0, h * w, size=per - a.size)
        # the first and the last position of the image as well
        pos.append(np.concatenate([a, c, [0, h * w - 1]]).astype(np.int64) + int(b) * h * w)
    return np.unique(np.concatenate(pos))


def _check_large(n, h, w, ci, co, k, p, mask, seed, samples=2000, images=None, expect_mfma=True):
    torch = G.torch_mod()
    dtype = synth.BF16
    x = synth.activations_large((n, h, w, ci), dtype, seed, 1)
    wt = synth.he_weights(co, k, k, ci, dtype, seed, 2)
    bias = synth.bias(co, seed, 3)
    shape = O.ConvShape(n, h, w, ci, co, k, k, (1, 1), (p, p), (1, 1), relu=True)
    m_out = O.mask_downsample(mask, k, k, (1, 1), (p, p))
    pos = _positions(m_out, samples, seed, images)
    want = O.focused_conv2d_at(shape, x, wt, pos, bias=bias, mask_in=mask, dtype=dtype)
    keep_rows = m_out.reshape(-1)[pos] != 0
    assert keep_rows.any() and not keep_rows.all()
    rms = float(np.sqrt(np.mean(want[keep_rows] ** 2)))
    xd = G.to_dev(x, dtype)
    del x
    desc = B.conv_desc(n, h, w, ci, co, (k, k), (1, 1), (p, p), (1, 1), dtype, B.F32, B.RELU)
    ho, wo = B.out_dims(desc)
    out = torch.full((n, ho, wo, co), 7.0, dtype=torch.float32, device=G.dev())
    md = G.mask_dev(mask)
    B.focused_conv2d(desc, xd, G.to_dev(wt, dtype), torch.from_numpy(bias).to(G.dev()), mask_in=md, out=out)
    torch.cuda.synchronize()
    got = out.reshape(-1, co)[torch.from_numpy(pos).to(G.dev())].to(torch.float64).cpu().numpy()
    err = float(np.abs(got - want).max()) / rms
    assert err <= TOL_F32_OUT, err
    assert not got[~keep_rows].any()
    # every irrelevant row all-zero bytes, every kept row written (no canary left), image by image
    keep_d = torch.from_numpy(m_out != 0).to(G.dev())
    for b in range(n):
        o = out[b].view(torch.int32)
        assert not bool(o[~keep_d[b]].any()), "image %d: an irrelevant row is not zero" % b
        assert not bool((out[b][keep_d[b]] == 7.0).all(dim=-1).any()), "image %d: a kept row was not written" % b
    return err


def test_vgg16_first_layer_hd_batch8():
    n, h, w = 8, 1080, 1920
    mask = synth.mask_depth_ramp(n, h, w, 0.5, 4, 0, 4)
    _check_large(n, h, w, 3, 64, 3, 1, mask, 901)


def test_vgg16_second_layer_hd_batch8():
    """64 -> 64 channels on 8 x 1080 x 1920 positions: the input tensor is 2.1 GB."""
    n, h, w = 8, 1080, 1920
    mask = synth.mask_depth_ramp(n, h, w, 0.5, 4, 0, 4)
    _check_large(n, h, w, 64, 64, 3, 1, mask, 902)


def test_vgg16_512_channel_layer_at_135x240_batch8():
    n, h, w = 8, 135, 240
    mask = synth.mask_depth_ramp(n, 1080, 1920, 0.5, 4, 0, 4)[:, ::8, ::8].copy()
    _check_large(n, h, w, 512, 512, 3, 1, mask, 903, samples=1200)


def test_masked_pool_hd_batch8():
    """The 2 x 2 pool after the second layer, with the propagated mask: kept positions hold the
    maximum of their window, the others +0."""
    torch = G.torch_mod()
    n, h, w, c = 8, 1080, 1920, 64
    dtype = synth.BF16
    mask = synth.mask_depth_ramp(n, h, w, 0.5, 4, 0, 4)
    x = synth.activations_large((n, h, w, c), dtype, 904, 1)
    keep = O.mask_downsample(mask, 2, 2, (2, 2), (0, 0))
    keep_d = G.mask_dev(keep)
    out = B.maxpool2d(G.to_dev(x, dtype), 2, 2, 0, B.BF16, keep=keep_d)
    torch.cuda.synchronize()
    g = synth.rng(904, 5)
    for b in range(n):
        xf = synth.from_storage(x[b], dtype)
        ref = xf.reshape(h // 2, 2, w // 2, 2, c).max(axis=(1, 3))
        ref[keep[b] == 0] = 0.0
        rows = g.integers(0, h // 2, size=40)
        got = out[b][torch.from_numpy(rows).to(G.dev())].to(torch.float32).cpu().numpy()
        np.testing.assert_array_equal(got, ref[rows])
        assert not bool(out[b][keep_d[b] == 0].view(torch.int16).any())


def test_byte_offsets_beyond_two_gib_on_the_matrix_cores():
    """Twelve HD frames of 64 channels: 3.2 GB, so the last five images lie beyond 2^31 bytes but
    inside the 32-bit offsets of the buffer descriptors.  Sampled in the last images."""
    n, h, w = 12, 1080, 1920
    assert 2 ** 31 < n * h * w * 64 * 2 < 0xF0000000
    mask = synth.mask_depth_ramp(n, h, w, 0.5, 905)
    _check_large(n, h, w, 64, 64, 3, 1, mask, 906, samples=1500, images=[7, 8, 10, 11])


def test_tensor_beyond_the_descriptor_range_takes_the_direct_kernel():
    """Sixteen HD frames of 64 channels are 4.2 GB: more than a buffer descriptor addresses, so the
    layer (a 1x1 projection here) runs on the direct kernel; the result must not change."""
    n, h, w = 16, 1080, 1920
    assert n * h * w * 64 * 2 >= 0xF0000000
    mask = synth.mask_depth_ramp(n, h, w, 0.5, 907)
    _check_large(n, h, w, 64, 8, 1, 0, mask, 908, samples=1500, images=[0, 7, 8, 15])


def test_single_layer_workload_as_stated():
    """One 3x3 layer, 64 -> 64 channels, batch 1, 56 x 56, fp32 storage, ReLU; irrelevant = a top band
    plus three boxes, 48 %.  Checked in full."""
    torch = G.torch_mod()
    n, h, w, c = 1, 56, 56, 64
    dtype = synth.F32
    x = synth.activations((n, h, w, c), dtype, 0, 0, 1)
    wt = synth.he_weights(c, 3, 3, c, dtype, 0, 0, 2)
    bias = synth.bias(c, 0, 0, 3)
    mask = synth.mask_band_and_boxes(n, h, w, 0.48, 0, 0, 4)
    assert abs(synth.irrelevant_fraction(mask) - 0.48) <= 0.01
    desc = B.conv_desc(n, h, w, c, c, in_dtype=B.F32, out_dtype=B.F32, flags=B.RELU)
    out = torch.full((n, h, w, c), 7.0, dtype=torch.float32, device=G.dev())
    md = G.mask_dev(mask)
    B.focused_conv2d(desc, G.to_dev(x, dtype), G.to_dev(wt, dtype), torch.from_numpy(bias).to(G.dev()), mask_in=md, out=out)
    torch.cuda.synchronize()
    want = O.focused_conv2d(O.ConvShape(n, h, w, c, c, relu=True), x, wt, bias=bias, mask_in=mask, dtype=dtype)
    keep = mask != 0
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_F32_OUT
    assert not out.cpu().numpy()[~keep].view(np.uint32).any()
    idx, count = B.active_index_compact(B.mask_downsample(md))
    want_idx, want_cnt = O.active_index_compact(O.mask_downsample(mask, 3, 3, (1, 1), (1, 1)))
    assert int(count.item()) == want_cnt and np.array_equal(idx[:want_cnt].cpu().numpy(), want_idx)
