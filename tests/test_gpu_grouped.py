"""GPU parity of the grouped layer (fc_focused_gconv2d) against the CPU oracle: fp32 output
within 1e-4 of the RMS of the kept outputs, +0.0 at irrelevant positions, 16-bit output equal to
the rounding of the fp32 output."""
import numpy as np
import pytest

from oracle import fc_oracle as O
from paper_2207_10741_amd import binding as B, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

TOL_F32_OUT = 1e-4

GROUPED_LAYERS = [
    # n, h, w, ci, co, k, s, p, groups
    (2, 28, 28, 128, 128, 3, 1, 1, 32),     # ResNeXt-style: 4 channels per group
    (1, 30, 41, 64, 128, 3, 1, 1, 4),
    (2, 19, 23, 96, 48, 3, 2, 1, 3),        # stride 2, fewer output channels per group
    (1, 17, 13, 24, 40, 1, 1, 0, 8),        # 1x1, 3 -> 5 channels per group
    (1, 12, 12, 10, 15, 5, 1, 2, 5),        # odd channel counts
    (3, 64, 64, 256, 256, 3, 1, 1, 32),     # many rows
    (1, 14, 14, 32, 32, 3, 1, 1, 32),       # one channel per group: runs the depthwise kernel
    (1, 14, 14, 32, 64, 3, 1, 1, 1),        # one group: runs the full layer
]


def _run(layer, dtype, out_dtype, mask_kind="objects", irr=0.48, relu=True, precomputed=False, flags_extra=0):
    torch = G.torch_mod()
    n, h, w, ci, co, k, s, p, groups = layer
    x = synth.activations((n, h, w, ci), dtype, 400, 1)
    wt = synth.he_weights(co, k, k, ci // groups, dtype, 400, 2)
    bias = synth.bias(co, 400, 3)
    mask = None if mask_kind is None else (synth.mask_bernoulli if mask_kind == "bernoulli" else synth.mask_objects)(
        n, h, w, irr, 400, 4)
    desc = B.conv_desc(n, h, w, ci, co, (k, k), (s, s), (p, p), (1, 1), dtype, out_dtype,
                       (B.RELU if relu else 0) | flags_extra)
    ho, wo = B.out_dims(desc)
    out = torch.full((n, ho, wo, co), 7.0, dtype=B.torch_dtype(out_dtype), device=G.dev())
    md = None if mask is None else G.mask_dev(mask)
    kw = {}
    if precomputed and mask is not None:
        m_out = B.mask_downsample(md, (k, k), (s, s), (p, p))
        idx, count = B.active_index_compact(m_out)
        kw = dict(mask_out=m_out, idx=idx, count=count)
    wd = G.to_dev(wt, dtype)
    B.focused_gconv2d(desc, groups, G.to_dev(x, dtype), wd, torch.from_numpy(bias).to(G.dev()), mask_in=md, out=out, **kw)
    torch.cuda.synchronize()
    want = O.focused_gconv2d(O.ConvShape(n, h, w, ci, co, k, k, (s, s), (p, p), (1, 1), relu=relu), groups, x, wt,
                             bias=bias, mask_in=mask, dtype=dtype)
    keep = (O.mask_downsample(mask, k, k, (s, s), (p, p)) != 0) if mask is not None else np.ones(want.shape[:3], bool)
    return out, want, keep


@pytest.mark.parametrize("layer", GROUPED_LAYERS)
@pytest.mark.parametrize("dtype", [synth.BF16, synth.F16, synth.F32])
def test_grouped_layer_matches_oracle(layer, dtype):
    out, want, keep = _run(layer, dtype, B.F32)
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_F32_OUT
    assert not out.cpu().numpy()[~keep].view(np.uint32).any()


@pytest.mark.parametrize("layer", GROUPED_LAYERS[:6])
@pytest.mark.parametrize("mask_kind,irr", [("bernoulli", 0.5), (None, 0.0), ("objects", 1.0), ("objects", 0.0)])
def test_grouped_layer_mask_structures_and_given_lists(layer, mask_kind, irr):
    out, want, keep = _run(layer, synth.BF16, B.F32, mask_kind=mask_kind, irr=irr, relu=False, precomputed=True)
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_F32_OUT
    assert not out.cpu().numpy()[~keep].view(np.uint32).any()


@pytest.mark.parametrize("layer", [GROUPED_LAYERS[0], GROUPED_LAYERS[2], GROUPED_LAYERS[4]])
@pytest.mark.parametrize("dtype", [synth.BF16, synth.F16])
def test_grouped_layer_16bit_out_is_rounded_fp32_out_and_skip_zero_fill(layer, dtype):
    torch = G.torch_mod()
    out32, _, keep = _run(layer, dtype, B.F32)
    out16, _, _ = _run(layer, dtype, dtype)
    assert torch.equal(out16, out32.to(out16.dtype))
    # irrelevant rows stay as they were when the caller asks for that
    left, _, _ = _run(layer, dtype, B.F32, flags_extra=B.SKIP_ZERO_FILL)
    got = left.cpu().numpy()
    assert (got[~keep] == 7.0).all() and np.array_equal(got[keep], out32.cpu().numpy()[keep])


def test_grouped_layer_argument_errors():
    torch = G.torch_mod()
    a = torch.zeros((1 << 16,), dtype=torch.uint8, device=G.dev())
    o = torch.zeros((1 << 18,), dtype=torch.uint8, device=G.dev())
    d = B.conv_desc(1, 8, 8, 24, 36, in_dtype=B.BF16, out_dtype=B.F32)
    for groups, status in ((5, -2), (0, -2), (-3, -2)):
        with pytest.raises(B.FcError) as e:
            B.focused_gconv2d(d, groups, a, a, None, out=o.view(torch.float32))
        assert e.value.status == status
    d8 = B.conv_desc(1, 8, 8, 32, 32, in_dtype=B.FP8, out_dtype=B.F32)
    with pytest.raises(B.FcError) as e:
        B.focused_gconv2d(d8, 2, a, a, None, out=o.view(torch.float32))
    assert e.value.status == -3


@pytest.mark.parametrize("layer", [GROUPED_LAYERS[0], GROUPED_LAYERS[1], GROUPED_LAYERS[5], (1, 20, 20, 64, 96, 1, 1, 0, 4)])
@pytest.mark.parametrize("dtype", [synth.BF16, synth.F32, synth.FP8])
def test_expanded_group_weights_run_the_grouped_layer_on_the_full_layer_path(layer, dtype):
    """Block-diagonal weights: bit-exact expansion (against numpy), and the full layer run with
    them matches the oracle's grouped layer."""
    torch = G.torch_mod()
    n, h, w, ci, co, k, s_, p, groups = layer
    if dtype == synth.FP8 and (ci % 16 or co % 8):
        pytest.skip("not an 8-bit matrix-core shape")
    x = synth.activations((n, h, w, ci), dtype, 401, 1)
    wt = synth.he_weights(co, k, k, ci // groups, dtype, 401, 2)
    bias = synth.bias(co, 401, 3)
    mask = synth.mask_objects(n, h, w, 0.48, 401, 4)
    full = B.expand_group_weights(G.to_dev(wt, dtype), groups, dtype)
    cig, cog = ci // groups, co // groups
    want_w = np.zeros((co, k, k, ci), wt.dtype)
    for g in range(groups):
        want_w[g * cog:(g + 1) * cog, :, :, g * cig:(g + 1) * cig] = wt[g * cog:(g + 1) * cog]
    np.testing.assert_array_equal(G.to_storage_np(full, dtype), want_w)
    desc = B.conv_desc(n, h, w, ci, co, (k, k), (s_, s_), (p, p), (1, 1), dtype, B.F32, B.RELU)
    out = B.focused_conv2d(desc, G.to_dev(x, dtype), full, torch.from_numpy(bias).to(G.dev()), mask_in=G.mask_dev(mask))
    want = O.focused_gconv2d(O.ConvShape(n, h, w, ci, co, k, k, (s_, s_), (p, p), (1, 1), relu=True), groups, x, wt,
                             bias=bias, mask_in=mask, dtype=dtype)
    keep = O.mask_downsample(mask, k, k, (s_, s_), (p, p)) != 0
    assert G.rel_err(G.to_f64(out), want, keep) <= (5e-4 if dtype == synth.FP8 else TOL_F32_OUT)
