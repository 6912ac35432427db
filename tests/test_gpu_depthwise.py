"""GPU parity of the depthwise focused layer (fc_focused_dwconv2d, through the C ABI) against
the CPU oracle on the same seeded inputs.  Bars as for the full layer: fp32 output within 1e-4
of the oracle relative to the RMS of the kept outputs; 16-bit output equal to the
round-to-nearest-even of the fp32 output; irrelevant rows all-zero bytes."""
import numpy as np
import pytest

from oracle import fc_oracle as O
from paper_2207_10741_amd import binding as B, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

TOL_F32_OUT = 1e-4


def _pair(v):
    return tuple(v) if isinstance(v, (tuple, list)) else (v, v)


def _inputs(n, h, w, c, k, dtype, seed, mask_kind, irr):
    kh, kw = _pair(k)
    x = synth.activations((n, h, w, c), dtype, seed, 1)
    wt = np.ascontiguousarray(synth.he_weights(c, kh, kw, 1, dtype, seed, 2)[..., 0])
    bias = synth.bias(c, seed, 3)
    if mask_kind == "objects":
        mask = synth.mask_objects(n, h, w, irr, seed, 4)
    elif mask_kind == "bernoulli":
        mask = synth.mask_bernoulli(n, h, w, irr, seed, 4)
    else:
        mask = None
    return x, wt, bias, mask


def _run(n, h, w, c, k, s, p, d, dtype, *, mask_kind="objects", irr=0.48, relu=True, use_bias=True,
         out_dtype=B.F32, seed=300, flags_extra=0, x_override=None):
    torch = G.torch_mod()
    kh, kw = _pair(k)
    s, p, d = _pair(s), _pair(p), _pair(d)
    x, wt, bias, mask = _inputs(n, h, w, c, k, dtype, seed, mask_kind, irr)
    if x_override is not None:
        x = x_override(x, mask)
    if not use_bias:
        bias = None
    desc = B.conv_desc(n, h, w, c, c, (kh, kw), s, p, d, dtype, out_dtype, (B.RELU if relu else 0) | flags_extra)
    ho, wo = B.out_dims(desc)
    # the output starts full of a canary, so a row nobody writes cannot pass as zero
    out = torch.full((n, ho, wo, c), 7.0, dtype=B.torch_dtype(out_dtype), device=G.dev())
    B.focused_dwconv2d(desc, G.to_dev(x, dtype), G.to_dev(wt, dtype),
                       None if bias is None else torch.from_numpy(bias).to(G.dev()),
                       mask_in=None if mask is None else G.mask_dev(mask), out=out)
    torch.cuda.synchronize()
    shape = O.ConvShape(n, h, w, c, c, kh, kw, s, p, d, relu=relu)
    want = O.focused_dwconv2d(shape, x, wt, bias=bias, mask_in=mask, dtype=dtype)
    keep = (O.mask_downsample(mask, kh, kw, s, p, d) != 0) if mask is not None else np.ones(want.shape[:3], bool)
    return out, want, keep


DW_LAYERS = [
    # n, h, w, c, k, s, p, d
    (2, 56, 56, 32, 3, 1, 1, 1),               # 4 lanes per position
    (2, 37, 53, 96, 3, 2, 1, 1),               # stride 2, ragged size, 12 lanes per position
    (1, 28, 28, 144, 3, 1, 1, 1),              # 18 lanes per position: 252 of 256 lanes used
    (3, 9, 7, 960, 3, 1, 1, 1),                # 120 lanes per position, two positions per step
    (1, 6, 5, 2304, 3, 1, 1, 1),               # more chunks than lanes: two channel tiles
    (2, 30, 41, 40, 5, 1, 2, 1),               # 5 x 5 filters kept packed in registers
    (1, 33, 29, 72, 5, 2, 2, 1),
    (2, 21, 40, 64, 3, (2, 1), (0, 2), (2, 1)),  # vertical stride and dilation, wide padding
    (1, 25, 31, 24, (3, 5), 1, (1, 2), 1),     # not square: filters read per tap
    (1, 40, 36, 16, 7, 2, 3, 1),
    (2, 19, 23, 20, 3, 1, 1, 1),               # channel count not a multiple of 8: one channel per lane
    (1, 17, 13, 7, (2, 3), (2, 1), 0, 1),      # even kernel height, odd channel count
    (1, 1, 1, 8, 3, 1, 1, 1),                  # a single position
    (2, 70, 75, 32, 3, 1, 1, 1),               # several tiles each way, ragged last tiles
    (1, 45, 50, 24, 5, 1, 2, 1),               # 5 x 5 over several tiles
    (1, 64, 64, 128, 3, 1, 30, 30),            # dilation too wide for a staged patch: direct kernel
]


@pytest.mark.parametrize("layer", DW_LAYERS)
@pytest.mark.parametrize("dtype", [synth.BF16, synth.F16])
def test_depthwise_matches_oracle_fp32_out(layer, dtype):
    out, want, keep = _run(*layer, dtype)
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_F32_OUT
    assert not out.cpu().numpy()[~keep].view(np.uint32).any()


@pytest.mark.parametrize("layer", [DW_LAYERS[0], DW_LAYERS[5], DW_LAYERS[8], DW_LAYERS[10], DW_LAYERS[11]])
def test_depthwise_fp32_storage(layer):
    out, want, keep = _run(*layer, synth.F32)
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_F32_OUT
    assert not out.cpu().numpy()[~keep].view(np.uint32).any()


@pytest.mark.parametrize("layer", [DW_LAYERS[1], DW_LAYERS[2], DW_LAYERS[5], DW_LAYERS[8]])
@pytest.mark.parametrize("mask_kind", ["bernoulli", None])
def test_depthwise_mask_structures(layer, mask_kind):
    out, want, keep = _run(*layer, synth.BF16, mask_kind=mask_kind, irr=0.5, seed=301)
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_F32_OUT
    assert not out.cpu().numpy()[~keep].view(np.uint32).any()


@pytest.mark.parametrize("irr", [0.0, 1.0, 0.97])
def test_depthwise_extreme_densities(irr):
    out, want, keep = _run(2, 24, 30, 48, 3, 1, 1, 1, synth.BF16, mask_kind="bernoulli", irr=irr, seed=302)
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_F32_OUT
    assert not out.cpu().numpy()[~keep].view(np.uint32).any()


@pytest.mark.parametrize("layer", [DW_LAYERS[0], DW_LAYERS[5], DW_LAYERS[10]])
@pytest.mark.parametrize("dtype", [synth.BF16, synth.F16])
def test_depthwise_16bit_output_is_rne_of_fp32_output(layer, dtype):
    torch = G.torch_mod()
    a, _, _ = _run(*layer, dtype, seed=303)
    b, _, _ = _run(*layer, dtype, seed=303, out_dtype=dtype)
    assert torch.equal(b, a.to(b.dtype))


def test_depthwise_without_bias_and_relu():
    out, want, keep = _run(*DW_LAYERS[1], synth.BF16, relu=False, use_bias=False, seed=304)
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_F32_OUT
    assert (G.to_f64(out) < 0).any()


def test_depthwise_nan_at_irrelevant_inputs_does_not_leak():
    def poison(x, mask):
        x = x.copy()
        x[mask == 0] = 0x7FC0          # bf16 NaN bit pattern
        return x
    clean, want, keep = _run(*DW_LAYERS[0], synth.BF16, seed=305)
    dirty, _, _ = _run(*DW_LAYERS[0], synth.BF16, seed=305, x_override=poison)
    assert G.torch_mod().equal(clean, dirty)
    assert np.isfinite(G.to_f64(dirty)).all()


def test_depthwise_skip_zero_fill_leaves_irrelevant_rows_untouched():
    out, want, keep = _run(*DW_LAYERS[2], synth.BF16, seed=306, flags_extra=B.SKIP_ZERO_FILL)
    got = G.to_f64(out)
    assert (got[~keep] == 7.0).all()
    rms = float(np.sqrt(np.mean(np.square(want[keep]))))
    assert np.abs(got[keep] - want[keep]).max() / rms <= TOL_F32_OUT


def test_depthwise_sampled_positions_at_a_large_size():
    """A MobileNetV2-shaped layer at the batch the benchmark times: fp32 output checked on sampled
    rows, the bf16 output the benchmark writes checked as its rounding, zero rows checked in full."""
    torch = G.torch_mod()
    n, h, w, c = 32, 112, 112, 96
    x, wt, bias, mask = _inputs(n, h, w, c, 3, synth.BF16, 307, "objects", 0.48)
    xd, wd, bd, md = (G.to_dev(x, synth.BF16), G.to_dev(wt, synth.BF16), torch.from_numpy(bias).to(G.dev()),
                      G.mask_dev(mask))
    geom = (n, h, w, c, c, (3, 3), (1, 1), (1, 1), (1, 1), synth.BF16)
    out32 = B.focused_dwconv2d(B.conv_desc(*geom, synth.F32, B.RELU), xd, wd, bd, mask_in=md)
    out16 = B.focused_dwconv2d(B.conv_desc(*geom, synth.BF16, B.RELU), xd, wd, bd, mask_in=md)
    torch.cuda.synchronize()
    rng = np.random.default_rng(307)
    pos = np.unique(rng.integers(0, n * h * w, 20000))
    want = O.focused_dwconv2d_at(O.ConvShape(n, h, w, c, c, relu=True), x, wt, pos, bias=bias, mask_in=mask,
                                 dtype=synth.BF16)
    got = out32.reshape(-1, c)[torch.from_numpy(pos).to(G.dev())].to(torch.float64).cpu().numpy()
    keep = mask.reshape(-1)[pos] != 0
    rms = float(np.sqrt(np.mean(np.square(want[keep]))))
    assert np.abs(got - want).max() / rms <= TOL_F32_OUT
    assert torch.equal(out16, out32.to(torch.bfloat16))
    # every irrelevant row of the whole tensor is zero bytes
    assert not out16.view(torch.int16)[torch.from_numpy(mask == 0).to(G.dev())].any()
