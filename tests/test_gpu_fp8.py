"""GPU parity of the 8-bit (E4M3) layers: the matrix-core path fed bytes, against the CPU
oracle fed the same bytes.

Tolerance.  Products of two E4M3 values are exact, but the 8-bit matrix instruction
(v_mfma_f32_32x32x64_f8f6f4) does not add them in fp32 one by one: it adds each aligned run
of 8 products (8 consecutive input channels of one tap here) on a fixed-point grid of 2^-13
times the power of two at or below the run's largest product, dropping what falls below the
grid, and only the runs' sums and the accumulator are added in fp32 (measured with an
in-bounds probe of the instruction: a second product of 2^-13 of the largest survives, one of
2^-14 is lost; products in different runs keep all 24 bits).  An output is therefore off by
less than sum over runs of 7 * 2^-13 * (largest |product| of the run), which
test_fp8_error_stays_inside_the_bound_of_the_instruction checks element by element; a product
of two 4-bit significands has 8 bits, so only products below 2^-6 of their run's largest lose
anything, and the typical error is far below the bound: 2e-6 of the output RMS on average,
2e-4 at worst over the layers below.  The bar for fp32 output is 5e-4 of the RMS of the kept
outputs; bf16 output must equal the round-to-nearest-even of the fp32 output bit for bit.

8-bit output.  The stored code is a rounding decision taken on the fp32 result, so it is checked
three ways: (1) where every sum is a small integer the fp32 result is exact on both sides and the
codes must equal the oracle's, ties and saturation included; (2) on ordinary inputs the codes must
equal the oracle's narrowing of the kernel's own fp32 output bit for bit (the decision in the
kernel's precision); (3) against the oracle end to end, a stored value v may be off the exact
result y by the distance from y to the nearest E4M3 value plus twice the fp32 tolerance, which is
what a correct rounding of a result within that tolerance gives."""

import numpy as np
import pytest

from oracle import fc_oracle as O
from paper_2207_10741_amd import binding as B, synth
from tests import gpu_util as G
from tests.test_gpu_parity import _run_layer

pytestmark = pytest.mark.gpu

TOL_FP8 = 5e-4

FP8_LAYERS = [
    # n, h, w, ci, co, k, s, p, d
    (1, 56, 56, 64, 64, 3, 1, 1, 1),        # half a stage of channels, shared-halo loop
    (2, 30, 41, 128, 64, 3, 1, 1, 1),       # exactly one stage per tap, ragged spatial size
    (2, 28, 28, 256, 128, 3, 1, 1, 1),
    (1, 19, 23, 64, 128, 3, 2, 1, 1),       # stride-2 3x3 (tap by tap)
    (2, 20, 24, 64, 256, 1, 1, 0, 1),       # 1x1
    (1, 21, 21, 128, 256, 1, 2, 0, 1),      # 1x1 / 2 projection
    (1, 14, 14, 256, 256, 3, 1, 1, 1),
    (1, 7, 9, 512, 512, 3, 1, 1, 1),        # few rows, long K
    (1, 24, 24, 32, 48, 3, 1, 2, 2),        # dilation
    (1, 17, 13, 16, 40, 3, 1, 1, 1),        # the fewest channels the path takes
    (1, 20, 36, 144, 72, 3, 1, 1, 1),       # a second stage with a 16-channel tail
    (1, 16, 18, 48, 24, 5, 1, 2, 1),        # 25 taps
    (1, 40, 40, 208, 8, 1, 1, 0, 1),        # eight output channels
    (4, 64, 64, 64, 64, 3, 1, 1, 1),        # more positions than one workgroup ranks itself
]


@pytest.mark.parametrize("layer", FP8_LAYERS)
def test_fp8_layer_matches_oracle_fp32_out(layer):
    out, want, keep = _run_layer(*layer, synth.FP8)
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_FP8
    assert not out.cpu().numpy()[~keep].view(np.uint32).any()        # +0.0 bit pattern


@pytest.mark.parametrize("layer", FP8_LAYERS[:8])
@pytest.mark.parametrize("mask_kind", ["bernoulli", "mixed", None])
def test_fp8_layer_mask_structures(layer, mask_kind):
    out, want, keep = _run_layer(*layer, synth.FP8, mask_kind=mask_kind, irr=0.5, seed=211)
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_FP8


@pytest.mark.parametrize("layer", [FP8_LAYERS[0], FP8_LAYERS[3], FP8_LAYERS[4]])
@pytest.mark.parametrize("irr", [0.0, 1.0, 0.9])
def test_fp8_layer_extreme_densities(layer, irr):
    out, want, keep = _run_layer(*layer, synth.FP8, irr=irr, seed=212)
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_FP8


@pytest.mark.parametrize("layer", [FP8_LAYERS[0], FP8_LAYERS[2], FP8_LAYERS[4], FP8_LAYERS[7]])
def test_fp8_layer_bf16_out_is_rounded_fp32_out_and_list_paths_agree(layer):
    """bf16 output = RNE of the fp32 output, bit for bit; a call given the mask, the list and a
    workspace (split reductions for small layers) gives the same bits as one given the mask only."""
    torch = G.torch_mod()
    out32, want, keep = _run_layer(*layer, synth.FP8, seed=213)
    out16, _, _ = _run_layer(*layer, synth.FP8, seed=213, out_dtype=B.BF16)
    np.testing.assert_array_equal(out16.view(torch.int16).cpu().numpy(),
                                  out32.to(torch.bfloat16).view(torch.int16).cpu().numpy())
    pre32, _, _ = _run_layer(*layer, synth.FP8, seed=213, precomputed=True)
    assert G.rel_err(G.to_f64(pre32), want, keep) <= TOL_FP8
    again, _, _ = _run_layer(*layer, synth.FP8, seed=213, precomputed=True)
    assert torch.equal(pre32, again)                                  # deterministic


@pytest.mark.parametrize("layer", [(1, 12, 14, 64, 32, 1, 1, 0, 1), (1, 10, 12, 32, 16, 3, 1, 1, 1),
                                   (1, 9, 9, 144, 24, 3, 2, 1, 1)])
def test_fp8_error_stays_inside_the_bound_of_the_instruction(layer):
    """|gpu - oracle| <= sum over aligned runs of 8 input channels of one tap of
    7 * 2^-13 * max |x * w| over the run, plus fp32 rounding of the running sum (dense layer,
    no ReLU, so that every output is a plain sum)."""
    n, h, w, ci, co, k, s_, p, d = layer
    out, want, keep = _run_layer(*layer, synth.FP8, mask_kind=None, relu=False, seed=216)
    x = synth.from_storage(synth.activations((n, h, w, ci), synth.FP8, 216, 1), synth.FP8).astype(np.float64)
    wt = synth.from_storage(synth.he_weights(co, k, k, ci, synth.FP8, 216, 2), synth.FP8).astype(np.float64)
    ho, wo = want.shape[1:3]
    xp = np.zeros((n, h + 2 * p, w + 2 * p, ci))
    xp[:, p:p + h, p:p + w] = x
    bound = np.zeros_like(want)
    mag = np.zeros_like(want)
    for i in range(k):
        for j in range(k):
            sl = xp[:, i * d: i * d + (ho - 1) * s_ + 1: s_, j * d: j * d + (wo - 1) * s_ + 1: s_, :]
            prod = np.abs(sl[:, :, :, None, :] * wt[None, None, None, :, i, j, :])      # [n,ho,wo,co,ci]
            runs = prod.reshape(n, ho, wo, co, ci // 8, 8)
            bound += 7 * 2.0 ** -13 * runs.max(axis=-1).sum(axis=-1)
            mag += prod.sum(axis=-1)
    slack = mag * (2.0 ** -23) * (k * k * ci // 8 + 2)                                # fp32 adds of the runs
    err = np.abs(G.to_f64(out) - want)
    assert (err <= bound + slack).all()
    assert err.max() > 0                        # the instruction does round: the bound is not vacuous


def test_fp8_every_code_times_every_code():
    """A 1x1 layer whose inputs run over all 254 finite codes (every pixel holds each of them
    once, rotated from pixel to pixel) against weights drawn from the codes up to |2|: sums of
    256 exact products, checked against the oracle; then a NaN code in one kept pixel makes
    that pixel's outputs NaN and no other."""
    torch = G.torch_mod()
    finite = np.array([c for c in range(256) if c & 0x7F != 0x7F], np.uint8)        # 254 codes
    g = synth.rng(214)
    n, h, w, ci, co = 1, 16, 16, 256, 64
    x = finite[g.integers(0, 254, size=(n, h, w, ci))]
    x[0, :, :, :254] = finite[(np.arange(h * w)[:, None] + np.arange(254)[None, :]).reshape(h, w, 254) % 254]
    small = np.array([c for c in finite if (c & 0x7F) <= 0x40], np.uint8)           # |v| <= 2: sums stay tame
    wt = small[g.integers(0, small.size, size=(co, 1, 1, ci))]
    mask = synth.mask_objects(n, h, w, 0.3, 214, 1)
    desc = B.conv_desc(n, h, w, ci, co, (1, 1), (1, 1), (0, 0), (1, 1), B.FP8, B.F32, 0)
    out = B.focused_conv2d(desc, G.to_dev(x, synth.FP8), G.to_dev(wt, synth.FP8), None, mask_in=G.mask_dev(mask))
    want = O.focused_conv2d(O.ConvShape(n, h, w, ci, co, 1, 1, pad=(0, 0), relu=False), x, wt, mask_in=mask,
                            dtype=O.FP8)
    keep = mask != 0
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_FP8
    kept = np.argwhere(keep)
    b, r, c = kept[len(kept) // 2]
    x[b, r, c, 7] = 0x7F
    out = B.focused_conv2d(desc, G.to_dev(x, synth.FP8), G.to_dev(wt, synth.FP8), None, mask_in=G.mask_dev(mask))
    got = out.cpu().numpy()
    assert np.isnan(got[b, r, c]).all()
    got[b, r, c] = 0
    assert np.isfinite(got).all()


def test_fp8_large_layer_on_sampled_positions():
    """A bench-sized layer (C256 at 32x32, batch 16) on 4096 sampled positions plus all-zero
    irrelevant rows."""
    torch = G.torch_mod()
    n, side, c = 16, 32, 256
    x = synth.activations((n, side, side, c), synth.FP8, 215, 1)
    wt = synth.he_weights(c, 3, 3, c, synth.FP8, 215, 2)
    bias = synth.bias(c, 215, 3)
    mask = synth.mask_objects(n, side, side, 0.48, 215, 4)
    desc = B.conv_desc(n, side, side, c, c, in_dtype=B.FP8, out_dtype=B.F32, flags=B.RELU)
    ws = torch.zeros((B.workspace_bytes(desc),), dtype=torch.uint8, device=G.dev())
    out = B.focused_conv2d(desc, G.to_dev(x, synth.FP8), G.to_dev(wt, synth.FP8),
                           torch.from_numpy(bias).to(G.dev()), mask_in=G.mask_dev(mask), workspace=ws)
    got = out.cpu().numpy().reshape(-1, c)
    keep = (mask != 0).reshape(-1)
    assert not got[~keep].view(np.uint32).any()
    pos = synth.rng(215, 9).choice(np.flatnonzero(keep), size=4096, replace=False)
    want = O.focused_conv2d_at(O.ConvShape(n, side, side, c, c, relu=True), x, wt, pos, bias=bias, mask_in=mask,
                               dtype=O.FP8)
    rms = float(np.sqrt(np.mean(np.square(want))))
    assert float(np.abs(got[pos] - want).max()) / rms <= TOL_FP8


@pytest.mark.parametrize("layer", [
    (8, 96, 96, 64, 128, 3, 1, 1),      # many 128 x 128 tiles (one set of operand fragments), shared pixel line
    (8, 96, 96, 256, 256, 3, 1, 1),     # the same with two stages per tap
    (4, 64, 64, 128, 128, 3, 1, 1),     # 128 x 64, shared pixel line
    (6, 80, 80, 64, 64, 3, 1, 1),       # 64 output channels
    (4, 72, 72, 96, 192, 3, 2, 1),      # stride 2: tap by tap
    (4, 96, 96, 256, 320, 1, 1, 0),     # 1x1, 128 x 128 tiles
])
@pytest.mark.parametrize("mask_kind,irr", [("objects", 0.48), ("bernoulli", 0.5), ("objects", 0.0)])
def test_fp8_large_tile_instances_sampled(layer, mask_kind, irr):
    """Layers with enough tiles for the large-tile instances, on sampled positions (half of them
    near a mask edge or the image border) plus all-zero irrelevant rows."""
    from tests.test_gpu_stacks import _sample_positions
    torch = G.torch_mod()
    n, h, w, ci, co, k, s_, p = layer
    x = synth.activations((n, h, w, ci), synth.FP8, 217, 1)
    wt = synth.he_weights(co, k, k, ci, synth.FP8, 217, 2)
    bias = synth.bias(co, 217, 3)
    mask = (synth.mask_bernoulli if mask_kind == "bernoulli" else synth.mask_objects)(n, h, w, irr, 217, h, ci)
    desc = B.conv_desc(n, h, w, ci, co, (k, k), (s_, s_), (p, p), (1, 1), B.FP8, B.F32, B.RELU)
    out = B.focused_conv2d(desc, G.to_dev(x, synth.FP8), G.to_dev(wt, synth.FP8),
                           torch.from_numpy(bias).to(G.dev()), mask_in=G.mask_dev(mask))
    m_out = O.mask_downsample(mask, k, k, (s_, s_), (p, p))
    got = out.cpu().numpy().reshape(-1, co)
    assert not got[m_out.reshape(-1) == 0].view(np.uint32).any()
    pos = _sample_positions(m_out, 1500, 218)
    want = O.focused_conv2d_at(O.ConvShape(n, h, w, ci, co, k, k, (s_, s_), (p, p), (1, 1), relu=True), x, wt, pos,
                               bias=bias, mask_in=mask, dtype=O.FP8)
    kept = m_out.reshape(-1)[pos] != 0
    rms = float(np.sqrt(np.mean(want[kept] ** 2)))
    assert float(np.abs(got[pos] - want).max()) / rms <= TOL_FP8
    # the same instances with 8-bit output: the codes are the narrowing of the values above
    if co % 16 == 0 and mask_kind == "objects":
        desc8 = B.conv_desc(n, h, w, ci, co, (k, k), (s_, s_), (p, p), (1, 1), B.FP8, B.FP8, B.RELU)
        out8 = B.focused_conv2d(desc8, G.to_dev(x, synth.FP8), G.to_dev(wt, synth.FP8),
                                torch.from_numpy(bias).to(G.dev()), mask_in=G.mask_dev(mask))
        expect = O.narrow_fp8(got.astype(np.float64))
        expect[got == 0] = 0
        np.testing.assert_array_equal(_codes(out8).reshape(-1, co), expect)


def test_fp8_layers_the_matrix_path_cannot_take_are_refused():
    torch = G.torch_mod()
    a = torch.zeros((1 << 16,), dtype=torch.uint8, device=G.dev())
    o = torch.zeros((1 << 16,), dtype=torch.uint8, device=G.dev())
    for ci, co, k in ((24, 64, 3), (3, 64, 7), (64, 20, 1), (16, 16, 7)):      # 16 | ci, 8 | co, <= 32 taps
        d = B.conv_desc(1, 8, 8, ci, co, (k, k), (1, 1), (k // 2, k // 2), (1, 1), B.FP8, B.F32)
        with pytest.raises(B.FcError) as e:
            B.focused_conv2d(d, a, a, None, out=o.view(torch.float32))
        assert e.value.status == -3
    d = B.conv_desc(1, 8, 8, 64, 64, in_dtype=B.FP8, out_dtype=B.F16)           # fp8 rounds to bf16, fp8 or fp32 only
    with pytest.raises(B.FcError):
        B.focused_conv2d(d, a, a, None, out=o.view(torch.float16))
    d = B.conv_desc(1, 8, 8, 64, 64, in_dtype=B.FP8, out_dtype=B.BF16)
    with pytest.raises(B.FcError):
        B.focused_dwconv2d(d, a, a, None, out=o.view(torch.bfloat16))


# ---- 8-bit outputs --------------------------------------------------------------------------

def _codes(t):
    return t.view(G.torch_mod().uint8).cpu().numpy()


def test_fp8_out_integer_sums_equal_the_oracle_codes():
    """Inputs 0..3 and weights -2..2 (exact E4M3 values), bias a multiple of 1/2: every partial sum
    is exact in fp32 in any order, so the codes must be the oracle's: integers between two E4M3
    values, exact midpoints (17, 34, 36, ...: ties to the even code) and sums past 448."""
    torch = G.torch_mod()
    n, h, w, ci, co = 2, 19, 22, 32, 48
    r = synth.rng(220, 1)
    xv = r.integers(0, 4, (n, h, w, ci)).astype(np.float32)
    wv = r.integers(-2, 3, (co, 3, 3, ci)).astype(np.float32)
    wv[:8] = np.abs(wv[:8])                                    # some channels run past 448
    bias = (r.integers(-40, 41, co) / 2.0).astype(np.float32)
    x8, w8 = synth.f32_to_fp8_bits(xv), synth.f32_to_fp8_bits(wv)
    mask = synth.mask_objects(n, h, w, 0.4, 220, 4)
    for relu in (False, True):
        desc = B.conv_desc(n, h, w, ci, co, (3, 3), (1, 1), (1, 1), (1, 1), B.FP8, B.FP8, B.RELU if relu else 0)
        out = B.focused_conv2d(desc, G.to_dev(x8, synth.FP8), G.to_dev(w8, synth.FP8),
                               torch.from_numpy(bias).to(G.dev()), mask_in=G.mask_dev(mask))
        torch.cuda.synchronize()
        shape = O.ConvShape(n, h, w, ci, co, 3, 3, (1, 1), (1, 1), (1, 1), relu=relu)
        y = O.focused_conv2d(shape, x8, w8, bias=bias, mask_in=mask, dtype=O.FP8)
        want = O.narrow_fp8(y)
        keep = mask != 0
        got = _codes(out)
        # ReLU of a negative sum is +0 here; the oracle's max(y, 0) agrees (no -0 from integers)
        np.testing.assert_array_equal(got[keep], want[keep])
        assert not got[~keep].any()                            # irrelevant rows: the code of +0.0
        if not relu:
            yk = y[keep]
            assert (np.abs(yk) > 448).mean() > 0.01 and (np.abs(yk) < 16).mean() > 0.05
            grid = O.widen(np.arange(0x7F, dtype=np.uint8), O.FP8)
            mids = (grid[:-1] + grid[1:]) / 2
            assert np.isin(np.abs(yk), mids).mean() > 0.02     # ties are among the cases


def test_fp8_out_stores_a_nan_code_for_a_nan_result():
    """One NaN byte in a kept pixel of x: every output whose window holds it is NaN in the oracle
    and one of the two NaN codes in the stored bytes; all other codes are the oracle's."""
    torch = G.torch_mod()
    n, h, w, ci, co = 1, 12, 12, 16, 16
    r = synth.rng(224, 1)
    x8 = synth.f32_to_fp8_bits(r.integers(0, 3, (n, h, w, ci)).astype(np.float32))
    w8 = synth.f32_to_fp8_bits(r.integers(-1, 2, (co, 3, 3, ci)).astype(np.float32))
    w8[w8 == 0x00] = 0x38                                      # no zero weights: the NaN reaches every channel
    x8[0, 5, 6, 3] = 0x7F
    mask = np.ones((n, h, w), np.uint8)
    mask[0, :2] = 0
    desc = B.conv_desc(n, h, w, ci, co, (3, 3), (1, 1), (1, 1), (1, 1), B.FP8, B.FP8, 0)
    out = B.focused_conv2d(desc, G.to_dev(x8, synth.FP8), G.to_dev(w8, synth.FP8), None, mask_in=G.mask_dev(mask))
    torch.cuda.synchronize()
    y = O.focused_conv2d(O.ConvShape(n, h, w, ci, co, 3, 3, (1, 1), (1, 1), (1, 1), relu=False), x8, w8,
                         bias=None, mask_in=mask, dtype=O.FP8)
    got = _codes(out)
    nan = np.isnan(y)
    assert nan.sum() == 9 * co
    assert ((got[nan] & 0x7F) == 0x7F).all()
    np.testing.assert_array_equal(got[~nan], O.narrow_fp8(y)[~nan])


@pytest.mark.parametrize("layer", [FP8_LAYERS[0], FP8_LAYERS[1], FP8_LAYERS[3], FP8_LAYERS[4], FP8_LAYERS[6],
                                   FP8_LAYERS[7], FP8_LAYERS[8], FP8_LAYERS[2], FP8_LAYERS[13]])
@pytest.mark.parametrize("relu", [True, False])
def test_fp8_out_is_the_narrowed_fp32_out_and_within_rounding_of_the_oracle(layer, relu):
    out32, want, keep = _run_layer(*layer, synth.FP8, seed=221, relu=relu)
    out8, _, _ = _run_layer(*layer, synth.FP8, seed=221, relu=relu, out_dtype=B.FP8)
    got = _codes(out8)
    f32 = out32.cpu().numpy()
    expect = O.narrow_fp8(f32.astype(np.float64))
    if relu:
        expect[f32 == 0] = 0            # the sign-bit rule stores +0 for -0
    np.testing.assert_array_equal(got[keep], expect[keep])
    assert not got[~keep].any()
    # end to end: v within (distance of y to the grid) + 2 tol of y
    grid = O.widen(np.arange(0x7F, dtype=np.uint8), O.FP8)
    grid = np.concatenate([-grid[:0:-1], grid])
    v = O.widen(got, O.FP8)
    rms = float(np.sqrt(np.mean(np.square(want[keep]))))
    yk, vk = want[keep], v[keep]
    j = np.searchsorted(grid, np.clip(yk, grid[0], grid[-1]))
    lo, hi = grid[np.maximum(j - 1, 0)], grid[np.minimum(j, grid.size - 1)]
    dist = np.minimum(np.abs(yk - lo), np.abs(hi - yk))
    assert (np.abs(vk - yk) <= dist + 2 * TOL_FP8 * rms).all()
    # and the codes mostly are the oracle's own (they differ only next to a rounding boundary)
    assert (got[keep] != O.narrow_fp8(want)[keep]).mean() < 0.01


def test_fp8_out_list_path_split_reduction_and_chain_of_two_layers():
    """The precomputed-list call (split reduction for this small layer) stores the same codes as
    the mask-only call; a second 8-bit layer fed the first one's bytes matches the oracle fed the
    same bytes."""
    torch = G.torch_mod()
    layer = FP8_LAYERS[7]
    a, _, keep = _run_layer(*layer, synth.FP8, seed=222, out_dtype=B.FP8)
    b, _, _ = _run_layer(*layer, synth.FP8, seed=222, out_dtype=B.FP8, precomputed=True)
    np.testing.assert_array_equal(_codes(a), _codes(b))
    n, h, w, ci, co = 2, 24, 20, 64, 64
    x = synth.activations((n, h, w, ci), synth.FP8, 223, 1)
    w1 = synth.he_weights(co, 3, 3, ci, synth.FP8, 223, 2)
    w2 = synth.he_weights(co, 1, 1, co, synth.FP8, 223, 3)
    mask = synth.mask_objects(n, h, w, 0.48, 223, 4)
    md = G.mask_dev(mask)
    d1 = B.conv_desc(n, h, w, ci, co, (3, 3), (1, 1), (1, 1), (1, 1), B.FP8, B.FP8, B.RELU)
    d2 = B.conv_desc(n, h, w, co, co, (1, 1), (1, 1), (0, 0), (1, 1), B.FP8, B.F32, 0)
    y1 = B.focused_conv2d(d1, G.to_dev(x, synth.FP8), G.to_dev(w1, synth.FP8), None, mask_in=md)
    y2 = B.focused_conv2d(d2, y1, G.to_dev(w2, synth.FP8), None, mask_in=md)
    torch.cuda.synchronize()
    s2 = O.ConvShape(n, h, w, co, co, 1, 1, (1, 1), (0, 0), (1, 1), relu=False)
    want = O.focused_conv2d(s2, _codes(y1), w2, bias=None, mask_in=mask, dtype=O.FP8)
    assert G.rel_err(G.to_f64(y2), want, mask != 0) <= TOL_FP8


@pytest.mark.parametrize("dtype", [synth.BF16, synth.F16])
@pytest.mark.parametrize("layer", [
    (1, 56, 56, 64, 64, 3, 1, 1, 1), (2, 20, 24, 64, 256, 1, 1, 0, 1), (1, 7, 9, 512, 512, 3, 1, 1, 1),
    (1, 64, 48, 3, 64, 7, 2, 3, 1),         # RGB stem
    (1, 40, 40, 3, 64, 3, 1, 1, 1),         # VGG first layer
    (1, 17, 13, 24, 48, 3, 1, 1, 1),
])
def test_fp8_out_from_16_bit_storage(layer, dtype):
    """16-bit activations and weights, 8-bit output (where an 8-bit chain starts): the codes are
    the oracle's narrowing of the kernel's own fp32 output, and within rounding of the oracle."""
    out32, want, keep = _run_layer(*layer, dtype, seed=225)
    out8, _, _ = _run_layer(*layer, dtype, seed=225, out_dtype=B.FP8)
    got = _codes(out8)
    f32 = out32.cpu().numpy()
    expect = O.narrow_fp8(f32.astype(np.float64))
    expect[f32 == 0] = 0
    np.testing.assert_array_equal(got[keep], expect[keep])
    assert not got[~keep].any()
    assert (got[keep] != O.narrow_fp8(want)[keep]).mean() < 0.01
    v = O.widen(got, O.FP8)
    rms = float(np.sqrt(np.mean(np.square(want[keep]))))
    # half the spacing of E4M3 values (2^-4 relative, 2^-10 absolute below 2^-6) + the fp32 tolerance
    assert (np.abs(v[keep] - want[keep]) <= np.maximum(np.abs(want[keep]) / 16, 2.0 ** -10) + 2e-4 * rms).all()


def test_fp8_out_refusals():
    torch = G.torch_mod()
    # 8-bit output needs a matrix-core layer (not fp32 storage, not odd channel counts) and whole 16-byte rows
    for in_dt, ci, co in ((B.F32, 64, 64), (B.FP8, 64, 40), (B.BF16, 64, 40), (B.BF16, 12, 64)):
        desc = B.conv_desc(1, 8, 8, ci, co, (3, 3), (1, 1), (1, 1), (1, 1), in_dt, B.FP8, 0)
        x = torch.zeros((1, 8, 8, ci), dtype=B.torch_dtype(in_dt), device=G.dev())
        w = torch.zeros((co, 3, 3, ci), dtype=B.torch_dtype(in_dt), device=G.dev())
        with pytest.raises(B.FcError) as e:
            B.focused_conv2d(desc, x, w, None)
        assert e.value.status == -3
