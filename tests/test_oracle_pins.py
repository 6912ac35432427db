"""Pins for the CPU oracle: what the paper prints and what mathematics fixes.

None of these tests touches the GPU library.  Each one is chosen so that a
plausible slip in oracle/focused_conv_oracle.c (a dropped term, a wrong sign or
index, a transposed operand, a wrong centre tap) fails it.
"""
import os

import numpy as np
import pytest

from oracle import fc_oracle as O
from paper_2207_10741_amd import synth, workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


# ---------------------------------------------------------------- Fig. 5 ----

def test_fig5_column_counts():
    """Fig. 5 caption: 4x6 input, 3x3 kernel, stride 1 -> 9x8 matrix; focused 9x6."""
    (row,) = _rows("fig5_im2col_counts.txt")
    n, h, w, c, kh, kw, s, p, k_rows, cols_dense, cols_focused = map(int, row)
    ho, wo = O.out_dim(h, kh, s, p), O.out_dim(w, kw, s, p)
    assert n * ho * wo == cols_dense          # fixes the "+1" in the output-size formula
    assert kh * kw * c == k_rows
    # any mask that marks the centres of two patches irrelevant must leave 6 columns
    centres = [(oh + 1, ow + 1) for oh in range(ho) for ow in range(wo)]
    for drop in ((0, 1), (3, 4), (0, 7), (5, 2)):
        mask = np.ones((n, h, w), np.uint8)
        for d in drop:
            mask[0][centres[d]] = 0
        m_out = O.mask_downsample(mask, kh, kw, (s, s), (p, p))
        idx, cnt = O.active_index_compact(m_out)
        assert cnt == cols_focused
        assert sorted(set(range(cols_dense)) - set(idx.tolist())) == sorted(drop)


@pytest.mark.parametrize("size,k,s,p,d,want", [
    (224, 7, 2, 3, 1, 112), (112, 3, 2, 1, 1, 56), (56, 3, 1, 1, 1, 56), (56, 1, 2, 0, 1, 28),
    (135, 2, 2, 0, 1, 67), (5, 3, 1, 0, 2, 1), (5, 3, 1, 2, 2, 5), (2, 3, 1, 0, 1, 0),
])
def test_out_dim_known_sizes(size, k, s, p, d, want):
    assert O.out_dim(size, k, s, p, d) == want


# ----------------------------------------------------- hand-computed cases ----

X33 = np.array([[1, 2, 3], [4, 5, 6], [7, 8, 9]], np.float32).reshape(1, 3, 3, 1)


def test_hand_sobel_valid():
    w = np.array([[1, 0, -1], [2, 0, -2], [1, 0, -1]], np.float32).reshape(1, 3, 3, 1)
    s = O.ConvShape(1, 3, 3, 1, 1, pad=(0, 0))
    assert O.focused_conv2d(s, X33, w).reshape(-1).tolist() == [-8.0]
    b = np.array([0.5], np.float32)
    assert O.focused_conv2d(s, X33, w, bias=b).reshape(-1).tolist() == [-7.5]
    s.relu = True
    assert O.focused_conv2d(s, X33, w, bias=b).reshape(-1).tolist() == [0.0]
    assert O.focused_conv2d(s, X33, -w, bias=b).reshape(-1).tolist() == [8.5]


def test_hand_box_filter_same_pad_and_mask():
    w = np.ones((1, 3, 3, 1), np.float32)
    s = O.ConvShape(1, 3, 3, 1, 1)
    dense = O.focused_conv2d(s, X33, w)[0, :, :, 0]
    assert dense.tolist() == [[12, 21, 16], [27, 45, 33], [24, 39, 28]]
    mask = np.ones((1, 3, 3), np.uint8)
    mask[0, 0, 0] = 0   # value 1
    mask[0, 1, 1] = 0   # value 5
    foc = O.focused_conv2d(s, X33, w, mask_in=mask)[0, :, :, 0]
    assert foc.tolist() == [[0, 15, 11], [21, 0, 28], [19, 34, 23]]


def test_hand_two_channels_stride2_even_kernel():
    x = np.zeros((1, 4, 4, 2), np.float32)
    x[0, :, :, 0] = np.arange(16).reshape(4, 4)
    x[0, :, :, 1] = 1
    w = np.zeros((2, 2, 2, 2), np.float32)
    w[0, :, :, 0] = 1
    w[1, :, :, 1] = [[1, 2], [3, 4]]
    s = O.ConvShape(1, 4, 4, 2, 2, kh=2, kw=2, stride=(2, 2), pad=(0, 0))
    out = O.focused_conv2d(s, x, w)
    assert out[0, :, :, 0].tolist() == [[10, 18], [42, 50]]
    assert out[0, :, :, 1].tolist() == [[10, 10], [10, 10]]
    # even kernel: the centre tap is the window's top-left pixel (2oh, 2ow)
    mask = np.ones((1, 4, 4), np.uint8)
    mask[0, 2, 0] = 0
    out = O.focused_conv2d(s, x, w, mask_in=mask)
    assert out[0, :, :, 0].tolist() == [[10, 18], [0, 50]]
    mask[:] = 1
    mask[0, 3, 1] = 0    # inside window (1,0) but not its centre: value 13 drops out
    out = O.focused_conv2d(s, x, w, mask_in=mask)
    assert out[0, :, :, 0].tolist() == [[10, 18], [29, 50]]
    assert out[0, :, :, 1].tolist() == [[10, 10], [6, 10]]


def test_hand_dilation():
    x = np.arange(25, dtype=np.float32).reshape(1, 5, 5, 1)
    w = np.ones((1, 3, 3, 1), np.float32)
    s = O.ConvShape(1, 5, 5, 1, 1, pad=(0, 0), dil=(2, 2))
    assert O.focused_conv2d(s, x, w).reshape(-1).tolist() == [108.0]
    s = O.ConvShape(1, 5, 5, 1, 1, pad=(2, 2), dil=(2, 2))
    out = O.focused_conv2d(s, x, w)[0, :, :, 0]
    assert out.shape == (5, 5)
    assert out[0, 0] == 24.0 and out[2, 2] == 108.0 and out[4, 4] == 12 + 14 + 22 + 24


def test_hand_weight_orientation():
    """One-hot weight picks x at (oh+kh-1, ow+kw-1): correlation, not flipped; co/ci not swapped."""
    x = synth.small_integers((1, 5, 6, 3), -4, 4, synth.F32, 11)
    s = O.ConvShape(1, 5, 6, 3, 2)
    for (co, kh, kw, ci) in [(0, 0, 2, 1), (1, 2, 0, 2), (1, 1, 1, 0)]:
        w = np.zeros((2, 3, 3, 3), np.float32)
        w[co, kh, kw, ci] = 1
        out = O.focused_conv2d(s, x, w)
        xp = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)))
        np.testing.assert_array_equal(out[0, :, :, co], xp[0, kh:kh + 5, kw:kw + 6, ci])
        np.testing.assert_array_equal(out[0, :, :, 1 - co], 0)


# --------------------------- the paper's own construction, written separately ----

def _im2col_gemm(x, w, bias, stride, pad, dil, mask=None, relu=False):
    """Fig. 5a/5b: build the patch matrix, drop the irrelevant patches' columns,
    multiply by the flattened weights.  Written with slicing, in float64."""
    n, h, wd, c = x.shape
    co, kh, kw, _ = w.shape
    x = x.astype(np.float64)
    if mask is not None:
        x = x * (mask != 0)[..., None]
    xp = np.pad(x, ((0, 0), (pad[0], pad[0]), (pad[1], pad[1]), (0, 0)))
    ho = (h + 2 * pad[0] - dil[0] * (kh - 1) - 1) // stride[0] + 1
    wo = (wd + 2 * pad[1] - dil[1] * (kw - 1) - 1) // stride[1] + 1
    cols = np.empty((kh * kw * c, n * ho * wo))
    for i in range(kh):
        for j in range(kw):
            sl = xp[:, i * dil[0]: i * dil[0] + (ho - 1) * stride[0] + 1: stride[0],
                    j * dil[1]: j * dil[1] + (wo - 1) * stride[1] + 1: stride[1], :]
            cols[(i * kw + j) * c:(i * kw + j + 1) * c, :] = sl.reshape(n * ho * wo, c).T
    keep = np.ones(n * ho * wo, bool)
    if mask is not None:
        ch = np.clip(np.arange(ho) * stride[0] - pad[0] + dil[0] * ((kh - 1) // 2), 0, h - 1)
        cw = np.clip(np.arange(wo) * stride[1] - pad[1] + dil[1] * ((kw - 1) // 2), 0, wd - 1)
        keep = (mask[:, ch][:, :, cw] != 0).reshape(-1)
    wm = w.astype(np.float64).reshape(co, kh * kw * c)
    res = wm @ cols[:, keep]                      # fewer columns, same weights
    if bias is not None:
        res = res + bias.astype(np.float64)[:, None]
    if relu:
        res = np.maximum(res, 0)
    out = np.zeros((n * ho * wo, co))
    out[keep] = res.T
    return out.reshape(n, ho, wo, co), keep


CASES = [
    # n, h, w, ci, co, kh, kw, stride, pad, dil
    (1, 7, 9, 3, 4, 3, 3, (1, 1), (1, 1), (1, 1)),
    (2, 8, 8, 5, 6, 3, 3, (2, 2), (1, 1), (1, 1)),
    (2, 9, 7, 4, 3, 1, 1, (2, 2), (0, 0), (1, 1)),
    (1, 12, 10, 2, 5, 3, 3, (1, 1), (2, 2), (2, 2)),
    (1, 11, 13, 3, 2, 7, 7, (2, 2), (3, 3), (1, 1)),
    (2, 6, 9, 4, 4, 3, 1, (1, 2), (1, 0), (1, 1)),
    (1, 9, 9, 2, 3, 2, 2, (2, 2), (0, 0), (1, 1)),
    (1, 10, 9, 3, 3, 5, 3, (2, 1), (0, 2), (1, 2)),
]


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("masked", [False, True])
def test_matches_im2col_gemm(case, masked):
    n, h, w, ci, co, kh, kw, st, pd, dl = case
    x = synth.from_storage(synth.activations((n, h, w, ci), synth.F32, 1, h, w) - 0.3, synth.F32)
    wt = synth.he_weights(co, kh, kw, ci, synth.F32, 2, h, w)
    b = synth.bias(co, 3, h)
    mask = synth.mask_bernoulli(n, h, w, 0.4, 4, h, w) if masked else None
    s = O.ConvShape(n, h, w, ci, co, kh, kw, st, pd, dl, relu=masked)
    got = O.focused_conv2d(s, x, wt, bias=b, mask_in=mask)
    want, keep = _im2col_gemm(x, wt, b, st, pd, dl, mask, relu=masked)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    if masked:
        m_out = O.mask_downsample(mask, kh, kw, st, pd, dl)
        np.testing.assert_array_equal(m_out.reshape(-1) != 0, keep)
        idx, cnt = O.active_index_compact(m_out)
        np.testing.assert_array_equal(idx, np.flatnonzero(keep))
        assert cnt == keep.sum()


@pytest.mark.parametrize("case", CASES)
def test_dense_matches_library_convolution(case):
    """No mask -> the standard convolution (Sec. III-A): compare with torch's conv2d in float64."""
    torch = pytest.importorskip("torch")
    n, h, w, ci, co, kh, kw, st, pd, dl = case
    x = synth.from_storage(synth.activations((n, h, w, ci), synth.F32, 5, h, w) - 0.2, synth.F32)
    wt = synth.he_weights(co, kh, kw, ci, synth.F32, 6, h, w)
    b = synth.bias(co, 7, h)
    s = O.ConvShape(n, h, w, ci, co, kh, kw, st, pd, dl)
    got = O.focused_conv2d(s, x, wt, bias=b)
    ref = torch.nn.functional.conv2d(
        torch.from_numpy(x).double().permute(0, 3, 1, 2), torch.from_numpy(wt).double().permute(0, 3, 1, 2),
        torch.from_numpy(b).double(), stride=st, padding=pd, dilation=dl).permute(0, 2, 3, 1).numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_array_equal(got, O.focused_conv2d(s, x, wt, bias=b, mask_in=np.ones((n, h, w), np.uint8)))


# ------------------------------------------------------------- closed forms ----

def test_rectangle_counts_and_indices():
    """Sec. III-A: a kept rectangle of p % of the positions leaves p % of the columns."""
    n, h, w = 2, 24, 32
    r0, r1, c0, c1 = 4, 20, 8, 24
    mask = np.zeros((n, h, w), np.uint8)
    mask[1, r0:r1, c0:c1] = 1
    m1 = O.mask_downsample(mask, 3, 3, (1, 1), (1, 1))
    np.testing.assert_array_equal(m1, mask)
    idx, cnt = O.active_index_compact(m1)
    assert cnt == (r1 - r0) * (c1 - c0)
    want = [(1 * h + r) * w + c for r in range(r0, r1) for c in range(c0, c1)]
    assert idx.tolist() == want
    for (k, p) in ((3, 1), (1, 0), (7, 3)):
        m2 = O.mask_downsample(mask, k, k, (2, 2), (p, p))
        assert m2.shape == (n, h // 2, w // 2)
        assert O.active_index_compact(m2)[1] == (r1 - r0) * (c1 - c0) // 4
        np.testing.assert_array_equal(m2, mask[:, ::2, ::2])      # nearest-neighbour rescale
    m4 = O.mask_downsample(mask, 2, 2, (2, 2), (0, 0))
    np.testing.assert_array_equal(m4, mask[:, ::2, ::2])


def test_mask_values_normalised_and_clamped():
    mask = np.array([[[0, 7, 255], [3, 0, 1]]], np.uint8)
    np.testing.assert_array_equal(O.mask_downsample(mask, 1, 1, (1, 1), (0, 0)), [[[0, 1, 1], [1, 0, 1]]])
    # pad larger than the kernel's half-width: centre taps outside the image clamp to the border
    m = O.mask_downsample(mask, 1, 1, (1, 1), (1, 1))
    assert m.shape == (1, 4, 5)
    np.testing.assert_array_equal(m[0], [[0, 0, 1, 1, 1], [0, 0, 1, 1, 1], [1, 1, 0, 1, 1], [1, 1, 0, 1, 1]])


def test_all_ones_counts_taps():
    """x = 1, w = 1, no bias: a kept output equals C_in times the number of taps that
    are inside the image and relevant; counted here with shifted adds."""
    n, h, w, ci, co = 1, 9, 11, 4, 2
    mask = synth.mask_band_and_boxes(n, h, w, 0.45, 21)
    x = np.ones((n, h, w, ci), np.float32)
    wt = np.ones((co, 3, 3, ci), np.float32)
    got = O.focused_conv2d(O.ConvShape(n, h, w, ci, co), x, wt, mask_in=mask)
    mp = np.pad((mask != 0).astype(np.int64), ((0, 0), (1, 1), (1, 1)))
    taps = sum(mp[:, i:i + h, j:j + w] for i in range(3) for j in range(3))
    want = (taps * ci) * (mask != 0)
    for c in range(co):
        np.testing.assert_array_equal(got[..., c], want)


# --------------------------------------------------------------- invariants ----

def _setup(seed, n=2, h=13, w=15, ci=6, co=5, dtype=synth.F32):
    x = synth.activations((n, h, w, ci), dtype, seed, 1)
    wt = synth.he_weights(co, 3, 3, ci, dtype, seed, 2)
    b = synth.bias(co, seed, 3)
    mask = synth.mask_objects(n, h, w, 0.48, seed, 4)
    return O.ConvShape(n, h, w, ci, co), x, wt, b, mask


def test_all_irrelevant_is_all_zero_bytes():
    s, x, wt, b, mask = _setup(31)
    out = O.focused_conv2d(s, x, wt, bias=b, mask_in=np.zeros_like(mask))
    assert not out.view(np.uint8).any()           # +0.0, not -0.0, not bias
    assert O.active_index_compact(np.zeros_like(mask))[1] == 0


def test_irrelevant_inputs_do_not_matter_even_nan():
    s, x, wt, b, mask = _setup(32)
    base = O.focused_conv2d(s, x, wt, bias=b, mask_in=mask)
    for poison in (1e6, np.nan, np.inf):
        xp = x.copy()
        xp[mask == 0] = poison
        np.testing.assert_array_equal(O.focused_conv2d(s, xp, wt, bias=b, mask_in=mask), base)
    xz = x * (mask != 0)[..., None]
    np.testing.assert_array_equal(O.focused_conv2d(s, xz.astype(np.float32), wt, bias=b, mask_in=mask), base)
    dense_of_masked = O.focused_conv2d(s, xz.astype(np.float32), wt, bias=b)
    keep = mask != 0
    np.testing.assert_array_equal(base[keep], dense_of_masked[keep])
    assert not base[~keep].any()
    assert np.abs(dense_of_masked[~keep]).max() > 0       # the dense layer does compute there


def test_linearity_without_relu():
    s, _, _, b, mask = _setup(33)
    # small integers, so that the combined operands are exact in float32
    x = synth.small_integers((s.n, s.h, s.w, s.c_in), -8, 8, synth.F32, 33, 8)
    x2 = synth.small_integers(x.shape, -8, 8, synth.F32, 33, 9)
    wt = synth.small_integers((s.c_out, 3, 3, s.c_in), -5, 5, synth.F32, 33, 10)
    w2 = synth.small_integers(wt.shape, -5, 5, synth.F32, 33, 11)
    f = lambda xx, ww: O.focused_conv2d(s, xx, ww, mask_in=mask)
    np.testing.assert_array_equal(f(2 * x + x2, wt), 2 * f(x, wt) + f(x2, wt))
    np.testing.assert_array_equal(f(x, wt - 3 * w2), f(x, wt) - 3 * f(x, w2))
    assert np.abs(f(x, wt)).max() > 10
    # bias enters once per kept position and never at irrelevant ones
    with_b = O.focused_conv2d(s, x, wt, bias=b, mask_in=mask)
    np.testing.assert_allclose(with_b - f(x, wt), (mask != 0)[..., None] * b.astype(np.float64), atol=1e-12)


def test_translation_by_stride_multiple():
    n, h, w, ci, co = 1, 20, 22, 3, 4
    x = synth.from_storage(synth.activations((n, h, w, ci), synth.F32, 34, 1), synth.F32)
    wt = synth.he_weights(co, 3, 3, ci, synth.F32, 34, 2)
    mask = synth.mask_bernoulli(n, h, w, 0.3, 34, 3)
    s = O.ConvShape(n, h, w, ci, co, stride=(2, 2))
    a = O.focused_conv2d(s, x, wt, mask_in=mask)
    xs, ms = np.roll(x, (4, 2), axis=(1, 2)), np.roll(mask, (4, 2), axis=(1, 2))
    bb = O.focused_conv2d(s, xs, wt, mask_in=ms)
    np.testing.assert_array_equal(bb[:, 3:-1, 2:-1], a[:, 1:-3, 1:-2])


def test_sampled_positions_equal_whole_layer():
    s, x, wt, b, mask = _setup(35)
    s.relu = True
    s.stride = (2, 1)
    full = O.focused_conv2d(s, x, wt, bias=b, mask_in=mask)
    ho, wo = O.out_dims(s)
    pos = synth.rng(35, 7).permutation(s.n * ho * wo)[:60]
    np.testing.assert_array_equal(O.focused_conv2d_at(s, x, wt, pos, bias=b, mask_in=mask),
                                  full.reshape(-1, s.c_out)[pos])
    with pytest.raises(ValueError):
        O.focused_conv2d_at(s, x, wt, [s.n * ho * wo], bias=b, mask_in=mask)


@pytest.mark.parametrize("dtype", [synth.BF16, synth.F16])
def test_16bit_storage_is_widened_exactly(dtype):
    """The oracle fed raw 16-bit patterns equals the oracle fed the same values as float32;
    the float32 values come from numpy's own conversions."""
    s, x, wt, b, mask = _setup(36, dtype=dtype)
    got = O.focused_conv2d(s, x, wt, bias=b, mask_in=mask, dtype=dtype)
    ref = O.focused_conv2d(s, synth.from_storage(x, dtype), synth.from_storage(wt, dtype), bias=b, mask_in=mask)
    np.testing.assert_array_equal(got, ref)
    if dtype == synth.F16:   # subnormals, signed zero and the largest finite half
        bits = np.array([0x0001, 0x03FF, 0x8001, 0x0400, 0x7BFF, 0x8000, 0x3C00, 0xC000], np.uint16)
        xs = np.zeros((1, 1, 8, 1), np.uint16)
        xs[0, 0, :, 0] = bits
        one = np.array([0x3C00], np.uint16).reshape(1, 1, 1, 1)
        out = O.focused_conv2d(O.ConvShape(1, 1, 8, 1, 1, kh=1, kw=1, pad=(0, 0)), xs, one, dtype=dtype)
        np.testing.assert_array_equal(out.reshape(-1), bits.view(np.float16).astype(np.float64))


@pytest.mark.parametrize("case", [(2, 9, 11, 8, 12, 3, (1, 1), (1, 1), 4), (1, 10, 8, 6, 6, 3, (2, 2), (1, 1), 3),
                                  (2, 7, 9, 12, 4, 1, (1, 1), (0, 0), 2), (1, 8, 8, 4, 8, 5, (1, 1), (2, 2), 4)])
@pytest.mark.parametrize("masked", [False, True])
def test_grouped_layer_against_the_full_layer_a_library_and_its_limits(case, masked):
    """groups = 1 is the full layer; groups = C is the depthwise layer; any groups equals the full
    layer with block-diagonal weights (exactly: the extra terms are zeros) and, dense, torch's
    grouped conv2d in float64."""
    n, h, w, ci, co, k, st, pd, groups = case
    x = synth.from_storage(synth.activations((n, h, w, ci), synth.F32, 39, h, w) - 0.3, synth.F32)
    wt = synth.he_weights(co, k, k, ci // groups, synth.F32, 39, h, 2)
    b = synth.bias(co, 39, 3)
    mask = synth.mask_bernoulli(n, h, w, 0.4, 39, h, 4) if masked else None
    s = O.ConvShape(n, h, w, ci, co, k, k, st, pd, (1, 1), relu=masked)
    got = O.focused_gconv2d(s, groups, x, wt, bias=b, mask_in=mask)
    cig, cog = ci // groups, co // groups
    full = np.zeros((co, k, k, ci), np.float32)
    for g in range(groups):
        full[g * cog:(g + 1) * cog, :, :, g * cig:(g + 1) * cig] = wt[g * cog:(g + 1) * cog]
    np.testing.assert_allclose(got, O.focused_conv2d(s, x, full, bias=b, mask_in=mask), rtol=1e-13, atol=1e-13)
    np.testing.assert_array_equal(O.focused_gconv2d(s, 1, x, full, bias=b, mask_in=mask),
                                  O.focused_conv2d(s, x, full, bias=b, mask_in=mask))
    if not masked:
        torch = pytest.importorskip("torch")
        ref = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2),
                                         torch.from_numpy(wt.astype(np.float64)).permute(0, 3, 1, 2),
                                         torch.from_numpy(b.astype(np.float64)), stride=st, padding=pd, groups=groups)
        np.testing.assert_allclose(got, ref.permute(0, 2, 3, 1).numpy(), rtol=1e-11, atol=1e-11)
    if ci == co:
        wd = synth.he_weights(ci, k, k, 1, synth.F32, 39, 5)
        np.testing.assert_array_equal(O.focused_gconv2d(s, ci, x, wd, bias=b, mask_in=mask),
                                      O.focused_dwconv2d(s, x, np.ascontiguousarray(wd[..., 0]), bias=b, mask_in=mask))
    with pytest.raises(ValueError):
        O.focused_gconv2d(s, 5, x, wt, bias=b, mask_in=mask)


def test_tile_ordered_list_is_a_reordering_sorted_by_tile():
    """The tile-ordered list holds exactly the ascending list's positions, sorted by (image, tile
    row, tile column, row, column) - checked with numpy's lexsort, on ragged sizes - and a hand
    case."""
    hand = np.array([[[1, 0, 1, 1, 0],
                      [0, 1, 1, 0, 1],
                      [1, 1, 0, 0, 1]]], np.uint8)
    idx, cnt = O.active_index_compact_tiled(hand, 2, 2)
    # tiles of 2x2: (rows 0-1, cols 0-1): 0, 6; (cols 2-3): 2, 3, 7; (col 4): 9; (row 2, cols 0-1): 10, 11; (col 4): 14
    assert cnt == 9 and idx.tolist() == [0, 6, 2, 3, 7, 9, 10, 11, 14]
    for (n, h, w, th, tw) in ((2, 13, 37, 8, 16), (1, 16, 32, 8, 16), (3, 7, 5, 3, 4), (1, 1, 9, 8, 16), (2, 9, 16, 1, 16)):
        mask = synth.mask_bernoulli(n, h, w, 0.4, 37, h, w) * np.uint8(5)
        idx, cnt = O.active_index_compact_tiled(mask, th, tw)
        plain, pcnt = O.active_index_compact(mask.reshape(-1))
        assert cnt == pcnt and np.array_equal(np.sort(idx), plain[:pcnt])
        b, y, x = np.unravel_index(plain[:pcnt], (n, h, w))
        order = np.lexsort((x % tw, y % th, x // tw, y // th, b))      # last key is the primary one
        np.testing.assert_array_equal(idx, plain[:pcnt][order])
    # one tile as large as the image is the ascending order
    mask = synth.mask_objects(2, 11, 14, 0.5, 38)
    np.testing.assert_array_equal(O.active_index_compact_tiled(mask, 11, 14)[0], O.active_index_compact(mask.reshape(-1))[0][:int(np.count_nonzero(mask))])


def test_fp8_storage_decoder_and_encoder_against_the_format_and_a_library():
    """E4M3 bytes (OCP 8-bit floating point, the variant without infinities): the oracle's
    decoder against closed forms of the format and against torch's float8_e4m3fn for all 256
    codes; the input generator's encoder against torch's conversion; the layer fed bytes equals
    the layer fed the library-decoded values as float32."""
    codes = np.arange(256, dtype=np.uint8)
    vals = O.widen(codes, O.FP8)
    # closed forms: one, the largest finite value, the smallest subnormal and normal, signed zero
    assert vals[0x38] == 1.0 and vals[0x7E] == 448.0 and vals[0x01] == 2.0 ** -9 and vals[0x08] == 2.0 ** -6
    assert vals[0x00] == 0.0 and vals[0x80] == 0.0 and np.signbit(vals[0x80]) and not np.signbit(vals[0x00])
    assert np.isnan(vals[0x7F]) and np.isnan(vals[0xFF]) and np.isfinite(np.delete(vals, [0x7F, 0xFF])).all()
    np.testing.assert_array_equal(vals[0x81:0xFF], -vals[0x01:0x7F])
    assert (np.diff(vals[:0x7F]) > 0).all()                       # codes order like their values
    # spacing: 8 values per binade, the subnormals continue the first binade's step
    np.testing.assert_array_equal(np.diff(vals[0:16]), np.full(15, 2.0 ** -9))
    np.testing.assert_array_equal(vals[0x40:0x48], 2.0 * (1 + np.arange(8) / 8.0))
    torch = pytest.importorskip("torch")
    lib_vals = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    np.testing.assert_array_equal(vals, lib_vals)                 # NaN positions compare equal here
    np.testing.assert_array_equal(synth.fp8_bits_to_f32(codes).astype(np.float64), lib_vals)
    # the encoder: exact values round-trip, everything else goes where the library puts it
    np.testing.assert_array_equal(synth.f32_to_fp8_bits(lib_vals[:0x7F].astype(np.float32)), codes[:0x7F])
    a = synth.rng(36, 8).standard_normal(20000).astype(np.float32) * np.float32(3.0)
    a[:2000] *= np.float32(1e-2)                                  # into the subnormals
    a[2000:2100] = np.linspace(-440, 440, 100, dtype=np.float32)
    halfway = (lib_vals[1:0x7E] + lib_vals[2:0x7F]) / 2           # ties: to the even code
    a = np.concatenate([a, halfway.astype(np.float32), -halfway.astype(np.float32)])
    want = torch.from_numpy(a).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    np.testing.assert_array_equal(synth.f32_to_fp8_bits(a), want)
    # the layer on bytes = the layer on the same values held as float32
    s, x, wt, b, mask = _setup(36, dtype=synth.FP8)
    assert x.dtype == np.uint8 and wt.dtype == np.uint8
    got = O.focused_conv2d(s, x, wt, bias=b, mask_in=mask, dtype=O.FP8)
    xf = torch.from_numpy(x).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    wf = torch.from_numpy(wt).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    np.testing.assert_array_equal(got, O.focused_conv2d(s, xf, wf, bias=b, mask_in=mask))
    assert np.count_nonzero(got) > got.size // 8


def test_fp8_output_narrowing_against_the_format_and_a_library():
    """The code an 8-bit output is stored as: every value of the format is its own code, a value
    between two neighbours goes to the nearer one (brute force over the table of all values), a
    midpoint to the even code, magnitudes past 448 stay at 448, NaN keeps its sign; in range it
    agrees with torch's float8_e4m3fn conversion."""
    codes = np.arange(256, dtype=np.uint8)
    vals = O.widen(codes, O.FP8)
    finite = np.delete(codes, [0x7F, 0xFF])
    np.testing.assert_array_equal(O.narrow_fp8(vals[finite]), finite)        # fixed points, -0 included
    np.testing.assert_array_equal(O.narrow_fp8(np.array([np.nan, -np.nan])) & 0x7F, [0x7F, 0x7F])
    np.testing.assert_array_equal(O.narrow_fp8(np.array([449.0, 464.0, 1e9, np.inf, -470.0, -np.inf])),
                                  [0x7E, 0x7E, 0x7E, 0x7E, 0xFE, 0xFE])
    pos = vals[:0x7F]                                                         # ascending, 0 .. 448
    mid = (pos[:-1] + pos[1:]) / 2
    even = np.where(codes[:0x7E] % 2 == 0, codes[:0x7E], codes[1:0x7F])
    np.testing.assert_array_equal(O.narrow_fp8(mid), even)                    # ties
    np.testing.assert_array_equal(O.narrow_fp8(-mid), even | 0x80)
    np.testing.assert_array_equal(O.narrow_fp8(np.nextafter(mid, 0)), codes[:0x7E])      # just below
    np.testing.assert_array_equal(O.narrow_fp8(np.nextafter(mid, np.inf)), codes[1:0x7F])  # just above
    # brute force: nearest table value for random magnitudes over all binades
    r = synth.rng(37, 1)
    a = np.concatenate([np.ldexp(r.uniform(0.5, 1.0, 40000), r.integers(-12, 10, 40000)),
                        r.uniform(0, 2.0 ** -6, 4000)])
    a = a[a < 448.0]
    near = np.abs(a[:, None] - pos[None, :]).argmin(axis=1)
    got = O.narrow_fp8(a)
    dist = np.abs(pos[got] - a)
    assert (dist <= np.abs(pos[near] - a)).all()
    np.testing.assert_array_equal(O.narrow_fp8(-a), got | 0x80)
    torch = pytest.importorskip("torch")
    a32 = a.astype(np.float32)
    want = torch.from_numpy(a32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    np.testing.assert_array_equal(O.narrow_fp8(a32.astype(np.float64)), want)


# ------------------------------------------- Table I: multiply-adds follow the kept share ----

def test_table1_ratio_is_kept_fraction():
    """Table I: focused / normal multiply-adds equals 1 - irrelevant share, for both networks."""
    for name, irr, ed_n, ed_f, sl_n, sl_f in _rows("table1_multiply_adds.txt"):
        keep = 1.0 - float(irr) / 100.0
        assert abs(float(ed_f) / float(ed_n) - keep) < 2e-3, name
        assert abs(float(sl_f) / float(sl_n) - keep) < 2e-3, name


def test_stack_multiply_adds_follow_kept_fraction():
    """Propagating the mask with the centre-tap rule keeps each layer's kept share, and so
    the whole stack's multiply-add ratio, at the image's kept share (what Table I shows)."""
    h = w = 224
    mask = synth.mask_objects(1, h, w, 0.48, 41)
    keep0 = 1.0 - synth.irrelevant_fraction(mask)
    masks = {-1: mask}
    dense = focused = 0
    for i, op in enumerate(workloads.resnet18()):
        m_in = masks[op.src]
        m_out = O.mask_downsample(m_in, op.k, op.k, (op.stride,) * 2, (op.pad,) * 2)
        masks[i] = m_out
        if op.kind != "conv":
            continue
        idx, cnt = O.active_index_compact(m_out)
        macs = op.k * op.k * op.c_in * op.c_out
        dense += m_out.size * macs
        focused += cnt * macs
        # coarse maps quantise the share (a 7x7 map moves in steps of 2 %)
        assert abs(cnt / m_out.size - keep0) < (0.04 if m_out.size >= 784 else 0.12), op.name
    assert masks[len(masks) - 2].shape == (1, 7, 7)
    assert abs(focused / dense - keep0) < 0.03


def test_window_rules_would_not_keep_the_share():
    """Why the centre tap: labelling a patch by ANY relevant pixel in its window grows the
    kept region layer after layer, by ALL pixels shrinks it; neither reproduces Table I's
    constant ratio.  (Rules written here with shifted ORs / ANDs, only to show the drift.)"""
    h = w = 224
    m = synth.mask_objects(1, h, w, 0.48, 41)[0] != 0
    keep0 = m.mean()
    any_m, all_m = m.copy(), m.copy()
    for _ in range(8):                       # eight 3x3 stride-1 layers
        pa = np.pad(any_m, 1)
        pl = np.pad(all_m, 1)
        any_m = np.any([pa[i:i + h, j:j + w] for i in range(3) for j in range(3)], axis=0)
        all_m = np.all([pl[i:i + h, j:j + w] for i in range(3) for j in range(3)], axis=0)
    centre = m[None].astype(np.uint8)
    for _ in range(8):
        centre = O.mask_downsample(centre, 3, 3, (1, 1), (1, 1))
    assert centre[0].mean() == keep0
    assert any_m.mean() - keep0 > 0.05 and keep0 - all_m.mean() > 0.05


# ---------------------------------------------------------- depthwise layer ----

DW_CASES = [
    # n, h, w, c, kh, kw, stride, pad, dil
    (1, 7, 9, 5, 3, 3, (1, 1), (1, 1), (1, 1)),
    (2, 8, 8, 6, 3, 3, (2, 2), (1, 1), (1, 1)),
    (1, 12, 10, 3, 5, 5, (1, 1), (2, 2), (1, 1)),
    (1, 11, 13, 4, 3, 3, (1, 2), (2, 0), (2, 1)),
    (2, 9, 7, 8, 5, 3, (2, 1), (0, 1), (1, 1)),
]


def _dw_inputs(case, seed):
    n, h, w, c, kh, kw, st, pd, dl = case
    x = synth.from_storage(synth.activations((n, h, w, c), synth.F32, seed, h, w) - 0.3, synth.F32)
    wt = synth.he_weights(c, kh, kw, 1, synth.F32, seed + 1, h, w)[..., 0]
    b = synth.bias(c, seed + 2, h)
    return O.ConvShape(n, h, w, c, c, kh, kw, st, pd, dl), x, np.ascontiguousarray(wt), b


def test_depthwise_hand_case():
    """3x3 image, two channels with different 2x2 filters, written out by hand."""
    x = np.zeros((1, 3, 3, 2), np.float32)
    x[0, :, :, 0] = [[1, 2, 3], [4, 5, 6], [7, 8, 9]]
    x[0, :, :, 1] = [[1, 0, -1], [2, 0, -2], [3, 0, -3]]
    w = np.zeros((2, 2, 2), np.float32)
    w[0] = [[1, 0], [0, -1]]          # x[r][c] - x[r+1][c+1]
    w[1] = [[0, 2], [1, 0]]           # 2 x[r][c+1] + x[r+1][c]
    s = O.ConvShape(1, 3, 3, 2, 2, 2, 2, (1, 1), (0, 0), (1, 1))
    got = O.focused_dwconv2d(s, x, w, bias=np.array([0.5, -1.0], np.float32))
    want0 = np.array([[1 - 5, 2 - 6], [4 - 8, 5 - 9]]) + 0.5
    want1 = np.array([[2 * 0 + 2, 2 * -1 + 0], [2 * 0 + 3, 2 * -2 + 0]]) - 1.0
    np.testing.assert_array_equal(got[0, :, :, 0], want0)
    np.testing.assert_array_equal(got[0, :, :, 1], want1)
    # centre tap of an even kernel is its top-left pixel: dropping pixel (1,1) drops output (1,1)
    # and removes that pixel from the three other windows that contain it
    m = np.ones((1, 3, 3), np.uint8)
    m[0, 1, 1] = 0
    gm = O.focused_dwconv2d(s, x, w, mask_in=m)
    assert not gm[0, 1, 1].any()
    np.testing.assert_array_equal(gm[0, 0, 0], [1 - 0, 2 * 0 + 2])
    np.testing.assert_array_equal(gm[0, 0, 1], [2 - 6, 2 * -1 + 0])
    np.testing.assert_array_equal(gm[0, 1, 0], [4 - 8, 2 * 0 + 3])


@pytest.mark.parametrize("case", DW_CASES)
@pytest.mark.parametrize("masked", [False, True])
def test_depthwise_is_the_full_layer_with_diagonal_weights(case, masked):
    """A depthwise layer is the ordinary layer whose weight is zero off the channel diagonal;
    the ordinary layer's oracle is pinned above by independent means."""
    s, x, wt, b = _dw_inputs(case, 41)
    mask = synth.mask_bernoulli(s.n, s.h, s.w, 0.4, 44, s.h, s.w) if masked else None
    full = np.zeros((s.c_out, s.kh, s.kw, s.c_in), np.float32)
    for k in range(s.c_out):
        full[k, :, :, k] = wt[k]
    s_relu = O.ConvShape(s.n, s.h, s.w, s.c_in, s.c_out, s.kh, s.kw, s.stride, s.pad, s.dil, relu=masked)
    got = O.focused_dwconv2d(s_relu, x, wt, bias=b, mask_in=mask)
    want = O.focused_conv2d(s_relu, x, full, bias=b, mask_in=mask)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("case", DW_CASES)
def test_depthwise_dense_matches_library_grouped_convolution(case):
    torch = pytest.importorskip("torch")
    s, x, wt, b = _dw_inputs(case, 51)
    got = O.focused_dwconv2d(s, x, wt, bias=b)
    ref = torch.nn.functional.conv2d(
        torch.from_numpy(x).double().permute(0, 3, 1, 2), torch.from_numpy(wt).double()[:, None],
        torch.from_numpy(b).double(), stride=s.stride, padding=s.pad, dilation=s.dil,
        groups=s.c_in).permute(0, 2, 3, 1).numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)


def test_depthwise_invariants_and_sampled_positions():
    s, x, wt, b = _dw_inputs((2, 14, 11, 6, 3, 3, (1, 1), (1, 1), (1, 1)), 61)
    mask = synth.mask_objects(s.n, s.h, s.w, 0.48, 61, 4)
    base = O.focused_dwconv2d(s, x, wt, bias=b, mask_in=mask)
    keep = mask != 0
    assert not base[~keep].view(np.uint8).any() and np.abs(base[keep]).max() > 0
    assert not O.focused_dwconv2d(s, x, wt, bias=b, mask_in=np.zeros_like(mask)).view(np.uint8).any()
    for poison in (1e6, np.nan):
        xp = x.copy()
        xp[~keep] = poison
        np.testing.assert_array_equal(O.focused_dwconv2d(s, xp, wt, bias=b, mask_in=mask), base)
    # channels do not mix: changing channel 2 of the input changes channel 2 of the output only
    x2 = x.copy()
    x2[..., 2] += 1.0
    d = O.focused_dwconv2d(s, x2, wt, bias=b, mask_in=mask) - base
    assert np.abs(d[..., 2]).max() > 0 and not np.delete(d, 2, axis=-1).any()
    pos = np.array([0, 5, 17, s.h * s.w, 2 * s.h * s.w - 1])
    np.testing.assert_array_equal(O.focused_dwconv2d_at(s, x, wt, pos, bias=b, mask_in=mask),
                                  base.reshape(-1, s.c_out)[pos])
    # 16-bit storage widens exactly
    xb = synth.activations((s.n, s.h, s.w, s.c_in), synth.BF16, 62, 1)
    wb = np.ascontiguousarray(synth.he_weights(s.c_out, s.kh, s.kw, 1, synth.BF16, 63, 2)[..., 0])
    np.testing.assert_array_equal(
        O.focused_dwconv2d(s, xb, wb, mask_in=mask, dtype=O.BF16),
        O.focused_dwconv2d(s, synth.from_storage(xb, synth.BF16), synth.from_storage(wb, synth.BF16), mask_in=mask))


# ----------------------------------------------------- window rules for labels ----

def _window_labels_by_shifts(mask, kh, kw, st, pd, dl, rule):
    """Independent formulation: pad with a marker, gather every tap as a strided view."""
    n, h, w = mask.shape
    ho = (h + 2 * pd[0] - dl[0] * (kh - 1) - 1) // st[0] + 1
    wo = (w + 2 * pd[1] - dl[1] * (kw - 1) - 1) // st[1] + 1
    rel = np.pad((mask != 0).astype(np.int8), ((0, 0), (pd[0], pd[0]), (pd[1], pd[1])), constant_values=-1)
    taps = np.stack([rel[:, i * dl[0]: i * dl[0] + (ho - 1) * st[0] + 1: st[0],
                         j * dl[1]: j * dl[1] + (wo - 1) * st[1] + 1: st[1]]
                     for i in range(kh) for j in range(kw)])
    inside = (taps >= 0).sum(0)
    relevant = (taps == 1).sum(0)
    return (relevant > 0) if rule == O.RULE_ANY else ((inside > 0) & (relevant == inside))


RULE_CASES = [
    # n, h, w, kh, kw, stride, pad, dil
    (2, 9, 11, 3, 3, (1, 1), (1, 1), (1, 1)),
    (1, 12, 10, 3, 3, (2, 2), (1, 1), (1, 1)),
    (1, 10, 13, 5, 3, (1, 2), (2, 0), (1, 2)),
    (2, 8, 8, 2, 2, (2, 2), (0, 0), (1, 1)),
    (1, 7, 7, 3, 3, (1, 1), (4, 4), (1, 1)),      # windows that lie wholly outside the image
    (1, 9, 9, 1, 1, (2, 2), (0, 0), (1, 1)),
]


@pytest.mark.parametrize("case", RULE_CASES)
@pytest.mark.parametrize("rule", [O.RULE_ANY, O.RULE_ALL])
def test_window_rule_labels_match_shifted_views(case, rule):
    n, h, w, kh, kw, st, pd, dl = case
    mask = synth.mask_bernoulli(n, h, w, 0.5, 71, h, w) * np.uint8(5)
    got = O.mask_downsample_rule(mask, kh, kw, st, pd, dl, rule)
    np.testing.assert_array_equal(got != 0, _window_labels_by_shifts(mask, kh, kw, st, pd, dl, rule))
    assert set(np.unique(got)) <= {0, 1}
    # rule 0 is the centre tap
    np.testing.assert_array_equal(O.mask_downsample_rule(mask, kh, kw, st, pd, dl, O.RULE_CENTRE),
                                  O.mask_downsample(mask, kh, kw, st, pd, dl))


def test_window_rules_against_library_morphology_and_closed_forms():
    """3x3 / stride 1 / pad 1: ANY is a binary dilation, ALL (inside the image) an erosion whose
    border treats outside pixels as relevant; a kept r x c rectangle away from the border becomes
    (r + 2) x (c + 2) and (r - 2) x (c - 2); ALL <= centre <= ANY."""
    ndi = pytest.importorskip("scipy.ndimage")
    mask = synth.mask_objects(2, 40, 37, 0.48, 72, 4)
    any_l = O.mask_downsample_rule(mask, 3, 3, (1, 1), (1, 1), (1, 1), O.RULE_ANY)
    all_l = O.mask_downsample_rule(mask, 3, 3, (1, 1), (1, 1), (1, 1), O.RULE_ALL)
    box = np.ones((3, 3), bool)
    for b in range(2):
        np.testing.assert_array_equal(any_l[b] != 0, ndi.binary_dilation(mask[b] != 0, structure=box))
        np.testing.assert_array_equal(all_l[b] != 0, ndi.binary_erosion(mask[b] != 0, structure=box, border_value=1))
    assert (all_l <= (mask != 0)).all() and ((mask != 0) <= any_l).all()
    rect = np.zeros((1, 20, 20), np.uint8)
    rect[0, 5:11, 4:13] = 1                                   # 6 x 9
    assert O.mask_downsample_rule(rect, 3, 3, (1, 1), (1, 1), (1, 1), O.RULE_ANY).sum() == 8 * 11
    assert O.mask_downsample_rule(rect, 3, 3, (1, 1), (1, 1), (1, 1), O.RULE_ALL).sum() == 4 * 7


def test_labelled_layer_is_the_layer_when_labels_are_the_centre_taps_and_follows_any_labels():
    n, h, w, ci, co = 2, 11, 13, 4, 5
    x = synth.from_storage(synth.activations((n, h, w, ci), synth.F32, 73, 1) - 0.3, synth.F32)
    wt = synth.he_weights(co, 3, 3, ci, synth.F32, 73, 2)
    b = synth.bias(co, 73, 3)
    mask = synth.mask_bernoulli(n, h, w, 0.5, 73, 4)
    s = O.ConvShape(n, h, w, ci, co, 3, 3, (2, 1), (1, 1), (1, 1), relu=True)
    centre = O.mask_downsample(mask, 3, 3, s.stride, s.pad, s.dil)
    np.testing.assert_array_equal(O.focused_conv2d_labelled(s, x, wt, centre, bias=b, mask_in=mask),
                                  O.focused_conv2d(s, x, wt, bias=b, mask_in=mask))
    # any-pixel labels: kept rows equal the dense layer of the masked input, the rest is zero
    lab = O.mask_downsample_rule(mask, 3, 3, s.stride, s.pad, s.dil, O.RULE_ANY)
    got = O.focused_conv2d_labelled(s, x, wt, lab, bias=b, mask_in=mask)
    xz = (x * (mask != 0)[..., None]).astype(np.float32)
    dense = O.focused_conv2d(s, xz, wt, bias=b)
    keep = lab != 0
    np.testing.assert_array_equal(got[keep], dense[keep])
    assert not got[~keep].view(np.uint8).any() and keep.sum() > (centre != 0).sum()
