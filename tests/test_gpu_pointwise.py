"""GPU parity of the pointwise (1x1, no padding) matrix-core kernel that keeps the layer's weights in
LDS: layers of more than 4096 positions whose channel counts are multiples of 8, against the CPU
oracle (the two layers of 256 input channels and at most 128 output channels in the list run on
the tiled kernel and are held to the same bars).  fp32 outputs within 1e-4 of the RMS of the kept outputs (fp32 accumulation of at
most 256 products of 16-bit values); 16-bit and 8-bit outputs are the one rounding of the kernel's
own fp32 output, bit for bit."""
import numpy as np
import pytest

from oracle import fc_oracle as O
from paper_2207_10741_amd import binding as B, synth
from tests import gpu_util as G
from tests.test_gpu_packed_masks import bits_dev
from tests.test_gpu_parity import _run_layer, TOL_F32_OUT

pytestmark = pytest.mark.gpu

PW_LAYERS = [
    # n, h, w, ci, co, k, s, p, d
    (2, 60, 70, 64, 64, 1, 1, 0, 1),          # 8400 positions, ragged last unit of 32 rows
    (2, 50, 47, 64, 256, 1, 1, 0, 1),         # eight blocks of output channels, two groups of four
    (1, 80, 81, 256, 64, 1, 1, 0, 1),         # 256 input channels: the tiled kernel
    (2, 48, 50, 256, 128, 1, 1, 0, 1),
    (1, 70, 66, 128, 128, 1, 1, 0, 1),        # two chunks of input channels per unit
    (3, 41, 37, 128, 64, 1, 1, 0, 1),
    (2, 95, 97, 128, 128, 1, 2, 0, 1),        # strided projection: 4704 positions
    (1, 121, 83, 64, 256, 1, (2, 1), 0, 1),   # vertical stride only
    (1, 300, 310, 64, 64, 1, 1, 0, 1),        # 93000 positions: several units per wave
    (2, 50, 47, 128, 512, 1, 1, 0, 1),        # four slices of 128 output channels
    (1, 80, 81, 256, 1024, 1, 1, 0, 1),       # eight slices, four chunks of input channels
    (1, 70, 66, 64, 512, 1, 1, 0, 1),         # two slices of 256 output channels
    (2, 95, 97, 256, 192, 1, 2, 0, 1),        # three slices of 64: not a divisor of the workgroups per XCD
    (1, 71, 67, 256, 2048, 1, 1, 0, 1),       # sixteen slices
    (2, 50, 47, 512, 128, 1, 1, 0, 1),        # eight chunks of input channels, two slices of 64
    (1, 80, 81, 512, 2048, 1, 1, 0, 1),       # thirty-two slices: a whole XCD per group of rows
]

# channel counts off the chunk and slice sizes (MobileNetV2's expansions and projections among them)
PW_TAIL_LAYERS = [
    (2, 60, 70, 16, 96, 1, 1, 0, 1),          # a quarter of a chunk in, three blocks out
    (2, 60, 70, 24, 144, 1, 1, 0, 1),         # 48-byte rows in; a slice of eight blocks, 144 channels of it real
    (2, 60, 70, 144, 24, 1, 1, 0, 1),         # three chunks, the last a quarter full; 48-byte rows out
    (2, 50, 47, 32, 16, 1, 1, 0, 1),
    (1, 80, 81, 192, 64, 1, 1, 0, 1),
    (1, 80, 81, 384, 96, 1, 1, 0, 1),         # six chunks, two slices of 64, the second half full
    (1, 80, 81, 576, 160, 1, 1, 0, 1),        # nine chunks (72 KB of weights), three slices: two workgroups per XCD spare
    (1, 70, 66, 160, 960, 1, 1, 0, 1),        # eight slices of 128, the last half full
    (1, 70, 66, 320, 1280, 1, 1, 0, 1),       # ten slices: three groups per XCD
    (1, 71, 67, 8, 8, 1, 1, 0, 1),            # one piece in, one piece out
    (1, 71, 67, 72, 40, 1, 2, 0, 1),          # one piece in the second chunk; strided
    (1, 71, 67, 64, 384, 1, 1, 0, 1),         # two slices of 256, the second half full
]


def _check_f32(out, want, keep, zero_filled=True):
    got = G.to_f64(out)
    if keep.any():
        rms = float(np.sqrt(np.mean(np.square(want[keep]))))
        assert float(np.abs(got[keep] - want[keep]).max()) / rms <= TOL_F32_OUT
    if zero_filled:
        assert not out.cpu().numpy()[~keep].view(np.uint32).any()      # +0, bit for bit
    else:
        assert (got[~keep] == 7.0).all()


@pytest.mark.parametrize("layer", PW_LAYERS)
@pytest.mark.parametrize("mask_kind", ["objects", "bernoulli", "mixed", None])
def test_pointwise_layers_match_oracle(layer, mask_kind):
    out, want, keep = _run_layer(*layer, synth.BF16, mask_kind=mask_kind, seed=231)
    _check_f32(out, want, keep)


@pytest.mark.parametrize("layer", PW_TAIL_LAYERS)
@pytest.mark.parametrize("mask_kind", ["objects", "bernoulli", None])
def test_pointwise_channel_tails_match_oracle(layer, mask_kind):
    torch = G.torch_mod()
    out, want, keep = _run_layer(*layer, synth.BF16, mask_kind=mask_kind, seed=242)
    _check_f32(out, want, keep)
    # 16-bit output: the same sums rounded once, through the staged stores
    o16, _, _ = _run_layer(*layer, synth.BF16, mask_kind=mask_kind, seed=242, out_dtype=synth.BF16)
    assert torch.equal(o16, out.to(o16.dtype))
    # chained: irrelevant rows untouched, also past a short last slice
    oc, _, _ = _run_layer(*layer, synth.BF16, mask_kind=mask_kind, seed=242, out_dtype=synth.BF16,
                          flags_extra=B.SKIP_ZERO_FILL, precomputed=True)
    k = torch.from_numpy(keep).to(G.dev())
    assert torch.equal(oc[k], o16[k]) and bool((oc[~k] == 7.0).all())


@pytest.mark.parametrize("layer", [PW_TAIL_LAYERS[0], PW_TAIL_LAYERS[4], PW_TAIL_LAYERS[6], PW_TAIL_LAYERS[7]])
def test_pointwise_channel_tails_f16_and_fp8_output(layer):
    torch = G.torch_mod()
    o32, want, keep = _run_layer(*layer, synth.F16, seed=243)
    _check_f32(o32, want, keep)
    o8, _, _ = _run_layer(*layer, synth.F16, seed=243, out_dtype=B.FP8)
    got = o8.view(torch.uint8).cpu().numpy()
    f32 = o32.cpu().numpy()
    expect = O.narrow_fp8(f32.astype(np.float64))
    expect[f32 == 0] = 0
    np.testing.assert_array_equal(got[keep], expect[keep])
    assert not got[~keep].any()


@pytest.mark.parametrize("layer", [PW_LAYERS[0], PW_LAYERS[1], PW_LAYERS[3], PW_LAYERS[6]])
@pytest.mark.parametrize("irr", [0.0, 1.0, 0.97])
def test_pointwise_extreme_densities(layer, irr):
    out, want, keep = _run_layer(*layer, synth.BF16, irr=irr, seed=232)
    _check_f32(out, want, keep)


@pytest.mark.parametrize("layer", [PW_LAYERS[0], PW_LAYERS[2], PW_LAYERS[4], PW_LAYERS[7]])
def test_pointwise_f16_no_bias_no_relu_precomputed_list(layer):
    out, want, keep = _run_layer(*layer, synth.F16, relu=False, use_bias=False, precomputed=True, seed=233)
    _check_f32(out, want, keep)
    again, _, _ = _run_layer(*layer, synth.F16, relu=False, use_bias=False, seed=233)
    torch = G.torch_mod()
    assert torch.equal(out, again)                      # the list built inside the call gives the same rows


@pytest.mark.parametrize("layer", [PW_LAYERS[0], PW_LAYERS[1], PW_LAYERS[3], PW_LAYERS[6]])
@pytest.mark.parametrize("mask_kind,irr", [("objects", 0.48), ("bernoulli", 0.5), ("objects", 1.0)])
def test_pointwise_chained_leaves_irrelevant_rows_untouched(layer, mask_kind, irr):
    out, want, keep = _run_layer(*layer, synth.BF16, mask_kind=mask_kind, irr=irr, seed=234,
                                 flags_extra=B.SKIP_ZERO_FILL, precomputed=True)
    _check_f32(out, want, keep, zero_filled=False)


@pytest.mark.parametrize("layer", PW_LAYERS[:7])
@pytest.mark.parametrize("dtype", [synth.BF16, synth.F16])
def test_pointwise_16bit_output_is_rne_of_fp32_output(layer, dtype):
    torch = G.torch_mod()
    o32, _, keep = _run_layer(*layer, dtype, seed=235)
    o16, _, _ = _run_layer(*layer, dtype, seed=235, out_dtype=dtype)
    assert torch.equal(o16, o32.to(o16.dtype))          # kept rows rounded once, the others +0
    assert not o16.cpu().view(torch.int16).numpy()[~keep].any()


@pytest.mark.parametrize("layer", [PW_LAYERS[0], PW_LAYERS[1], PW_LAYERS[3]])
def test_pointwise_fp8_output_is_the_narrowing_of_fp32_output(layer):
    torch = G.torch_mod()
    o32, want, keep = _run_layer(*layer, synth.BF16, seed=236)
    o8, _, _ = _run_layer(*layer, synth.BF16, seed=236, out_dtype=B.FP8)
    got = o8.view(torch.uint8).cpu().numpy()
    f32 = o32.cpu().numpy()
    expect = O.narrow_fp8(f32.astype(np.float64))
    expect[f32 == 0] = 0
    np.testing.assert_array_equal(got[keep], expect[keep])
    assert not got[~keep].any()


@pytest.mark.parametrize("with_list", [False, True])
@pytest.mark.parametrize("layer", [PW_LAYERS[0], PW_LAYERS[3], PW_LAYERS[6]])
def test_pointwise_with_packed_masks_equals_byte_masks(layer, with_list):
    torch = G.torch_mod()
    n, h, w, ci, co, k, s, p, d = layer
    dtype = synth.BF16
    x = synth.activations((n, h, w, ci), dtype, 237, 1)
    wt = synth.he_weights(co, k, k, ci, dtype, 237, 2)
    bias = synth.bias(co, 237, 3)
    mask = synth.mask_objects(n, h, w, 0.48, 237, 4)
    xd, wd, bd = G.to_dev(x, dtype), G.to_dev(wt, dtype), torch.from_numpy(bias).to(G.dev())
    md = G.mask_dev(mask)
    mbits = bits_dev(mask)
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
    _check_f32(outs[1], want, keep)


@pytest.mark.parametrize("irr", [0.48, 0.0, 0.97, 1.0])
@pytest.mark.parametrize("c_mid,c_out", [(64, 256), (128, 64), (128, 128), (24, 144), (144, 24), (320, 1280)])
def test_pointwise_on_compacted_activations(c_mid, c_out, irr):
    """A 1x1 layer that reads and writes compacted rows (rows in list order) gives, bit for bit, the
    rows the spatial layout holds at the list's entries; rows past the count stay untouched."""
    torch = G.torch_mod()
    n, h, w = 2, 61, 70
    dtype = synth.BF16
    x = synth.activations((n, h, w, c_mid), dtype, 238, 1)
    w1 = synth.he_weights(c_out, 1, 1, c_mid, dtype, 238, 2)
    b1 = synth.bias(c_out, 238, 3)
    mask = synth.mask_objects(n, h, w, irr, 238, 4)
    md = G.mask_dev(mask)
    idx, count = B.active_index_compact(md)
    cnt = int(count.item())
    lists = dict(mask_in=md, mask_out=md, idx=idx, count=count)
    xd, w1d, b1d = G.to_dev(x, dtype), G.to_dev(w1, dtype), torch.from_numpy(b1).to(G.dev())
    li = idx[:cnt].long()
    x_compact = torch.zeros((n * h * w, c_mid), dtype=xd.dtype, device=G.dev())
    x_compact[:cnt] = xd.reshape(-1, c_mid)[li]
    geom = ((1, 1), (1, 1), (0, 0), (1, 1))
    for out_dtype in (B.F32, dtype):
        d1 = B.conv_desc(n, h, w, c_mid, c_out, *geom, dtype, out_dtype, B.RELU)
        z_spatial = B.focused_conv2d(d1, xd, w1d, b1d, **lists)
        for flags in (B.COMPACT_OUT, B.COMPACT_IN | B.COMPACT_OUT):
            dc = B.conv_desc(n, h, w, c_mid, c_out, *geom, dtype, out_dtype, B.RELU | flags)
            z = torch.full((n * h * w, c_out), 7.0, dtype=B.torch_dtype(out_dtype), device=G.dev())
            B.focused_conv2d(dc, x_compact if flags & B.COMPACT_IN else xd, w1d, b1d, out=z, **lists)
            assert torch.equal(z[:cnt], z_spatial.reshape(-1, c_out)[li])
            assert bool((z[cnt:] == 7.0).all())
    want = O.focused_conv2d(O.ConvShape(n, h, w, c_mid, c_out, 1, 1, pad=(0, 0), relu=True), x, w1, bias=b1,
                            mask_in=mask, dtype=dtype)
    d32 = B.conv_desc(n, h, w, c_mid, c_out, *geom, dtype, B.F32, B.RELU)
    _check_f32(B.focused_conv2d(d32, xd, w1d, b1d, **lists), want, mask != 0)


def test_pointwise_two_runs_are_bit_identical_and_nan_does_not_leak():
    torch = G.torch_mod()
    n, h, w, ci, co = 2, 60, 70, 64, 256
    dtype = synth.BF16
    x = synth.activations((n, h, w, ci), dtype, 239, 1)
    wt = synth.he_weights(co, 1, 1, ci, dtype, 239, 2)
    mask = synth.mask_objects(n, h, w, 0.48, 239, 4)
    md = G.mask_dev(mask)
    xd, wd = G.to_dev(x, dtype), G.to_dev(wt, dtype)
    desc = B.conv_desc(n, h, w, ci, co, (1, 1), (1, 1), (0, 0), (1, 1), dtype, B.F32, 0)
    a = B.focused_conv2d(desc, xd, wd, None, mask_in=md)
    b = B.focused_conv2d(desc, xd, wd, None, mask_in=md)
    assert torch.equal(a, b)
    # NaN under every irrelevant pixel: no kept row reads it, every irrelevant row is +0
    xn = xd.clone()
    xn[~md.bool().reshape(n, h, w)] = float("nan")
    c = B.focused_conv2d(desc, xn, wd, None, mask_in=md)
    assert torch.equal(a, c)


@pytest.mark.parametrize("irr", [None, 0.1])
def test_pointwise_at_the_bench_size_with_a_streamed_output(irr):
    """64 -> 256 channels on 32 x 120 x 160 positions: more than 256 MB of 16-bit rows, which the
    kernel streams past the memory-side cache.  The fp32 output is checked against the oracle on a
    sample of positions; the 16-bit output must be its rounding everywhere."""
    torch = G.torch_mod()
    n, h, w, ci, co = 32, 120, 160, 64, 256
    dtype = synth.BF16
    x = synth.activations_large((n, h, w, ci), dtype, 240, 1)
    wt = synth.he_weights(co, 1, 1, ci, dtype, 240, 2)
    bias = synth.bias(co, 240, 3)
    mask = None if irr is None else synth.mask_objects(n, h, w, irr, 240, 4)
    g = synth.rng(240, 5)
    pos = np.unique(np.concatenate([g.integers(0, n * h * w, size=3000), [0, n * h * w - 1]])).astype(np.int64)
    shape = O.ConvShape(n, h, w, ci, co, 1, 1, (1, 1), (0, 0), (1, 1), relu=True)
    want = O.focused_conv2d_at(shape, x, wt, pos, bias=bias, mask_in=mask, dtype=dtype)
    keep_rows = np.ones(pos.size, bool) if mask is None else mask.reshape(-1)[pos] != 0
    xd, wd, bd = G.to_dev(x, dtype), G.to_dev(wt, dtype), torch.from_numpy(bias).to(G.dev())
    md = None if mask is None else G.mask_dev(mask)
    if md is not None:
        assert int(md.sum().item()) * co * 2 > (256 << 20)
    outs = {}
    for out_dtype in (B.F32, dtype):
        desc = B.conv_desc(n, h, w, ci, co, (1, 1), (1, 1), (0, 0), (1, 1), dtype, out_dtype, B.RELU)
        out = torch.full((n, h, w, co), 7.0, dtype=B.torch_dtype(out_dtype), device=G.dev())
        B.focused_conv2d(desc, xd, wd, bd, mask_in=md, out=out)
        outs[out_dtype] = out
    torch.cuda.synchronize()
    got = outs[B.F32].reshape(-1, co)[torch.from_numpy(pos).to(G.dev())].to(torch.float64).cpu().numpy()
    rms = float(np.sqrt(np.mean(want[keep_rows] ** 2)))
    assert float(np.abs(got - want).max()) / rms <= TOL_F32_OUT
    assert not got[~keep_rows].any()
    assert torch.equal(outs[dtype], outs[B.F32].to(outs[dtype].dtype))


def test_pointwise_many_launches_of_a_many_stage_layer_are_bit_identical():
    """512 -> 2048 channels on 6480 positions: 32 slices, eight chunk loads per unit, 37 000 waits for
    a load into LDS per launch.  Every launch must give the same bits (a load into a ring buffer that
    overtakes the last read of the chunk before shows up as one differing block in about one launch
    of ten), and the first one must match the oracle."""
    torch = G.torch_mod()
    n, h, w, ci, co = 1, 80, 81, 512, 2048
    dtype = synth.BF16
    x = synth.activations((n, h, w, ci), dtype, 241, 1)
    wt = synth.he_weights(co, 1, 1, ci, dtype, 241, 2)
    bias = synth.bias(co, 241, 3)
    mask = synth.mask_bernoulli(n, h, w, 0.3, 241, 4)
    xd, wd, bd, md = G.to_dev(x, dtype), G.to_dev(wt, dtype), torch.from_numpy(bias).to(G.dev()), G.mask_dev(mask)
    idx, count = B.active_index_compact(md)
    outs = {}
    for out_dtype in (B.F32, dtype):
        desc = B.conv_desc(n, h, w, ci, co, (1, 1), (1, 1), (0, 0), (1, 1), dtype, out_dtype, B.RELU)
        first = None
        for it in range(40):
            out = torch.full((n, h, w, co), 7.0, dtype=B.torch_dtype(out_dtype), device=G.dev())
            B.focused_conv2d(desc, xd, wd, bd, mask_in=md, mask_out=md, idx=idx, count=count, out=out)
            if first is None:
                first = out
            else:
                assert torch.equal(out, first), "launch %d differs from the first" % it
        outs[out_dtype] = first
    want = O.focused_conv2d(O.ConvShape(n, h, w, ci, co, 1, 1, pad=(0, 0), relu=True), x, wt, bias=bias, mask_in=mask,
                            dtype=dtype)
    _check_f32(outs[B.F32], want, mask != 0)
    assert torch.equal(outs[dtype], outs[B.F32].to(outs[dtype].dtype))


# ---- 8-bit (E4M3) storage: chunks of 128 channels, the 8-bit matrix instruction ----
PW_FP8_LAYERS = [
    (2, 60, 70, 128, 128, 1, 1, 0, 1),        # one chunk
    (2, 50, 47, 64, 256, 1, 1, 0, 1),         # half a chunk, a slice of eight blocks
    (1, 80, 81, 256, 1024, 1, 1, 0, 1),       # two chunks, eight slices
    (1, 80, 81, 512, 128, 1, 1, 0, 1),        # four chunks into one slice: the tiled kernel
    (1, 80, 81, 1024, 256, 1, 1, 0, 1),       # eight chunks, slices of 64
    (1, 70, 66, 144, 48, 1, 2, 0, 1),         # tails on both sides, strided
    (1, 300, 310, 64, 64, 1, 1, 0, 1),        # several units per wave
]


@pytest.mark.parametrize("layer", PW_FP8_LAYERS)
@pytest.mark.parametrize("mask_kind", ["objects", "bernoulli", None])
def test_pointwise_fp8_storage_matches_oracle(layer, mask_kind):
    from tests.test_gpu_fp8 import TOL_FP8
    torch = G.torch_mod()
    out, want, keep = _run_layer(*layer, synth.FP8, mask_kind=mask_kind, seed=244)
    got = G.to_f64(out)
    rms = float(np.sqrt(np.mean(np.square(want[keep]))))
    assert float(np.abs(got[keep] - want[keep]).max()) / rms <= TOL_FP8
    assert not out.cpu().numpy()[~keep].view(np.uint32).any()
    # bf16 output: the fp32 output rounded once; 8-bit output: its narrowing (+0 for -0 under ReLU)
    o16, _, _ = _run_layer(*layer, synth.FP8, mask_kind=mask_kind, seed=244, out_dtype=B.BF16)
    assert torch.equal(o16, out.to(torch.bfloat16))
    if layer[4] % 16 == 0:
        o8, _, _ = _run_layer(*layer, synth.FP8, mask_kind=mask_kind, seed=244, out_dtype=B.FP8)
        codes = o8.view(torch.uint8).cpu().numpy()
        f32 = out.cpu().numpy()
        expect = O.narrow_fp8(f32.astype(np.float64))
        expect[f32 == 0] = 0
        np.testing.assert_array_equal(codes[keep], expect[keep])
        assert not codes[~keep].any()
        # chained, list given: the same codes on kept rows, the canary elsewhere
        oc, _, _ = _run_layer(*layer, synth.FP8, mask_kind=mask_kind, seed=244, out_dtype=B.FP8,
                              flags_extra=B.SKIP_ZERO_FILL, precomputed=True)
        cc = oc.view(torch.uint8).cpu().numpy()
        np.testing.assert_array_equal(cc[keep], codes[keep])
        assert (cc[~keep] == 0x4E).all()


# ---- 3x3 layers whose pixels are one 128-byte chunk (64 channels of a 16-bit type, 128 of the
# 8-bit one): the same kernel, a chunk per tap, the weights of a 64-channel slice resident ----
# ---- 3x3 layers whose pixels are one 128-byte chunk, on the same kernel (nine chunks per row: the
# nine taps).  The library sends such layers there by measured size rules (tens of thousands of
# positions and more); the tests ask for the kernel with FC_RESIDENT_WEIGHTS so that sizes the
# oracle finishes in seconds reach it, and one test runs a size the rule itself sends there ----
RW = B.RESIDENT_WEIGHTS

PW_3X3_LAYERS = [
    # n, h, w, ci, co, k, s, p, d
    (2, 60, 70, 64, 64, 3, 1, 1, 1),
    (2, 50, 47, 64, 128, 3, 1, 1, 1),                 # two slices
    (2, 120, 121, 64, 64, 3, 2, 1, 1),                # stride 2
    (1, 90, 77, 64, 64, 3, 1, 2, 2),                  # dilation 2
    (2, 61, 67, 64, 40, 3, (2, 1), (3, 2), (2, 1)),   # wide padding, mixed stride and dilation, a short slice
    (1, 80, 83, 64, 64, 3, 1, 0, 1),                  # no padding
    (1, 300, 310, 64, 64, 3, 1, 1, 1),                # several units per wave
]


@pytest.mark.parametrize("layer", PW_3X3_LAYERS)
@pytest.mark.parametrize("mask_kind", ["objects", "bernoulli", "mixed", None])
def test_pointwise_kernel_on_3x3_layers_matches_oracle(layer, mask_kind):
    torch = G.torch_mod()
    out, want, keep = _run_layer(*layer, synth.BF16, mask_kind=mask_kind, seed=245, flags_extra=RW)
    _check_f32(out, want, keep)
    o16, _, _ = _run_layer(*layer, synth.BF16, mask_kind=mask_kind, seed=245, out_dtype=synth.BF16, flags_extra=RW)
    assert torch.equal(o16, out.to(o16.dtype))
    # chained, list given
    oc, _, _ = _run_layer(*layer, synth.BF16, mask_kind=mask_kind, seed=245, flags_extra=B.SKIP_ZERO_FILL | RW,
                          precomputed=True)
    _check_f32(oc, want, keep, zero_filled=False)


@pytest.mark.parametrize("layer", [PW_3X3_LAYERS[0], PW_3X3_LAYERS[2], PW_3X3_LAYERS[4]])
@pytest.mark.parametrize("irr", [0.0, 1.0, 0.97])
def test_pointwise_kernel_on_3x3_layers_extreme_densities_f16(layer, irr):
    out, want, keep = _run_layer(*layer, synth.F16, irr=irr, seed=246, flags_extra=RW)
    _check_f32(out, want, keep)


@pytest.mark.parametrize("layer", [(2, 60, 70, 128, 64, 3, 1, 1, 1), (2, 61, 67, 128, 128, 3, 2, 1, 1)])
@pytest.mark.parametrize("mask_kind", ["objects", "bernoulli", None])
def test_pointwise_kernel_on_3x3_layers_fp8_storage(layer, mask_kind):
    from tests.test_gpu_fp8 import TOL_FP8
    torch = G.torch_mod()
    out, want, keep = _run_layer(*layer, synth.FP8, mask_kind=mask_kind, seed=247, flags_extra=RW)
    got = G.to_f64(out)
    rms = float(np.sqrt(np.mean(np.square(want[keep]))))
    assert float(np.abs(got[keep] - want[keep]).max()) / rms <= TOL_FP8
    assert not out.cpu().numpy()[~keep].view(np.uint32).any()
    o8, _, _ = _run_layer(*layer, synth.FP8, mask_kind=mask_kind, seed=247, out_dtype=B.FP8, flags_extra=RW)
    codes = o8.view(torch.uint8).cpu().numpy()
    f32 = out.cpu().numpy()
    expect = O.narrow_fp8(f32.astype(np.float64))
    expect[f32 == 0] = 0
    np.testing.assert_array_equal(codes[keep], expect[keep])
    assert not codes[~keep].any()


def test_pointwise_kernel_on_3x3_layer_nan_under_irrelevant_pixels_and_packed_masks():
    """NaN under every irrelevant pixel must not reach a kept row (every tap is gated by the input
    mask), with byte masks and with bit masks alike."""
    torch = G.torch_mod()
    n, h, w, ci, co = 2, 60, 70, 64, 64
    dtype = synth.BF16
    x = synth.activations((n, h, w, ci), dtype, 248, 1)
    wt = synth.he_weights(co, 3, 3, ci, dtype, 248, 2)
    mask = synth.mask_objects(n, h, w, 0.48, 248, 4)
    md, mbits = G.mask_dev(mask), bits_dev(mask)
    xd, wd = G.to_dev(x, dtype), G.to_dev(wt, dtype)
    xn = xd.clone()
    xn[~md.bool().reshape(n, h, w)] = float("nan")
    outs = []
    for packed, xin in ((False, xd), (False, xn), (True, xn)):
        desc = B.conv_desc(n, h, w, ci, co, in_dtype=dtype, out_dtype=B.F32, flags=RW | (B.PACKED_MASKS if packed else 0))
        outs.append(B.focused_conv2d(desc, xin, wd, None, mask_in=mbits if packed else md))
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    want = O.focused_conv2d(O.ConvShape(n, h, w, ci, co, 3, 3, (1, 1), (1, 1), (1, 1), relu=False), x, wt, bias=None,
                            mask_in=mask, dtype=dtype)
    _check_f32(outs[0], want, mask != 0)


@pytest.mark.parametrize("n,h,w", [(1, 300, 310), (16, 128, 128)])
def test_3x3_layer_sent_to_the_resident_weights_kernel_by_the_size_rule_matches_the_flagged_run(n, h, w):
    """93 000 positions, and the benchmark's C64 layer at its batch (262 144 positions), without a
    mask and chained, are sizes the dispatch rule sends to the resident-weights kernel by itself:
    the same bits as with the flag, and within tolerance of the oracle on sampled positions."""
    torch = G.torch_mod()
    ci, co = 64, 64
    dtype = synth.BF16
    x = synth.activations((n, h, w, ci), dtype, 249, 1)
    wt = synth.he_weights(co, 3, 3, ci, dtype, 249, 2)
    bias = synth.bias(co, 249, 3)
    mask = synth.mask_objects(n, h, w, 0.48, 249, 4)
    xd, wd, bd, md = G.to_dev(x, dtype), G.to_dev(wt, dtype), torch.from_numpy(bias).to(G.dev()), G.mask_dev(mask)
    idx, count = B.active_index_compact(md)
    for masked in (False, True):
        outs = []
        for extra in (0, RW):
            desc = B.conv_desc(n, h, w, ci, co, (3, 3), (1, 1), (1, 1), (1, 1), dtype, B.F32,
                               B.RELU | extra | (B.SKIP_ZERO_FILL if masked else 0))
            out = torch.zeros((n, h, w, co), dtype=torch.float32, device=G.dev())
            kw = dict(mask_in=md, mask_out=md, idx=idx, count=count) if masked else {}
            B.focused_conv2d(desc, xd, wd, bd, out=out, **kw)
            outs.append(out)
        assert torch.equal(outs[0], outs[1])
        # sampled kept positions against the oracle's definition, one by one
        rng = np.random.default_rng(249)
        kept = np.flatnonzero(mask.reshape(-1)) if masked else np.arange(n * h * w)
        pos = np.sort(rng.choice(kept, size=2000, replace=False))
        shape = O.ConvShape(n, h, w, ci, co, 3, 3, (1, 1), (1, 1), (1, 1), relu=True)
        want = O.focused_conv2d_at(shape, x, wt, pos, bias=bias, mask_in=mask if masked else None, dtype=dtype)
        got = outs[0].reshape(-1, co)[torch.from_numpy(pos).to(G.dev())].cpu().numpy().astype(np.float64)
        rms = float(np.sqrt(np.mean(np.square(want))))
        assert float(np.abs(got - want).max()) / rms <= TOL_F32_OUT


def test_many_launches_of_a_3x3_layer_on_the_resident_weights_kernel_are_bit_identical():
    """One unit per wave at most (2 906 units of 32 rows on 2 048 waves): every wave is in its
    start-up, where the loads of the list entries, of the tap masks and of the first chunks
    follow one another most closely.  Forty launches each, masked and dense, fp32 and bf16
    outputs: every launch the same bits, the bf16 output the rounding of the fp32 one."""
    torch = G.torch_mod()
    n, h, w, ci, co = 1, 300, 310, 64, 64
    dtype = synth.BF16
    x = synth.activations((n, h, w, ci), dtype, 250, 1)
    wt = synth.he_weights(co, 3, 3, ci, dtype, 250, 2)
    mask = synth.mask_objects(n, h, w, 0.48, 250, 4)
    xd, wd, md = G.to_dev(x, dtype), G.to_dev(wt, dtype), G.mask_dev(mask)
    idx, count = B.active_index_compact(md)
    for masked in (True, False):
        kw = dict(mask_in=md, mask_out=md, idx=idx, count=count) if masked else {}
        firsts = {}
        for out_dtype in (B.F32, dtype):
            desc = B.conv_desc(n, h, w, ci, co, (3, 3), (1, 1), (1, 1), (1, 1), dtype, out_dtype, B.RELU | RW)
            for it in range(40):
                out = torch.full((n, h, w, co), 7.0, dtype=B.torch_dtype(out_dtype), device=G.dev())
                B.focused_conv2d(desc, xd, wd, None, out=out, **kw)
                if out_dtype not in firsts:
                    firsts[out_dtype] = out
                else:
                    assert torch.equal(out, firsts[out_dtype]), "launch %d differs from the first" % it
        assert torch.equal(firsts[dtype], firsts[B.F32].to(firsts[dtype].dtype))
