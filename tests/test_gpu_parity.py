"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on
the same seeded inputs.  Bars: index and mask work bit-exact; features with fp32
output within 1e-4 of the oracle relative to the RMS of the kept outputs (any storage
type: products of stored values, fp32 accumulation); bf16/f16 output equal to the
round-to-nearest-even of the fp32 output, and within 2e-2 of RMS."""
import numpy as np
import pytest

from oracle import fc_oracle as O
from paper_2207_10741_amd import binding as B, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

TOL_F32_OUT = 1e-4
TOL_16BIT_OUT = 2e-2


# ------------------------------------------------------------------ masks ----

@pytest.mark.parametrize("n,h,w,k,s,p,d", [
    (1, 56, 56, 3, 1, 1, 1), (2, 57, 43, 3, 2, 1, 1), (3, 224, 224, 7, 2, 3, 1), (2, 135, 241, 2, 2, 0, 1),
    (1, 9, 300, 1, 2, 0, 1), (2, 33, 35, 3, 1, 2, 2), (1, 5, 5, 1, 1, 1, 1), (1, 1, 1, 1, 1, 0, 1),
])
def test_mask_downsample_bit_exact(n, h, w, k, s, p, d):
    mask = synth.mask_bernoulli(n, h, w, 0.45, 101, h, w) * np.uint8(3)      # nonzero, not just 1
    got = B.mask_downsample(G.mask_dev(mask), (k, k), (s, s), (p, p), (d, d)).cpu().numpy()
    want = O.mask_downsample(mask, k, k, (s, s), (p, p), (d, d))
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("n,h,w,k,s,p,d", [
    (2, 57, 43, 3, 1, 1, 1), (1, 56, 56, 3, 2, 1, 1), (2, 33, 35, (5, 3), (1, 2), (2, 0), (1, 2)),
    (1, 135, 241, 2, 2, 0, 1), (1, 7, 7, 3, 1, 4, 1), (1, 9, 300, 1, 2, 0, 1), (3, 224, 224, 7, 2, 3, 1),
])
@pytest.mark.parametrize("rule", [B.RULE_CENTRE, B.RULE_ANY, B.RULE_ALL])
def test_window_rule_labels_bit_exact(n, h, w, k, s, p, d, rule):
    pair = lambda v: tuple(v) if isinstance(v, (tuple, list)) else (v, v)
    k, s, p, d = pair(k), pair(s), pair(p), pair(d)
    mask = synth.mask_bernoulli(n, h, w, 0.5, 103, h, w) * np.uint8(7)
    got = B.mask_downsample_rule(G.mask_dev(mask), k, s, p, d, rule).cpu().numpy()
    np.testing.assert_array_equal(got, O.mask_downsample_rule(mask, k[0], k[1], s, p, d, rule))


@pytest.mark.parametrize("rule", [B.RULE_ANY, B.RULE_ALL])
@pytest.mark.parametrize("layer", [(2, 40, 56, 64, 128, 3, 1, 1, 1), (1, 19, 23, 64, 128, 3, 2, 1, 1),
                                   (2, 30, 41, 24, 40, 3, 1, 1, 1)])
def test_layer_with_window_rule_labels_matches_oracle(layer, rule):
    """Labels from the any-pixel / all-pixels rule, compacted and handed to the layer."""
    torch = G.torch_mod()
    n, h, w, ci, co, k, s, p, d = layer
    dtype = synth.BF16
    x = synth.activations((n, h, w, ci), dtype, 104, 1)
    wt = synth.he_weights(co, k, k, ci, dtype, 104, 2)
    bias = synth.bias(co, 104, 3)
    mask = synth.mask_objects(n, h, w, 0.48, 104, 4)
    md = G.mask_dev(mask)
    labels = B.mask_downsample_rule(md, (k, k), (s, s), (p, p), (d, d), rule)
    idx, count = B.active_index_compact(labels)
    desc = B.conv_desc(n, h, w, ci, co, (k, k), (s, s), (p, p), (d, d), dtype, B.F32, B.RELU)
    ho, wo = B.out_dims(desc)
    out = torch.full((n, ho, wo, co), 7.0, dtype=torch.float32, device=G.dev())
    B.focused_conv2d(desc, G.to_dev(x, dtype), G.to_dev(wt, dtype), torch.from_numpy(bias).to(G.dev()), mask_in=md,
                     mask_out=labels, idx=idx, count=count, out=out)
    torch.cuda.synchronize()
    want_labels = O.mask_downsample_rule(mask, k, k, (s, s), (p, p), (d, d), rule)
    np.testing.assert_array_equal(labels.cpu().numpy(), want_labels)
    want = O.focused_conv2d_labelled(O.ConvShape(n, h, w, ci, co, k, k, (s, s), (p, p), (d, d), relu=True), x, wt,
                                     want_labels, bias=bias, mask_in=mask, dtype=dtype)
    keep = want_labels != 0
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_F32_OUT
    assert not out.cpu().numpy()[~keep].view(np.uint32).any()


@pytest.mark.parametrize("rule", [B.RULE_ANY, B.RULE_ALL])
@pytest.mark.parametrize("layer", [(1, 40, 56, 64, 128, 3, 1, 1, 1),      # 2240 positions: a layer that could rank its own rows
                                   (4, 40, 56, 64, 128, 3, 1, 1, 1),      # 8960 positions
                                   (2, 30, 41, 24, 40, 3, 1, 1, 1)])      # off the matrix-core tile sizes
def test_layer_with_labels_but_no_list_follows_the_labels(layer, rule):
    """Labels handed over without a kept list: the call compacts exactly these labels, so the rows it
    computes and the rows it clears agree with them (not with the centre tap of the input mask)."""
    torch = G.torch_mod()
    n, h, w, ci, co, k, s, p, d = layer
    dtype = synth.BF16
    x = synth.activations((n, h, w, ci), dtype, 114, 1)
    wt = synth.he_weights(co, k, k, ci, dtype, 114, 2)
    bias = synth.bias(co, 114, 3)
    mask = synth.mask_objects(n, h, w, 0.48, 114, 4)
    md = G.mask_dev(mask)
    labels = B.mask_downsample_rule(md, (k, k), (s, s), (p, p), (d, d), rule)
    desc = B.conv_desc(n, h, w, ci, co, (k, k), (s, s), (p, p), (d, d), dtype, B.F32, B.RELU)
    ho, wo = B.out_dims(desc)
    out = torch.full((n, ho, wo, co), 7.0, dtype=torch.float32, device=G.dev())
    ws = torch.empty((B.workspace_bytes(desc),), dtype=torch.uint8, device=G.dev())
    B.focused_conv2d(desc, G.to_dev(x, dtype), G.to_dev(wt, dtype), torch.from_numpy(bias).to(G.dev()), mask_in=md,
                     mask_out=labels, out=out, workspace=ws)
    torch.cuda.synchronize()
    want_labels = O.mask_downsample_rule(mask, k, k, (s, s), (p, p), (d, d), rule)
    centre = O.mask_downsample(mask, k, k, (s, s), (p, p), (d, d))
    assert (want_labels != centre).any()                       # the two labellings really differ here
    want = O.focused_conv2d_labelled(O.ConvShape(n, h, w, ci, co, k, k, (s, s), (p, p), (d, d), relu=True), x, wt,
                                     want_labels, bias=bias, mask_in=mask, dtype=dtype)
    keep = want_labels != 0
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_F32_OUT
    assert not out.cpu().numpy()[~keep].view(np.uint32).any()


@pytest.mark.parametrize("margin", [1, 2, 4])
def test_context_margin_is_the_any_rule_with_a_wider_window(margin):
    """A mask grown by a margin of context pixels (every pixel within `margin` of a relevant
    one, Chebyshev distance) is the any-pixel rule over a (2*margin+1)^2 window at stride 1:
    bit-exact against the oracle and against a library dilation; a layer run with the grown
    mask as its input mask matches the oracle run with the same mask."""
    ndimage = pytest.importorskip("scipy.ndimage")
    torch = G.torch_mod()
    n, h, w, ci, co = 2, 45, 61, 32, 48
    mask = synth.mask_objects(n, h, w, 0.6, 105, margin)
    k = 2 * margin + 1
    grown = B.mask_downsample_rule(G.mask_dev(mask), (k, k), (1, 1), (margin, margin), (1, 1), B.RULE_ANY)
    got = grown.cpu().numpy()
    np.testing.assert_array_equal(got, O.mask_downsample_rule(mask, k, k, (1, 1), (margin, margin), (1, 1), O.RULE_ANY))
    lib = np.stack([ndimage.binary_dilation(m != 0, structure=np.ones((k, k), bool)) for m in mask])
    np.testing.assert_array_equal(got != 0, lib)
    assert got.sum() > np.count_nonzero(mask)
    dtype = synth.BF16
    x = synth.activations((n, h, w, ci), dtype, 105, 1)
    wt = synth.he_weights(co, 3, 3, ci, dtype, 105, 2)
    desc = B.conv_desc(n, h, w, ci, co, in_dtype=dtype, out_dtype=B.F32, flags=B.RELU)
    out = B.focused_conv2d(desc, G.to_dev(x, dtype), G.to_dev(wt, dtype), None, mask_in=grown)
    want = O.focused_conv2d(O.ConvShape(n, h, w, ci, co, relu=True), x, wt, mask_in=got, dtype=dtype)
    assert G.rel_err(G.to_f64(out), want, got != 0) <= TOL_F32_OUT


@pytest.mark.parametrize("m", [1, 15, 16, 17, 63, 64, 65, 4095, 4096, 4097, 8192, 12289, 100003, 1 << 20, 3000017])
@pytest.mark.parametrize("irr", [0.48, 0.0, 1.0, 0.97])
def test_active_index_compact_bit_exact(m, irr):
    mask = synth.mask_bernoulli(1, 1, m, irr, 102, m).reshape(-1) * np.uint8(255)
    idx, count = B.active_index_compact(G.mask_dev(mask))
    want_idx, want_cnt = O.active_index_compact(mask)
    cnt = int(count.cpu().item())
    assert cnt == want_cnt
    np.testing.assert_array_equal(idx[:cnt].cpu().numpy(), want_idx)


@pytest.mark.parametrize("n,h,w,th,tw", [(2, 13, 37, 8, 16), (1, 16, 32, 8, 16), (3, 7, 5, 3, 4), (1, 1, 9, 8, 16),
                                        (2, 9, 16, 1, 16), (16, 128, 128, 8, 16), (3, 120, 160, 8, 16), (2, 57, 83, 4, 32),
                                        (1, 300, 500, 16, 8), (2, 33, 64, 40, 16)])
@pytest.mark.parametrize("irr", [0.48, 0.0, 1.0])
def test_tile_ordered_list_bit_exact(n, h, w, th, tw, irr):
    mask = synth.mask_bernoulli(n, h, w, irr, 106, h, w) * np.uint8(9)
    idx, count = B.active_index_compact_tiled(G.mask_dev(mask), th, tw)
    want_idx, want_cnt = O.active_index_compact_tiled(mask, th, tw)
    assert int(count.cpu().item()) == want_cnt
    np.testing.assert_array_equal(idx[:want_cnt].cpu().numpy(), want_idx)


@pytest.mark.parametrize("layer", [(2, 40, 56, 64, 128, 3, 1, 1, 1), (1, 19, 23, 64, 128, 3, 2, 1, 1),
                                   (4, 64, 64, 128, 128, 3, 1, 1, 1), (2, 30, 41, 24, 40, 3, 1, 1, 1),
                                   (2, 20, 24, 64, 256, 1, 1, 0, 1)])
@pytest.mark.parametrize("mask_kind", ["objects", "bernoulli"])
def test_layer_with_tile_ordered_list_matches(layer, mask_kind):
    """The layer takes the kept positions in any order: with the tile-ordered list every output
    row gets the same terms; only the order of its fp32 sum can differ (a tile whose pixel line is
    too long for the shared-line loop goes tap by tap), so the result equals the ascending list's
    to fp32 rounding of the sum, and the oracle within the bar."""
    torch = G.torch_mod()
    n, h, w, ci, co, k, s, p, d = layer
    dtype = synth.BF16
    x = synth.activations((n, h, w, ci), dtype, 107, 1)
    wt = synth.he_weights(co, k, k, ci, dtype, 107, 2)
    bias = synth.bias(co, 107, 3)
    mask = (synth.mask_objects if mask_kind == "objects" else synth.mask_bernoulli)(n, h, w, 0.48, 107, 4)
    md = G.mask_dev(mask)
    m_out = B.mask_downsample(md, (k, k), (s, s), (p, p), (d, d))
    desc = B.conv_desc(n, h, w, ci, co, (k, k), (s, s), (p, p), (d, d), dtype, B.F32, B.RELU)
    ho, wo = B.out_dims(desc)
    outs = []
    for tiled in (False, True):
        idx, count = B.active_index_compact_tiled(m_out, 8, 16) if tiled else B.active_index_compact(m_out)
        out = torch.full((n, ho, wo, co), 7.0, dtype=torch.float32, device=G.dev())
        ws = torch.zeros((B.workspace_bytes(desc),), dtype=torch.uint8, device=G.dev())
        B.focused_conv2d(desc, G.to_dev(x, dtype), G.to_dev(wt, dtype), torch.from_numpy(bias).to(G.dev()), mask_in=md,
                         mask_out=m_out, idx=idx, count=count, out=out, workspace=ws)
        outs.append(out)
    torch.cuda.synchronize()
    want = O.focused_conv2d(O.ConvShape(n, h, w, ci, co, k, k, (s, s), (p, p), (d, d), relu=True), x, wt, bias=bias,
                            mask_in=mask, dtype=dtype)
    keep = O.mask_downsample(mask, k, k, (s, s), (p, p), (d, d)) != 0
    assert G.rel_err(G.to_f64(outs[1]), G.to_f64(outs[0]), keep) <= 1e-5
    assert G.rel_err(G.to_f64(outs[1]), want, keep) <= TOL_F32_OUT
    assert not outs[1].cpu().numpy()[~keep].view(np.uint32).any()


@pytest.mark.parametrize("dtype", [synth.BF16, synth.FP8])
@pytest.mark.parametrize("irr", [0.48, 0.0, 0.97])
def test_compacted_activations_through_a_bottleneck(dtype, irr):
    """1x1 -> 3x3 -> 1x1 with the activations between the last two layers, and the block's output,
    stored compacted (rows in list order): the 3x3 writes compact rows (FC_COMPACT_OUT), the second
    1x1 reads and writes them (FC_COMPACT_IN | FC_COMPACT_OUT).  Every compact row equals, bit for
    bit, the row the spatial layout holds at that list entry; rows past the count stay untouched;
    the oracle checks the values."""
    torch = G.torch_mod()
    n, h, w, c_mid, c_out = 2, 36, 44, 64, 256
    x = synth.activations((n, h, w, c_mid), dtype, 108, 1)
    w3 = synth.he_weights(c_mid, 3, 3, c_mid, dtype, 108, 2)
    w1 = synth.he_weights(c_out, 1, 1, c_mid, dtype, 108, 3)
    b3, b1 = synth.bias(c_mid, 108, 4), synth.bias(c_out, 108, 5)
    mask = synth.mask_objects(n, h, w, irr, 108, 6)
    md = G.mask_dev(mask)
    m_out = B.mask_downsample(md)
    idx, count = B.active_index_compact(m_out)
    cnt = int(count.item())
    act = B.BF16 if dtype == synth.FP8 else dtype            # 8-bit layers write bf16
    d3 = B.conv_desc(n, h, w, c_mid, c_mid, in_dtype=dtype, out_dtype=act, flags=B.RELU)
    d3c = B.conv_desc(n, h, w, c_mid, c_mid, in_dtype=dtype, out_dtype=act, flags=B.RELU | B.COMPACT_OUT)
    xd, w3d, b3d = G.to_dev(x, dtype), G.to_dev(w3, dtype), torch.from_numpy(b3).to(G.dev())
    lists = dict(mask_in=md, mask_out=m_out, idx=idx, count=count)
    y_spatial = B.focused_conv2d(d3, xd, w3d, b3d, **lists)
    y_compact = torch.full((n * h * w, c_mid), 7.0, dtype=B.torch_dtype(act), device=G.dev())
    B.focused_conv2d(d3c, xd, w3d, b3d, out=y_compact, **lists)
    li = idx[:cnt].long()
    assert torch.equal(y_compact[:cnt], y_spatial.reshape(-1, c_mid)[li])
    assert bool((y_compact[cnt:] == 7.0).all())
    if dtype == synth.FP8:
        return                                               # (the next layer would mix storage types)
    # second layer: compact in, compact out, against spatial in / spatial out
    w1d, b1d = G.to_dev(w1, dtype), torch.from_numpy(b1).to(G.dev())
    d1 = B.conv_desc(n, h, w, c_mid, c_out, (1, 1), (1, 1), (0, 0), (1, 1), dtype, B.F32, B.RELU)
    d1c = B.conv_desc(n, h, w, c_mid, c_out, (1, 1), (1, 1), (0, 0), (1, 1), dtype, B.F32,
                      B.RELU | B.COMPACT_IN | B.COMPACT_OUT)
    z_spatial = B.focused_conv2d(d1, y_spatial, w1d, b1d, **lists)
    z_compact = torch.full((n * h * w, c_out), 7.0, dtype=torch.float32, device=G.dev())
    B.focused_conv2d(d1c, y_compact, w1d, b1d, out=z_compact, **lists)
    assert torch.equal(z_compact[:cnt], z_spatial.reshape(-1, c_out)[li])
    assert bool((z_compact[cnt:] == 7.0).all())
    # and the oracle on the second layer, fed the GPU's own (spatial) input
    y_host = G.to_storage_np(y_spatial, dtype)
    want = O.focused_conv2d(O.ConvShape(n, h, w, c_mid, c_out, 1, 1, pad=(0, 0), relu=True), y_host, w1, bias=b1,
                            mask_in=mask, dtype=dtype)
    keep = mask != 0
    assert G.rel_err(G.to_f64(z_spatial), want, keep) <= TOL_F32_OUT
    if cnt:
        got = z_compact[:cnt].to(torch.float64).cpu().numpy()
        rms = float(np.sqrt(np.mean(want[keep] ** 2)))
        assert float(np.abs(got - want.reshape(-1, c_out)[idx[:cnt].cpu().numpy()]).max()) / rms <= TOL_F32_OUT


def test_compacted_activations_argument_checks():
    torch = G.torch_mod()
    a = torch.zeros((1 << 18,), dtype=torch.uint8, device=G.dev())
    o = torch.zeros((1 << 18,), dtype=torch.uint8, device=G.dev())
    i32 = torch.zeros((64,), dtype=torch.int32, device=G.dev())
    d = B.conv_desc(1, 8, 8, 64, 64, in_dtype=B.BF16, out_dtype=B.BF16, flags=B.COMPACT_OUT)
    with pytest.raises(B.FcError) as e:                       # no list
        B.focused_conv2d(d, a.view(torch.bfloat16), a.view(torch.bfloat16), None, mask_in=a, out=o.view(torch.bfloat16))
    assert e.value.status == -1
    d = B.conv_desc(1, 8, 8, 64, 64, in_dtype=B.BF16, out_dtype=B.BF16, flags=B.COMPACT_IN)   # 3x3 cannot read compact rows
    with pytest.raises(B.FcError) as e:
        B.focused_conv2d(d, a.view(torch.bfloat16), a.view(torch.bfloat16), None, mask_in=a, mask_out=a, idx=i32,
                         count=i32, out=o.view(torch.bfloat16))
    assert e.value.status == -2
    d = B.conv_desc(1, 8, 8, 5, 7, (1, 1), (1, 1), (0, 0), in_dtype=B.F32, flags=B.COMPACT_OUT)     # not a matrix-core layer
    with pytest.raises(B.FcError) as e:
        B.focused_conv2d(d, a.view(torch.float32), a.view(torch.float32), None, mask_in=a, mask_out=a, idx=i32,
                         count=i32, out=o.view(torch.float32))
    assert e.value.status == -3


def test_active_index_compact_blobs_large():
    mask = synth.mask_objects(3, 480, 640, [0.3, 0.5, 0.7], 103)
    idx, count = B.active_index_compact(G.mask_dev(mask))
    want_idx, want_cnt = O.active_index_compact(mask)
    assert int(count.cpu().item()) == want_cnt
    np.testing.assert_array_equal(idx[:want_cnt].cpu().numpy(), want_idx)


@pytest.mark.parametrize("n,h,w,steps", [
    (16, 128, 128, [((3, 3), (1, 1), (1, 1), (1, 1)), ((3, 3), (2, 2), (1, 1), (1, 1)),
                    ((3, 3), (2, 2), (1, 1), (1, 1)), ((3, 3), (2, 2), (1, 1), (1, 1))]),
    (3, 57, 83, [((7, 7), (2, 2), (3, 3), (1, 1)), ((3, 3), (2, 2), (1, 1), (1, 1)), ((1, 1), (2, 2), (0, 0), (1, 1)),
                 ((2, 2), (2, 2), (0, 0), (1, 1)), ((3, 3), (1, 1), (1, 1), (1, 1))]),
    (1, 224, 224, [((7, 7), (2, 2), (3, 3), (1, 1)), ((3, 3), (2, 2), (1, 1), (1, 1)), ((3, 3), (2, 2), (1, 1), (1, 1)),
                   ((3, 3), (2, 2), (1, 1), (1, 1)), ((3, 3), (2, 2), (1, 1), (1, 1))]),
    (2, 33, 47, [((3, 5), (1, 2), (0, 4), (2, 1))]),
    (2, 300, 500, [((3, 3), (1, 1), (1, 1), (1, 1)), ((5, 5), (3, 3), (0, 0), (1, 1))]),
    # many blocks of 4096 positions per level
    (8, 256, 256, [((3, 3), (1, 1), (1, 1), (1, 1)), ((3, 3), (2, 2), (1, 1), (1, 1))]),
])
@pytest.mark.parametrize("irr", [0.48, 0.0, 1.0])
def test_mask_pyramid_matches_the_chain_of_rescalings(n, h, w, steps, irr):
    """All levels' masks and lists from one launch pair equal, bit for bit, the oracle's
    level-by-level rescaling and compaction."""
    mask = synth.mask_objects(n, h, w, irr, 120, h) * np.uint8(3)        # any nonzero byte counts
    md = G.mask_dev(mask)
    pyr = B.PreparedPyramid(md, steps)
    for m_out, idx, count in pyr.levels:
        m_out.fill_(9)
        idx.fill_(-7)
        count.fill_(-1)
    levels = pyr()
    G.torch_mod().cuda.synchronize()
    cur = mask
    for (k, s_, p, d), (m_out, idx, count) in zip(steps, levels):
        cur = O.mask_downsample(cur, k[0], k[1], s_, p, d)
        np.testing.assert_array_equal(m_out.cpu().numpy(), cur)
        want_idx, want_count = O.active_index_compact(cur)
        assert int(count.item()) == want_count
        np.testing.assert_array_equal(idx.cpu().numpy()[:want_count], want_idx[:want_count])


# ------------------------------------------------------------- conv layers ----

def _run_layer(n, h, w, ci, co, k, s, p, d, dtype, *, irr=0.48, relu=True, use_bias=True, out_dtype=B.F32,
               mask_kind="objects", seed=200, flags_extra=0, precomputed=False):
    torch = G.torch_mod()
    x = synth.activations((n, h, w, ci), dtype, seed, 1)
    wt = synth.he_weights(co, k, k, ci, dtype, seed, 2)
    bias = synth.bias(co, seed, 3) if use_bias else None
    if mask_kind == "objects":
        mask = synth.mask_objects(n, h, w, irr, seed, 4)
    elif mask_kind == "bernoulli":
        mask = synth.mask_bernoulli(n, h, w, irr, seed, 4)
    elif mask_kind == "band":
        mask = synth.mask_band_and_boxes(n, h, w, irr, seed, 4)
    elif mask_kind == "mixed":
        # left part of every image row fragmented, right part solid, a few rows empty: tiles
        # with long runs of adjacent kept positions next to tiles with none
        mask = synth.mask_bernoulli(n, h, w, 0.5, seed, 4)
        mask[:, :, w // 3:] = 1
        mask[:, ::7, :] = 0
    else:
        mask = None
    flags = (B.RELU if relu else 0) | flags_extra
    pair = lambda v: tuple(v) if isinstance(v, (tuple, list)) else (v, v)
    s, p, d = pair(s), pair(p), pair(d)
    desc = B.conv_desc(n, h, w, ci, co, (k, k), s, p, d, dtype, out_dtype, flags)
    xd, wd = G.to_dev(x, dtype), G.to_dev(wt, dtype)
    bd = None if bias is None else torch.from_numpy(bias).to(G.dev())
    md = None if mask is None else G.mask_dev(mask)
    kw = {}
    if precomputed and mask is not None:
        m_out = B.mask_downsample(md, (k, k), s, p, d)
        idx, count = B.active_index_compact(m_out)
        # same workspace size as the internal path, so that small layers split their
        # reduction the same way (the result is then bit-identical by construction)
        ws = torch.empty((B.workspace_bytes(desc),), dtype=torch.uint8, device=G.dev())
        kw = dict(mask_out=m_out, idx=idx, count=count, workspace=ws)
    # the output buffer starts full of a canary, so a row nobody writes cannot pass as zero
    ho, wo = B.out_dims(desc)
    if out_dtype == B.FP8:       # the code of 7.0
        out = torch.full((n, ho, wo, co), 0x4E, dtype=torch.uint8, device=G.dev()).view(B.torch_dtype(out_dtype))
    else:
        out = torch.full((n, ho, wo, co), 7.0, dtype=B.torch_dtype(out_dtype), device=G.dev())
    B.focused_conv2d(desc, xd, wd, bd, mask_in=md, out=out, **kw)
    torch.cuda.synchronize()
    shape = O.ConvShape(n, h, w, ci, co, k, k, s, p, d, relu=relu)
    want = O.focused_conv2d(shape, x, wt, bias=bias, mask_in=mask, dtype=dtype)
    keep = (O.mask_downsample(mask, k, k, s, p, d) != 0) if mask is not None \
        else np.ones(want.shape[:3], bool)
    return out, want, keep


LAYERS = [
    # n, h, w, ci, co, k, s, p, d
    (1, 56, 56, 64, 64, 3, 1, 1, 1),        # the single-layer config
    (2, 30, 41, 64, 64, 3, 1, 1, 1),        # ragged spatial size
    (2, 28, 28, 128, 128, 3, 1, 1, 1),
    (1, 19, 23, 64, 128, 3, 2, 1, 1),       # stride-2 3x3
    (2, 20, 24, 64, 256, 1, 1, 0, 1),       # 1x1
    (1, 21, 21, 128, 256, 1, 2, 0, 1),      # 1x1 / 2 projection
    (1, 14, 14, 256, 256, 3, 1, 1, 1),
    (1, 7, 9, 512, 512, 3, 1, 1, 1),        # few rows, long K
    (1, 64, 48, 3, 64, 7, 2, 3, 1),         # RGB stem
    (1, 40, 40, 3, 64, 3, 1, 1, 1),         # VGG first layer
    (1, 24, 24, 32, 48, 3, 1, 2, 2),        # dilation
    (1, 17, 13, 24, 40, 3, 1, 1, 1),        # channel counts off the tile sizes
    (1, 12, 12, 5, 7, 3, 1, 1, 1),          # odd channel counts
]


@pytest.mark.parametrize("layer", LAYERS)
@pytest.mark.parametrize("dtype", [synth.BF16, synth.F16, synth.F32])
def test_layer_matches_oracle_fp32_out(layer, dtype):
    out, want, keep = _run_layer(*layer, dtype)
    got = G.to_f64(out)
    assert G.rel_err(got, want, keep) <= TOL_F32_OUT
    assert not out.cpu().numpy()[~keep].view(np.uint32).any()        # +0.0 bit pattern


@pytest.mark.parametrize("layer", LAYERS[:8])
@pytest.mark.parametrize("mask_kind", ["bernoulli", "band", None])
def test_layer_mask_structures(layer, mask_kind):
    out, want, keep = _run_layer(*layer, synth.BF16, mask_kind=mask_kind, irr=0.5, seed=201)
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_F32_OUT


@pytest.mark.parametrize("layer", [LAYERS[0], LAYERS[3], LAYERS[4], LAYERS[8]])
@pytest.mark.parametrize("irr", [0.0, 1.0, 0.9])
def test_layer_extreme_densities(layer, irr):
    out, want, keep = _run_layer(*layer, synth.BF16, irr=irr, seed=202)
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_F32_OUT
    if irr == 1.0:
        assert not out.cpu().numpy().view(np.uint32).any()


@pytest.mark.parametrize("layer", [LAYERS[1], LAYERS[3], LAYERS[5], LAYERS[9]])
def test_variants_no_bias_no_relu_precomputed_list(layer):
    a, want, keep = _run_layer(*layer, synth.BF16, relu=False, use_bias=False, seed=203)
    assert G.rel_err(G.to_f64(a), want, keep) <= TOL_F32_OUT
    assert (want < 0).any()
    b, _, _ = _run_layer(*layer, synth.BF16, relu=False, use_bias=False, seed=203, precomputed=True)
    assert G.torch_mod().equal(a, b)          # same kernels, same order: bit-identical


@pytest.mark.parametrize("layer", [LAYERS[0], LAYERS[2], LAYERS[4], LAYERS[8], LAYERS[11]])
@pytest.mark.parametrize("dtype", [synth.BF16, synth.F16])
def test_16bit_output_is_rne_of_fp32_output(layer, dtype):
    torch = G.torch_mod()
    o32, want, keep = _run_layer(*layer, dtype, seed=204)
    o16, _, _ = _run_layer(*layer, dtype, seed=204, out_dtype=dtype)
    assert torch.equal(o16, o32.to(o16.dtype))                      # one rounding, to nearest even
    err = G.rel_err(G.to_f64(o16), want, keep)
    if err > TOL_16BIT_OUT:
        # an outlier activation can exceed the RMS-relative bar through output rounding alone;
        # then every element must still be within one unit in the last place of the oracle
        ulp = np.abs(want) * (2.0 ** -8 if dtype == synth.BF16 else 2.0 ** -11)
        assert (np.abs(G.to_f64(o16) - want) <= ulp + 1e-30).all()
    assert not o16.view(torch.int16).cpu().numpy()[~keep].any()


# 3x3 layers that step one pixel at a time horizontally and are at least 32 wide: the three
# horizontal taps share one gathered pixel line per tile (runs of adjacent kept positions), and
# tiles whose line would be too long (fragmented masks) take the tap-by-tap loop
HALO_LAYERS = [
    # n, h, w, ci, co, k, s, p, d
    (2, 40, 56, 64, 128, 3, 1, 1, 1),               # 128 x 64 tiles
    (8, 96, 96, 64, 128, 3, 1, 1, 1),               # 128 x 128 tiles (576 of them)
    (1, 36, 64, 64, 64, 3, 1, 1, 1),                # narrow layer, reduction split over workgroups
    (1, 33, 47, 72, 136, 3, (2, 1), (0, 2), (2, 1)),  # vertical stride and dilation, wide padding, channel tails
    (3, 17, 32, 128, 72, 3, (1, 1), (1, 0), (1, 1)),  # no horizontal padding: the output is narrower
    (128, 16, 16, 64, 256, 3, 1, 1, 1),             # 16-pixel rows, 512 tiles of 128 x 128: short runs on the pixel line
    (2, 30, 70, 64, 128, 3, 1, (3, 2), (3, 1)),     # three padded rows and two padded pixels: first taps far outside
]


@pytest.mark.parametrize("layer", HALO_LAYERS)
@pytest.mark.parametrize("mask_kind", ["objects", "bernoulli", "mixed", None])
def test_shared_halo_layers_match_oracle(layer, mask_kind):
    out, want, keep = _run_layer(*layer, synth.BF16, mask_kind=mask_kind, irr=0.45, seed=207)
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_F32_OUT
    assert not out.cpu().numpy()[~keep].view(np.uint32).any()


@pytest.mark.parametrize("layer", [HALO_LAYERS[0], HALO_LAYERS[2], HALO_LAYERS[3]])
def test_shared_halo_precomputed_list_and_16bit_output(layer):
    torch = G.torch_mod()
    a, want, keep = _run_layer(*layer, synth.F16, mask_kind="mixed", seed=208)
    b, _, _ = _run_layer(*layer, synth.F16, mask_kind="mixed", seed=208, precomputed=True)
    assert torch.equal(a, b)
    c, _, _ = _run_layer(*layer, synth.F16, mask_kind="mixed", seed=208, out_dtype=synth.F16)
    assert torch.equal(c, a.to(c.dtype))
    assert G.rel_err(G.to_f64(a), want, keep) <= TOL_F32_OUT


# Chained 3x3 layers (irrelevant rows left unwritten) of 65 .. 128 output channels and up to 65536
# positions run on the one-workgroup-per-CU kernel: kept rows dealt out in 32-row blocks, one
# pixel line per tile, tap by tap where a tile's line would not fit or the geometry has none
CHAINED_LINE_LAYERS = [
    # n, h, w, ci, co, k, s, p, d
    (2, 40, 56, 64, 128, 3, 1, 1, 1),               # 4480 positions: a block or two per workgroup
    (8, 96, 64, 64, 128, 3, 1, 1, 1),               # 49152 positions: several blocks per workgroup
    (16, 64, 64, 128, 128, 3, 1, 1, 1),             # the bench shape: two channel chunks, eight blocks when dense
    (3, 47, 61, 72, 96, 3, 1, 1, 1),                # channel tails on both sides, ragged rows
    (2, 61, 47, 64, 128, 3, (2, 1), (0, 2), (2, 1)),  # vertical stride and dilation, wide padding
    (2, 63, 65, 64, 128, 3, 2, 1, 1),               # stride 2: no shared line, tap by tap
    (1, 70, 70, 64, 104, 3, 1, 1, 2),               # dilation 2: tap by tap
]


@pytest.mark.parametrize("layer", CHAINED_LINE_LAYERS)
@pytest.mark.parametrize("mask_kind,irr", [("objects", 0.48), ("bernoulli", 0.5), ("mixed", 0.5), ("objects", 0.95),
                                           ("objects", 0.0), ("objects", 1.0)])
def test_chained_layers_on_the_one_workgroup_per_cu_kernel(layer, mask_kind, irr):
    torch = G.torch_mod()
    out, want, keep = _run_layer(*layer, synth.BF16, mask_kind=mask_kind, irr=irr, seed=209,
                                 flags_extra=B.SKIP_ZERO_FILL, precomputed=True)
    got = G.to_f64(out)
    if keep.any():
        rms = float(np.sqrt(np.mean(np.square(want[keep]))))
        assert float(np.abs(got[keep] - want[keep]).max()) / rms <= TOL_F32_OUT
    assert (got[~keep] == 7.0).all()                    # irrelevant rows untouched
    # 16-bit outputs: the same sums, rounded once
    o16, _, _ = _run_layer(*layer, synth.BF16, mask_kind=mask_kind, irr=irr, seed=209, flags_extra=B.SKIP_ZERO_FILL,
                           precomputed=True, out_dtype=synth.BF16)
    k = torch.from_numpy(keep).to(G.dev())
    assert torch.equal(o16[k], out[k].to(o16.dtype))


# layers with at most 4 input channels run on the matrix cores through an element-wise gather
STEM_LAYERS = [
    # n, h, w, ci, co, k, s, p, d
    (2, 37, 53, 3, 64, 3, 1, 1, 1),
    (1, 64, 48, 3, 64, 7, 2, 3, 1),
    (1, 33, 29, 1, 72, 5, 1, 2, 1),             # one channel, 25 taps, a partial channel tile
    (2, 31, 40, 4, 16, 3, (2, 1), (2, 0), (2, 1)),
    (1, 300, 200, 3, 128, 3, 1, 1, 1),          # many tiles per workgroup, two channel tiles
]


@pytest.mark.parametrize("layer", STEM_LAYERS)
@pytest.mark.parametrize("mask_kind", ["objects", "bernoulli", None])
def test_stem_layers_match_oracle(layer, mask_kind):
    out, want, keep = _run_layer(*layer, synth.BF16, mask_kind=mask_kind, irr=0.45, seed=211)
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_F32_OUT
    assert not out.cpu().numpy()[~keep].view(np.uint32).any()


def test_stem_16bit_output_and_precomputed_list():
    torch = G.torch_mod()
    layer = STEM_LAYERS[0]
    a, want, keep = _run_layer(*layer, synth.F16, seed=212)
    b, _, _ = _run_layer(*layer, synth.F16, seed=212, precomputed=True)
    assert torch.equal(a, b)
    c, _, _ = _run_layer(*layer, synth.F16, seed=212, out_dtype=synth.F16)
    assert torch.equal(c, a.to(c.dtype))
    assert G.rel_err(G.to_f64(a), want, keep) <= TOL_F32_OUT


def test_dense_path_is_standard_convolution():
    out, want, keep = _run_layer(2, 21, 27, 64, 128, 3, 1, 1, 1, synth.BF16, mask_kind=None, seed=205)
    assert keep.all() and G.rel_err(G.to_f64(out), want, keep) <= TOL_F32_OUT


def test_nan_at_irrelevant_inputs_does_not_leak():
    torch = G.torch_mod()
    n, h, w, c = 1, 30, 30, 64
    x = synth.activations((n, h, w, c), synth.BF16, 206, 1)
    wt = synth.he_weights(c, 3, 3, c, synth.BF16, 206, 2)
    mask = synth.mask_objects(n, h, w, 0.48, 206, 4)
    desc = B.conv_desc(n, h, w, c, c, in_dtype=B.BF16, out_dtype=B.F32)
    md = G.mask_dev(mask)
    clean = B.focused_conv2d(desc, G.to_dev(x, synth.BF16), G.to_dev(wt, synth.BF16), mask_in=md)
    xp = x.copy()
    xp[mask == 0] = 0x7FC0            # bf16 quiet NaN
    dirty = B.focused_conv2d(desc, G.to_dev(xp, synth.BF16), G.to_dev(wt, synth.BF16), mask_in=md)
    assert torch.equal(clean, dirty)


def test_skip_zero_fill_leaves_irrelevant_rows_untouched_and_guard_bytes_intact():
    torch = G.torch_mod()
    n, h, w, ci, co = 2, 25, 31, 64, 64
    x = synth.activations((n, h, w, ci), synth.BF16, 207, 1)
    wt = synth.he_weights(co, 3, 3, ci, synth.BF16, 207, 2)
    mask = synth.mask_objects(n, h, w, 0.48, 207, 4)
    guard = 4096
    for flags in (B.SKIP_ZERO_FILL, 0):
        desc = B.conv_desc(n, h, w, ci, co, in_dtype=B.BF16, out_dtype=B.BF16, flags=flags)
        buf = torch.full((n * h * w * co + 2 * guard,), 7.0, dtype=torch.bfloat16, device=G.dev())
        out = buf[guard:guard + n * h * w * co].view(n, h, w, co)
        B.focused_conv2d(desc, G.to_dev(x, synth.BF16), G.to_dev(wt, synth.BF16), mask_in=G.mask_dev(mask), out=out)
        torch.cuda.synchronize()
        assert (buf[:guard] == 7.0).all() and (buf[-guard:] == 7.0).all()
        o = out.float().cpu().numpy()
        keep = mask != 0
        if flags:
            assert (o[~keep] == 7.0).all()
        else:
            assert not o[~keep].any()
        want = O.focused_conv2d(O.ConvShape(n, h, w, ci, co), x, wt, mask_in=mask, dtype=O.BF16)
        assert np.abs(o[keep] - want[keep]).max() <= TOL_16BIT_OUT * np.sqrt(np.mean(want[keep] ** 2))


def test_workspace_ready_flag_skips_the_clear_and_leaves_the_counters_zero():
    """A layer small enough to split its reduction: with the counters cleared once and
    FC_WORKSPACE_READY on every call, repeated calls (dense and masked, sharing the workspace)
    reproduce the result of the ordinary call bit for bit, and the counters read zero after."""
    torch = G.torch_mod()
    n, h, w, c = 1, 20, 24, 256
    x = G.to_dev(synth.activations((n, h, w, c), synth.BF16, 209, 1), synth.BF16)
    wt = G.to_dev(synth.he_weights(c, 3, 3, c, synth.BF16, 209, 2), synth.BF16)
    md = G.mask_dev(synth.mask_objects(n, h, w, 0.4, 209, 4))
    m_out = B.mask_downsample(md)
    idx, count = B.active_index_compact(m_out)
    plain = B.conv_desc(n, h, w, c, c, in_dtype=B.BF16, out_dtype=B.F32)
    ws = torch.empty((B.workspace_bytes(plain),), dtype=torch.uint8, device=G.dev())
    ws.fill_(0xAB)                                            # garbage an ordinary call must cope with
    want_masked = B.focused_conv2d(plain, x, wt, mask_in=md, mask_out=m_out, idx=idx, count=count, workspace=ws)
    want_dense = B.focused_conv2d(plain, x, wt, workspace=ws)
    B.ready_workspace(ws)
    masked = B.PreparedConv(plain, x, wt, mask_in=md, mask_out=m_out, idx=idx, count=count, workspace=ws,
                            workspace_ready=True)
    dense = B.PreparedConv(plain, x, wt, workspace=ws, workspace_ready=True)
    for _ in range(3):
        assert torch.equal(masked().clone(), want_masked)
        assert torch.equal(dense().clone(), want_dense)
        assert not ws[:B.WORKSPACE_COUNTER_BYTES].any()


def test_two_runs_are_bit_identical():
    torch = G.torch_mod()
    a, _, _ = _run_layer(2, 28, 28, 128, 128, 3, 1, 1, 1, synth.BF16, seed=208)
    b, _, _ = _run_layer(2, 28, 28, 128, 128, 3, 1, 1, 1, synth.BF16, seed=208)
    assert torch.equal(a, b)


def test_maxpool_helper():
    torch = G.torch_mod()
    x = synth.from_storage(synth.activations((2, 13, 17, 24), synth.F32, 209) - 0.5, synth.F32)
    xd = torch.from_numpy(x).to(G.dev())
    for (k, s, p) in ((2, 2, 0), (3, 2, 1)):
        got = B.maxpool2d(xd, k, s, p, B.F32).cpu()
        ref = torch.nn.functional.max_pool2d(torch.from_numpy(x).permute(0, 3, 1, 2), k, s, p).permute(0, 2, 3, 1)
        assert torch.equal(got, ref.contiguous())
    # 16-bit storage: channel counts on and off the 8-channel vector path, negative values too
    for dtype, c in ((synth.BF16, 24), (synth.F16, 64), (synth.BF16, 20)):
        bits = synth.to_storage(synth.from_storage(synth.activations((2, 13, 17, c), synth.F32, 210, c), synth.F32) - 0.7, dtype)
        xd = G.to_dev(bits, dtype)
        for (k, s, p) in ((2, 2, 0), (3, 2, 1)):
            got = B.maxpool2d(xd, k, s, p, dtype)
            ref = torch.nn.functional.max_pool2d(xd.float().permute(0, 3, 1, 2), k, s, p).permute(0, 2, 3, 1)
            assert torch.equal(got.float(), ref.contiguous())
            # with a keep mask: kept positions as above, the others all-zero bytes, and NaN in
            # windows that only dropped positions see is never read
            ho, wo = got.shape[1:3]
            keep = synth.mask_bernoulli(2, ho, wo, 0.5, 211, c, k)
            canary = torch.full_like(got, 7.0)
            B.maxpool2d(xd, k, s, p, dtype, out=canary, keep=G.mask_dev(keep))
            kd = torch.from_numpy(keep != 0).to(G.dev())
            assert torch.equal(canary[kd], got[kd])
            assert not canary[~kd].view(torch.int16).any()


def test_issue_probe_runs_and_counts_cycles():
    """fc_calibrate_issue: every mode and wave count runs, reports positive cycle counts, and two
    matrix instructions cannot take less than their 2 x 8 passes of four cycles."""
    torch = G.torch_mod()
    src = torch.ones((1 << 18,), dtype=torch.int32, device=G.dev())
    for waves in (1, 2, 4):
        for mode in range(5):
            cyc = B.calibrate_issue(mode, waves, 200, 8, src)
            torch.cuda.synchronize()
            per_step = cyc.double().cpu().numpy() / 200
            assert (per_step >= 40).all() and (per_step < 5000).all()
    with pytest.raises(B.FcError):
        B.calibrate_issue(7, 1, 10, 1, src)
    with pytest.raises(B.FcError):
        B.calibrate_issue(0, 3, 10, 1, src)

