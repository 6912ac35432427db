"""GPU parity at the benchmark's sizes and through whole conv stacks.

Large layers are checked on sampled output positions the oracle computes one by one
(half of the sample within two pixels of a mask edge or the image border), plus a
full check on the device that every irrelevant row is all-zero bytes.  Stacks are
checked layer by layer with the oracle fed the GPU's own input of that layer, so that
rounding of intermediate activations does not compound into the gate."""
import numpy as np
import pytest

from oracle import fc_oracle as O
from paper_2207_10741_amd import binding as B, synth, workloads
from paper_2207_10741_amd.stacks import ConvStack
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

TOL_F32_OUT = 1e-4
TOL_16BIT_OUT = 2e-2


def _sample_positions(mask_out: np.ndarray, count: int, seed: int) -> np.ndarray:
    """Flat output positions: half near a mask edge or the image border, half anywhere."""
    n, h, w = mask_out.shape
    m = mask_out != 0
    edge = np.zeros_like(m)
    edge[:, :2, :] = edge[:, -2:, :] = True
    edge[:, :, :2] = edge[:, :, -2:] = True
    for d in (1, 2):
        edge[:, d:, :] |= m[:, d:, :] != m[:, :-d, :]
        edge[:, :-d, :] |= m[:, d:, :] != m[:, :-d, :]
        edge[:, :, d:] |= m[:, :, d:] != m[:, :, :-d]
        edge[:, :, :-d] |= m[:, :, d:] != m[:, :, :-d]
    g = synth.rng(seed, 77)
    near = np.flatnonzero(edge & m)
    anywhere = np.arange(m.size)
    a = g.choice(near, size=min(count // 2, near.size), replace=False) if near.size else np.empty(0, np.int64)
    b = g.choice(anywhere, size=count - a.size, replace=False)
    return np.unique(np.concatenate([a, b]).astype(np.int64))


def _check_sampled(n, h, w, ci, co, k, s, p, mask, seed, samples=3000, dtype=synth.BF16):
    torch = G.torch_mod()
    x = synth.activations((n, h, w, ci), dtype, seed, 1)
    wt = synth.he_weights(co, k, k, ci, dtype, seed, 2)
    bias = synth.bias(co, seed, 3)
    xd, wd = G.to_dev(x, dtype), G.to_dev(wt, dtype)
    bd = torch.from_numpy(bias).to(G.dev())
    md = G.mask_dev(mask)
    shape = O.ConvShape(n, h, w, ci, co, k, k, (s, s), (p, p), (1, 1), relu=True)
    m_out = O.mask_downsample(mask, k, k, (s, s), (p, p))
    pos = _sample_positions(m_out, samples, seed)
    want = O.focused_conv2d_at(shape, x, wt, pos, bias=bias, mask_in=mask, dtype=dtype)
    keep_rows = m_out.reshape(-1)[pos] != 0
    rms = float(np.sqrt(np.mean(want[keep_rows] ** 2))) if keep_rows.any() else 1.0
    outs = {}
    for out_dtype in (B.F32, dtype):
        desc = B.conv_desc(n, h, w, ci, co, (k, k), (s, s), (p, p), (1, 1), dtype, out_dtype, B.RELU)
        ho, wo = B.out_dims(desc)
        out = torch.full((n, ho, wo, co), 7.0, dtype=B.torch_dtype(out_dtype), device=G.dev())
        B.focused_conv2d(desc, xd, wd, bd, mask_in=md, out=out)
        torch.cuda.synchronize()
        outs[out_dtype] = out
        got = out.reshape(-1, co)[torch.from_numpy(pos).to(G.dev())].to(torch.float64).cpu().numpy()
        err = float(np.abs(got - want).max()) / rms
        if out_dtype == B.F32:
            assert err <= TOL_F32_OUT, err
        elif err > TOL_16BIT_OUT:
            # rounding an outlier activation to 8 (11) significant bits can alone exceed the
            # RMS-relative bar; every element must then be within half a unit in the last place
            # of the oracle (plus the accumulation bound)
            half_ulp = np.abs(want) * (2.0 ** -8 if dtype == synth.BF16 else 2.0 ** -11)
            assert (np.abs(got - want) <= half_ulp + TOL_F32_OUT * rms).all(), err
        keep_d = torch.from_numpy(m_out != 0).to(G.dev())
        assert bool((out[~keep_d].view(torch.int16 if out.element_size() == 2 else torch.int32) == 0).all())
    assert torch.equal(outs[dtype], outs[B.F32].to(outs[dtype].dtype))     # one rounding, to nearest even
    # the kept list the library derives is the oracle's
    idx, count = B.active_index_compact(B.mask_downsample(md, (k, k), (s, s), (p, p)))
    want_idx, want_cnt = O.active_index_compact(m_out)
    assert int(count.cpu().item()) == want_cnt
    assert np.array_equal(idx[:want_cnt].cpu().numpy(), want_idx)


@pytest.mark.parametrize("c,side", workloads.sweep_shapes())
@pytest.mark.parametrize("mask_kind", ["blobs", "bernoulli"])
def test_sweep_shapes_full_batch_sampled(c, side, mask_kind):
    """The benchmark's four layers at its batch size and launch configuration."""
    n = workloads.SWEEP_BATCH
    if mask_kind == "blobs":
        mask = synth.mask_objects(n, side, side, workloads.HEADLINE_IRRELEVANT, 5, c, 4)
    else:
        mask = synth.mask_bernoulli(n, side, side, workloads.HEADLINE_IRRELEVANT, 5, c, 4)
    _check_sampled(n, side, side, c, c, 3, 1, 1, mask, 300 + c)


@pytest.mark.parametrize("layer", [
    # ResNet-50 bottleneck layers at 480x640 input, batch 32 (post-stem 120x160)
    (32, 120, 160, 64, 64, 3, 1, 1),
    (32, 120, 160, 64, 256, 1, 1, 0),
    (32, 120, 160, 256, 128, 1, 1, 0),
    (32, 120, 160, 128, 128, 3, 2, 1),
    (32, 30, 40, 256, 256, 3, 1, 1),
    (32, 30, 40, 1024, 512, 1, 1, 0),
    (32, 15, 20, 512, 512, 3, 1, 1),
    (32, 15, 20, 512, 2048, 1, 1, 0),
])
def test_resnet50_layers_full_batch_sampled(layer):
    n, h, w, ci, co, k, s, p = layer
    fr = synth.rng(330, h).uniform(0.3, 0.7, size=n)
    mask = synth.mask_objects(n, h, w, fr, 331, h, ci)
    _check_sampled(n, h, w, ci, co, k, s, p, mask, 332 + ci + co, samples=2000)


@pytest.mark.parametrize("layer", [
    # layers with enough tiles for each of the large-tile instances (small layers run 64 x 64 tiles)
    (8, 96, 96, 64, 128, 3, 1, 1),      # many 128 x 128 tiles, shared pixel line
    (4, 64, 64, 128, 128, 3, 1, 1),     # fewer tiles: 128 x 64, shared pixel line, reduction may be split
    (6, 80, 80, 64, 64, 3, 1, 1),       # 64 output channels
    (4, 72, 72, 96, 192, 3, 2, 1),      # stride 2: tap by tap
    (4, 60, 64, 256, 320, 1, 1, 0),     # 1x1
    (2, 48, 160, 32, 64, 5, 1, 2),      # 25 taps
])
@pytest.mark.parametrize("mask_kind,irr", [("bernoulli", 0.5), ("mixed", 0.5), ("band", 0.48), ("objects", 0.9),
                                           ("objects", 0.0), ("objects", 1.0)])
def test_large_tile_instances_mask_structures_sampled(layer, mask_kind, irr):
    n, h, w, ci, co, k, s, p = layer
    if mask_kind == "bernoulli":
        mask = synth.mask_bernoulli(n, h, w, irr, 345, h, ci)
    elif mask_kind == "band":
        mask = synth.mask_band_and_boxes(n, h, w, irr, 345, h, ci)
    elif mask_kind == "mixed":
        mask = synth.mask_bernoulli(n, h, w, irr, 345, h, ci)
        mask[:, :, w // 3:] = 1
        mask[:, ::7, :] = 0
    else:
        mask = synth.mask_objects(n, h, w, irr, 345, h, ci)
    _check_sampled(n, h, w, ci, co, k, s, p, mask, 346 + ci + co, samples=1500)


def test_hd_frame_first_layers_sampled():
    """VGG-16's first two convs on full-HD frames (batch 2 here), depth-ramp mask."""
    n, h, w = 2, 1080, 1920
    mask = synth.mask_depth_ramp(n, h, w, 0.5, 340)
    assert abs(synth.irrelevant_fraction(mask) - 0.5) < 0.02
    _check_sampled(n, h, w, 3, 64, 3, 1, 1, mask, 341, samples=1500)
    _check_sampled(n, h, w, 64, 64, 3, 1, 1, mask, 342, samples=1500)


@pytest.mark.parametrize("irr", [0.0, 0.1, 0.3, 0.5, 0.7, 0.9, 1.0])
@pytest.mark.parametrize("mask_kind", ["blobs", "bernoulli"])
def test_density_sweep_small(irr, mask_kind):
    n, side, c = 3, 32, 64
    mask = (synth.mask_objects if mask_kind == "blobs" else synth.mask_bernoulli)(n, side, side, irr, 350)
    x = synth.activations((n, side, side, c), synth.BF16, 351, 1)
    wt = synth.he_weights(c, 3, 3, c, synth.BF16, 351, 2)
    desc = B.conv_desc(n, side, side, c, c, in_dtype=B.BF16, out_dtype=B.F32)
    torch = G.torch_mod()
    out = torch.full((n, side, side, c), 7.0, dtype=torch.float32, device=G.dev())
    B.focused_conv2d(desc, G.to_dev(x, synth.BF16), G.to_dev(wt, synth.BF16), mask_in=G.mask_dev(mask), out=out)
    want = O.focused_conv2d(O.ConvShape(n, side, side, c, c), x, wt, mask_in=mask, dtype=O.BF16)
    keep = mask != 0
    assert G.rel_err(G.to_f64(out), want, keep) <= TOL_F32_OUT
    if irr == 0.0:
        assert keep.all()
    if irr == 1.0:
        assert not keep.any() and not out.cpu().numpy().view(np.uint32).any()


# ------------------------------------------------------------------ stacks ----

def _check_stack(ops, n, h, w, c_in, mask, seed, dtype=synth.BF16):
    torch = G.torch_mod()
    tol = 5e-4 if dtype == synth.FP8 else TOL_F32_OUT     # the 8-bit matrix instruction's summation
    stack = ConvStack(ops, n, h, w, dtype, seed=seed)
    x = synth.activations((n, h, w, c_in), dtype, seed, 1)
    outs, masks = stack.run(G.to_dev(x, dtype), G.mask_dev(mask))
    torch.cuda.synchronize()
    host_masks = {-1: mask}
    dense_macs = kept_macs = 0
    for i, op in enumerate(ops):
        m_in = host_masks[op.src]
        m_out = O.mask_downsample(m_in, op.k, op.k, (op.stride,) * 2, (op.pad,) * 2)
        host_masks[i] = m_out
        np.testing.assert_array_equal(masks[i].cpu().numpy(), m_out, err_msg=op.name)
        src = G.to_storage_np(outs[op.src], dtype)
        hi, wi = src.shape[1:3]
        if op.kind == "maxpool":
            # the pool computes the positions its mask keeps and writes zeros elsewhere
            ref = torch.nn.functional.max_pool2d(outs[op.src].float().permute(0, 3, 1, 2), op.k, op.stride, op.pad)
            kd = torch.from_numpy(m_out != 0).to(G.dev())
            assert torch.equal(outs[i].float()[kd], ref.permute(0, 2, 3, 1).contiguous()[kd]), op.name
            assert not outs[i][~kd].view(torch.int16).any(), op.name
            continue
        shape = O.ConvShape(n, hi, wi, op.c_in, op.c_out, op.k, op.k, (op.stride,) * 2, (op.pad,) * 2, (1, 1), relu=True)
        keep = m_out != 0
        # accumulation gate on an fp32-output call with the same device inputs
        if op.kind == "dwconv":
            want = O.focused_dwconv2d(shape, src, stack.host_weights[i], bias=stack.host_biases[i], mask_in=m_in,
                                      dtype=dtype)
            o32 = B.focused_dwconv2d(stack.desc(i, out_dtype=B.F32), outs[op.src], stack.weights[i], stack.biases[i],
                                     mask_in=masks[op.src])
        else:
            want = O.focused_conv2d(shape, src, stack.host_weights[i], bias=stack.host_biases[i], mask_in=m_in,
                                    dtype=dtype)
            o32 = B.focused_conv2d(stack.desc(i, out_dtype=B.F32), outs[op.src], stack.weights[i], stack.biases[i],
                                   mask_in=masks[op.src])
        assert G.rel_err(G.to_f64(o32), want, keep) <= tol, op.name
        if dtype == synth.FP8:
            # the stored codes are the oracle's narrowing of the fp32-output call's values
            f32 = o32.cpu().numpy()
            expect = O.narrow_fp8(f32.astype(np.float64))
            expect[f32 == 0] = 0
            np.testing.assert_array_equal(G.to_storage_np(outs[i], dtype), expect, err_msg=op.name)
        else:
            assert torch.equal(outs[i], o32.to(outs[i].dtype)), op.name
        assert not G.to_storage_np(outs[i], dtype)[~keep].any(), op.name
        macs = op.k * op.k * op.c_in * (op.c_out if op.kind == "conv" else 1)
        dense_macs += keep.size * macs
        kept_macs += int(keep.sum()) * macs
    return kept_macs / dense_macs


def test_resnet18_stack_layer_by_layer():
    """All 20 convs of the ResNet-18-shaped stack, batch 1, 224x224x3, ~48 % irrelevant."""
    mask = synth.mask_objects(1, 224, 224, 0.48, 360)
    ratio = _check_stack(workloads.resnet18(), 1, 224, 224, 3, mask, 361)
    # Table I: the multiply-add ratio follows the kept share of the image
    # (coarse 7x7 and 14x14 maps quantise the share, hence the loose band)
    assert abs(ratio - (1.0 - synth.irrelevant_fraction(mask))) < 0.07


def test_vgg16_stack_small_frames():
    """VGG-16's 13 convs and 4 pools on small frames (the layer list of the HD workload)."""
    n, h, w = 2, 72, 128
    mask = synth.mask_depth_ramp(n, h, w, 0.5, 362)
    _check_stack(workloads.vgg16(), n, h, w, 3, mask, 363)


def test_resnet50_bottlenecks_small_batch():
    """All 52 convs of the bottleneck stack at reduced size (batch 2, 48x64 post-stem)."""
    n, h, w = 2, 48, 64
    mask = synth.mask_objects(n, h, w, [0.35, 0.65], 364)
    _check_stack(workloads.resnet50_bottlenecks(), n, h, w, 64, mask, 365)


def test_resnet50_bottlenecks_8bit_chain():
    """The same 52 convs with 8-bit (E4M3) activations and weights all the way: every layer reads
    the previous layer's bytes and is checked against the oracle fed those bytes."""
    n, h, w = 2, 48, 64
    mask = synth.mask_objects(n, h, w, [0.35, 0.65], 366)
    _check_stack(workloads.resnet50_bottlenecks(), n, h, w, 64, mask, 367, dtype=synth.FP8)


def test_mobilenetv2_stack_layer_by_layer():
    """All 52 convs of the MobileNetV2-shaped stack (1x1 / depthwise 3x3 / 1x1 blocks) on small images."""
    n, h, w = 2, 96, 128
    mask = synth.mask_objects(n, h, w, [0.4, 0.55], 372)
    ops = workloads.mobilenetv2()
    assert sum(op.kind == "dwconv" for op in ops) == 17 and sum(op.kind == "conv" for op in ops) == 35
    ratio = _check_stack(ops, n, h, w, 3, mask, 373)
    assert abs(ratio - (1.0 - synth.irrelevant_fraction(mask))) < 0.07


def test_chain_mode_never_reads_the_unwritten_rows():
    """Convs read only by convs leave their irrelevant rows unwritten; the readers gate their
    taps by the same mask, so every kept output is bit-identical to the zero-filled run even
    when the unwritten rows hold NaN.  Outputs that a pool or nobody reads stay zero-filled."""
    torch = G.torch_mod()
    dtype = synth.BF16
    for ops, (n, h, w, c_in), mask in (
        (workloads.resnet50_bottlenecks()[:13], (2, 48, 64, 64), synth.mask_objects(2, 48, 64, [0.4, 0.6], 366)),
        (workloads.vgg16()[:8], (1, 48, 64, 3), synth.mask_depth_ramp(1, 48, 64, 0.5, 367)),
        (workloads.mobilenetv2()[:12], (2, 64, 96, 3), synth.mask_objects(2, 64, 96, [0.4, 0.6], 369)),
    ):
        stack = ConvStack(ops, n, h, w, dtype, seed=368)
        x = G.to_dev(synth.activations((n, h, w, c_in), dtype, 368, 1), dtype)
        md = G.mask_dev(mask)
        strict, masks = stack.run(x, md)
        chained, _ = stack.run(x, md, chain=True, canary=float("nan"))
        torch.cuda.synchronize()
        readers = {}
        for op in ops:
            readers.setdefault(op.src, []).append(op.kind)
        skipped = 0
        for i, op in enumerate(ops):
            keep = masks[i].bool()
            a, b = strict[i], chained[i]
            assert torch.equal(a[keep].view(torch.int16), b[keep].view(torch.int16)), op.name
            if op.kind not in ("conv", "dwconv"):
                continue
            if readers.get(i) and all(k in ("conv", "dwconv") for k in readers[i]):
                assert torch.isnan(b[~keep].float()).all(), op.name      # untouched canary
                skipped += 1
            else:
                assert not b[~keep].view(torch.int16).any(), op.name     # zero-filled as usual
        assert skipped >= 3


def test_compact_mode_holds_the_same_rows_as_the_spatial_layout():
    """With compacted activations (rows in list order between a conv and the 1x1 convs that read
    it) every layer's kept rows are, bit for bit, those of the chained spatial run, wherever they
    are stored; rows past the kept count keep the canary."""
    torch = G.torch_mod()
    dtype = synth.BF16
    ops = workloads.resnet50_bottlenecks()[:23]
    n, h, w, c_in = 2, 48, 64, 64
    mask = synth.mask_objects(n, h, w, [0.4, 0.6], 371)
    stack = ConvStack(ops, n, h, w, dtype, seed=372)
    x = G.to_dev(synth.activations((n, h, w, c_in), dtype, 372, 1), dtype)
    md = G.mask_dev(mask)
    chained, masks = stack.run(x, md, chain=True)
    compact, _ = stack.run(x, md, chain=True, compact=True, canary=float("nan"))
    torch.cuda.synchronize()
    n_compact = 0
    for i, op in enumerate(ops):
        keep = masks[i].bool()
        a, b = chained[i], compact[i]
        if b.dim() == 2:                               # stored compacted: [positions, channels]
            cnt = int(keep.sum().item())
            assert torch.equal(b[:cnt].view(torch.int16), a[keep].view(torch.int16)), op.name
            assert torch.isnan(b[cnt:].float()).all(), op.name
            n_compact += 1
        else:
            assert torch.equal(a[keep].view(torch.int16), b[keep].view(torch.int16)), op.name
    assert n_compact >= 8


# ------------------------------------------------------- graph capture ----

def test_graph_replays_match_eager():
    """The library only enqueues kernels on the given stream, so a call can be recorded
    into a HIP graph; every replay must reproduce the eager result, with eager work and
    synchronisations between the replays."""
    torch = G.torch_mod()
    n, side, c = 4, 40, 128
    x = synth.activations((n, side, side, c), synth.BF16, 370, 1)
    wt = synth.he_weights(c, 3, 3, c, synth.BF16, 370, 2)
    bias = synth.bias(c, 370, 3)
    mask = synth.mask_objects(n, side, side, 0.48, 370, 4)
    desc = B.conv_desc(n, side, side, c, c, in_dtype=B.BF16, out_dtype=B.BF16, flags=B.RELU)
    xd, wd, bd, md = G.to_dev(x, synth.BF16), G.to_dev(wt, synth.BF16), torch.from_numpy(bias).to(G.dev()), G.mask_dev(mask)
    eager = B.focused_conv2d(desc, xd, wd, bd, mask_in=md).clone()
    call = B.PreparedConv(desc, xd, wd, bd, mask_in=md)
    call()
    torch.cuda.synchronize()
    side_stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side_stream):
        call()
    for rep in range(4):
        call.out.fill_(3.0)
        other = B.focused_conv2d(desc, xd * 0.5, wd, bd, mask_in=md)     # eager work in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(call.out, eager), rep
        assert not torch.equal(other, eager)
