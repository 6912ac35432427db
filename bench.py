#!/usr/bin/env python3
"""Benchmark of the focused-convolution hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: mask
propagation and ordered compaction of the kept positions for every layer of the
workload (one mask pyramid call), then per layer the focused convolution itself
(gather + matrix-core GEMM + bias/ReLU/scatter + zero-fill of the irrelevant rows),
with all inputs already resident in HBM.

Default workload: the four 3x3 layer shapes of ResNet-50 (C = 64/128/256/512 at
128/64/32/16 pixels a side), batch 16, bf16, seeded blob masks with 48 % of the
pixels irrelevant - the operating point the paper's census gives (Sec. II-B) and
the one the metric is quoted on.  `value` is effective TFLOP/s counted on kept
positions only; the same JSON line carries the speed-up over the library's own
dense path, ms per image, the roofline fraction of the dominant kernel and the
CPU oracle's throughput on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "focused-conv effective TFLOP/s + speedup vs dense at 48% irrelevant pixels"
BF16_MFMA_PEAK_TFLOPS = 2500.0
FP8_MFMA_PEAK_TFLOPS = 5000.0
# HBM bytes per launch of the conv kernels on the default workload (mean of the four layers)
# come from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, each scaled by what the counter read
# for a streaming copy of known size.  The summary of those runs is the one tracked place the
# figure lives in; it also records the hash of the kernel sources it was measured on, and the
# bench line carries the figure only while that hash is the one of the tree that runs.
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "k_conv_resnet50_3x3_b16_48pct.md")
HBM_PEAK_GBPS = 8000.0


def kernel_source_hash():
    """sha256 (first 16 hex digits) over the library's kernel sources, in name order."""
    import glob
    import hashlib
    h = hashlib.sha256()
    base = os.path.join(ROOT, "paper_2207_10741_amd", "csrc")
    for f in sorted(glob.glob(os.path.join(base, "*.hip")) + glob.glob(os.path.join(base, "*.hpp"))):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def measured_traffic():
    """(bytes per launch, note): the figure of the tracked profile summary, or None when the summary is
    missing or was measured on other kernel sources."""
    import re
    try:
        text = open(TRAFFIC_PROFILE).read()
    except OSError:
        return None, "no counter summary in profiles/"
    m_t = re.search(r"traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)", text)
    m_h = re.search(r"kernel_source_hash\s*=\s*([0-9a-f]+)", text)
    if not m_t or not m_h:
        return None, "counter summary carries no figure"
    if m_h.group(1) != kernel_source_hash():
        return None, "counter summary was measured on other kernel sources (%s)" % m_h.group(1)
    return float(m_t.group(1)), "rocprofv3 FETCH_SIZE + WRITE_SIZE, " + os.path.relpath(TRAFFIC_PROFILE, ROOT)


def calibrate_peaks(torch, B, in_dtype):
    """What this machine delivers: matrix-core rate of a register-only loop of independent matrix
    instructions on every SIMD, and the rate of a streaming copy far larger than the memory-side
    cache (bytes read + bytes written).  Best of three launches each, HIP events on the launch stream."""
    dev = torch.device("cuda:0")
    sink = torch.zeros((4096 * 256,), dtype=torch.float32, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    best_f = 0.0
    for _ in range(4):
        a, b = ev(), ev()
        a.record()
        flop = B.calibrate_mfma(in_dtype, 2000, 4096, sink)
        b.record()
        torch.cuda.synchronize()
        best_f = max(best_f, flop / (a.elapsed_time(b) * 1e-3))
    src = torch.ones((128 << 20,), dtype=torch.int32, device=dev)     # 512 MiB
    dst = torch.empty_like(src)
    best_b = 0.0
    for _ in range(4):
        a, b = ev(), ev()
        a.record()
        nbytes = B.calibrate_copy(src, dst)
        b.record()
        torch.cuda.synchronize()
        best_b = max(best_b, 2.0 * nbytes / (a.elapsed_time(b) * 1e-3))
    del src, dst, sink
    torch.cuda.empty_cache()
    return {"mfma_tflops": round(best_f / 1e12, 1), "copy_gbps": round(best_b / 1e9, 1),
            "how": "register-only loop of 8 independent matrix instructions per wave, 16 waves per CU; "
                   "streaming copy of 512 MiB (read + written bytes); best of 4 launches each"}


ISSUE_ITEMS = ("two matrix instructions only", "+ one 1 KB load into LDS", "+ twelve dependent integer instructions",
               "+ one 16-byte-per-lane LDS read (the next operand)", "+ the LDS load and the LDS read")


def issue_probe(torch, B):
    """What a SIMD can do beside its matrix instructions (fc_calibrate_issue): every wave runs steps
    of two 32x32x16 bf16 matrix instructions plus one item, with 1, 2 and 4 waves per SIMD on
    every CU.  Reported: wall time of the launch per step (HIP events, best of three; a step of
    the launch is one step of every wave) and the shader cycles per step that the first wave of
    a workgroup counted for itself (the oldest wave is served first, so with several waves per
    SIMD it finishes before the others)."""
    dev = torch.device("cuda:0")
    src = torch.ones((1 << 18,), dtype=torch.int32, device=dev)     # 1 MiB
    steps, blocks = 4000, torch.cuda.get_device_properties(0).multi_processor_count
    ev = lambda: torch.cuda.Event(enable_timing=True)
    table = {}
    for waves in (1, 2, 4):
        row = {}
        for mode, name in enumerate(ISSUE_ITEMS):
            best, cyc = None, None
            for _ in range(3):
                a, b = ev(), ev()
                a.record()
                cyc = B.calibrate_issue(mode, waves, steps, blocks, src)
                b.record()
                torch.cuda.synchronize()
                t = a.elapsed_time(b) * 1e6 / steps
                best = t if best is None else min(best, t)
            row[name] = {"ns_per_step": round(best, 1),
                         "ns_per_matrix_instruction": round(best / (2 * waves), 2),
                         "first_wave_cycles_per_step": round(float(cyc.double().mean().item()) / steps, 1)}
        table["%d waves per SIMD" % waves] = row
    return {"per_step": table, "steps": steps, "workgroups": blocks,
            "how": "every wave: steps of two independent 32x32x16 bf16 matrix instructions plus the item; one launch, "
                   "HIP events around it (launch overhead of about 10 us included), best of three"}


def build_sweep_layers(torch, B, synth, workloads, irrelevant, mask_kind, batch, in_dtype=None, out_dtype=None):
    """Device tensors for the four ResNet-50 3x3 shapes (bf16 storage, or E4M3 bytes with
    bf16 or E4M3 outputs)."""
    in_dtype = B.BF16 if in_dtype is None else in_dtype
    out_dtype = B.BF16 if out_dtype is None else out_dtype
    dev = torch.device("cuda:0")
    layers = []
    for li, (c, side) in enumerate(workloads.sweep_shapes()):
        key = (5, li)
        x = synth.activations((batch, side, side, c), in_dtype, *key, 1)
        w = synth.he_weights(c, 3, 3, c, in_dtype, *key, 2)
        bias = synth.bias(c, *key, 3)
        if mask_kind == "bernoulli":
            mask = synth.mask_bernoulli(batch, side, side, irrelevant, *key, 4)
        else:
            mask = synth.mask_objects(batch, side, side, irrelevant, *key, 4)
        desc = B.conv_desc(batch, side, side, c, c, in_dtype=in_dtype, out_dtype=out_dtype, flags=B.RELU)
        if in_dtype == B.FP8:
            to_dev = lambda codes: torch.from_numpy(codes).to(dev).view(torch.float8_e4m3fn)
        else:
            to_dev = lambda bits: torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
        L = dict(name="c%d@%d" % (c, side), desc=desc, c=c, side=side,
                 x=to_dev(x), w=to_dev(w), bias=torch.from_numpy(bias).to(dev),
                 mask=torch.from_numpy(mask).to(dev), host=(x, w, bias, mask),
                 kept=int(np.count_nonzero(mask)), m=mask.size, k=9 * c)
        L["out"] = torch.empty((batch, side, side, c), dtype=B.torch_dtype(out_dtype), device=dev)
        # one workspace per layer, counters cleared once: the timed calls carry FC_WORKSPACE_READY
        L["ws"] = B.ready_workspace(torch.empty((B.workspace_bytes(desc),), dtype=torch.uint8, device=dev))
        L["flops_kept"] = 2.0 * L["kept"] * L["k"] * c
        L["flops_dense"] = 2.0 * L["m"] * L["k"] * c
        layers.append(L)
    return layers


def time_loop(torch, fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def capture(torch, fn):
    """One step recorded into a HIP graph (the layers take a few microseconds each, so
    eager launches from Python would measure the host).  The library only enqueues
    kernels on the stream it is given: no memsets, no allocation, no host sync."""
    fn()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        fn()
    torch.cuda.synchronize()
    return graph


def cpu_baseline(layers, images):
    """The oracle as it stands, on `images` images of every layer, all host threads."""
    from oracle import fc_oracle as O
    O.lib()
    flops = 0.0
    t = 0.0
    for L in layers:
        x, w, bias, mask = L["host"]
        c, side = L["c"], L["side"]
        s = O.ConvShape(images, side, side, c, c, relu=True)
        t0 = time.perf_counter()
        O.focused_conv2d(s, x[:images], w, bias=bias, mask_in=mask[:images], dtype=L["desc"].in_dtype)
        t += time.perf_counter() - t0
        flops += 2.0 * int(np.count_nonzero(mask[:images])) * L["k"] * c
    return flops / t / 1e12, O.num_threads(), t


def sweep(torch, B, synth, workloads, args, batch):
    """Mask-density sweep of the four layer shapes: irrelevant share 0, 0.1, ... 1 for blob and
    Bernoulli masks; per layer the conv kernel alone (kept list given) and the whole call
    (mask propagation + compaction + conv + zero-fill), each as a HIP-graph replay; a
    least-squares line t = a + b * kept_share per layer and mask structure."""
    shares = [round(0.1 * i, 1) for i in range(11)]
    out = {"sweep": True, "batch": batch, "unit": "us", "launch_floor_us": None, "layers": {}}
    # what one (near-)empty kernel costs inside a replayed graph: 16 of them, divided by 16
    tiny = torch.zeros((64,), dtype=torch.int32, device="cuda:0")
    def sixteen():
        for _ in range(16):
            tiny.add_(1)
    g = capture(torch, sixteen)
    out["launch_floor_us"] = round(time_loop(torch, g.replay, args.steps, args.warmup) / 16 * 1e6, 2)
    layers = build_sweep_layers(torch, B, synth, workloads, 0.0, "blobs", batch)   # tensors made once
    for L in layers:
        L["dense"] = B.PreparedConv(L["desc"], L["x"], L["w"], L["bias"], out=L["out"], workspace=L["ws"], workspace_ready=True)

    def timed(call):
        def fn():
            for _ in range(4):
                call()
        return time_loop(torch, capture(torch, fn).replay, args.steps, args.warmup) / 4 * 1e6

    for li, L in enumerate(layers):
        L["dense_us"] = timed(L["dense"])
    for kind in ("blobs", "bernoulli"):
        gen = synth.mask_bernoulli if kind == "bernoulli" else synth.mask_objects
        for li, L in enumerate(layers):
            pts = []
            for f in shares:
                mask_host = gen(batch, L["side"], L["side"], f, 5, li, 4)
                L["mask"].copy_(torch.from_numpy(mask_host))
                m_out = B.mask_downsample(L["mask"])
                idx, count = B.active_index_compact(m_out)
                d = L["desc"]
                full = B.PreparedConv(d, L["x"], L["w"], L["bias"], mask_in=L["mask"], out=L["out"], workspace=L["ws"], workspace_ready=True)
                conv = B.PreparedConv(d, L["x"], L["w"], L["bias"], mask_in=L["mask"], mask_out=m_out, idx=idx,
                                      count=count, out=L["out"], workspace=L["ws"], workspace_ready=True)
                pts.append((float(np.count_nonzero(mask_host)) / mask_host.size, timed(conv), timed(full)))
            r = np.array([p[0] for p in pts])
            entry = {"kept_share": [round(float(v), 4) for v in r], "dense_us": round(L["dense_us"], 2)}
            for col, name in ((1, "conv_only_us"), (2, "whole_call_us")):
                t = np.array([p[col] for p in pts])
                b, a = np.polyfit(r, t, 1)
                ss_res = float(np.sum((t - (a + b * r)) ** 2))
                ss_tot = float(np.sum((t - t.mean()) ** 2))
                entry[name] = [round(float(v), 2) for v in t]
                entry[name + "_fit"] = {"a_us": round(float(a), 2), "b_us": round(float(b), 2),
                                        "r2": round(1.0 - ss_res / ss_tot, 4) if ss_tot > 0 else None}
            out["layers"].setdefault(L["name"], {})[kind] = entry
    print(json.dumps(out))


STACKS = {
    # name: (layer list, batch, height, width, input channels, what it stands for)
    "resnet18": ("resnet18", 1, 224, 224, 3, "ResNet-18-shaped stack, batch 1, 224x224x3, boxes + sky band, 48 % irrelevant"),
    "resnet50": ("resnet50_bottlenecks", 32, 120, 160, 64,
                 "ResNet-50 bottleneck convs on the post-stem activation of 480x640 images, batch 32, "
                 "per-image irrelevant share uniform in [0.3, 0.7]"),
    "vgg16": ("vgg16", 8, 1080, 1920, 3, "VGG-16 convs on 1080x1920 frames, batch 8, depth-ramp mask, 50 % irrelevant"),
    "mobilenetv2": ("mobilenetv2", 32, 224, 224, 3,
                    "MobileNetV2 backbone convs (1x1 / depthwise 3x3 / 1x1 blocks), batch 32, 224x224x3, boxes + sky "
                    "band, 48 % irrelevant"),
}


def stack_bench(torch, B, synth, workloads, args):
    """A whole conv stack (every conv one library call, masks and kept lists built once per
    resolution): dense, focused with every output zero-filled, and focused with conv-to-conv
    outputs left unwritten at irrelevant rows.  One HIP graph replay per pass."""
    from paper_2207_10741_amd.stacks import ConvStack
    fn_name, n, h, w, c_in, what = STACKS[args.stack]
    if args.batch is not None:
        what = what.replace("batch %d" % n, "batch %d" % args.batch)
        n = args.batch
    ops = getattr(workloads, fn_name)()
    if args.stack == "resnet50":
        shares = list(synth.rng(3, 0, 5).uniform(0.3, 0.7, size=n))
        mask = synth.mask_objects(n, h, w, shares, 3, 0, 4)
    elif args.stack == "vgg16":
        mask = synth.mask_depth_ramp(n, h, w, 0.5, 4, 0, 4)
    else:
        mask = synth.mask_objects(n, h, w, workloads.HEADLINE_IRRELEVANT, 2, 0, 4)
    fp8 = args.in_dtype == "fp8"    # 8-bit activations and weights all the way (stacks of matrix-core convs only)
    stack = ConvStack(ops, n, h, w, B.FP8 if fp8 else B.BF16, seed=len(args.stack))
    x_host = synth.activations((n, h, w, c_in), synth.FP8 if fp8 else synth.BF16, 9, 0, 1)
    if fp8:
        x = torch.from_numpy(x_host).to("cuda:0").view(torch.float8_e4m3fn)
    else:
        x = torch.from_numpy(x_host.view(np.int16)).to("cuda:0").view(torch.bfloat16)
    md = torch.from_numpy(mask).to("cuda:0")
    del x_host

    # kept rows per conv, from the propagated masks of one eager pass
    _, masks = stack.run(x, md, keep_outputs=False)
    torch.cuda.synchronize()
    dense_flops = kept_flops = 0.0
    for i, op in enumerate(ops):
        if op.kind not in ("conv", "dwconv"):
            continue
        per_pos = 2.0 * op.k * op.k * op.c_in * (op.c_out if op.kind == "conv" else 1)
        dense_flops += masks[i].numel() * per_pos
        kept_flops += float(torch.count_nonzero(masks[i]).item()) * per_pos
    del masks

    def timed(**kw):
        def one():
            stack.run(x, kw.get("mask"), keep_outputs=False, chain=kw.get("chain", False),
                      compact=kw.get("compact", False))
        try:
            graph = capture(torch, one)
            t = time_loop(torch, graph.replay, args.steps, args.warmup)
            del graph
            how = "one HIP graph replay per pass"
        except Exception:   # capture not possible: time the eager calls
            torch.cuda.synchronize()
            t = time_loop(torch, one, args.steps, args.warmup)
            how = "eager calls"
        torch.cuda.empty_cache()
        return t, how

    t_dense, how = timed()
    t_strict, _ = timed(mask=md)
    t_chain, _ = timed(mask=md, chain=True)
    t_compact, _ = timed(mask=md, chain=True, compact=True)
    print(json.dumps({
        "stack": args.stack, "workload": what, "batch": n, "convs": sum(op.kind in ("conv", "dwconv") for op in ops),
        "launch": how, "steps": args.steps, "dtype": args.in_dtype, "data": "synthetic",
        "kept_flop_share": round(kept_flops / dense_flops, 4),
        "dense_ms": round(t_dense * 1e3, 4), "dense_tflops": round(dense_flops / t_dense / 1e12, 2),
        "focused_ms": round(t_strict * 1e3, 4), "focused_effective_tflops": round(kept_flops / t_strict / 1e12, 2),
        "speedup_vs_dense": round(t_dense / t_strict, 3),
        "focused_chain_ms": round(t_chain * 1e3, 4), "speedup_chain_vs_dense": round(t_dense / t_chain, 3),
        "focused_compact_ms": round(t_compact * 1e3, 4), "speedup_compact_vs_dense": round(t_dense / t_compact, 3),
        "ms_per_image": round(t_strict * 1e3 / n, 5),
    }))


def depthwise_bench(torch, B, synth, workloads, args):
    """The 3x3 depthwise layers of a MobileNetV2 backbone, batch 32, bf16, blob masks: per layer
    the focused call and the same call without a mask, each as a HIP-graph replay of four
    calls.  The layer is bound by memory traffic: algorithmic bytes = input mask + relevant
    input pixels once + filters and bias + every output row once (kept rows and zero rows)."""
    irr = workloads.HEADLINE_IRRELEVANT if args.irrelevant is None else args.irrelevant
    n = workloads.DEPTHWISE_BATCH if args.batch is None else args.batch
    dev = torch.device("cuda:0")
    gen = synth.mask_bernoulli if args.mask == "bernoulli" else synth.mask_objects
    rows, t_f, t_d, bytes_f, bytes_d = [], 0.0, 0.0, 0.0, 0.0
    for li, (c, side, stride) in enumerate(workloads.mobilenetv2_depthwise()):
        x = synth.activations((n, side, side, c), synth.BF16, 6, li, 1)
        w = np.ascontiguousarray(synth.he_weights(c, 3, 3, 1, synth.BF16, 6, li, 2)[..., 0])
        bias = synth.bias(c, 6, li, 3)
        mask = gen(n, side, side, irr, 6, li, 4)
        to_dev = lambda bits: torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
        desc = B.conv_desc(n, side, side, c, c, (3, 3), (stride, stride), (1, 1), (1, 1), B.BF16, B.BF16, B.RELU)
        ho, wo = B.out_dims(desc)
        xd, wd, bd, md = to_dev(x), to_dev(w), torch.from_numpy(bias).to(dev), torch.from_numpy(mask).to(dev)
        out = torch.empty((n, ho, wo, c), dtype=torch.bfloat16, device=dev)
        focused = B.PreparedDwConv(desc, xd, wd, bd, mask_in=md, out=out)
        dense = B.PreparedDwConv(desc, xd, wd, bd, out=out)

        def timed(call):
            def fn():
                for _ in range(4):
                    call()
            return time_loop(torch, capture(torch, fn).replay, args.steps, args.warmup) / 4

        tf, td = timed(focused), timed(dense)
        kept_in = float(np.count_nonzero(mask))
        m = n * ho * wo
        common = c * 9 * 2 + c * 4 + m * c * 2
        bf = mask.size + kept_in * c * 2 + common
        bd_ = mask.size * c * 2 + common
        rows.append({"layer": "c%d@%d/s%d" % (c, side, stride), "focused_us": round(tf * 1e6, 2),
                     "dense_us": round(td * 1e6, 2), "speedup": round(td / tf, 3),
                     "focused_GBps": round(bf / tf / 1e9, 1), "dense_GBps": round(bd_ / td / 1e9, 1)})
        t_f, t_d, bytes_f, bytes_d = t_f + tf, t_d + td, bytes_f + bf, bytes_d + bd_
        del xd, out, focused, dense
    print(json.dumps({
        "depthwise": True, "workload": "MobileNetV2 3x3 depthwise layers, batch %d, 224x224 images, bf16, %s masks, "
        "%d %% irrelevant" % (n, args.mask, round(irr * 100)), "launch": "HIP graph replay of four calls",
        "steps": args.steps, "layers": rows, "focused_ms": round(t_f * 1e3, 4), "dense_ms": round(t_d * 1e3, 4),
        "speedup_vs_dense": round(t_d / t_f, 3),
        "roofline": {"bound": "hbm", "achieved": round(bytes_f / t_f / 1e9, 1), "peak": 8000.0, "unit": "GB/s",
                     "frac": round(bytes_f / t_f / 8e12, 4), "traffic": None},
        "dense_GBps": round(bytes_d / t_d / 1e9, 1)}))


def pointwise_kernel_of(ci, co, m):
    """Which matrix-core kernel the library gives a 1x1 layer (the rule of its dispatch, restated
    for the bench's table: the profiler's kernel names are the evidence)."""
    kch = (ci + 63) // 64
    fits = kch == 1 or kch * 64 * 128 + 1024 + 8 * 8448 <= 160 * 1024
    if m <= 4096 or ci % 8 or co % 8 or not fits or (ci == 256 and co <= 128):
        return "k_conv_dma"
    if kch >= 3 and co <= (64 if kch > 4 else 128) and m < 100000:
        return "k_conv_dma"
    return "k_conv_pw"


def pointwise_bench(torch, B, synth, workloads, args):
    """1x1 layers of a ResNet-50 (up to 512 input channels) at the resolutions its stages see them
    on 480x640 images, batch 32, bf16, blob masks with the list given: per layer the dense call,
    the focused call (irrelevant rows cleared) and the chained call (irrelevant rows left alone),
    each as a HIP-graph replay of four calls.  These layers are bound by memory traffic:
    algorithmic bytes = kept input rows + kept output rows (+ the cleared rows) + the list +
    weights and bias."""
    irr = workloads.HEADLINE_IRRELEVANT if args.irrelevant is None else args.irrelevant
    mbv2 = args.pointwise == "mobilenetv2"    # the 1x1 layers of a MobileNetV2 on 224x224 images, batch 256
    n = (256 if mbv2 else workloads.POINTWISE_BATCH) if args.batch is None else args.batch
    dev = torch.device("cuda:0")
    gen = synth.mask_bernoulli if args.mask == "bernoulli" else synth.mask_objects
    mask0 = gen(n, 224, 224, irr, 9, 0, 4) if mbv2 else gen(n, workloads.POINTWISE_H, workloads.POINTWISE_W, irr, 9, 0, 4)
    to_dev = lambda bits: torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
    rows, tot = [], {"dense": [0.0, 0.0], "focused": [0.0, 0.0], "chained": [0.0, 0.0]}
    kept0 = float(np.count_nonzero(mask0)) / mask0.size
    for li, (ci, co, div) in enumerate(workloads.mobilenetv2_pointwise() if mbv2 else workloads.resnet50_pointwise()):
        mask = np.ascontiguousarray(mask0[:, ::div, ::div])      # the centre-tap labels at that stage
        h, w_ = mask.shape[1], mask.shape[2]
        md = torch.from_numpy(mask).to(dev)
        idx, count = B.active_index_compact(md)
        kept, m = int(count.item()), n * h * w_
        xd = to_dev(synth.activations_large((n, h, w_, ci), synth.BF16, 9, li, 1))
        wd = to_dev(synth.he_weights(co, 1, 1, ci, synth.BF16, 9, li, 2))
        bd = torch.from_numpy(synth.bias(co, 9, li, 3)).to(dev)
        out = torch.empty((n, h, w_, co), dtype=torch.bfloat16, device=dev)
        fixed = ci * co * 2 + co * 4
        row = {"layer": "%d->%d@%dx%d" % (ci, co, h, w_),
               "kernel": pointwise_kernel_of(ci, co, m)}
        for kind in ("dense", "focused", "chained"):
            flags = B.RELU | (B.SKIP_ZERO_FILL if kind == "chained" else 0)
            desc = B.conv_desc(n, h, w_, ci, co, (1, 1), (1, 1), (0, 0), (1, 1), B.BF16, B.BF16, flags)
            kw = {} if kind == "dense" else dict(mask_in=md, mask_out=md, idx=idx, count=count)
            call = B.PreparedConv(desc, xd, wd, bd, out=out, **kw)

            def fn():
                for _ in range(4):
                    call()
            t = time_loop(torch, capture(torch, fn).replay, args.steps, args.warmup) / 4
            r = m if kind == "dense" else kept
            by = r * (ci + co) * 2 + fixed + (0 if kind == "dense" else kept * 4) \
                + ((m - kept) * co * 2 if kind == "focused" else 0)
            row[kind + "_us"] = round(t * 1e6, 2)
            row[kind + "_GBps"] = round(by / t / 1e9, 1)
            tot[kind][0] += t
            tot[kind][1] += by
        rows.append(row)
        del xd, out
    copy_gbps = calibrate_peaks(torch, B, B.BF16)["copy_gbps"]
    t_f, by_f = tot["focused"]
    print(json.dumps({
        "pointwise": True, "workload": ("MobileNetV2 1x1 layers, batch %d, 224x224 images, bf16, %s masks, %d %% "
                                        "irrelevant, kept list given" if mbv2 else
                                        "ResNet-50 1x1 layers of up to 512 input channels, batch %d, 480x640 images "
                                        "(120x160 positions after the stem, halved per stage), bf16, %s masks, %d %% "
                                        "irrelevant, kept list given") % (n, args.mask, round(irr * 100)),
        "launch": "HIP graph replay of four calls", "steps": args.steps, "kept_fraction": round(kept0, 4),
        "layers": rows, "dense_ms": round(tot["dense"][0] * 1e3, 4), "focused_ms": round(t_f * 1e3, 4),
        "chained_ms": round(tot["chained"][0] * 1e3, 4), "speedup_vs_dense": round(tot["dense"][0] / t_f, 3),
        "roofline": {"bound": "hbm", "achieved": round(by_f / t_f / 1e9, 1), "peak": 8000.0, "unit": "GB/s",
                     "frac": round(by_f / t_f / 8e12, 4), "traffic": None, "measured_copy_gbps": copy_gbps},
        "dense_GBps": round(tot["dense"][1] / tot["dense"][0] / 1e9, 1),
        "chained_GBps": round(tot["chained"][1] / tot["chained"][0] / 1e9, 1)}))


def grouped_bench(torch, B, synth, workloads, args):
    """The 3x3 grouped layers of a ResNeXt-50 (32 groups of 4 to 32 channels), bf16, blob masks:
    per layer the focused call (list given) and the dense call, each as a HIP-graph replay of four
    calls.  These layers run on the vector ALUs (fp32 multiply-adds), so the bound quoted is the
    fp32 vector peak; their arithmetic intensity (a few dozen FLOP per byte) puts the memory
    roofline far above what they reach."""
    irr = workloads.HEADLINE_IRRELEVANT if args.irrelevant is None else args.irrelevant
    n = 16 if args.batch is None else args.batch
    dev = torch.device("cuda:0")
    gen = synth.mask_bernoulli if args.mask == "bernoulli" else synth.mask_objects
    rows, t_f, t_d, fl_f, fl_d = [], 0.0, 0.0, 0.0, 0.0
    t_mf = t_md = 0.0
    for li, (c, side) in enumerate(((128, 56), (256, 28), (512, 14), (1024, 7))):
        groups = 32
        x = synth.activations((n, side, side, c), synth.BF16, 8, li, 1)
        w = synth.he_weights(c, 3, 3, c // groups, synth.BF16, 8, li, 2)
        bias = synth.bias(c, 8, li, 3)
        mask = gen(n, side, side, irr, 8, li, 4)
        to_dev = lambda bits: torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
        desc = B.conv_desc(n, side, side, c, c, in_dtype=B.BF16, out_dtype=B.BF16, flags=B.RELU)
        xd, wd, bd, md = to_dev(x), to_dev(w), torch.from_numpy(bias).to(dev), torch.from_numpy(mask).to(dev)
        out = torch.empty((n, side, side, c), dtype=torch.bfloat16, device=dev)
        m_out = B.mask_downsample(md)
        idx, count = B.active_index_compact(m_out)

        def timed(**kw):
            def fn():
                for _ in range(4):
                    B.focused_gconv2d(desc, groups, xd, wd, bd, out=out, **kw)
            return time_loop(torch, capture(torch, fn).replay, args.steps, args.warmup) / 4

        tf = timed(mask_in=md, mask_out=m_out, idx=idx, count=count)
        td = timed()
        # the same layer as a full layer with block-diagonal weights, on the matrix cores
        w_full = B.expand_group_weights(wd, groups, B.BF16)
        ws = B.ready_workspace(torch.empty((B.workspace_bytes(desc),), dtype=torch.uint8, device=dev))
        on_mfma_f = B.PreparedConv(desc, xd, w_full, bd, mask_in=md, mask_out=m_out, idx=idx, count=count, out=out,
                                   workspace=ws, workspace_ready=True)
        on_mfma_d = B.PreparedConv(desc, xd, w_full, bd, out=out, workspace=ws, workspace_ready=True)

        def timed_call(call):
            def fn():
                for _ in range(4):
                    call()
            return time_loop(torch, capture(torch, fn).replay, args.steps, args.warmup) / 4

        tmf, tmd = timed_call(on_mfma_f), timed_call(on_mfma_d)
        per_pos = 2.0 * 9 * (c // groups) * c
        ff, fd = float(np.count_nonzero(mask)) * per_pos, float(mask.size) * per_pos
        rows.append({"layer": "c%d@%d/g%d" % (c, side, groups), "focused_us": round(tf * 1e6, 2),
                     "dense_us": round(td * 1e6, 2), "speedup": round(td / tf, 3),
                     "focused_TFLOPs": round(ff / tf / 1e12, 2), "dense_TFLOPs": round(fd / td / 1e12, 2),
                     "block_diagonal_on_matrix_cores_focused_us": round(tmf * 1e6, 2),
                     "block_diagonal_on_matrix_cores_dense_us": round(tmd * 1e6, 2)})
        t_f, t_d, fl_f, fl_d = t_f + tf, t_d + td, fl_f + ff, fl_d + fd
        t_mf, t_md = t_mf + tmf, t_md + tmd
        del xd, out, on_mfma_f, on_mfma_d
    print(json.dumps({
        "grouped": True, "workload": "ResNeXt-50 (32x4d) 3x3 grouped layers, batch %d, 224x224 images, bf16, %s masks, "
        "%d %% irrelevant" % (n, args.mask, round(irr * 100)), "launch": "HIP graph replay of four calls",
        "steps": args.steps, "layers": rows, "focused_ms": round(t_f * 1e3, 4), "dense_ms": round(t_d * 1e3, 4),
        "speedup_vs_dense": round(t_d / t_f, 3),
        "block_diagonal_on_matrix_cores": {"focused_ms": round(t_mf * 1e3, 4), "dense_ms": round(t_md * 1e3, 4),
                                           "speedup_vs_dense": round(t_md / t_mf, 3)},
        "roofline": {"bound": "alu", "achieved": round(fl_f / t_f / 1e12, 3), "peak": 157.3, "unit": "TFLOP/s",
                     "frac": round(fl_f / t_f / 157.3e12, 4), "traffic": None},
        "dense_TFLOPs": round(fl_d / t_d / 1e12, 2)}))


def masks_bench(torch, B, synth, workloads, args):
    """Mask propagation + ordered compaction at the mask sizes of the workloads, with byte masks and
    with packed masks (one bit per pixel): the mask pyramid (every level's mask and kept list from the
    one input mask, two launches) and the single-level compaction of the first level.  Each figure is
    a HIP-graph replay of four calls; GB/s = algorithmic bytes / time, where the algorithmic bytes are
    the input mask once, every level's mask written once and read once (the list pass), and four
    bytes per kept position."""
    dev = torch.device("cuda:0")
    s1, s2, pool = ((3, 3), (1, 1), (1, 1), (1, 1)), ((3, 3), (2, 2), (1, 1), (1, 1)), ((2, 2), (2, 2), (0, 0), (1, 1))
    cases = [
        ("bench workload: 16 x 128 x 128, four resolutions", 16, 128, 128, [s1, s2, s2, s2], "objects", 0.48),
        ("ResNet-50 bottlenecks: 32 x 120 x 160, four resolutions", 32, 120, 160, [s1, s2, s2, s2], "objects", 0.5),
        ("VGG-16 on HD frames: 8 x 1080 x 1920, five resolutions", 8, 1080, 1920, [s1, pool, pool, pool, pool], "ramp", 0.5),
    ]

    def timed(call):
        def fn():
            for _ in range(4):
                call()
        return time_loop(torch, capture(torch, fn).replay, args.steps, args.warmup) / 4

    rows = []
    for what, n, h, w, steps, kind, irr in cases:
        mask = synth.mask_depth_ramp(n, h, w, irr, 7, 0, 4) if kind == "ramp" else synth.mask_objects(n, h, w, irr, 7, 0, 4)
        md = torch.from_numpy(mask).to(dev)
        bits = B.mask_pack(md)
        m0 = mask.size
        pyr_b = B.PreparedPyramid(md, steps)
        pyr_p = B.PreparedPyramid(md, steps, packed=True)
        pyr_pp = B.PreparedPyramid(bits, steps, packed=True, packed_in=True, shape=(n, h, w))
        levels = pyr_b()
        torch.cuda.synchronize()
        sizes = [lv[0].numel() for lv in levels]
        kept = [int(lv[2].item()) for lv in levels]
        for a_, b_ in zip(pyr_p(), levels):       # same lists either way
            assert torch.equal(a_[1][:int(b_[2].item())], b_[1][:int(b_[2].item())])
        lists = 4 * sum(kept)
        bytes_b = m0 + 2 * sum(sizes) + lists
        bytes_p = m0 + 2 * sum(sizes) / 8 + lists
        bytes_pp = m0 / 8 + 2 * sum(sizes) / 8 + lists
        t_b, t_p, t_pp = timed(pyr_b), timed(pyr_p), timed(pyr_pp)
        # single-level compaction of the first level (labels given), bytes and bits
        idx = torch.empty((sizes[0],), dtype=torch.int32, device=dev)
        cnt = torch.empty((1,), dtype=torch.int32, device=dev)
        ws = torch.empty((B.compact_workspace_bytes(sizes[0]),), dtype=torch.uint8, device=dev)
        lab_b, lab_p = levels[0][0], pyr_p.levels[0][0]
        t_cb = timed(lambda: B.active_index_compact(lab_b, idx, cnt, ws))
        t_cp = timed(lambda: B.active_index_compact_packed(lab_p, sizes[0], idx, cnt, ws))
        t_pack = timed(lambda: B.mask_pack(md, bits))
        c_b, c_p = sizes[0] + 4 * kept[0], sizes[0] / 8 + 4 * kept[0]
        gb = lambda nbytes, t: round(nbytes / t / 1e9, 1)
        rows.append({
            "masks": what, "positions_per_level": sizes, "kept_share": round(kept[0] / sizes[0], 3),
            "pyramid_byte_masks": {"us": round(t_b * 1e6, 2), "algorithmic_MB": round(bytes_b / 1e6, 3), "GBps": gb(bytes_b, t_b)},
            "pyramid_bytes_in_bits_out": {"us": round(t_p * 1e6, 2), "algorithmic_MB": round(bytes_p / 1e6, 3), "GBps": gb(bytes_p, t_p)},
            "pyramid_bits_in_bits_out": {"us": round(t_pp * 1e6, 2), "algorithmic_MB": round(bytes_pp / 1e6, 3), "GBps": gb(bytes_pp, t_pp)},
            "compaction_level0_bytes": {"us": round(t_cb * 1e6, 2), "algorithmic_MB": round(c_b / 1e6, 3), "GBps": gb(c_b, t_cb)},
            "compaction_level0_bits": {"us": round(t_cp * 1e6, 2), "algorithmic_MB": round(c_p / 1e6, 3), "GBps": gb(c_p, t_cp)},
            "pack": {"us": round(t_pack * 1e6, 2), "GBps": gb(m0 * 9 / 8, t_pack)},
        })
        del pyr_b, pyr_p, pyr_pp, levels
    print(json.dumps({"masks_bench": True, "launch": "HIP graph replay of four calls", "steps": args.steps,
                      "hbm_peak_GBps": HBM_PEAK_GBPS, "cases": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--irrelevant", type=float, default=None, help="irrelevant-pixel share (default 0.48)")
    ap.add_argument("--mask", choices=["blobs", "bernoulli"], default="blobs")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-images", type=int, default=16)
    ap.add_argument("--in-dtype", choices=("bf16", "fp8"), default="bf16",
                    help="storage type of activations and weights of the bench line (fp8 = E4M3 bytes, "
                         "outputs bf16; the headline is bf16)")
    ap.add_argument("--out-dtype", choices=("bf16", "fp8"), default="bf16",
                    help="with --in-dtype fp8: store the outputs as E4M3 bytes too")
    ap.add_argument("--roofline-only", action="store_true",
                    help="run only the dominant-kernel loop (for rocprofv3 --kernel-trace --stats)")
    ap.add_argument("--sweep", action="store_true",
                    help="mask-density sweep (irrelevant share 0..1, blob and Bernoulli masks) with a "
                         "linear fit of time against kept share per layer, instead of the bench line")
    ap.add_argument("--stack", choices=sorted(STACKS), default=None,
                    help="time a whole conv stack (dense / focused / focused without zero-fill between "
                         "convs) instead of the bench line")
    ap.add_argument("--pointwise", nargs="?", const="resnet50", default=None, choices=["resnet50", "mobilenetv2"],
                    help="time the 1x1 layers of a ResNet-50 (default) or of a MobileNetV2 at their stages' "
                         "resolutions (dense, focused, chained) and exit")
    ap.add_argument("--depthwise", action="store_true",
                    help="time the depthwise layers of a MobileNetV2 backbone (focused and dense) "
                         "instead of the bench line")
    ap.add_argument("--grouped", action="store_true",
                    help="time the 3x3 grouped layers of a ResNeXt-50 (focused and dense) instead of the bench line")
    ap.add_argument("--masks", action="store_true",
                    help="time mask propagation + compaction (byte masks and packed masks) at the workloads' mask sizes")
    ap.add_argument("--peaks", action="store_true",
                    help="only measure this box's matrix-core and streaming-copy rates (the on-box rooflines)")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: one 256 MiB streaming copy (fc_calibrate_copy: calibrates the "
                         "FETCH_SIZE / WRITE_SIZE counters), then --steps eager steps; no timing")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2207_10741_amd import binding as B, synth, workloads
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    B.lib()

    irr = workloads.HEADLINE_IRRELEVANT if args.irrelevant is None else args.irrelevant
    batch = workloads.SWEEP_BATCH if args.batch is None else args.batch
    if args.peaks:
        out = {"peaks": True}
        for name, code in (("bf16", B.BF16), ("fp8", B.FP8)):
            out[name] = calibrate_peaks(torch, B, code)
        out["issue"] = issue_probe(torch, B)
        print(json.dumps(out))
        return
    if args.masks:
        masks_bench(torch, B, synth, workloads, args)
        return
    if args.sweep:
        sweep(torch, B, synth, workloads, args, batch)
        return
    if args.stack:
        stack_bench(torch, B, synth, workloads, args)
        return
    if args.pointwise:
        pointwise_bench(torch, B, synth, workloads, args)
        return
    if args.depthwise:
        depthwise_bench(torch, B, synth, workloads, args)
        return
    if args.grouped:
        grouped_bench(torch, B, synth, workloads, args)
        return
    in_dtype = B.FP8 if args.in_dtype == "fp8" else B.BF16
    peak = FP8_MFMA_PEAK_TFLOPS if in_dtype == B.FP8 else BF16_MFMA_PEAK_TFLOPS
    if args.out_dtype == "fp8" and in_dtype != B.FP8:
        sys.exit("bench.py: --out-dtype fp8 needs --in-dtype fp8")
    out_dtype = B.FP8 if args.out_dtype == "fp8" else B.BF16
    layers = build_sweep_layers(torch, B, synth, workloads, irr, args.mask, batch, in_dtype, out_dtype)

    # The four shapes are the four resolutions of one network, so they see ONE mask, rescaled
    # (Sec. III-B): the mask of the first layer, subsampled by two per resolution change.
    mask0 = layers[0]["host"][3]
    for li, L in enumerate(layers):
        mh = np.ascontiguousarray(mask0[:, ::1 << li, ::1 << li])
        assert mh.shape == (batch, L["side"], L["side"])
        L["mask"] = torch.from_numpy(mh).to("cuda:0")
        L["host"] = L["host"][:3] + (mh,)
        L["kept"] = int(np.count_nonzero(mh))
        L["flops_kept"] = 2.0 * L["kept"] * L["k"] * L["c"]
    # ... which the library builds, with all kept lists, from the first mask in two launches:
    # the layer's own window, then three stride-2 3x3 windows
    pyramid = B.PreparedPyramid(layers[0]["mask"], [((3, 3), (1, 1), (1, 1), (1, 1))] +
                                [((3, 3), (2, 2), (1, 1), (1, 1))] * (len(layers) - 1))
    for L, (m_out, idx, count) in zip(layers, pyramid()):
        assert torch.equal(m_out != 0, L["mask"] != 0) and int(count.item()) == L["kept"]
        L["m_out"], L["idx"], L["count"] = m_out, idx, count

    # ---- the whole hot path: a1 + a2 + a3..a6 for every layer ------------------
    for L in layers:
        d = L["desc"]
        L["call_focused"] = B.PreparedConv(d, L["x"], L["w"], L["bias"], mask_in=L["mask"], out=L["out"],
                                           workspace=L["ws"], workspace_ready=True)
        L["call_dense"] = B.PreparedConv(d, L["x"], L["w"], L["bias"], out=L["out"], workspace=L["ws"], workspace_ready=True)
        L["call_conv_only"] = B.PreparedConv(d, L["x"], L["w"], L["bias"], mask_in=L["mask"], mask_out=L["m_out"],
                                             idx=L["idx"], count=L["count"], out=L["out"], workspace=L["ws"], workspace_ready=True)
        dk = B.conv_desc(batch, L["side"], L["side"], L["c"], L["c"], in_dtype=in_dtype, out_dtype=out_dtype,
                         flags=B.RELU | B.SKIP_ZERO_FILL)
        L["call_kernel"] = B.PreparedConv(dk, L["x"], L["w"], L["bias"], mask_in=L["mask"], mask_out=L["m_out"],
                                          idx=L["idx"], count=L["count"], out=L["out"], workspace=L["ws"], workspace_ready=True)

    if args.traffic_probe:
        src = torch.ones((64 << 20,), dtype=torch.int32, device="cuda:0")   # 256 MiB
        dst = torch.empty_like(src)
        B.calibrate_copy(src, dst)               # k_calibrate_copy: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        for _ in range(args.steps):
            for L in layers:
                L["call_conv_only"]()        # the launch the step makes: kept list given, zero-fill included
            torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": True, "copy_bytes_each_way": src.numel() * 4, "steps": args.steps,
                          "kernel_source_hash": kernel_source_hash(),
                          "kept_rows": {L["name"]: L["kept"] for L in layers}}))
        return

    def step_of(key):
        if key == "whole":          # mask pyramid (a1 + a2 for all four layers), then the four layers
            calls = [pyramid] + [L["call_conv_only"] for L in layers]
        else:
            calls = [L[key] for L in layers]

        def step():
            for c in calls:
                c()
        return step

    # A step takes about 0.1 ms, so a short --steps would time a couple of milliseconds: every timed
    # "step" is `inner` replays of the step's graph (stated in the line), at least 100 replays in all.
    inner = max(1, -(-100 // max(1, args.steps)))
    timings = {}
    for key in (() if args.roofline_only else ("whole", "call_focused", "call_dense", "call_conv_only")):
        step = step_of(key)
        timings[key + "_eager"] = time_loop(torch, step, args.steps, args.warmup)
        graph = capture(torch, step)
        timings[key] = time_loop(torch, graph.replay, args.steps * inner, args.warmup)
    if not args.roofline_only:
        t_focused, t_dense, t_conv_only = (timings[k] for k in ("whole", "call_dense", "call_conv_only"))
        # spread of the focused step: ten chunks of at least 20 replays each (a second pass)
        graph = capture(torch, step_of("whole"))
        chunk = max(20, args.steps * inner // 10)
        chunks = sorted(time_loop(torch, graph.replay, chunk, 0) for _ in range(10))
        t_min, t_median = chunks[0], 0.5 * (chunks[4] + chunks[5])
        # the same step with the activations coming from HBM: the four layers' tensors of one
        # set are 126 MB and stay in the 256 MB memory-side cache between replays, so rotate
        # through four sets (503 MB)
        sets = 4
        cold_calls = []
        for k in range(sets):
            cold_calls.append(pyramid)
            for L in layers:
                xk = L["x"] if k == 0 else L["x"].clone()
                ok = L["out"] if k == 0 else torch.empty_like(L["out"])
                cold_calls.append(B.PreparedConv(L["desc"], xk, L["w"], L["bias"], mask_in=L["mask"],
                                                 mask_out=L["m_out"], idx=L["idx"], count=L["count"], out=ok,
                                                 workspace=L["ws"], workspace_ready=True))

        def cold_step():
            for c in cold_calls:
                c()
        graph = capture(torch, cold_step)
        t_cold = time_loop(torch, graph.replay, max(1, args.steps // sets), max(1, args.warmup // sets)) / sets
        del graph, cold_calls

    # ---- dominant kernel: the matrix-core conv kernel exactly as the step launches it (kept
    # list given, zero-fill of the irrelevant rows in the same launch), one launch per call,
    # timed with events on the stream it is launched on -----------------------------
    per_layer_ms = []
    for L in layers:
        call = L["call_conv_only"]
        for _ in range(args.warmup):
            call()
        # events bracket runs of 10 back-to-back launches of this one kernel, so that the
        # cost of the event records themselves is spread thin
        burst = 10
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(max(10, args.steps // burst))]
        for a, b in evs:
            a.record()
            for _ in range(burst):
                call()
            b.record()
        torch.cuda.synchronize()
        per_layer_ms.append(float(np.mean([a.elapsed_time(b) for a, b in evs])) / burst)
    if args.roofline_only:
        # the same launches without the zero-fill of the irrelevant rows (what a chained layer runs)
        skip_ms = []
        for L in layers:
            call = L["call_kernel"]
            for _ in range(args.warmup):
                call()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
            for a, b in evs:
                a.record()
                for _ in range(10):
                    call()
                b.record()
            torch.cuda.synchronize()
            skip_ms.append(float(np.mean([a.elapsed_time(b) for a, b in evs])) / 10)
    flops_kept = sum(L["flops_kept"] for L in layers)
    kern_avg_s = sum(per_layer_ms) / 1e3 / len(layers)
    achieved = (flops_kept / len(layers)) / kern_avg_s / 1e12
    default_workload = (args.irrelevant is None and args.mask == "blobs" and args.batch is None and
                        in_dtype == B.BF16 and out_dtype == B.BF16)
    # algorithmic HBM bytes of a launch: input mask (gate and labels) + labels + the kept list once +
    # every needed input pixel once (for these 3x3 unit-stride layers: the relevant pixels) + weights
    # and bias once + every output row once (kept rows and zero-filled rows)
    e_in, e_out = (1 if in_dtype == B.FP8 else 2), (1 if out_dtype == B.FP8 else 2)
    algo_bytes = sum(2 * L["m"] + 4 * L["kept"] + L["kept"] * L["c"] * e_in + L["k"] * L["c"] * e_in + 4 * L["c"] +
                     L["m"] * L["c"] * e_out for L in layers) / len(layers)
    traffic, traffic_note = measured_traffic() if default_workload else (None, "not the workload of the counter summary")
    peaks = calibrate_peaks(torch, B, in_dtype)
    roofline = {
        "bound": "mfma", "kernel": "k_conv_dma / k_conv_line (one launch per layer, zero-fill included)",
        "achieved": round(achieved, 3), "peak": peak,
        "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
        "traffic": traffic, "traffic_source": traffic_note,
        "algorithmic_bytes_per_launch": round(algo_bytes),
        "traffic_over_algorithmic": None if traffic is None else round(traffic / algo_bytes, 3),
        "avg_launch_us": round(kern_avg_s * 1e6, 3),
        "flops_per_launch": round(flops_kept / len(layers)),
        "measured_peak": peaks["mfma_tflops"], "frac_of_measured_peak": round(achieved / peaks["mfma_tflops"], 4),
        "measured_copy_gbps": peaks["copy_gbps"], "peaks_how": peaks["how"],
    }
    if args.roofline_only:
        print(json.dumps({"roofline": roofline,
                          "per_layer_conv_kernel_ms": {L["name"]: round(ms, 5) for L, ms in zip(layers, per_layer_ms)},
                          "per_layer_without_zero_fill_ms": {L["name"]: round(ms, 5) for L, ms in zip(layers, skip_ms)}}))
        return

    value = flops_kept / t_focused / 1e12
    result = {
        "metric": METRIC,
        "value": round(value, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(t_focused * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": args.in_dtype,
        "data": "synthetic",
        "config": {
            "workload": ("" if in_dtype == B.BF16 else "E4M3 storage, %s outputs: " % ("E4M3" if out_dtype == B.FP8 else "bf16")) +
                        "ResNet-50 3x3 layer shapes (C64@128, C128@64, C256@32, C512@16), batch %d, "
                        "one %s mask per image with %.0f %% irrelevant, rescaled to the four resolutions; step = "
                        "mask pyramid (propagation + compaction for all four layers, two launches) + focused "
                        "conv + zero-fill per layer" % (batch, args.mask, 100 * irr),
            "batch": batch, "irrelevant": irr, "mask": args.mask,
            "kept_fraction": round(sum(L["kept"] for L in layers) / sum(L["m"] for L in layers), 4),
        },
        "launch": "one HIP graph replay per step",
        "replays_per_timed_step": inner, "timed_replays": args.steps * inner,
        "ms_per_step_min": round(t_min * 1e3, 4), "ms_per_step_median": round(t_median * 1e3, 4),
        "cold_ms_per_step": round(t_cold * 1e3, 4),
        "eager_ms_per_step": round(timings["whole_eager"] * 1e3, 4),
        "per_call_ms_per_step": round(timings["call_focused"] * 1e3, 4),
        "speedup_vs_dense": round(t_dense / t_focused, 3),
        "dense_ms_per_step": round(t_dense * 1e3, 4),
        "dense_tflops": round(sum(L["flops_dense"] for L in layers) / t_dense / 1e12, 3),
        "conv_only_ms_per_step": round(t_conv_only * 1e3, 4),
        "conv_only_tflops": round(flops_kept / t_conv_only / 1e12, 3),
        "ms_per_image": round(t_focused * 1e3 / batch, 6),
        "per_layer_conv_kernel_ms": {L["name"]: round(ms, 5) for L, ms in zip(layers, per_layer_ms)},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        v, cores, secs = cpu_baseline(layers, min(args.cpu_images, batch))
        result["cpu_baseline"] = {
            "value": round(v, 6), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": "%d of the %d images of each of the four layers, same masks, %.1f s" % (
                min(args.cpu_images, batch), batch, secs),
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
