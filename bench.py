#!/usr/bin/env python3
"""Benchmark of the COMET activation codec on one MI355X.

A step = one pass of the whole hot path over the ResNet-50-shaped activation set
(batch 64, five fp32 post-BN-ReLU tensors, 590.9 MB): compress every layer in
forward order, keep the five containers, decompress them in reverse order.
Inputs are resident in HBM before the timed region; all ten calls are enqueued
asynchronously (the layers are dealt to --streams contexts, each on a stream of
its own) and the region ends with a device synchronisation.

Prints ONE JSON line: round-trip throughput in GB/s of fp32 input, the roofline
figures of the dominant kernel (per-kernel durations from HIP events recorded by
the library on its own stream) and the CPU oracle timed on the same data.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_resnet50_set_batch64.txt")


def traffic_from_profiles():
    """HBM bytes per mean launch of every kernel, from the rocprofv3 counter summary under profiles/
    (FETCH_SIZE + WRITE_SIZE, scaled by the same counters on a plain copy of known size): the lines
    `TRAFFIC <kernel> <bytes>` of that file.  Empty if the file is missing."""
    out = {}
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                w = line.split()
                if len(w) == 3 and w[0] == "TRAFFIC":
                    out[w[1]] = int(w[2])
    except OSError:
        pass
    return out


def valu_issue_from_profiles():
    """Share of the vector-ALU issue slots each kernel uses (rocprofv3 SQ counters): the lines
    `VALU_ISSUE <kernel> <fraction>` of the counter summary under profiles/."""
    out = {}
    try:
        with open(os.path.join(ROOT, "profiles", "sq_counters_resnet50_set_batch64.txt")) as f:
            for line in f:
                w = line.split()
                if len(w) == 3 and w[0] == "VALU_ISSUE":
                    out[w[1]] = float(w[2])
    except OSError:
        pass
    return out


def other_configs(comet, synth, torch, np, chunk_syms, reps=5):
    """Throughput and ratio of the configurations that are not the headline workload: config 0, the VGG-16-shaped
    set (config 2), the error-bound sweep (config 3, primary curve) and the two large tensors of config 4, each
    alone and with one stream compressing while the other decompresses.  One context, one call at a time
    (median of `reps`), except where config 4 overlaps two."""
    def med(fn, sync, n=reps):
        ts = []
        for _ in range(n):
            sync()
            t = time.perf_counter()
            fn()
            sync()
            ts.append(time.perf_counter() - t)
        return sorted(ts)[len(ts) // 2]

    def cell(ctx, xd, e, cont, out):
        used = ctx.comet_compress(xd, e["eb"], e["nbins"], cont)
        ctx.comet_decompress(cont, used, xd.shape, out)
        ctx.comet_sync()
        tc = med(lambda: ctx.comet_compress(xd, e["eb"], e["nbins"], cont, sync=False), torch.cuda.synchronize)
        td = med(lambda: ctx.comet_decompress(cont, used, xd.shape, out), torch.cuda.synchronize)
        ctx.comet_sync()
        n = xd.numel()
        b = used / n
        return dict(elements=n, container_bytes=used, ratio=round(4 * n / used, 3), compress_GBps=round(4 * n / tc / 1e9, 1), decompress_GBps=round(4 * n / td / 1e9, 1),
                    roundtrip_GBps=round(4 * n / (tc + td) / 1e9, 1),
                    compress_frac_hbm_two_pass_floor=round((8 + b) * n / tc / 1e9 / HBM_PEAK_GBS, 4),
                    decompress_frac_hbm_fused_floor=round((4 + b) * n / td / 1e9 / HBM_PEAK_GBS, 4))

    res = {}
    # config 0 and config 2: per set, the sums over its tensors
    for name, entries in (("config0", synth.config0()), ("config2_vgg16_batch32", synth.config2(32))):
        ctx = comet.Context(max(int(np.prod(e["shape"])) for e in entries), max(e["nbins"] for e in entries))
        ctx.comet_set_chunk_syms(chunk_syms)
        cells = []
        for e in entries:
            xd = torch.from_numpy(synth.make(e)).cuda()
            cont = torch.empty(comet.comet_compress_bound(xd.shape, e["nbins"], chunk_syms), dtype=torch.uint8, device="cuda")
            out = torch.empty_like(xd)
            cells.append(cell(ctx, xd, e, cont, out))
            del xd, cont, out
        ctx.close()
        n = sum(c["elements"] for c in cells)
        tc = sum(4 * c["elements"] / c["compress_GBps"] for c in cells)
        td = sum(4 * c["elements"] / c["decompress_GBps"] for c in cells)
        used = sum(c["container_bytes"] for c in cells)
        b = used / n
        res[name] = dict(eb=entries[0]["eb"], nbins=entries[0]["nbins"], elements=n, ratio=round(4 * n / used, 3),
                         compress_GBps=round(4 * n / tc, 1), decompress_GBps=round(4 * n / td, 1), roundtrip_GBps=round(4 * n / (tc + td), 1),
                         compress_frac_hbm_two_pass_floor=round((8 + b) * n / tc / HBM_PEAK_GBS, 4),
                         decompress_frac_hbm_fused_floor=round((4 + b) * n / td / HBM_PEAK_GBS, 4),
                         per_layer_ratio=[c["ratio"] for c in cells])
    # zero chunks (container version 2) on the headline set (55 % zeros) and on sparser ones (the same recipe with the
    # shift before the ReLU at -1.0, -2.0, -2.5: 84 %, 98 %, 99 % zeros)
    zc = {}
    for name, shift in (("resnet50_set_batch64", -0.2), ("resnet50_set_batch64_zeros84", -1.0), ("resnet50_set_batch64_zeros98", -2.0),
                        ("resnet50_set_batch64_zeros99", -2.5)):
        entries = [dict(e, shift=shift) for e in synth.config1(64)]
        ctx = comet.Context(max(int(np.prod(e["shape"])) for e in entries), 1024)
        ctx.comet_set_chunk_syms(chunk_syms)
        tot = {}
        for e in entries:
            xd = torch.from_numpy(synth.make(e)).cuda()
            cont = torch.empty(comet.comet_compress_bound(xd.shape, e["nbins"], chunk_syms), dtype=torch.uint8, device="cuda")
            out = torch.empty_like(xd)
            for v, on in (("v1", False), ("v2", True)):
                ctx.comet_set_zero_chunks(on)
                r = cell(ctx, xd, e, cont, out)
                t = tot.setdefault(v, dict(bytes=0, n=0, tc=0.0, td=0.0))
                t["bytes"] += r["container_bytes"]; t["n"] += r["elements"]
                t["tc"] += 4 * r["elements"] / r["compress_GBps"]; t["td"] += 4 * r["elements"] / r["decompress_GBps"]
            del xd, cont, out
        ctx.close()
        zc[name] = {v: dict(ratio=round(4 * t["n"] / t["bytes"], 3), compress_GBps=round(4 * t["n"] / t["tc"], 1),
                            decompress_GBps=round(4 * t["n"] / t["td"], 1)) for v, t in tot.items()}
    res["zero_chunks"] = zc
    # config 3: one tensor, seven error bounds with their alphabets
    entries = synth.config3(64)
    xd = torch.from_numpy(synth.make(entries[0])).cuda()
    ctx = comet.Context(xd.numel(), 65536)
    ctx.comet_set_chunk_syms(chunk_syms)
    cont = torch.empty(comet.comet_compress_bound(xd.shape, 65536, chunk_syms), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(xd)
    res["config3_eb_sweep"] = [dict(eb=float(f"{e['eb']:.3g}"), nbins=e["nbins"], **{k: v for k, v in cell(ctx, xd, e, cont, out).items() if k not in ("elements", "container_bytes")})
                               for e in entries]
    ctx.close()
    del xd, cont, out
    # config 4: two large tensors, each alone, then one being compressed while the other is decompressed
    entries = synth.config4()
    n = int(np.prod(entries[0]["shape"]))
    ctxs = [comet.Context(n, entries[0]["nbins"]) for _ in entries]
    for c in ctxs:
        c.comet_set_chunk_syms(chunk_syms)
    sts = [torch.cuda.Stream(), torch.cuda.Stream()]
    xds, conts, outs, used, alone = [], [], [], [], []
    for i, e in enumerate(entries):
        xd = torch.from_numpy(synth.make(e)).cuda()
        cont = torch.empty(comet.comet_compress_bound(xd.shape, e["nbins"], chunk_syms), dtype=torch.uint8, device="cuda")
        out = torch.empty_like(xd)
        alone.append(cell(ctxs[i], xd, e, cont, out))
        used.append(alone[-1]["container_bytes"])
        xds.append(xd); conts.append(cont); outs.append(out)

    def both():
        ctxs[0].comet_compress(xds[0], entries[0]["eb"], entries[0]["nbins"], conts[0], stream=sts[0], sync=False)
        ctxs[1].comet_decompress(conts[1], used[1], xds[1].shape, outs[1], stream=sts[1])
    t_both = med(both, torch.cuda.synchronize)
    for c, st in zip(ctxs, sts):
        c.comet_sync(st)
        c.close()
    t_sum = 4 * n / alone[0]["compress_GBps"] / 1e9 + 4 * n / alone[1]["decompress_GBps"] / 1e9
    res["config4_two_tensors"] = dict(eb=entries[0]["eb"], nbins=entries[0]["nbins"], alone=alone,
                                      overlapped=dict(ms=round(t_both * 1e3, 3), GBps_of_input=round(8 * n / t_both / 1e9, 1),
                                                      one_after_the_other_ms=round(t_sum * 1e3, 3)))
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=64, help="batch of the activation set (64 = the metric's workload)")
    ap.add_argument("--chunk-syms", type=int, default=64)
    ap.add_argument("--streams", type=int, default=5,
                    help="contexts (each on its own stream) the layers are dealt to; the single-workgroup kernels of "
                         "one layer then overlap the streaming kernels of another")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--overlap-conv", action="store_true",
                    help="also time the step next to fp32 3x3 convolutions of the five layers on a stream of their own "
                         "(the paper's future work: hiding the codec behind the layers' compute); adds path.overlap_with_conv")
    ap.add_argument("--per-layer", action="store_true", help="also print a per-layer table to stderr")
    ap.add_argument("--no-split", action="store_true", help="skip the compress-only and decompress-only passes")
    ap.add_argument("--no-configs", action="store_true", help="skip the other configurations (path.configs)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="first run one plain device-to-device copy of the largest layer (a kernel of known traffic "
                         "that hardware-counter runs are scaled by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the codec shards with zero exchange (every GPU compresses its own batch "
              "shard), so --gpus above 1 is not run here.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2111_09562_amd import comet, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    layers = synth.config1(args.batch)
    t0 = time.time()
    xs_host = [synth.make(e) for e in layers]
    gen_s = time.time() - t0
    xs = [torch.from_numpy(x).cuda() for x in xs_host]
    n_total = sum(x.numel() for x in xs)
    in_bytes = 4 * n_total

    if args.copy_probe:
        probe = torch.empty_like(xs[0])
        probe.copy_(xs[0])
        torch.cuda.synchronize()
        print(f"copy probe: {xs[0].numel() * 4} bytes read, {xs[0].numel() * 4} bytes written", file=sys.stderr)
        del probe

    n_ctx = max(1, min(args.streams, len(xs)))
    ctxs = [comet.Context(max_elems=max(x.numel() for x in xs), max_nbins=1024) for _ in range(n_ctx)]
    for c in ctxs:
        c.comet_set_chunk_syms(args.chunk_syms)
    # context 0 runs on torch's current stream, the others on streams of their own (default priority)
    streams = [torch.cuda.current_stream()] + [torch.cuda.Stream() for _ in range(n_ctx - 1)]
    owner = [i % n_ctx for i in range(len(xs))]            # layer -> context / stream
    # containers: 60 % of the input is ample for these tensors; a low ratio would raise COMET_ERR_CAPACITY
    conts = [torch.empty(int(x.numel() * 4 * 0.6) // 16 * 16, dtype=torch.uint8, device="cuda") for x in xs]
    outs = [torch.empty_like(x) for x in xs]

    def compress_all():
        for i, (x, e, c) in enumerate(zip(xs, layers, conts)):
            ctxs[owner[i]].comet_compress(x, e["eb"], e["nbins"], c, stream=streams[owner[i]], sync=False)

    def decompress_all():
        for i in reversed(range(len(xs))):
            ctxs[owner[i]].comet_decompress(conts[i], conts[i].numel(), xs[i].shape, outs[i], stream=streams[owner[i]])

    def sync_all():
        for c, st in zip(ctxs, streams):
            c.comet_sync(st)

    def step():
        compress_all()
        decompress_all()

    for _ in range(args.warmup):
        step()
    sync_all()
    sizes = [int(ctxs[0].comet_peek(c, c.numel()).total_bytes) for c in conts]

    # ---- the timed region: exactly K steps ----
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    sync_all()                                     # raises if any call of the region reported an error
    ms_per_step = dt / args.steps * 1e3
    value = in_bytes / (dt / args.steps) / 1e9

    # compress-only and decompress-only rates (same launch configuration)
    tc = td = tr = t16 = None
    if not args.no_split:
        def timed(fn):
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t) / args.steps
        tc = timed(compress_all)
        td = timed(decompress_all)
        sync_all()
        # code book reuse: the same compression with the length tables of the containers just written (copied out,
        # a table may not lie inside the buffer that is being written); same tensors, so the containers must not change
        tables = [c[comet.HEADER_BYTES: comet.HEADER_BYTES + e["nbins"]].clone() for c, e in zip(conts, layers)]

        def compress_reuse_all():
            for i, (x, e, c) in enumerate(zip(xs, layers, conts)):
                ctxs[owner[i]].comet_compress_with_codebook(x, e["eb"], e["nbins"], tables[i], c, stream=streams[owner[i]], sync=False)
        compress_reuse_all()
        sync_all()
        tr = timed(compress_reuse_all)
        sync_all()
        assert [int(ctxs[0].comet_peek(c, c.numel()).total_bytes) for c in conts] == sizes, "code book reuse changed a container"
        # 16-bit activations: the same step on the set rounded to bfloat16 (half the input and output bytes)
        xs16 = [x.to(torch.bfloat16) for x in xs]
        outs16 = [torch.empty_like(x) for x in xs16]

        def step16():
            for i, (x, e, c) in enumerate(zip(xs16, layers, conts)):
                ctxs[owner[i]].comet_compress_16(x, e["eb"], e["nbins"], c, stream=streams[owner[i]], sync=False)
            for i in reversed(range(len(xs16))):
                ctxs[owner[i]].comet_decompress_16(conts[i], conts[i].numel(), xs16[i].shape, outs16[i], stream=streams[owner[i]])
        step16()
        sync_all()
        t16 = timed(step16)
        sync_all()
        del xs16, outs16

    # ---- optional: the codec next to convolutions (one more stream, default priority) ----
    overlap = None
    if args.overlap_conv:
        import torch.nn.functional as F
        conv_stream = torch.cuda.Stream()
        ws = [torch.randn(x.shape[1], x.shape[1], 3, 3, device="cuda") * 0.05 for x in xs]

        def convs():
            with torch.cuda.stream(conv_stream):
                for x, w in zip(xs, ws):
                    F.conv2d(x, w, padding=1)

        def timed_pair(f, g, reps):
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(reps):
                if f:
                    f()
                if g:
                    g()
            torch.cuda.synchronize()
            return (time.perf_counter() - t) / reps
        convs(); torch.cuda.synchronize()                     # algorithm selection happens here
        reps = max(3, args.steps // 2)
        t_conv = timed_pair(convs, None, reps)
        t_codec = timed_pair(None, step, reps)
        t_both = timed_pair(convs, step, reps)
        overlap = dict(conv_ms=round(t_conv * 1e3, 3), codec_ms=round(t_codec * 1e3, 3), both_ms=round(t_both * 1e3, 3),
                       hidden_frac_of_codec=round((t_conv + t_codec - t_both) / t_codec, 3),
                       note="five fp32 3x3 convolutions (C -> C, padding 1) of the layers' shapes on one stream, the codec "
                            "step on its streams; hidden = (conv + codec - both) / codec")

    # ---- per-kernel durations: K more steps with the library bracketing every launch with two HIP events on
    # the launch's stream.  This pass runs one call at a time (a synchronisation after each), so that a
    # kernel has the chip to itself and its duration says something about the kernel; the timed region above
    # runs without brackets and with the layers overlapped ----
    for c in ctxs:
        c.comet_profile_enable(True)
        c.comet_profile_reset()
    for _ in range(args.steps):
        for i, (x, e, c) in enumerate(zip(xs, layers, conts)):
            ctxs[owner[i]].comet_compress(x, e["eb"], e["nbins"], c, stream=streams[owner[i]], sync=False)
            torch.cuda.synchronize()
        for i in reversed(range(len(xs))):
            ctxs[owner[i]].comet_decompress(conts[i], conts[i].numel(), xs[i].shape, outs[i], stream=streams[owner[i]])
            torch.cuda.synchronize()
    sync_all()
    kern = {}
    for kid, name in enumerate(comet.KERNEL_NAMES):
        launches, ms = 0, 0.0
        for c in ctxs:
            l, m = c.comet_profile_read(kid)
            launches += l
            ms += m
        kern[name] = dict(launches=launches, total_ms=ms, avg_us=(ms / launches * 1e3 if launches else 0.0))
    for c in ctxs:
        c.comet_profile_enable(False)

    # the same step with every call on one stream (what a training loop that compresses a layer while the next
    # one computes sees: the single-workgroup kernels of a layer are then on the step's critical path)
    def step_one_stream():
        for x, e, c in zip(xs, layers, conts):
            ctxs[0].comet_compress(x, e["eb"], e["nbins"], c, stream=streams[0], sync=False)
        for i in reversed(range(len(xs))):
            ctxs[0].comet_decompress(conts[i], conts[i].numel(), xs[i].shape, outs[i], stream=streams[0])
    step_one_stream()
    torch.cuda.synchronize()
    t1s = time.perf_counter()
    for _ in range(args.steps):
        step_one_stream()
    torch.cuda.synchronize()
    one_stream_s = (time.perf_counter() - t1s) / args.steps
    ctxs[0].comet_sync(streams[0])

    cont_bytes = sum(sizes)
    b = cont_bytes / n_total                       # container bytes per element
    # algorithmic bytes per element of each streaming kernel (what its interface makes it read + write):
    # quantise: fp32 in, u16 code out; encode: codes in (count pass), codes in and container out (pack pass);
    # decode: container in, int16 residual out; scan + store: int16 in, fp32 out
    alg = {"k_quantize_rows": 4.0 + 2.0, "k_encode_count": 2.0, "k_encode_pack": 2.0 + b, "k_decode_chunks": b + 2.0,
           "k_scan_store": 2.0 + 4.0, "k_decode_scan": b + 4.0}
    traffic = traffic_from_profiles()
    dom = max(alg.keys(), key=lambda k: kern[k]["total_ms"])
    launches = kern[dom]["launches"]
    # every launch of a kernel handles one layer; the five layers differ in size, so
    # "per launch" is the mean over the set: bytes of the set / 5 per mean launch time
    alg_bytes_per_launch = alg[dom] * n_total / len(xs)
    avg_s = kern[dom]["total_ms"] / launches / 1e3
    achieved = alg_bytes_per_launch / avg_s / 1e9
    roofline = dict(bound="hbm", kernel=dom, achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(achieved / HBM_PEAK_GBS, 4), traffic=traffic.get(dom), valu_issue=valu_issue_from_profiles().get(dom),
                    avg_launch_us=round(avg_s * 1e6, 2), launches=launches,
                    alg_bytes_per_elem=round(alg[dom], 4),
                    note="mean over the five layers of the set; durations from HIP events recorded by the library on "
                         "the stream of each launch, in a pass of K more steps after the timed region in which the "
                         "calls run one at a time (in the timed region the layers overlap on several streams and a "
                         "kernel shares the chip, so its duration there measures the mix, not the kernel); traffic = "
                         "HBM bytes per mean launch from rocprofv3 FETCH_SIZE + WRITE_SIZE scaled by a copy of known "
                         "size (profiles/hbm_traffic_resnet50_set_batch64.txt)")
    # path-level figures: bytes the kernels of a path move per element (compress: 6 + 4 + b, decompress in one
    # kernel: b + 4), the floors of the method (two passes to compress: 8 + b; b + 4 to decompress) and the
    # smallest any codec could move (4 + b each way)
    step_s = dt / args.steps
    path = dict(ratio=round(in_bytes / cont_bytes, 3),
                per_layer_ratio=[round(4 * x.numel() / s, 3) for x, s in zip(xs, sizes)],
                roundtrip_frac_hbm_kernel_bytes=round((14.0 + 2 * b) * n_total / step_s / 1e9 / HBM_PEAK_GBS, 4),
                roundtrip_frac_hbm_method_floor=round((12.0 + 2 * b) * n_total / step_s / 1e9 / HBM_PEAK_GBS, 4),
                roundtrip_frac_hbm_min_bytes=round((8.0 + 2 * b) * n_total / step_s / 1e9 / HBM_PEAK_GBS, 4),
                one_stream=dict(ms_per_step=round(one_stream_s * 1e3, 4), GBps=round(in_bytes / one_stream_s / 1e9, 1),
                                note="every call of the step on one stream, nothing overlaps"),
                kernels={k: dict(launches=v["launches"], avg_us=round(v["avg_us"], 2)) for k, v in kern.items()},
                # the same roofline arithmetic for every streaming kernel (mean launch, algorithmic bytes / duration)
                kernel_frac_hbm={k: round(alg[k] * n_total / len(xs) / (kern[k]["total_ms"] / kern[k]["launches"] / 1e3) / 1e9
                                          / HBM_PEAK_GBS, 4) for k in alg if kern[k]["launches"]})
    if overlap is not None:
        path["overlap_with_conv"] = overlap
    if tc is not None:
        path.update(compress_GBps=round(in_bytes / tc / 1e9, 1), decompress_GBps=round(in_bytes / td / 1e9, 1),
                    compress_with_codebook_GBps=round(in_bytes / tr / 1e9, 1),
                    bf16_roundtrip_Gelem_per_s=round(n_total / t16 / 1e9, 2), fp32_roundtrip_Gelem_per_s=round(n_total / (dt / args.steps) / 1e9, 2),
                    compress_frac_hbm_kernel_bytes=round((10.0 + b) * n_total / tc / 1e9 / HBM_PEAK_GBS, 4),
                    decompress_frac_hbm_kernel_bytes=round((4.0 + b) * n_total / td / 1e9 / HBM_PEAK_GBS, 4),
                    # floors of the method itself: two passes over the data to compress (8 + b bytes per element),
                    # a fused decode + reconstruction to decompress (b + 4), and what a codec with a known code book
                    # could reach (4 + b)
                    compress_frac_hbm_two_pass_floor=round((8.0 + b) * n_total / tc / 1e9 / HBM_PEAK_GBS, 4),
                    decompress_frac_hbm_fused_floor=round((4.0 + b) * n_total / td / 1e9 / HBM_PEAK_GBS, 4),
                    compress_frac_hbm_ideal_floor=round((4.0 + b) * n_total / tc / 1e9 / HBM_PEAK_GBS, 4))
        # what a plain device-to-device copy of the largest layer reaches in this run (read + write bytes)
        big = max(range(len(xs)), key=lambda i: xs[i].numel())

        def copy_big():
            outs[big].copy_(xs[big])
        copy_big()
        t_copy = timed(copy_big)
        copy_gbs = 8.0 * xs[big].numel() / t_copy / 1e9
        path.update(copy_ceiling_GBps=round(copy_gbs, 1),
                    roundtrip_frac_copy_ceiling_kernel_bytes=round((14.0 + 2 * b) * n_total / step_s / 1e9 / copy_gbs, 4),
                    roundtrip_frac_copy_ceiling_min_bytes=round((8.0 + 2 * b) * n_total / step_s / 1e9 / copy_gbs, 4))
    prop = torch.cuda.get_device_properties(0)
    path["device"] = dict(name=prop.name, compute_units=prop.multi_processor_count, memory_GB=round(prop.total_memory / 2**30, 1),
                          l2_MB_per_xcd=round(getattr(prop, "L2_cache_size", 0) / 2**20, 1))

    cpu = None
    if not args.no_cpu_baseline:
        from concurrent.futures import ThreadPoolExecutor

        from oracle import comet_oracle as oracle
        t0 = time.perf_counter()
        bufs = [oracle.compress(x, e["eb"], e["nbins"], args.chunk_syms) for x, e in zip(xs_host, layers)]
        t1 = time.perf_counter()
        for bf in reversed(bufs):
            oracle.decompress(bf)
        t2 = time.perf_counter()
        assert [len(bf) for bf in bufs] == sizes, "GPU and oracle container sizes differ"
        for bf, c in zip(bufs, conts):                 # the containers of the last step, byte for byte
            assert np.array_equal(c[:len(bf)].cpu().numpy(), bf), "a GPU container differs from the oracle's"
        # secondary: every host core at once, each on a slice of the batch as a tensor of its own (throughput only:
        # such containers differ from those of the whole tensors)
        cores = max(1, min(os.cpu_count() or 1, 16))
        slices = []
        for x, e in zip(xs_host, layers):
            per = max(1, x.shape[0] // cores)
            slices += [(np.ascontiguousarray(x[i:i + per]), e) for i in range(0, x.shape[0], per)]

        def one(job):
            xx, e = job
            oracle.decompress(oracle.compress(xx, e["eb"], e["nbins"], args.chunk_syms))
        t3 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=cores) as pool:
            list(pool.map(one, slices))
        t4 = time.perf_counter()
        cpu = dict(value=round(in_bytes / (t2 - t0) / 1e9, 4), unit="GB/s", cores=1, kind="oracle",
                   sample=f"the whole set once ({in_bytes / 1e6:.1f} MB): compress {t1 - t0:.1f} s, decompress {t2 - t1:.1f} s; "
                          "its containers equal the GPU's byte for byte",
                   compress_GBps=round(in_bytes / (t1 - t0) / 1e9, 4), decompress_GBps=round(in_bytes / (t2 - t1) / 1e9, 4),
                   all_cores=dict(value=round(in_bytes / (t4 - t3) / 1e9, 4), unit="GB/s", cores=cores,
                                  note="throughput only: the same set cut into batch slices, one oracle round trip per slice, "
                                       f"{cores} threads; containers differ from those of the whole tensors"))

    if not args.no_configs:
        del xs, outs, conts
        torch.cuda.empty_cache()
        path["configs"] = other_configs(comet, synth, torch, np, args.chunk_syms)

    if args.per_layer:
        for e, x, s in zip(layers, xs, sizes):
            print(f"  {tuple(x.shape)} eb={e['eb']} nbins={e['nbins']}: {4 * x.numel()} B -> {s} B (x{4 * x.numel() / s:.2f})", file=sys.stderr)
        print(f"  generation {gen_s:.1f} s", file=sys.stderr)

    line = dict(metric="compress+decompress GB/s (fp32 in)", value=round(value, 2), unit="GB/s", n_gpus=1,
                steps=args.steps, warmup=args.warmup, ms_per_step=round(ms_per_step, 4), higher_is_better=True,
                scaling="weak", vs_baseline=None, dtype="f32", data="synthetic",
                config=dict(workload=f"ResNet-50-shaped activation set, batch {args.batch}: compress 5 layers forward, "
                                     f"decompress reverse; eb per layer {[e['eb'] for e in layers]}, 1024 bins, "
                                     f"chunk {args.chunk_syms}; layers dealt to {n_ctx} contexts/streams", elements=n_total,
                            input_bytes=in_bytes),
                roofline=roofline, cpu_baseline=cpu, path=path)
    print(json.dumps(line))
    for c in ctxs:
        c.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
