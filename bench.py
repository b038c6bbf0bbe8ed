#!/usr/bin/env python3
"""Benchmark of the W6A6 / W6A8 linear-layer hot path on one MI355X.

Workload: the four linear layers of one LLaMA-2-70B decoder block (fused QKV,
attention output, fused gate+up, down projection) on seeded synthetic weights
and outlier-channel activations.  One step = one pass over the four layers:
per-token activation quantization, then the packed-6-bit GEMM with the fused
scale epilogue; W6A6 everywhere except W6A8 on the down projection, the
paper's policy (Section 4.1.2).

Two timed regions, each of exactly --steps steps after --warmup warm-ups:
  prefill  M = 4096 tokens  -> GEMM TOPS (2*M*N*K per layer), the headline value
  decode   M = 1 token      -> GEMV GB/s of algorithmic bytes
Prints ONE JSON line.  Inputs are resident in HBM before timing starts.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "W6A8/W6A6 GEMM TOPS (M\u22651024) + decode GEMV HBM GB/s, LLaMA-2-70B linears"
PEAK_I8_TOPS = 5000.0      # MI355X dense int8 MFMA, published
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E, published
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "bench_llama2_70b_linears_hbm_traffic.md")
SIGMA = 0.015
LAYERS = [("qkv", 8192, 10240, 6), ("o", 8192, 8192, 6), ("gate_up", 8192, 57344, 6),
          ("down", 28672, 8192, 8)]          # name, K, N, activation bits


def kernel_sources_key():
    """Short hash of the kernel sources: names the build a counter profile was taken on."""
    import hashlib
    csrc = os.path.join(ROOT, "paper_2508_04405_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def profiled_traffic():
    """Bytes past L2 per launch (fetched + written, averaged over the four layers) of the GEMM at
    M = 4096 and of the GEMV at M = 1, from the rocprofv3 FETCH_SIZE / WRITE_SIZE summary under
    profiles/ -- only if that summary was taken on exactly these kernel sources (its `kernel-sources`
    line carries their hash); otherwise None, None: a stale figure is not printed beside live timings."""
    import re
    try:
        text = open(TRAFFIC_PROFILE).read()
    except OSError:
        return None, None
    key = re.search(r"kernel-sources:\s*([0-9a-f]{16})", text)
    gemm = re.search(r"gemm-m4096-traffic-bytes-per-launch:\s*([0-9.]+)", text)
    gemv = re.search(r"gemv-m1-traffic-bytes-per-launch:\s*([0-9.]+)", text)
    if not (key and gemm and gemv) or key.group(1) != kernel_sources_key():
        return None, None
    return float(gemm.group(1)), float(gemv.group(1))


def algorithmic_bytes(M, N, K):
    """Packed weights + weight scales + fp16 activations in + int8 codes out and in again
    + activation scales + fp16 output."""
    return 0.75 * N * K + 2 * N + 2 * M * K + 2 * M * K + 2 * M + 2 * M * N


def gemm_bytes(M, N, K):
    return 0.75 * N * K + 2 * N + M * K + 2 * M + 2 * M * N


def sweep(args, torch, fq, fqdev, synth, dev):
    """Per-layer time of the linear-layer call (pre-quantized activations) for each token
    count, the four layers cycled so that every launch streams its weights from HBM."""
    gen = torch.Generator(device=dev)
    packed = []
    for i, (name, K, N, bits) in enumerate(LAYERS):
        gen.manual_seed(3000 + 10 * i)
        wq = torch.empty((N, K), dtype=torch.int8, device=dev)
        sw = torch.empty((N,), dtype=torch.float16, device=dev)
        for r0 in range(0, N, 8192):
            r1 = min(N, r0 + 8192)
            w = torch.randn((r1 - r0, K), generator=gen, device=dev, dtype=torch.float32) * SIGMA
            wq[r0:r1], sw[r0:r1] = fq.quant_w6(w)
            del w
        packed.append(fq.pack_w6(wq, sw))
        del wq, sw
    print("| M | " + " | ".join("%s us kernel (TOP/s, GB/s)" % L[0] for L in LAYERS) + " |")
    print("|---|" + "---|" * len(LAYERS))
    for M in (1, 4, 8, 16, 32, 64, 128, 256, 512, 768, 1024, 1536, 2048, 3072, 4096):
        bufs = []
        for i, (name, K, N, bits) in enumerate(LAYERS):
            x = torch.from_numpy(synth.activations(M, K, seed=3000 + 10 * i + 1,
                                                   outlier_frac=0.01)).to(dev)
            xq, sx = fq.quant_act(x, bits)
            bufs.append((xq, sx, torch.empty((M, N), dtype=torch.float16, device=dev),
                         fq.make_workspace(M, N, K, dev)))
        times = [[] for _ in LAYERS]
        kinds = [None for _ in LAYERS]

        def cycle(record):
            for i, (name, K, N, bits) in enumerate(LAYERS):
                xq, sx, y, ws = bufs[i]
                fn = fqdev.gemm_w6a6 if bits == 6 else fqdev.gemm_w6a8   # (reports what it launched)
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                fn(packed[i], N, K, 0, xq=xq, sx=sx, workspace=ws, out=y)
                e1.record()
                if record:
                    times[i].append((e0, e1))
                    kinds[i] = fqdev.last_dispatch()

        # warm up for at least 50 ms of GPU work (the host-side input generation above
        # leaves the GPU idle, and its clock takes a while to come back up)
        t_warm = time.perf_counter()
        reps = 0
        while reps < args.warmup or time.perf_counter() - t_warm < 0.05:
            cycle(False)
            torch.cuda.synchronize()
            reps += 1
        for rep in range(args.steps):
            cycle(True)
        torch.cuda.synchronize()
        cells = []
        for i, (name, K, N, bits) in enumerate(LAYERS):
            us = sorted(a.elapsed_time(b) * 1e3 for a, b in times[i])[len(times[i]) // 2]
            kern, splits = kinds[i]
            label = {1: "s", 5: "h", 7: "a", 8: "b", 12: "c", 13: "p", 14: "t", 15: "l", 16: "k"}.get(kern, "?")
            if splits > 1:
                label += str(splits)
            cells.append("%.1f %s (%.0f, %.0f)" % (us, label, 2.0 * M * N * K / us / 1e6,
                                                   gemm_bytes(M, N, K) / us / 1e3))
        print("| %d | " % M + " | ".join(cells) + " |", flush=True)
        del bufs


def replay_time(args, torch, enqueue):
    """Microseconds per call of `enqueue()`, its launches captured in a HIP graph and the graph
    replayed (at least 50 ms of warm-up replays: the host-side set-up leaves the GPU idle and its
    clock low)."""
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        enqueue()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            enqueue()
        t_warm = time.perf_counter()
        reps = 0
        while reps < args.warmup or time.perf_counter() - t_warm < 0.05:
            graph.replay()
            torch.cuda.synchronize()
            reps += 1
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / args.steps


def layer_table(args, torch, fq, fqdev, synth, dev):
    """One decoder layer's seven linears through flexq_layer_linears (fused QKV, O, fused gate+up,
    down, each fed by the producer that quantizes its input: RMS norm + quantize before QKV and
    gate+up, the quantize node before O, gated SiLU + quantize before down).  Two policies: the
    paper's (A8 on the down projection only) and a layer running all seven linears at A8 (the
    flagged layers of the 13B configuration).  The call's launches are captured in a HIP graph and
    replayed; one layer's weights stay resident in the Infinity Cache between replays (the cold
    figure for a whole stack of layers is --stack13b's)."""
    models = [("LLaMA-2-7B", 4096, 11008, 4096 * 3, 0, (1, 8, 512, 2048, 4096)),
              ("LLaMA-2-13B, group-128 weight scales", 5120, 13824, 5120 * 3, 128, (32, 2048)),
              ("LLaMA-2-70B (GQA: 10240-wide QKV)", 8192, 28672, 10240, 0, (1, 16, 1024, 4096))]
    print("| model | M | policy | us per layer | TOP/s | weight GB/s |")
    print("|---|---|---|---|---|---|")
    for name, H, F, QKV, group, Ms in models:
        gen = torch.Generator(device=dev)
        gen.manual_seed(5)

        def make(N, K):
            w = torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * 0.02
            p = fq.pack_w6(*fq.quant_w6(w, group), group)
            del w
            return p
        w_qkv, w_o, w_gu, w_dn = make(QKV, H), make(H, H), make(2 * F, H), make(H, F)
        gamma = torch.from_numpy(synth.norm_gain(H, seed=6)).to(dev)
        wbytes = 0.75 * (QKV * H + H * H + 2 * F * H + H * F)
        ops1 = 2.0 * (QKV * H + H * H + 2 * F * H + H * F)
        for M in Ms:
            x = torch.from_numpy(synth.activations(M, H, seed=7, outlier_frac=0.01)).to(dev)
            attn = torch.from_numpy(synth.activations(M, H, seed=8, outlier_frac=0.01)).to(dev)
            outs = {k: torch.empty((M, n), dtype=torch.float16, device=dev)
                    for k, n in (("qkv", QKV), ("o", H), ("gate_up", 2 * F), ("down", H))}
            for policy, bits in (("A6, A8 on down (the paper's)", (6, 6, 6, 8)),
                                 ("all seven linears A8", (8, 8, 8, 8))):
                layer = fq.Layer(H, F, QKV, group, w_qkv, w_o, w_gu, w_dn, gamma, gamma, 1e-5, bits)
                ws = layer.make_workspace(M, dev)
                us = replay_time(args, torch, lambda: fq.layer_linears(layer, M, ws, x=x, attn=attn,
                                                                         x_ffn=outs["o"], **outs))
                print("| %s | %d | %s | %.1f | %.0f | %.0f |" % (name, M, policy, us, ops1 * M / us / 1e6,
                                                              wbytes / us / 1e3), flush=True)
        del w_qkv, w_o, w_gu, w_dn


def stack13b(args, torch, fq, fqdev, synth, dev):
    """The LLaMA-2-13B-shaped stack of 40 decoder layers' linears (hidden 5120, FFN 13824, fused QKV
    15360), every layer with packed weights of its own (group-128 scales, 9.5 GB resident: a pass
    streams them from HBM, cold by construction).  A seeded quarter of the layers carries outlier
    channels x50 in its input and runs all seven linears at W6A8; the others run W6A6 (Section
    4.1.2's selective precision, per layer as the 13B configuration states it).  Each layer is one
    flexq_layer_linears call on its own synthetic input and attention output; the 40 calls are
    captured in one HIP graph.  Reports the aggregate time of the seven linears (with their fused
    producers) over all 40 layers for batched decode (M = 32) and prefill (M = 2048)."""
    H, F, QKV, group, n_layers = 5120, 13824, 15360, 128, 40
    rng = __import__("numpy").random.default_rng(13)
    flagged = rng.random(n_layers) < 0.25
    gen = torch.Generator(device=dev)
    layers = []
    for i in range(n_layers):
        gen.manual_seed(13000 + i)

        def make(N, K):
            w = torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * 0.02
            p = fq.pack_w6(*fq.quant_w6(w, group), group)
            del w
            return p
        gamma = torch.from_numpy(synth.norm_gain(H, seed=13100 + i)).to(dev)
        bits = (8, 8, 8, 8) if flagged[i] else (6, 6, 6, 6)
        layers.append(fq.Layer(H, F, QKV, group, make(QKV, H), make(H, H), make(2 * F, H), make(H, F),
                               gamma, gamma, 1e-5, bits))
    torch.cuda.synchronize()
    wbytes = n_layers * (0.75 + 2.0 / 128) * (QKV * H + H * H + 2 * F * H + H * F)
    ops1 = n_layers * 2.0 * (QKV * H + H * H + 2 * F * H + H * F)
    print("%d layers, %d of them W6A8 (outlier channels x50): %s; packed weights %.2f GB" %
          (n_layers, int(flagged.sum()), " ".join(str(i) for i in range(n_layers) if flagged[i]), wbytes / 1e9))
    print("| M | us, all 40 layers x 7 linears | us per layer | TOP/s | weight GB/s |")
    print("|---|---|---|---|---|")
    for M in (32, 2048):
        xs, attns = [], []
        for i in range(n_layers):
            scale = 50.0 if flagged[i] else 1.0        # no outlier channels in the other layers
            frac = 0.01 if flagged[i] else 0.0
            xs.append(torch.from_numpy(synth.activations(M, H, seed=13200 + i, outlier_frac=frac,
                                                         outlier_scale=scale)).to(dev))
            attns.append(torch.from_numpy(synth.activations(M, H, seed=13300 + i, outlier_frac=frac,
                                                            outlier_scale=scale)).to(dev))
        outs = {k: torch.empty((M, n), dtype=torch.float16, device=dev)
                for k, n in (("qkv", QKV), ("o", H), ("gate_up", 2 * F), ("down", H))}
        ws = layers[0].make_workspace(M, dev)

        def step():
            for i, layer in enumerate(layers):
                fq.layer_linears(layer, M, ws, x=xs[i], attn=attns[i], x_ffn=outs["o"], **outs)
        us = replay_time(args, torch, step)
        print("| %d | %.0f | %.1f | %.0f | %.0f |" % (M, us, us / n_layers, ops1 * M / us / 1e6, wbytes / us / 1e3),
              flush=True)
        del xs, attns


def probe_table(args, torch, fq, fqdev, synth, dev):
    """Decode GEMV against a kernel that only reads the same packed buffer (the development
    library's read probe), layer by layer, the four layers cycled so that every launch streams from
    HBM: how much of a layer's time is the weight stream itself, launch, ramp-up and drain
    included."""
    packs = []
    for name, K, N, bits in LAYERS:
        packed = torch.randint(0, 256, (fq.packed_bytes(N, K, 0),), dtype=torch.uint8, device=dev)
        sw = (torch.rand(N, device=dev) * 1e-3 + 1e-4).half()
        packed[N * K * 6 // 8: N * K * 6 // 8 + 2 * N] = sw.view(torch.uint8)
        packs.append(packed)
    sink = torch.zeros(16, dtype=torch.int32, device=dev)
    print("| M | layer | packed MB | read probe us (GB/s) | GEMV us (GB/s) | GEMV / probe |")
    print("|---|---|---|---|---|---|")
    for M in (1, 16):
        bufs = []
        for name, K, N, bits in LAYERS:
            xq = torch.randint(-31, 32, (M, K), dtype=torch.int8, device=dev)
            sx = torch.ones(M, dtype=torch.float16, device=dev)
            bufs.append((xq, sx, torch.empty((M, N), dtype=torch.float16, device=dev),
                         fq.make_workspace(M, N, K, dev)))
        tp = [[] for _ in LAYERS]
        tg = [[] for _ in LAYERS]
        for rep in range(args.warmup + args.steps):
            for i, (name, K, N, bits) in enumerate(LAYERS):
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                fqdev.probe_hbm_read(packs[i], sink)
                e1.record()
                if rep >= args.warmup:
                    tp[i].append((e0, e1))
            for i, (name, K, N, bits) in enumerate(LAYERS):
                xq, sx, y, ws = bufs[i]
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                (fq.gemv_w6a6 if bits == 6 else fq.gemv_w6a8)(packs[i], N, K, 0, xq=xq, sx=sx, workspace=ws, out=y)
                e1.record()
                if rep >= args.warmup:
                    tg[i].append((e0, e1))
        torch.cuda.synchronize()
        med = lambda t: sorted(a.elapsed_time(b) * 1e3 for a, b in t)[len(t) // 2]
        for i, (name, K, N, bits) in enumerate(LAYERS):
            mb = packs[i].numel() / 1e6
            p_us, g_us = med(tp[i]), med(tg[i])
            print("| %d | %s | %.1f | %.1f (%.0f) | %.1f (%.0f) | %.2f |" %
                  (M, name, mb, p_us, mb / p_us * 1e3, g_us, mb / g_us * 1e3, g_us / p_us), flush=True)


def mix_table(args, torch, fq, fqdev, synth, dev):
    """What the chip sustains on a stream of int8 MFMAs accompanied by the other work of a GEMM
    wavefront (development library's mix probe: no global loads, no barriers): the context for
    reading the GEMM's fraction of the published peak on a power-limited machine."""
    K, N = 8192, 8192
    gen = torch.Generator(device=dev)
    gen.manual_seed(3010)
    w = torch.randn((256, K), generator=gen, device=dev, dtype=torch.float32) * SIGMA
    wq, sw = fq.quant_w6(w)
    b_ops = fq.pack_w6(wq, sw)
    x = torch.from_numpy(synth.activations(64, K, seed=3011, outlier_frac=0.01)).to(dev)
    a_ops, _ = fq.quant_act(x, 6)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    print("| wavefronts per SIMD | vector operations per MFMA | 16-byte LDS reads per 8 MFMAs | TOP/s | of the 5000 peak |")
    print("|---|---|---|---|---|")
    iters = 4000
    for waves, v, l in ((4, 0, 0), (8, 0, 0), (8, 2, 0), (8, 3, 0), (8, 4, 0), (8, 6, 0), (8, 8, 0), (8, 0, 4), (8, 3, 4),
                        (8, 3, 8)):
        t_start = time.perf_counter()
        while time.perf_counter() - t_start < 0.05:
            fqdev.probe_mfma_mix(a_ops, b_ops, v, l, 400, 256, waves, sink)
            torch.cuda.synchronize()
        best = []
        for _ in range(5):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            fqdev.probe_mfma_mix(a_ops, b_ops, v, l, iters, 256, waves, sink)
            e1.record()
            torch.cuda.synchronize()
            best.append(e0.elapsed_time(e1))
        ms = sorted(best)[2]
        tops = 2.0 * 32768 * 8 * iters * waves * 256 / (ms * 1e-3) / 1e12
        print("| %d | %d | %d | %.0f | %.1f %% |" % (waves // 4, v, l, tops, tops / 50.0), flush=True)


def tiles_table(args, torch, fq, fqdev, synth, dev):
    """Batched decode from fp16 activations, per layer and token count: the quantizer writing
    row-major int8 codes against the quantizer writing tile order (6-bit activations packed at
    0.75 byte per value), each followed by the streaming kernel; and what the library picks by
    itself.  Each figure is the whole call (quantize launch + GEMV), the four layers cycled so
    that the weights stream from HBM."""
    packs = []
    for name, K, N, bits in LAYERS:
        packed = torch.randint(0, 256, (fq.packed_bytes(N, K, 0),), dtype=torch.uint8, device=dev)
        sw = (torch.rand(N, device=dev) * 1e-3 + 1e-4).half()
        packed[N * K * 6 // 8: N * K * 6 // 8 + 2 * N] = sw.view(torch.uint8)
        packs.append(packed)
    print("| M | layer | activations | row-major codes us | tile order us | library's choice us (kernel) |")
    print("|---|---|---|---|---|---|")
    for M in (4, 8, 12, 16, 20, 24, 28, 32):
        bufs = []
        for i, (name, K, N, bits) in enumerate(LAYERS):
            x = torch.from_numpy(synth.activations(M, K, seed=3001 + 10 * i, outlier_frac=0.01)).to(dev)
            bufs.append((x, torch.empty((M, N), dtype=torch.float16, device=dev), fq.make_workspace(M, N, K, dev)))
        res = {}
        for mode in (2, 1, 0):
            fqdev.set_tiles(mode)
            times = [[] for _ in LAYERS]

            def cycle(record):
                for i, (name, K, N, bits) in enumerate(LAYERS):
                    x, y, ws = bufs[i]
                    e0 = torch.cuda.Event(enable_timing=True)
                    e1 = torch.cuda.Event(enable_timing=True)
                    e0.record()
                    (fqdev.gemv_w6a6 if bits == 6 else fqdev.gemv_w6a8)(packs[i], N, K, 0, x_fp16=x, workspace=ws, out=y)
                    e1.record()
                    if record:
                        times[i].append((e0, e1, fqdev.last_dispatch()))

            t_start = time.perf_counter()
            while time.perf_counter() - t_start < 0.05:     # the clock settles under load
                cycle(False)
                torch.cuda.synchronize()
            for _ in range(args.warmup):
                cycle(False)
            for _ in range(args.steps):                      # back to back, as a decode loop issues them
                cycle(True)
            torch.cuda.synchronize()
            res[mode] = [(sorted(a.elapsed_time(b) * 1e3 for a, b, _ in t)[len(t) // 2], t[0][2]) for t in times]
        fqdev.set_tiles(0)
        for i, (name, K, N, bits) in enumerate(LAYERS):
            kern, code = res[0][i][1]
            what = ("streaming, tiles" if code >= 500 else "streaming, rows") if kern == 1 else "64x128 tiles GEMM"
            print("| %d | %s | A%d | %.1f | %.1f | %.1f (%s) |" %
                  (M, name, bits, res[2][i][0], res[1][i][0], res[0][i][0], what), flush=True)


def ablation(args, torch, fq, fqdev, synth, dev):
    """GEMV time with one design choice of the streaming kernel undone per row (the paper's
    Table 6 on this machine).  Each shape is replicated until the copies exceed twice the
    Infinity Cache, the launches over all copies are captured in a HIP graph and the graph is
    replayed, so a row is kernel time from cold HBM without host launch overhead."""
    shapes = [("(1,4096)x(4096,4096) W6A6", 4096, 4096, 6, 44),
              ("(1,28672)x(28672,8192) W6A8", 28672, 8192, 8, 3)]
    rows = [("full design (automatic dispatch)", dict()),
            ("no K split across workgroups", dict(split=1)),
            ("4 wavefronts per workgroup instead of 8", dict(waves=4)),
            ("16 wavefronts per workgroup", dict(waves=16)),
            ("cached instead of non-temporal weight loads", dict(ablate=1)),
            ("one weight tile in flight per wavefront instead of four", dict(ablate=2)),
            ("two weight tiles in flight", dict(ablate=3)),
            ("activations from global memory per tile, not staged in LDS", dict(ablate=4)),
            ("separate quantize launch (kernel pair) instead of the fused prologue", dict(pair=True)),
            ("fused quantize prologue (one launch from fp16 activations)", dict(fused=True))]
    print("| variant | " + " | ".join(s[0] + " us (GB/s)" for s in shapes) + " |")
    print("|---|" + "---|" * len(shapes))
    table = {r[0]: [] for r in rows}
    for name, K, N, bits, copies in shapes:
        gen = torch.Generator(device=dev)
        gen.manual_seed(77)
        w = torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * 0.02
        one = fq.pack_w6(*fq.quant_w6(w))
        del w
        packed = [one.clone() for _ in range(copies)]
        x = torch.from_numpy(synth.activations(1, K, seed=78, outlier_frac=0.01)).to(dev)
        xq, sx = fq.quant_act(x, bits)
        y = torch.empty((1, N), dtype=torch.float16, device=dev)
        ws = fq.make_workspace(1, N, K, dev)
        gemv = fqdev.gemv_w6a6 if bits == 6 else fqdev.gemv_w6a8
        nbytes = gemm_bytes(1, N, K)
        for label, opt in rows:
            fqdev.set_dispatch(1, opt.get("split", 0), opt.get("waves", 8 if "ablate" in opt else 0), 0)
            fqdev.set_ablation(opt.get("ablate", 0))

            def launches():
                for p in packed:
                    if opt.get("fused"):
                        gemv(p, N, K, 0, x_fp16=x, workspace=ws, out=y)
                    else:
                        if opt.get("pair"):
                            fq.quant_act(x, bits, out=(xq, sx))
                        gemv(p, N, K, 0, xq=xq, sx=sx, workspace=ws, out=y)
            try:
                stream = torch.cuda.Stream()
                stream.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(stream):
                    launches()
                    torch.cuda.synchronize()
                    graph = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(graph, stream=stream):
                        launches()
                    for _ in range(args.warmup):
                        graph.replay()
                    e0 = torch.cuda.Event(enable_timing=True)
                    e1 = torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for _ in range(args.steps):
                        graph.replay()
                    e1.record()
                    torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / (args.steps * copies)
                table[label].append("%.2f (%.0f)" % (us, nbytes / us / 1e3))
            finally:
                fqdev.set_ablation(0)
                fqdev.set_dispatch(0, 0, 0, 0)
    for label, _ in rows:
        print("| %s | " % label + " | ".join(table[label]) + " |", flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--prefill-m", type=int, default=4096)
    ap.add_argument("--decode-m", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sources-key", action="store_true",
                    help="print the hash of the kernel sources (what a counter profile is tagged with) and exit")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="only run a plain device copy of known size (for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    ap.add_argument("--gemm-cfg", type=int, default=0,
                    help="force a tile configuration of the tiled kernel (0 = the library's choice)")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line, print a table of per-layer GEMM / GEMV "
                         "times over token counts M = 1 .. 4096 (library's own dispatch)")
    ap.add_argument("--layer", action="store_true",
                    help="instead of the benchmark line, print the time of one decoder layer's "
                         "seven linears (four GEMM calls fed by the fused producers) for the "
                         "LLaMA-2 7B / 13B / 70B shapes")
    ap.add_argument("--probe", action="store_true",
                    help="instead of the benchmark line, print the decode GEMV against a read-only kernel "
                         "over the same packed buffers, per layer, at M = 1 and 16")
    ap.add_argument("--mix", action="store_true",
                    help="instead of the benchmark line, print what the chip sustains on int8 MFMA streams "
                         "accompanied by vector operations and LDS reads (development library's mix probe)")
    ap.add_argument("--tiles", action="store_true",
                    help="instead of the benchmark line, print batched decode (4 to 32 tokens, fp16 in) with the "
                         "quantized activations row-major against in tile order (6-bit ones packed)")
    ap.add_argument("--stack13b", action="store_true",
                    help="instead of the benchmark line, print the aggregate time of the LLaMA-2-13B-shaped "
                         "40-layer linear stack (group-128 weight scales, a seeded quarter of the layers at "
                         "W6A8) at M = 32 and M = 2048")
    ap.add_argument("--ablation", action="store_true",
                    help="instead of the benchmark line, print the decode-kernel ablation table "
                         "(one design choice undone per row) on the paper's Table-6 shapes")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (--gpus 1); "
                 "there is no multi-GPU path to measure")
    if args.sources_key:
        print(kernel_sources_key())
        return

    import numpy as np
    import torch
    import paper_2508_04405_amd as fq
    from paper_2508_04405_amd import dev as fqdev, synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.traffic_calibration:
        nbytes = 1 << 30
        src = torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)          # one elementwise copy kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "5 copies", "bytes_read_per_copy": nbytes,
                          "bytes_written_per_copy": nbytes}))
        return
    fq.load()
    # the product library runs the benchmark; a forced tile configuration needs the
    # development library (same sources, per-call overrides)
    lin = fq
    if args.gemm_cfg:
        fqdev.set_dispatch(0, 0, 0, args.gemm_cfg)
        lin = fqdev

    if args.sweep:
        return sweep(args, torch, fq, fqdev, synth, dev)
    if args.ablation:
        return ablation(args, torch, fq, fqdev, synth, dev)
    if args.layer:
        return layer_table(args, torch, fq, fqdev, synth, dev)
    if args.stack13b:
        return stack13b(args, torch, fq, fqdev, synth, dev)
    if args.probe:
        return probe_table(args, torch, fq, fqdev, synth, dev)
    if args.tiles:
        return tiles_table(args, torch, fq, fqdev, synth, dev)
    if args.mix:
        return mix_table(args, torch, fq, fqdev, synth, dev)

    # ---- resident inputs: packed weights, fp16 activations -----------------
    gen = torch.Generator(device=dev)
    layers = []
    for i, (name, K, N, bits) in enumerate(LAYERS):
        gen.manual_seed(3000 + 10 * i)
        wq = torch.empty((N, K), dtype=torch.int8, device=dev)
        sw = torch.empty((N,), dtype=torch.float16, device=dev)
        for r0 in range(0, N, 8192):
            r1 = min(N, r0 + 8192)
            w = torch.randn((r1 - r0, K), generator=gen, device=dev, dtype=torch.float32) * SIGMA
            q, s = fq.quant_w6(w)
            wq[r0:r1], sw[r0:r1] = q, s
            del w, q, s
        packed = fq.pack_w6(wq, sw)
        del wq, sw
        layer = {"name": name, "K": K, "N": N, "bits": bits, "packed": packed}
        for tag, M in (("prefill", args.prefill_m), ("decode", args.decode_m)):
            x = torch.from_numpy(synth.activations(M, K, seed=3000 + 10 * i + 1,
                                                   outlier_frac=0.01, outlier_scale=20.0)).to(dev)
            layer[tag] = {
                "M": M, "x": x,
                "xq": torch.empty((M, K), dtype=torch.int8, device=dev),
                "sx": torch.empty((M,), dtype=torch.float16, device=dev),
                "y": torch.empty((M, N), dtype=torch.float16, device=dev),
                "ws": fq.make_workspace(M, N, K, dev),
            }
        layers.append(layer)
    torch.cuda.synchronize()

    def run_layer(layer, tag, events=None):
        b = layer[tag]
        if tag == "decode":     # small batch: the GEMV call quantizes the fp16 activations itself
            gemv = fq.gemv_w6a6 if layer["bits"] == 6 else fq.gemv_w6a8
            gemv(layer["packed"], layer["N"], layer["K"], 0, x_fp16=b["x"], workspace=b["ws"],
                 out=b["y"])
            return
        fq.quant_act(b["x"], layer["bits"], out=(b["xq"], b["sx"]))
        gemm = lin.gemm_w6a6 if layer["bits"] == 6 else lin.gemm_w6a8
        if events is not None:
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
        gemm(layer["packed"], layer["N"], layer["K"], 0, xq=b["xq"], sx=b["sx"],
             workspace=b["ws"], out=b["y"])
        if events is not None:
            e1.record()
            events.append((layer["name"], e0, e1))

    preroll_ms = {}

    def timed(tag, per_kernel_events):
        # pre-roll: the host-side set-up above left the GPU idle, and its clock takes tens of
        # milliseconds of load to settle; run the step for at least 50 ms before the declared
        # warm-up steps (reported as preroll_ms)
        t_roll = time.perf_counter()
        while time.perf_counter() - t_roll < 0.05:
            for layer in layers:
                run_layer(layer, tag)
            torch.cuda.synchronize()
        preroll_ms[tag] = round((time.perf_counter() - t_roll) * 1e3, 1)
        for _ in range(args.warmup):
            for layer in layers:
                run_layer(layer, tag)
        events = [] if per_kernel_events else None
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            for layer in layers:
                run_layer(layer, tag, events)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        return (t1 - t0) / args.steps, events

    # ---- prefill: the headline ------------------------------------------------
    Mp = args.prefill_m
    step_s, events = timed("prefill", True)
    ops_step = sum(2.0 * Mp * L["N"] * L["K"] for L in layers)
    tops = ops_step / step_s / 1e12
    per_layer = {}
    for name, e0, e1 in events:
        per_layer.setdefault(name, []).append(e0.elapsed_time(e1) * 1e-3)
    gemm_s = sum(sum(v) for v in per_layer.values()) / args.steps       # the 4 GEMM launches
    gemm_tops = ops_step / gemm_s / 1e12
    launches = 4 * args.steps
    traffic_gemm, traffic_gemv = profiled_traffic()
    roofline = {
        "bound": "mfma",
        "kernel": "gemm_wlds_kernel (256-row tiles, both operands through LDS, persistent; the 10240-wide "
                  "qkv adds a tail of half tiles or K-cut tiles), i8 MFMA 32x32x32",
        "achieved": round(gemm_tops, 2), "peak": PEAK_I8_TOPS / 1.0, "unit": "TOP/s",
        "frac": round(gemm_tops / PEAK_I8_TOPS, 4),
        "avg_launch_ms": round(gemm_s / 4 * 1e3, 4), "launches": launches,
        "per_layer_tops": {n: round(2.0 * Mp * L["N"] * L["K"] / (sum(per_layer[n]) / args.steps) / 1e12, 2)
                           for n, L in ((L["name"], L) for L in layers)},
        "traffic": traffic_gemm if Mp == 4096 else None,
        "algorithmic_bytes": sum(gemm_bytes(Mp, L["N"], L["K"]) for L in layers) / 4,
    }

    # ---- decode: weight-streaming GEMV ---------------------------------------
    Md = args.decode_m

    dstep_s, _ = timed("decode", False)
    dbytes = sum(algorithmic_bytes(Md, L["N"], L["K"]) for L in layers)
    # kernel-only rate: the same four GEMV launches back to back, no quantize pass, one event pair
    # (eager launches: replaying them as a HIP graph was measured 3-4 % slower -- graph nodes start
    # strictly after one another, eager launches on one stream overlap their ramp-up and drain)
    for layer in layers:
        b = layer["decode"]
        fq.quant_act(b["x"], layer["bits"], out=(b["xq"], b["sx"]))

    def gemv_step():
        for layer in layers:
            b = layer["decode"]
            (fq.gemv_w6a6 if layer["bits"] == 6 else fq.gemv_w6a8)(
                layer["packed"], layer["N"], layer["K"], 0, xq=b["xq"], sx=b["sx"],
                workspace=b["ws"], out=b["y"])
    for _ in range(args.warmup):
        gemv_step()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        gemv_step()
    e1.record()
    torch.cuda.synchronize()
    gemv_s = e0.elapsed_time(e1) * 1e-3 / args.steps
    gbytes = sum(gemm_bytes(Md, L["N"], L["K"]) for L in layers)
    roofline_decode = {
        "bound": "hbm", "kernel": "skinny_kernel (streaming GEMV, M=%d)" % Md,
        "achieved": round(gbytes / gemv_s / 1e9, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
        "frac": round(gbytes / gemv_s / 1e9 / PEAK_HBM_GBS, 4),
        "avg_launch_us": round(gemv_s / 4 * 1e6, 2), "launches": 4 * args.steps,
        "bytes_per_step": int(gbytes), "algorithmic_bytes": gbytes / 4,
        "traffic": traffic_gemv if Md == 1 else None,
    }

    # ---- measured ceilings on this machine (context for the fractions above) ------
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    for layer in layers:                                   # warm-up
        fqdev.probe_hbm_read(layer["packed"], sink)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        for layer in layers:                               # 642 MB per pass: cold, like the GEMV
            fqdev.probe_hbm_read(layer["packed"], sink)
    e1.record()
    torch.cuda.synchronize()
    read_gbs = sum(L["packed"].numel() for L in layers) * args.steps / (e0.elapsed_time(e1) * 1e-3) / 1e9
    a_ops, b_ops = layers[0]["prefill"]["xq"], layers[0]["packed"]
    def mix_tops(valu, lds_reads):
        # the MFMA stream in the GEMM kernel's operand pattern, with `valu` vector operations per
        # MFMA and `lds_reads` LDS reads per eight MFMAs beside it: ~1 ms, like one GEMM launch
        iters = 4000
        t_roll = time.perf_counter()
        while time.perf_counter() - t_roll < 0.03:
            fqdev.probe_mfma_mix(a_ops, b_ops, valu, lds_reads, 400, 256, 8, sink)
            torch.cuda.synchronize()
        e0.record()
        fqdev.probe_mfma_mix(a_ops, b_ops, valu, lds_reads, iters, 256, 8, sink)
        e1.record()
        torch.cuda.synchronize()
        return 2.0 * 32768 * 8 * iters * 8 * 256 / (e0.elapsed_time(e1) * 1e-3) / 1e12

    mfma_only, mfma_mix = mix_tops(0, 0), mix_tops(3, 4)
    roofline["measured_ceiling"] = {
        "value": round(mfma_mix, 1), "unit": "TOP/s",
        "what": "v_mfma_i32_32x32x32_i8 stream in this kernel's operand pattern on this workload's "
                "activation codes and weight bytes, with three vector operations per MFMA and one LDS "
                "read per two MFMAs beside it and nothing else (no global loads, barriers, epilogue); "
                "the chip is power-limited: the clock drops with the work",
        "mfma_only": round(mfma_only, 1),
        "frac_of_ceiling": round(gemm_tops / mfma_mix, 4)}
    roofline_decode["measured_ceiling"] = {
        "value": round(read_gbs, 1), "unit": "GB/s",
        "what": "read-only kernel over the same four packed weight buffers",
        "frac_of_ceiling": round(roofline_decode["achieved"] / read_gbs, 4)}

    # ---- the CPU oracle on a bounded sample of the same workload --------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        K, N = 8192, 8192
        w = synth.weights(N, K, SIGMA, seed=3010)
        wq, sw = oracle.quantize(w, 6, 0)
        del w
        x = synth.activations(Mp, K, seed=3011, outlier_frac=0.01)
        rows = min(32, Mp)
        t0 = time.perf_counter()
        xq, sx = oracle.quantize(x[:rows].astype(np.float32), 6, 0)
        oracle.dequant(oracle.matmul(xq, wq), sx, sw)
        probe = time.perf_counter() - t0
        rows = int(max(1, min(Mp, rows * 15.0 / max(probe, 1e-3))))
        t0 = time.perf_counter()
        xq, sx = oracle.quantize(x[:rows].astype(np.float32), 6, 0)
        oracle.dequant(oracle.matmul(xq, wq), sx, sw)
        dt = time.perf_counter() - t0
        cpu = {"value": round(2.0 * rows * N * K / dt / 1e12, 5), "unit": "TOPS",
               "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "o_proj layer (K=8192, N=8192), %d of the %d prefill tokens: quantize + "
                         "int64 matmul + fp64 dequant, %.1f s" % (rows, Mp, dt)}

    out = {
        "metric": METRIC, "value": round(tops, 2), "unit": "TOPS", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "preroll_ms": preroll_ms,
        "ms_per_step": round(step_s * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": "LLaMA-2-70B linears (configs[3]): qkv 8192x10240, o 8192x8192, "
                               "gate_up 8192x57344 (W6A6), down 28672x8192 (W6A8); prefill M=%d, "
                               "decode M=%d; step = quantize activations + GEMM for all four" % (Mp, Md),
                   "prefill_tokens": Mp, "decode_tokens": Md},
        "decode": {"value": round(dbytes / dstep_s / 1e9, 1), "unit": "GB/s",
                   "us_per_step": round(dstep_s * 1e6, 2),
                   "note": "algorithmic bytes of quantize + GEMV for the four layers / step time"},
        "roofline": roofline, "roofline_decode": roofline_decode, "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
