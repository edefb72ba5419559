"""Benchmark of the XNOR-Net binary convolution block on one MI355X.

One step = one pass of the hot path over one batch resident in HBM:
    xnor_binactiv (BatchNorm fold, sign + bit-pack, A)  ->  xnor_conv2d (binary dot, K from A, K*alpha).
The weights are packed once before the timed region (at inference only B and alpha exist; the
packing time is reported separately).  Prints ONE JSON line on stdout.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload alexnet_conv2] [--algo auto]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# command (scaled by a 256 MiB copy: reads x2.00, writes x1.00), see profiles/; None where not measured.
MEASURED_TRAFFIC = {("alexnet_conv2", "mfma_f4"): 1830.6 * 1024 * 2.0 + 49229.0 * 1024}

PEAKS = {  # MI355X published dense peaks
    "mfma_f4": {"bound": "mfma", "peak": 10100.0, "unit": "TFLOP/s"},     # fp4 10.1 PFLOP/s, 2 flops per MAC
    "mfma_i8": {"bound": "mfma", "peak": 5000.0, "unit": "TOP/s"},        # int8 5.0 POP/s, 2 ops per MAC
    # vector ALU bitcount: 2 instructions (XOR, bitcount-accumulate) per 32 binary MACs:
    # 256 CUs x 64 lanes x 2.4 GHz x 16 MAC per lane-instruction
    "popcount": {"bound": "alu", "peak": 256 * 64 * 2.4e9 * 16 / 1e12, "unit": "Tbinop/s"},
}


def algo_bytes(layer, fused=False):
    """Bytes one xnor_conv2d launch must move: packed activations, matrix-core weight image (fp4),
    A, alpha and the float output."""
    cw = (layer.c + 31) // 32
    taps = layer.kh * layer.kw
    wimg = ((layer.k_out + 31) // 32) * ((taps * cw + 1) // 2) * 1024
    m = layer.n * layer.h_out * layer.w_out
    # result: the float tensor, or (fused epilogue) the next layer's sign words and A
    result = m * ((layer.k_out + 31) // 32 * 4 + 4) if fused else m * layer.k_out * 4
    return layer.n * layer.h * layer.w * (cw * 4 + 4) + wimg + layer.k_out * 4 + result


def cpu_baseline(layers, inputs):
    """The oracle as it stands, whole block, on this machine's host cores."""
    from oracle import xnor_oracle as xo
    xo.binary_conv2d(inputs[0]["x"][:1], inputs[0]["w"], (1, 1), (0, 0))   # load + warm the library
    t0 = time.perf_counter()
    macs = 0
    for layer, d in zip(layers, inputs):
        xo.binary_conv2d(d["x"], d["w"], (layer.stride,) * 2, (layer.pad,) * 2, d["bn_scale"], d["bn_shift"])
        macs += layer.bit_macs
    dt = time.perf_counter() - t0
    return {"value": macs / dt / 1e9, "unit": "Gbinop/s", "cores": xo.threads(), "kind": "oracle",
            "sample": f"full workload ({len(layers)} layer(s), batch {layers[0].n}), {dt:.2f} s wall"}


def report(args):
    """Per-layer table over all five configurations (markdown on stdout): median of `--steps` HIP-event
    timed launches after warm-up (L2 not flushed between launches), for the convolution alone with each
    inner loop, BinActiv alone, and the whole block; throughput, algorithmic GB/s and roofline fractions
    of the fastest loop; the weight packing once; the CPU oracle on the same inputs."""
    import statistics

    import torch
    from paper_1603_05279_amd import workloads as wl
    from paper_1603_05279_amd import xnor

    torch.cuda.set_device(0)
    runs = max(args.steps, 50)

    def median_us(fn):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(runs)]
        for a, b in ev:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        return statistics.median(a.elapsed_time(b) for a, b in ev) * 1e3

    # streaming copy: the practical HBM rate the fractions below are also quoted against
    src = torch.empty(256 * 1024 * 1024 // 4, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    copy_us = median_us(lambda: dst.copy_(src))
    copy_gbs = 2 * src.numel() * 4 / (copy_us * 1e-6) / 1e9
    del src, dst
    print(f"Streaming copy 256 MiB: {copy_us:.1f} us = {copy_gbs:.0f} GB/s (read + write); published peak 8000 GB/s.")
    print(f"Every figure: median of {runs} single launches bracketed by HIP events (the bracket itself adds "
          "about 3 us of dispatch latency to a launch); L2 not flushed between launches.\n")
    print("| config / layer | G binop | conv fp4 us | conv int8 us | conv popcount us | BinActiv us | block us | "
          "Tbinop/s (conv fp4) | alg. GB/s | % fp4 peak | % HBM peak | % attainable | pack us | oracle Gbinop/s |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    from oracle import xnor_oracle as xo
    for cfg in ("tiny", "alexnet_conv2", "alexnet_conv345", "resnet18", "fc"):
        for i, layer in enumerate(wl.config_layers(cfg)):
            seed = wl.config_seed(cfg, i)
            if cfg == "fc":
                d = wl.linear_inputs(layer, seed)
                n, c, h, w_, k, kh, kw, st, pd = layer.batch, layer.in_features, 1, 1, layer.out_features, 1, 1, 1, 0
                x = torch.from_numpy(d["x"]).cuda().reshape(n, c, 1, 1)
                wt = torch.from_numpy(d["w"]).cuda().reshape(k, c, 1, 1)
                sc = sf = None
            else:
                d = wl.conv_inputs(layer, seed)
                n, c, h, w_, k, kh, kw, st, pd = (layer.n, layer.c, layer.h, layer.w, layer.k_out, layer.kh,
                                                  layer.kw, layer.stride, layer.pad)
                x, wt = torch.from_numpy(d["x"]).cuda(), torch.from_numpy(d["w"]).cuda()
                sc = torch.from_numpy(d["bn_scale"]).cuda() if d["bn_scale"] is not None else None
                sf = torch.from_numpy(d["bn_shift"]).cuda() if d["bn_shift"] is not None else None
            desc = xnor.make_desc(n, c, h, w_, k, kh, kw, st, pd)
            pw = xnor.PackedWeights(wt)
            bufs = xnor.ConvBuffers(desc)
            pack_us = median_us(lambda: xnor.xnor_pack_weights(wt, pw.wbits, pw.alpha, pw.wmfma, k, c, kh, kw))
            ba_us = median_us(lambda: xnor.xnor_binactiv(x, sc, sf, bufs.xbits, bufs.A, None, desc))
            conv = {a: median_us(lambda a=a: xnor.xnor_conv2d(bufs.xbits, pw.wbits, pw.wmfma, None, bufs.A, pw.alpha,
                                                               bufs.out, None, desc, xnor.ALGOS[a]))
                    for a in ("mfma_f4", "mfma_i8", "popcount")}

            def block():
                xnor.xnor_binactiv(x, sc, sf, bufs.xbits, bufs.A, None, desc)
                xnor.xnor_conv2d(bufs.xbits, pw.wbits, pw.wmfma, None, bufs.A, pw.alpha, bufs.out, None, desc,
                                 xnor.XNOR_ALGO_MFMA_F4)
            block_us = median_us(block)
            macs = layer.bit_macs
            ho, wo = xnor.output_hw(desc)
            cw = (c + 31) // 32
            nbytes = (n * h * w_ * (cw * 4 + 4) + ((k + 31) // 32) * ((kh * kw * cw + 1) // 2) * 1024 + k * 4 +
                      n * k * ho * wo * 4)
            t = conv["mfma_f4"] * 1e-6
            tb, gbs = macs / t / 1e12, nbytes / t / 1e9
            attain = max(2 * macs / 10.1e15, nbytes / 8e12) / t        # against min(peak, AI x BW)
            t0 = time.perf_counter()
            if cfg == "fc":
                xo.binary_linear(d["x"], d["w"])
            else:
                xo.binary_conv2d(d["x"], d["w"], (st, st), (pd, pd), d["bn_scale"], d["bn_shift"])
            orc = macs / (time.perf_counter() - t0) / 1e9
            print(f"| {cfg} / {layer.name} | {macs / 1e9:.2f} | {conv['mfma_f4']:.1f} | {conv['mfma_i8']:.1f} | "
                  f"{conv['popcount']:.1f} | {ba_us:.1f} | {block_us:.1f} | {tb:.0f} | {gbs:.0f} | "
                  f"{100 * 2 * tb / 10100:.1f} | {100 * gbs / 8000:.1f} | {100 * attain:.1f} | {pack_us:.1f} | "
                  f"{orc:.1f} |", flush=True)
    # the widened rows: Binary-Weight-Network convolution and binary-gradient backward convolution
    print("\n| config / layer | BWN split us | BWN conv us | bf16 TFLOP/s (3 parts) | % bf16 peak | fp32-equiv TFLOP/s | "
          "grad binarize us | grad conv us | Tbinop/s (grad conv) | 2-bit pack us | 2x2-bit conv us | "
          "pool 3x3/2 + BinActiv of the output us |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|")
    for cfg in ("alexnet_conv2", "alexnet_conv345", "resnet18"):
        for i, layer in enumerate(wl.config_layers(cfg)):
            n, c, h, w_, k, kh, kw, st, pd = (layer.n, layer.c, layer.h, layer.w, layer.k_out, layer.kh, layer.kw,
                                              layer.stride, layer.pad)
            gen = torch.Generator(device="cuda")
            gen.manual_seed(wl.config_seed(cfg, i))
            x = torch.randn((n, c, h, w_), device="cuda", generator=gen)
            wt = torch.randn((k, c, kh, kw), device="cuda", generator=gen)
            desc = xnor.make_desc(n, c, h, w_, k, kh, kw, st, pd)
            ho, wo = xnor.output_hw(desc)
            u8 = lambda nbytes: torch.empty((nbytes,), dtype=torch.uint8, device="cuda")
            parts, wimg = u8(xnor.bwn_parts_bytes(n, c, h, w_)), u8(xnor.bwn_wimg_bytes(k, c, kh, kw))
            alpha = torch.empty((k,), device="cuda")
            out = torch.empty((n, k, ho, wo), device="cuda")
            xnor.xnor_bwn_pack_weights(wt, alpha, wimg, k, c, kh, kw)
            split_us = median_us(lambda: xnor.xnor_bwn_split(x, parts, n, c, h, w_))
            bwn_us = median_us(lambda: xnor.xnor_bwn_conv2d(parts, wimg, alpha, out, desc))
            flops = 2.0 * layer.bit_macs
            row = (f"| {cfg} / {layer.name} | {split_us:.1f} | {bwn_us:.1f} | {3 * flops / bwn_us / 1e6:.0f} | "
                   f"{100 * 3 * flops / bwn_us / 1e6 / 2500:.1f} | {flops / bwn_us / 1e6:.0f} |")
            if st == 1:
                Kp = torch.rand((n, ho, wo), device="cuda", generator=gen) + 0.5
                kw32 = xnor.words_per_pixel(k)
                wtbits = torch.empty((c, kh * kw, kw32), dtype=torch.int32, device="cuda")
                wtmfma = u8(xnor.wmfma_bytes(c, k, kh, kw))
                ones, gmax = torch.empty((c,), device="cuda"), torch.empty((n,), device="cuda")
                gbits = torch.empty((n, ho, wo, kw32), dtype=torch.int32, device="cuda")
                plane, gin = torch.empty((n, h, w_), device="cuda"), torch.empty((n, c, h, w_), device="cuda")
                xnor.xnor_bingrad_pack_weights(wt, wtbits, ones, wtmfma, k, c, kh, kw)
                gb_us = median_us(lambda: xnor.xnor_bingrad_binarize(out, Kp, alpha, gbits, gmax, desc))
                gc_us = median_us(lambda: xnor.xnor_bingrad_conv2d(gbits, wtbits, wtmfma, gmax, ones, plane, gin, None,
                                                                   desc, xnor.XNOR_ALGO_AUTO))
                row += f" {gb_us:.1f} | {gc_us:.1f} | {layer.bit_macs / gc_us / 1e6:.0f} |"
            else:
                row += " - | - | - |"
            # 2-bit inputs x 2-bit weights (inputs scaled into [-1, 1])
            xs = torch.tanh(x)
            xq, wq2 = u8(xnor.kbit_input_bytes(n, c, h, w_)), u8(xnor.kbit_wimg_bytes(k, c, kh, kw))
            scale2 = torch.empty((k,), device="cuda")
            xnor.xnor_kbit_pack_weights(torch.tanh(wt), scale2, wq2, 2, 2, k, c, kh, kw)
            kp_us = median_us(lambda: xnor.xnor_kbit_pack_input(xs, xq, 2, n, c, h, w_))
            kc_us = median_us(lambda: xnor.xnor_kbit_conv2d(xq, wq2, scale2, out, None, desc, 2, 2))
            row += f" {kp_us:.1f} | {kc_us:.1f} |"
            del xq, wq2
            # max-pool 3x3 stride 2 of this layer's output fused into the next block's BinActiv
            if ho >= 3 and wo >= 3:
                hp_, wp_ = (ho - 3) // 2 + 1, (wo - 3) // 2 + 1
                pb = torch.empty((n, hp_, wp_, xnor.words_per_pixel(k)), dtype=torch.int32, device="cuda")
                pa = torch.empty((n, hp_, wp_), device="cuda")
                pl_us = median_us(lambda: xnor.xnor_pool_binactiv(out, None, None, pb, pa, n, k, ho, wo, (3, 3), (2, 2)))
                row += f" {pl_us:.1f} |"
            else:
                row += " - |"
            print(row, flush=True)
    # the oracle on one thread, tiny configuration (the other oracle figures use every host thread)
    import ctypes
    gomp = ctypes.CDLL("libgomp.so.1")
    nthreads = xo.threads()
    tiny = wl.config_layers("tiny")[0]
    dt_in = wl.conv_inputs(tiny, wl.config_seed("tiny"))
    gomp.omp_set_num_threads(1)
    t0 = time.perf_counter()
    for _ in range(20):
        xo.binary_conv2d(dt_in["x"], dt_in["w"], (tiny.stride, tiny.stride), (tiny.pad, tiny.pad))
    one = 20 * tiny.bit_macs / (time.perf_counter() - t0) / 1e9
    gomp.omp_set_num_threads(nthreads)
    print(f"\nOracle on one thread, tiny configuration: {one:.2f} Gbinop/s.  One binop = one +-1 multiply-accumulate; "
          "counting XNOR and bitcount as two operations doubles every Tbinop/s figure above.")
    print(f"Oracle: {xo.threads()} host threads.  % attainable = floor time at min(fp4 peak, arithmetic "
          "intensity x 8 TB/s) / measured time.  The paper's own figures: 58x measured, 62.27x modelled speed-up of "
          "binary over float convolution on its CPU, memory access excluded (sec. 4.1).")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="alexnet_conv2",
                    choices=["tiny", "alexnet_conv2", "alexnet_conv345", "resnet18"])
    ap.add_argument("--algo", default="fastest", choices=["fastest", "popcount", "mfma_i8", "mfma_f4"],
                    help="inner loop of the binary convolution; 'fastest' times all three and keeps the winner")
    ap.add_argument("--chain", default="none", choices=["none", "layerwise", "fused"],
                    help="alexnet_conv345 only: feed each layer the previous layer's output instead of its own "
                         "synthetic input; 'layerwise' = xnor_binactiv + xnor_conv2d per layer, 'fused' = one "
                         "xnor_binactiv, then xnor_conv2d_binactiv emits the next layer's bits and A directly")
    ap.add_argument("--report", action="store_true",
                    help="print a per-layer table over all configurations instead of the one JSON line")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy, so a rocprofv3 --pmc run of this command holds "
                         "a kernel of known HBM traffic to scale FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.chain != "none" and args.workload != "alexnet_conv345":
        sys.exit("bench.py: --chain needs --workload alexnet_conv345 (the only workload whose layers feed each other)")
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path shards over the batch with no "
                 "exchange step, each GPU running these same kernels on its share of the images). Run with --gpus 1.")

    import torch
    from paper_1603_05279_amd import workloads as wl
    from paper_1603_05279_amd import xnor

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    if args.report:
        report(args)
        return
    torch.cuda.set_device(0)
    layers = wl.config_layers(args.workload)
    inputs = [wl.conv_inputs(l, wl.config_seed(args.workload, i)) for i, l in enumerate(layers)]

    # device state: inputs, packed weights, preallocated activation buffers
    dev = []
    pack_ms = 0.0
    for layer, d in zip(layers, inputs):
        x = torch.from_numpy(d["x"]).cuda()
        w = torch.from_numpy(d["w"]).cuda()
        sc = torch.from_numpy(d["bn_scale"]).cuda() if d["bn_scale"] is not None else None
        sf = torch.from_numpy(d["bn_shift"]).cuda() if d["bn_shift"] is not None else None
        desc = xnor.make_desc(layer.n, layer.c, layer.h, layer.w, layer.k_out, layer.kh, layer.kw,
                              layer.stride, layer.pad)
        pw = xnor.PackedWeights(w)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        xnor.xnor_pack_weights(w, pw.wbits, pw.alpha, pw.wmfma, *pw.shape)
        e1.record()
        torch.cuda.synchronize()
        pack_ms += e0.elapsed_time(e1)
        dev.append((x, sc, sf, pw, xnor.ConvBuffers(desc)))

    def conv_only_ms(name, iters=10):
        """Average conv-kernel time of one pass over all layers with inner loop `name` (HIP events)."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for it in range(iters + 2):
            if it == 2:
                e0.record()
            for (x, sc, sf, pw, bufs) in dev:
                xnor.xnor_conv2d(bufs.xbits, pw.wbits, pw.wmfma, None, bufs.A, pw.alpha, bufs.out, None, bufs.desc,
                                 xnor.ALGOS[name])
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    for (x, sc, sf, pw, bufs) in dev:
        xnor.xnor_binactiv(x, sc, sf, bufs.xbits, bufs.A, None, bufs.desc)
    compare = {name: conv_only_ms(name) for name in ("popcount", "mfma_i8", "mfma_f4")}
    used = min(compare, key=compare.get) if args.algo == "fastest" else args.algo
    if args.chain == "fused" and used == "popcount":
        sys.exit("bench.py: the fused epilogue exists in the matrix-core kernels only (--algo mfma_f4 or mfma_i8)")
    algo = xnor.ALGOS[used]

    workspaces = [torch.empty((max(16, xnor.conv2d_binactiv_workspace_bytes(b.desc)),), dtype=torch.uint8,
                              device="cuda") for (_, _, _, _, b) in dev] if args.chain == "fused" else None

    def step(events=None):
        for i, (x, sc, sf, pw, bufs) in enumerate(dev):
            last = i + 1 == len(dev)
            if args.chain == "none":
                xnor.xnor_binactiv(x, sc, sf, bufs.xbits, bufs.A, None, bufs.desc)
            elif args.chain == "layerwise" or i == 0:
                src = x if i == 0 else dev[i - 1][4].out
                xnor.xnor_binactiv(src, sc, sf, bufs.xbits, bufs.A, None, bufs.desc)
            if events is not None:
                events[i][0].record()
            if args.chain == "fused" and not last:
                nxt = dev[i + 1]
                xnor.xnor_conv2d_binactiv(bufs.xbits, pw.wbits, pw.wmfma, None, bufs.A, pw.alpha, nxt[1], nxt[2],
                                          nxt[4].xbits, nxt[4].A, None, workspaces[i], bufs.desc, algo)
            else:
                xnor.xnor_conv2d(bufs.xbits, pw.wbits, pw.wmfma, None, bufs.A, pw.alpha, bufs.out, None, bufs.desc,
                                 algo)
            if events is not None:
                events[i][1].record()

    if args.copy_calibration:
        src = torch.empty(256 * 1024 * 1024 // 4, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # HIP events around the convolution launch on every 8th step only: an event record is a stream
    # command of its own and costs about 3 us, which would otherwise inflate every step by 6 us
    sampled = [s for s in range(args.steps) if s % 8 == 0]
    ev = {s: [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in dev]
          for s in sampled}
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(ev.get(s))
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    macs = sum(l.bit_macs for l in layers)
    ms_per_step = dt / args.steps * 1e3
    # dominant kernel = the binary convolution; average launch duration from the HIP events
    conv_ms = [sum(ev[s][i][0].elapsed_time(ev[s][i][1]) for s in sampled) / len(sampled)
               for i in range(len(dev))]
    dom = max(range(len(dev)), key=lambda i: conv_ms[i])
    pk = PEAKS[used]
    per_mac = 1.0 if used == "popcount" else 2.0
    sec = conv_ms[dom] * 1e-3
    compute = {"bound": pk["bound"], "achieved": layers[dom].bit_macs * per_mac / sec / 1e12, "peak": pk["peak"],
               "unit": pk["unit"]}
    dom_fused = args.chain == "fused" and dom + 1 < len(dev)
    hbm = {"bound": "hbm", "achieved": algo_bytes(layers[dom], dom_fused) / sec / 1e9, "peak": 8000.0,
           "unit": "GB/s"}
    for r in (compute, hbm):
        r["frac"] = r["achieved"] / r["peak"]
    # the binding roof is the one whose floor time at the published peak is longer; at the same measured
    # duration that is the one with the larger fraction.  The other one is reported next to it.
    bind, other = (hbm, compute) if hbm["frac"] >= compute["frac"] else (compute, hbm)
    roofline = dict(bind)
    roofline.update({"traffic": MEASURED_TRAFFIC.get((args.workload, used)),
                     "algorithmic_bytes": algo_bytes(layers[dom], dom_fused),
                     "kernel": f"{'xnor_conv2d_binactiv' if dom_fused else 'xnor_conv2d'}[{layers[dom].name}]",
                     "other_roof": other})
    out = {
        "metric": "binary conv throughput (Gbinop/s) + % of popcount/MFMA roofline",
        "value": macs / (dt / args.steps) / 1e9, "unit": "Gbinop/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"mfma_f4": "fp4", "mfma_i8": "i8", "popcount": "u32"}[used], "data": "synthetic",
        "config": {"workload": args.workload, "layers": [l.name for l in layers], "batch": layers[0].n,
                   "algo": used, "algo_conv_ms": compare, "step": {"none": "xnor_binactiv + xnor_conv2d per layer, each layer on its own synthetic input",
                            "layerwise": "xnor_binactiv + xnor_conv2d per layer, each layer on the previous output",
                            "fused": "xnor_binactiv, then xnor_conv2d_binactiv per layer (plain xnor_conv2d last)"
                            }[args.chain],
                   "conv_ms": conv_ms, "pack_weights_ms_once": pack_ms,
                   "conv_only_Gbinop_s": [l.bit_macs / (t * 1e-3) / 1e9 for l, t in zip(layers, conv_ms)]},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(layers, inputs)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
