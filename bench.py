"""Benchmark of the XNOR-Net binary convolution block on one MI355X.

One step = one pass of the hot path over one batch of every layer of the workload, inputs resident in HBM:
    xnor_binactiv (BatchNorm fold, sign + bit-pack, A)  ->  xnor_conv2d / xnor_linear (binary dot, K from A, K*alpha).
The default workload is all five benchmark configurations (ten layers).  Weights are packed once before the
timed region (at inference only B and alpha exist; the packing time is reported separately).

Buffers: by default every layer owns a ring of input / packed / output buffer sets whose total exceeds three
times the chip's 256 MB last-level cache and each step uses the next set, so that what is timed moves through
HBM ("cold"); `--buffers fixed` re-uses one set (the "warm" figure is reported in the same line either way).

Prints ONE JSON line on stdout:  value = whole-step throughput; `layers` = per-layer kernel times (HIP events
around >= 50 back-to-back launches, independent of --steps) with their roofline fractions; `roofline` = the
binary convolution kernel over all its launches of a step; `measured_peaks` = what this GPU delivers on the
register-only inner loops and on streaming (xnor_ubench); `cpu_baseline` = the CPU oracle on the same inputs.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all] [--buffers rotating]
    python bench.py --report            # markdown tables instead of the JSON line
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PEAKS = {  # MI355X published dense peaks
    "mfma_f4": {"bound": "mfma", "peak": 10100.0, "unit": "TFLOP/s", "per_mac": 2.0},   # fp4 10.1 PFLOP/s
    "mfma_i8": {"bound": "mfma", "peak": 5000.0, "unit": "TOP/s", "per_mac": 2.0},      # int8 5.0 POP/s
    # vector ALU: 2 instructions (XOR, bitcount-accumulate) per 32 binary MACs:
    # 256 CUs x 64 lanes x 2.4 GHz x 16 MAC per lane-instruction
    "popcount": {"bound": "alu", "peak": 256 * 64 * 2.4e9 * 16 / 1e12, "unit": "Tbinop/s", "per_mac": 1.0},
}
LLC_BYTES = 256 << 20          # last-level cache of the chip; rotating rings hold at least three times this
WORKLOADS = ["all", "tiny", "alexnet_conv2", "alexnet_conv345", "resnet18", "fc"]

# HBM bytes per launch of the convolution kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (each
# scaled by the same counter over a plain copy of known size); source: the named file under profiles/.
# None = not profiled.
PROFILED_TRAFFIC = {
    "tiny_64x14x14_k3": 386648, "alexnet_conv2": 56262886, "alexnet_conv3": 42855315, "alexnet_conv4": 43883570,
    "alexnet_conv5": 28248434, "resnet18_64x56": 216580891, "resnet18_128x28": 121813565, "resnet18_256x14": 60139770,
    "resnet18_512x7": 39470434, "fc_9216x4096": 25778613,
}
PROFILED_TRAFFIC_SOURCE = "profiles/conv_hbm_traffic.md"


class Shape:
    """One layer as the kernels see it (a fully connected layer is the 1x1 image with in_features channels)."""

    def __init__(self, cfg, idx, layer):
        self.cfg, self.idx, self.layer, self.name = cfg, idx, layer, layer.name
        self.fc = cfg == "fc"
        if self.fc:
            self.n, self.c, self.h, self.w = layer.batch, layer.in_features, 1, 1
            self.k, self.kh, self.kw, self.stride, self.pad = layer.out_features, 1, 1, 1, 0
        else:
            self.n, self.c, self.h, self.w = layer.n, layer.c, layer.h, layer.w
            self.k, self.kh, self.kw, self.stride, self.pad = layer.k_out, layer.kh, layer.kw, layer.stride, layer.pad
        self.ho = (self.h + 2 * self.pad - self.kh) // self.stride + 1
        self.wo = (self.w + 2 * self.pad - self.kw) // self.stride + 1
        self.cw = (self.c + 31) // 32
        self.macs = layer.bit_macs

    def conv_bytes(self, fused=False):
        """Algorithmic bytes of one xnor_conv2d launch: packed activations, packed 1-bit weights, the K map,
        the float output (fused epilogue: the next block's sign words and A instead)."""
        m = self.n * self.ho * self.wo
        result = m * ((self.k + 31) // 32 * 4 + 4) if fused else m * self.k * 4
        return self.n * self.h * self.w * self.cw * 4 + self.k * self.kh * self.kw * self.cw * 4 + m * 4 + result

    def binactiv_bytes(self):
        """Algorithmic bytes of one xnor_binactiv launch: the float input once, sign words and A out."""
        px = self.n * self.h * self.w
        return px * self.c * 4 + px * self.cw * 4 + px * 4

    def roofs(self, seconds, algo="mfma_f4", fused=False):
        pk = PEAKS[algo]
        comp = {"bound": pk["bound"], "achieved": self.macs * pk["per_mac"] / seconds / 1e12, "peak": pk["peak"],
                "unit": pk["unit"]}
        hbm = {"bound": "hbm", "achieved": self.conv_bytes(fused) / seconds / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
        for r in (comp, hbm):
            r["frac"] = r["achieved"] / r["peak"]
        # the binding roof is the one with the longer floor time, i.e. the larger fraction at the same duration
        return (hbm, comp) if hbm["frac"] >= comp["frac"] else (comp, hbm)


def workload_shapes(wl, name):
    cfgs = ["tiny", "alexnet_conv2", "alexnet_conv345", "resnet18", "fc"] if name == "all" else [name]
    return [Shape(c, i, l) for c in cfgs for i, l in enumerate(wl.config_layers(c))]


class LayerState:
    """Device tensors of one layer: the synthetic input, packed weights and a ring of buffer sets."""

    def __init__(self, torch, wl, xnor, sh, ring_bytes):
        seed = wl.config_seed(sh.cfg, sh.idx)
        self.sh = sh
        if sh.fc:
            d = wl.linear_inputs(sh.layer, seed)
            x = torch.from_numpy(d["x"]).reshape(sh.n, sh.c, 1, 1)
            w = torch.from_numpy(d["w"]).reshape(sh.k, sh.c, 1, 1)
            d = {"x": d["x"], "w": d["w"], "bn_scale": None, "bn_shift": None}
        else:
            d = wl.conv_inputs(sh.layer, seed)
            x, w = torch.from_numpy(d["x"]), torch.from_numpy(d["w"])
        self.host = d
        self.sc = torch.from_numpy(d["bn_scale"]).cuda() if d["bn_scale"] is not None else None
        self.sf = torch.from_numpy(d["bn_shift"]).cuda() if d["bn_shift"] is not None else None
        self.desc = xnor.make_desc(sh.n, sh.c, sh.h, sh.w, sh.k, sh.kh, sh.kw, sh.stride, sh.pad)
        wdev = w.cuda()
        pw = xnor.PackedWeights(wdev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        xnor.xnor_pack_weights(wdev, pw.wbits, pw.alpha, pw.wmfma, *pw.shape)
        e0.record()
        xnor.xnor_pack_weights(wdev, pw.wbits, pw.alpha, pw.wmfma, *pw.shape)
        e1.record()
        torch.cuda.synchronize()
        self.pack_ms = e0.elapsed_time(e1)
        per_set = x.numel() * 4 + sh.n * sh.h * sh.w * (sh.cw * 4 + 4) + sh.n * sh.k * sh.ho * sh.wo * 4
        w_bytes = pw.wmfma.numel() + pw.wbits.numel() * 4
        rotate_w = ring_bytes > 0 and w_bytes > per_set            # weight-heavy layers (FC) rotate their weights too
        if rotate_w:
            per_set += w_bytes
        self.ring = 1 if ring_bytes <= 0 else max(2, min(24, -(-ring_bytes // per_set)))
        xd = x.cuda()
        self.x = [xd] + [xd.clone() for _ in range(self.ring - 1)]
        self.bufs = [xnor.ConvBuffers(self.desc) for _ in range(self.ring)]
        self.pw = [pw]
        for _ in range(self.ring - 1 if rotate_w else 0):
            q = xnor.PackedWeights(wdev)
            q.wbits.copy_(pw.wbits), q.alpha.copy_(pw.alpha), q.wmfma.copy_(pw.wmfma)
            self.pw.append(q)
        del wdev
        self.xnor = xnor

    def binactiv(self, r):
        b = self.bufs[r % self.ring]
        # every layer's input comes from memory (its ring, or nothing has touched it since the previous step's nine
        # other layers): the entry point for inputs that are in no cache
        self.xnor.xnor_binactiv_streamed(self.x[r % self.ring], self.sc, self.sf, b.xbits, b.A, None, self.desc)

    def conv(self, r, algo):
        b, pw, sh, xn = self.bufs[r % self.ring], self.pw[r % len(self.pw)], self.sh, self.xnor
        if sh.fc:       # K of a 1x1 filter over a 1x1 image is A itself
            xn.xnor_linear(b.xbits, pw.wbits, pw.wmfma, b.A, pw.alpha, b.out, None, sh.n, sh.c, sh.k, algo)
        else:
            xn.xnor_conv2d(b.xbits, pw.wbits, pw.wmfma, None, b.A, pw.alpha, b.out, None, self.desc, algo)


def event_us(torch, fn, launches):
    """Average duration of `launches` back-to-back calls fn(i) between two HIP events on the current stream."""
    for i in range(min(10, launches)):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(launches):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / launches


def measured_peaks(torch, xnor):
    """What this GPU delivers on the register-only inner loops and on streaming (xnor_ubench), next to the
    published peaks the fractions are quoted against."""
    buf = torch.empty((1 << 30) + (256 << 20), dtype=torch.uint8, device="cuda")
    out = {}
    wgs, iters = 2048, 2000            # two waves per SIMD, about 0.3 ms per launch
    us = event_us(torch, lambda i: xnor.ubench("mfma_f4", wgs, iters, buf), 20)
    out["mfma_f4_TFLOP_s"] = wgs * 4 * iters * 8 * 2.0 * 32 * 32 * 64 / us / 1e6
    # the same loop on operands that change with every instruction, sustained and as a burst of one convolution's length
    us = event_us(torch, lambda i: xnor.ubench("mfma_f4_data", wgs, iters, buf), 20)
    out["mfma_f4_changing_operands_TFLOP_s"] = wgs * 4 * iters * 8 * 2.0 * 32 * 32 * 64 / us / 1e6
    torch.cuda.synchronize()
    clk = buf[:16].view(torch.int64).cpu()
    out["core_clock_GHz_sustained_mfma"] = round(float(clk[0]) / (float(clk[1]) * 10.0), 3)
    event_us(torch, lambda i: xnor.ubench("mfma_f4_data", 512, 30, buf), 20)
    torch.cuda.synchronize()
    clk = buf[:16].view(torch.int64).cpu()
    out["core_clock_GHz_10us_mfma_bursts"] = round(float(clk[0]) / (float(clk[1]) * 10.0), 3)
    # 16-byte loads of a 4 MiB buffer that stays in L2, 64 KiB per workgroup and pass (the weight stream of the convolution)
    us = event_us(torch, lambda i: xnor.ubench("l2_read", 2048, 64, buf, 4 << 20), 20)
    out["l2_read_GB_s"] = 2048 * 64 * 65536 / us / 1e3
    out["l2_read_bytes_per_clock_per_cu_at_2.4GHz"] = round(2048 * 64 * 65536 / (us * 1e-6) / 256 / 2.4e9, 1)
    us = event_us(torch, lambda i: xnor.ubench("mfma_i8", wgs, iters, buf), 20)
    out["mfma_i8_TOP_s"] = wgs * 4 * iters * 8 * 2.0 * 32 * 32 * 32 / us / 1e6
    us = event_us(torch, lambda i: xnor.ubench("popcount", wgs, 500, buf), 20)
    out["valu_xor_bitcount_Tbinop_s"] = wgs * 256 * 500 * 128 * 32.0 / us / 1e6
    for name, nbytes in (("48MiB_llc_resident", 48 << 20), ("1GiB_through_hbm", 1 << 30)):
        for kind, moved in (("fill", nbytes), ("fill_nt", nbytes), ("read", nbytes), ("copy", nbytes)):
            us = event_us(torch, lambda i: xnor.ubench(kind, 4096, 0, buf, nbytes), 30)
            out[f"{kind}_{name}_GB_s"] = moved / us / 1e3
    out["note"] = ("copy moves bytes/2 from the first half to the second (read + write counted); the 48 MiB figures "
                   "stay in the 256 MB last-level cache, the 1 GiB ones pass through HBM; fill_nt stores with the "
                   "non-temporal hint")
    del buf
    return out


def cpu_baseline(states):
    """The oracle as it stands, whole block per layer, on this machine's host cores."""
    from oracle import xnor_oracle as xo
    first = states[0]
    xo.binary_conv2d(first.host["x"].reshape(first.sh.n, first.sh.c, first.sh.h, first.sh.w)[:1],
                     first.host["w"].reshape(first.sh.k, first.sh.c, first.sh.kh, first.sh.kw), (1, 1), (0, 0))
    t0 = time.perf_counter()
    macs = 0
    for st in states:
        sh, d = st.sh, st.host
        if sh.fc:
            xo.binary_linear(d["x"], d["w"])
        else:
            xo.binary_conv2d(d["x"], d["w"], (sh.stride,) * 2, (sh.pad,) * 2, d["bn_scale"], d["bn_shift"])
        macs += sh.macs
    dt = time.perf_counter() - t0
    return {"value": macs / dt / 1e9, "unit": "Gbinop/s", "cores": xo.threads(), "kind": "oracle",
            "sample": f"the full workload once ({len(states)} layer(s), {macs / 1e9:.1f} G binop), {dt:.2f} s wall"}


def chain_config3(torch, wl, xnor, launches, profile_runs=0):
    """Config 3 as the chain it is: block i+1 consumes block i's output.  Layer by layer (xnor_binactiv +
    xnor_conv2d per block) against the fused form (one xnor_binactiv, then xnor_conv2d_binactiv emits the next
    block's sign words and A; the float tensor between the blocks is never written)."""
    shapes = workload_shapes(wl, "alexnet_conv345")
    sts = [LayerState(torch, wl, xnor, sh, 0) for sh in shapes]
    ws = [torch.empty((max(16, xnor.conv2d_binactiv_workspace_bytes(s.desc)),), dtype=torch.uint8, device="cuda")
          for s in sts]
    f4 = xnor.XNOR_ALGO_MFMA_F4

    def layerwise(_):
        for i, s in enumerate(sts):
            b = s.bufs[0]
            xnor.xnor_binactiv(s.x[0] if i == 0 else sts[i - 1].bufs[0].out, s.sc, s.sf, b.xbits, b.A, None, s.desc)
            xnor.xnor_conv2d(b.xbits, s.pw[0].wbits, s.pw[0].wmfma, None, b.A, s.pw[0].alpha, b.out, None, s.desc, f4)

    def fused(_):
        s0 = sts[0]
        xnor.xnor_binactiv(s0.x[0], s0.sc, s0.sf, s0.bufs[0].xbits, s0.bufs[0].A, None, s0.desc)
        for i, s in enumerate(sts):
            b, pw = s.bufs[0], s.pw[0]
            if i + 1 < len(sts):
                nx = sts[i + 1]
                xnor.xnor_conv2d_binactiv(b.xbits, pw.wbits, pw.wmfma, None, b.A, pw.alpha, nx.sc, nx.sf,
                                          nx.bufs[0].xbits, nx.bufs[0].A, None, ws[i], s.desc, f4)
            else:
                xnor.xnor_conv2d(b.xbits, pw.wbits, pw.wmfma, None, b.A, pw.alpha, b.out, None, s.desc, f4)

    if profile_runs:           # rocprofv3 runs: the fused chain alone
        for i in range(profile_runs):
            fused(i)
        torch.cuda.synchronize()
        return None
    macs = sum(s.sh.macs for s in sts)
    res = {"G_binop": macs / 1e9}
    for name, fn in (("layerwise", layerwise), ("fused", fused)):
        us = event_us(torch, fn, launches)
        res[name + "_us"] = us
        res[name + "_Tbinop_s"] = macs / us / 1e6
    # the fused convolution kernel alone (no float output: bound by the matrix cores)
    per = []
    for i, s in enumerate(sts[:-1]):
        b, pw, nx = s.bufs[0], s.pw[0], sts[i + 1]
        us = event_us(torch, lambda _: xnor.xnor_conv2d_binactiv(b.xbits, pw.wbits, pw.wmfma, None, b.A, pw.alpha, nx.sc,
                                                                 nx.sf, nx.bufs[0].xbits, nx.bufs[0].A, None, ws[i],
                                                                 s.desc, f4), launches)
        bind, other = s.sh.roofs(us * 1e-6, "mfma_f4", fused=True)
        per.append({"layer": s.sh.name, "conv2d_binactiv_us": us, "bound": bind["bound"], "frac": bind["frac"],
                    "other_frac": other["frac"]})
    res["conv2d_binactiv"] = per
    return res


def bwn_conv2_profile(torch, wl, xnor, runs):
    """rocprofv3 runs: the Binary-Weight-Network convolution (sec. 3.1) on the alexnet_conv2 shape,
    xnor_bwn_split + xnor_bwn_conv2d per run."""
    sh = workload_shapes(wl, "alexnet_conv2")[0]
    d = wl.conv_inputs(sh.layer, wl.config_seed("alexnet_conv2"))
    x, w = torch.from_numpy(d["x"]).cuda(), torch.from_numpy(d["w"]).cuda()
    desc = xnor.make_desc(sh.n, sh.c, sh.h, sh.w, sh.k, sh.kh, sh.kw, sh.stride, sh.pad)
    parts = torch.empty((xnor.bwn_parts_bytes(sh.n, sh.c, sh.h, sh.w),), dtype=torch.uint8, device="cuda")
    wimg = torch.empty((xnor.bwn_wimg_bytes(sh.k, sh.c, sh.kh, sh.kw),), dtype=torch.uint8, device="cuda")
    alpha = torch.empty((sh.k,), dtype=torch.float32, device="cuda")
    out = torch.empty((sh.n, sh.k, sh.ho, sh.wo), dtype=torch.float32, device="cuda")
    xnor.xnor_bwn_pack_weights(w, alpha, wimg, sh.k, sh.c, sh.kh, sh.kw)
    for _ in range(runs):
        xnor.xnor_bwn_split(x, parts, sh.n, sh.c, sh.h, sh.w)
        xnor.xnor_bwn_conv2d(parts, wimg, alpha, out, desc)
    torch.cuda.synchronize()


def measure_layers(torch, xnor, states, launches, compare_algos=True):
    """Per-layer kernel times, independent of --steps: `launches` back-to-back launches between HIP events."""
    rows = []
    f4 = xnor.XNOR_ALGO_MFMA_F4
    for st in states:
        sh = st.sh
        for r in range(st.ring):
            st.binactiv(r)
        row = {"config": sh.cfg, "layer": sh.name, "G_binop": sh.macs / 1e9, "ring": st.ring}
        row["conv_us"] = event_us(torch, lambda i: st.conv(i, f4), launches)                    # through the ring
        row["conv_us_warm"] = event_us(torch, lambda i: st.conv(0, f4), launches)               # one buffer set
        row["binactiv_us"] = event_us(torch, lambda i: st.binactiv(i), launches)
        row["binactiv_us_warm"] = event_us(torch, lambda i: st.binactiv(0), launches)
        if compare_algos:
            row["conv_us_warm_mfma_i8"] = event_us(torch, lambda i: st.conv(0, xnor.XNOR_ALGO_MFMA_I8), launches)
            row["conv_us_warm_popcount"] = event_us(torch, lambda i: st.conv(0, xnor.XNOR_ALGO_POPCOUNT), launches)
        sec = row["conv_us"] * 1e-6
        bind, other = sh.roofs(sec)
        row.update({"Tbinop_s": sh.macs / sec / 1e12, "algorithmic_bytes": sh.conv_bytes(),
                    "flop": 2.0 * sh.macs, "bound": bind["bound"], "frac": bind["frac"],
                    "other_roof": other["bound"], "other_frac": other["frac"],
                    "frac_warm": sh.roofs(row["conv_us_warm"] * 1e-6)[0]["frac"],
                    "binactiv_GB_s": sh.binactiv_bytes() / row["binactiv_us"] / 1e3,
                    "pack_weights_ms_once": st.pack_ms,
                    "profiled_hbm_bytes": PROFILED_TRAFFIC.get(sh.name)})
        rows.append(row)
    return rows


def print_report(rows, peaks, chain, cpu):
    print("Measured peaks (xnor_ubench): " + ", ".join(f"{k} {v:.0f}" if v >= 100 else f"{k} {v:.3g}" for k, v in peaks.items() if k != "note"))
    print("\n| config / layer | G binop | conv fp4 us (ring) | conv fp4 us (one set) | conv int8 us | conv popcount us | "
          "BinActiv us (ring) | Tbinop/s | alg. MB | bound | frac of bound | frac of other roof | BinActiv GB/s | pack ms |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    for r in rows:
        print(f"| {r['config']} / {r['layer']} | {r['G_binop']:.2f} | {r['conv_us']:.1f} | {r['conv_us_warm']:.1f} | "
              f"{r.get('conv_us_warm_mfma_i8', float('nan')):.1f} | {r.get('conv_us_warm_popcount', float('nan')):.1f} | "
              f"{r['binactiv_us']:.1f} | {r['Tbinop_s']:.0f} | {r['algorithmic_bytes'] / 1e6:.1f} | {r['bound']} | "
              f"{r['frac']:.3f} | {r['other_frac']:.3f} | {r['binactiv_GB_s']:.0f} | {r['pack_weights_ms_once']:.3f} |")
    if chain:
        print(f"\nConfig 3 as a chain ({chain['G_binop']:.2f} G binop): layer by layer {chain['layerwise_us']:.1f} us, "
              f"fused {chain['fused_us']:.1f} us; xnor_conv2d_binactiv alone: " +
              ", ".join(f"{p['layer']} {p['conv2d_binactiv_us']:.1f} us ({p['bound']} {p['frac']:.3f})"
                        for p in chain["conv2d_binactiv"]))
    if cpu:
        print(f"\nCPU oracle: {cpu['value']:.1f} Gbinop/s on {cpu['cores']} threads ({cpu['sample']}).")
    print("\nring = rotating buffer sets (HBM), one set = re-used buffers (last-level cache).  frac = achieved / "
          "published peak of the binding roof (HBM 8 TB/s on algorithmic bytes, or fp4 matrix cores 10.1 PFLOP/s).  "
          "One binop = one +-1 multiply-accumulate.  The paper's own figures: 58x measured, 62.27x modelled "
          "speed-up of binary over float convolution on its CPU, memory access excluded (sec. 4.1).")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="all", choices=WORKLOADS)
    ap.add_argument("--algo", default="mfma_f4", choices=["auto", "popcount", "mfma_i8", "mfma_f4"],
                    help="inner loop of the binary convolution in the timed step")
    ap.add_argument("--buffers", default="rotating", choices=["rotating", "fixed"],
                    help="rotating: each step uses the next of a ring of buffer sets larger than the last-level cache")
    ap.add_argument("--launches", type=int, default=60, help="back-to-back launches per per-layer kernel timing")
    ap.add_argument("--report", action="store_true", help="markdown tables instead of the JSON line")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-pass", action="store_true",
                    help="for rocprofv3 runs: three 256 MiB calibration copies (xnor_ubench), then only the warm-up and "
                         "timed steps; prints a short JSON line and skips every other measurement")
    ap.add_argument("--profile-extra", action="store_true",
                    help="with --profile-pass: instead of the steps, --steps runs of the fused config-3 chain "
                         "(xnor_binactiv, two xnor_conv2d_binactiv, xnor_conv2d), then of xnor_bwn_split + xnor_bwn_conv2d "
                         "on the alexnet_conv2 shape")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip measured peaks, the inner-loop comparison and the config-3 chain (profiling runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path shards over the batch with no "
                 "exchange step, each GPU running these same kernels on its share of the images). Run with --gpus 1.")

    import torch
    from paper_1603_05279_amd import workloads as wl
    from paper_1603_05279_amd import xnor

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    torch.cuda.set_device(0)
    shapes = workload_shapes(wl, args.workload)
    ring_bytes = 3 * LLC_BYTES if args.buffers == "rotating" else 0
    states = [LayerState(torch, wl, xnor, sh, ring_bytes) for sh in shapes]
    algo = xnor.ALGOS[args.algo]

    def step(s):
        for st in states:
            st.binactiv(s)
            st.conv(s, algo)

    def timed(nsteps, offset):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(nsteps):
            step(offset + s)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    if args.profile_pass:
        # a kernel of known HBM traffic for scaling FETCH_SIZE / WRITE_SIZE: reads 128 MiB, writes 128 MiB
        cal = torch.empty((256 << 20,), dtype=torch.uint8, device="cuda")
        for _ in range(3):
            xnor.ubench("copy", 4096, 0, cal)
        torch.cuda.synchronize()
        del cal
        if args.profile_extra:
            chain_config3(torch, wl, xnor, 0, profile_runs=args.steps)
            bwn_conv2_profile(torch, wl, xnor, args.steps)
            print(json.dumps({"profile_pass": True, "profile_extra": True, "runs": args.steps,
                              "fused_chain_launches_per_run": "xnor_binactiv, xnor_conv2d_binactiv x2 (each + sum_planes), "
                              "xnor_conv2d", "bwn_launches_per_run": "xnor_bwn_split, xnor_bwn_conv2d"}))
            return
    for s in range(args.warmup):
        step(s)
    dt = timed(args.steps, args.warmup)
    macs = sum(sh.macs for sh in shapes)
    if args.profile_pass:
        print(json.dumps({"profile_pass": True, "workload": args.workload, "buffers": args.buffers,
                          "layers": [sh.name for sh in shapes], "rings": [st.ring for st in states],
                          "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
                          "kernels_per_step": 2 * len(shapes)}))
        return
    # the same steps on one buffer set (served by the last-level cache where the layer fits it)
    for s in range(min(args.warmup, 5)):
        for st in states:
            st.binactiv(0), st.conv(0, algo)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        for st in states:
            st.binactiv(0), st.conv(0, algo)
    torch.cuda.synchronize()
    dt_warm = time.perf_counter() - t0

    rows = measure_layers(torch, xnor, states, max(50, args.launches), compare_algos=not args.no_extras)
    peaks = None if args.no_extras else measured_peaks(torch, xnor)
    chain = None if args.no_extras else chain_config3(torch, wl, xnor, max(50, args.launches))
    cpu = None if args.no_cpu_baseline else cpu_baseline(states)
    if args.report:
        print_report(rows, peaks or {}, chain, cpu)
        return

    # dominant kernel: the binary convolution, over all its launches of one step
    conv_s = sum(r["conv_us"] for r in rows) * 1e-6
    nbytes, flop = sum(r["algorithmic_bytes"] for r in rows), sum(r["flop"] for r in rows)
    hbm = {"bound": "hbm", "achieved": nbytes / conv_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    mfma = {"bound": "mfma", "achieved": flop / conv_s / 1e12, "peak": PEAKS["mfma_f4"]["peak"], "unit": "TFLOP/s"}
    for r in (hbm, mfma):
        r["frac"] = r["achieved"] / r["peak"]
    bind, other = (hbm, mfma) if hbm["frac"] >= mfma["frac"] else (mfma, hbm)
    traffic = [r["profiled_hbm_bytes"] for r in rows]
    roofline = dict(bind)
    roofline.update({
        "traffic": sum(traffic) if all(t is not None for t in traffic) else None,
        "traffic_source": PROFILED_TRAFFIC_SOURCE + " (rocprofv3 FETCH_SIZE / WRITE_SIZE, not measured in this run)",
        "kernel": "conv_mfma_kernel (xnor_conv2d / xnor_linear, 4-bit-float matrix instructions), all launches of one step",
        "launches_per_step": len(rows), "algorithmic_bytes": nbytes, "flop": flop,
        "avg_launch_us": conv_s * 1e6 / len(rows), "timing": f"HIP events around {max(50, args.launches)} back-to-back "
        "launches per layer, rotating buffer sets" if args.buffers == "rotating" else "HIP events, one buffer set",
        "other_roof": other})
    out = {
        "metric": "binary conv throughput (Gbinop/s) + % of popcount/MFMA roofline",
        "value": macs / (dt / args.steps) / 1e9, "unit": "Gbinop/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"mfma_f4": "fp4", "mfma_i8": "i8", "popcount": "u32", "auto": "fp4"}[args.algo], "data": "synthetic",
        "config": {"workload": "all_five_configs" if args.workload == "all" else args.workload,
                   "layers": [sh.name for sh in shapes], "algo": args.algo,
                   "step": "xnor_binactiv + xnor_conv2d (xnor_linear) per layer, each layer on its own synthetic input",
                   "buffers": (f"rotating rings, >= {3 * LLC_BYTES >> 20} MB per layer (through HBM)"
                               if args.buffers == "rotating" else "one buffer set per layer"),
                   "bn_eps": wl.BN_EPS},
        "value_one_buffer_set": macs / (dt_warm / args.steps) / 1e9,
        "ms_per_step_one_buffer_set": dt_warm / args.steps * 1e3,
        "layers": rows,
        "roofline": roofline,
    }
    if peaks:
        out["measured_peaks"] = peaks
    if chain:
        out["chain_config3"] = chain
    if cpu:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))


if __name__ == "__main__":
    main()
