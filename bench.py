#!/usr/bin/env python3
"""Benchmark of the convolution hot path on one MI355X.

A step is one forward + backward-data + backward-weight pass of one layer
through the C ABI (default: the ResNet-50 3x3 bottleneck layer, N=64,
C=K=256, 14x14), inputs resident in HBM.  Prints ONE JSON line:
whole-step TFLOP/s (nominal 2*N*K*P*Q*Cg*R*S FLOPs per pass), the roofline
figures of the dominant kernel measured with HIP events, the same layer's
figures against the clock the GPU actually ran at, the depthwise layer's
three passes against the HBM peak (`secondary`), and the CPU oracle timed on
the host cores as a baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--layer 2a] [--dtype f32|bf16]
"""
import argparse
import glob
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0, "bf16out": 2500.0}   # dense MFMA, MI355X published
PEAK_HBM_GBS = 8000.0
NUM_CUS = 256
MFMA_FLOP_PER_CLK_PER_CU = {"f32": 256, "bf16": 4096, "bf16out": 4096}   # 157.3 TFLOP/s = 256 CUs x 256 x 2.4 GHz
PASSES = ("fwd", "bwd_data", "bwd_weight")
METRIC = "conv fwd+bwd TFLOP/s and % FP32 MFMA peak (ResNet-50 3x3 layer)"
CSRC = os.path.join(ROOT, "paper_1912_01703_amd", "csrc")
TRAFFIC_PROFILES = ("profiles/conv2d_hbm_traffic_pmc.md", "profiles/conv2d_layer4a_bf16_hbm_traffic_pmc.md")
# The paper's own throughput figures (Section 6.3, Table 1: whole-model training, one Quadro GP100, fp32).
# Another machine and another unit: quoted for context only, never compared with `value`.
PAPER_CONTEXT = {
    "source": "paper Section 6.3, Table 1 (PyTorch row), 2x Xeon E5-2698 v4 + 1x Quadro GP100, fp32, whole-model training",
    "alexnet_images_per_s": 1547, "vgg19_images_per_s": 119, "resnet50_images_per_s": 212,
    "mobilenet_images_per_s": 463, "comparable_to_value": False,
}
# Source files whose change invalidates a stored HBM-traffic figure, per kernel family (the shared header with the
# declarations and the buffer-load helpers is left out: it changes whenever a kernel family is added).
FAMILY_SOURCES = {
    "mfma/tile": ("mfma_tile_kernel.h", "mfma_tile.hip"),
    "mfma/tile_merge2": ("mfma_tile_kernel.h", "mfma_tile_phase.hip"),
    "mfma/tile_phase": ("mfma_tile_kernel.h", "mfma_tile_phase.hip"),
    "mfma/wgrad": ("mfma_wgrad.hip",),
    "mfma/smallc": ("mfma_smallc.hip",),
    "mfma/bf16_tile": ("mfma_bf16.hip",),
    "mfma/bf16_wgrad": ("mfma_bf16_wgrad.hip",),
    "mfma/bf16_gemm": ("mfma_bf16_gemm.hip",),
    "depthwise/strip": ("depthwise.hip",),
    "depthwise/rows": ("depthwise.hip",),
    "depthwise/lds": ("depthwise.hip",),
    "direct": ("direct.hip",),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--layer", default="2a")
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16", "bf16out"],
                    help="bf16: bf16 inputs, float results; bf16out: bf16 inputs, y and dx stored as bf16 (dw float)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--epilogue", action="store_true",
                    help="time the fused calls instead: conv2d_fwd_bias_relu and conv2d_bwd_data_relu_mask (mask = x); "
                         "backward-weight is unchanged.  Not the headline configuration: no cpu baseline, no secondary")
    ap.add_argument("--no-secondary", action="store_true",
                    help="skip the depthwise layer's figures that the default run reports beside the headline layer")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, run --steps plain device-to-device copies of MIB mebibytes "
                         "(a kernel of known HBM traffic, used to scale the rocprofv3 FETCH_SIZE/WRITE_SIZE counters)")
    ap.add_argument("--settle-ms", type=float, default=60.0,
                    help="untimed steps are run for this long before the warm-up steps so that the GPU clock has ramped up")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark, time further ResNet / VGG / MobileNet layer shapes (fp32, seeded "
                         "inputs) and print one JSON line with a list of per-pass timings")
    ap.add_argument("--rotate", type=int, default=0,
                    help="number of distinct buffer sets cycled between steps (0: auto; "
                         "bandwidth-bound layers use enough to exceed the 256 MB Infinity Cache)")
    ap.add_argument("--all-layers", action="store_true",
                    help="instead of the benchmark, time every benchmark layer (fp32; the two VGG layers also with bf16 "
                         "inputs) and print one JSON line per layer and dtype: per pass time, TFLOP/s, GB/s, fraction of the "
                         "roof that bounds it, kernel family and (layers the oracle finishes in seconds) the largest "
                         "normalised error against the oracle")
    ap.add_argument("--traffic-lines", metavar="DIR",
                    help="instead of the benchmark, read the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE csv files under DIR "
                         "(sub-folders copy_<COUNTER>, l<layer>[bf16]_<COUNTER>) and print the per-kernel table and the "
                         "`traffic` lines that the profile summaries under profiles/ store (host only, no GPU)")
    return ap.parse_args()


def algorithmic_bytes(L, pass_name, in_bytes, out_bytes=4):
    """Unique bytes one pass must move: its two inputs once, its output once (dw is always float)."""
    nx, nw, ny = (L.N * L.C * L.H * L.W, L.K * (L.C // L.groups) * L.R * L.S, L.N * L.K * L.P * L.Q)
    if pass_name == "fwd":
        return (nx + nw) * in_bytes + ny * out_bytes
    if pass_name == "bwd_data":
        return (ny + nw) * in_bytes + nx * out_bytes
    return (nx + ny) * in_bytes + nw * 4


# ------------------------------------------------------------------------------------------ stored HBM traffic
def source_digest(family):
    """Short sha256 of the kernel sources behind a kernel family (what a stored traffic figure is tied to)."""
    h = hashlib.sha256()
    for name in FAMILY_SOURCES.get(family, ("api.cpp",)):
        with open(os.path.join(CSRC, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def stored_traffic(layer, dtype, pass_name, family):
    """HBM bytes per launch measured earlier with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy) and
    stored as a `traffic` line in a profile summary.  The figure is only reported while the kernel's sources are
    the ones it was measured on; otherwise value is null and `reason` says why."""
    pat = re.compile(r"^traffic layer=(\S+) dtype=(\S+) pass=(\S+) bytes=(\d+) family=(\S+) sources=(\S+)\s*$")
    for rel in TRAFFIC_PROFILES:
        path = os.path.join(ROOT, rel)
        if not os.path.exists(path):
            continue
        for line in open(path):
            m = pat.match(line.strip())
            if not m or (m.group(1), m.group(2), m.group(3)) != (layer, dtype, pass_name):
                continue
            if m.group(5) != family:
                return {"value": None, "source": rel, "reason": f"stored for kernel family {m.group(5)}, now {family}"}
            if m.group(6) != source_digest(family):
                return {"value": None, "source": rel,
                        "reason": "kernel sources changed since the stored figure was measured "
                                  f"(stored {m.group(6)}, now {source_digest(family)})"}
            return {"value": int(m.group(4)), "source": rel, "kind": "stored rocprofv3 --pmc figure, not measured in this run",
                    "sources_sha256_16": m.group(6)}
    return {"value": None, "source": None, "reason": "no stored measurement for this layer, dtype and pass"}


def traffic_lines(directory):
    """Summarises rocprofv3 --pmc csv output (see the commands in profiles/conv2d_hbm_traffic_pmc.md)."""
    import csv
    from paper_1912_01703_amd import binding as mc
    from paper_1912_01703_amd import workloads as wl

    def counters(folder):
        agg = {}
        for path in glob.glob(os.path.join(directory, folder, "**", "*counter_collection.csv"), recursive=True):
            for r in csv.DictReader(open(path)):
                agg.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
        return {k: sum(v) / len(v) for k, v in agg.items()}

    scale = {}
    for c in ("FETCH_SIZE", "WRITE_SIZE"):
        cal = counters("copy_" + c)
        kib = [v for k, v in cal.items() if "copyBuffer" in k]
        if not kib:
            raise SystemExit(f"no copy calibration for {c} under {directory}")
        log = json.loads(next(l for l in open(os.path.join(directory, f"copy_{c}.log")) if l.startswith('{"copy_calibration"')))
        scale[c] = log["bytes_read_per_copy"] / 1024.0 / kib[0]
        print(f"- {c} reads {kib[0]:.1f} KiB per {log['bytes_read_per_copy'] >> 20} MiB copy -> scale factor {scale[c]:.3f}")
    print("\n| run | kernel | FETCH_SIZE KiB | WRITE_SIZE KiB | read MB | written MB | total MB |\n|---|---|---|---|---|---|---|")
    lines = []
    for folder in sorted({os.path.basename(p).rsplit("_", 2)[0] for p in glob.glob(os.path.join(directory, "l*_FETCH_SIZE"))}):
        layer, dtype = (folder[1:-4], "bf16") if folder.endswith("bf16") else (folder[1:], "f32")
        fetch, write = counters(folder + "_FETCH_SIZE"), counters(folder + "_WRITE_SIZE")
        per_pass = {p: 0.0 for p in PASSES}
        code = mc.BF16_F32ACC if dtype == "bf16" else mc.F32
        for k in sorted(fetch):
            if "miconv" not in k or "clock_sampler" in k:
                continue
            rd, wr = fetch[k] * scale["FETCH_SIZE"] * 1024, write.get(k, 0.0) * scale["WRITE_SIZE"] * 1024
            short = re.sub(r"\(anonymous namespace\)::|void |miconv::", "", k)
            short = re.sub(r"\(.*\)$", "", short)
            print(f"| {layer} {dtype} | `{short}` | {fetch[k]:.0f} | {write.get(k, 0.0):.0f} | {rd / 1e6:.1f} | {wr / 1e6:.1f} | {(rd + wr) / 1e6:.1f} |")
            # which pass a kernel belongs to: backward-weight kernels and their reductions, backward-data instances,
            # everything else forward; kernels shared by forward and backward-data count for both
            if re.search(r"wgrad|reduce", short):
                per_pass["bwd_weight"] += rd + wr
            elif re.search(r"conv_tile_kernel<[^>]*?, true, (true|false), (true|false), \d", short) or "bwd" in short:
                per_pass["bwd_data"] += rd + wr
            elif re.search(r"dw_strip_stencil|dw_rows_kernel|dw_stencil|pack_|bf16_tile_kernel", short):
                per_pass["fwd"] += rd + wr
                per_pass["bwd_data"] += rd + wr
            else:
                per_pass["fwd"] += rd + wr
        for p, name in enumerate(PASSES):
            fam = mc.miconv_kernel_path(p, *wl.LAYERS[layer].conv_args(), code)
            lines.append(f"traffic layer={layer} dtype={dtype} pass={name} bytes={per_pass[name]:.0f} family={fam} "
                         f"sources={source_digest(fam)}")
    print("\n" + "\n".join(lines))


# ------------------------------------------------------------------------------------------------ CPU baseline
def cpu_baseline(L, dtype, gpu_results=None):
    """Times the oracle (as it stands) on the host cores for the same layer.
    Layers whose full oracle run would exceed ~30 s are timed on a subset of
    images and the rate is reported per FLOP, which is the metric's unit.
    When the whole layer was run and gpu_results() returns the HIP path's (y, dx, dw) for the same seeded
    inputs, the oracle's results are also used to report each pass's maximum normalised error
    |gpu - oracle| / sum |a||b| (the untimed part of this leg)."""
    import numpy as np
    from oracle import convref as ref
    from paper_1912_01703_amd import workloads as wl
    budget_flops = 60e9          # about 10-30 s of scalar fp64 on 8-16 cores
    n_sub = max(1, min(L.N, int(L.N * budget_flops / (3.0 * L.flops))))
    sub = wl.custom_layer(L.name + "-cpu", n_sub, L.C, L.H, L.W, L.K, L.R, L.S, L.strides, L.pads, L.groups,
                          seed=L.seed, x_dist=L.x_dist)
    x, w, dy = wl.make_inputs(sub)
    if dtype == "bf16":
        x, w, dy = wl.to_bf16_bits(x), wl.to_bf16_bits(w), wl.to_bf16_bits(dy)
    tiny = wl.LAYERS["1"]
    tx, tw, _ = wl.make_inputs(tiny)
    ref.conv2d_fwd(tx, tw, tiny.strides, tiny.pads, tiny.groups)     # warm-up: library load, thread pool
    t0 = time.perf_counter()
    refs = (ref.conv2d_fwd(x, w, sub.strides, sub.pads, sub.groups),
            ref.conv2d_bwd_data(dy, w, sub.x_shape, sub.strides, sub.pads, sub.groups),
            ref.conv2d_bwd_weight(x, dy, sub.w_shape, sub.strides, sub.pads, sub.groups))
    dt = time.perf_counter() - t0
    errs = None
    if gpu_results is not None and n_sub == L.N:
        ab = (lambda t: t & np.uint16(0x7FFF)) if dtype == "bf16" else np.abs
        dens = (ref.conv2d_fwd(ab(x), ab(w), sub.strides, sub.pads, sub.groups),
                ref.conv2d_bwd_data(ab(dy), ab(w), sub.x_shape, sub.strides, sub.pads, sub.groups),
                ref.conv2d_bwd_weight(ab(x), ab(dy), sub.w_shape, sub.strides, sub.pads, sub.groups))
        errs = {}
        for name, got, want, den in zip(PASSES, gpu_results(), refs, dens):
            live = den > 0
            errs[name] = float(np.max(np.abs(got.astype(np.float64)[live] - want[live]) / den[live]))
            if not np.all(got[~live] == 0):
                errs[name] = 1e30    # a value where no tap reaches: reported as a failed bound
    model = ""
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {"value": 3.0 * sub.flops / dt / 1e12, "unit": "TFLOP/s", "cores": ref.num_threads(), "kind": "oracle",
            "seconds": dt, "cpu_model": model, "max_norm_err_vs_gpu": errs,
            "sample": f"layer {L.name} with N={n_sub} of {L.N} images, fwd+bwd_data+bwd_weight once, fp64 accumulate"}


# ------------------------------------------------------------------------------------------------ GPU clock
class ClockSampler:
    """Average shader clock while benchmark kernels run: a one-wave kernel of the library on a second stream reads
    the shader-clock counter and the GPU's constant-rate counter at both ends of an interval (see
    miconv_sample_shader_clock in include/miconv.h)."""

    def __init__(self, mc, torch):
        self.mc, self.torch = mc, torch
        self.stream = torch.cuda.Stream()          # default priority
        self.counts = torch.zeros(2, dtype=torch.int64, device="cuda:0")
        self.khz = None

    def start(self, duration_us):
        self.counts.zero_()
        self.torch.cuda.synchronize()
        self.khz = self.mc.miconv_sample_shader_clock(self.counts, duration_us, self.stream.cuda_stream)

    def mhz(self):
        """Call after a device synchronisation."""
        c = self.counts.cpu().numpy()
        if self.khz is None or c[1] <= 0:
            return None
        return float(c[0]) / float(c[1]) * self.khz / 1e3


# ------------------------------------------------------------------------------------------------ one layer
def make_sets(L, dtype, nsets, torch, np, wl, dev):
    x, w, dy = wl.make_inputs(L)
    if dtype != "f32":
        x, w, dy = (wl.to_bf16_bits(t).view(np.int16) for t in (x, w, dy))
    odt = torch.int16 if dtype == "bf16out" else torch.float32
    sets = []
    for _ in range(nsets):
        sets.append(dict(x=torch.from_numpy(x).to(dev), w=torch.from_numpy(w).to(dev), dy=torch.from_numpy(dy).to(dev),
                         y=torch.empty(L.y_shape, dtype=odt, device=dev),
                         dx=torch.empty(L.x_shape, dtype=odt, device=dev),
                         dw=torch.empty(L.w_shape, dtype=torch.float32, device=dev)))
    return sets


def measure_layer(L, dtype, steps, warmup, settle_ms, rotate, mc, wl, torch, np, fused=False):
    """Times `steps` steps of layer L (wall clock between two synchronisations) and then, in a second region of
    the same launches, each pass's average launch duration with HIP events.  Returns a dict of figures."""
    code = {"f32": mc.F32, "bf16": mc.BF16_F32ACC, "bf16out": mc.BF16_BF16OUT}[dtype]
    in_bytes = 4 if dtype == "f32" else 2
    out_bytes = 2 if dtype == "bf16out" else 4
    args = L.conv_args()
    dev = "cuda:0"
    # Which roof bounds the layer: below the ridge (peak FLOP/s over 8 TB/s) it is HBM.  That is every depthwise
    # layer, and the 224x224x64 layer with bf16 inputs (192 FLOP per byte against a ridge of 312).
    intensity = L.flops / max(algorithmic_bytes(L, p, in_bytes, out_bytes) for p in PASSES)
    hbm_bound = intensity < PEAK_TFLOPS[dtype] * 1e12 / (PEAK_HBM_GBS * 1e9)
    # HBM-bound layers rotate over buffer sets so that no launch finds its inputs in the 256 MB Infinity
    # Cache: also within a group of launches of one pass, more than 256 MB are touched between two
    # uses of a buffer.
    pass_bytes = min(algorithmic_bytes(L, p, in_bytes, out_bytes) for p in PASSES)
    nsets = rotate if rotate > 0 else (max(4, int(300e6 // max(1, pass_bytes)) + 2) if hbm_bound else 1)
    nsets = min(nsets, 64)
    sets = make_sets(L, dtype, nsets, torch, np, wl, dev)
    ws_bytes = [mc.conv2d_workspace_bytes(p, *args, code) for p in range(3)]
    ws = torch.empty(max(ws_bytes + [256]), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    bias = torch.from_numpy(wl.make_epilogue_inputs(L)[0]).to(dev) if fused else None

    def run_pass(p, s):
        if p == 0 and fused:
            mc.conv2d_fwd_bias_relu(s["x"], s["w"], bias, s["y"], *args, code, ws, stream)
        elif p == 1 and fused:
            mc.conv2d_bwd_data_relu_mask(s["dy"], s["w"], s["x"], s["dx"], *args, code, ws, stream)
        elif p == 0:
            mc.conv2d_fwd(s["x"], s["w"], s["y"], *args, code, ws, stream)
        elif p == 1:
            mc.conv2d_bwd_data(s["dy"], s["w"], s["dx"], *args, code, ws, stream)
        else:
            mc.conv2d_bwd_weight(s["x"], s["dy"], s["dw"], *args, code, ws, stream)

    def step(i):
        s = sets[i % nsets]
        for p in range(3):
            run_pass(p, s)

    # The GPU takes about 25 ms of sustained load to reach its full clock (layer 2a kernels go from 137 to
    # 117 us over their first 200 launches): steps run untimed until that much time has passed, then the
    # W warm-up steps, then the K timed ones.
    t_settle = time.perf_counter()
    i = 0
    while (time.perf_counter() - t_settle) * 1e3 < settle_ms:
        for _ in range(8):
            step(i)
            i += 1
        torch.cuda.synchronize()
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / steps

    # Second region, same launches: HIP events (recorded on the stream the kernels are launched on)
    # around GROUP back-to-back launches of one pass, each on the next buffer set; the bracket's time
    # divided by GROUP is that pass's average launch duration.  One launch per bracket would add the
    # events' own cost (2-3 us) to kernels that run for 25 us.  MFMA-bound layers keep the order of a
    # training step (fwd, bwd_data, bwd_weight groups alternate).  HBM-bound layers run pass by pass,
    # each after a few untimed launches: in step order the pass that only reads (bwd_weight) is charged
    # the write-back of the 256 MB of results that the passes before it left in the Infinity Cache
    # (31 instead of 25 us on layer 5a).
    GROUP = 16
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(3)]
          for _ in range(steps)]

    def bracket(i, p):
        ev[i][p][0].record()
        for j in range(GROUP):
            run_pass(p, sets[(i * GROUP + j) % nsets])
        ev[i][p][1].record()

    if hbm_bound:
        for p in range(3):
            for j in range(2 * GROUP):
                run_pass(p, sets[j % nsets])
            for i in range(steps):
                bracket(i, p)
    else:
        for i in range(steps):
            for p in range(3):
                bracket(i, p)
    torch.cuda.synchronize()
    times = [[ev[i][p][0].elapsed_time(ev[i][p][1]) / GROUP for i in range(steps)] for p in range(3)]
    # HBM-bound layers: the same brackets on one buffer set, i.e. with whatever fits already in the Infinity Cache
    pass_warm = None
    if hbm_bound:
        evw = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(3)]
               for _ in range(steps)]
        for p in range(3):
            for i in range(steps):
                evw[i][p][0].record()
                for j in range(GROUP):
                    run_pass(p, sets[0])
                evw[i][p][1].record()
        torch.cuda.synchronize()
        pass_warm = [float(np.mean([evw[i][p][0].elapsed_time(evw[i][p][1]) for i in range(steps)])) / GROUP for p in range(3)]
    # Third region, untimed: the same steps once more while a one-wave kernel on a second stream samples the shader
    # clock (at most 20 ms, about two thirds of the region's expected length).  It has a region of its own because a
    # second active stream slows passes that consist of two dependent kernels (split reductions: +20 % on layer 2c).
    sampler = ClockSampler(mc, torch)
    clock_steps = max(steps, int(3.0 / max(ms_per_step, 1e-3)))          # at least 3 ms of work
    sampler.start(int(min(20000.0, max(200.0, 0.66 * ms_per_step * 1e3 * clock_steps))))
    for i in range(clock_steps):
        step(i)
    torch.cuda.synchronize()
    sclk_mhz = sampler.mhz()
    passes = {}
    for p, name in enumerate(PASSES):
        ms = float(np.mean(times[p]))
        passes[name] = {"ms_avg": ms, "ms_median": float(np.median(times[p])), "ms_min": float(np.min(times[p])),
                        "algo": mc.miconv_last_algo(p), "kernel_path": mc.miconv_kernel_path(p, *args, code),
                        "tflops": L.flops / (ms * 1e-3) / 1e12,
                        "gbs": algorithmic_bytes(L, name, in_bytes, out_bytes) / (ms * 1e-3) / 1e9}
        if pass_warm is not None:
            passes[name]["ms_avg_warm"] = pass_warm[p]
    del sets, ws
    torch.cuda.empty_cache()
    return {"ms_per_step": ms_per_step, "passes": passes, "hbm_bound": hbm_bound, "nsets": nsets, "group": GROUP,
            "sclk_mhz": sclk_mhz, "in_bytes": in_bytes, "out_bytes": out_bytes}


def roofline_of(L, dtype, m, layer_name):
    passes = m["passes"]
    dom = max(PASSES, key=lambda p: passes[p]["ms_avg"])
    traffic = stored_traffic(layer_name, dtype, dom, passes[dom]["kernel_path"])
    common = {"kernel": dom, "kernel_path": passes[dom]["kernel_path"], "traffic": traffic["value"], "traffic_detail": traffic,
              "algorithmic_bytes_per_launch": algorithmic_bytes(L, dom, m["in_bytes"], m["out_bytes"]),
              "avg_launch_ms": passes[dom]["ms_avg"], "launches_per_event_pair": m["group"]}
    if m["hbm_bound"]:
        ach = passes[dom]["gbs"]
        return dict({"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
                     "event_region_order": "pass by pass", "buffer_sets_rotated": m["nsets"]}, **common)
    ach = passes[dom]["tflops"]
    return dict({"bound": "mfma", "achieved": ach, "peak": PEAK_TFLOPS[dtype], "unit": "TFLOP/s",
                 "frac": ach / PEAK_TFLOPS[dtype], "algorithmic_flops_per_launch": L.flops,
                 "event_region_order": "step by step"}, **common)


def secondary_depthwise(steps, warmup, settle_ms, mc, wl, torch, np):
    """Layer 5a (MobileNet depthwise 3x3), every pass cold: the HBM-bound half of the target."""
    L = wl.LAYERS["5a"]
    m = measure_layer(L, "f32", steps, warmup, settle_ms, 0, mc, wl, torch, np)
    out = {"workload": f"layer 5a ({L.note}): N={L.N} C={L.C} HxW={L.H}x{L.W} 3x3 stride 1 pad 1 groups {L.groups}, fp32",
           "bound": "hbm", "peak": PEAK_HBM_GBS, "unit": "GB/s", "target_frac": 0.60,
           "inputs": f"cold: {m['nsets']} buffer sets rotated, pass by pass, {m['group']} launches per event pair",
           "passes": {}}
    for name in PASSES:
        p = m["passes"][name]
        out["passes"][name] = {"us": p["ms_avg"] * 1e3, "us_min": p["ms_min"] * 1e3, "us_warm": p["ms_avg_warm"] * 1e3,
                               "gbs": p["gbs"], "frac": p["gbs"] / PEAK_HBM_GBS, "kernel_path": p["kernel_path"],
                               "algorithmic_bytes_per_launch": algorithmic_bytes(L, name, 4)}
    slow = min(PASSES, key=lambda n: out["passes"][n]["frac"])
    out["slowest_pass"] = slow
    out["frac_slowest"] = out["passes"][slow]["frac"]
    return out


def batchnorm_figures(mc, wl, torch, np, reps=20):
    """batchnorm2d_fwd / batchnorm2d_bwd on the two benchmark shapes, cold (buffer sets rotated so that more than
    the 256 MB Infinity Cache passes between two uses of a buffer), against the HBM peak.  Algorithmic bytes:
    forward x once + y once (8 B per element), backward x, dy once + dx once (12 B per element)."""
    dev = "cuda:0"
    stream = torch.cuda.current_stream().cuda_stream
    out = {"bound": "hbm", "peak": PEAK_HBM_GBS, "unit": "GB/s", "shapes": {}}
    for idx, (name, N, C, H, W) in enumerate(wl.BN_SHAPES):
        elems = N * C * H * W
        nsets = max(4, int(600e6 // (elems * 12)) + 2)
        x, dy, gamma, beta = wl.make_bn_inputs(N, C, H, W, 512 + idx)
        sets = [dict(x=torch.from_numpy(x).to(dev), dy=torch.from_numpy(dy).to(dev),
                     y=torch.empty((N, C, H, W), device=dev), dx=torch.empty((N, C, H, W), device=dev)) for _ in range(nsets)]
        g, b = torch.from_numpy(gamma).to(dev), torch.from_numpy(beta).to(dev)
        mean, inv_std, dg, db = (torch.empty(C, device=dev) for _ in range(4))
        ws = torch.empty(max(256, max(mc.batchnorm2d_workspace_bytes(p, N, C, H, W) for p in (0, 1))), dtype=torch.uint8, device=dev)
        fwd = lambda s: mc.batchnorm2d_fwd(s["x"], g, b, s["y"], mean, inv_std, N, C, H, W, 1e-5, mc.F32, ws, stream)
        bwd = lambda s: mc.batchnorm2d_bwd(s["x"], s["dy"], g, mean, inv_std, s["dx"], dg, db, N, C, H, W, mc.F32, ws, stream)
        row = {"N": N, "C": C, "H": H, "W": W, "buffer_sets_rotated": nsets}
        for pname, call, bpe in (("fwd", fwd, 8), ("bwd", bwd, 12)):
            for j in range(nsets):
                call(sets[j])
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for j in range(reps):
                call(sets[j % nsets])
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / reps
            gbs = elems * bpe / (us * 1e-6) / 1e9
            row[pname] = {"us": us, "algorithmic_bytes_per_launch": elems * bpe, "gbs": gbs, "frac": gbs / PEAK_HBM_GBS}
        out["shapes"][name] = row
        del sets
        torch.cuda.empty_cache()
    return out


def all_layers(a, mc, wl, torch, np):
    """One JSON line per (layer, dtype) of the benchmark configurations."""
    from oracle import convref as ref
    runs = [(n, "f32") for n in wl.LAYERS] + [("4a", "bf16"), ("4b", "bf16")]
    for name, dtype in runs:
        L = wl.LAYERS[name]
        steps = max(5, min(a.steps, int(400.0 / max(1e-3, 3 * L.flops / 100e12 * 1e3))))   # about 0.4 s of timed work per region
        m = measure_layer(L, dtype, steps, min(a.warmup, steps), a.settle_ms, a.rotate, mc, wl, torch, np)
        peak = PEAK_HBM_GBS if m["hbm_bound"] else PEAK_TFLOPS[dtype]
        line = {"layer": name, "note": L.note, "dtype": dtype, "seed": L.seed, "bound": "hbm" if m["hbm_bound"] else "mfma",
                "peak": peak, "unit": "GB/s" if m["hbm_bound"] else "TFLOP/s", "steps": steps,
                "step_tflops": 3.0 * L.flops / (m["ms_per_step"] * 1e-3) / 1e12, "passes": {}}
        errs = None
        if 3.0 * L.flops <= 60e9:      # the oracle finishes the layer (and its absolute-value twin) in seconds
            def gpu_results(L=L, dtype=dtype):
                s = make_sets(L, dtype, 1, torch, np, wl, "cuda:0")[0]
                code = mc.BF16_F32ACC if dtype == "bf16" else mc.F32
                args = L.conv_args()
                ws = torch.empty(max([256] + [mc.conv2d_workspace_bytes(p, *args, code) for p in range(3)]), dtype=torch.uint8, device="cuda:0")
                st = torch.cuda.current_stream().cuda_stream
                mc.conv2d_fwd(s["x"], s["w"], s["y"], *args, code, ws, st)
                mc.conv2d_bwd_data(s["dy"], s["w"], s["dx"], *args, code, ws, st)
                mc.conv2d_bwd_weight(s["x"], s["dy"], s["dw"], *args, code, ws, st)
                torch.cuda.synchronize()
                return s["y"].cpu().numpy(), s["dx"].cpu().numpy(), s["dw"].cpu().numpy()
            errs = cpu_baseline(L, dtype, gpu_results)["max_norm_err_vs_gpu"]
        for pname in PASSES:
            p = m["passes"][pname]
            ach = p["gbs"] if m["hbm_bound"] else p["tflops"]
            line["passes"][pname] = {"us_avg": p["ms_avg"] * 1e3, "us_median": p["ms_median"] * 1e3, "us_min": p["ms_min"] * 1e3,
                                     "tflops": p["tflops"], "gbs": p["gbs"], "frac_of_roof": ach / peak,
                                     "kernel_path": p["kernel_path"], "max_norm_err": errs[pname] if errs else None}
        print(json.dumps(line), flush=True)


def sweep(mc, wl, torch):
    """Times every pass of wl.MORE_SHAPES (fp32, seeded inputs of the workloads module, back-to-back launches between
    two events)."""
    dev = "cuda:0"
    stream = torch.cuda.current_stream().cuda_stream
    rows = []
    for idx, (name, N, C, H, W, K, R, st, pd, g) in enumerate(wl.MORE_SHAPES):
        L = wl.custom_layer(name, N, C, H, W, K, R, R, st, pd, g, seed=256 + idx)
        args = L.conv_args()
        x, w, dy = (torch.from_numpy(t).to(dev) for t in wl.make_inputs(L))
        y, dx, dw = (torch.empty(sh, device=dev) for sh in (L.y_shape, L.x_shape, L.w_shape))
        ws = torch.empty(max([256] + [mc.conv2d_workspace_bytes(p, *args, mc.F32) for p in range(3)]),
                         dtype=torch.uint8, device=dev)
        calls = [lambda: mc.conv2d_fwd(x, w, y, *args, mc.F32, ws, stream),
                 lambda: mc.conv2d_bwd_data(dy, w, dx, *args, mc.F32, ws, stream),
                 lambda: mc.conv2d_bwd_weight(x, dy, dw, *args, mc.F32, ws, stream)]
        row = {"layer": name, "seed": L.seed, "flops_per_pass": L.flops, "bytes_x_plus_y": (x.numel() + y.numel()) * 4}
        for p, call in enumerate(calls):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            call()
            torch.cuda.synchronize()
            e0.record(); call(); e1.record()
            torch.cuda.synchronize()
            reps = max(3, min(200, int(30.0 / max(e0.elapsed_time(e1), 1e-3))))
            for _ in range(reps):
                call()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                call()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            row[PASSES[p]] = {"ms": ms, "tflops": L.flops / (ms * 1e-3) / 1e12, "algo": mc.miconv_last_algo(p),
                              "kernel_path": mc.miconv_kernel_path(p, *args, mc.F32)}
        rows.append(row)
        sys.stderr.write("%-32s " % name + " | ".join("%9.1f us %6.1f TF a%d" % (row[k]["ms"] * 1e3, row[k]["tflops"], row[k]["algo"])
                                                     for k in PASSES) + "\n")
        del x, w, dy, y, dx, dw, ws
    print(json.dumps({"sweep": rows}), flush=True)


def main():
    a = parse()
    if a.gpus != 1:
        sys.stderr.write("bench.py: this build measures one GPU only; run with --gpus 1\n")
        sys.exit(2)
    if a.traffic_lines:
        traffic_lines(a.traffic_lines)
        return
    import numpy as np
    import torch
    from paper_1912_01703_amd import binding as mc
    from paper_1912_01703_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible\n")
        sys.exit(3)
    if a.copy_calibration > 0:
        nbytes = a.copy_calibration << 20
        src = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(a.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "bytes_read_per_copy": nbytes, "bytes_written_per_copy": nbytes,
                          "copies": a.steps}), flush=True)
        return
    if a.sweep:
        sweep(mc, wl, torch)
        return
    if a.all_layers:
        all_layers(a, mc, wl, torch, np)
        return
    L = wl.LAYERS[a.layer]
    m = measure_layer(L, a.dtype, a.steps, a.warmup, a.settle_ms, a.rotate, mc, wl, torch, np, fused=a.epilogue)
    tflops = 3.0 * L.flops / (m["ms_per_step"] * 1e-3) / 1e12
    out = {
        "metric": METRIC, "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": m["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": a.dtype, "data": "synthetic",
        "config": {"workload": f"layer {L.name} ({L.note}): N={L.N} C={L.C} HxW={L.H}x{L.W} K={L.K} "
                               f"{L.R}x{L.S} stride {L.stride} pad {L.pad} groups {L.groups}; "
                               "step = fwd + bwd_data + bwd_weight",
                   "layer": L.name, "seed": L.seed, "flops_per_pass": L.flops},
        "pct_of_peak": 100.0 * tflops / PEAK_TFLOPS[a.dtype],
        "passes": m["passes"],
        "roofline": roofline_of(L, a.dtype, m, a.layer),
        "device": torch.cuda.get_device_name(0),
        "paper_context": PAPER_CONTEXT,
    }
    # Against the clock the GPU ran at: the published peak assumes 2.4 GHz, the part settles lower under this load.
    if m["sclk_mhz"]:
        peak_at_clock = NUM_CUS * MFMA_FLOP_PER_CLK_PER_CU[a.dtype] * m["sclk_mhz"] * 1e6 / 1e12
        out["measured_clock"] = {"sclk_mhz": m["sclk_mhz"],
                                 "source": "ratio of the shader-clock counter to the constant-rate counter, read by a one-wave "
                                           "kernel on a second stream (miconv_sample_shader_clock) while the timed steps "
                                           "were repeated in an untimed region of their own",
                                 "peak_at_clock": peak_at_clock, "unit": "TFLOP/s",
                                 "formula": f"{NUM_CUS} CUs x {MFMA_FLOP_PER_CLK_PER_CU[a.dtype]} FLOP/clk x sclk"}
        out["pct_of_measured_clock_peak"] = 100.0 * tflops / peak_at_clock
    else:
        out["measured_clock"] = None
        out["pct_of_measured_clock_peak"] = None
    if a.epilogue:
        out["config"]["epilogue"] = "fwd: bias + ReLU; bwd_data: ReLU mask (x); fused=%s" % [
            mc.miconv_epilogue_is_fused(p, *L.conv_args(), mc.BF16_F32ACC if a.dtype == "bf16" else mc.F32) for p in (0, 1)]
        print(json.dumps(out), flush=True)
        return
    if a.layer == "2a" and a.dtype == "f32" and not a.no_secondary:
        out["secondary"] = secondary_depthwise(max(10, min(a.steps, 30)), a.warmup, a.settle_ms, mc, wl, torch, np)
        out["batchnorm"] = batchnorm_figures(mc, wl, torch, np)
    if not a.no_cpu_baseline:
        def gpu_results():
            s = make_sets(L, a.dtype, 1, torch, np, wl, "cuda:0")[0]
            code = mc.BF16_F32ACC if a.dtype == "bf16" else mc.F32
            args = L.conv_args()
            ws = torch.empty(max([256] + [mc.conv2d_workspace_bytes(p, *args, code) for p in range(3)]),
                             dtype=torch.uint8, device="cuda:0")
            st = torch.cuda.current_stream().cuda_stream
            mc.conv2d_fwd(s["x"], s["w"], s["y"], *args, code, ws, st)
            mc.conv2d_bwd_data(s["dy"], s["w"], s["dx"], *args, code, ws, st)
            mc.conv2d_bwd_weight(s["x"], s["dy"], s["dw"], *args, code, ws, st)
            torch.cuda.synchronize()
            return s["y"].cpu().numpy(), s["dx"].cpu().numpy(), s["dw"].cpu().numpy()
        # (bf16 results: the oracle is timed on the same bf16 inputs; the per-pass error check is the tests' business)
        out["cpu_baseline"] = cpu_baseline(L, "f32" if a.dtype == "f32" else "bf16", None if a.dtype == "bf16out" else gpu_results)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
