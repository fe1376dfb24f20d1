#!/usr/bin/env python3
"""Benchmark of the convolution hot path on one MI355X.

A step is one forward + backward-data + backward-weight pass of one layer
through the C ABI (default: the ResNet-50 3x3 bottleneck layer, N=64,
C=K=256, 14x14), inputs resident in HBM.  Prints ONE JSON line:
whole-step TFLOP/s (nominal 2*N*K*P*Q*Cg*R*S FLOPs per pass), the roofline
figures of the dominant kernel measured with HIP events, and the CPU oracle
timed on the host cores as a baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--layer 2a] [--dtype f32|bf16]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}   # dense MFMA, MI355X published
PEAK_HBM_GBS = 8000.0
PASSES = ("fwd", "bwd_data", "bwd_weight")
# HBM bytes per launch (read + written), from rocprofv3 FETCH_SIZE / WRITE_SIZE runs scaled by a plain
# copy of known size; see profiles/conv2d_hbm_traffic_pmc.md for the commands and the raw counters.
MEASURED_TRAFFIC = {
    ("2a", "f32"): {"fwd": 45.2e6, "bwd_data": 45.2e6, "bwd_weight": 79.7e6},
    ("5a", "f32"): {"fwd": 102.9e6, "bwd_data": 102.9e6, "bwd_weight": 103.0e6},
}
METRIC = "conv fwd+bwd TFLOP/s and % FP32 MFMA peak (ResNet-50 3x3 layer)"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--layer", default="2a")
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, run --steps plain device-to-device copies of MIB mebibytes "
                         "(a kernel of known HBM traffic, used to scale the rocprofv3 FETCH_SIZE/WRITE_SIZE counters)")
    ap.add_argument("--settle-ms", type=float, default=60.0,
                    help="untimed steps are run for this long before the warm-up steps so that the GPU clock has ramped up")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark, time further ResNet / VGG / MobileNet layer shapes (fp32) and print "
                         "one JSON line with a list of per-pass timings")
    ap.add_argument("--rotate", type=int, default=0,
                    help="number of distinct buffer sets cycled between steps (0: auto; "
                         "bandwidth-bound layers use enough to exceed the 256 MB Infinity Cache)")
    return ap.parse_args()


def algorithmic_bytes(L, pass_name, in_bytes):
    """Unique bytes one pass must move: its two inputs once, its output once."""
    nx, nw, ny = (L.N * L.C * L.H * L.W, L.K * (L.C // L.groups) * L.R * L.S, L.N * L.K * L.P * L.Q)
    if pass_name == "fwd":
        return (nx + nw) * in_bytes + ny * 4
    if pass_name == "bwd_data":
        return (ny + nw) * in_bytes + nx * 4
    return (nx + ny) * in_bytes + nw * 4


def cpu_baseline(L, dtype):
    """Times the oracle (as it stands) on the host cores for the same layer.
    Layers whose full oracle run would exceed ~30 s are timed on a subset of
    images and the rate is reported per FLOP, which is the metric's unit."""
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
    ref.conv2d_fwd(x, w, sub.strides, sub.pads, sub.groups)
    ref.conv2d_bwd_data(dy, w, sub.x_shape, sub.strides, sub.pads, sub.groups)
    ref.conv2d_bwd_weight(x, dy, sub.w_shape, sub.strides, sub.pads, sub.groups)
    dt = time.perf_counter() - t0
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
            "seconds": dt, "cpu_model": model,
            "sample": f"layer {L.name} with N={n_sub} of {L.N} images, fwd+bwd_data+bwd_weight once, fp64 accumulate"}


def sweep(mc, wl, torch):
    """Times every pass of wl.MORE_SHAPES (fp32, random inputs, back-to-back launches between two events)."""
    dev = "cuda:0"
    stream = torch.cuda.current_stream().cuda_stream
    rows = []
    for (name, N, C, H, W, K, R, st, pd, g) in wl.MORE_SHAPES:
        L = wl.custom_layer(name, N, C, H, W, K, R, R, st, pd, g)
        args = L.conv_args()
        x = torch.randn(L.x_shape, device=dev)
        w = torch.randn(L.w_shape, device=dev)
        dy = torch.randn(L.y_shape, device=dev)
        y, dx, dw = (torch.empty(sh, device=dev) for sh in (L.y_shape, L.x_shape, L.w_shape))
        ws = torch.empty(max([256] + [mc.conv2d_workspace_bytes(p, *args, mc.F32) for p in range(3)]),
                         dtype=torch.uint8, device=dev)
        calls = [lambda: mc.conv2d_fwd(x, w, y, *args, mc.F32, ws, stream),
                 lambda: mc.conv2d_bwd_data(dy, w, dx, *args, mc.F32, ws, stream),
                 lambda: mc.conv2d_bwd_weight(x, dy, dw, *args, mc.F32, ws, stream)]
        row = {"layer": name, "flops_per_pass": L.flops, "bytes_x_plus_y": (x.numel() + y.numel()) * 4}
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
            row[PASSES[p]] = {"ms": ms, "tflops": L.flops / (ms * 1e-3) / 1e12, "algo": mc.miconv_last_algo(p)}
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
    L = wl.LAYERS[a.layer]
    code = mc.BF16_F32ACC if a.dtype == "bf16" else mc.F32
    in_bytes = 2 if a.dtype == "bf16" else 4
    args = L.conv_args()
    dev = "cuda:0"
    x, w, dy = wl.make_inputs(L)
    if a.dtype == "bf16":
        x, w, dy = (wl.to_bf16_bits(t).view(np.int16) for t in (x, w, dy))

    # Which roof bounds the layer: below the ridge (peak FLOP/s over 8 TB/s) it is HBM.  That is every depthwise
    # layer, and the 224x224x64 layer with bf16 inputs (192 FLOP per byte against a ridge of 312).
    intensity = L.flops / max(algorithmic_bytes(L, p, in_bytes) for p in PASSES)
    hbm_bound = intensity < PEAK_TFLOPS[a.dtype] * 1e12 / (PEAK_HBM_GBS * 1e9)
    # HBM-bound layers rotate over buffer sets so that no launch finds its inputs in the 256 MB Infinity
    # Cache: also within a group of launches of one pass, more than 256 MB are touched between two
    # uses of a buffer.
    pass_bytes = min(algorithmic_bytes(L, p, in_bytes) for p in PASSES)
    nsets = a.rotate if a.rotate > 0 else (max(4, int(300e6 // max(1, pass_bytes)) + 2) if hbm_bound else 1)
    nsets = min(nsets, 64)
    sets = []
    for i in range(nsets):
        s = dict(x=torch.from_numpy(x).to(dev), w=torch.from_numpy(w).to(dev), dy=torch.from_numpy(dy).to(dev),
                 y=torch.empty(L.y_shape, dtype=torch.float32, device=dev),
                 dx=torch.empty(L.x_shape, dtype=torch.float32, device=dev),
                 dw=torch.empty(L.w_shape, dtype=torch.float32, device=dev))
        sets.append(s)
    ws_bytes = [mc.conv2d_workspace_bytes(p, *args, code) for p in range(3)]
    ws = torch.empty(max(ws_bytes + [256]), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream

    def run_pass(p, s):
        if p == 0:
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
    while (time.perf_counter() - t_settle) * 1e3 < a.settle_ms:
        for _ in range(8):
            step(i)
            i += 1
        torch.cuda.synchronize()
    for i in range(a.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(a.steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / a.steps
    tflops = 3.0 * L.flops / (ms_per_step * 1e-3) / 1e12

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
          for _ in range(a.steps)]

    def bracket(i, p):
        ev[i][p][0].record()
        for j in range(GROUP):
            run_pass(p, sets[(i * GROUP + j) % nsets])
        ev[i][p][1].record()

    if hbm_bound:
        for p in range(3):
            for j in range(2 * GROUP):
                run_pass(p, sets[j % nsets])
            for i in range(a.steps):
                bracket(i, p)
    else:
        for i in range(a.steps):
            for p in range(3):
                bracket(i, p)
    torch.cuda.synchronize()
    pass_ms = [float(np.mean([ev[i][p][0].elapsed_time(ev[i][p][1]) for i in range(a.steps)])) / GROUP for p in range(3)]
    pass_min = [float(np.min([ev[i][p][0].elapsed_time(ev[i][p][1]) for i in range(a.steps)])) / GROUP for p in range(3)]
    pass_med = [float(np.median([ev[i][p][0].elapsed_time(ev[i][p][1]) for i in range(a.steps)])) / GROUP for p in range(3)]
    # HBM-bound layers: the same brackets on one buffer set, i.e. with whatever fits already in the Infinity Cache
    pass_warm = None
    if hbm_bound:
        evw = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(3)]
               for _ in range(a.steps)]
        for p in range(3):
            for i in range(a.steps):
                evw[i][p][0].record()
                for j in range(GROUP):
                    run_pass(p, sets[0])
                evw[i][p][1].record()
        torch.cuda.synchronize()
        pass_warm = [float(np.mean([evw[i][p][0].elapsed_time(evw[i][p][1]) for i in range(a.steps)])) / GROUP for p in range(3)]
    algos = [mc.miconv_last_algo(p) for p in range(3)]

    passes = {}
    for p, name in enumerate(PASSES):
        passes[name] = {"ms_avg": pass_ms[p], "ms_median": pass_med[p], "ms_min": pass_min[p], "algo": algos[p],
                        "tflops": L.flops / (pass_ms[p] * 1e-3) / 1e12,
                        "gbs": algorithmic_bytes(L, name, in_bytes) / (pass_ms[p] * 1e-3) / 1e9}
        if pass_warm is not None:
            passes[name]["ms_avg_warm"] = pass_warm[p]
    dom = int(np.argmax(pass_ms))
    traffic = MEASURED_TRAFFIC.get((a.layer, a.dtype), {}).get(PASSES[dom])
    if hbm_bound:
        ach = passes[PASSES[dom]]["gbs"]
        roof = {"bound": "hbm", "kernel": PASSES[dom], "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": ach / PEAK_HBM_GBS, "traffic": traffic,
                "algorithmic_bytes_per_launch": algorithmic_bytes(L, PASSES[dom], in_bytes),
                "avg_launch_ms": pass_ms[dom], "launches_per_event_pair": GROUP, "event_region_order": "pass by pass",
                "buffer_sets_rotated": nsets}
    else:
        ach = passes[PASSES[dom]]["tflops"]
        peak = PEAK_TFLOPS[a.dtype]
        roof = {"bound": "mfma", "kernel": PASSES[dom], "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                "frac": ach / peak, "traffic": traffic, "algorithmic_flops_per_launch": L.flops,
                "algorithmic_bytes_per_launch": algorithmic_bytes(L, PASSES[dom], in_bytes),
                "avg_launch_ms": pass_ms[dom], "launches_per_event_pair": GROUP, "event_region_order": "step by step"}

    out = {
        "metric": METRIC, "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": a.dtype, "data": "synthetic",
        "config": {"workload": f"layer {L.name} ({L.note}): N={L.N} C={L.C} HxW={L.H}x{L.W} K={L.K} "
                               f"{L.R}x{L.S} stride {L.stride} pad {L.pad} groups {L.groups}; "
                               "step = fwd + bwd_data + bwd_weight",
                   "layer": L.name, "seed": L.seed, "flops_per_pass": L.flops},
        "pct_of_peak": 100.0 * tflops / PEAK_TFLOPS[a.dtype],
        "passes": passes,
        "roofline": roof,
        "device": torch.cuda.get_device_name(0),
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(L, a.dtype)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
