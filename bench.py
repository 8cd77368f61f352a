#!/usr/bin/env python3
"""Benchmark of the convolution hot path on one MI355X.

One step = conv_fwd + conv_bwd_data + conv_bwd_weight through the C ABI on one batch of
seeded synthetic tensors that are already resident in HBM.  Prints ONE JSON line:
throughput in TFLOP/s on nominal FLOPs (3 * 2*N*Ks*P*Q*C*R*S per step), a roofline
object for the slowest matrix-core kernel (timed live with HIP events placed around it by
the library's one-shot probe), and the CPU oracle timed on a bounded sample of the same
layer as a reported baseline.

`--table` instead measures every benchmark configuration (fp32, and bf16 for the
larger-image layers) and prints one JSON line per configuration plus a markdown table
on stderr; it is not the default contract line.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}   # MI355X dense MFMA peaks
HBM_PEAK_GBS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.md")


def measured_traffic():
    """HBM-side bytes per launch of the matrix-core kernels, read from the committed rocprofv3 counter summary
    (profiles/hbm_traffic.md: FETCH_SIZE and WRITE_SIZE runs scaled by a copy kernel of known size).
    Returns {(config, dtype, kernel): bytes}; empty when the file is not there."""
    table = {}
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                cells = [c.strip() for c in line.strip().strip("|").split("|")]
                if len(cells) >= 6 and cells[0].startswith("cfg") and cells[1] in ("f32", "bf16"):
                    try:
                        table[(cells[0], cells[1], cells[2])] = int(float(cells[-2])) + int(float(cells[-1]))
                    except ValueError:
                        pass
    except OSError:
        pass
    return table


METRIC = "conv fwd+bwd TFLOP/s and % of MFMA peak, 1500-kernel 5x5 layer, batch 128"


def find_hip_runtime():
    """The libamdhip64 already mapped into this process (torch's and libconvslice's)."""
    with open("/proc/self/maps") as f:
        for line in f:
            if "libamdhip64" in line:
                return ctypes.CDLL(line.split()[-1])
    return ctypes.CDLL("libamdhip64.so")


class HipEvents:
    def __init__(self, count):
        self.hip = find_hip_runtime()
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.ev = []
        for _ in range(count):
            e = ctypes.c_void_p()
            rc = self.hip.hipEventCreate(ctypes.byref(e))
            if rc != 0:
                raise RuntimeError(f"hipEventCreate failed: {rc}")
            self.ev.append(e)

    def elapsed_ms(self, i, j):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.ev[i], self.ev[j])
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(ms.value)

    def destroy(self):
        for e in self.ev:
            self.hip.hipEventDestroy(e)
        self.ev = []


def cpu_baseline(cfg, x, w, dy, images):
    """The oracle as it stands on the first `images` images of the batch (default: all of them), all
    kernels of the slice, compiled -O3 -march=native on this host when a compiler is there."""
    import oracle
    try:
        flags = oracle.use_native_build()
    except Exception as e:   # no compiler on this host: the portable in-tree build is timed instead
        flags = f"-O2 -fopenmp (portable build; native build failed: {type(e).__name__})"
    k0, k1 = cfg.slice
    n = min(images, cfg.N)
    sh = oracle.Shape(n, cfg.C, cfg.H, cfg.W, cfg.K, cfg.R, cfg.S, cfg.stride, cfg.stride, cfg.pad, cfg.pad, k0, k1)
    xs, dys = x[:n], dy[:n]
    t0 = time.perf_counter()
    oracle.conv_fwd(sh, xs, w)
    oracle.conv_bwd_data(sh, dys, w)
    oracle.conv_bwd_weight(sh, xs, dys)
    dt = time.perf_counter() - t0
    flops = 3 * 2 * n * (k1 - k0) * cfg.P * cfg.Q * cfg.C * cfg.R * cfg.S
    which = f"all {cfg.N} images" if n == cfg.N else f"first {n} of {cfg.N} images"
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"{which} of {cfg.name}, all {k1 - k0} kernels of the slice (the whole layer), "
                      f"fwd+bwd_data+bwd_weight, fp64 direct loops, gcc {flags}, {dt:.1f} s"}


PASS_OF = {"conv_fwd": 0, "conv_bwd_data": 1, "conv_bwd_weight": 2}


def measure(cfg_name, dtype_name, steps, warmup, cpu_images=0, per_pass=False, graph=False):
    """Times `steps` steps of one configuration; returns the result dictionary."""
    import numpy as np
    import torch

    import paper_1712_02546_amd as cs
    from paper_1712_02546_amd import synth

    cfg = synth.CONFIGS[cfg_name]
    dtype = cs.CONV_F32 if dtype_name == "f32" else cs.CONV_BF16
    k0, k1 = cfg.slice
    x, w, dy = synth.make_inputs(cfg)
    if dtype == cs.CONV_BF16:
        x, w, dy = (synth.round_to_bf16(a) for a in (x, w, dy))
    dev = torch.device("cuda:0")

    def up(a):
        if dtype == cs.CONV_BF16:
            return torch.from_numpy(synth.f32_to_bf16_bits(a).view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    xd, wd, dyd = up(x), up(w), up(dy)
    tdt = torch.float32 if dtype == cs.CONV_F32 else torch.bfloat16
    y = torch.zeros((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=tdt, device=dev)
    dx = torch.zeros((cfg.N, cfg.C, cfg.H, cfg.W), dtype=tdt, device=dev)
    dw = torch.zeros((cfg.K, cfg.C, cfg.R, cfg.S), dtype=torch.float32, device=dev)
    desc = cs.ConvDesc(cfg.N, cfg.C, cfg.H, cfg.W, cfg.K, cfg.R, cfg.S, cfg.stride, cfg.stride, cfg.pad, cfg.pad,
                       k0, k1, dtype, 0)
    ws = torch.empty(max(cs.conv_workspace_bytes(desc, p) for p in (0, 1, 2)), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream

    passes = (("conv_fwd", cs.conv_fwd, (xd, wd, y)),
              ("conv_bwd_data", cs.conv_bwd_data, (dyd, wd, dx)),
              ("conv_bwd_weight", cs.conv_bwd_weight, (xd, dyd, dw)))

    def step(events=None, base=0):
        for i, (_, fn, (a, b, out)) in enumerate(passes):
            if events is not None:
                cs.conv_probe_next_call(events.ev[base + 2 * i], events.ev[base + 2 * i + 1])
            fn(desc, a, b, out, ws, stream)

    for _ in range(warmup):
        step()
    events = HipEvents(6 * steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        step(events, 6 * s)
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / steps
    F = cfg.flops_per_pass
    value = 3 * F / (ms_per_step * 1e-3) / 1e12
    kern = []
    es = 4 if dtype == cs.CONV_F32 else 2
    # bytes a pass must move at least: each of x, the slice of w and the slice of y once (dw is fp32)
    nx, ny, nw = x.size, y.numel() * (k1 - k0) // cfg.K, w.size * (k1 - k0) // cfg.K
    pass_bytes = {"conv_fwd": (nx + nw + ny) * es, "conv_bwd_data": (nx + nw + ny) * es,
                  "conv_bwd_weight": (nx + ny) * es + nw * 4}
    for i, (name, _, _) in enumerate(passes):
        d = [events.elapsed_ms(6 * s + 2 * i, 6 * s + 2 * i + 1) for s in range(steps)]
        avg = sum(d) / len(d)
        path = cs.conv_pass_path(desc, PASS_OF[name])
        kern.append({"entry": name, "kernel": path.split(":")[0], "path": path, "avg_ms": avg, "min_ms": min(d),
                     "tflops": F / (avg * 1e-3) / 1e12, "algorithmic_bytes": pass_bytes[name],
                     "gbs_on_algorithmic_bytes": pass_bytes[name] / (avg * 1e-3) / 1e9})
    events.destroy()
    if per_pass:  # whole entry point (layout kernels included), each pass timed on its own
        for k, (name, fn, (a, b, out)) in zip(kern, passes):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                fn(desc, a, b, out, ws, stream)
            torch.cuda.synchronize()
            k["entry_ms"] = (time.perf_counter() - t0) * 1e3 / steps
    graph_ms = None
    if graph:  # the same step recorded once into a HIP graph and replayed (what a launch-bound caller would do)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _, fn, (a, b, out) in passes:
                fn(desc, a, b, out, ws, torch.cuda.current_stream().cuda_stream)
        for _ in range(warmup):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / steps
        del g
    dom = max(kern, key=lambda k: k["avg_ms"])
    peak = PEAK_TFLOPS[dtype_name]
    # A converted-operand path multiplies on the fp32 matrix cores whatever the tensor dtype is.
    kpeak = PEAK_TFLOPS["f32"] if "fp32 MFMA" in dom["path"] else PEAK_TFLOPS["bf16"]
    min_bytes = sum(pass_bytes.values())
    f_mfma = dom["tflops"] / kpeak
    f_hbm = dom["gbs_on_algorithmic_bytes"] / HBM_PEAK_GBS
    traffic = measured_traffic().get((cfg_name, dtype_name, dom["kernel"]))
    # The roofline that binds the dominant kernel is the one it is closer to; the other fraction is reported beside it.
    if f_mfma >= f_hbm:
        roofline = {"bound": "mfma", "kernel": dom["kernel"], "achieved": dom["tflops"], "peak": kpeak, "unit": "TFLOP/s",
                    "frac": f_mfma, "avg_ms": dom["avg_ms"], "traffic": traffic,
                    "hbm_side": {"achieved": dom["gbs_on_algorithmic_bytes"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                 "frac": f_hbm}}
    else:
        roofline = {"bound": "hbm", "kernel": dom["kernel"], "achieved": dom["gbs_on_algorithmic_bytes"],
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": f_hbm, "avg_ms": dom["avg_ms"], "traffic": traffic,
                    "mfma_side": {"achieved": dom["tflops"], "peak": kpeak, "unit": "TFLOP/s", "frac": f_mfma}}
    out = {
        "metric": METRIC,
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype_name, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: batch {cfg.N}, input {cfg.C}x{cfg.H}x{cfg.W}, {cfg.K} kernels "
                               f"{cfg.R}x{cfg.S} stride {cfg.stride} pad {cfg.pad}, slice [{k0},{k1}), "
                               "fwd + bwd_data + bwd_weight",
                   "flops_per_step": 3 * F},
        "frac_of_mfma_peak": value / peak,
        "min_hbm_bytes_per_step": min_bytes,
        "hbm_gbs_on_min_bytes": min_bytes / (ms_per_step * 1e-3) / 1e9,
        "roofline": roofline,
        "kernels": kern,
    }
    if graph_ms is not None:
        out["ms_per_step_graph_replay"] = graph_ms
    if cpu_images > 0:
        out["cpu_baseline"] = cpu_baseline(cfg, x, w, dy, cpu_images)
    del xd, wd, dyd, y, dx, dw, ws
    torch.cuda.empty_cache()
    return out


def measure_partition(cfg_name, dtype_name, times, steps, warmup):
    """Times the layer split by Eq. (1) for the given probe times (all slices on this one GPU,
    conv_layer_*) next to the same layer as one slice; also runs the calibration probe."""
    import numpy as np
    import torch

    import paper_1712_02546_amd as cs
    from paper_1712_02546_amd import synth

    cfg = synth.CONFIGS[cfg_name]
    cfg = cfg.with_slice(0, cfg.K)
    dtype = cs.CONV_F32 if dtype_name == "f32" else cs.CONV_BF16
    x, w, dy = synth.make_inputs(cfg)
    dev = torch.device("cuda:0")

    def up(a):
        if dtype == cs.CONV_BF16:
            return torch.from_numpy(synth.f32_to_bf16_bits(synth.round_to_bf16(a)).view(np.int16)).to(dev).view(
                torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    xd, wd, dyd = up(x), up(w), up(dy)
    tdt = torch.float32 if dtype == cs.CONV_F32 else torch.bfloat16
    y = torch.zeros((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=tdt, device=dev)
    dx = torch.zeros((cfg.N, cfg.C, cfg.H, cfg.W), dtype=tdt, device=dev)
    dw = torch.zeros((cfg.K, cfg.C, cfg.R, cfg.S), dtype=torch.float32, device=dev)
    desc = cs.ConvDesc(cfg.N, cfg.C, cfg.H, cfg.W, cfg.K, cfg.R, cfg.S, cfg.stride, cfg.stride, cfg.pad, cfg.pad,
                       0, cfg.K, dtype, 0)
    shares, bounds = cs.conv_partition(times, cfg.K)
    mask = cs.pass_mask(cs.PASS_FWD, cs.PASS_BWD_DATA, cs.PASS_BWD_WEIGHT)
    need = max([cs.conv_layer_workspace_bytes(desc, bounds, p) for p in (0, 1, 2)] +
               [cs.conv_layer_workspace_bytes(desc, [0, cfg.K], p) for p in (0, 1, 2)] +
               [cs.conv_calibrate_workspace_bytes(desc, mask)])
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream

    def layer(b):
        cs.conv_layer_fwd(desc, b, xd, wd, y, ws, stream)
        cs.conv_layer_bwd_data(desc, b, dyd, wd, dx, ws, stream)
        cs.conv_layer_bwd_weight(desc, b, xd, dyd, dw, ws, stream)

    def timed(b):
        for _ in range(warmup):
            layer(b)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            layer(b)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    one = timed([0, cfg.K])
    split = timed(bounds)
    probe_s = cs.conv_calibrate(desc, mask, max(steps // 2, 1), ws, stream)
    finish, speedup = cs.conv_partition_estimate(times, shares)
    F3 = 3 * cfg.flops_per_pass
    return {"what": "layer split by Eq. (1), all slices on one GPU", "config": cfg.name, "dtype": dtype_name,
            "probe_times": times, "shares": shares, "bounds": bounds,
            "estimated_finish_of_slowest": finish, "estimated_speedup_over_fastest_alone": speedup,
            "ms_one_slice": one, "ms_partitioned": split, "partitioned_over_one": split / one,
            "tflops_one_slice": F3 / (one * 1e-3) / 1e12, "tflops_partitioned": F3 / (split * 1e-3) / 1e12,
            "calibration_probe_ms": probe_s * 1e3, "steps": steps, "warmup": warmup}


def scaling_study(cfg_name, dtype_name, max_devices, link_gbytes, comp_fraction, reps):
    """The form of the paper's scalability study (Section 4.2) with this GPU's numbers: the
    calibration probe gives the convolution time of one device, Eq. (1) the blocks of n equal
    devices, Eq. (2) (per-partition form) the elements the master exchanges, and one xGMI link
    of the master the bandwidth.  Returns one row per device count."""
    import torch

    import paper_1712_02546_amd as cs
    from paper_1712_02546_amd import synth

    cfg = synth.CONFIGS[cfg_name]
    dtype = cs.CONV_F32 if dtype_name == "f32" else cs.CONV_BF16
    desc = cs.ConvDesc(cfg.N, cfg.C, cfg.H, cfg.W, cfg.K, cfg.R, cfg.S, cfg.stride, cfg.stride, cfg.pad, cfg.pad,
                       0, cfg.K, dtype, 0)
    mask = cs.pass_mask(cs.PASS_FWD, cs.PASS_BWD_DATA, cs.PASS_BWD_WEIGHT)
    ws = torch.empty(cs.conv_calibrate_workspace_bytes(desc, mask), dtype=torch.uint8, device="cuda:0")
    t_conv = cs.conv_calibrate(desc, mask, reps, ws)
    t_comp = t_conv * comp_fraction / (1.0 - comp_fraction)
    layer = (cfg.H, cfg.C, cfg.R, cfg.K, cfg.P)
    es = 4 if dtype == cs.CONV_F32 else 2
    rows = []
    n = 1
    while n <= max_devices:
        shares, bounds = cs.conv_partition([t_conv] * n, cfg.K)
        # forward traffic of Eq. (2); the backward passes move the same maps the other way
        elements = 2 * cs.conv_comm_elements_partition(layer, cfg.N, bounds, 0)
        sec, sp, am = cs.conv_scaling_estimate([t_conv] * n, shares, t_comp, elements, es, link_gbytes * 8e9)
        rows.append({"devices": n, "kernels_per_device": bounds[1] - bounds[0], "elements": elements,
                     "batch_ms": sec * 1e3, "speedup": sp, "amdahl_bound": am})
        n *= 2
    return {"what": "scalability estimate in the form of Section 4.2", "config": cfg.name, "dtype": dtype_name,
            "probe_ms_fwd_bwd": t_conv * 1e3, "other_layers_fraction": comp_fraction,
            "link_GB_per_s": link_gbytes, "rows": rows}


def net_study(steps, warmup, batches, sizes):
    """Training step of the paper's network (Section 4.1) for its four sizes: time in the
    convolutions against time in the other layers ("Comp. time", Section 4.2)."""
    import torch

    from paper_1712_02546_amd import net as pnet

    rows = []
    for k1, k2 in sizes:
        for batch in batches:
            net = pnet.PaperNet(batch, k1, k2, seed=1)
            x = torch.rand((batch, 3, 32, 32), device="cuda:0")
            labels = torch.randint(0, 10, (batch,), device="cuda:0", dtype=torch.int32)
            for _ in range(warmup):
                net.step(x, labels)
            conv = other = 0.0
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                net.step(x, labels)
                c, o = net.times_ms()
                conv += c
                other += o
            wall = (time.perf_counter() - t0) * 1e3 / steps
            conv /= steps
            other /= steps
            rows.append({"kernels": f"{k1}:{k2}", "batch": batch, "conv_ms": conv, "other_ms": other,
                         "other_share": other / (conv + other), "amdahl_bound": (conv + other) / other,
                         "wall_ms_per_step": wall, "images_per_s": batch / ((conv + other) * 1e-3)})
            del net, x, labels
            torch.cuda.empty_cache()
    return {"what": "training step of the paper's network, convolutions against the other layers", "steps": steps,
            "warmup": warmup, "rows": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="cfg3", help="cfg1..cfg5b (default: the 1500-kernel layer)")
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--cpu-images", type=int, default=1 << 30,
                    help="images in the CPU-oracle sample (default: the whole batch; 0 = skip)")
    ap.add_argument("--table", action="store_true", help="measure all configurations (not the contract line)")
    ap.add_argument("--graph", action="store_true",
                    help="also record the step into a HIP graph and time its replay (extra key ms_per_step_graph_replay)")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="first run one plain device copy of this many MiB (a kernel of known HBM traffic "
                         "to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings with)")
    ap.add_argument("--partition", default="",
                    help="comma-separated probe times of pretend devices: time the layer split by Eq. (1) "
                         "(all slices on this GPU) against one slice (not the contract line)")
    ap.add_argument("--scaling", type=int, default=0,
                    help="largest device count of a scalability estimate in the form of the paper's "
                         "(measured probe time, Eq. (1), Eq. (2), one xGMI link; not the contract line)")
    ap.add_argument("--link-gbytes", type=float, default=153.0, help="bandwidth of the master's link, GB/s")
    ap.add_argument("--comp-fraction", type=float, default=0.13,
                    help="share of the other layers in the single-device time (the paper measured 13-25 %%)")
    ap.add_argument("--net", action="store_true",
                    help="time training steps of the paper's four network sizes: convolutions against the other "
                         "layers (not the contract line)")
    ap.add_argument("--net-batches", default="64,128,1024")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only; --gpus must be 1 "
                 "(the kernel-slice argument is how the layer would be sharded across devices)")

    import torch

    import paper_1712_02546_amd as cs

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    cs.load()

    if args.calib_copy_mib > 0:
        src = torch.ones(args.calib_copy_mib * (1 << 18), dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)   # reads and writes calib_copy_mib MiB each
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    if args.net:
        sizes = [(50, 500), (150, 800), (300, 1000), (500, 1500)]
        print(json.dumps(net_study(args.steps, args.warmup, [int(b) for b in args.net_batches.split(",")], sizes)))
        return

    if args.scaling > 0:
        print(json.dumps(scaling_study(args.config, args.dtype, args.scaling, args.link_gbytes, args.comp_fraction,
                                       max(args.steps // 2, 1))))
        return

    if args.partition:
        times = [float(v) for v in args.partition.split(",")]
        print(json.dumps(measure_partition(args.config, args.dtype, times, args.steps, args.warmup)))
        return

    if not args.table:
        print(json.dumps(measure(args.config, args.dtype, args.steps, args.warmup, args.cpu_images, graph=args.graph)))
        return

    runs = [("cfg1", "f32"), ("cfg2", "f32"), ("cfg3", "f32"), ("cfg4", "f32"), ("cfg5a", "f32"), ("cfg5b", "f32"),
            ("cfg5a", "bf16"), ("cfg5b", "bf16"), ("cfg3", "bf16")]
    rows = []
    for name, dt in runs:
        # Short steps need many repetitions before the start of the timed region (the host's first launches, which
        # nothing hides) stops showing: time about a quarter of a second per configuration, at least args.steps steps.
        est = measure(name, dt, 3, 2, 0)["ms_per_step"]
        steps = max(args.steps, min(1000, int(250.0 / est)))
        r = measure(name, dt, steps, args.warmup, 0, per_pass=True, graph=True)
        print(json.dumps(r), flush=True)
        rows.append((name, dt, r))
    print("| cfg | dtype | steps | fwd ms | bwd_data ms | bwd_weight ms | step ms | TFLOP/s | % MFMA peak | "
          "GB/s on minimal bytes | step ms replayed from a HIP graph |", file=sys.stderr)
    print("|---|---|---|---|---|---|---|---|---|---|---|", file=sys.stderr)
    for name, dt, r in rows:
        k = {x["entry"]: x for x in r["kernels"]}
        print(f"| {name} | {dt} | {r['steps']} | {k['conv_fwd']['entry_ms']:.3f} | {k['conv_bwd_data']['entry_ms']:.3f} | "
              f"{k['conv_bwd_weight']['entry_ms']:.3f} | {r['ms_per_step']:.3f} | {r['value']:.2f} | "
              f"{100 * r['frac_of_mfma_peak']:.1f} | {r['hbm_gbs_on_min_bytes']:.0f} | "
              f"{r['ms_per_step_graph_replay']:.3f} |", file=sys.stderr)


if __name__ == "__main__":
    main()
