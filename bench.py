#!/usr/bin/env python3
"""Throughput of the fused fake-quantization hot path on one MI355X.

One step = fq_forward + fq_backward (Eq. (3)-(5) and the STE backward with the per-channel
scale-gradient reduction) over the headline tensor: FP16 1x384x120x160, 384 learnable scales,
signed 8-bit codes.  Inputs are synthetic (seeded, DPVO-feature-map shaped) and resident in HBM
before the timed region.  Successive steps rotate over a ring of distinct buffer sets larger than
the 256 MB Infinity Cache, so every step streams from HBM rather than from cache.

The timed steps are enqueued as one HIP graph (captured before the timed region, the way a
training loop over a static tensor list would run them; --launch eager enqueues every kernel from
Python instead and is bound by the interpreter at these kernel sizes).

Prints one JSON line: whole-job GB/s (algorithmic bytes: forward 2b + backward 3b per element),
the roofline position of the dominant kernel (the backward kernel, 3b bytes per element: mean,
median and minimum over a dense series of back-to-back launches on the cold ring, timed with HIP
events on the launch stream), what plain streaming kernels of the same launch shape take for the
same bytes, and the CPU oracle timed on this host on one core and on all cores.

Other workloads (--workload), the forward alone (--pass forward: 2b bytes per element) and the
int8 code-emission forward (--pass codes: x in, packed int8 codes out, b+1 bytes per element) use
the same machinery; lists of tensors go through the multi-tensor entry points, one launch per
pass.  --pass distill times fq_distill_loss on a student/teacher pair of the workload's shape.
--floor-sweep adds the plain streaming kernel's time over a range of sizes and the fit
time = launch + bytes / bandwidth that bounds a launch of a given size.
"""
import argparse
import ctypes
import glob
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
RING_BYTES = 1200 << 20        # total footprint of the rotating buffer sets
SERIES_TRAINS = 40             # dense series: this many event-bracketed trains ...
SERIES_MIN_PER_TRAIN = 60      # ... of at least this many back-to-back launches each

# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this command with --copy-calibration (each counter scaled by what it reads for a plain copy of
# known size in the same run); the tables are in profiles/.  An entry is None until its kernel's
# counters have been taken, and is reset to None whenever that kernel changes.
TRAFFIC_BYTES_PER_LAUNCH = {
    ("feature_fp16_per_channel", "train"): 44488995,      # backward_kernel<f16>: 1.006 x the algorithmic bytes
    ("feature_fp16_per_channel", "forward"): 29591391,    # forward_kernel<f16>: 1.003 x
    ("feature_fp16_per_channel", "codes"): 22228614,      # forward_kernel<f16, codes only>: 1.005 x
    ("train_batch_fp16", "train"): 222084135,             # 1.004 x
    ("multi_tensor_mixed", "train"): 3359498369,          # backward_multi_kernel: 1.012 x
    ("conv_weights_fp32", "train"): 17958351,             # 1.015 x
    ("act_fp32_per_tensor", "train"): 1995130,            # 1.082 x (a 1.8 MB launch: theta, partial sums, tickets count)
    ("feature_fp16_per_channel", "distill"): 44372788,    # fused kernel + the block that adds the tile sums: 1.003 x
    ("train_batch_fp16", "distill"): 221381819,           # 1.001 x
}

WORKLOAD_TEXT = {
    "act_fp32_per_tensor": "act_fp32_per_tensor: FP32 1x128x30x40, one scale, codes -128..127",
    "feature_fp16_per_channel": "feature_fp16_per_channel: FP16 1x384x120x160 NCHW, 384 per-channel scales, "
                                "codes -128..127",
    "conv_weights_fp32": "conv_weights_fp32: FP32 384x384x3x3 + 128x128x3x3, per-output-channel scales, codes "
                         "-127..127, one multi-tensor launch per pass",
    "train_batch_fp16": "train_batch_fp16: FP16 15x128x120x160, 128 per-channel scales, codes -128..127",
    "multi_tensor_mixed": "multi_tensor_mixed: 64 mixed FP16/FP32, 4/8-bit, per-tensor/per-channel tensors, "
                          "about 1 GiB of inputs, one multi-tensor launch per pass",
}


class Events:
    """Raw HIP events on a given stream (torch.cuda.Event only sees torch's current stream)."""

    def __init__(self):
        hip = ctypes.CDLL("libamdhip64.so")
        hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.hip = hip

    def new(self):
        e = ctypes.c_void_p()
        if self.hip.hipEventCreate(ctypes.byref(e)) != 0:
            sys.exit("bench.py: hipEventCreate failed")
        return e

    def record(self, e, stream_ptr):
        if self.hip.hipEventRecord(e, stream_ptr) != 0:
            sys.exit("bench.py: hipEventRecord failed")

    def elapsed_us(self, a, z):
        ms = ctypes.c_float()
        if self.hip.hipEventSynchronize(z) != 0 or self.hip.hipEventElapsedTime(ctypes.byref(ms), a, z) != 0:
            sys.exit("bench.py: hipEventElapsedTime failed")
        return ms.value * 1e3


def dense_series(ev, torch, launch, ring, trains=SERIES_TRAINS, min_per_train=SERIES_MIN_PER_TRAIN):
    """Per-launch duration of `launch(k, stream_ptr)` (k = buffer set).  A train of back-to-back
    launches that walks the ring is captured once into a HIP graph; each of `trains` replays is
    bracketed by one pair of HIP events on the replaying stream, and a replay's time divided by
    the launches in it is one sample.  (Launched one by one from Python, kernels shorter than
    about 7 us would show the interpreter's enqueue rate instead of their own duration; an event
    pair around a single launch would add several microseconds of its own.)  Returns statistics
    over the trains' per-launch means."""
    per_train = ring * -(-min_per_train // ring)
    side = torch.cuda.Stream()
    sp = side.cuda_stream
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        for k in range(ring):                               # untimed pass over the ring
            launch(k, sp)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            for n in range(per_train):
                launch(n % ring, sp)
        side.synchronize()
        graph.replay()                                      # untimed: the graph's first-use costs
        side.synchronize()
        pairs = []
        for _ in range(trains):
            a, z = ev.new(), ev.new()
            ev.record(a, sp)
            graph.replay()
            ev.record(z, sp)
            pairs.append((a, z))
        side.synchronize()
    us = sorted(ev.elapsed_us(a, z) / per_train for a, z in pairs)
    for a, z in pairs:
        ev.hip.hipEventDestroy(a)
        ev.hip.hipEventDestroy(z)
    del graph
    return {"mean_us": sum(us) / len(us), "median_us": us[len(us) // 2], "min_us": us[0], "max_us": us[-1],
            "trains": trains, "launches": trains * per_train}


def gpu_clock_state():
    """Current shader / memory clock and the power policy as the driver reports them (sysfs)."""
    out = {}
    for dev in sorted(glob.glob("/sys/class/drm/card*/device")):
        try:
            for key, name in (("sclk_mhz", "pp_dpm_sclk"), ("mclk_mhz", "pp_dpm_mclk")):
                cur = [ln for ln in open(os.path.join(dev, name)).read().splitlines() if ln.strip().endswith("*")]
                if cur:
                    out[key] = cur[0].split(":")[1].replace("*", "").strip()
            out["performance_level"] = open(os.path.join(dev, "power_dpm_force_performance_level")).read().strip()
        except OSError:
            continue
        if out:
            out["device"] = os.path.basename(os.path.dirname(dev))
            break
    return out or None


def host_threads():
    """Threads for the all-cores oracle baseline: the cores this process may use."""
    n = os.cpu_count() or 1
    try:
        n = min(n, len(os.sched_getaffinity(0)))
    except (AttributeError, OSError):
        pass
    env = os.environ.get("OMP_NUM_THREADS", "")
    if env.isdigit() and int(env) > 0:
        n = min(n, int(env))
    return max(1, n)


def time_cpu(fn, target_s=5.0):
    """Median wall time of fn() over 3 to 15 runs, aiming at about target_s of CPU work."""
    reps, times, rep = 3, [], 0
    while rep < reps:
        rep += 1
        c0 = time.perf_counter()
        fn()
        times.append(time.perf_counter() - c0)
        if rep == 1:
            reps = int(min(15, max(3, round(target_s / max(times[0], 1e-3)))))
    return sorted(times)[len(times) // 2], reps


def floor_sweep(ev, torch, fq, inputs):
    """Plain streaming kernel (fq_probe_stream, `inputs` inputs and one output) over a range of
    sizes on a cold ring, and the least-squares line time = launch + bytes / bandwidth."""
    pool = 640 << 20
    a = torch.empty(pool, dtype=torch.uint8, device="cuda").fill_(1)
    b = torch.empty(pool, dtype=torch.uint8, device="cuda").fill_(2) if inputs == 2 else None
    o = torch.empty(pool, dtype=torch.uint8, device="cuda")
    pa, po = a.data_ptr(), o.data_ptr()
    pb = b.data_ptr() if inputs == 2 else 0
    rows = []
    for per_stream in (1843200, 3686400, 7372800, 14745600, 29491200, 58982400, 117964800):
        ring = pool // per_stream

        def launch(k, sp, n=per_stream):
            fq.fq_probe_stream_raw(inputs, pa + k * n, pb + k * n if pb else 0, po + k * n, n, sp)

        st = dense_series(ev, torch, launch, ring, trains=20)
        rows.append({"bytes_per_stream": per_stream, "bytes_moved": (inputs + 1) * per_stream,
                     "mean_us": round(st["mean_us"], 2), "min_us": round(st["min_us"], 2)})
    xs = [r["bytes_moved"] for r in rows[2:]]               # the line is fitted from 22 MB upwards
    ys = [r["mean_us"] for r in rows[2:]]
    n = len(xs)
    mx, my = sum(xs) / n, sum(ys) / n
    slope = sum((x - mx) * (y - my) for x, y in zip(xs, ys)) / sum((x - mx) ** 2 for x in xs)
    return {"kernel": "fq_probe_stream, %d input(s) + 1 output, 256-thread blocks of 20 KiB per stream" % inputs,
            "rows": rows, "fit_launch_us": round(my - slope * mx, 2), "fit_bandwidth_GBs": round(1e-3 / slope, 1)}


def distill_bench(args, cases, fq, torch, np):
    """--pass distill: fq_distill_loss (loss and gradient with respect to the student) on one
    student/teacher pair shaped like the workload's tensor.  A step is one call.  Algorithmic
    bytes per element: read student, read teacher, write the gradient = 3 b; anything the
    implementation moves beyond that is its own traffic and is not counted."""
    if len(cases) != 1:
        sys.exit("bench.py: --pass distill takes a single-tensor workload")
    cs = cases[0]
    io_bytes = cs.numel * cs.itemsize
    set_bytes = 3 * io_bytes
    ring = max(2, RING_BYTES // set_bytes) if set_bytes < RING_BYTES else 1
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream
    hs, ht = torch.from_numpy(cs.x.reshape(-1)), torch.from_numpy(cs.gy.reshape(-1))
    out = torch.zeros(3, dtype=torch.float64, device="cuda")
    descs, keep = [], []
    for _ in range(ring):
        a, b = hs.cuda(), ht.cuda()
        g = torch.empty_like(a)
        keep.append((a, b, g))
        descs.append(fq.FqDistill.from_torch(cs.outer, cs.channels, cs.inner, a, b, out, g, lam=0.5))
    ws_bytes = fq.fq_distill_workspace_bytes(descs[0])
    ws = torch.empty(max(ws_bytes, 8) // 8, dtype=torch.float64, device="cuda")
    ev = Events()

    for i in range(args.warmup):
        fq.fq_distill_loss(descs[i % ring], ws, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        fq.fq_distill_loss(descs[(args.warmup + i) % ring], ws, stream)
    t_enq = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    series = dense_series(ev, torch, lambda k, p: fq.fq_distill_loss(descs[k], ws, p), ring)
    for i in range(args.copy_calibration):           # plain copies of known size for --pmc runs
        a, _, g = keep[i % ring]
        g.copy_(a)
    torch.cuda.synchronize()
    sec_per_step = (t1 - t0) / args.steps
    step_bytes = 3 * io_bytes
    value = step_bytes / sec_per_step / 1e9
    achieved = step_bytes / (series["mean_us"] * 1e-6) / 1e9
    roofline = {"bound": "hbm", "kernel": "fq_distill_loss: all kernels of one call",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": TRAFFIC_BYTES_PER_LAUNCH.get((args.workload, "distill")),
                "bytes_per_launch": step_bytes, "avg_us": round(series["mean_us"], 2),
                "median_us": round(series["median_us"], 2), "min_us": round(series["min_us"], 2),
                "samples": series["launches"], "trains": series["trains"],
                "method": "HIP events around replays of a HIP graph holding a train of back-to-back calls over "
                          "the cold ring; statistics over the trains' per-call means"}
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import fq_oracle
        fq_oracle.lib()
        x3 = cs.x.reshape(cs.outer, cs.channels, cs.inner)
        t3 = cs.gy.reshape(cs.outer, cs.channels, cs.inner)
        take = max(1, min(cs.outer, 40_000_000 // max(1, cs.channels * cs.inner)))
        x3, t3 = x3[:take], t3[:take]
        med, reps = time_cpu(lambda: fq_oracle.distill(x3, t3, 0.5))
        cpu = {"value": round(3 * x3.size * cs.itemsize / med / 1e9, 4), "unit": "GB/s", "cores": 1,
               "kind": "oracle", "sample": "%d of %d images of the pair (%d elements), loss and gradient, "
                                           "median of %d runs, %.2f s each" % (take, cs.outer, x3.size, reps, med)}
    print(json.dumps({
        "metric": "distillation loss + gradient GB/s", "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.workload] + ", as one student/teacher pair [n, channels, "
                               "h*w]: loss of Eq. (7) and its gradient",
                   "launch": "eager", "elements": cs.numel, "bytes_per_step": step_bytes,
                   "ring_buffer_sets": int(ring), "workspace_bytes": ws_bytes},
        "host_enqueue_us_per_step": round((t_enq - t0) / args.steps * 1e6, 2),
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "gpu_clocks": gpu_clock_state(),
        "roofline": roofline, "cpu_baseline": cpu}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="feature_fp16_per_channel",
                    help="one of paper_2511_12653_amd.workloads.WORKLOAD_NAMES (default: the headline "
                         "tensor); lists of tensors go through the multi-tensor entry points")
    ap.add_argument("--pass", dest="which", default="train", choices=["train", "forward", "codes", "distill"],
                    help="train: forward + STE backward (default); forward: the forward alone (x in, y "
                         "out); codes: forward that writes only the packed int8 codes; distill: the "
                         "distillation loss and its gradient for one student/teacher pair of the "
                         "workload's shape (single-tensor workloads)")
    ap.add_argument("--launch", default="graph", choices=["graph", "eager"],
                    help="graph (default): the timed steps are captured once into a HIP graph and the "
                         "timed region is one replay; eager: every kernel is enqueued from Python")
    ap.add_argument("--cache-warm", action="store_true",
                    help="use one buffer set for every step instead of the HBM-cold ring (labelled in the "
                         "output; a different, cache-assisted figure)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="N",
                    help="after the timed region also run N plain device copies of the first tensor "
                         "(torch copy_), so that a rocprofv3 --pmc run of this command holds a copy "
                         "kernel of known size to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--no-kernel-series", action="store_true",
                    help="skip the dense per-kernel series and the streaming context (roofline becomes "
                         "null); for profiler runs that should hold the timed steps only")
    ap.add_argument("--floor-sweep", action="store_true",
                    help="also time the plain streaming kernel over a range of sizes and fit launch cost "
                         "and bandwidth")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on one GPU (got --gpus %d); several GPUs would each take "
                 "their own tensors or channel ranges, which this benchmark does not launch" % args.gpus)

    import numpy as np
    import torch
    from paper_2511_12653_amd import build as lib_build
    lib_build.ensure_built()
    from paper_2511_12653_amd import binding as fq
    from paper_2511_12653_amd import workloads

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; there is no CPU fallback")
    torch.cuda.set_device(0)
    if args.workload not in workloads.WORKLOAD_NAMES:
        sys.exit("bench.py: unknown workload %r (choose from %s)" % (
            args.workload, ", ".join(workloads.WORKLOAD_NAMES)))
    train = args.which == "train"
    codes = args.which == "codes"

    cases = workloads.make(args.workload)
    if args.which == "distill":
        return distill_bench(args, cases, fq, torch, np)
    if codes:
        cases = [cs for cs in cases if cs.qmin >= -128 and cs.qmax <= 127]
    multi = len(cases) > 1
    numel = sum(cs.numel for cs in cases)
    io_bytes = sum(cs.numel * cs.itemsize for cs in cases)        # sum over tensors of b * elements
    fwd_bytes = io_bytes + numel if codes else 2 * io_bytes      # bytes one forward launch moves
    set_bytes = 4 * io_bytes if train else fwd_bytes
    ring = max(2, RING_BYTES // set_bytes) if set_bytes < RING_BYTES else 1
    if args.cache_warm:
        ring = 1
    ev = Events()

    # ---- device buffers: `ring` independent sets, descriptors marshalled once ------------------
    per_case = [(torch.from_numpy(cs.x.reshape(-1)), torch.from_numpy(cs.gy.reshape(-1)),
                 torch.from_numpy(cs.theta).cuda(), torch.empty(cs.channels, device="cuda"),
                 torch.empty(cs.channels, device="cuda")) for cs in cases]
    sets, keep, first_bufs = [], [], []
    for _ in range(ring):
        group = []
        for j, (cs, (hx, hg, theta, gs, gtheta)) in enumerate(zip(cases, per_case)):
            common = dict(theta=theta, eps=cs.eps, s_min=cs.s_min, s_max=cs.s_max, flags=cs.flags)
            x = hx.cuda()
            if train:
                gy = hg.cuda()
                y, gx = torch.empty_like(x), torch.empty_like(x)
                keep.append((x, y, gy, gx))
                group.append(fq.FqTensor.from_torch(cs.outer, cs.channels, cs.inner, cs.qmin, cs.qmax, x=x,
                                                    y=y, gy=gy, gx=gx, gs=gs, gtheta=gtheta, **common))
            elif codes:
                q = torch.empty(cs.numel, dtype=torch.int8, device="cuda")
                y = torch.empty_like(x) if (j == 0 and args.copy_calibration) else None
                keep.append((x, q, y))
                group.append(fq.FqTensor.from_torch(cs.outer, cs.channels, cs.inner, cs.qmin, cs.qmax, x=x,
                                                    q=q, s=gs, **common))
            else:
                y = torch.empty_like(x)
                keep.append((x, y))
                group.append(fq.FqTensor.from_torch(cs.outer, cs.channels, cs.inner, cs.qmin, cs.qmax, x=x,
                                                    y=y, s=gs, **common))
            if j == 0:
                first_bufs.append((x, y))
        sets.append(fq.fq_tensor_array(group) if multi else group[0])

    def zeros(nbytes):
        t = torch.zeros(nbytes // 4, dtype=torch.int32, device="cuda")
        keep.append(t)
        return t

    # ---- the launches of one step, on the stream whose handle is passed ---------------------------
    if multi:
        # a static tensor list: prepare once (descriptor table resident in a workspace of its own
        # per plan), then each pass is one kernel launch and nothing else
        plans = []
        for d in sets:
            pf = fq.fq_plan_create(d, fq.FQ_MODE_FORWARD, zeros(fq.fq_workspace_bytes(d, fq.FQ_MODE_FORWARD)))
            pb = None
            if train:
                pb = fq.fq_plan_create(d, fq.FQ_MODE_BACKWARD, zeros(fq.fq_workspace_bytes(d, fq.FQ_MODE_BACKWARD)))
            plans.append((pf, pb))
        torch.cuda.synchronize()

        def forward(k, sp):
            fq.fq_plan_run(plans[k][0], sp)

        def backward(k, sp):
            fq.fq_plan_run(plans[k][1], sp)
    else:
        ws = zeros(fq.fq_workspace_bytes(sets[0], fq.FQ_MODE_BACKWARD)) if train else None

        def forward(k, sp):
            fq.fq_forward(sets[k], sp)

        def backward(k, sp):
            fq.fq_backward(sets[k], ws, sp)

    def step(i, sp):
        k = i % ring
        forward(k, sp)
        if train:
            backward(k, sp)

    # ---- the timed region: exactly `steps` steps, after `warmup` untimed ones ---------------------
    main_sp = torch.cuda.current_stream().cuda_stream
    for i in range(args.warmup):
        step(i, main_sp)
    torch.cuda.synchronize()
    if args.launch == "graph":
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for i in range(args.steps):
                    step(args.warmup + i, side.cuda_stream)
        torch.cuda.synchronize()
        graph.replay()                                   # one untimed replay: the graph's own first-use costs
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        graph.replay()
        t_enq = time.perf_counter()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    else:
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(args.warmup + i, main_sp)
        t_enq = time.perf_counter()
        torch.cuda.synchronize()
        t1 = time.perf_counter()

    sec_per_step = (t1 - t0) / args.steps
    step_bytes = 5 * io_bytes if train else fwd_bytes
    value = step_bytes / sec_per_step / 1e9
    # ---- the dominant kernel alone: dense series on the cold ring ---------------------------------
    roofline, context, sweep = None, None, None
    if not args.no_kernel_series:
        dominant = backward if train else forward
        series = dense_series(ev, torch, dominant, ring)
        kernel_bytes = 3 * io_bytes if train else fwd_bytes
        achieved = kernel_bytes / (series["mean_us"] * 1e-6) / 1e9
        dt = "f16" if cases[0].itemsize == 2 else "f32"
        if train:
            kname = "backward_multi_kernel<fused>" if multi else "backward_kernel<%s, fused>" % dt
        elif codes:
            kname = "forward_multi_kernel<codes>" if multi else "forward_kernel<%s, codes>" % dt
        else:
            kname = "forward_multi_kernel" if multi else "forward_kernel<%s>" % dt
        traffic = None if args.cache_warm else TRAFFIC_BYTES_PER_LAUNCH.get((args.workload, args.which))
        roofline = {"bound": "hbm", "kernel": kname, "achieved": round(achieved, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": traffic, "bytes_per_launch": kernel_bytes,
                    "avg_us": round(series["mean_us"], 2), "median_us": round(series["median_us"], 2),
                    "min_us": round(series["min_us"], 2), "max_us": round(series["max_us"], 2),
                    "samples": series["launches"], "trains": series["trains"],
                    "method": "after the timed region: HIP events on the launch stream around replays of a HIP "
                              "graph that holds a train of back-to-back launches of this kernel over the cold "
                              "ring; avg/median/min/max over the trains' per-launch means"}

        # ---- context: what kernels without arithmetic take for the same traffic --------------------
        # (single-tensor training workloads).  fq_probe_stream has the library's launch shape;
        # torch's device copy and torch.add are the platform library's kernels for the same bytes.
        if train and not multi:
            us = lambda fn: round(dense_series(ev, torch, fn, ring, trains=20)["mean_us"], 2)
            nbytes = io_bytes
            ptr = [tuple(t.data_ptr() for t in keep[k]) for k in range(ring)]      # x, y, gy, gx of set k
            context = {
                "note": "us per launch, back-to-back launches over the same cold ring (graph trains)",
                "fq_forward_us": us(forward), "fq_backward_us": round(series["mean_us"], 2),
                "empty_launch_us": us(lambda k, sp: fq.fq_probe_stream_raw(0, 0, 0, 0, nbytes, sp)),
                "probe_1in_1out_us": us(lambda k, sp: fq.fq_probe_stream_raw(1, ptr[k][0], 0, ptr[k][1], nbytes, sp)),
                "probe_2in_1out_us": us(lambda k, sp: fq.fq_probe_stream_raw(2, ptr[k][0], ptr[k][2], ptr[k][3],
                                                                             nbytes, sp)),
                "torch_copy_us": us(lambda k, sp: keep[k][1].copy_(keep[k][0])),
                "torch_add_us": us(lambda k, sp: torch.add(keep[k][0], keep[k][2], out=keep[k][3])),
            }
        if args.floor_sweep:
            sweep = floor_sweep(ev, torch, fq, 2 if train else 1)

    for i in range(args.copy_calibration):
        x, y = first_bufs[i % ring]
        y.copy_(x)
    torch.cuda.synchronize()

    # ---- the CPU oracle beside it: one core, then all cores (channels split over threads) ---------
    cpu, cpu_all = None, None
    if not args.no_cpu_baseline:
        from oracle import fq_oracle
        fq_oracle.lib()
        # bounded sample: whole tensors of the workload, in order, until about 40 M elements
        sample, n_sample = [], 0
        for cs in cases:
            if sample and n_sample + cs.numel > 40_000_000:
                break
            sample.append(cs)
            n_sample += cs.numel
        per_el = lambda cs: 5 * cs.itemsize if train else (cs.itemsize + 1 if codes else 2 * cs.itemsize)
        sample_bytes = sum(per_el(cs) * cs.numel for cs in sample)

        def oracle_pass():
            for cs in sample:
                s_, active = fq_oracle.scale(cs.theta, cs.eps, cs.s_min, cs.s_max)
                fq_oracle.forward(cs.x, s_, cs.qmin, cs.qmax, cs.outer, cs.channels, cs.inner, want_q=codes)
                if train:
                    fq_oracle.backward(cs.x, cs.gy, s_, cs.theta, active, cs.qmin, cs.qmax,
                                       cs.outer, cs.channels, cs.inner)

        what = "fwd+bwd" if train else ("forward with codes" if codes else "forward")
        legs = []
        for threads in (1, host_threads()):
            used = fq_oracle.set_threads(threads)
            med, reps = time_cpu(oracle_pass)
            legs.append({"value": round(sample_bytes / med / 1e9, 4), "unit": "GB/s", "cores": used,
                         "kind": "oracle",
                         "sample": "%d of %d tensors of the workload (%d elements, %s), median of %d runs, "
                                   "%.2f s each%s" % (len(sample), len(cases), n_sample, what, reps, med,
                                                      "" if used == 1 else "; channels split over threads"),
                         "elements_per_s": round(n_sample / med, 1)})
        fq_oracle.set_threads(1)
        cpu, cpu_all = legs

    out = {
        "metric": ("fake-quant fwd+bwd GB/s" if train else
                   "fake-quant int8 code emission GB/s" if codes else "fake-quant forward GB/s"),
        "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.workload] + (", forward + STE backward" if train else
                                                               ", forward writing int8 codes only" if codes
                                                               else ", forward only"),
                   "launch": ("one HIP graph holding the %d timed steps, replayed once" % args.steps
                              if args.launch == "graph" else "eager: each kernel enqueued from Python"),
                   "tensors": len(cases), "launches_per_step": 2 if train else 1, "elements": numel,
                   "bytes_per_step": step_bytes, "ring_buffer_sets": int(ring),
                   "ring_bytes": int(ring * set_bytes),
                   "residency": "cache-warm: the same buffers every step" if args.cache_warm else
                                "HBM-cold: steps rotate over the ring" if ring > 1 else
                                "one buffer set larger than the caches"},
        "elements_per_s": round(numel / sec_per_step, 1),
        "host_enqueue_us_per_step": round((t_enq - t0) / args.steps * 1e6, 2),
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "gpu_clocks": gpu_clock_state(),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "cpu_baseline_all_cores": cpu_all,
        "streaming_context": context,
        "floor_sweep": sweep,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
