#!/usr/bin/env python3
"""Throughput of the fused fake-quantization hot path on one MI355X.

One step = fq_forward + fq_backward (Eq. (3)-(5) and the STE backward with the per-channel
scale-gradient reduction) over the headline tensor: FP16 1x384x120x160, 384 learnable scales,
signed 8-bit codes.  Inputs are synthetic (seeded, DPVO-feature-map shaped) and resident in HBM
before the timed region.  Successive steps rotate over a ring of distinct buffer sets larger than
the 256 MB Infinity Cache, so every step streams from HBM rather than from cache.

Prints one JSON line: whole-job GB/s (algorithmic bytes: forward 2b + backward 3b per element),
the roofline position of the dominant kernel (the backward kernel, 3b bytes per element, timed
inside the timed region with HIP events on the launch stream) and the CPU oracle timed on this
host beside it.

Other workloads (--workload), the forward alone (--pass forward: 2b bytes per element) and the
int8 code-emission forward (--pass codes: x in, packed int8 codes out, b+1 bytes per element) use
the same machinery; lists of tensors go through the multi-tensor entry points, one launch per
pass.  --pass distill times fq_distill_loss on a student/teacher pair of the workload's shape.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
RING_BYTES = 1200 << 20        # total footprint of the rotating buffer sets
EVENT_EVERY = 8                # one bracketed step in this many
# HBM bytes per backward launch on the headline tensor, from the rocprofv3 FETCH_SIZE / WRITE_SIZE
# counter runs summarised in profiles/ (each scaled by a plain copy of known size in the same run).
# Set to None whenever the backward kernel changes until the counters are taken again.
TRAFFIC_BYTES_PER_LAUNCH = 44454849
# The same for the forward kernel (y only) on the headline tensor, from the same counter runs.
FORWARD_TRAFFIC_BYTES_PER_LAUNCH = 29578918

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


# HBM bytes per fq_distill_loss call (both kernels) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# of this command with --copy-calibration, scaled by the plain copy in the same run; see
# profiles/distill_kernels_feature_and_train_batch.md.  Set an entry to None when its kernels change.
DISTILL_TRAFFIC_BYTES_PER_CALL = {"feature_fp16_per_channel": 76335808, "train_batch_fp16": 378033465}


def distill_bench(args, cases, fq, torch, np):
    """--pass distill: fq_distill_loss (loss and gradient with respect to the student) on one
    student/teacher pair shaped like the workload's tensor.  A step is one call (two kernels).
    Algorithmic bytes per element: read student, read teacher, write the gradient = 3 b; the
    second read of the pair by the gradient kernel and the per-position statistics are the
    implementation's own traffic and are not counted."""
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
    ws = torch.empty(ws_bytes // 8, dtype=torch.float64, device="cuda")

    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]

    def new_event():
        e = ctypes.c_void_p()
        if hip.hipEventCreate(ctypes.byref(e)) != 0:
            sys.exit("bench.py: hipEventCreate failed")
        return e

    for i in range(args.warmup):
        fq.fq_distill_loss(descs[i % ring], ws, stream)
    torch.cuda.synchronize()
    ev_a, ev_z = new_event(), new_event()
    t0 = time.perf_counter()
    hip.hipEventRecord(ev_a, sp)
    for i in range(args.steps):
        fq.fq_distill_loss(descs[(args.warmup + i) % ring], ws, stream)
    hip.hipEventRecord(ev_z, sp)
    t_enq = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms = ctypes.c_float()
    hip.hipEventElapsedTime(ctypes.byref(ms), ev_a, ev_z)
    for i in range(args.copy_calibration):           # plain copies of known size for --pmc runs
        a, _, g = keep[i % ring]
        g.copy_(a)
    torch.cuda.synchronize()
    sec_per_step = (t1 - t0) / args.steps
    gpu_sec_per_step = ms.value * 1e-3 / args.steps
    step_bytes = 3 * io_bytes
    value = step_bytes / sec_per_step / 1e9
    achieved = step_bytes / gpu_sec_per_step / 1e9
    roofline = {"bound": "hbm", "kernel": "fq_distill_loss: distill_stats_kernel + distill_grad_kernel of one call",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": DISTILL_TRAFFIC_BYTES_PER_CALL.get(args.workload),
                "bytes_per_launch": step_bytes, "avg_us": round(gpu_sec_per_step * 1e6, 2),
                "method": "one HIP event pair on the launch stream around all timed calls, divided by "
                          "the number of calls"}
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import fq_oracle
        fq_oracle.lib()
        x3 = cs.x.reshape(cs.outer, cs.channels, cs.inner)
        t3 = cs.gy.reshape(cs.outer, cs.channels, cs.inner)
        take = max(1, min(cs.outer, 40_000_000 // max(1, cs.channels * cs.inner)))
        x3, t3 = x3[:take], t3[:take]
        reps, times, rep = 3, [], 0
        while rep < reps:
            rep += 1
            c0 = time.perf_counter()
            fq_oracle.distill(x3, t3, 0.5)
            times.append(time.perf_counter() - c0)
            if rep == 1:
                reps = int(min(15, max(3, round(5.0 / max(times[0], 1e-3)))))
        med = sorted(times)[len(times) // 2]
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
                   "launches_per_step": 2, "elements": cs.numel, "bytes_per_step": step_bytes,
                   "ring_buffer_sets": int(ring), "workspace_bytes": ws_bytes},
        "host_enqueue_us_per_step": round((t_enq - t0) / args.steps * 1e6, 2),
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
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
                         "out); codes: forward that writes only the packed int8 codes; distill: the distillation loss and its gradient for one "
                         "student/teacher pair of the workload's shape (single-tensor workloads)")
    ap.add_argument("--cache-warm", action="store_true",
                    help="use one buffer set for every step instead of the HBM-cold ring (labelled in the "
                         "output; a different, cache-assisted figure)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="N",
                    help="after the timed region also run N plain device copies of the first tensor "
                         "(torch copy_), so that a rocprofv3 --pmc run of this command holds a copy "
                         "kernel of known size to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="put no timing events into the timed region (roofline becomes null)")
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
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream

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

    # ---- the launches of one step ---------------------------------------------------------------
    if multi:
        # a static tensor list: prepare once (descriptor table resident in a workspace of its own
        # per plan), then each pass is one kernel launch and nothing else
        plans = []
        for d in sets:
            pf = fq.fq_plan_create(d, fq.FQ_MODE_FORWARD, zeros(fq.fq_workspace_bytes(d, fq.FQ_MODE_FORWARD)), stream)
            pb = None
            if train:
                pb = fq.fq_plan_create(d, fq.FQ_MODE_BACKWARD, zeros(fq.fq_workspace_bytes(d, fq.FQ_MODE_BACKWARD)),
                                       stream)
            plans.append((pf, pb))

        def forward(k):
            fq.fq_plan_run(plans[k][0], stream)

        def backward(k):
            fq.fq_plan_run(plans[k][1], stream)
    else:
        ws = zeros(fq.fq_workspace_bytes(sets[0], fq.FQ_MODE_BACKWARD)) if train else None

        def forward(k):
            fq.fq_forward(sets[k], stream)

        def backward(k):
            fq.fq_backward(sets[k], ws, stream)

    def launches_of_step(i):
        k = i % ring
        return [(forward, k), (backward, k)] if train else [(forward, k)]

    # ---- kernel timing inside the timed region --------------------------------------------------
    # Raw HIP events on the launch stream.  A pair of event records costs the queue about as much
    # as a small kernel, so (a) only every EVENT_EVERY-th step carries a pair and (b) the timed
    # kernel's duration is a difference that cancels the pair's own cost: brackets of kind A span
    # two consecutive launches, brackets of kind B only the first of them, and
    # t(second launch) = mean(A) - mean(B).  In a training step the second launch is the backward
    # kernel; in the codes pass it is the next step's forward kernel.
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def new_event():
        e = ctypes.c_void_p()
        if hip.hipEventCreate(ctypes.byref(e)) != 0:
            sys.exit("bench.py: hipEventCreate failed")
        return e

    timed = []
    for i in range(args.steps):
        timed.extend(launches_of_step(args.warmup + i))
    per_step = len(timed) // args.steps
    record_before = {}                      # launch index -> events to record just before it
    brackets = []
    if not args.no_kernel_events:
        every = min(EVENT_EVERY, max(2, args.steps // 4))        # short runs still get both kinds
        for n, i in enumerate(range(every - 1, args.steps, every)):
            first = i * per_step
            span = 2 if n % 2 == 0 else 1
            if first + span > len(timed):
                break
            a, z = new_event(), new_event()
            record_before.setdefault(first, []).append(a)
            record_before.setdefault(first + span, []).append(z)
            brackets.append((a, z, span))

    for i in range(args.warmup):
        for fn, k in launches_of_step(i):
            fn(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for idx, (fn, k) in enumerate(timed):
        for e in record_before.get(idx, ()):
            hip.hipEventRecord(e, sp)
        fn(k)
    for e in record_before.get(len(timed), ()):
        hip.hipEventRecord(e, sp)
    t_enq = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    for i in range(args.copy_calibration):
        x, y = first_bufs[i % ring]
        y.copy_(x)
    torch.cuda.synchronize()

    sec_per_step = (t1 - t0) / args.steps
    step_bytes = 5 * io_bytes if train else fwd_bytes
    value = step_bytes / sec_per_step / 1e9

    roofline = None
    if brackets:
        dur = {1: [], 2: []}
        for a, z, span in brackets:
            ms = ctypes.c_float()
            if hip.hipEventElapsedTime(ctypes.byref(ms), a, z) != 0:
                sys.exit("bench.py: hipEventElapsedTime failed")
            dur[span].append(ms.value * 1e-3)
            hip.hipEventDestroy(a)
            hip.hipEventDestroy(z)
        if dur[1] and dur[2]:
            t_two, t_one = float(np.mean(dur[2])), float(np.mean(dur[1]))
            t_kernel = t_two - t_one
            kernel_bytes = 3 * io_bytes if train else fwd_bytes
            achieved = kernel_bytes / t_kernel / 1e9
            dt = "f16" if cases[0].itemsize == 2 else "f32"
            if train:
                kname = "backward_multi_kernel<fused>" if multi else "backward_kernel<%s, fused>" % dt
            elif codes:
                kname = "forward_multi_kernel<codes>" if multi else "forward_kernel<%s, codes>" % dt
            else:
                kname = "forward_multi_kernel" if multi else "forward_kernel<%s>" % dt
            headline = args.workload == "feature_fp16_per_channel"
            traffic = None
            if args.cache_warm:
                pass                                   # the counters were taken on the HBM-cold ring
            elif headline and train:
                traffic = TRAFFIC_BYTES_PER_LAUNCH
            elif headline and not codes:
                traffic = FORWARD_TRAFFIC_BYTES_PER_LAUNCH
            roofline = {"bound": "hbm", "kernel": kname, "achieved": round(achieved, 1),
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                        "traffic": traffic,
                        "bytes_per_launch": kernel_bytes, "avg_us": round(t_kernel * 1e6, 2),
                        "method": "HIP events on the launch stream in the timed region: mean(bracket of two "
                                  "launches) - mean(bracket of the first); cancels the event pair's own cost",
                        "bracket_two_us": round(t_two * 1e6, 2), "bracket_one_us": round(t_one * 1e6, 2),
                        "samples": [len(dur[2]), len(dur[1])]}

    # ---- context: what plain library streaming kernels reach on the same buffers ---------------
    # (outside the timed region; single-tensor training workloads only).  torch's device copy moves
    # the forward's bytes (read b, write b per element), torch.add the backward's (read 2b, write
    # b): neither does any of the quantizer's arithmetic, so their time per launch is the
    # streaming floor of this machine for that traffic, launched back to back over the same ring.
    floors = None
    if train and not multi and not args.no_kernel_events:
        def train_of(fn, reps=10 * ring):
            a, z = new_event(), new_event()
            for i in range(ring):
                fn(i)
            torch.cuda.synchronize()
            hip.hipEventRecord(a, sp)
            for i in range(reps):
                fn(i % ring)
            hip.hipEventRecord(z, sp)
            torch.cuda.synchronize()
            ms = ctypes.c_float()
            hip.hipEventElapsedTime(ctypes.byref(ms), a, z)
            return ms.value / reps * 1e3

        per_set = len(cases)
        t_copy = train_of(lambda k: keep[k * per_set][1].copy_(keep[k * per_set][0]))
        t_add = train_of(lambda k: torch.add(keep[k * per_set][0], keep[k * per_set][2], out=keep[k * per_set][3]))
        t_fwd = train_of(forward)
        t_bwd = train_of(backward)
        floors = {"note": "us per launch, back-to-back launches over the same cold ring, one event pair "
                          "around the whole train",
                  "torch_copy_us": round(t_copy, 2), "fq_forward_us": round(t_fwd, 2),
                  "torch_add_us": round(t_add, 2), "fq_backward_us": round(t_bwd, 2)}

    cpu = None
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
        reps, times = 3, []
        rep = 0
        while rep < reps:
            rep += 1
            c0 = time.perf_counter()
            for cs in sample:
                s_, active = fq_oracle.scale(cs.theta, cs.eps, cs.s_min, cs.s_max)
                fq_oracle.forward(cs.x, s_, cs.qmin, cs.qmax, cs.outer, cs.channels, cs.inner, want_q=codes)
                if train:
                    fq_oracle.backward(cs.x, cs.gy, s_, cs.theta, active, cs.qmin, cs.qmax,
                                       cs.outer, cs.channels, cs.inner)
            times.append(time.perf_counter() - c0)
            if rep == 1:                      # aim at about 5 s of CPU work, 3 to 15 repetitions
                reps = int(min(15, max(3, round(5.0 / max(times[0], 1e-3)))))
        med = sorted(times)[len(times) // 2]
        cpu = {"value": round(sample_bytes / med / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": "%d of %d tensors of the workload (%d elements, %s), median of %d runs, "
                         "%.2f s each" % (len(sample), len(cases), n_sample,
                                          "fwd+bwd" if train else ("forward with codes" if codes else "forward"), reps, med),
               "elements_per_s": round(n_sample / med, 1)}

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
                   "tensors": len(cases), "launches_per_step": per_step, "elements": numel,
                   "bytes_per_step": step_bytes, "ring_buffer_sets": int(ring),
                   "ring_bytes": int(ring * set_bytes),
                   "residency": "cache-warm: the same buffers every step" if args.cache_warm else
                                "HBM-cold: steps rotate over the ring" if ring > 1 else
                                "one buffer set larger than the caches"},
        "elements_per_s": round(numel / sec_per_step, 1),
        "host_enqueue_us_per_step": round((t_enq - t0) / args.steps * 1e6, 2),
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "streaming_context": floors,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
