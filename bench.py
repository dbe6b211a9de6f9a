#!/usr/bin/env python3
"""Throughput of the fused fake-quantization hot path on one MI355X.

One step = fq_forward + fq_backward (Eq. (3)-(5) and the STE backward with the per-channel
scale-gradient reduction) over the headline tensor: FP16 1x384x120x160, 384 learnable scales,
signed 8-bit codes.  Inputs are synthetic (seeded, DPVO-feature-map shaped) and resident in HBM
before the timed region.  Successive steps rotate over a ring of distinct buffer sets larger than
the 256 MB Infinity Cache, so every step streams from HBM rather than from cache.

Prints one JSON line: whole-job GB/s (algorithmic bytes: forward 2b + backward 3b per element),
the roofline position of the dominant kernel (the backward kernel, 3b bytes per element, timed
in every step of the timed region by HIP events that ride on the kernel's own dispatch) and the
CPU oracle timed on this host beside it.
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
# HBM bytes per backward launch from rocprofv3 FETCH_SIZE / WRITE_SIZE counters (see profiles/);
# None until counters have been taken for the current kernel.
TRAFFIC_BYTES_PER_LAUNCH = None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="N",
                    help="after the timed region also run N plain device copies of the 14745600-byte "
                         "x tensor (torch copy_), so that a rocprofv3 --pmc run of this command holds a "
                         "copy kernel of known size to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="do not attach timing events to the backward kernel (roofline becomes null)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (got --gpus %d); "
                 "the path shards by tensor / channel range, see DESIGN.md" % args.gpus)

    import numpy as np
    import torch
    from paper_2511_12653_amd import binding as fq
    from paper_2511_12653_amd import workloads

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; there is no CPU fallback")
    torch.cuda.set_device(0)

    case = workloads.make("feature_fp16_per_channel")[0]
    numel, b = case.numel, case.itemsize
    set_bytes = 4 * numel * b
    ring = max(2, RING_BYTES // set_bytes)

    hx = torch.from_numpy(case.x.reshape(-1))
    hg = torch.from_numpy(case.gy.reshape(-1))
    theta = torch.from_numpy(case.theta).cuda()
    c = case.channels
    gs = torch.empty(c, device="cuda")
    gtheta = torch.empty(c, device="cuda")
    descs, keep = [], []
    for _ in range(ring):
        x, gy = hx.cuda(), hg.cuda()
        y, gx = torch.empty_like(x), torch.empty_like(x)
        keep.append((x, gy, y, gx))
        descs.append(fq.FqTensor.from_torch(case.outer, c, case.inner, case.qmin, case.qmax,
                                            x=x, y=y, theta=theta, gy=gy, gx=gx, gs=gs, gtheta=gtheta))
    ws = torch.zeros(fq.fq_workspace_bytes(descs[0], fq.FQ_MODE_BACKWARD) // 4, dtype=torch.int32,
                     device="cuda")
    stream = torch.cuda.current_stream()

    # Kernel timing inside the timed region, with raw HIP events on the launch stream.  A pair of
    # event records costs the queue about as much as a small kernel, so (a) only every
    # EVENT_EVERY-th step carries a pair, and (b) the backward kernel's duration is taken as a
    # difference that cancels the pair's own overhead: steps of kind A bracket forward+backward,
    # steps of kind B bracket the forward alone, and  t(backward) = mean(A) - mean(B).
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
    sp = stream.cuda_stream

    def new_event():
        e = ctypes.c_void_p()
        if hip.hipEventCreate(ctypes.byref(e)) != 0:
            sys.exit("bench.py: hipEventCreate failed")
        return e

    def step(i, ev=None, kind=None):
        d = descs[i % ring]
        if ev is not None:
            hip.hipEventRecord(ev[0], sp)
        fq.fq_forward(d, stream)
        if kind == "fwd":
            hip.hipEventRecord(ev[1], sp)
        fq.fq_backward(d, ws, stream)
        if kind == "fwd+bwd":
            hip.hipEventRecord(ev[1], sp)

    for i in range(args.warmup):
        step(i)
    events = {}
    if not args.no_kernel_events:
        for n, i in enumerate(range(EVENT_EVERY - 1, args.steps, EVENT_EVERY)):
            events[i] = ((new_event(), new_event()), "fwd+bwd" if n % 2 == 0 else "fwd")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i in events:
            step(args.warmup + i, *events[i])
        else:
            step(args.warmup + i)
    t_enq = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    for i in range(args.copy_calibration):
        x, _, y, _ = keep[i % ring]
        y.copy_(x)
    torch.cuda.synchronize()

    sec_per_step = (t1 - t0) / args.steps
    step_bytes = 5 * b * numel
    value = step_bytes / sec_per_step / 1e9

    roofline = None
    if events:
        dur = {"fwd+bwd": [], "fwd": []}
        for (a, z), kind in events.values():
            ms = ctypes.c_float()
            if hip.hipEventElapsedTime(ctypes.byref(ms), a, z) != 0:
                sys.exit("bench.py: hipEventElapsedTime failed")
            dur[kind].append(ms.value * 1e-3)
            hip.hipEventDestroy(a)
            hip.hipEventDestroy(z)
        if dur["fwd"] and dur["fwd+bwd"]:
            t_both, t_fwd = float(np.mean(dur["fwd+bwd"])), float(np.mean(dur["fwd"]))
            t_bwd = t_both - t_fwd
            bwd_bytes = 3 * b * numel
            achieved = bwd_bytes / t_bwd / 1e9
            roofline = {"bound": "hbm", "kernel": "backward_kernel<f16, fused>", "achieved": round(achieved, 1),
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                        "traffic": TRAFFIC_BYTES_PER_LAUNCH, "bytes_per_launch": bwd_bytes,
                        "avg_us": round(t_bwd * 1e6, 2),
                        "method": "HIP events on the launch stream in the timed region: mean(bracket "
                                  "fwd+bwd) - mean(bracket fwd); cancels the event pair's own cost",
                        "bracket_fwd_bwd_us": round(t_both * 1e6, 2), "bracket_fwd_us": round(t_fwd * 1e6, 2),
                        "samples": [len(dur["fwd+bwd"]), len(dur["fwd"])]}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import fq_oracle
        fq_oracle.lib()
        reps, times = 3, []
        for _ in range(reps):
            c0 = time.perf_counter()
            s, active = fq_oracle.scale(case.theta)
            fq_oracle.forward(case.x, s, case.qmin, case.qmax, case.outer, c, case.inner, want_q=False)
            fq_oracle.backward(case.x, case.gy, s, case.theta, active, case.qmin, case.qmax,
                               case.outer, c, case.inner)
            times.append(time.perf_counter() - c0)
        med = sorted(times)[len(times) // 2]
        cpu = {"value": round(step_bytes / med / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": "the whole workload tensor (7372800 elements, fwd+bwd), median of %d runs, "
                         "%.2f s each" % (reps, med),
               "elements_per_s": round(numel / med, 1)}

    out = {
        "metric": "fake-quant fwd+bwd GB/s", "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "feature_fp16_per_channel: FP16 1x384x120x160 NCHW, 384 per-channel "
                               "scales, codes -128..127, forward + STE backward",
                   "io_dtype": "f16", "elements": numel, "bytes_per_step": step_bytes,
                   "ring_buffer_sets": int(ring), "ring_bytes": int(ring * set_bytes)},
        "elements_per_s": round(numel / sec_per_step, 1),
        "host_enqueue_us_per_step": round((t_enq - t0) / args.steps * 1e6, 2),
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
