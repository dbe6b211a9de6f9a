"""The launching calls enqueue kernels only, so they can be captured in a HIP graph and replayed."""
import numpy as np
import pytest
import torch

from paper_2511_12653_amd import workloads
from paper_2511_12653_amd import binding as fq

import _gpu_harness as H

pytestmark = pytest.mark.gpu


def _snapshot(dcs):
    return [[getattr(d, k).clone() for k in ("y", "gx", "gs", "gtheta")] for d in dcs]


def _poison(dcs):
    for d in dcs:
        d.y.zero_()
        d.gx.zero_()
        d.gs.fill_(float("nan"))
        d.gtheta.fill_(float("nan"))


def _same(a, b):
    return all(torch.equal(x.view(torch.uint8), y.view(torch.uint8)) for p, q in zip(a, b) for x, y in zip(p, q))


def test_single_tensor_calls_in_a_graph():
    case = workloads.feature_fp16_per_channel(shape=(2, 12, 60, 80))[0]
    H.say("graph capture: fq_forward + fq_backward, 5 replays with eager work in between")
    dc = H.DeviceCase(case, want_q=False)
    ws = H.workspace_for(dc.desc, fq.FQ_MODE_BACKWARD)
    fq.fq_forward(dc.desc)
    fq.fq_backward(dc.desc, ws)
    torch.cuda.synchronize()
    eager = _snapshot([dc])
    ref = H.oracle_forward(case)
    H.check_forward(dc, ref, "graph/eager fwd")
    H.check_backward(dc, ref[0], ref[1], "graph/eager bwd")

    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            fq.fq_forward(dc.desc)                   # stream=None: the capturing stream
            fq.fq_backward(dc.desc, ws)
    torch.cuda.synchronize()
    scratch = torch.zeros(1 << 20, device="cuda")
    for rep in range(5):
        _poison([dc])
        scratch.add_(1.0)                            # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert _same(_snapshot([dc]), eager), "replay %d differs from the eager result" % rep


def test_plan_run_in_a_graph():
    cases = workloads.multi_tensor_mixed(n_act=4, n_wgt=3, target_bytes=6 << 20, max_batch=2)
    H.say("graph capture: fq_plan_run forward + backward over %d tensors" % len(cases))
    dcs = [H.DeviceCase(c, want_q=False) for c in cases]
    arr = fq.fq_tensor_array([d.desc for d in dcs])
    ws_f = H.workspace_for(arr, fq.FQ_MODE_FORWARD)
    ws_b = H.workspace_for(arr, fq.FQ_MODE_BACKWARD)
    plan_f = fq.fq_plan_create(arr, fq.FQ_MODE_FORWARD, ws_f)
    plan_b = fq.fq_plan_create(arr, fq.FQ_MODE_BACKWARD, ws_b)
    try:
        fq.fq_plan_run(plan_f)
        fq.fq_plan_run(plan_b)
        torch.cuda.synchronize()
        eager = _snapshot(dcs)
        for i, (c, d) in enumerate(zip(cases, dcs)):
            ref = H.oracle_forward(c)
            H.check_forward(d, ref, "graph/plan[%d] fwd" % i)
            H.check_backward(d, ref[0], ref[1], "graph/plan[%d] bwd" % i)
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                fq.fq_plan_run(plan_f)
                fq.fq_plan_run(plan_b)
        torch.cuda.synchronize()
        for rep in range(4):
            _poison(dcs)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert _same(_snapshot(dcs), eager), "replay %d differs from the eager result" % rep
    finally:
        fq.fq_plan_destroy(plan_f)
        fq.fq_plan_destroy(plan_b)


def test_distillation_step_in_a_graph():
    """forward -> distillation loss and gradient -> backward, captured once and replayed with new
    data at the same addresses; every replay equals the eager chain bit for bit."""
    rng = np.random.Generator(np.random.Philox(31))
    n, c, m = 2, 20, 1536
    H.say("graph capture: fq_forward + fq_distill_loss + fq_backward, shape (%d, %d, %d)" % (n, c, m))
    x = torch.from_numpy((rng.standard_normal((n, c, m)) * 1.3).astype(np.float16)).cuda()
    teacher = torch.from_numpy((rng.standard_normal((n, c, m)) * 1.3).astype(np.float16)).cuda()
    theta = torch.from_numpy(workloads.theta_for_scale(rng.uniform(0.01, 0.05, c))).cuda()
    y, gy, gx = torch.empty_like(x), torch.empty_like(x), torch.empty_like(x)
    gs, gth = torch.empty(c, device="cuda"), torch.empty(c, device="cuda")
    out = torch.zeros(3, dtype=torch.float64, device="cuda")
    t = fq.FqTensor.from_torch(n, c, m, -127, 127, x=x, y=y, theta=theta, gy=gy, gx=gx, gs=gs, gtheta=gth)
    d = fq.FqDistill.from_torch(n, c, m, y, teacher, out, gy, lam=0.5, upstream=256.0)
    ws_b = H.workspace_for(t, fq.FQ_MODE_BACKWARD)
    ws_d = torch.empty(fq.fq_distill_workspace_bytes(d) // 8, dtype=torch.float64, device="cuda")

    def chain():
        fq.fq_forward(t)
        fq.fq_distill_loss(d, ws_d)
        fq.fq_backward(t, ws_b)

    def snapshot():
        return [v.clone() for v in (y, gy, gx, gs, gth, out)]

    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    chain()                                           # warm up outside the capture
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            chain()
    torch.cuda.synchronize()
    for rep in range(4):
        x.mul_(1.0 + 0.125 * rep)                     # new data, same addresses
        teacher.add_(0.01 * rep)
        torch.cuda.synchronize()
        chain()
        torch.cuda.synchronize()
        eager = snapshot()
        for v in (y, gy, gx):
            v.zero_()
        for v in (gs, gth, out):
            v.fill_(float("nan"))
        ws_d.fill_(float("nan"))                      # the distillation workspace carries no state
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(snapshot(), eager):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), "replay %d differs" % rep
    assert torch.isfinite(out).all() and float(out[0]) > 0.0
