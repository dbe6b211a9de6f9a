"""Fused Adam step on theta at the end of the backward pass, against the oracle's backward
followed by the oracle's Adam step.  Every step starts from the oracle's state (uploaded), so a
last-bit difference cannot carry over into the next step's quantizer."""
import numpy as np
import pytest
import torch

from paper_2511_12653_amd import workloads
from paper_2511_12653_amd import binding as fq
from oracle import fq_oracle

import _gpu_harness as H

pytestmark = pytest.mark.gpu

HYPER = dict(lr=3e-3, beta1=0.9, beta2=0.999, eps=1e-8)


def _close(got, ref, what):
    got, ref = got.astype(np.float64), ref.astype(np.float64)
    err = np.abs(got - ref)
    assert np.all(err <= 1e-6 * np.abs(ref) + 1e-12), "%s: max err %.3e" % (what, err.max())
    return float(np.mean(got == ref))


def _short_slab_case(outer):
    """4200 channels of 96 FP16 elements each: one wavefront per slab, `outer` units per channel."""
    rng = np.random.Generator(np.random.Philox(900 + outer))
    c, inner = 4200, 96
    x = (rng.standard_normal((outer, c, inner)) * 1.5).astype(np.float16)
    gy = rng.standard_normal(x.shape).astype(np.float16)
    theta = workloads.theta_for_scale(rng.uniform(0.02, 0.05, c))
    return workloads.TensorCase("short", x.shape, outer, c, inner, -128, 127, x, theta, gy)


@pytest.mark.parametrize("in_place", [True, False])
@pytest.mark.parametrize("flags", [0, fq.FQ_FLAG_TWO_PASS])
@pytest.mark.parametrize("shape", ["blocks", "waves1", "waves2", "waves6"])
def test_adam_steps_single_tensor(in_place, flags, shape):
    case = (workloads.train_batch_fp16(shape=(3, 10, 60, 80))[0] if shape == "blocks"
            else _short_slab_case(int(shape[5:])))
    H.say("adam single %s in_place=%s flags=%d" % (shape, in_place, flags))
    c = case.channels
    dc = H.DeviceCase(case, want_q=False, flags=flags)
    assert fq.fq_layout(dc.desc).wave_units == (0 if shape == "blocks" else 1)
    ws = H.workspace_for(dc.desc, fq.FQ_MODE_BACKWARD)
    m_d, v_d = torch.zeros(c, device="cuda"), torch.zeros(c, device="cuda")
    out_d = dc.theta if in_place else torch.full((c,), float("nan"), device="cuda")
    theta, m, v = case.theta.copy(), np.zeros(c, np.float32), np.zeros(c, np.float32)
    for step in range(1, 5):
        dc.theta.copy_(H.dev(theta)); m_d.copy_(H.dev(m)); v_d.copy_(H.dev(v))
        dc.desc.set_adam(fq.FqAdam.from_torch(m_d, v_d, out_d, step=step, **HYPER))
        fq.fq_backward(dc.desc, ws)
        torch.cuda.synchronize()
        s, active = fq_oracle.scale(theta)
        r = fq_oracle.backward(case.x, case.gy, s, theta, active, case.qmin, case.qmax,
                               case.outer, c, case.inner)
        th_ref, m_ref, v_ref = fq_oracle.adam(r["gtheta"], m, v, theta, step=step, **HYPER)
        exact = _close(out_d.cpu().numpy(), th_ref, "theta step %d" % step)
        _close(m_d.cpu().numpy(), m_ref, "m step %d" % step)
        _close(v_d.cpu().numpy(), v_ref, "v step %d" % step)
        assert exact >= 0.9, "theta should be bit-exact for nearly every channel (%.2f)" % exact
        if not in_place:
            assert np.array_equal(dc.theta.cpu().numpy(), theta)        # input untouched
        theta, m, v = th_ref, m_ref, v_ref
    assert not np.array_equal(theta, case.theta)


def test_adam_skips_non_finite_gradient_and_clamped_channels():
    rng = np.random.default_rng(8)
    c, inner = 4, 2000
    x = rng.standard_normal((1, c, inner)).astype(np.float32)
    x[0, 1, 5] = np.nan                                  # channel 1: NaN scale gradient
    gy = rng.standard_normal((1, c, inner)).astype(np.float32)
    theta = np.array([0.0, 0.0, -9.0, 0.3], np.float32)   # channel 2: below s_min, clamp active
    case = workloads.TensorCase("adamnan", x.shape, 1, c, inner, -128, 127, x, theta, gy, s_min=0.01)
    H.say("adam with a NaN channel and a clamped channel")
    dc = H.DeviceCase(case, want_q=False)
    ws = H.workspace_for(dc.desc, fq.FQ_MODE_BACKWARD)
    m0 = np.array([0.1, 0.2, 0.3, 0.4], np.float32)
    v0 = np.array([0.01, 0.02, 0.03, 0.04], np.float32)
    m_d, v_d, out_d = H.dev(m0), H.dev(v0), torch.full((c,), float("nan"), device="cuda")
    dc.desc.set_adam(fq.FqAdam.from_torch(m_d, v_d, out_d, step=7, **HYPER))
    fq.fq_backward(dc.desc, ws)
    torch.cuda.synchronize()
    s, active = fq_oracle.scale(theta, 0.0, 0.01)
    assert list(active) == [0, 0, 1, 0]
    r = fq_oracle.backward(x, gy, s, theta, active, -128, 127, 1, c, inner)
    assert np.isnan(r["gtheta"][1]) and r["gtheta"][2] == 0
    th_ref, m_ref, v_ref = fq_oracle.adam(r["gtheta"], m0, v0, theta, step=7, **HYPER)
    _close(out_d.cpu().numpy(), th_ref, "theta")
    _close(m_d.cpu().numpy(), m_ref, "m")
    _close(v_d.cpu().numpy(), v_ref, "v")
    assert out_d[1].item() == 0.0 and m_d[1].item() == np.float32(0.2)   # untouched
    assert out_d[2].item() != -9.0                                        # momentum still moves it


def test_adam_in_multi_tensor_calls_and_plans():
    """Three Adam steps over a list, once through fq_multi_tensor (descriptors rebuilt per step)
    and once through a plan replayed with fq_plan_run_adam: identical bits, and equal to the
    oracle after the first step."""
    cases = workloads.multi_tensor_mixed(n_act=4, n_wgt=3, target_bytes=6 << 20, max_batch=2)
    H.say("adam multi + plan: %d tensors" % len(cases))

    def fresh():
        dcs = [H.DeviceCase(cs, want_q=False) for cs in cases]
        state = [(torch.zeros(cs.channels, device="cuda"), torch.zeros(cs.channels, device="cuda")) for cs in cases]
        return dcs, state

    def attach(dcs, state, step):
        for d, (m_d, v_d) in zip(dcs, state):
            d.desc.set_adam(fq.FqAdam.from_torch(m_d, v_d, d.theta, step=step, **HYPER))     # in place
        return fq.fq_tensor_array([d.desc for d in dcs])

    # (a) fq_multi_tensor, descriptors rebuilt for each step
    dcs_a, st_a = fresh()
    ws_a = H.workspace_for(attach(dcs_a, st_a, 1), fq.FQ_MODE_BACKWARD)
    for step in (1, 2, 3):
        fq.fq_multi_tensor(attach(dcs_a, st_a, step), fq.FQ_MODE_BACKWARD, ws_a)
        torch.cuda.synchronize()
        if step == 1:
            for cs, d, (m_d, v_d) in zip(cases, dcs_a, st_a):
                s, active = fq_oracle.scale(cs.theta)
                r = fq_oracle.backward(cs.x, cs.gy, s, cs.theta, active, cs.qmin, cs.qmax, cs.outer,
                                       cs.channels, cs.inner)
                z = np.zeros(cs.channels, np.float32)
                th_ref, m_ref, v_ref = fq_oracle.adam(r["gtheta"], z, z, cs.theta, step=1, **HYPER)
                _close(d.theta.cpu().numpy(), th_ref, cs.name + " theta")
                _close(m_d.cpu().numpy(), m_ref, cs.name + " m")
                _close(v_d.cpu().numpy(), v_ref, cs.name + " v")

    # (b) one plan, replayed
    dcs_b, st_b = fresh()
    arr = attach(dcs_b, st_b, 1)
    ws_b = H.workspace_for(arr, fq.FQ_MODE_BACKWARD)
    plan = fq.fq_plan_create(arr, fq.FQ_MODE_BACKWARD, ws_b)
    try:
        for step in (1, 2, 3):
            fq.fq_plan_run_adam(plan, step)
        torch.cuda.synchronize()
    finally:
        fq.fq_plan_destroy(plan)
    for da, db, (ma, va), (mb, vb) in zip(dcs_a, dcs_b, st_a, st_b):
        for x, y in ((da.theta, db.theta), (ma, mb), (va, vb), (da.gx, db.gx), (da.gs, db.gs)):
            assert torch.equal(x.view(torch.uint8), y.view(torch.uint8))
