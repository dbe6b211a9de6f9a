"""fq_backward_static (the backward whose partial sums and slots live in the library's built-in
scratch array, for callers that cannot allocate) against fq_backward with a caller's workspace:
same bits in gx, gs, gtheta and s, on calls in a row that share the one array -- a large tensor
first (tickets in two levels), then smaller ones with other protocols (exchange, exchange tree,
one unit per channel, two launches), then the large one again."""
import numpy as np
import pytest
import torch

from paper_2511_12653_amd import workloads
from paper_2511_12653_amd import binding as fq

import _gpu_harness as H

pytestmark = pytest.mark.gpu


def _case(dtype, outer, channels, inner, seed):
    rng = np.random.Generator(np.random.Philox(seed))
    x = (rng.standard_normal((outer, channels, inner)) * 2).astype(dtype)
    gy = rng.standard_normal(x.shape).astype(dtype)
    theta = workloads.theta_for_scale(rng.uniform(0.02, 0.05, channels))
    return workloads.TensorCase("static", x.shape, outer, channels, inner, -128, 127, x, theta, gy)


def _both(case, label, flags=0):
    """Run fq_backward (own workspace) and fq_backward_static on the same inputs; compare bits."""
    H.say("no-alloc: %s %s, flags %d" % (label, "x".join(map(str, case.shape)), flags))
    ref = H.DeviceCase(case, want_q=False, flags=flags)
    got = H.DeviceCase(case, want_q=False, flags=flags)
    info = fq.fq_layout(ref.desc)
    ws = H.workspace_for(ref.desc, fq.FQ_MODE_BACKWARD)
    fq.fq_backward(ref.desc, ws)
    fq.fq_backward_static(got.desc)
    torch.cuda.synchronize()
    got.check_guards(label)
    for name in ("gx", "gs", "gtheta", "s"):
        a, b = ref.host(name), got.host(name)
        if a is None:                          # no gx with FQ_FLAG_NO_DX
            continue
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), "%s: %s differs" % (label, name)
    assert not np.isnan(got.host("gs")).any()
    return ref, info


def test_static_backward_equals_workspace_backward_on_calls_in_a_row():
    big = _case(np.float16, 9, 96, 19200, 41)          # 18 units per channel: two-level tickets
    ref, info = _both(big, "first, large")
    assert info.units_per_channel == 18 and info.extra_slots == 16
    s, active, _, _ = H.oracle_forward(big)
    H.check_backward(ref, s, active, "no-alloc/oracle")          # and both equal the oracle
    small = _case(np.float16, 1, 384, 19200, 42)       # 2 units per channel: exchange
    _, info = _both(small, "second, smaller")
    assert info.units_per_channel == 2
    _, info = _both(_case(np.float32, 1, 384, 28800, 43), "tickets on one slot")
    assert info.units_per_channel == 6 and info.extra_slots == 0
    _, info = _both(_case(np.float16, 1, 384, 28800, 44), "exchange tree")
    assert info.units_per_channel == 3 and info.extra_slots == 2
    _, info = _both(_case(np.float16, 1, 128, 30 * 40, 45), "one unit per channel")
    assert info.units_per_channel == 1
    _both(small, "two launches", flags=fq.FQ_FLAG_TWO_PASS)
    _both(small, "no gx", flags=fq.FQ_FLAG_NO_DX)
    _both(big, "large again")


def test_static_backward_refuses_a_tensor_beyond_its_scratch():
    # validation only: nothing is enqueued, the fake addresses are never touched
    d = fq.FqTensor(outer=1, channels=1, inner=98305 * 10240, dtype=fq.FQ_F16, qmin=-128, qmax=127, eps=0.0,
                    s_min=fq.FLT_MIN, s_max=float("inf"), flags=0, x=1 << 40, y=None, q=None, theta=0x30000,
                    s=None, gy=2 << 40, gx=3 << 40, gs=None, gtheta=0x60000)
    with pytest.raises(fq.FqError):
        fq.fq_backward_static(d)
