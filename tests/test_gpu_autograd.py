"""The torch.autograd wrapper is marshalling only: its results are those of fq_forward / fq_backward,
checked here against the oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from paper_2511_12653_amd import workloads
from paper_2511_12653_amd.autograd import fake_quantize

import _gpu_harness as H

pytestmark = pytest.mark.gpu


def _check(oracle, x, theta, gy, qmin, qmax, channel_dim, view, x_requires_grad=True):
    outer, c, inner = view
    xd = torch.from_numpy(x).cuda().requires_grad_(x_requires_grad)
    td = torch.from_numpy(theta).cuda().requires_grad_(True)
    y = fake_quantize(xd, td, qmin, qmax, channel_dim=channel_dim)
    y.backward(torch.from_numpy(gy).cuda())
    torch.cuda.synchronize()
    s, active = oracle.scale(theta)
    ry, _ = oracle.forward(x, s, qmin, qmax, outer, c, inner, want_q=False)
    rb = oracle.backward(x, gy, s, theta, active, qmin, qmax, outer, c, inner)
    assert y.shape == xd.shape and H.ulp_distance(y.detach().cpu().numpy(), ry.reshape(x.shape)).max() == 0
    if x_requires_grad:
        got = xd.grad.cpu().numpy()
        assert np.array_equal(got.view(np.uint16 if x.dtype == np.float16 else np.uint32),
                              rb["gx"].reshape(x.shape).view(np.uint16 if x.dtype == np.float16 else np.uint32))
    else:
        assert xd.grad is None
    gt = td.grad.cpu().numpy().reshape(-1).astype(np.float64)
    ref = rb["gtheta"].astype(np.float64)
    assert td.grad.shape == td.shape
    assert np.all(np.abs(gt - ref) <= 1e-5 * np.maximum(np.abs(ref), 1e-30)), (gt, ref)


def test_per_channel_activation_fp16(oracle):
    case = workloads.feature_fp16_per_channel(shape=(2, 12, 30, 40))[0]
    H.say("autograd: FP16 activation (2, 12, 30, 40), scales along dim 1")
    x = case.x.reshape(2, 12, 30, 40)
    _check(oracle, x, case.theta, case.gy.reshape(x.shape), -128, 127, 1, (2, 12, 1200))


def test_per_tensor_fp32(oracle):
    rng = np.random.Generator(np.random.Philox(5))
    x = (rng.standard_normal((3, 5, 17)) * 40).astype(np.float32)
    gy = rng.standard_normal(x.shape).astype(np.float32)
    H.say("autograd: FP32 per-tensor")
    _check(oracle, x, np.array([0.5], np.float32), gy, -127, 127, None, (1, 1, x.size))


@pytest.mark.parametrize("frozen", [False, True])
def test_conv_weight_scales_along_dim0(oracle, frozen):
    rng = np.random.Generator(np.random.Philox(6))
    w = (rng.standard_normal((16, 8, 3, 3)) * 0.05).astype(np.float32)
    gy = (rng.standard_normal(w.shape) * 0.1).astype(np.float32)
    theta = workloads.theta_for_scale(np.abs(w).reshape(16, -1).max(axis=1) / 127.0)
    H.say("autograd: conv weight (16, 8, 3, 3), frozen=%s" % frozen)
    _check(oracle, w, theta, gy, -127, 127, 0, (1, 16, 72), x_requires_grad=not frozen)


def test_non_contiguous_input_and_cpu_tensors(oracle):
    rng = np.random.Generator(np.random.Philox(7))
    base = (rng.standard_normal((6, 4, 10))).astype(np.float32)
    theta = np.full(4, -2.0, np.float32)
    xd = torch.from_numpy(base).cuda().transpose(0, 2)        # (10, 4, 6), not contiguous
    y = fake_quantize(xd, torch.from_numpy(theta).cuda(), -8, 7, channel_dim=1)
    xc = np.ascontiguousarray(base.transpose(2, 1, 0))
    s, _ = oracle.scale(theta)
    ry, _ = oracle.forward(xc, s, -8, 7, 10, 4, 6, want_q=False)
    assert H.ulp_distance(y.cpu().numpy(), ry.reshape(xc.shape)).max() == 0
    with pytest.raises(RuntimeError):
        fake_quantize(torch.zeros(4), torch.zeros(1))
