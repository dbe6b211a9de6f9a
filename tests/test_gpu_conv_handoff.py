"""One quantized convolution layer the way the front end runs it (Sec. 3.2-3.3): fake-quantize the
activation (per-tensor scale) and the frozen weight (per-output-channel scales), hand both to the
platform library's float convolution, and on the way back take the convolution's gradients as the
upstream gradients of the two STE backward passes.  The convolution itself is the library's on both
sides (MIOpen through torch on the GPU, torch's CPU routine in binary64 beside the oracle); what is
checked is that the library's outputs feed it and its gradients feed the library, end to end."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from paper_2511_12653_amd import workloads
from paper_2511_12653_amd.autograd import fake_quantize

import _gpu_harness as H

pytestmark = pytest.mark.gpu


def test_quantized_conv_layer_forward_and_backward(oracle):
    rng = np.random.Generator(np.random.Philox(41))
    n, cin, cout, h, w = 2, 16, 24, 30, 40
    x = rng.standard_normal((n, cin, h, w)).astype(np.float32)
    wt = (rng.standard_normal((cout, cin, 3, 3)) * np.sqrt(2.0 / (cin * 9))).astype(np.float32)
    gout = rng.standard_normal((n, cout, h, w)).astype(np.float32)
    theta_a = workloads.theta_for_scale(np.array([np.abs(x).max() / 127.0 * 0.7]))      # some clipping
    theta_w = workloads.theta_for_scale(np.abs(wt).reshape(cout, -1).max(axis=1) / 127.0)
    H.say("conv hand-off: x %s, w %s" % (x.shape, wt.shape))

    xd = torch.from_numpy(x).cuda().requires_grad_(True)
    wd = torch.from_numpy(wt).cuda()                              # frozen: only its scales train
    ta = torch.from_numpy(theta_a).cuda().requires_grad_(True)
    tw = torch.from_numpy(theta_w).cuda().requires_grad_(True)
    xq = fake_quantize(xd, ta, -128, 127, channel_dim=None)
    wq = fake_quantize(wd, tw, -127, 127, channel_dim=0)
    y = F.conv2d(xq, wq, padding=1)
    y.backward(torch.from_numpy(gout).cuda())
    torch.cuda.synchronize()
    assert wd.grad is None

    # the same layer beside the oracle: its fake quantization, the CPU convolution in binary64
    sa, act_a = oracle.scale(theta_a)
    sw, act_w = oracle.scale(theta_w)
    rxq, _ = oracle.forward(x, sa, -128, 127, 1, 1, x.size, want_q=False)
    rwq, _ = oracle.forward(wt, sw, -127, 127, 1, cout, cin * 9, want_q=False)
    assert np.array_equal(xq.detach().cpu().numpy().view(np.uint32), rxq.reshape(x.shape).view(np.uint32))
    assert np.array_equal(wq.detach().cpu().numpy().view(np.uint32), rwq.reshape(wt.shape).view(np.uint32))
    cx = torch.from_numpy(rxq.reshape(x.shape).astype(np.float64)).requires_grad_(True)
    cw = torch.from_numpy(rwq.reshape(wt.shape).astype(np.float64)).requires_grad_(True)
    cy = F.conv2d(cx, cw, padding=1)
    cy.backward(torch.from_numpy(gout.astype(np.float64)))
    np.testing.assert_allclose(y.detach().cpu().numpy(), cy.detach().numpy(), rtol=1e-4, atol=1e-4)

    g_xq = cx.grad.numpy().astype(np.float32)                     # upstream of the activation's backward
    g_wq = cw.grad.numpy().astype(np.float32)
    ra = oracle.backward(x, g_xq, sa, theta_a, act_a, -128, 127, 1, 1, x.size)
    rw = oracle.backward(wt, g_wq, sw, theta_w, act_w, -127, 127, 1, cout, cin * 9)
    # gx is a masked copy of the convolution's input gradient: same mask, values to conv accuracy
    got_gx = xd.grad.cpu().numpy()
    ref_gx = ra["gx"].reshape(x.shape)
    assert np.array_equal(got_gx == 0.0, ref_gx == 0.0) and (ref_gx == 0.0).mean() > 0.001
    np.testing.assert_allclose(got_gx, ref_gx, rtol=1e-4, atol=1e-4)
    # scale gradients: sums of gy*t with cancellation; the upstream gradients differ at conv
    # accuracy (1e-6 relative per element), so compare against the sum of magnitudes
    for name, got, r in (("theta_a", ta.grad, ra), ("theta_w", tw.grad, rw)):
        g = got.cpu().numpy().reshape(-1).astype(np.float64)
        bound = 1e-5 * r["aabs"] + 1e-5 * np.abs(r["gtheta"])
        assert np.all(np.abs(g - r["gtheta"].astype(np.float64)) <= bound), (name, g, r["gtheta"])
        assert np.abs(g).max() > 0.0
