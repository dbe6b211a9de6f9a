"""Scale-only training end to end (Sec. 3.2): forward, a distillation-style loss against the
unquantized tensor, STE backward with the fused Adam step, repeated.  The teacher is x itself and
the loss is mean((FQ(x) - x)^2), so learning the scales must reduce the quantization error; the
same loop run with the CPU oracle must follow the same trajectory."""
import numpy as np
import pytest
import torch

from paper_2511_12653_amd import workloads
from paper_2511_12653_amd import binding as fq
from oracle import fq_oracle

import _gpu_harness as H

pytestmark = pytest.mark.gpu

HYPER = dict(lr=2e-2, beta1=0.9, beta2=0.999, eps=1e-8)


def test_scale_only_training_reduces_quantization_error():
    rng = np.random.default_rng(12)
    outer, c, inner, steps = 2, 6, 4096, 40
    sigma = rng.uniform(0.3, 2.0, c).astype(np.float32)
    x = (rng.standard_normal((outer, c, inner)).astype(np.float32) * sigma[None, :, None])
    # start far from the optimum: scales 4x too small for half the channels (heavy clipping),
    # 4x too large for the others (coarse steps)
    s0 = sigma * 4.0 / 127.0 * np.where(np.arange(c) % 2 == 0, 0.25, 4.0)
    theta0 = workloads.theta_for_scale(s0)
    n = x.size
    H.say("training loop: %d steps, %d channels" % (steps, c))

    # ---- GPU loop: the loss gradient is plain torch, everything else goes through the C ABI
    xd = H.dev(x.reshape(-1))
    y, gy, gx = torch.empty_like(xd), torch.empty_like(xd), torch.empty_like(xd)
    theta, m, v = H.dev(theta0), torch.zeros(c, device="cuda"), torch.zeros(c, device="cuda")
    gs, gt = torch.empty(c, device="cuda"), torch.empty(c, device="cuda")
    d = fq.FqTensor.from_torch(outer, c, inner, -128, 127, x=xd, y=y, theta=theta, gy=gy, gx=gx, gs=gs, gtheta=gt)
    ws = H.workspace_for(d, fq.FQ_MODE_BACKWARD)
    gpu_loss, gpu_theta = [], []
    for step in range(1, steps + 1):
        fq.fq_forward(d)
        diff = y - xd
        gpu_loss.append(float((diff.double() ** 2).mean().item()))
        torch.mul(diff, 2.0 / n, out=gy)
        d.set_adam(fq.FqAdam.from_torch(m, v, theta, step=step, **HYPER))      # in place
        fq.fq_backward(d, ws)
        torch.cuda.synchronize()
        gpu_theta.append(theta.cpu().numpy().copy())

    # ---- the same loop with the oracle
    th, mo, vo = theta0.copy(), np.zeros(c, np.float32), np.zeros(c, np.float32)
    ref_loss, ref_theta = [], []
    for step in range(1, steps + 1):
        s, active = fq_oracle.scale(th)
        yo, _ = fq_oracle.forward(x, s, -128, 127, outer, c, inner, want_q=False)
        diff = yo - x
        ref_loss.append(float((diff.astype(np.float64) ** 2).mean()))
        gyo = (diff * np.float32(2.0 / n)).astype(np.float32)
        r = fq_oracle.backward(x, gyo, s, th, active, -128, 127, outer, c, inner)
        th, mo, vo = fq_oracle.adam(r["gtheta"], mo, vo, th, step=step, **HYPER)
        ref_theta.append(th.copy())

    assert gpu_loss[-1] < 0.2 * gpu_loss[0], (gpu_loss[0], gpu_loss[-1])
    assert ref_loss[-1] < 0.2 * ref_loss[0]
    np.testing.assert_allclose(gpu_loss, ref_loss, rtol=1e-4)
    np.testing.assert_allclose(np.array(gpu_theta), np.array(ref_theta), rtol=1e-4, atol=1e-5)
    # the learned scales moved toward each other: clipped channels grew, coarse channels shrank
    s_end, _ = fq_oracle.scale(gpu_theta[-1])
    assert np.all(s_end[0::2] > s0[0::2]) and np.all(s_end[1::2] < s0[1::2])
