"""Repeat the backward pass many times on the same inputs and workspace: the cross-block
combination (atomic exchange for two blocks per channel, tickets for more) must hand every
channel's finisher the other blocks' sums of THIS launch -- a stale or missing sum would change
bits.  Outputs are poisoned before every launch and compared on the device."""
import numpy as np
import pytest
import torch

from paper_2511_12653_amd import workloads
from paper_2511_12653_amd import binding as fq

import _gpu_harness as H

pytestmark = pytest.mark.gpu


def _repeat(case, label, iters):
    H.say("%s: %d launches" % (label, iters))
    dc = H.DeviceCase(case, want_q=False)
    ws = H.workspace_for(dc.desc, fq.FQ_MODE_BACKWARD)
    fq.fq_backward(dc.desc, ws)
    torch.cuda.synchronize()
    ref = H.oracle_forward(case)
    H.check_backward(dc, ref[0], ref[1], label)
    want = [t.clone() for t in (dc.gs, dc.gtheta, dc.gx)]
    bad = torch.zeros((), dtype=torch.int64, device="cuda")
    for _ in range(iters):
        dc.gs.fill_(float("nan"))
        dc.gtheta.fill_(float("nan"))
        fq.fq_backward(dc.desc, ws)
        for got, w in zip((dc.gs, dc.gtheta), want[:2]):
            bad += (got.view(torch.int32) != w.view(torch.int32)).sum()
    torch.cuda.synchronize()
    assert int(bad.item()) == 0, "%s: %d mismatching words over %d launches" % (label, int(bad.item()), iters)
    assert torch.equal(dc.gx.view(torch.uint8), want[2].view(torch.uint8))


def test_two_blocks_per_channel_exchange():
    case = workloads.make("feature_fp16_per_channel")[0]            # 384 channels x 2 blocks
    _repeat(case, "stress/exchange", 300)


def test_many_blocks_per_channel_tickets():
    case = workloads.train_batch_fp16(shape=(6, 64, 120, 160))[0]   # 64 channels x 12 blocks
    _repeat(case, "stress/tickets", 200)


def test_one_channel_many_blocks():
    rng = np.random.default_rng(5)
    n = 3_000_000                                                   # one channel, 586 blocks
    x = (rng.standard_normal(n) * 2).astype(np.float32)
    gy = rng.standard_normal(n).astype(np.float32)
    case = workloads.TensorCase("one", (n,), 1, 1, n, -128, 127, x, workloads.theta_for_scale([0.03]), gy)
    _repeat(case, "stress/one_channel", 200)


@pytest.mark.parametrize("dtype, outer, channels, inner", [
    (np.float16, 32, 3, 19200),     # 2 blocks per slab: 64 per channel, the last count that shares one slot
    (np.float16, 33, 3, 19200),     # 66 per channel: two-level tickets, first-level slots see 3 or 2 arrivals
    (np.float32, 1, 1, 65 * 5120),  # one scale, well over a hundred blocks
    (np.float32, 1, 1, 97 * 5120 + 13),   # ragged last block
])
def test_ticket_levels_around_the_threshold(dtype, outer, channels, inner):
    rng = np.random.Generator(np.random.Philox(outer * 1000 + channels))
    x = (rng.standard_normal((outer, channels, inner)) * 2).astype(dtype)
    gy = rng.standard_normal(x.shape).astype(dtype)
    theta = workloads.theta_for_scale(rng.uniform(0.02, 0.05, channels))
    case = workloads.TensorCase("lv", x.shape, outer, channels, inner, -128, 127, x, theta, gy)
    _repeat(case, "stress/levels %dx%dx%d" % (outer, channels, inner), 20)


@pytest.mark.parametrize("blocks_per_channel", [1, 2, 3, 4, 5, 8, 64, 66, 130])
def test_every_combination_protocol_equals_the_two_launch_mode_bitwise(blocks_per_channel):
    """One block per slab (8192 FP16 elements), so a channel has exactly `outer` blocks: direct
    write, exchange, exchange tree, tickets, two-level tickets.  Each must give the bits of the
    two-launch mode (and the oracle's values); channel 0 has an all-zero upstream gradient."""
    outer, channels, inner = blocks_per_channel, 5, 8192
    rng = np.random.Generator(np.random.Philox(7000 + outer))
    x = (rng.standard_normal((outer, channels, inner)) * 2).astype(np.float16)
    gy = rng.standard_normal(x.shape).astype(np.float16)
    gy[:, 0, :] = 0.0
    theta = workloads.theta_for_scale(rng.uniform(0.02, 0.05, channels))
    case = workloads.TensorCase("proto", x.shape, outer, channels, inner, -128, 127, x, theta, gy)
    H.say("stress/protocols: %d blocks per channel" % outer)
    got = {}
    for flags in (0, fq.FQ_FLAG_TWO_PASS):
        dc = H.DeviceCase(case, want_q=False, flags=flags)
        ws = H.workspace_for(dc.desc, fq.FQ_MODE_BACKWARD)
        for rep in range(3):                       # the slots must be back at zero after every call
            dc.gs.fill_(float("nan"))
            dc.gtheta.fill_(float("nan"))
            fq.fq_backward(dc.desc, ws)
        torch.cuda.synchronize()
        if flags == 0:
            ref = H.oracle_forward(case)
            H.check_backward(dc, ref[0], ref[1], "stress/protocols")
        got[flags] = (dc.host("gs"), dc.host("gtheta"))
    for a, b in zip(got[0], got[fq.FQ_FLAG_TWO_PASS]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), (blocks_per_channel, a, b)
    assert got[0][0][0] == 0.0 and not np.signbit(got[0][0][0])
