"""Repeat the backward pass many times on one workspace: the cross-block combination (atomic
exchange for two blocks per channel, tickets for more) must hand every channel's finisher the
other blocks' sums of THIS launch.  Two cases of the same shape but different upstream gradients
take turns on the workspace, so a partial sum left over from the launch before belongs to the
other case and would change bits; outputs are poisoned before every launch and compared on the
device."""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2511_12653_amd import workloads
from paper_2511_12653_amd import binding as fq

import _gpu_harness as H

pytestmark = pytest.mark.gpu


def _other_gradient(case):
    """The same tensor with another upstream gradient (every partial sum differs)."""
    rng = np.random.Generator(np.random.Philox(991))
    gy = (case.gy.astype(np.float32) * -0.75 + rng.standard_normal(case.gy.shape).astype(np.float32)).astype(
        case.gy.dtype)
    return dataclasses.replace(case, gy=gy)


def _repeat(case, label, iters):
    H.say("%s: %d launches, two gradients alternating on one workspace" % (label, iters))
    cases = (case, _other_gradient(case))
    dcs = [H.DeviceCase(c, want_q=False) for c in cases]
    ws = H.workspace_for(dcs[0].desc, fq.FQ_MODE_BACKWARD)
    assert fq.fq_workspace_bytes(dcs[1].desc, fq.FQ_MODE_BACKWARD) == ws.numel() * 4
    want = []
    for c, dc in zip(cases, dcs):
        fq.fq_backward(dc.desc, ws)
        torch.cuda.synchronize()
        ref = H.oracle_forward(c)
        H.check_backward(dc, ref[0], ref[1], label)
        want.append([t.clone() for t in (dc.gs, dc.gtheta, dc.gx)])
    assert not torch.equal(want[0][0], want[1][0]), label + ": the two cases must differ"
    bad = torch.zeros((), dtype=torch.int64, device="cuda")
    for i in range(iters):
        dc, w = dcs[i % 2], want[i % 2]
        dc.gs.fill_(float("nan"))
        dc.gtheta.fill_(float("nan"))
        fq.fq_backward(dc.desc, ws)
        for got, ww in zip((dc.gs, dc.gtheta), w[:2]):
            bad += (got.view(torch.int32) != ww.view(torch.int32)).sum()
    torch.cuda.synchronize()
    assert int(bad.item()) == 0, "%s: %d mismatching words over %d launches" % (label, int(bad.item()), iters)
    for dc, w in zip(dcs, want):
        assert torch.equal(dc.gx.view(torch.uint8), w[2].view(torch.uint8))


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


def _protocol_case(dtype, outer, channels, inner, units, waves, extra, iters=3):
    """Fused backward against the two-launch mode, bit for bit, and against the oracle, on a shape
    whose layout (fq_layout) is asserted first so that the intended protocol is the one running.
    Channel 0 has an all-zero upstream gradient (a sum of +0.0 travels as -0.0 in the exchanges)."""
    rng = np.random.Generator(np.random.Philox(7000 + outer * 31 + channels))
    x = (rng.standard_normal((outer, channels, inner)) * 2).astype(dtype)
    gy = rng.standard_normal(x.shape).astype(dtype)
    gy[:, 0, :] = 0.0
    theta = workloads.theta_for_scale(rng.uniform(0.02, 0.05, channels))
    case = workloads.TensorCase("proto", x.shape, outer, channels, inner, -128, 127, x, theta, gy)
    got = {}
    for flags in (0, fq.FQ_FLAG_TWO_PASS):
        dc = H.DeviceCase(case, want_q=False, flags=flags)
        info = fq.fq_layout(dc.desc)
        assert (info.units_per_channel, info.wave_units, info.extra_slots) == (units, waves, extra), (
            info.units_per_channel, info.wave_units, info.extra_slots)
        H.say("stress/protocols: %dx%dx%d %s: %d units per channel, wave units %d, extra slots %d, flags %d" % (
            outer, channels, inner, np.dtype(dtype).name, units, waves, extra, flags))
        ws = H.workspace_for(dc.desc, fq.FQ_MODE_BACKWARD)
        for rep in range(iters):                   # the slots must be back at zero after every call
            dc.gs.fill_(float("nan"))
            dc.gtheta.fill_(float("nan"))
            fq.fq_backward(dc.desc, ws)
        torch.cuda.synchronize()
        if flags == 0:
            ref = H.oracle_forward(case)
            H.check_backward(dc, ref[0], ref[1], "stress/protocols")
        got[flags] = (dc.host("gs"), dc.host("gtheta"), dc.host("gx"))
    for a, b in zip(got[0], got[fq.FQ_FLAG_TWO_PASS]):
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), (units, a, b)
    assert got[0][0][0] == 0.0 and not np.signbit(got[0][0][0])


@pytest.mark.parametrize("outer, extra", [(1, 0), (2, 0), (3, 2), (4, 2), (5, 0), (8, 0), (16, 0), (17, 16),
                                          (40, 16), (66, 16), (130, 16), (256, 16), (257, 32), (300, 32)])
def test_wavefront_units_every_protocol(outer, extra):
    """Short slabs (40 FP16 elements) and thousands of them: one wavefront per slab, so a channel
    has exactly `outer` units: direct write, exchange, exchange tree, tickets, two-level tickets."""
    _protocol_case(np.float16, outer, 4100, 40, outer, 1, extra, iters=2)


@pytest.mark.parametrize("dtype, outer, inner, units, extra", [
    (np.float16, 1, 19200, 2, 0),        # the headline layout: exchange
    (np.float16, 1, 28800, 3, 2),        # exchange tree, three blocks
    (np.float16, 1, 22560, 4, 2),        # exchange tree, four blocks
    (np.float32, 1, 9600 * 3, 6, 0),     # tickets on one slot
    (np.float16, 8, 19200, 16, 0),       # the last count that shares one slot
    (np.float16, 9, 19200, 18, 16),      # two-level tickets
])
def test_block_units_every_protocol(dtype, outer, inner, units, extra):
    _protocol_case(dtype, outer, 384, inner, units, 0, extra, iters=2)


def test_one_scale_many_blocks_two_level_tickets():
    rng = np.random.Generator(np.random.Philox(77))
    n = 97 * 5120 + 13                                              # ragged last block
    x = (rng.standard_normal(n) * 2).astype(np.float32)
    gy = rng.standard_normal(n).astype(np.float32)
    case = workloads.TensorCase("one", (n,), 1, 1, n, -128, 127, x, workloads.theta_for_scale([0.03]), gy)
    dc = H.DeviceCase(case, want_q=False)
    info = fq.fq_layout(dc.desc)
    assert info.units_per_channel > 16 and info.extra_slots in (16, 32) and info.wave_units == 0
    _repeat(case, "stress/one_scale %d blocks" % info.units_per_channel, 20)


def test_one_workspace_serves_lists_of_other_shapes_after_zeroing():
    """What a call leaves in a workspace (partial sums, where the slots lie) belongs to its tensor
    list: fq_workspace_init between two lists of different shapes makes the workspace fit for the
    next one, on the stream, with no host synchronisation in between."""
    rng = np.random.Generator(np.random.Philox(4242))

    def case(outer, channels, inner, dtype):
        x = (rng.standard_normal((outer, channels, inner)) * 2).astype(dtype)
        gy = rng.standard_normal(x.shape).astype(dtype)
        theta = workloads.theta_for_scale(rng.uniform(0.02, 0.05, channels))
        return workloads.TensorCase("reuse", x.shape, outer, channels, inner, -128, 127, x, theta, gy)

    # tickets on many partial sums, then an exchange layout whose slots lie where those sums were,
    # then two-level tickets, then the first one again
    cases = [case(6, 48, 19200, np.float16), case(1, 384, 19200, np.float16), case(1, 1, 97 * 5120 + 13, np.float32)]
    cases.append(cases[0])
    dcs = [H.DeviceCase(c, want_q=False) for c in cases]
    need = max(fq.fq_workspace_bytes(dc.desc, fq.FQ_MODE_BACKWARD) for dc in dcs)
    ws = torch.full((need // 4,), 0x7fc00000, dtype=torch.int32, device="cuda")      # not zero: must be initialised
    for i, dc in enumerate(dcs):
        H.say("stress/reuse: list %d of %d on one workspace of %d bytes" % (i + 1, len(dcs), need))
        fq.fq_workspace_init(ws)
        fq.fq_backward(dc.desc, ws)
    torch.cuda.synchronize()
    for c, dc in zip(cases, dcs):
        ref = H.oracle_forward(c)
        H.check_backward(dc, ref[0], ref[1], "stress/reuse")


def test_calls_on_two_streams_with_a_workspace_each():
    """Two streams, each with its own tensors and workspace, launching at the same time: calls
    that do not share a workspace do not disturb each other (forward and backward, tickets on one
    stream, exchange on the other)."""
    a = workloads.train_batch_fp16(shape=(4, 32, 120, 160))[0]      # 8 blocks per channel: tickets
    b = workloads.make("feature_fp16_per_channel")[0]               # 2 blocks per channel: exchange
    want = []
    for c in (a, b):
        dc = H.DeviceCase(c, want_q=False)
        fq.fq_forward(dc.desc)
        fq.fq_backward(dc.desc, H.workspace_for(dc.desc, fq.FQ_MODE_BACKWARD))
        torch.cuda.synchronize()
        ref = H.oracle_forward(c)
        H.check_forward(dc, ref, "stress/streams reference")
        H.check_backward(dc, ref[0], ref[1], "stress/streams reference")
        want.append([t.clone() for t in (dc.y, dc.gx, dc.gs, dc.gtheta)])
    dcs = [H.DeviceCase(c, want_q=False) for c in (a, b)]
    wss = [H.workspace_for(dc.desc, fq.FQ_MODE_BACKWARD) for dc in dcs]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    bad = [torch.zeros((), dtype=torch.int64, device="cuda") for _ in dcs]
    H.say("stress/streams: 60 rounds of forward + backward on two streams at once")
    for i in range(60):
        for k, (dc, ws, st) in enumerate(zip(dcs, wss, streams)):
            with torch.cuda.stream(st):
                for t in (dc.y, dc.gx):
                    t.view(torch.uint8).fill_(0xff)
                dc.gs.fill_(float("nan"))
                dc.gtheta.fill_(float("nan"))
                fq.fq_forward(dc.desc, st.cuda_stream)
                fq.fq_backward(dc.desc, ws, st.cuda_stream)
                for got, w in zip((dc.y, dc.gx, dc.gs, dc.gtheta), want[k]):
                    bad[k] += (got.view(torch.uint8) != w.view(torch.uint8)).sum()
    torch.cuda.synchronize()
    assert [int(x.item()) for x in bad] == [0, 0]
