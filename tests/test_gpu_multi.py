"""GPU parity of fq_multi_tensor: a whole list of tensors in one launch."""
import numpy as np
import pytest
import torch

from paper_2511_12653_amd import workloads
from paper_2511_12653_amd import binding as fq

import _gpu_harness as H

pytestmark = pytest.mark.gpu


def _run_list(cases, label, flags=0, want_q=True):
    H.say("%s: %d tensors, %.1f MiB of inputs, flags=%d" % (
        label, len(cases), sum(c.x.nbytes for c in cases) / 2 ** 20, flags))
    dcs = [H.DeviceCase(c, want_q=want_q and c.qmin >= -128, flags=flags) for c in cases]
    descs = [d.desc for d in dcs]
    ws = H.workspace_for(descs, fq.FQ_MODE_BACKWARD)
    assert fq.fq_workspace_bytes(descs, fq.FQ_MODE_FORWARD) <= ws.numel() * 4
    fq.fq_multi_tensor(descs, fq.FQ_MODE_FORWARD, ws)
    fq.fq_multi_tensor(descs, fq.FQ_MODE_BACKWARD, ws)
    torch.cuda.synchronize()
    for i, (c, d) in enumerate(zip(cases, dcs)):
        ref = H.oracle_forward(c)
        H.check_forward(d, ref, "%s[%d] fwd" % (label, i))
        H.check_backward(d, ref[0], ref[1], "%s[%d] bwd" % (label, i),
                         want_gx=not (flags & fq.FQ_FLAG_NO_DX))
        if i % 8 == 7:
            H.say("%s: %d of %d tensors match" % (label, i + 1, len(cases)))
    return dcs, ws


@pytest.mark.parametrize("flags", [0, fq.FQ_FLAG_TWO_PASS])
def test_small_mixed_list(flags):
    cases = workloads.multi_tensor_mixed(n_act=10, n_wgt=6, target_bytes=24 << 20, max_batch=2)
    _run_list(cases, "multi/small", flags=flags)


def test_list_with_empty_and_tiny_members():
    rng = np.random.default_rng(4)
    cases = workloads.multi_tensor_mixed(n_act=3, n_wgt=2, target_bytes=4 << 20, max_batch=1)
    x1 = rng.standard_normal((1, 1, 1)).astype(np.float32)
    tiny = workloads.TensorCase("tiny", (1,), 1, 1, 1, -8, 7, x1, np.array([0.1], np.float32), x1.copy())
    empty = workloads.TensorCase("empty", (0, 4, 9), 0, 4, 9, -128, 127, np.zeros((0, 4, 9), np.float16),
                                 np.array([0.1, 0.2, 0.3, 0.4], np.float32),
                                 np.zeros((0, 4, 9), np.float16))
    lst = [empty, cases[0], tiny, cases[1], empty, cases[2], cases[3], cases[4], empty]
    dcs, _ = _run_list(lst, "multi/empty_members")
    for d in (dcs[0], dcs[4], dcs[8]):
        assert torch.all(d.gs == 0) and torch.all(d.gtheta == 0)


def test_multi_equals_single_calls_bitwise():
    cases = workloads.multi_tensor_mixed(n_act=6, n_wgt=4, target_bytes=12 << 20, max_batch=2)
    dcs, _ = _run_list(cases, "multi/vs_single", want_q=False)
    H.say("multi/vs_single: single-tensor calls")
    for c, d in zip(cases, dcs):
        one = H.DeviceCase(c, want_q=False)
        fq.fq_forward(one.desc)
        ws = H.workspace_for(one.desc, fq.FQ_MODE_BACKWARD)
        fq.fq_backward(one.desc, ws)
        torch.cuda.synchronize()
        for name in ("y", "gx", "gs", "gtheta", "s"):
            a, b = getattr(one, name), getattr(d, name)
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), name


def test_list_of_a_thousand_tiny_tensors():
    """1000 tensors of 0..3000 elements each, every dtype / granularity / code range: the block ->
    tensor search, the descriptor table and the per-channel finalisation across many members."""
    rng = np.random.default_rng(99)
    cases = []
    for t in range(1000):
        dtype = np.float16 if rng.integers(0, 2) else np.float32
        c = int(rng.integers(1, 6))
        outer = int(rng.integers(1, 4))
        inner = int(rng.integers(0, 200)) if t % 97 else 0           # a few empty members
        if rng.integers(0, 2) == 0:
            outer, c, inner = 1, 1, outer * c * inner                 # per-tensor
        qmin, qmax = [(-128, 127), (-8, 7), (-127, 127)][int(rng.integers(0, 3))]
        x = (rng.standard_normal((outer, c, inner)) * 2).astype(dtype)
        gy = rng.standard_normal((outer, c, inner)).astype(dtype)
        theta = workloads.theta_for_scale(rng.uniform(0.01, 0.5, c))
        cases.append(workloads.TensorCase("t%d" % t, x.shape, outer, c, inner, qmin, qmax, x, theta, gy))
    _run_list(cases, "multi/thousand")


@pytest.mark.timeout(600)
def test_plan_replay_equals_direct_calls_bitwise():
    """fq_plan_create once, fq_plan_run several times with changing data and theta: every replay
    equals a fresh fq_multi_tensor call bit for bit (and the oracle once)."""
    cases = workloads.multi_tensor_mixed(n_act=5, n_wgt=3, target_bytes=8 << 20, max_batch=2)
    H.say("multi/plan: %d tensors" % len(cases))
    dcs = [H.DeviceCase(c, want_q=False) for c in cases]
    arr = fq.fq_tensor_array([d.desc for d in dcs])
    ws_f = H.workspace_for(arr, fq.FQ_MODE_FORWARD)
    ws_b = H.workspace_for(arr, fq.FQ_MODE_BACKWARD)
    plan_f = fq.fq_plan_create(arr, fq.FQ_MODE_FORWARD, ws_f)
    plan_b = fq.fq_plan_create(arr, fq.FQ_MODE_BACKWARD, ws_b)
    ws_ref = H.workspace_for(arr, fq.FQ_MODE_BACKWARD)
    try:
        for rep in range(3):
            if rep:
                for d in dcs:                       # new data, new theta, same addresses
                    d.x.mul_(1.25)
                    d.theta.add_(0.01 * rep)
            fq.fq_plan_run(plan_f)
            fq.fq_plan_run(plan_b)
            torch.cuda.synchronize()
            got = [[getattr(d, k).clone() for k in ("y", "gx", "gs", "gtheta", "s")] for d in dcs]
            if rep == 0:
                for i, (c, d) in enumerate(zip(cases, dcs)):
                    ref = H.oracle_forward(c)
                    H.check_forward(d, ref, "plan[%d] fwd" % i)
                    H.check_backward(d, ref[0], ref[1], "plan[%d] bwd" % i)
            for d in dcs:
                for k in ("y", "gx"):
                    getattr(d, k).zero_()
                for k in ("gs", "gtheta", "s"):
                    getattr(d, k).fill_(float("nan"))
            fq.fq_multi_tensor(arr, fq.FQ_MODE_FORWARD, ws_ref)
            fq.fq_multi_tensor(arr, fq.FQ_MODE_BACKWARD, ws_ref)
            torch.cuda.synchronize()
            for d, g in zip(dcs, got):
                for k, t in zip(("y", "gx", "gs", "gtheta", "s"), g):
                    assert torch.equal(getattr(d, k).view(torch.uint8), t.view(torch.uint8)), (rep, k)
    finally:
        fq.fq_plan_destroy(plan_f)
        fq.fq_plan_destroy(plan_b)


@pytest.mark.timeout(600)
def test_full_size_list_about_1GiB():
    """The 64-tensor, ~1 GiB list in the launch configuration used for timing: one forward launch
    and one backward launch, every element checked against the oracle."""
    cases = workloads.make("multi_tensor_mixed")
    total = sum(c.x.nbytes for c in cases)
    assert len(cases) == 64 and abs(total - 2 ** 30) <= 0.05 * 2 ** 30
    _run_list(cases, "multi/full", want_q=False)


@pytest.mark.timeout(300)
def test_list_mixing_block_and_wavefront_units_with_codes():
    """A list with enough blocks that its short-slab members are cut per wavefront (checked with
    fq_workspace_bytes: one partial sum per slab), next to ordinary members, int8 codes wanted for
    all: forward with codes, backward, against the oracle and against the single-tensor calls."""
    rng = np.random.Generator(np.random.Philox(5150))
    big = workloads.train_batch_fp16(shape=(4, 96, 120, 160))[0]            # 768 blocks

    def short(outer, c, inner, dtype):
        x = (rng.standard_normal((outer, c, inner)) * 2).astype(dtype)
        gy = rng.standard_normal(x.shape).astype(dtype)
        return workloads.TensorCase("short", x.shape, outer, c, inner, -128, 127, x,
                                    workloads.theta_for_scale(rng.uniform(0.01, 0.03, c)), gy)

    cases = [short(2, 1500, 147, np.float16), big, short(1, 900, 333, np.float32), short(5, 300, 8, np.float16)]
    dcs, ws = _run_list(cases, "multi/mixed_units", want_q=True)
    descs = [d.desc for d in dcs]
    # 3000 + 900 + 1500 slabs in block units would be 5400 blocks on top of 768: the launch has blocks
    # to spare, so those members need one partial per slab but only a quarter of the blocks
    alone = [fq.fq_layout(d) for d in descs]
    assert [a.wave_units for a in alone] == [0, 0, 0, 0]                   # each on its own: too small
    total = fq.fq_workspace_bytes(descs, fq.FQ_MODE_BACKWARD)
    separately = sum(fq.fq_workspace_bytes([d], fq.FQ_MODE_BACKWARD) for d in descs)
    assert total <= separately
    H.say("multi/mixed_units: single-tensor calls")
    for c, d in zip(cases, dcs):
        one = H.DeviceCase(c, want_q=True)
        fq.fq_forward(one.desc)
        ws1 = H.workspace_for(one.desc, fq.FQ_MODE_BACKWARD)
        fq.fq_backward(one.desc, ws1)
        torch.cuda.synchronize()
        for name in ("y", "q", "gx", "gs", "gtheta", "s"):
            a, b = getattr(one, name), getattr(d, name)
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), name


def _random_case(rng, name, budget):
    """One tensor of a random list: short slabs in bulk, a per-tensor scale, a feature map or an
    arbitrary small shape, any dtype and code range, at most `budget` elements."""
    dtype = np.float16 if rng.integers(0, 2) else np.float32
    kind = int(rng.integers(0, 4))
    if kind == 0:
        inner, c, outer = int(rng.choice([9, 40, 147, 1200, 2520, 2552, 2560])), int(rng.integers(1, 200)), int(rng.integers(1, 40))
    elif kind == 1:
        inner, c, outer = int(rng.integers(1, 300000)), 1, int(rng.integers(1, 4))
    elif kind == 2:
        inner, c, outer = int(rng.choice([19200, 4800, 22560, 28800, 9600, 9601])), int(rng.integers(1, 48)), int(rng.integers(1, 6))
    else:
        inner, c, outer = int(rng.integers(1, 20000)), int(rng.integers(1, 16)), int(rng.integers(1, 5))
    while outer * c * inner > budget and (outer > 1 or c > 1):
        if outer > 1:
            outer = (outer + 1) // 2
        else:
            c = (c + 1) // 2
    inner = min(inner, budget)
    qmin, qmax = [(-128, 127), (-127, 127), (-8, 7), (0, 15), (-2048, 2047)][int(rng.integers(0, 5))]
    spread = float(np.exp(rng.uniform(-2, 2)))
    x = (rng.standard_normal((outer, c, inner)) * spread).astype(dtype)
    gy = rng.standard_normal((outer, c, inner)).astype(dtype)
    s = spread * rng.uniform(0.5, 4.0, c) / max(abs(qmin), qmax)
    return workloads.TensorCase(name, x.shape, outer, c, inner, qmin, qmax, x, workloads.theta_for_scale(s), gy)


def test_randomised_lists():
    """Sixteen seeded random lists of 2..29 tensors (every unit shape, combination protocol, dtype
    and code range mixed in one launch; some lists have enough blocks for wavefront units)."""
    for seed in range(16):
        rng = np.random.default_rng(20_100 + seed)
        n = int(rng.integers(2, 30))
        budget = int(rng.choice([20_000, 200_000, 1_500_000]))
        cases = [_random_case(rng, "r%d_%d" % (seed, i), budget) for i in range(n)]
        flags = int(rng.choice([0, 0, fq.FQ_FLAG_TWO_PASS, fq.FQ_FLAG_NO_DX]))
        _run_list(cases, "multi/random[%d] budget=%d" % (seed, budget), flags=flags, want_q=bool(rng.integers(0, 2)))
