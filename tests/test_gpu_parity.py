"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Sizes here are ones the oracle finishes in seconds; they span several chunks per slab,
ragged tails, misaligned bases and every dtype / granularity."""
import numpy as np
import pytest
import torch

from paper_2511_12653_amd import workloads
from paper_2511_12653_amd import binding as fq

import _gpu_harness as H

pytestmark = pytest.mark.gpu


def _fwd_bwd(case, label, flags=0, inplace=False, misalign=0, want_q=True):
    H.say("%s: shape=%s view=(%d,%d,%d) dtype=%s q=[%d,%d] flags=%d inplace=%s misalign=%d" % (
        label, case.shape, case.outer, case.channels, case.inner, case.x.dtype, case.qmin, case.qmax,
        flags, inplace, misalign))
    ref = H.oracle_forward(case)
    s, active = ref[0], ref[1]
    dc = H.DeviceCase(case, want_q=want_q, flags=flags, inplace=False, misalign=misalign)
    fq.fq_forward(dc.desc)
    torch.cuda.synchronize()
    info = H.check_forward(dc, ref, label + " fwd")
    if case.gy is not None:
        ws = H.workspace_for(dc.desc, fq.FQ_MODE_BACKWARD)
        fq.fq_backward(dc.desc, ws)
        torch.cuda.synchronize()
        H.check_backward(dc, s, active, label + " bwd", want_gx=not (flags & fq.FQ_FLAG_NO_DX))
    if inplace:
        dci = H.DeviceCase(case, want_q=want_q, flags=flags, inplace=True, misalign=misalign)
        fq.fq_forward(dci.desc)
        torch.cuda.synchronize()
        assert torch.equal(dci.y, dc.y)
    return info


def test_act_fp32_per_tensor():
    case = workloads.make("act_fp32_per_tensor")[0]
    info = _fwd_bwd(case, "act_fp32_per_tensor")
    assert info["y_exact"]


def test_act_fp32_per_tensor_two_pass():
    case = workloads.make("act_fp32_per_tensor")[0]
    _fwd_bwd(case, "act_fp32_per_tensor/two_pass", flags=fq.FQ_FLAG_TWO_PASS)


@pytest.mark.parametrize("flags", [0, fq.FQ_FLAG_TWO_PASS])
def test_feature_fp16_per_channel_reduced(flags):
    # 37 channels x (48 x 67 = 3216 elements): one chunk per slab, ragged (3216 % 8 == 0 but
    # the slab is not a whole number of 256-lane rows)
    case = workloads.feature_fp16_per_channel(shape=(2, 37, 48, 67))[0]
    _fwd_bwd(case, "feature_fp16/reduced", flags=flags)


def test_feature_fp16_full_size():
    case = workloads.make("feature_fp16_per_channel")[0]
    info = _fwd_bwd(case, "feature_fp16_per_channel 1x384x120x160")
    assert info["y_exact"]


@pytest.mark.parametrize("flags", [0, fq.FQ_FLAG_NO_DX, fq.FQ_FLAG_TWO_PASS])
def test_conv_weights_fp32(flags):
    for case in workloads.make("conv_weights_fp32"):
        _fwd_bwd(case, "conv_weights_fp32/" + case.name, flags=flags)


def test_train_batch_fp16_reduced():
    # 3 frames x 16 channels x 120x160: three chunks per slab, reduction across frames
    case = workloads.train_batch_fp16(shape=(3, 16, 120, 160))[0]
    _fwd_bwd(case, "train_batch_fp16/reduced")


@pytest.mark.timeout(600)
def test_train_batch_fp16_full_size():
    """15x128x120x160 FP16, the reduction runs over 15 frames x 2 chunks = 30 blocks per channel."""
    case = workloads.make("train_batch_fp16")[0]
    info = _fwd_bwd(case, "train_batch_fp16 15x128x120x160", want_q=False)
    assert info["y_exact"]


@pytest.mark.parametrize("dtype", [np.float16, np.float32])
@pytest.mark.parametrize("inner", [1, 7, 8, 9, 147, 1023, 8191, 8200, 20001])
def test_odd_inner_and_misaligned_slabs(dtype, inner):
    """inner not a multiple of the vector width: slabs start off the 16-byte grid."""
    rng = np.random.default_rng(1000 + inner)
    outer, c = 2, 5
    x = (rng.standard_normal((outer, c, inner)) * 2).astype(dtype)
    gy = rng.standard_normal((outer, c, inner)).astype(dtype)
    s = rng.uniform(0.01, 0.03, c)
    case = workloads.TensorCase("odd", (outer, c, inner), outer, c, inner, -128, 127, x,
                                workloads.theta_for_scale(s), gy)
    _fwd_bwd(case, "odd_inner=%d/%s" % (inner, np.dtype(dtype).name))


@pytest.mark.parametrize("dtype", [np.float16, np.float32])
@pytest.mark.parametrize("misalign", [1, 3])
def test_misaligned_base_pointers(dtype, misalign):
    rng = np.random.default_rng(77 + misalign)
    outer, c, inner = 1, 3, 5000
    x = (rng.standard_normal((outer, c, inner)) * 2).astype(dtype)
    gy = rng.standard_normal((outer, c, inner)).astype(dtype)
    case = workloads.TensorCase("mis", (outer, c, inner), outer, c, inner, -8, 7, x,
                                workloads.theta_for_scale(rng.uniform(0.2, 0.4, c)), gy)
    _fwd_bwd(case, "misaligned_base=%d/%s" % (misalign, np.dtype(dtype).name), misalign=misalign)


def test_x_and_y_misaligned_relative_to_each_other():
    rng = np.random.default_rng(5)
    n = 4099
    x = rng.standard_normal(n).astype(np.float32)
    case = workloads.TensorCase("rel", (n,), 1, 1, n, -128, 127, x, np.array([-3.0], np.float32))
    ref = H.oracle_forward(case)
    H.say("x/y relative misalignment, n=%d" % n)
    xb = torch.empty(n + 4, dtype=torch.float32, device="cuda")
    yb = torch.empty(n + 4, dtype=torch.float32, device="cuda")
    xv, yv = xb[:n], yb[1:n + 1]
    xv.copy_(H.dev(x))
    yb.fill_(-7.0)
    theta = H.dev(case.theta)
    d = fq.FqTensor.from_torch(1, 1, n, -128, 127, x=xv, y=yv, theta=theta)
    fq.fq_forward(d)
    torch.cuda.synchronize()
    assert np.array_equal(yv.cpu().numpy(), ref[2])
    assert yb[0].item() == -7.0 and torch.all(yb[n + 1:] == -7.0)        # no write outside y


def test_in_place_forward_and_backward():
    case = workloads.feature_fp16_per_channel(shape=(1, 9, 40, 52))[0]
    _fwd_bwd(case, "in_place", inplace=True)
    H.say("in-place backward (gx aliases gy)")
    s, active = H.oracle_forward(case)[:2]
    dc = H.DeviceCase(case, want_q=False, inplace=True)
    ws = H.workspace_for(dc.desc, fq.FQ_MODE_BACKWARD)
    fq.fq_backward(dc.desc, ws)
    torch.cuda.synchronize()
    H.check_backward(dc, s, active, "in_place bwd")


def test_all_finite_fp16_inputs():
    """Every finite FP16 value, for several scales (one channel each)."""
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    h = h[np.isfinite(h)]
    scales = np.array([2.0 ** -6, 0.0236, 0.9740769863128662, 1.0 / 127, 3.0, 0.3333, 1e-3, 17.0])
    c = len(scales)
    x = np.broadcast_to(h, (c, h.size)).copy()
    gy = np.random.default_rng(3).standard_normal((c, h.size)).astype(np.float16)
    case = workloads.TensorCase("allhalf", (c, h.size), 1, c, h.size, -128, 127, x,
                                workloads.theta_for_scale(scales), gy)
    info = _fwd_bwd(case, "all_finite_fp16")
    assert info["y_exact"]


def test_code_ranges_and_clip_edges():
    rng = np.random.default_rng(9)
    for qmin, qmax in [(-128, 127), (-127, 127), (-8, 7), (0, 255), (-32768, 32767)]:
        n = 6000
        s = 0.05
        x = (rng.uniform(qmin - 4, qmax + 4, n) * s).astype(np.float32)
        x[:600] = ((np.arange(600) - 300) * 0.5 * s + (qmax if qmax < 300 else 0) * s).astype(np.float32)
        gy = rng.standard_normal(n).astype(np.float32)
        case = workloads.TensorCase("rng", (n,), 1, 1, n, qmin, qmax, x,
                                    workloads.theta_for_scale([s]), gy)
        _fwd_bwd(case, "code_range[%d,%d]" % (qmin, qmax), want_q=(qmin >= -128 and qmax <= 127))


def test_scale_clamp_and_eps():
    rng = np.random.default_rng(21)
    c, inner = 6, 3000
    theta = np.array([-9.0, -2.0, 0.0, 1.0, 4.0, 9.0], np.float32)
    x = rng.standard_normal((1, c, inner)).astype(np.float16)
    gy = rng.standard_normal((1, c, inner)).astype(np.float16)
    case = workloads.TensorCase("clamp", (1, c, inner), 1, c, inner, -128, 127, x, theta, gy,
                                eps=1e-3, s_min=2.0 ** -7, s_max=3.0)
    _fwd_bwd(case, "scale_clamp_eps")


@pytest.mark.parametrize("dtype", [np.float16, np.float32])
@pytest.mark.parametrize("q_offset", [0, 1, 3])
def test_codes_only_forward(dtype, q_offset):
    """y = NULL: only the packed int8 codes (and the scales) are written; q at any byte offset."""
    rng = np.random.default_rng(40 + q_offset)
    outer, c, inner = 2, 6, 5003
    x = (rng.standard_normal((outer, c, inner)) * 2).astype(dtype)
    case = workloads.TensorCase("codes", x.shape, outer, c, inner, -128, 127, x,
                                workloads.theta_for_scale(rng.uniform(0.01, 0.03, c)))
    H.say("codes only %s q_offset=%d" % (np.dtype(dtype).name, q_offset))
    s_ref, _, _, q_ref = H.oracle_forward(case)
    n = case.numel
    xd, theta = H.dev(x.reshape(-1)), H.dev(case.theta)
    qbuf = torch.full((n + 16,), 99, dtype=torch.int8, device="cuda")
    qv = qbuf[q_offset:q_offset + n]
    s = torch.empty(c, device="cuda")
    d = fq.FqTensor.from_torch(outer, c, inner, -128, 127, x=xd, q=qv, theta=theta, s=s)
    fq.fq_forward(d)
    torch.cuda.synchronize()
    assert np.array_equal(s.cpu().numpy(), s_ref)
    assert np.array_equal(qv.cpu().numpy().astype(np.int32), q_ref)
    assert torch.all(qbuf[:q_offset] == 99) and torch.all(qbuf[q_offset + n:] == 99)


def test_scale_sweep_bit_exact():
    """Eq. (3)-(4) over two million theta values (dense sweep, random, specials), through the
    scale-only path of a tensor with channels but no elements."""
    from oracle import fq_oracle
    rng = np.random.default_rng(2511)
    theta = np.concatenate([
        np.linspace(-120.0, 100.0, 1 << 20), rng.standard_normal(1 << 19) * 4.0,
        rng.uniform(-20.0, 20.0, 1 << 19),
        [0.0, -0.0, 0.5, 20.0, -20.0, 88.7, -87.3, -103.9, -104.0, -745.0, -800.0, 745.0, 1e30, -1e30,
         3.4e38, -3.4e38, np.inf, -np.inf, 1e-30, -1e-30, 1e-45]]).astype(np.float32)
    for eps, s_min, s_max in [(0.0, fq.FLT_MIN, float("inf")), (1e-4, 2.0 ** -14, 512.0)]:
        H.say("scale sweep: %d thetas eps=%g s_min=%g s_max=%g" % (theta.size, eps, s_min, s_max))
        th = H.dev(theta)
        s = torch.full((theta.size,), float("nan"), device="cuda")
        d = fq.FqTensor.from_torch(0, theta.size, 8, -128, 127, theta=th, s=s, dtype=fq.FQ_F16,
                                   eps=eps, s_min=s_min, s_max=s_max)
        fq.fq_forward(d)
        torch.cuda.synchronize()
        ref, _ = fq_oracle.scale(theta, eps, s_min, s_max)
        got = s.cpu().numpy()
        bad = np.nonzero(got.view(np.uint32) != ref.view(np.uint32))[0]
        assert bad.size == 0, "scale differs for theta=%r: %r vs %r" % (
            theta[bad[:5]], got[bad[:5]], ref[bad[:5]])


def test_non_finite_inputs():
    x = np.array([np.inf, -np.inf, np.nan, 1.0, -0.0, 0.0, 1e-40, 65504.0] * 40, np.float32)
    gy = np.array([1.0, np.nan, 2.0, 3.0, np.inf, 4.0, 5.0, 6.0] * 40, np.float32)
    for dtype in (np.float32, np.float16):
        # channel 0 holds the non-finite values (its scale gradient is NaN), channel 1 is clean
        xx = np.stack([x, np.linspace(-3, 3, x.size).astype(np.float32)]).astype(dtype)
        gg = np.stack([gy, np.ones_like(gy)]).astype(dtype)
        case = workloads.TensorCase("nonfinite", xx.shape, 1, 2, x.size, -128, 127, xx,
                                    np.array([0.5, -1.0], np.float32), gg)
        _fwd_bwd(case, "non_finite/" + np.dtype(dtype).name)


def test_empty_tensors():
    H.say("empty tensors")
    theta = H.dev(np.array([0.5, 1.5], np.float32))
    s = torch.full((2,), float("nan"), device="cuda")
    gs = torch.full((2,), float("nan"), device="cuda")
    gt = torch.full((2,), float("nan"), device="cuda")
    d = fq.FqTensor.from_torch(0, 2, 64, -128, 127, theta=theta, s=s, gs=gs, gtheta=gt, dtype=fq.FQ_F16)
    fq.fq_forward(d)
    ws = H.workspace_for(d, fq.FQ_MODE_BACKWARD)
    fq.fq_backward(d, ws)
    torch.cuda.synchronize()
    from oracle import fq_oracle
    ref, _ = fq_oracle.scale(np.array([0.5, 1.5], np.float32))
    assert np.array_equal(s.cpu().numpy(), ref)
    assert torch.all(gs == 0) and torch.all(gt == 0)
    d0 = fq.FqTensor.from_torch(3, 0, 5, -128, 127, dtype=fq.FQ_F32)
    fq.fq_forward(d0)
    fq.fq_backward(d0, ws)
    torch.cuda.synchronize()


def test_backward_is_bitwise_reproducible():
    """Same inputs, same workspace, repeated calls: identical bits every time (no float atomics;
    the ticket counters must come back to zero or the second call would not finish its sums)."""
    case = workloads.train_batch_fp16(shape=(3, 16, 120, 160))[0]
    H.say("run-twice determinism, fused and two-pass")
    first = None
    for flags in (0, fq.FQ_FLAG_TWO_PASS):
        dc = H.DeviceCase(case, want_q=False, flags=flags)
        ws = H.workspace_for(dc.desc, fq.FQ_MODE_BACKWARD)
        for rep in range(3):
            dc.gs.fill_(float("nan"))
            dc.gtheta.fill_(float("nan"))
            dc.gx.zero_()
            fq.fq_backward(dc.desc, ws)
            torch.cuda.synchronize()
            out = (dc.host("gs"), dc.host("gtheta"), dc.host("gx"))
            assert not np.isnan(out[0]).any() and not np.isnan(out[1]).any()
            if first is None:
                first = out
            for a, b in zip(first, out):
                assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), (flags, rep)


@pytest.mark.timeout(600)
def test_more_than_2_31_elements():
    """One per-tensor FP16 tensor of 2^31 + 4099 elements (64-bit element offsets, 209 719 blocks,
    as many partial sums for one channel).  Outputs are checked against the oracle on slices
    (a per-tensor scale makes every slice a valid tensor of its own): the head, a window across
    element 2^31, the ragged tail, and windows at odd offsets; the scale gradient of the whole
    tensor is checked against the binary64 sum of the scale gradients of eight pieces."""
    from oracle import fq_oracle
    n = (1 << 31) + 4099
    H.say("large tensor: %d FP16 elements" % n)
    g = torch.Generator(device="cuda").manual_seed(20251112)
    x = torch.empty(n, dtype=torch.float16, device="cuda")
    gy = torch.empty(n, dtype=torch.float16, device="cuda")
    step = 1 << 28
    for a in range(0, n, step):
        b = min(n, a + step)
        x[a:b] = torch.randn(b - a, generator=g, device="cuda", dtype=torch.float32).mul_(3.0)
        gy[a:b] = torch.randn(b - a, generator=g, device="cuda", dtype=torch.float32)
    y, gx = torch.empty_like(x), torch.empty_like(x)
    theta_h = workloads.theta_for_scale([0.05])
    theta = H.dev(theta_h)
    s, gs, gt = (torch.full((1,), float("nan"), device="cuda") for _ in range(3))
    d = fq.FqTensor.from_torch(1, 1, n, -128, 127, x=x, y=y, theta=theta, s=s, gy=gy, gx=gx, gs=gs, gtheta=gt)
    ws = H.workspace_for(d, fq.FQ_MODE_BACKWARD)
    fq.fq_forward(d)
    fq.fq_backward(d, ws)
    torch.cuda.synchronize()
    so, active = fq_oracle.scale(theta_h)
    assert np.array_equal(s.cpu().numpy(), so)
    windows = [(0, 1 << 20), ((1 << 31) - (1 << 19), n), (123457, 123457 + 300001),
               ((1 << 30) + 7, (1 << 30) + 7 + 262147), (n - 4099 - 1283, n - 5)]
    for a, b in windows:
        H.say("  window [%d, %d)" % (a, b))
        xs, gys = x[a:b].cpu().numpy(), gy[a:b].cpu().numpy()
        yo, _ = fq_oracle.forward(xs, so, -128, 127, 1, 1, b - a, want_q=False)
        ro = fq_oracle.backward(xs, gys, so, theta_h, active, -128, 127, 1, 1, b - a)
        assert np.array_equal(y[a:b].cpu().numpy().view(np.uint16), yo.view(np.uint16))
        assert np.array_equal(gx[a:b].cpu().numpy().view(np.uint16), ro["gx"].view(np.uint16))
    # whole-tensor scale gradient vs eight pieces run separately
    total, pieces = float(gs.item()), []
    cut = [0] + [k * (n // 8) + 3 * k for k in range(1, 8)] + [n]
    gsp = torch.empty(1, device="cuda")
    for a, b in zip(cut[:-1], cut[1:]):
        dp = fq.FqTensor.from_torch(1, 1, b - a, -128, 127, x=x[a:b], theta=theta, gy=gy[a:b], gs=gsp,
                                    flags=fq.FQ_FLAG_NO_DX)
        wsp = H.workspace_for(dp, fq.FQ_MODE_BACKWARD)
        fq.fq_backward(dp, wsp)
        torch.cuda.synchronize()
        pieces.append(float(gsp.item()))
    assert abs(total - sum(pieces)) <= 1e-6 * sum(abs(p) for p in pieces), (total, pieces)


def test_randomised_shapes_alignments_and_flags():
    """Eighty seeded random single-tensor cases: extents (including chunk boundaries +-1), dtype,
    code range, scale clamp, base misalignment, NO_DX / TWO_PASS flags."""
    rng = np.random.default_rng(777)
    edges = [1, 2, 63, 64, 65, 511, 512, 513, 1279 * 4, 1280 * 4, 1280 * 4 + 1, 1280 * 8 - 1, 1280 * 8,
             1280 * 8 + 3, 2 * 1280 * 8 + 5]
    for k in range(80):
        dtype = np.float16 if rng.integers(0, 2) else np.float32
        inner = int(rng.choice(edges)) if rng.integers(0, 2) else int(rng.integers(1, 30000))
        outer, c = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        if outer * c * inner > 400_000:
            outer = 1
        qmin, qmax = [(-128, 127), (-127, 127), (-8, 7), (0, 15), (-2048, 2047)][int(rng.integers(0, 5))]
        flags = int(rng.choice([0, 0, fq.FQ_FLAG_NO_DX, fq.FQ_FLAG_TWO_PASS, fq.FQ_FLAG_NO_DX | fq.FQ_FLAG_TWO_PASS]))
        spread = float(np.exp(rng.uniform(-3, 3)))
        x = (rng.standard_normal((outer, c, inner)) * spread).astype(dtype)
        gy = rng.standard_normal((outer, c, inner)).astype(dtype)
        s = spread * rng.uniform(0.5, 4.0, c) / max(abs(qmin), qmax) * rng.choice([0.2, 1.0, 1.0, 3.0], c)
        kw = {}
        if rng.integers(0, 3) == 0:
            kw = dict(eps=float(rng.uniform(0, 1e-3)), s_min=float(s.min() * 1.5), s_max=float(s.max() * 0.9))
            if kw["s_max"] < kw["s_min"]:
                kw["s_max"] = kw["s_min"]
        case = workloads.TensorCase("rnd%d" % k, x.shape, outer, c, inner, qmin, qmax, x,
                                    workloads.theta_for_scale(s), gy, **kw)
        _fwd_bwd(case, "random[%d]" % k, flags=flags, misalign=int(rng.integers(0, 8)),
                 want_q=(qmin >= -128 and qmax <= 127))


@pytest.mark.parametrize("dtype, inner", [(np.float16, 1), (np.float16, 7), (np.float16, 147), (np.float16, 1001),
                                          (np.float16, 2551), (np.float32, 5), (np.float32, 333),
                                          (np.float32, 1275)])
@pytest.mark.parametrize("flags, misalign", [(0, 0), (fq.FQ_FLAG_NO_DX, 1), (fq.FQ_FLAG_TWO_PASS, 0)])
def test_wavefront_units_short_slabs(dtype, inner, flags, misalign):
    """Thousands of short slabs: every wavefront owns a whole slab (fq_layout says so).  Odd slab
    lengths put most slabs off the 16-byte grid (scalar heads and tails inside a wavefront), the
    longest cases fill a wavefront's five rows; codes, y, gx and the scale gradients against the
    oracle, in place as well."""
    rng = np.random.default_rng(4000 + inner)
    outer, c = 2, 2100
    x = (rng.standard_normal((outer, c, inner)) * 2).astype(dtype)
    gy = rng.standard_normal((outer, c, inner)).astype(dtype)
    case = workloads.TensorCase("waves", (outer, c, inner), outer, c, inner, -128, 127, x,
                                workloads.theta_for_scale(rng.uniform(0.01, 0.03, c)), gy)
    probe = H.DeviceCase(case, want_q=False)
    info = fq.fq_layout(probe.desc)
    assert info.wave_units == 1 and info.units_per_channel == outer and info.blocks == (outer * c + 3) // 4
    del probe
    _fwd_bwd(case, "wave_units inner=%d/%s" % (inner, np.dtype(dtype).name), flags=flags, misalign=misalign,
             inplace=(flags == 0))
