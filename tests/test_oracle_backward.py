"""Pins for the oracle's straight-through-estimator backward (round differentiated as the
identity, as stated next to Eq. (5) with the LSQ citation)."""
import os

import numpy as np
import pytest

from test_oracle_forward import _table, _bits


def _bwd(oracle, x, gy, s, qmin, qmax, outer, c, inner, theta=None, active=None):
    theta = np.zeros(c, np.float32) if theta is None else theta
    active = np.zeros(c, np.uint8) if active is None else active
    return oracle.backward(x, gy, s, theta, active, qmin, qmax, outer, c, inner)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_table_T(oracle, dtype):
    t = _table("table_T.txt")
    x, gy = t[:, 0].astype(dtype), t[:, 4].astype(dtype)
    theta = np.array([np.log(np.expm1(0.5))], np.float32)
    s, active = oracle.scale(theta)
    assert s[0] == 0.5 and active[0] == 0
    r = oracle.backward(x, gy, s, theta, active, -128, 127, 1, 1, x.size)
    assert np.array_equal(_bits(r["gx"]), _bits(t[:, 5].astype(dtype)))
    assert r["acc"][0] == -261.0 and r["gs"][0] == np.float32(-261.0)
    assert r["aabs"][0] == 0.5 + 1.0 + 1.5 + 2.0 + 762 + 1024
    # sigmoid(theta) = 1 - e^-0.5 ; theta itself is rounded to binary32, hence 1e-7
    np.testing.assert_allclose(r["gtheta"][0], -102.69549781500268, rtol=2e-7)
    # symmetric range: v = -128 is now outside, t = -127 there and for the last row
    r = oracle.backward(x, gy, s, theta, active, -127, 127, 1, 1, x.size)
    assert list(r["gx"].astype(np.float64)) == [1, 2, 3, 4, 5, 0, 0, 0]
    assert r["acc"][0] == -0.5 + 1.0 - 1.5 + 2.0 + 0 + 6 * 127 - 7 * 127 - 8 * 127


def test_surrogate_finite_difference(oracle):
    """Freeze delta_i = round(clip(v_i)) - clip(v_i) at s0; then y~_i(s) = s*(clip(x_i/s)+delta_i)
    is differentiable in s and its derivative at s0 is exactly the STE scale gradient."""
    rng = np.random.default_rng(23)
    n = 4000
    s0 = np.float32(0.0371)
    x = (rng.standard_normal(n) * 3).astype(np.float32)        # about 12 % of |v| beyond 127
    gy = rng.standard_normal(n).astype(np.float32)
    r = _bwd(oracle, x, gy, np.array([s0]), -128, 127, 1, 1, n)
    xd, gd = x.astype(np.float64), gy.astype(np.float64)
    v0 = np.clip(xd / float(s0), -128, 127)
    delta = np.rint(v0) - v0

    def loss(sv):
        return np.sum(gd * sv * (np.clip(xd / sv, -128, 127) + delta))

    h = 1e-7
    fd = (loss(float(s0) + h) - loss(float(s0) - h)) / (2 * h)
    # the oracle forms v in binary32 (relative error 6e-8 on |v| <= 128): scale tolerance by sum|terms|
    assert abs(r["acc"][0] - fd) <= 2e-5 * r["aabs"][0] / np.sqrt(n) + 1e-6 * abs(fd)
    assert abs(r["acc"][0] - fd) <= 1e-5 * abs(fd)


def test_true_finite_difference_on_saturated_and_interior(oracle):
    """Where |v| is far outside the range the true function is y = s*qmax (or s*qmin): slope
    qmax/qmin, equal to the STE value.  Inside the range the true slope is q, NOT q - v: the
    STE deliberately differs there (this guards against 'fixing' the formula)."""
    s0 = np.float32(0.05)
    x = np.array([100.0, -100.0, 0.26], np.float32)            # v = 2000, -2000, 5.2
    gy = np.ones(3, np.float32)
    one = lambda i: _bwd(oracle, x[i:i + 1], gy[i:i + 1], np.array([s0]), -128, 127, 1, 1, 1)["acc"][0]
    assert one(0) == 127.0 and one(1) == -128.0

    def y_at(sv, i):
        yy, _ = oracle.forward(x[i:i + 1], np.array([sv], np.float32), -128, 127, 1, 1, 1)
        return float(yy[0])

    h = np.float32(2.0 ** -12)
    for i, want in [(0, 127.0), (1, -128.0), (2, 5.0)]:
        slope = (y_at(s0 + h, i) - y_at(s0 - h, i)) / (float(s0 + h) - float(s0 - h))
        assert abs(slope - want) < 1e-3
    assert abs(one(2) - (5.0 - 5.2)) < 1e-5                   # STE: q - v


def test_torch_autograd_float64_composite(oracle):
    """Autograd of clamp / detach-round / multiply in float64.  With a power-of-two scale the
    binary32 quotient is exact, so the two agree to float64 rounding."""
    import torch
    rng = np.random.default_rng(29)
    outer, c, inner = 2, 3, 500
    s = np.array([2.0 ** -5, 2.0 ** -4, 2.0 ** -6], np.float32)
    theta = np.log(np.expm1(s.astype(np.float64))).astype(np.float32)
    x = (rng.standard_normal((outer, c, inner)) * 3).astype(np.float32)
    gy = rng.standard_normal((outer, c, inner)).astype(np.float32)
    r = oracle.backward(x, gy, s, theta, np.zeros(c, np.uint8), -128, 127, outer, c, inner)

    ts = torch.tensor(s.astype(np.float64), requires_grad=True)
    tx = torch.tensor(x.astype(np.float64), requires_grad=True)
    v = tx / ts[None, :, None]
    vc = torch.clamp(v, -128, 127)
    y = (vc + (torch.round(vc) - vc).detach()) * ts[None, :, None]
    (y * torch.tensor(gy.astype(np.float64))).sum().backward()
    np.testing.assert_allclose(r["acc"], ts.grad.numpy(), rtol=1e-12, atol=1e-12)
    assert np.array_equal(r["gx"].astype(np.float64), tx.grad.numpy())

    # chain rule through Eq. (3)-(4) for a general theta, autograd through softplus in float64
    theta = rng.uniform(-4, 1, c).astype(np.float32)
    s, active = oracle.scale(theta)
    r = oracle.backward(x, gy, s, theta, active, -128, 127, outer, c, inner)
    tt = torch.tensor(theta.astype(np.float64), requires_grad=True)
    ts = torch.nn.functional.softplus(tt)
    v = torch.tensor(x.astype(np.float64)) / ts[None, :, None]
    vc = torch.clamp(v, -128, 127)
    y = (vc + (torch.round(vc) - vc).detach()) * ts[None, :, None]
    (y * torch.tensor(gy.astype(np.float64))).sum().backward()
    # the oracle's s and v carry binary32 rounding: compare relative to sum|terms|
    err = np.abs(r["gtheta"].astype(np.float64) - tt.grad.numpy())
    assert np.all(err <= 1e-5 * r["aabs"] * torch.sigmoid(tt).detach().numpy())


def test_mask_is_on_the_unrounded_quotient(oracle):
    s = np.array([1.0], np.float32)
    hi, lo = np.float32(127.0), np.float32(-128.0)
    x = np.array([hi, np.nextafter(hi, np.float32(np.inf)), 127.4, lo,
                  np.nextafter(lo, np.float32(-np.inf)), -128.4, np.inf, -np.inf, np.nan], np.float32)
    gy = np.array([1, 2, 3, 4, 5, 6, np.nan, np.inf, 7], np.float32)
    r = _bwd(oracle, x[:6], gy[:6], s, -128, 127, 1, 1, 6)
    assert list(r["gx"]) == [1, 0, 0, 4, 0, 0]
    assert r["acc"][0] == 0 + 2 * 127 + 3 * 127 + 0 - 5 * 128 - 6 * 128
    r = _bwd(oracle, x, gy, s, -128, 127, 1, 1, 9)
    # masked slots hold +0 bits whatever gy was
    assert list(_bits(r["gx"])[6:]) == [0, 0, 0]
    assert np.isnan(r["acc"][0])


def test_reduction_properties(oracle):
    rng = np.random.default_rng(31)
    outer, c, inner = 3, 4, 900
    s = rng.uniform(0.02, 0.05, c).astype(np.float32)
    x = (rng.standard_normal((outer, c, inner)) * 3).astype(np.float32)
    gy = rng.standard_normal((outer, c, inner)).astype(np.float32)
    r = _bwd(oracle, x, gy, s, -128, 127, outer, c, inner)
    # permutation inside a channel leaves the sum unchanged (binary64 accumulation)
    perm = rng.permutation(inner)
    rp = _bwd(oracle, x[:, :, perm], gy[:, :, perm], s, -128, 127, outer, c, inner)
    np.testing.assert_allclose(rp["acc"], r["acc"], rtol=1e-12, atol=1e-12)
    # channels are independent
    x2, gy2 = x.copy(), gy.copy()
    x2[:, 2, :] *= 1.7
    gy2[:, 2, :] += 1
    r2 = _bwd(oracle, x2, gy2, s, -128, 127, outer, c, inner)
    keep = [0, 1, 3]
    assert np.array_equal(r2["acc"][keep], r["acc"][keep]) and r2["acc"][2] != r["acc"][2]
    # the reduction runs over outer AND inner: equals the sum of per-slab calls
    per = np.zeros(c)
    for o in range(outer):
        for ch in range(c):
            per[ch] += _bwd(oracle, x[o, ch], gy[o, ch], s[ch:ch + 1], -128, 127, 1, 1, inner)["acc"][0]
    np.testing.assert_allclose(per, r["acc"], rtol=1e-12)


def test_scale_clamp_gates_theta_gradient(oracle):
    rng = np.random.default_rng(37)
    theta = np.array([-6.0, 0.0, 6.0], np.float32)
    s, active = oracle.scale(theta, s_min=0.05, s_max=2.0)
    assert list(active) == [1, 0, 1]
    x = rng.standard_normal((1, 3, 200)).astype(np.float32)
    gy = rng.standard_normal((1, 3, 200)).astype(np.float32)
    r = oracle.backward(x, gy, s, theta, active, -128, 127, 1, 3, 200)
    assert r["gtheta"][0] == 0 and r["gtheta"][2] == 0
    assert r["gtheta"][1] == np.float32(r["acc"][1] * 0.5)       # sigmoid(0) = 1/2
    assert np.all(r["gs"] == r["acc"].astype(np.float32))


def test_threads_change_nothing(oracle):
    """The benchmark's all-cores baseline splits channels over threads: every output must have the
    same bits as with one thread (each channel's sum is still one thread's sequential sum)."""
    rng = np.random.Generator(np.random.Philox(4242))
    outer, channels, inner = 3, 37, 501
    for dtype in (np.float16, np.float32):
        x = (rng.standard_normal((outer, channels, inner)) * 3).astype(dtype)
        gy = rng.standard_normal(x.shape).astype(dtype)
        theta = rng.uniform(-4, -2, channels).astype(np.float32)
        s, active = oracle.scale(theta)
        ref = None
        for threads in (1, 4, 7):
            assert oracle.set_threads(threads) == threads
            y, q = oracle.forward(x, s, -128, 127, outer, channels, inner)
            r = oracle.backward(x, gy, s, theta, active, -128, 127, outer, channels, inner)
            got = [y.view(np.uint8), q, r["gx"].view(np.uint8), r["acc"].view(np.uint64), r["aabs"].view(np.uint64),
                   r["gs"].view(np.uint32), r["gtheta"].view(np.uint32)]
            if ref is None:
                ref = got
            for a, b in zip(ref, got):
                assert np.array_equal(a, b)
        oracle.set_threads(1)
