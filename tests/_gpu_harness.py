"""Shared helpers of the GPU parity tests: upload a seeded TensorCase, run the HIP path through
the C-ABI binding, run the CPU oracle on the same bytes, compare.

Bars (element by element):  scales bit-exact; integer codes q bit-exact; y within 1 ulp of the
I/O dtype (-0 == +0; in practice bit-exact); gx bit-exact; gs and gtheta within 1e-5 relative of
the oracle's binary64 sum.
"""
import sys

import numpy as np
import torch

from paper_2511_12653_amd import binding as fq
from oracle import fq_oracle

GS_RTOL = 1e-5
GUARD = 8
SENTINEL = -24576.0          # exactly representable in FP16 and FP32


def say(msg):
    print("[gpu-case] " + msg, flush=True)
    sys.stderr.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def ordered(a):
    """Map float bit patterns to integers whose difference is the distance in ulps (-0 == +0)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        b = a.view(np.uint16).astype(np.int64)
        sign, mag = b >> 15, b & 0x7FFF
    else:
        b = a.view(np.uint32).astype(np.int64)
        sign, mag = b >> 31, b & 0x7FFFFFFF
    return np.where(sign == 1, -mag, mag)


def ulp_distance(a, b):
    nan_a, nan_b = np.isnan(a), np.isnan(b)
    assert np.array_equal(nan_a, nan_b), "NaN positions differ"
    d = np.abs(ordered(a) - ordered(b))
    d[nan_a] = 0
    return d


class DeviceCase:
    """Device buffers + descriptor for one TensorCase."""

    def __init__(self, case, want_q=True, flags=0, inplace=False, misalign=0, want_s=True):
        self.case = case
        n = case.numel
        tdt = torch.float16 if case.x.dtype == np.float16 else torch.float32

        self._guards = []

        def buf(src=None):
            # `misalign` elements of slack in front (base pointers off the 16-byte grid) and eight
            # behind; both are filled with a sentinel that check_guards() looks for afterwards
            t = torch.full((n + misalign + GUARD,), SENTINEL, dtype=tdt, device="cuda")
            v = t[misalign:misalign + n]
            if src is not None:
                v.copy_(dev(src.reshape(-1)))
            self._guards.append((t, misalign, n))
            return v

        self.x = buf(case.x)
        self.y = self.x if inplace else buf()
        self.q = torch.empty(n, dtype=torch.int8, device="cuda") if want_q else None
        self.theta = dev(case.theta)
        c = case.channels
        self.s = torch.full((c,), float("nan"), dtype=torch.float32, device="cuda") if want_s else None
        self.gy = buf(case.gy) if case.gy is not None else None
        self.gx = None
        if case.gy is not None and not (flags & fq.FQ_FLAG_NO_DX):
            self.gx = self.gy if inplace else buf()
        self.gs = torch.full((c,), float("nan"), dtype=torch.float32, device="cuda")
        self.gtheta = torch.full((c,), float("nan"), dtype=torch.float32, device="cuda")
        self.desc = fq.FqTensor.from_torch(
            case.outer, case.channels, case.inner, case.qmin, case.qmax, x=self.x, y=self.y,
            q=self.q, theta=self.theta, s=self.s, gy=self.gy, gx=self.gx, gs=self.gs,
            gtheta=self.gtheta, eps=case.eps, s_min=case.s_min, s_max=case.s_max,
            flags=flags | case.flags,
            dtype=fq.FQ_F16 if case.x.dtype == np.float16 else fq.FQ_F32)

    def check_guards(self, label=""):
        """Nothing may be written outside [base, base + numel)."""
        for t, front, n in self._guards:
            assert bool(torch.all(t[:front] == SENTINEL)) and bool(torch.all(t[front + n:] == SENTINEL)), \
                label + ": wrote outside a tensor"

    def host(self, name):
        t = getattr(self, name)
        return None if t is None else t.cpu().numpy()


def workspace_for(descs, mode):
    nbytes = fq.fq_workspace_bytes(descs, mode)
    assert nbytes > 0
    return torch.zeros(nbytes // 4, dtype=torch.int32, device="cuda")


def oracle_forward(case):
    s, active = fq_oracle.scale(case.theta, case.eps, case.s_min, case.s_max)
    y, q = fq_oracle.forward(case.x, s, case.qmin, case.qmax, case.outer, case.channels, case.inner)
    return s, active, y.reshape(-1), q.reshape(-1)


def oracle_backward(case, s, active, want_gx=True):
    return fq_oracle.backward(case.x, case.gy, s, case.theta, active, case.qmin, case.qmax,
                              case.outer, case.channels, case.inner, want_gx=want_gx)


def check_forward(dc, ref=None, label=""):
    case = dc.case
    dc.check_guards(label)
    s, active, y, q = ref if ref is not None else oracle_forward(case)
    if dc.s is not None and case.channels:
        gs_ = dc.host("s")
        if not np.array_equal(gs_.view(np.uint32), s.view(np.uint32)):
            bad = np.nonzero(gs_.view(np.uint32) != s.view(np.uint32))[0]
            c = int(bad[0])
            # Both sides evaluate softplus in binary64 (each within a few ulp of binary64) and round to
            # binary32 once, so they can differ by one binary32 ulp only where the exact value lies
            # within ~1e-15 relative of a rounding boundary: about once in 1e8 channels.  Anything
            # else is a bug; say which it looks like.
            ulps = int(abs(int(ordered(gs_[c:c + 1])[0]) - int(ordered(s[c:c + 1])[0])))
            raise AssertionError("%s: scales differ in %d channel(s); channel %d: theta=%r gpu=%r oracle=%r (%d ulp)%s" % (
                label, bad.size, c, float(case.theta[c]), float(gs_[c]), float(s[c]), ulps,
                ": a one-ulp difference in one channel can be a binary64 rounding coincidence (reseed the case); "
                "several channels or more ulps cannot" if ulps == 1 and bad.size == 1 else ""))
    if case.numel == 0:
        return
    gy_ = dc.host("y").reshape(-1)
    d = ulp_distance(gy_, y)
    assert d.max() <= 1, "%s: y differs by %d ulp at %d" % (label, d.max(), int(d.argmax()))
    if dc.q is not None:
        gq = dc.host("q").astype(np.int32)
        bad = np.nonzero(gq != q)[0]
        assert bad.size == 0, "%s: %d codes differ, first at %d (%d vs %d)" % (
            label, bad.size, bad[0], gq[bad[0]], q[bad[0]])
    return dict(y_exact=bool((d == 0).all()))


def check_backward(dc, s, active, label="", want_gx=True):
    case = dc.case
    dc.check_guards(label)
    r = oracle_backward(case, s, active, want_gx=want_gx)
    if want_gx and case.numel:
        ggx = dc.host("gx").reshape(-1)
        ref = r["gx"].reshape(-1)
        it = np.uint16 if ref.dtype == np.float16 else np.uint32
        bad = np.nonzero(ggx.view(it) != ref.view(it))[0]
        assert bad.size == 0, "%s: %d gx words differ, first at %d" % (label, bad.size, bad[0])
    if case.channels == 0:
        return r
    for name, ref in (("gs", r["acc"]), ("gtheta", r["gtheta"].astype(np.float64))):
        got = dc.host(name).astype(np.float64)
        if name == "gtheta":
            # reference in binary64: acc * sigmoid(theta), 0 where the scale clamp is active
            sig = 1.0 / (1.0 + np.exp(-case.theta.astype(np.float64)))
            ref = np.where(active == 1, 0.0, r["acc"] * sig)
        nan = np.isnan(ref)
        assert np.array_equal(np.isnan(got), nan), label + ": NaN channels differ in " + name
        err = np.abs(got - ref)[~nan]
        tol = GS_RTOL * np.abs(ref)[~nan] + 1e-30
        worst = int(np.argmax(err - tol)) if err.size else 0
        assert np.all(err <= tol), "%s: %s off by %.3e (tol %.3e) in channel %d, cond %.1f" % (
            label, name, err[worst], tol[worst], worst,
            r["aabs"][~nan][worst] / max(abs(r["acc"][~nan][worst]), 1e-300))
    return r
