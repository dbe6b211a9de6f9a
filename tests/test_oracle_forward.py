"""Pins for the oracle's forward pass, Eq. (5): y = s * round(clip(x/s, qmin, qmax)).

None of these tests retype the oracle: they use hand-worked values (tests/golden/), exact
rational arithmetic, numpy / torch library routines and properties the definition implies.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _table(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([float(t) for t in line.split()])
    return np.array(rows, dtype=np.float64)


def _bits(a):
    a = np.ascontiguousarray(a)
    return a.view(np.uint16 if a.dtype == np.float16 else np.uint32)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_table_T(oracle, dtype):
    t = _table("table_T.txt")
    x = t[:, 0].astype(dtype)
    s = np.array([0.5], np.float32)
    y, q = oracle.forward(x, s, -128, 127, 1, 1, x.size)
    assert np.array_equal(q, t[:, 2].astype(np.int32))
    assert np.array_equal(_bits(y), _bits(t[:, 3].astype(dtype)))      # includes the -0.0
    # the paper's symmetric range, Eq. (5)-(6): [-127, 127]
    y, q = oracle.forward(x, s, -127, 127, 1, 1, x.size)
    assert list(q[-2:]) == [-127, -127] and list(y[-2:]) == [-63.5, -63.5]
    assert np.array_equal(q[:-2], t[:-2, 2].astype(np.int32))


def test_table_4bit(oracle):
    t = _table("table_4bit.txt")
    y, q = oracle.forward(t[:, 0].astype(np.float32), np.ones(1, np.float32), -8, 7, 1, 1, len(t))
    assert np.array_equal(q, t[:, 1].astype(np.int32))
    assert np.array_equal(y, t[:, 2].astype(np.float32))


def _round_half_even(fr: Fraction) -> int:
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


def test_brute_force_exact_rationals(oracle):
    """Tiny inputs, each step carried out on exact rationals: the binary32 quotient (numpy's
    IEEE divide) is clipped and rounded half-to-even as a Fraction, the product q*s is formed
    exactly and rounded to binary32 once by numpy."""
    rng = np.random.default_rng(3)
    s = np.array([0.0236], np.float32)
    x = np.concatenate([rng.standard_normal(300) * 1.2, (np.arange(-140, 141) + 0.5) * float(s[0]),
                        np.arange(-140, 141) * float(s[0]), [3.2, -3.3, 1e-30, -1e-30]]
                       ).astype(np.float32)
    y, q = oracle.forward(x, s, -128, 127, 1, 1, x.size)
    for xi, yi, qi in zip(x, y, q):
        v = Fraction(float(np.float32(xi) / s[0]))
        code = _round_half_even(min(max(v, Fraction(-128)), Fraction(127)))
        assert qi == code
        want = np.float32(float(Fraction(code) * Fraction(float(s[0]))))   # exact, then one RNE
        assert yi == want


@pytest.mark.parametrize("qmin,qmax", [(-128, 127), (-127, 127), (-8, 7)])
def test_clip_round_order_is_immaterial(oracle, qmin, qmax):
    """round(clip(v)) == clip(round(v)) for integer bounds; the right-hand side is evaluated
    with numpy library calls."""
    rng = np.random.default_rng(5)
    s = np.array([0.0371], np.float32)
    x = (rng.standard_normal(200_000) * 2.0).astype(np.float32)
    x[:4000] = (np.linspace(qmin - 3, qmax + 3, 4000) * s[0]).astype(np.float32)
    y, q = oracle.forward(x, s, qmin, qmax, 1, 1, x.size)
    ref_q = np.clip(np.rint(x / s[0]), qmin, qmax)
    assert np.array_equal(q, ref_q.astype(np.int32))
    assert np.array_equal(y, (ref_q * s[0]).astype(np.float32))


def test_invariants(oracle):
    rng = np.random.default_rng(9)
    c, inner, outer = 5, 777, 3
    s = rng.uniform(0.01, 0.2, c).astype(np.float32)
    x = (rng.standard_normal((outer, c, inner)) * 4).astype(np.float32)
    y, q = oracle.forward(x, s, -128, 127, outer, c, inner)
    assert q.min() >= -128 and q.max() <= 127
    assert np.array_equal(y, q.astype(np.float32) * s[None, :, None])      # y == s*q exactly
    v = x / s[None, :, None]
    inside = (v >= -128) & (v <= 127)
    assert np.all(np.abs(y - x)[inside] <= (0.5 * s[None, :, None] * (1 + 1e-6) + 0 * x)[inside])
    # monotone in x within a channel
    for ch in range(c):
        xs = np.sort(x[:, ch, :].reshape(-1))
        _, qs = oracle.forward(xs, s[ch:ch + 1], -128, 127, 1, 1, xs.size)
        assert np.all(np.diff(qs) >= 0)
    # odd symmetry for a symmetric range
    yp, qp = oracle.forward(x, s, -127, 127, outer, c, inner)
    yn, qn = oracle.forward(-x, s, -127, 127, outer, c, inner)
    assert np.array_equal(qp, -qn) and np.array_equal(yp, -yn)


def test_per_channel_layout(oracle):
    """[outer, C, inner] indexing: each (o, c) slab must equal a per-tensor call with s[c]."""
    rng = np.random.default_rng(13)
    outer, c, inner = 4, 7, 33
    s = rng.uniform(0.02, 0.5, c).astype(np.float32)
    x = rng.standard_normal((outer, c, inner)).astype(np.float32) * 3
    y, q = oracle.forward(x, s, -8, 7, outer, c, inner)
    ref = np.clip(np.rint(x / s[None, :, None]), -8, 7)
    assert np.array_equal(q, ref.astype(np.int32))
    # a transposed operand (treating the tensor as [C, outer, inner]) must NOT match
    bad = np.clip(np.rint(x / s[np.arange(outer * c) // outer % c].reshape(outer, c, 1)), -8, 7)
    assert not np.array_equal(ref, bad)


def test_fp16_all_finite_values(oracle):
    """Every finite binary16 input for several scales; reference via numpy float32 math and
    numpy's own float16 narrowing."""
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    h = h[np.isfinite(h)]
    assert h.size == 63488
    for sv in [2.0 ** -6, 0.0236, 0.9740769863128662, 1.0 / 127, 3.0]:
        s = np.array([sv], np.float32)
        y, q = oracle.forward(h, s, -128, 127, 1, 1, h.size)
        ref_q = np.rint(np.clip(h.astype(np.float32) / s[0], -128, 127))
        assert np.array_equal(q, ref_q.astype(np.int32))
        ref_y = (ref_q * s[0]).astype(np.float32).astype(np.float16)
        assert np.array_equal(_bits(y), _bits(ref_y))


def test_idempotent_inside_safe_domain(oracle):
    """fq(fq(x)) == fq(x) when y neither overflows nor goes subnormal in the I/O dtype."""
    rng = np.random.default_rng(17)
    for dtype, scales in [(np.float32, [1e-3, 0.0236, 0.77, 12.5]), (np.float16, [2.0 ** -9, 0.0236, 0.77, 100.0])]:
        for sv in scales:
            s = np.array([sv], np.float32)
            x = (rng.standard_normal(50_000) * 60 * sv).astype(dtype)
            y1, q1 = oracle.forward(x, s, -128, 127, 1, 1, x.size)
            y2, q2 = oracle.forward(y1, s, -128, 127, 1, 1, x.size)
            assert np.array_equal(q1, q2) and np.array_equal(_bits(y1), _bits(y2))


def test_torch_fake_quantize_almost_everywhere(oracle):
    """torch.fake_quantize_per_channel_affine (zero_point 0) documents the same function; it may
    use a reciprocal multiply, so disagreement is tolerated only within an ulp of a rounding tie
    or a clip edge."""
    import torch
    rng = np.random.default_rng(19)
    c, inner = 6, 4000
    s = rng.uniform(0.01, 0.3, c).astype(np.float32)
    x = (rng.standard_normal((1, c, inner)) * 5).astype(np.float32)
    y, q = oracle.forward(x, s, -128, 127, 1, c, inner)
    ty = torch.fake_quantize_per_channel_affine(torch.from_numpy(x), torch.from_numpy(s),
                                                torch.zeros(c, dtype=torch.int32), 1, -128, 127).numpy()
    diff = y != ty
    assert diff.mean() < 1e-3
    v = (x.astype(np.float64) / s[None, :, None].astype(np.float64))[diff]
    frac = np.abs(v - np.floor(v) - 0.5)
    assert np.all(frac < 1e-4)


def test_non_finite_inputs(oracle):
    x = np.array([np.inf, -np.inf, np.nan, 1.0], np.float32)
    y, q = oracle.forward(x, np.array([0.5], np.float32), -128, 127, 1, 1, 4)
    assert list(q) == [127, -128, 0, 2]
    assert y[0] == 63.5 and y[1] == -64.0 and np.isnan(y[2]) and y[3] == 1.0
