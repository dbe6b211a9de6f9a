"""The kernels form the quotient as (float)((double)x * RN64(1/s)) instead of the binary32
division x/s.  This checks the identity the kernel relies on with numpy's IEEE arithmetic: equal
bits for every tested pair whose quotient is a normal binary32 number, including pairs
constructed to sit as close to a rounding boundary as a quotient of two binary32 numbers can."""
import numpy as np


def _both(x, s):
    x, s = x.astype(np.float32), s.astype(np.float32)
    with np.errstate(all="ignore"):
        ref = x / s
        rd = np.float64(1.0) / s.astype(np.float64)
        got = (x.astype(np.float64) * rd).astype(np.float32)
    return ref, got


def _assert_same(ref, got):
    normal = np.isfinite(ref) & (np.abs(ref) >= np.finfo(np.float32).tiny)
    same = (ref.view(np.uint32) == got.view(np.uint32)) | (np.isnan(ref) & np.isnan(got))
    bad = np.nonzero(normal & ~same)[0]
    assert bad.size == 0, (bad[:5], ref[bad[:5]], got[bad[:5]])
    # outside the normal range: zero / subnormal quotients may differ by one subnormal ulp
    sub = ~normal & np.isfinite(ref)
    diff = np.abs(ref[sub].astype(np.float64) - got[sub].astype(np.float64))
    assert np.all(diff <= 2.0 ** -149)
    inf = np.isinf(ref)
    assert np.array_equal(ref[inf], got[inf])


def test_random_bit_patterns():
    rng = np.random.default_rng(1)
    for _ in range(4):
        x = rng.integers(0, 2 ** 32, 2_000_000, dtype=np.uint64).astype(np.uint32).view(np.float32)
        s = rng.integers(0x00800000, 0x7F800000, 2_000_000, dtype=np.uint64).astype(np.uint32).view(np.float32)
        _assert_same(*_both(x, s))


def test_fp16_inputs_and_typical_scales():
    rng = np.random.default_rng(2)
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16).astype(np.float32)
    for _ in range(40):
        s = np.float32(np.exp(rng.uniform(-12, 4)))
        _assert_same(*_both(h, np.full(h.shape, s, np.float32)))


def test_quotients_next_to_rounding_boundaries():
    """x = RN(s * m) for m a half-way point between consecutive binary32 numbers (and its two
    neighbours): the exact quotient x/s then lies within a few 2^-25 ulp of a rounding boundary,
    the hardest case for any division shortcut."""
    rng = np.random.default_rng(3)
    n = 1_000_000
    s = (rng.integers(0x3F000000, 0x40000000, n, dtype=np.uint64).astype(np.uint32)).view(np.float32)
    q = rng.integers(1 << 23, 1 << 24, n).astype(np.float64)            # 24-bit integers
    mid = (q + 0.5) * 2.0 ** rng.integers(-30, 8, n)                    # half-way points, scaled
    for delta in (0.0, 2.0 ** -30, -2.0 ** -30):
        x = (s.astype(np.float64) * mid * (1.0 + delta)).astype(np.float32)
        _assert_same(*_both(x, s))
    # scales with all-ones and power-of-two significands
    for sv in (np.float32(1.9999999), np.float32(0.99999994), np.float32(2.0 ** -7), np.float32(3.0)):
        x = rng.standard_normal(n).astype(np.float32) * np.float32(50)
        _assert_same(*_both(x, np.full(n, sv, np.float32)))


def test_special_values():
    x = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 3.4e38, -3.4e38, 1e-45, 65504.0], np.float32)
    for sv in (1.1754944e-38, 1e-30, 0.5, 3.0, 1e30, 3.4e38):
        ref, got = _both(x, np.full(x.shape, sv, np.float32))
        _assert_same(ref, got)
        assert np.array_equal(np.signbit(ref[:2]), np.signbit(got[:2]))
