"""Pins for the oracle's own binary16 <-> binary32 conversions: numpy's float16 is an
independent implementation of the same IEEE-754 format."""
import numpy as np


def test_half_to_float_all_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def _check_narrow(oracle, vals):
    vals = np.asarray(vals, dtype=np.float32)
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).view(np.uint16)
    got = np.array([oracle.float_to_half(v) for v in vals], dtype=np.uint16)
    nan = np.isnan(vals)
    assert np.all((got[nan] & 0x7c00) == 0x7c00) and np.all((got[nan] & 0x3ff) != 0)
    assert np.array_equal(got[~nan], ref[~nan])


def test_float_to_half_exact_values_roundtrip(oracle):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    h = bits.view(np.float16)
    keep = ~np.isnan(h)
    _check_narrow(oracle, h[keep].astype(np.float32))


def test_float_to_half_midpoints_and_neighbours(oracle):
    # every tie between two adjacent non-negative halfs, and the floats just around it
    bits = np.arange(0, 0x7c00, dtype=np.uint16)
    lo = bits.view(np.float16).astype(np.float64)
    hi = np.concatenate([lo[1:], [65536.0]])
    mid = ((lo + hi) / 2).astype(np.float32)          # exact: one extra bit
    vals = np.concatenate([mid, np.nextafter(mid, np.float32(np.inf)),
                           np.nextafter(mid, np.float32(-np.inf))])
    vals = np.concatenate([vals, -vals])
    _check_narrow(oracle, vals)


def test_float_to_half_random_bit_patterns(oracle):
    rng = np.random.default_rng(7)
    pat = rng.integers(0, 2**32, size=150_000, dtype=np.uint64).astype(np.uint32)
    _check_narrow(oracle, pat.view(np.float32))
    # concentrate on the binary16 range, where rounding is not trivially 0 or inf
    v = (rng.standard_normal(150_000) * np.exp(rng.uniform(-20, 11, 150_000))).astype(np.float32)
    _check_narrow(oracle, v)
    _check_narrow(oracle, [np.inf, -np.inf, 0.0, -0.0, 65504.0, 65519.99, 65520.0, 2.0**-24,
                           2.0**-25, np.nextafter(np.float32(2.0**-25), np.float32(1)), 1e-45])
