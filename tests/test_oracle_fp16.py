"""Pins for the oracle's fp16 conversions: numpy's IEEE binary16 is the
independent reference (a library routine, not the oracle's own formula)."""
import numpy as np


def test_half_to_real_all_bit_patterns(orc):
    bits = np.arange(65536, dtype=np.uint16)
    h = bits.view(np.float16)
    got = orc.half_to_real(h)
    want = h.astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_real_to_half_round_trip_is_identity(orc):
    bits = np.arange(65536, dtype=np.uint16)
    h = bits.view(np.float16)
    ok = ~np.isnan(h)
    back = orc.real_to_half(h.astype(np.float64))
    assert np.array_equal(back.view(np.uint16)[ok], bits[ok])


def test_real_to_half_matches_numpy_rne(orc):
    rng = np.random.default_rng(7)
    vals = np.concatenate([
        rng.standard_normal(200000) * 10.0 ** rng.integers(-9, 6, 200000),
        # exact midpoints between neighbouring halves (ties) and their neighbours
        *[(np.arange(65535, dtype=np.uint16)[:31743].view(np.float16).astype(np.float64)
           + np.arange(1, 31744, dtype=np.uint16).view(np.float16).astype(np.float64)) / 2 * s
          for s in (1.0, -1.0)],
        np.array([0.0, -0.0, 65504.0, 65519.999, 65520.0, 65536.0, 1e9, -1e9, np.inf, -np.inf,
                  2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0000001, 2.0 ** -26, 6.1e-5, 6.104e-5]),
    ])
    got = orc.real_to_half(vals).view(np.uint16)
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)
    assert np.array_equal(got, want)
    assert orc.real_to_half(np.array([np.nan])).view(np.uint16)[0] & 0x7c00 == 0x7c00


def test_f32_variant_conversions(orc32):
    rng = np.random.default_rng(8)
    v = (rng.standard_normal(50000) * 30).astype(np.float32)
    assert np.array_equal(orc32.real_to_half(v).view(np.uint16), v.astype(np.float16).view(np.uint16))
