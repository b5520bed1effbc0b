"""Pins for the oracle's binary16 conversions: numpy's float16 is the library reference."""
import numpy as np

import oracle


def test_f16_to_f64_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.f16_bits_to_f64(int(b)) for b in bits])
    both_nan = np.isnan(want) & np.isnan(got)
    assert np.all((want == got) | both_nan)
    assert np.all(np.signbit(want) == np.signbit(got))


def test_f64_to_f16_round_trip_is_identity():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = bits.view(np.float16).astype(np.float64)
    for b, v in zip(bits, vals):
        if np.isnan(v):
            continue
        assert oracle.f64_to_f16_bits(float(v)) == int(b)


def test_f64_to_f16_matches_numpy_on_random_and_tie_values():
    rng = np.random.default_rng(7)
    vals = [rng.standard_normal(20000) * s for s in (1e-8, 1e-6, 1e-4, 1e-2, 1.0, 300.0, 7e4)]
    # exact ties and their neighbours between every pair of adjacent positive halves
    hb = np.arange(0, 0x7c00, dtype=np.uint16)
    lo = hb.view(np.float16).astype(np.float64)
    hi = (hb + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    hi[-1] = 65536.0  # the value "after" the largest finite half, for the overflow tie
    mid = (lo + hi) / 2
    vals += [mid, -mid, np.nextafter(mid, 0), np.nextafter(mid, np.inf), np.array([0.0, -0.0, 1e300, -1e300])]
    v = np.concatenate(vals)
    with np.errstate(over="ignore"):
        want = v.astype(np.float16).view(np.uint16)
    got = np.array([oracle.f64_to_f16_bits(float(x)) for x in v], dtype=np.uint16)
    assert np.array_equal(want, got)
