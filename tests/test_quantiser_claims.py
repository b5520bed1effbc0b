"""Host-side pin of the arithmetic claim behind the quantiser that the fused prologues apply to 16-bit activations
(paper: Appendix table of quantisation configurations, per-token symmetric int4 activations; q = clamp(round(y / S))).

The kernels do not divide: they take q0 = y * (1/S), one Newton step q1 = q0 + (y - q0 S) (1/S) with fused multiply-adds,
and round q1.  The claim is that for y with at most 11 significant bits (fp16, bf16) and S an fp16 number this gives, after
clamping, exactly the integer that rounding the correctly rounded binary32 quotient y / S gives -- ties included -- and that
a reciprocal that is off by one unit in the last place does not change that.  The check below evaluates both sides with
numpy on every finite fp16 input (and a dense sample of bf16 inputs) for several hundred scales.  The fused multiply-adds
are evaluated in binary64, where the products and the first sum are exact.
"""
import numpy as np
import pytest


def _fma32(a, b, c):
    """Binary32 fused multiply-add of binary32 arrays, through binary64 (exact product; see the module text)."""
    return (a.astype(np.float64) * b.astype(np.float64) + c.astype(np.float64)).astype(np.float32)


def _kernel_side(y, s, rs):
    q0 = (y * rs).astype(np.float32)
    q1 = _fma32(_fma32(-q0, np.float32(s), y), np.float32(rs), q0)
    return np.clip(np.rint(q1), -8, 7).astype(np.int32)


def _definition(y, s):
    return np.clip(np.rint((y / np.float32(s)).astype(np.float32)), -8, 7).astype(np.int32)


def _scales():
    rng = np.random.default_rng(20250215)
    bits = np.concatenate([rng.integers(1, 0x7C00, size=300, dtype=np.int64),        # anywhere, subnormals included
                           rng.integers(0x2C00, 0x4400, size=200, dtype=np.int64),    # around the scales of real layers
                           np.array([1, 2, 0x03FF, 0x0400, 0x3400, 0x3C00, 0x3C01, 0x3BFF, 0x7BFF], dtype=np.int64)])
    return bits.astype(np.uint16).view(np.float16).astype(np.float32)


@pytest.mark.parametrize("ulp", [0, -1, 1])
def test_newton_step_quotient_rounds_like_the_division_for_fp16_inputs(ulp):
    allbits = np.arange(0x10000, dtype=np.uint32).astype(np.uint16)
    y_all = allbits.view(np.float16)
    y_all = y_all[np.isfinite(y_all)].astype(np.float32)
    ties = 0
    for s in _scales():
        y = y_all[np.abs(y_all) <= np.float32(40.0) * s]       # beyond that both sides clamp to the same end
        rs = np.float32(1.0) / np.float32(s)
        if ulp:
            rs = np.nextafter(rs, np.float32(np.inf) if ulp > 0 else np.float32(0.0), dtype=np.float32)
        got, want = _kernel_side(y, s, rs), _definition(y, s)
        assert np.array_equal(got, want), (float(s), y[got != want][:4])
        t = y.astype(np.float64) / np.float64(s)
        ties += int(np.count_nonzero((np.abs(t) < 8.5) & (np.abs(t - np.floor(t)) == 0.5)))
    assert ties > 1000       # the sweep really does sit on rounding ties, a couple of thousand times


def test_newton_step_quotient_rounds_like_the_division_for_bf16_inputs():
    rng = np.random.default_rng(7)
    # bf16 numbers: the upper 16 bits of a binary32; a dense sample over the exponents that matter plus every mantissa
    hi = np.concatenate([rng.integers(0x3000, 0x4800, size=200000, dtype=np.int64),
                         (np.arange(0x3800, 0x4400, dtype=np.int64))])
    hi = np.concatenate([hi, hi | 0x8000])
    y_all = (hi.astype(np.uint32) << 16).view(np.float32)
    for s in _scales()[300:]:
        y = y_all[np.abs(y_all) <= np.float32(40.0) * s]
        rs = np.float32(1.0) / np.float32(s)
        for r in (rs, np.nextafter(rs, np.float32(0.0), dtype=np.float32), np.nextafter(rs, np.float32(np.inf), dtype=np.float32)):
            got, want = _kernel_side(y, s, r), _definition(y, s)
            assert np.array_equal(got, want), (float(s), y[got != want][:4])


def test_plain_reciprocal_product_does_not_round_like_the_division():
    """The pin has teeth: without the Newton step the product y * (1/S) lands on the wrong side of some ties."""
    allbits = np.arange(0x10000, dtype=np.uint32).astype(np.uint16)
    y_all = allbits.view(np.float16)
    y_all = y_all[np.isfinite(y_all)].astype(np.float32)
    wrong = 0
    for s in _scales()[300:400]:
        y = y_all[np.abs(y_all) <= np.float32(40.0) * s]
        rs = np.float32(1.0) / np.float32(s)
        plain = np.clip(np.rint((y * rs).astype(np.float32)), -8, 7).astype(np.int32)
        wrong += int(np.count_nonzero(plain != _definition(y, s)))
    assert wrong > 0
