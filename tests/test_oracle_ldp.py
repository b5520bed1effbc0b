"""Pins for the oracle's LDP grid, index assignment and packing (Section 4.3)."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import rcp_synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _f16(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def _golden_uniform():
    vals = {}
    with open(os.path.join(GOLDEN, "ldp_uniform_init.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, num, den = line.split()
            vals[name] = Fraction(int(num), int(den))
    return vals


@pytest.mark.parametrize("lo,hi", [(0.0, 1.0), (-3.0, 3.0), (-0.046875, 0.0546875)])
def test_uniform_initial_point_matches_the_paper(lo, hi):
    g = _golden_uniform()
    p = [np.float32(float(g[k])) for k in ("p1", "p2", "p3")]
    T, L = oracle.ldp_grid(lo, hi, *p)
    rng_ = hi - lo
    for i, name in enumerate(("t1", "t2", "t3")):
        assert abs(float(T[i]) - (lo + rng_ * float(g[name]))) <= 2e-7 * max(1.0, abs(rng_))
    want = np.array([lo + rng_ * float(g[k]) for k in ("w0", "w1", "w2", "w3")])
    assert np.array_equal(L, want.astype(np.float16).view(np.uint16))


def test_grid_closed_forms_and_ordering():
    rng = np.random.default_rng(0)
    part = rcp_synth.partitions(0, "closed", 500)
    for h in range(500):
        lo = np.float32(-abs(rng.standard_normal()) - 0.5)
        hi = np.float32(abs(rng.standard_normal()) + 0.5)
        p1, p2, p3 = (float(v) for v in part[h])
        T, L = oracle.ldp_grid(lo, hi, p1, p2, p3)
        r = float(hi) - float(lo)
        t = np.array([p1 / 2, p1 + p2 / 2, (p1 + p2 + p3) - p3 / 2])  # centres of the partitions
        np.testing.assert_allclose(T, float(lo) + r * t, rtol=0, atol=3e-7 * r)
        w = np.array([0.0, (t[0] + t[1]) / 2, (t[1] + t[2]) / 2, 1.0])
        lv = _f16(L)
        np.testing.assert_allclose(lv, float(lo) + r * w, rtol=0, atol=2.0 ** -11 * max(abs(lo), abs(hi)))
        assert lv[0] == np.float64(np.float16(lo)) and lv[3] == np.float64(np.float16(hi))
        assert lv[0] < lv[1] < lv[2] < lv[3]                      # monotone inside [lo, hi]
        assert T[0] < T[1] < T[2]
        exact = float(lo) + r * w                                  # interior level inside its own bin
        assert T[0] < exact[1] < T[1] < exact[2] < T[2]


def test_step_function_takes_the_upper_bin_at_a_grid_point():
    # p = (1/2, 1/4, 1/4), range [0, 1]: t = (0.25, 0.625, 0.875), all exact in binary
    N, K = 4, 32
    W = np.zeros((N, K), dtype=np.float32)
    W[0, :8] = [0.25, np.nextafter(np.float32(0.25), np.float32(0)), 0.625, 0.62, 0.875, 0.87, -5.0, 5.0]
    lo, hi = np.zeros(N, np.float32), np.ones(N, np.float32)
    part = np.tile(np.array([0.5, 0.25, 0.25], np.float32), (N, 1))
    _, cb, idx = oracle.pack_weights(W, lo, hi, part, want_idx=True)
    assert list(idx[0, :8]) == [1, 0, 2, 1, 3, 2, 0, 3]
    np.testing.assert_array_equal(_f16(cb[0]), [0.0, (0.25 + 0.625) / 2, (0.625 + 0.875) / 2, 1.0])


def test_uniform_point_reduces_to_the_2bit_asymmetric_integer_quantizer():
    """Eqn. 1 with N = 2: Q(W) = clip(round(W/s) + z, 0, 3), s = range/3, z = -min/s.
    The range is chosen with min/s an integer so that the zero point is exact."""
    N, K = 8, 4096
    s = 2.0 ** -6
    lo_v, hi_v = -5 * s, -5 * s + 3 * s
    rng = np.random.default_rng(3)
    W = (rng.uniform(lo_v - s, hi_v + s, size=(N, K))).astype(np.float16).astype(np.float32)
    lo, hi = np.full(N, lo_v, np.float32), np.full(N, hi_v, np.float32)
    part = np.full((N, 3), 1.0 / 3.0, dtype=np.float32)
    _, cb, idx = oracle.pack_weights(W, lo, hi, part, want_idx=True)
    x = W.astype(np.float64) / s
    textbook = np.clip(np.rint(x) + 5, 0, 3)
    off_tie = np.abs((x - np.floor(x)) - 0.5) > 1e-4
    assert off_tie.mean() > 0.9
    assert np.array_equal(idx[off_tie], textbook[off_tie].astype(np.uint8))
    np.testing.assert_allclose(_f16(cb), np.tile(lo_v + s * np.arange(4), (N, 1)), atol=2.0 ** -11 * 0.1)


def test_indices_are_searchsorted_of_the_thresholds_and_fill_every_level():
    W, lo, hi, part = rcp_synth.linear_layer(0, "tiny", 256, 512)
    packed, cb, idx = oracle.pack_weights(W.astype(np.float32), lo, hi, part, want_idx=True)
    for h in range(0, 256, 5):
        T, L = oracle.ldp_grid(lo[h], hi[h], *part[h])
        want = np.searchsorted(T, W[h].astype(np.float32), side="right")
        assert np.array_equal(idx[h], want.astype(np.uint8))
        assert np.array_equal(cb[h], L)
        counts = np.bincount(idx[h], minlength=4)
        assert counts[0] >= 5 and counts[3] >= 5  # 1 % of 512 lies beyond each clip value
    assert packed.size == 256 * 512 // 4


def test_pack_unpack_round_trip_and_dequantised_levels():
    N, K = 36, 160
    idx = rcp_synth.random_indices(2, "rt", N, K)
    packed = oracle.pack_indices(idx)
    assert packed.dtype == np.uint8 and packed.size == N * K // 4
    assert np.array_equal(oracle.unpack_indices(packed, N, K), idx)
    W, lo, hi, part = rcp_synth.linear_layer(2, "rt", N, K)
    packed, cb, idx = oracle.pack_weights(W.astype(np.float32), lo, hi, part, want_idx=True)
    unpacked = oracle.unpack_indices(packed, N, K)
    assert np.array_equal(unpacked, idx)
    levels = _f16(cb)
    assert np.array_equal(np.take_along_axis(levels, unpacked.astype(np.int64), axis=1),
                          np.take_along_axis(levels, idx.astype(np.int64), axis=1))


def test_packed_layout_follows_the_written_bit_positions():
    """One index set at (h, k) lights exactly the documented bits: cell (h/4, k/8) at byte
    8*((h/4)*(K/8) + k/8), word 0 = low index bit, word 1 = high bit, bit 4*(k%8) + h%4."""
    N, K = 12, 96
    for h, k, v in [(0, 0, 1), (5, 17, 2), (11, 95, 3), (6, 40, 3), (3, 7, 1)]:
        idx = np.zeros((N, K), dtype=np.uint8)
        idx[h, k] = v
        words = oracle.pack_indices(idx).view("<u4").reshape(N // 4, K // 8, 2)
        want = np.zeros_like(words)
        bit = np.uint32(1) << np.uint32(4 * (k % 8) + h % 4)
        if v & 1:
            want[h // 4, k // 8, 0] = bit
        if v & 2:
            want[h // 4, k // 8, 1] = bit
        assert np.array_equal(words, want)


def test_buffer_sizes_match_the_paper_shapes():
    with open(os.path.join(GOLDEN, "gemv_shapes.txt")) as f:
        rows = [list(map(int, l.split())) for l in f if l.strip() and not l.startswith("#")]
    for C, H, wq, lut, xq, out in rows:
        assert wq == H * C // 4 and lut == H * 4 * 2 and xq == C // 2 and out == H * 2
    idx = rcp_synth.random_indices(0, "sz", 8, 64)
    assert oracle.pack_indices(idx).nbytes == 8 * 64 // 4


def test_shape_errors():
    with pytest.raises(RuntimeError):
        oracle.pack_indices(np.zeros((6, 32), np.uint8))
    with pytest.raises(RuntimeError):
        oracle.pack_indices(np.zeros((8, 24), np.uint8))
