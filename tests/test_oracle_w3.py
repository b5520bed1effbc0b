"""Pins for the oracle's 3-bit variant: LDP applied to the asymmetric normal-float format
(Section 4.3, paragraph on the NF3 format: centre point, the two scales, the rounding rule and
"multiply the scale back and add the centre") and the GEMV of Section 4.4 with an eight-entry
LUT per output channel."""
import numpy as np
import pytest

import oracle
import rcp_synth


def _f16(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def _levels64(lo, hi, p, grid):
    """The eight levels in float64, from the paragraph's own quantities."""
    lo, hi, p = float(np.float32(lo)), float(np.float32(hi)), float(np.float32(p))
    c = lo + (hi - lo) * p
    s_neg, s_pos = abs(c - lo), abs(hi - c)
    return np.array([c + (s_neg if g < 0 else s_pos) * float(g) for g in np.asarray(grid, np.float32)]), c, s_neg, s_pos


def test_levels_span_the_clip_range_and_hold_the_centre():
    grid = rcp_synth.normal_quantile_grid()
    assert grid[0] == -1 and grid[7] == 1 and grid[3] == 0 and np.all(np.diff(grid) > 0)
    rng = np.random.default_rng(5)
    for _ in range(50):
        lo, hi = np.float32(-rng.random() - 0.01), np.float32(rng.random() + 0.01)
        p = np.float32(rng.uniform(0.05, 0.95))
        T, L = oracle.w3_grid(lo, hi, p, grid)
        Lf = _f16(L)
        c = float(lo) + (float(hi) - float(lo)) * float(p)
        # the ends are the clip values, the level at grid value 0 is the centre (each within one fp16 rounding)
        assert abs(Lf[0] - float(lo)) <= 2.0 ** -11 * abs(float(lo)) + 2.0 ** -25
        assert abs(Lf[7] - float(hi)) <= 2.0 ** -11 * abs(float(hi)) + 2.0 ** -25
        assert abs(Lf[3] - c) <= 2.0 ** -11 * abs(c) + 2.0 ** -25
        assert np.all(np.diff(Lf) >= 0)
        assert np.all(np.diff(T) > 0) and np.all(T > Lf[:-1] - 1e-6) and np.all(T < Lf[1:] + 1e-6)
        # the two sides have their own scale: level spacings follow the grid on each side
        L64, _, s_neg, s_pos = _levels64(lo, hi, p, grid)
        assert np.allclose(np.diff(L64[:4]), s_neg * np.diff(grid[:4].astype(np.float64)), rtol=1e-12, atol=0)
        assert np.allclose(np.diff(L64[3:]), s_pos * np.diff(grid[3:].astype(np.float64)), rtol=1e-12, atol=0)
        assert np.allclose(Lf, L64, rtol=2.0 ** -11, atol=2.0 ** -25)


def test_integer_grid_is_the_printed_rounding_rule():
    """With the integers -3..4 as the grid, the index is clip(round((w - c)/s_side)) + 3: the
    quantisation equation of the paragraph as printed (s_pos above the centre, s_neg otherwise)."""
    grid = np.arange(-3, 5, dtype=np.float32)
    rng = np.random.default_rng(11)
    N, K = 8, 256
    lo = -rng.uniform(0.05, 0.2, N).astype(np.float32)
    hi = rng.uniform(0.05, 0.2, N).astype(np.float32)
    p = rng.uniform(0.2, 0.8, N).astype(np.float32)
    W = (rng.standard_normal((N, K)) * 0.5).astype(np.float32)
    _, _, idx = oracle.pack_weights_w3(W, lo, hi, p, grid, want_idx=True)
    checked = 0
    for h in range(N):
        _, c, s_neg, s_pos = _levels64(lo[h], hi[h], p[h], grid)
        w = W[h].astype(np.float64)
        t = np.where(w > c, (w - c) / s_pos, (w - c) / s_neg)
        clear = np.abs(t - np.floor(t) - 0.5) > 1e-4          # away from exact ties
        want = np.clip(np.rint(t), -3, 4).astype(np.int64) + 3
        assert np.array_equal(idx[h][clear], want[clear])
        checked += int(clear.sum())
        assert set(np.unique(idx[h])) == set(range(8))      # both clipped ends and every step occur
    assert checked > 0.99 * N * K


@pytest.mark.parametrize("seed", [1, 2])
def test_index_is_the_nearest_level(seed):
    N, K = 16, 512
    W, lo, hi, p, grid = rcp_synth.linear_layer_w3(seed, "near", N, K)
    packed, cb, idx = oracle.pack_weights_w3(W, lo, hi, p, grid, want_idx=True)
    assert np.array_equal(oracle.unpack_indices_w3(packed, N, K), idx)
    for h in range(N):
        L64, _, _, _ = _levels64(lo[h], hi[h], p[h], grid)
        w = W[h].astype(np.float64)
        d = np.abs(w[:, None] - L64[None, :])
        order = np.sort(d, axis=1)
        clear = order[:, 1] - order[:, 0] > 1e-7
        assert np.array_equal(idx[h][clear], np.argmin(d, axis=1)[clear])
        # reconstruction error inside the clip range: at most half the widest gap
        inside = (w >= L64[0]) & (w <= L64[7])
        rec = L64[idx[h]]
        assert np.all(np.abs(rec - w)[inside] <= np.diff(L64).max() / 2 + 1e-9)
        assert np.array_equal(_f16(cb[h]), L64.astype(np.float16).astype(np.float64))
    assert len(np.unique(idx)) == 8


@pytest.mark.parametrize("N,K", [(4, 32), (8, 64), (4, 2048), (8, 2080), (4, 4096), (8, 11008)])
def test_layout_round_trip_and_structure(N, K):
    idx = rcp_synth.random_indices(3, f"w3:{K}", N, K, levels=8)
    packed = oracle.pack_indices_w3(idx)
    assert packed.size == 3 * N * K // 8
    assert np.array_equal(oracle.unpack_indices_w3(packed, N, K), idx)
    # every (row, column, plane) owns its own bit: all-ones indices fill the buffer
    assert np.all(oracle.pack_indices_w3(np.full((N, K), 7, np.uint8)) == 0xFF)
    # structure: a single index bit p at (h, k) sets exactly one bit; inside a block of units the
    # three planes of one unit are R*16 bytes apart, units 16 bytes apart, row groups 48*K/32 bytes
    U = K // 32
    rng = np.random.default_rng(K + N)
    for _ in range(8):
        h, k = int(rng.integers(N)), int(rng.integers(K))
        pos = []
        for p in range(3):
            one = np.zeros((N, K), np.uint8)
            one[h, k] = 1 << p
            b = np.unpackbits(oracle.pack_indices_w3(one), bitorder="little")
            assert b.sum() == 1
            pos.append(int(np.flatnonzero(b)[0]))
        u = k // 32
        R = min(64, U - 64 * (u // 64))
        assert pos[1] - pos[0] == 8 * 16 * R and pos[2] - pos[1] == 8 * 16 * R
        within = pos[0] - 8 * (48 * U * (h // 4) + 3072 * (u // 64) + 16 * (u % 64))
        assert within == 32 * ((k % 32) // 8) + 4 * (k % 8) + h % 4
    if K >= 64:
        one = np.zeros((N, K), np.uint8)
        one[0, 0] = 1
        two = np.zeros((N, K), np.uint8)
        two[0, 32] = 1
        a = np.flatnonzero(np.unpackbits(oracle.pack_indices_w3(one), bitorder="little"))[0]
        b = np.flatnonzero(np.unpackbits(oracle.pack_indices_w3(two), bitorder="little"))[0]
        assert b - a == 8 * 16
    if N >= 8:
        one = np.zeros((N, K), np.uint8)
        one[4, 0] = 1
        b = np.flatnonzero(np.unpackbits(oracle.pack_indices_w3(one), bitorder="little"))[0]
        assert b == 8 * 48 * U


@pytest.mark.parametrize("N,K", [(4, 32), (8, 256), (12, 2080), (8, 4096)])
def test_gemv_partial_sums_and_output(N, K):
    idx = rcp_synth.random_indices(4, f"w3g:{K}", N, K, levels=8)
    q = rcp_synth.random_int4(4, f"w3g:{K}", 1, K)
    rng = np.random.default_rng(K)
    lut = np.sort(rng.standard_normal((N, 8)).astype(np.float16), axis=1)
    cb = lut.view(np.uint16)
    y = q.astype(np.float32)
    xq, sc, q2 = oracle.quantize_act(y, 1.0)               # amax 8 or 7 -> the int4 codes need not equal q
    packed = oracle.pack_indices_w3(idx)
    out, P = oracle.w3a4_gemv(packed, cb, N, K, xq, sc)
    onehot = (idx[:, :, None] == np.arange(8)[None, None, :]).astype(np.int64)
    assert np.array_equal(P, np.einsum("hkl,k->hl", onehot, q2[0].astype(np.int64)))
    assert np.array_equal(P.sum(axis=1), np.full(N, int(q2[0].astype(np.int64).sum())))
    S = float(_f16(sc)[0])
    dense = np.take_along_axis(lut.astype(np.float64), idx.astype(np.int64), axis=1)      # N x K dequantised weights
    want = dense @ (S * q2[0].astype(np.float64))
    assert np.allclose(out, want, rtol=1e-12, atol=1e-9)


def test_four_used_levels_reduce_to_the_two_bit_gemv():
    N, K = 8, 1024
    idx = rcp_synth.random_indices(6, "w3as2", N, K, levels=4)
    q = rcp_synth.random_int4(6, "w3as2", 1, K)
    xq, sc, _ = oracle.quantize_act(q.astype(np.float32), 1.0)
    rng = np.random.default_rng(3)
    lut8 = rng.standard_normal((N, 8)).astype(np.float16)
    out3, P3 = oracle.w3a4_gemv(oracle.pack_indices_w3(idx), lut8.view(np.uint16), N, K, xq, sc)
    out2, P2 = oracle.w2a4_gemv(oracle.pack_indices(idx), np.ascontiguousarray(lut8[:, :4]).view(np.uint16), N, K, xq, sc, 1)
    assert np.array_equal(P3[:, :4], P2[0]) and not P3[:, 4:].any()
    assert np.array_equal(out3, out2[0])


def test_relabelling_levels_leaves_the_output_unchanged():
    N, K = 4, 512
    idx = rcp_synth.random_indices(7, "perm", N, K, levels=8)
    q = rcp_synth.random_int4(7, "perm", 1, K)
    xq, sc, _ = oracle.quantize_act(q.astype(np.float32), 1.0)
    rng = np.random.default_rng(9)
    lut = rng.integers(-8, 9, size=(N, 8)).astype(np.float16)        # small integers: sums are exact in any order
    perm = rng.permutation(8)
    out_a, P_a = oracle.w3a4_gemv(oracle.pack_indices_w3(idx), lut.view(np.uint16), N, K, xq, sc)
    inv = np.argsort(perm)
    out_b, P_b = oracle.w3a4_gemv(oracle.pack_indices_w3(inv[idx].astype(np.uint8)),
                                  np.ascontiguousarray(lut[:, perm]).view(np.uint16), N, K, xq, sc)
    assert np.array_equal(out_a, out_b)
    assert np.array_equal(P_a[:, perm], P_b)
