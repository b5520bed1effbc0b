"""Pins for the oracle's W2A4 GEMV (Section 4.4): brute force in exact rational arithmetic,
numpy integer and fp64 matmuls, and the identities of the per-level partial sums."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import rcp_synth


def _f16(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def _case(seed, N, K, M):
    idx = rcp_synth.random_indices(seed, "g", N, K)
    q = rcp_synth.random_int4(seed, "g", M, K)
    rng = np.random.default_rng(seed)
    cb = np.sort(rng.standard_normal((N, 4)) * 0.05, axis=1).astype(np.float16).view(np.uint16)
    sc = (np.abs(rng.standard_normal(M)) + 0.1).astype(np.float16).view(np.uint16)
    xq = ((q[:, 0::2].astype(np.uint8) & 0xF) | ((q[:, 1::2].astype(np.uint8) & 0xF) << 4)).astype(np.uint8)
    return idx, q, cb, sc, xq


def test_brute_force_exact_rational_tiny():
    N, K, M = 8, 64, 2
    idx, q, cb, sc, xq = _case(0, N, K, M)
    O, P = oracle.w2a4_gemv(oracle.pack_indices(idx), cb, N, K, xq, sc, M)
    lv, s = _f16(cb), _f16(sc)
    for t in range(M):
        for h in range(N):
            acc = Fraction(0)
            Pl = [0, 0, 0, 0]
            for k in range(K):
                acc += Fraction(lv[h, idx[h, k]]) * Fraction(s[t]) * int(q[t, k])
                Pl[idx[h, k]] += int(q[t, k])
            assert list(P[t, h]) == Pl
            assert abs(Fraction(O[t, h]) - acc) <= abs(acc) * Fraction(1, 10 ** 13) + Fraction(1, 10 ** 18)


@pytest.mark.parametrize("N,K,M", [(4, 32, 1), (12, 96, 3), (256, 512, 1), (64, 2048, 4), (20, 11008, 1)])
def test_matches_dense_dequantise_and_dot(N, K, M):
    idx, q, cb, sc, xq = _case(N + K, N, K, M)
    packed = oracle.pack_indices(idx)
    O, P = oracle.w2a4_gemv(packed, cb, N, K, xq, sc, M)
    Wd = np.take_along_axis(_f16(cb), idx.astype(np.int64), axis=1)          # N x K dequantised weights
    xd = q.astype(np.float64) * _f16(sc)[:, None]                             # M x K dequantised activations
    want = xd @ Wd.T
    scale = (np.abs(xd) @ np.abs(Wd).T)
    assert np.all(np.abs(O - want) <= 1e-13 * scale + 1e-300)
    O2 = oracle.dequant_dot(packed, cb, N, K, xq, sc, M)
    assert np.all(np.abs(O2 - want) <= 1e-13 * scale + 1e-300)
    # per-level partial sums against one-hot integer matmuls
    for l in range(4):
        want_P = q.astype(np.int64) @ (idx == l).astype(np.int64).T
        assert np.array_equal(P[:, :, l], want_P)
    assert np.array_equal(P.sum(axis=2), np.broadcast_to(q.astype(np.int64).sum(axis=1)[:, None], (M, N)))


def test_integer_codebook_and_all_ones_activation():
    N, K = 16, 256
    idx, q, _, _, xq = _case(9, N, K, 1)
    cb = np.tile(np.array([0, 1, 2, 3], np.float16).view(np.uint16), (N, 1))
    one = np.array([1.0], np.float16).view(np.uint16)
    O, P = oracle.w2a4_gemv(oracle.pack_indices(idx), cb, N, K, xq, one, 1)
    assert np.array_equal(O[0], (idx.astype(np.int64) @ q[0].astype(np.int64)).astype(np.float64))
    ones = np.full((1, K // 2), 0x11, np.uint8)
    O, P = oracle.w2a4_gemv(oracle.pack_indices(idx), cb, N, K, ones, one, 1)
    for h in range(N):
        assert np.array_equal(P[0, h], np.bincount(idx[h], minlength=4))


def test_end_to_end_tiny_config_against_fp64_pipeline():
    """Config 'tiny': pack -> rotate -> quantise -> GEMV equals the same chain in numpy fp64."""
    (name, N, K, rot), = rcp_synth.CONFIGS["tiny"]
    W, lo, hi, part = rcp_synth.linear_layer(0, name, N, K)
    x = rcp_synth.activation(0, name, 1, K)
    packed, cb, idx = oracle.pack_weights(W.astype(np.float32), lo, hi, part, want_idx=True)
    y = oracle.rotate(x.astype(np.float64), oracle.ROT_WHT, n_wht=K)
    xq, sc, q = oracle.quantize_act(y.astype(np.float32))
    O, P = oracle.w2a4_gemv(packed, cb, N, K, xq, sc, 1)
    Wd = np.take_along_axis(_f16(cb), idx.astype(np.int64), axis=1)
    want = (q.astype(np.float64) * _f16(sc)[:, None]) @ Wd.T
    np.testing.assert_allclose(O, want, rtol=1e-12, atol=1e-15)
    # the quantised product approximates the clipped-weight fp product: loose sanity bound
    Wc = np.clip(W.astype(np.float64), lo[:, None], hi[:, None])
    full = y @ Wc.T
    # (random, untrained partitions at 2 bits: the error is large but the signal must dominate)
    cos = float((O * full).sum() / (np.linalg.norm(O) * np.linalg.norm(full)))
    assert cos > 0.7
