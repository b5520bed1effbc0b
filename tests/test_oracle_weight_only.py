"""Pins for the oracle's weight-only product (the W2-only variant of the paper's inference-latency
section): O[h] = sum_k LUT[h][idx[h][k]] * x[k] with 16-bit activations, binary64 accumulation."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import rcp_synth


def _f16(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def _case(seed, N, K, M=1):
    idx = rcp_synth.random_indices(seed, f"wo{N}x{K}", N, K)
    rng = np.random.default_rng(seed)
    cb = np.sort(rng.standard_normal((N, 4)) * 0.03, axis=1).astype(np.float16).view(np.uint16)
    x = rcp_synth.activation(seed, f"wo{K}", M, K)
    return idx, oracle.pack_indices(idx), cb, x


@pytest.mark.parametrize("N,K,M", [(4, 32, 1), (8, 96, 3), (64, 512, 1), (16, 2080, 2)])
def test_equals_dense_dequantised_matrix_product(N, K, M):
    idx, packed, cb, x = _case(1, N, K, M)
    Wd = np.take_along_axis(_f16(cb), idx.astype(np.int64), axis=1)      # N x K dequantised weights
    want = x.astype(np.float64) @ Wd.T
    got = oracle.w2a16_gemv(packed, cb, N, K, x)
    assert got.shape == (M, N)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-15)


def test_exact_rational_on_tiny_case():
    N, K = 4, 32
    idx, packed, cb, x = _case(2, N, K)
    got = oracle.w2a16_gemv(packed, cb, N, K, x)
    lut = _f16(cb)
    for h in range(N):
        exact = sum(Fraction(float(lut[h, idx[h, k]])) * Fraction(float(x[0, k])) for k in range(K))
        assert abs(Fraction(float(got[0, h])) - exact) <= abs(exact) * Fraction(1, 10 ** 13) + Fraction(1, 10 ** 18)


@pytest.mark.parametrize("N,K", [(8, 64), (32, 4096), (8, 11008)])
def test_agrees_with_the_w2a4_product_on_exactly_dequantised_int4_activations(N, K):
    """x = S*q with S a power of two is an fp16 vector; both statements of the product must then
    give the same number (the W2A4 oracle via per-level integer sums, this one via plain products)."""
    idx = rcp_synth.random_indices(3, f"woq{K}", N, K)
    packed = oracle.pack_indices(idx)
    rng = np.random.default_rng(3)
    cb = np.sort(rng.standard_normal((N, 4)) * 0.03, axis=1).astype(np.float16).view(np.uint16)
    q = rcp_synth.random_int4(3, f"woq{K}", 1, K)
    sc = np.array([0.125], np.float16).view(np.uint16)
    xq = ((q[:, 0::2].astype(np.uint8) & 0xF) | ((q[:, 1::2].astype(np.uint8) & 0xF) << 4)).astype(np.uint8)
    O_a4, _ = oracle.w2a4_gemv(packed, cb, N, K, xq, sc, 1)
    x = (q.astype(np.float64) * 0.125).astype(np.float16)
    assert np.array_equal(x.astype(np.float64), q * 0.125)
    O_wo = oracle.w2a16_gemv(packed, cb, N, K, x)
    assert np.allclose(O_wo, O_a4, rtol=1e-12, atol=1e-14)


def test_linear_in_x_and_one_hot_columns():
    N, K = 12, 96
    idx, packed, cb, x = _case(4, N, K, 2)
    lut = _f16(cb)
    # a unit vector picks one dequantised weight per row
    for k in (0, 7, 8, 31, 95):
        e = np.zeros((1, K)); e[0, k] = 1.0
        assert np.array_equal(oracle.w2a16_gemv(packed, cb, N, K, e)[0], lut[np.arange(N), idx[:, k]])
    a = oracle.w2a16_gemv(packed, cb, N, K, x[0:1].astype(np.float64))
    b = oracle.w2a16_gemv(packed, cb, N, K, x[1:2].astype(np.float64))
    ab = oracle.w2a16_gemv(packed, cb, N, K, x[0:1].astype(np.float64) * 2 + x[1:2].astype(np.float64))
    assert np.allclose(ab, 2 * a + b, rtol=1e-12, atol=1e-15)


def test_all_ones_activation_counts_levels():
    N, K = 8, 2080
    idx, packed, cb, _ = _case(5, N, K)
    lut = _f16(cb)
    got = oracle.w2a16_gemv(packed, cb, N, K, np.ones((1, K)))
    counts = np.stack([(idx == l).sum(axis=1) for l in range(4)], axis=1)
    assert np.allclose(got[0], (counts * lut).sum(axis=1), rtol=1e-13)


def test_shape_errors():
    idx, packed, cb, x = _case(6, 8, 64)
    with pytest.raises(RuntimeError):
        oracle.lib().rcp_ref_w2a16_gemv  # symbol exists
        oracle._check(oracle.lib().rcp_ref_w2a16_gemv(oracle._p(packed), oracle._p(cb), 6, 64,
                                                      oracle._p(x.astype(np.float64)), 1,
                                                      oracle._p(np.empty(8))), "w2a16_gemv")
