"""Pins for the oracle's group-wise (128 input channels per quantisation unit) export and GEMV:
the Appendix table of quantisation configurations (weights: groups of 128) and the LUT shape
H x N*4 of Section 4.4."""
import numpy as np
import pytest

import oracle
import rcp_synth

G = 128


def _f16(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def _lut(cb, N, NG):
    """Grouped LUT layout [N/4][NG][4 rows][4] -> float64 [N, NG, 4]."""
    return _f16(cb).reshape(N // 4, NG, 4, 4).transpose(0, 2, 1, 3).reshape(N, NG, 4)


def _params(seed, N, K):
    W = rcp_synth.weights(seed, "grouped", N, K)
    NG = K // G
    Wg = W.astype(np.float32).reshape(N, NG, G)
    lo = np.quantile(Wg, 0.02, axis=2).astype(np.float32)
    hi = np.quantile(Wg, 0.98, axis=2).astype(np.float32)
    part = rcp_synth.partitions(seed, "grouped", N * NG).reshape(N, NG, 3)
    return W, lo, hi, part


@pytest.mark.parametrize("N,K", [(4, 128), (8, 256), (12, 4096), (8, 11008), (4, 14336), (8, 4224)])
def test_round_trip_and_layout(N, K):
    idx = rcp_synth.random_indices(1, f"grp{K}", N, K)
    packed = oracle.pack_indices_grouped(idx)
    assert packed.size == N * K // 4
    assert np.array_equal(oracle.unpack_indices_grouped(packed, N, K), idx)
    # written layout: unit i of group g at unit position 256*(g/32) + i*R + g%32, R = min(32, NG - 32*(g/32))
    NG = K // G
    rng = np.random.default_rng(K)
    for _ in range(6):
        h, k = int(rng.integers(N)), int(rng.integers(K))
        one = np.zeros((N, K), np.uint8)
        one[h, k] = 3
        words = oracle.pack_indices_grouped(one).view("<u4")
        g, i = k // G, (k % G) // 16
        R = min(32, NG - 32 * (g // 32))
        pos = 256 * (g // 32) + i * R + g % 32
        cell = (h // 4) * (K // 16) * 2 + pos * 2 + (k % 16) // 8          # 8-byte cells
        want = np.zeros_like(words)
        want[2 * cell] = want[2 * cell + 1] = np.uint32(1) << np.uint32(4 * (k % 8) + h % 4)
        assert np.array_equal(words, want)


@pytest.mark.parametrize("N,K", [(8, 256), (12, 4096), (8, 11008)])
def test_equal_groups_reduce_to_the_per_channel_quantiser(N, K):
    """With the same clip range and partition in every group of a row, grouping changes nothing."""
    W, lo_c, hi_c, part_c = rcp_synth.linear_layer(2, "same", N, K)
    NG = K // G
    lo = np.repeat(lo_c[:, None], NG, axis=1)
    hi = np.repeat(hi_c[:, None], NG, axis=1)
    part = np.repeat(part_c[:, None, :], NG, axis=1)
    packed_g, cb_g, idx_g = oracle.pack_weights_grouped(W.astype(np.float32), lo, hi, part, want_idx=True)
    packed_c, cb_c, idx_c = oracle.pack_weights(W.astype(np.float32), lo_c, hi_c, part_c, want_idx=True)
    assert np.array_equal(idx_g, idx_c)
    assert np.array_equal(oracle.unpack_indices_grouped(packed_g, N, K), idx_c)
    lut = _lut(cb_g, N, NG)
    assert np.array_equal(lut, np.repeat(_f16(cb_c)[:, None, :], NG, axis=1))
    x = rcp_synth.activation(2, "same", 1, K).astype(np.float32)
    xq, sc, _ = oracle.quantize_act(x)
    O_g, P_g = oracle.w2a4_gemv_grouped(packed_g, cb_g, N, K, xq, sc)
    O_c, P_c = oracle.w2a4_gemv(packed_c, cb_c, N, K, xq, sc, 1)
    np.testing.assert_allclose(O_g, O_c[0], rtol=1e-12, atol=1e-15)
    assert np.array_equal(P_g.sum(axis=1), P_c[0])


@pytest.mark.parametrize("N,K", [(4, 128), (8, 512), (16, 4096), (8, 11008), (8, 14336)])
def test_gemv_matches_numpy_dequantise_and_dot(N, K):
    W, lo, hi, part = _params(3, N, K)
    NG = K // G
    packed, cb, idx = oracle.pack_weights_grouped(W.astype(np.float32), lo, hi, part, want_idx=True)
    # indices: searchsorted of each group's thresholds; LUT entries from the per-unit grid function
    for h, g in [(0, 0), (N - 1, NG - 1), (N // 2, NG // 2)]:
        T, L = oracle.ldp_grid(lo[h, g], hi[h, g], *part[h, g])
        want = np.searchsorted(T, W[h, g * G:(g + 1) * G].astype(np.float32), side="right")
        assert np.array_equal(idx[h, g * G:(g + 1) * G], want.astype(np.uint8))
        base = oracle.grouped_lut_index(h, g, NG)
        assert np.array_equal(cb[base:base + 4], L)
    x = rcp_synth.activation(3, f"x{K}", 1, K).astype(np.float32)
    xq, sc, q = oracle.quantize_act(x)
    O, P = oracle.w2a4_gemv_grouped(packed, cb, N, K, xq, sc)
    lut = _lut(cb, N, NG)                                                   # [N, NG, 4]
    Wd = np.take_along_axis(np.repeat(lut, G, axis=1), idx.astype(np.int64)[:, :, None], axis=2)[:, :, 0]
    xd = q[0].astype(np.float64) * _f16(sc)[0]
    want = Wd @ xd
    assert np.all(np.abs(O - want) <= 1e-13 * (np.abs(Wd) @ np.abs(xd)) + 1e-300)
    for l in range(4):
        onehot = (idx == l).astype(np.int64).reshape(N, NG, G)
        assert np.array_equal(P[:, :, l], (onehot * q[0].astype(np.int64).reshape(1, NG, G)).sum(axis=2))


@pytest.mark.parametrize("N,K,M", [(8, 256, 3), (12, 4096, 16), (8, 11008, 5)])
def test_several_tokens_match_numpy_dequantise_and_matmul(N, K, M):
    W, lo, hi, part = _params(5, N, K)
    NG = K // G
    packed, cb, idx = oracle.pack_weights_grouped(W.astype(np.float32), lo, hi, part, want_idx=True)
    x = rcp_synth.activation(5, f"xm{K}", M, K).astype(np.float32) * np.linspace(0.5, 2.0, M, dtype=np.float32)[:, None]
    xq, sc, q = oracle.quantize_act(x)
    O, P = oracle.w2a4_gemv_grouped(packed, cb, N, K, xq, sc, M=M)
    assert O.shape == (M, N) and P.shape == (M, N, NG, 4)
    lut = _lut(cb, N, NG)
    Wd = np.take_along_axis(np.repeat(lut, G, axis=1), idx.astype(np.int64)[:, :, None], axis=2)[:, :, 0]
    xd = q.astype(np.float64) * _f16(sc)[:, None]                           # [M, K]
    want = xd @ Wd.T
    assert np.all(np.abs(O - want) <= 1e-13 * (np.abs(xd) @ np.abs(Wd).T) + 1e-300)
    for l in range(4):
        onehot = (idx == l).astype(np.int64).reshape(1, N, NG, G)
        assert np.array_equal(P[..., l], (onehot * q.astype(np.int64).reshape(M, 1, NG, G)).sum(axis=3))
    # token by token it is the one-token call
    for t in (0, M - 1):
        O1, P1 = oracle.w2a4_gemv_grouped(packed, cb, N, K, xq[t:t + 1], sc[t:t + 1])
        assert np.array_equal(O1, O[t]) and np.array_equal(P1, P[t])


def test_shape_errors():
    with pytest.raises(RuntimeError):
        oracle.pack_indices_grouped(np.zeros((4, 192), np.uint8))
    with pytest.raises(RuntimeError):
        oracle.pack_indices_grouped(np.zeros((4, 256), np.uint8), group=64)
