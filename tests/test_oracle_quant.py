"""Pins for the oracle's per-token symmetric int4 quantiser (Appendix table of
quantisation configurations; Section 4.4 for the packed X_q / fp16 S)."""
import numpy as np
import pytest

import oracle
import rcp_synth


def _f16(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


@pytest.mark.parametrize("K,ratio", [(512, 1.0), (4096, 1.0), (11008, 1.0), (4096, 0.9)])
def test_error_bound_scale_and_range(K, ratio):
    x = rcp_synth.activation(0, f"quant{K}", 3, K).astype(np.float32)
    xq, sc, q = oracle.quantize_act(x, ratio)
    s = _f16(sc)
    a = np.abs(x.astype(np.float64)).max(axis=1)
    target = ratio * a / 7.0
    ulp = 2.0 ** (np.floor(np.log2(s)) - 10)
    assert np.all(np.abs(s - target) <= 0.5 * ulp + target * 2.0 ** -22)  # fp16 RNE of an fp32 value
    z = x.astype(np.float64) / s[:, None]
    inside = (z <= 7.5) & (z >= -8.5)
    assert np.all(np.abs(q[inside] - z[inside]) <= 0.5 + 1e-6)
    assert np.all(q[z > 7.5] == 7) and np.all(q[z < -8.5] == -8)
    assert q.min() >= -8 and q.max() <= 7
    if ratio == 1.0:
        assert np.all(np.abs(q).max(axis=1) >= 7)  # the largest entry maps to +-7
        assert np.all(inside | (np.abs(z) < 8.5))
    else:
        assert (~inside).sum() + (np.abs(z) > 7).sum() > 0  # clipping binds at ratio 0.9
    assert np.array_equal(oracle.unpack_act(xq, 3, K), q)


def test_ties_round_to_even_and_nibble_order():
    # a = 7 and ratio 1 give S = 1 exactly, so y is its own quotient
    y = np.array([[7.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5, -3.5, 6.5, -6.5, -7.0, 0.49, -0.51, 4.0, -4.0]],
                 dtype=np.float32)
    xq, sc, q = oracle.quantize_act(y, 1.0)
    assert sc[0] == 0x3C00
    assert list(q[0]) == [7, 0, 2, 2, 0, -2, -2, 4, -4, 6, -6, -7, 0, -1, 4, -4]
    # byte b = (q[2b] & 0xF) | (q[2b+1] << 4): even index in the low nibble
    want = [(int(q[0, 2 * b]) & 0xF) | ((int(q[0, 2 * b + 1]) & 0xF) << 4) for b in range(8)]
    assert list(xq[0]) == want
    assert xq[0, 0] == 0x07 and xq[0, 1] == 0x22


def test_degenerate_inputs():
    K = 64
    xq, sc, q = oracle.quantize_act(np.zeros((1, K), np.float32))
    assert sc[0] == 0x3C00 and not q.any() and not xq.any()
    y = np.zeros((1, K), np.float32)
    y[0, 13] = -1000.0  # single outlier: everything else quantises to zero
    xq, sc, q = oracle.quantize_act(y)
    assert q[0, 13] == -7 and np.count_nonzero(q) == 1
    tiny = np.full((1, K), 1e-9, np.float32)  # S underflows fp16 -> S = 1, q = 0
    xq, sc, q = oracle.quantize_act(tiny)
    assert sc[0] == 0x3C00 and not q.any()
    huge = np.full((1, K), 3e6, np.float32)  # S would overflow fp16 -> capped at 65504
    xq, sc, q = oracle.quantize_act(huge)
    assert sc[0] == 0x7BFF and np.all(q == 7)


def test_nibble_decoding_is_twos_complement_sign_extension():
    """Appendix, online dequantisation: X_hi = byte >> 4 (arithmetic), X_low = (byte << 4) >> 4."""
    b = np.arange(256, dtype=np.uint8)
    q = oracle.unpack_act(b, 1, 512)[0]
    lo = ((b & 0xF).astype(np.int16) ^ 8) - 8
    hi = ((b >> 4).astype(np.int16) ^ 8) - 8
    assert np.array_equal(q[0::2], lo) and np.array_equal(q[1::2], hi)
