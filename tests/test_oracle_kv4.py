"""Pins for the oracle's 4-bit KV cache: the asymmetric integer quantiser of Eqn. 1 with N = 4
on groups of 128 (Appendix table of quantisation configurations: asymmetric, group size 128,
clipping ratio 0.95) and one-token attention over the cache (Section 2.1: the cache is
compressed, attention itself is the usual softmax(q K^T) V)."""
import os

import numpy as np
import pytest
import scipy.special

import oracle
import rcp_synth

D = 128
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "kv_cache_quant_config.txt")


def _config():
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            bits, sym, group, ratio = line.split()
            return int(bits), sym == "yes", int(group), float(ratio)
    raise AssertionError("no data line in the fixture")


def test_configuration_is_the_papers():
    bits, symmetric, group, ratio = _config()
    assert (bits, symmetric, group, ratio) == (4, False, 128, 0.95)
    assert oracle.KV_D == group                                 # one head vector is one group
    x = rcp_synth.kv_vectors(2, "cfg", 50, 2).astype(np.float32)
    codes, params = _quantise(x, clip=ratio)
    c = _codes(codes)
    assert c.min() == 0 and c.max() == 2 ** bits - 1            # N bits, both ends used
    sb, z = oracle.kv4_params(params)
    lo, hi = ratio * x.min(axis=-1).T, ratio * x.max(axis=-1).T
    assert np.allclose(_f16(sb), (hi - lo) / (2 ** bits - 1), rtol=2.0 ** -10)      # s = h / (2^N - 1) on the clipped range
    assert np.all(np.abs(z + lo / _f16(sb)) <= 0.5 + 1e-4)                          # asymmetric: zero point -round(min / s)
    assert (z != 8).any()                                                           # not a symmetric grid
    # the product binding's default clipping ratio is the table's
    import inspect
    import paper_2502_15779_amd
    assert inspect.signature(paper_2502_15779_amd.kv4_append).parameters["clip_ratio"].default == ratio
    assert inspect.signature(paper_2502_15779_amd.kv4_append_batched).parameters["clip_ratio"].default == ratio


def _f16(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def _quantise(x, clip=0.95, S_max=None, pos=0):
    n, H, _ = x.shape
    codes, params = oracle.kv4_new_cache(H, S_max or n)
    oracle.kv4_append(x, pos, clip, codes, params)
    return codes, params


def _codes(codes):
    """uint8[H][S][128] of the nibbles in element order."""
    return np.stack([codes & 0xF, codes >> 4], axis=-1).reshape(codes.shape[0], codes.shape[1], D)


def test_integer_grid_is_reproduced_exactly():
    # values a + b*k, k = 0..15, b a power of two, clipping off: the step is b, the minimum
    # gets code 0, the maximum code 15, and every value comes back exactly
    rng = np.random.default_rng(1)
    for b, a in [(0.25, -2.0), (1.0, -8.0), (0.5, 0.0), (2.0, -30.0), (0.125, -0.5)]:
        k = rng.integers(0, 16, size=(3, 2, D))
        k[:, :, 0], k[:, :, 1] = 0, 15
        x = (a + b * k).astype(np.float32)
        codes, params = _quantise(x, clip=1.0)
        sb, z = oracle.kv4_params(params)
        assert np.all(_f16(sb) == b)
        assert np.all(z == -round(a / b))
        assert np.array_equal(_codes(codes).transpose(1, 0, 2), k.astype(np.uint8))
        assert np.array_equal(oracle.kv4_dequant(codes, params, 0, 3), x.astype(np.float64))


def test_codes_are_the_nearest_points_of_the_grid_inside_the_clip_range():
    x = rcp_synth.kv_vectors(3, "k", 40, 4).astype(np.float32)
    codes, params = _quantise(x)
    sb, z = oracle.kv4_params(params)
    s = _f16(sb).T[:, :, None]            # [n][H][1]
    zz = z.T.astype(np.float64)[:, :, None]
    c = _codes(codes).transpose(1, 0, 2).astype(np.float64)
    grid = s[..., None] * (np.arange(16)[None, None, None, :] - zz[..., None])   # [n][H][1][16]
    dist = np.abs(x.astype(np.float64)[..., None] - grid)
    best = dist.min(axis=-1)
    mine = np.abs(x - s * (c - zz))
    assert np.all(mine <= best + 1e-6 * s)      # ties and float rounding aside, the nearest point
    # the grid covers the clipped range: its ends lie within one step of ratio*min and ratio*max
    lo, hi = 0.95 * x.min(axis=-1), 0.95 * x.max(axis=-1)
    assert np.all(np.abs(grid[:, :, 0, 0] - lo) <= s[:, :, 0])
    assert np.all(np.abs(grid[:, :, 0, 15] - hi) <= 1.01 * s[:, :, 0])
    # the step is (hi - lo) / (2^N - 1), held in fp16
    assert np.allclose(s[:, :, 0], (hi - lo) / 15.0, rtol=2.0 ** -10)
    # inside the range the error is at most half a step; outside, the value saturates at an end code
    inside = (x >= grid[:, :, :, 0]) & (x <= grid[:, :, :, 15])
    assert np.all(mine[inside] <= (0.5 + 1e-6) * np.broadcast_to(s, x.shape)[inside])
    assert np.all(c[x < grid[:, :, :, 0]] == 0) and np.all(c[x > grid[:, :, :, 15]] == 15)
    assert inside.mean() > 0.9


def test_offset_groups_follow_eqn_1_on_the_clipped_range_in_double():
    """Groups far from zero (either sign), checked in binary64 against Eqn. 1 with the stored (s, z): every code whose
    value lies inside the clipped range [ratio*min, ratio*max] is within half a step of x/s + z and dequantises to
    within s/2 of x; values outside that range take the end codes.  Because the one clipping ratio of the table scales
    the minimum and the maximum (the form of the paper's clipping equation for weights), the range of a group that does
    not straddle zero moves towards zero instead of shrinking about the data: for x in [a, a + w] with a > 0 only values
    up to ratio*(a + w) keep their half-step accuracy.  That consequence of the reading is pinned here too."""
    rng = np.random.default_rng(12)
    for offset, width, ratio in [(0.0, 1.0, 0.95), (3.0, 1.0, 0.95), (-3.0, 2.0, 0.95), (40.0, 8.0, 1.0), (-250.0, 3.0, 1.0),
                                 (7.5, 0.25, 0.9), (1000.0, 0.9, 1.0)]:
        x = (offset + width * rng.random((6, 3, D))).astype(np.float32)
        codes, params = _quantise(x, clip=ratio)
        sb, z = oracle.kv4_params(params)
        s = _f16(sb).T[:, :, None]
        zz = z.T.astype(np.float64)[:, :, None]
        c = _codes(codes).transpose(1, 0, 2).astype(np.float64)
        x64 = x.astype(np.float64)
        lo = ratio * x64.min(axis=-1, keepdims=True)
        hi = ratio * x64.max(axis=-1, keepdims=True)
        assert np.all(np.abs(zz + lo / s) <= 0.5 + 1e-3)                 # z = -round(lo / s), |z| far below the int16 limit
        assert np.all(np.abs(s - (hi - lo) / 15.0) <= 2.0 ** -10 * s + 1e-12)
        t = x64 / s + zz                                                 # Eqn. 1 before rounding and clamping
        free = (t >= -0.5) & (t <= 15.5)                                 # rounds to a code without clamping
        eps = 1e-4 + 2.0 ** -22 * np.abs(x64 / s)                        # the rounding decision is taken in binary32
        assert np.all((np.abs(c - t) <= 0.5 + eps)[free])
        assert np.all((np.abs(s * (c - zz) - x64) <= (0.5 + eps) * s)[free])
        assert np.all(c[t < -0.5] == 0) and np.all(c[t > 15.5] == 15)
        if ratio == 1.0:
            assert free.mean() > 0.999           # nothing is clipped: the whole group keeps half-step accuracy
        elif offset > 0:
            clipped = x64 > hi + s               # the top of a positive group lies beyond ratio*max and saturates
            assert clipped.any() and np.all(c[clipped] == 15)
            if width < (1.0 - ratio) * offset:   # the whole group lies above ratio*max: every value takes the top code
                assert np.all(c == 15)
    # the zero point is stored in 16 bits: beyond |lo / s| = 32767 it saturates (both sides do the same)
    x = np.full((1, 1, D), 60000.0, dtype=np.float32)
    x[0, 0, 0] = 59999.0
    _, params = _quantise(x, clip=1.0)
    assert oracle.kv4_params(params)[1][0, 0] == -32768


def test_zero_point_follows_the_minimum():
    # shifting a group by a whole number of steps shifts the zero point and leaves the codes
    rng = np.random.default_rng(4)
    k = rng.integers(0, 16, size=(1, 1, D))
    k[0, 0, :2] = (0, 15)
    base = (0.5 * k).astype(np.float32)
    c0, p0 = _quantise(base, clip=1.0)
    for shift in (-20, -3, 7, 100):
        c1, p1 = _quantise(base + np.float32(0.5 * shift), clip=1.0)
        assert np.array_equal(c0, c1)
        assert oracle.kv4_params(p1)[1][0, 0] == oracle.kv4_params(p0)[1][0, 0] - shift
        assert oracle.kv4_params(p1)[0][0, 0] == oracle.kv4_params(p0)[0][0, 0]


def test_constant_and_zero_groups():
    x = np.zeros((2, 2, D), dtype=np.float32)
    x[1, 0, :] = 3.0
    codes, params = _quantise(x)
    sb, z = oracle.kv4_params(params)
    assert np.all(sb == 0x3C00)                      # zero range: the step is taken as 1
    deq = oracle.kv4_dequant(codes, params, 0, 2)
    assert np.all(deq[0] == 0.0) and np.all(deq[1, 1] == 0.0)
    assert np.all(np.abs(deq[1, 0] - 3.0) <= 0.5)


def test_layout_and_append_positions():
    H, S_max = 3, 10
    x = rcp_synth.kv_vectors(5, "v", 6, H).astype(np.float32)
    codes, params = oracle.kv4_new_cache(H, S_max)
    codes[:] = 0xEE
    params[:] = 0x77
    oracle.kv4_append(x[:2], 3, 0.95, codes, params)
    oracle.kv4_append(x[2:], 5, 0.95, codes, params)
    # untouched positions keep their bytes
    for t in (0, 1, 2, 9):
        assert np.all(codes[:, t] == 0xEE) and np.all(params[:, t] == 0x77)
    # a token's codes do not depend on where or with whom it was appended
    c2, p2 = _quantise(x)
    assert np.array_equal(codes[:, 3:9], c2) and np.array_equal(params[:, 3:9], p2)
    # element j sits in byte j // 2, low nibble first; head-major, then token
    one = np.zeros((1, H, D), dtype=np.float32)
    one[0, 1, 0], one[0, 1, 37] = -1.0, 14.0        # range 15, step 1: codes 0 and 15, the rest 1
    c3, p3 = _quantise(one, clip=1.0, S_max=4, pos=2)
    flat = c3.reshape(-1)
    base = (1 * 4 + 2) * 64
    assert flat[base + 0] == 0x10 and flat[base + 18] == 0xF1 and flat[base + 5] == 0x11
    pb = p3.reshape(-1)[(1 * 4 + 2) * 4:(1 * 4 + 2) * 4 + 4]
    assert pb[0] == 0x00 and pb[1] == 0x3C and pb[2] == 1 and pb[3] == 0


def test_rotated_append_is_the_append_of_the_rotated_vectors():
    # R3 (Section 2.1): with the flag set, what is quantised is H x / sqrt(128) per head vector; the
    # transform itself is pinned to the dense definition in the rotation tests
    x = rcp_synth.kv_vectors(12, "k", 9, 3).astype(np.float32)
    c1, p1 = oracle.kv4_new_cache(3, 9)
    oracle.kv4_append(x, 0, 0.95, c1, p1, rotate=True)
    dense = oracle.rotate(x.reshape(-1, D).astype(np.float64), oracle.ROT_WHT, D, 1).reshape(x.shape)
    fast = np.stack([oracle.fwht_f32(v) for v in x.reshape(-1, D)]).reshape(x.shape)
    assert np.allclose(fast, dense, rtol=0, atol=1e-5 * np.abs(dense).max())
    c2, p2 = _quantise(fast)
    assert np.array_equal(c1, c2) and np.array_equal(p1, p2)
    # scores are unchanged when queries and keys are both rotated (up to the quantisation of the keys):
    # the dequantised rotated keys stay within half a step of the rotated vectors inside the clip range
    deq = oracle.kv4_dequant(c1, p1, 0, 9)
    s = _f16(oracle.kv4_params(p1)[0]).T[:, :, None]
    inside = (dense >= 0.95 * dense.min(axis=-1, keepdims=True)) & (dense <= 0.95 * dense.max(axis=-1, keepdims=True))
    assert np.all(np.abs(deq - dense)[inside] <= (0.5 + 1e-3) * np.broadcast_to(s, dense.shape)[inside] + 1e-6)
    q = rcp_synth.query_vectors(12, "q", 3).astype(np.float64)
    qr = oracle.rotate(q, oracle.ROT_WHT, D, 1)
    assert np.allclose(np.einsum("hd,thd->th", qr, dense), np.einsum("hd,thd->th", q, x.astype(np.float64)), atol=1e-9)
    # a constant vector rotates onto its first coordinate
    one = np.full((1, 1, D), 0.5, dtype=np.float32)
    c3, p3 = oracle.kv4_new_cache(1, 1)
    oracle.kv4_append(one, 0, 1.0, c3, p3, rotate=True)
    d3 = oracle.kv4_dequant(c3, p3, 0, 1)[0, 0]
    assert abs(d3[0] - 0.5 * np.sqrt(128.0)) <= 0.5 * _f16(oracle.kv4_params(p3)[0])[0, 0] and np.all(d3[1:] == 0.0)


def _cache(seed, S, H, S_max=None):
    k = rcp_synth.kv_vectors(seed, "k", S, H).astype(np.float32)
    v = rcp_synth.kv_vectors(seed, "v", S, H).astype(np.float32)
    kc, kp = _quantise(k, S_max=S_max or S)
    vc, vp = _quantise(v, S_max=S_max or S)
    return kc, kp, vc, vp


def test_attention_equals_library_softmax_of_the_dequantised_cache():
    H, S = 4, 77
    kc, kp, vc, vp = _cache(7, S, H, S_max=80)
    q = rcp_synth.query_vectors(7, "q", H).astype(np.float64)
    out = oracle.kv4_attn_decode(q, S, kc, kp, vc, vp, 1.0 / np.sqrt(D))
    K = oracle.kv4_dequant(kc, kp, 0, S)        # [S][H][128]
    V = oracle.kv4_dequant(vc, vp, 0, S)
    for h in range(H):
        p = scipy.special.softmax(K[:, h] @ q[h] / np.sqrt(D))
        assert np.allclose(out[h], p @ V[:, h], rtol=1e-12, atol=1e-13)


def test_attention_special_cases():
    H, S = 2, 33
    kc, kp, vc, vp = _cache(8, S, H)
    q = rcp_synth.query_vectors(8, "q", H).astype(np.float64)
    V = oracle.kv4_dequant(vc, vp, 0, S)
    K = oracle.kv4_dequant(kc, kp, 0, S)
    # one cached token: the output is that token's value vector
    assert np.allclose(oracle.kv4_attn_decode(q, 1, kc, kp, vc, vp, 0.3), V[0], rtol=1e-14)
    # zero query (or zero scale): uniform weights, the output is the mean value vector
    assert np.allclose(oracle.kv4_attn_decode(np.zeros_like(q), S, kc, kp, vc, vp, 1.0), V.mean(axis=0), rtol=1e-13)
    assert np.allclose(oracle.kv4_attn_decode(q, S, kc, kp, vc, vp, 0.0), V.mean(axis=0), rtol=1e-13)
    # a query far along one key picks that key's value
    t = 11
    big = 50.0 * K[t]
    others = np.delete(np.arange(S), t)
    margin = np.array([(big[h] @ K[t, h]) - np.max(K[others, h] @ big[h]) for h in range(H)])
    assert np.all(margin > 40)
    assert np.allclose(oracle.kv4_attn_decode(big, S, kc, kp, vc, vp, 1.0), V[t], atol=1e-12)
    # only the first S tokens count
    full = oracle.kv4_attn_decode(q, 20, kc, kp, vc, vp, 0.1)
    kc2, vc2 = kc.copy(), vc.copy()
    kc2[:, 20:], vc2[:, 20:] = 0x5A, 0xA5
    assert np.array_equal(full, oracle.kv4_attn_decode(q, 20, kc2, kp, vc2, vp, 0.1))


def test_attention_is_invariant_to_token_order_and_handles_large_scores():
    H, S = 2, 50
    kc, kp, vc, vp = _cache(9, S, H)
    q = rcp_synth.query_vectors(9, "q", H).astype(np.float64)
    ref = oracle.kv4_attn_decode(q, S, kc, kp, vc, vp, 0.09)
    perm = np.random.default_rng(0).permutation(S)
    out = oracle.kv4_attn_decode(q, S, np.ascontiguousarray(kc[:, perm]), np.ascontiguousarray(kp[:, perm]),
                                 np.ascontiguousarray(vc[:, perm]), np.ascontiguousarray(vp[:, perm]), 0.09)
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-14)
    # scores in the thousands must not overflow
    out = oracle.kv4_attn_decode(200.0 * q, S, kc, kp, vc, vp, 1.0)
    assert np.all(np.isfinite(out))


def test_grouped_query_heads_share_a_cache_head():
    H_kv, rep, S = 2, 4, 19
    kc, kp, vc, vp = _cache(10, S, H_kv)
    q = rcp_synth.query_vectors(10, "q", H_kv * rep).astype(np.float64)
    out = oracle.kv4_attn_decode(q, S, kc, kp, vc, vp, 0.1)
    for h in range(H_kv * rep):
        hk = h // rep
        single = oracle.kv4_attn_decode(q[h:h + 1], S, kc[hk:hk + 1].copy(), kp[hk:hk + 1].copy(),
                                        vc[hk:hk + 1].copy(), vp[hk:hk + 1].copy(), 0.1)
        assert np.array_equal(single[0], out[h])


def test_shape_errors():
    codes, params = oracle.kv4_new_cache(2, 4)
    x = np.zeros((3, 2, D), dtype=np.float32)
    with pytest.raises(RuntimeError):
        oracle.kv4_append(x, 2, 0.95, codes, params)          # runs past S_max
    with pytest.raises(RuntimeError):
        oracle.kv4_attn_decode(np.zeros((2, D)), 5, codes, params, codes, params, 1.0)
    with pytest.raises(RuntimeError):
        oracle.kv4_attn_decode(np.zeros((3, D)), 2, codes, params, codes, params, 1.0)
