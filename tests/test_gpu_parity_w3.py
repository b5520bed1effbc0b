"""GPU-vs-oracle parity of the 3-bit variant through the C ABI: export (LDP on the asymmetric
normal-float format) bit-exact, per-level int32 partial sums of the eight-level GEMV bit-exact,
floating-point outputs within 1e-3 of the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2502_15779_amd as rcp
import rcp_synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _f16(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(autouse=True)
def _auto_options():
    yield
    for k in ("gemv_lanes", "gemv_blocks", "gemv_nt"):
        rcp.set_option(k, 0)


def _nibbles(q):
    return ((q[:, 0::2].astype(np.uint8) & 0xF) | ((q[:, 1::2].astype(np.uint8) & 0xF) << 4)).astype(np.uint8)


@pytest.mark.parametrize("N,K,dtype", [(4, 32, "f32"), (12, 96, "f16"), (36, 2080, "bf16"), (256, 2048, "f16"),
                                       (1024, 4096, "f16"), (64, 11008, "f16"), (8, 32768, "f16")])
def test_pack_w3_bit_exact(N, K, dtype):
    _say(f"pack w3 N={N} K={K} {dtype}")
    W, lo, hi, frac, grid = rcp_synth.linear_layer_w3(1, f"w3pack{N}x{K}", N, K)
    if dtype == "f16":
        Wd, W32 = _t(W), W.astype(np.float32)
    elif dtype == "f32":
        W32 = W.astype(np.float32) * np.float32(1.0009765)
        Wd = _t(W32)
    else:
        Wd = _t(W.astype(np.float32)).to(torch.bfloat16)
        W32 = Wd.to(torch.float32).cpu().numpy()
    packed, cb = rcp.pack_weights_w3(Wd, _t(lo), _t(hi), _t(frac), grid)
    idx = rcp.unpack_indices_w3(packed, N, K)
    torch.cuda.synchronize()
    ref_packed, ref_cb, ref_idx = oracle.pack_weights_w3(W32, lo, hi, frac, grid, want_idx=True)
    assert np.array_equal(cb.cpu().numpy().view(np.uint16), ref_cb)
    assert np.array_equal(idx.cpu().numpy(), ref_idx)
    assert np.array_equal(packed.cpu().numpy(), ref_packed)
    assert len(np.unique(ref_idx)) == 8


def test_pack_w3_weights_on_thresholds_and_integer_grid():
    """Weights sitting exactly on thresholds and levels; the integer grid of the printed rounding rule."""
    N, K = 8, 64
    grid = np.arange(-3, 5, dtype=np.float32)
    lo = np.array([-3, -1.5, -0.75, -3e-3, -6, -3, -0.3, -30000], np.float32) / 3
    hi = np.array([4, 2, 1, 4e-3, 2, 8, 0.1, 30000], np.float32) / 4
    frac = np.array([0.5, 0.5, 0.5, 0.5, 0.75, 0.25, 0.6, 0.5], np.float32)
    rng = np.random.default_rng(2)
    W = np.empty((N, K), np.float32)
    for h in range(N):
        T, L = oracle.w3_grid(lo[h], hi[h], frac[h], grid)
        pool = np.concatenate([T, np.nextafter(T, np.float32(-np.inf)), np.nextafter(T, np.float32(np.inf)),
                               _f16(L).astype(np.float32), [np.float32(-65504), np.float32(65504), 0.0]])
        W[h] = rng.choice(pool.astype(np.float32), size=K)
    packed, cb = rcp.pack_weights_w3(_t(W), _t(lo), _t(hi), _t(frac), grid)
    torch.cuda.synchronize()
    ref_packed, ref_cb = oracle.pack_weights_w3(W, lo, hi, frac, grid)
    assert np.array_equal(cb.cpu().numpy().view(np.uint16), ref_cb)
    assert np.array_equal(packed.cpu().numpy(), ref_packed)


def _w3_case(seed, N, K):
    idx = rcp_synth.random_indices(seed, f"w3gemv{N}x{K}", N, K, levels=8)
    q = rcp_synth.random_int4(seed, f"w3gemv{K}", 1, K)
    rng = np.random.default_rng(seed)
    cb = np.sort(rng.standard_normal((N, 8)) * 0.03, axis=1).astype(np.float16).view(np.uint16)
    sc = (np.abs(rng.standard_normal(1)) * 0.2 + 0.05).astype(np.float16).view(np.uint16)
    return oracle.pack_indices_w3(idx), cb, _nibbles(q), sc


def _check_w3(packed, cb, N, K, xq, sc, out_dtype):
    ref_O, ref_P = oracle.w3a4_gemv(packed, cb, N, K, xq, sc)
    out, P = rcp.w3a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, _t(xq), _t(sc.view(np.float16)),
                           out_dtype=out_dtype, want_partial_sums=True)
    torch.cuda.synchronize()
    assert np.array_equal(P.cpu().numpy(), ref_P), "per-level partial sums are not bit-exact"
    got = out.cpu().numpy().astype(np.float64).ravel()
    cond = _f16(sc)[0] * (np.abs(_f16(cb)) * np.abs(ref_P)).sum(axis=1)
    half = 2.0 ** -11 * np.abs(ref_O) if out_dtype == torch.float16 else 0.0
    assert np.all(np.abs(got - ref_O) <= 1e-3 * cond + half + 1e-30)
    assert np.linalg.norm(got - ref_O) <= 1e-3 * np.linalg.norm(ref_O) + 1e-30
    out2 = rcp.w3a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, _t(xq), _t(sc.view(np.float16)), out_dtype=out_dtype)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


@pytest.mark.parametrize("N,K", [(4, 32), (12, 96), (256, 512), (20, 2080), (1028, 4096), (72, 11008), (40, 14336),
                                 (2048, 2048), (16, 32768), (8200, 64)])
@pytest.mark.parametrize("lanes", [0, 64, 128, 256])
def test_w3_gemv_partial_sums_bit_exact_and_output_close(N, K, lanes):
    _say(f"w3 gemv N={N} K={K} lanes={lanes}")
    rcp.set_option("gemv_lanes", lanes)   # wavefronts per row group: automatic, 1, 2, 4
    packed, cb, xq, sc = _w3_case(N + K, N, K)
    _check_w3(packed, cb, N, K, xq, sc, torch.float32)
    _check_w3(packed, cb, N, K, xq, sc, torch.float16)


@pytest.mark.parametrize("N,K", [(12, 96), (1028, 4096), (72, 11008), (8200, 64)])
def test_w3_gemv_with_non_temporal_weight_loads(N, K):
    """The weight loads' cache hint that the launcher adds from 16 MB on, forced on small matrices: pre-quantised and
    fused calls, same partial sums."""
    _say(f"w3 gemv non-temporal N={N} K={K}")
    rcp.set_option("gemv_nt", 1)
    packed, cb, xq, sc = _w3_case(N + K + 1, N, K)
    _check_w3(packed, cb, N, K, xq, sc, torch.float32)
    xd, x32 = _x_as(rcp_synth.activation(9, f"w3nt{K}", 1, K), "f16")
    ref_xq, ref_sc, _ = oracle.quantize_act(x32, 1.0)
    _, ref_P = oracle.w3a4_gemv(packed, cb, N, K, ref_xq, ref_sc)
    _, P = rcp.quant_w3a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, xd, 1.0, out_dtype=torch.float32,
                               want_partial_sums=True)
    torch.cuda.synchronize()
    assert np.array_equal(P.cpu().numpy(), ref_P)


def test_w3_gemv_extreme_activations_and_integer_codebook():
    """q = -8 everywhere with index 7 everywhere drives every monomial sum to its largest magnitude;
    an integer codebook makes the fp32 epilogue exact."""
    N, K = 16, 14336
    idx = np.full((N, K), 7, np.uint8)
    idx[1::2] = rcp_synth.random_indices(0, "w3ext", N // 2, K, levels=8)
    cb = np.tile(np.arange(8).astype(np.float16).view(np.uint16), (N, 1))
    xq = np.full((1, K // 2), 0x88, np.uint8)
    one = np.array([1.0], np.float16).view(np.uint16)
    packed = oracle.pack_indices_w3(idx)
    ref_O, ref_P = oracle.w3a4_gemv(packed, cb, N, K, xq, one)
    out, P = rcp.w3a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, _t(xq), _t(one.view(np.float16)),
                           out_dtype=torch.float32, want_partial_sums=True)
    torch.cuda.synchronize()
    assert np.array_equal(P.cpu().numpy(), ref_P)
    assert np.array_equal(out.cpu().numpy().astype(np.float64).ravel(), ref_O)
    assert ref_P[0, 7] == -8 * K


@pytest.mark.parametrize("lanes", [64, 128, 256])
@pytest.mark.parametrize("blocks", [1, 3, 64])
def test_w3_gemv_grid_stride_with_few_workgroups(blocks, lanes):
    _say(f"w3 gemv grid-stride blocks={blocks} lanes={lanes}")
    rcp.set_option("gemv_blocks", blocks)
    rcp.set_option("gemv_lanes", lanes)
    N, K = 1028, 11008
    packed, cb, xq, sc = _w3_case(3, N, K)
    _check_w3(packed, cb, N, K, xq, sc, torch.float32)


@pytest.mark.parametrize("N,K", [(64, 4096), (32, 11008)])
def test_w3_whole_path(N, K):
    """export -> quantise -> GEMV against the oracle doing the same from the same inputs."""
    _say(f"w3 whole path N={N} K={K}")
    W, lo, hi, frac, grid = rcp_synth.linear_layer_w3(4, f"w3whole{N}x{K}", N, K)
    x = rcp_synth.activation(4, f"w3whole{K}", 1, K)
    packed, cb = rcp.pack_weights_w3(_t(W), _t(lo), _t(hi), _t(frac), grid)
    xq, sc = rcp.rotate_quant_act(_t(x))
    out, P = rcp.w3a4_gemv(packed, cb, N, K, xq, sc, out_dtype=torch.float32, want_partial_sums=True)
    torch.cuda.synchronize()
    ref_packed, ref_cb = oracle.pack_weights_w3(W.astype(np.float32), lo, hi, frac, grid)
    ref_xq, ref_sc, _ = oracle.quantize_act(x.astype(np.float32))
    assert np.array_equal(xq.cpu().numpy(), ref_xq) and np.array_equal(sc.cpu().numpy().view(np.uint16), ref_sc)
    ref_O, ref_P = oracle.w3a4_gemv(ref_packed, ref_cb, N, K, ref_xq, ref_sc)
    assert np.array_equal(P.cpu().numpy(), ref_P)
    got = out.cpu().numpy().astype(np.float64).ravel()
    assert np.linalg.norm(got - ref_O) <= 1e-3 * np.linalg.norm(ref_O)
    exact = W.astype(np.float64) @ x.astype(np.float64).ravel()
    cos = float(got @ exact / (np.linalg.norm(got) * np.linalg.norm(exact)))
    assert cos > 0.8


def _x_as(x16, dtype):
    if dtype == "f16":
        return _t(x16), x16.astype(np.float32)
    if dtype == "f32":
        x32 = x16.astype(np.float32) * np.float32(1.0009765)
        return _t(x32), x32
    xb = _t(x16.astype(np.float32)).to(torch.bfloat16)
    return xb, xb.float().cpu().numpy()


@pytest.mark.parametrize("N,K", [(4, 32), (12, 96), (256, 512), (20, 2080), (1028, 4096), (72, 11008), (40, 14336),
                                 (16, 32768), (8, 32736)])
@pytest.mark.parametrize("dtype,clip", [("f16", 1.0), ("f32", 0.9), ("bf16", 1.0)])
def test_w3_fused_quantiser_matches_oracle_and_the_two_calls(N, K, dtype, clip):
    """rcp_quant_w3a4_gemv: x_q, S and the per-level sums bit-exact against the oracle's quantiser + GEMV,
    output bits equal to rcp_rotate_quant_act followed by rcp_w3a4_gemv."""
    _say(f"w3 fused N={N} K={K} {dtype} clip={clip}")
    packed, cb, _, _ = _w3_case(N + K + 1, N, K)
    xd, x32 = _x_as(rcp_synth.activation(6, f"w3fused{K}", 1, K), dtype)
    ref_xq, ref_sc, _ = oracle.quantize_act(x32, clip)
    ref_O, ref_P = oracle.w3a4_gemv(packed, cb, N, K, ref_xq, ref_sc)
    pk, cbd = _t(packed), _t(cb.view(np.float16))
    xq_out = torch.zeros(K // 2, dtype=torch.uint8, device=DEV)
    sc_out = torch.zeros(1, dtype=torch.float16, device=DEV)
    for out_dtype in (torch.float32, torch.float16):
        out, P = rcp.quant_w3a4_gemv(pk, cbd, N, K, xd, clip, out_dtype=out_dtype, xq_out=xq_out, scale_out=sc_out,
                                     want_partial_sums=True)
        torch.cuda.synchronize()
        assert np.array_equal(xq_out.cpu().numpy(), ref_xq.ravel())
        assert np.array_equal(sc_out.cpu().numpy().view(np.uint16), ref_sc)
        assert np.array_equal(P.cpu().numpy(), ref_P)
        got = out.cpu().numpy().astype(np.float64).ravel()
        cond = _f16(ref_sc)[0] * (np.abs(_f16(cb)) * np.abs(ref_P)).sum(axis=1)
        half = 2.0 ** -11 * np.abs(ref_O) if out_dtype == torch.float16 else 0.0
        assert np.all(np.abs(got - ref_O) <= 1e-3 * cond + half + 1e-30)
        xq2, sc2 = rcp.rotate_quant_act(xd, None, clip)
        two = rcp.w3a4_gemv(pk, cbd, N, K, xq2, sc2, out_dtype=out_dtype)
        one = rcp.quant_w3a4_gemv(pk, cbd, N, K, xd, clip, out_dtype=out_dtype)     # without the optional outputs
        torch.cuda.synchronize()
        assert torch.equal(out, two) and torch.equal(one, two)


@pytest.mark.parametrize("lanes,blocks", [(128, 0), (256, 3), (64, 1)])
def test_w3_fused_quantiser_other_work_splits(lanes, blocks):
    _say(f"w3 fused lanes={lanes} blocks={blocks}")
    rcp.set_option("gemv_lanes", lanes)
    rcp.set_option("gemv_blocks", blocks)
    N, K = 1028, 11008
    packed, cb, _, _ = _w3_case(9, N, K)
    xd, x32 = _x_as(rcp_synth.activation(9, "w3fusedsplit", 1, K), "f16")
    ref_xq, ref_sc, _ = oracle.quantize_act(x32, 1.0)
    _, ref_P = oracle.w3a4_gemv(packed, cb, N, K, ref_xq, ref_sc)
    _, P = rcp.quant_w3a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, xd, 1.0, out_dtype=torch.float32,
                               want_partial_sums=True)
    torch.cuda.synchronize()
    assert np.array_equal(P.cpu().numpy(), ref_P)


@pytest.mark.parametrize("N,K", [(4096, 4096), (11008, 4096), (4096, 11008)])
def test_w3_full_size_as_benchmarked(N, K):
    _say(f"w3 full size N={N} K={K}")
    packed, cb, xq, sc = _w3_case(5, N, K)
    _check_w3(packed, cb, N, K, xq, sc, torch.float16)
    # the fused call on the same weights
    xd, x32 = _x_as(rcp_synth.activation(5, f"w3full{K}", 1, K), "f16")
    ref_xq, ref_sc, _ = oracle.quantize_act(x32, 1.0)
    ref_O, ref_P = oracle.w3a4_gemv(packed, cb, N, K, ref_xq, ref_sc)
    out, P = rcp.quant_w3a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, xd, 1.0, want_partial_sums=True)
    torch.cuda.synchronize()
    assert np.array_equal(P.cpu().numpy(), ref_P)
    got = out.float().cpu().numpy().astype(np.float64).ravel()
    assert np.linalg.norm(got - ref_O) <= 1e-3 * np.linalg.norm(ref_O) + 1e-30


def test_w3_argument_errors():
    N, K = 8, 64
    W = torch.zeros((N, K), dtype=torch.float16, device=DEV)
    v = torch.zeros(N, dtype=torch.float32, device=DEV)
    good = rcp_synth.normal_quantile_grid()
    for bad in (good[::-1], np.array([0, 0, 1, 2, 3, 4, 5, 6], np.float32),
                np.array([-1, 0, 1, 2, 3, 4, 5, np.inf], np.float32), np.array([np.nan] + [1, 2, 3, 4, 5, 6, 7], np.float32)):
        with pytest.raises(rcp.RcpError):
            rcp.pack_weights_w3(W, v, v, v, bad)
    packed, cb = rcp.pack_weights_w3(W, v, v + 1, v + 0.5, good)
    xq = torch.zeros(K // 2, dtype=torch.uint8, device=DEV)
    sc = torch.ones(1, dtype=torch.float16, device=DEV)
    with pytest.raises(rcp.RcpError):
        rcp.w3a4_gemv(packed, cb, 6, K, xq, sc)
    with pytest.raises(rcp.RcpError):
        rcp.w3a4_gemv(packed, cb, N, 48, xq, sc)
    out = rcp.w3a4_gemv(packed, cb, N, K, xq, sc)
    torch.cuda.synchronize()
    assert not out.any()


def test_w3_large_matrix_as_benchmarked():
    """131072 x 4096 (the bench line's `large_matrix.other_kernels.w3a4`): the launch configuration that size selects,
    every output against the oracle.  Any byte string is a valid packed matrix, so the weights are random bytes."""
    N, K = 131072, 4096
    _say("w3 large matrix 131072 x 4096")
    rng = np.random.default_rng(133)
    packed = rng.integers(0, 256, size=3 * N * K // 8, dtype=np.uint8)
    cb = np.sort(rng.standard_normal((N, 8)) * 0.03, axis=1).astype(np.float16).view(np.uint16)
    q = rcp_synth.random_int4(133, "w3large", 1, K)
    sc = np.array([0.07], np.float16).view(np.uint16)
    _check_w3(packed, cb, N, K, _nibbles(q), sc, torch.float32)
