"""GPU-vs-oracle parity through the C ABI (python binding = argument marshalling only).

Bars: packed bytes, LUT bit patterns, per-level int32 partial sums and (for pure Hadamard
sizes) the quantised activations are bit-exact; floating-point outputs are within 1e-3
(norm-wise, and per element relative to s * sum_l |LUT_l| |P_l|) of the fp64 oracle.
"""
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
    for k in ("gemv_lanes", "gemv_blocks", "gemv_unroll", "gemv_variant", "gemm_waves", "gemv_waves", "gemm_rows", "gemv_oneshot",
              "gemm_stage", "gemv_nt"):
        rcp.set_option(k, 0)


# ------------------------------------------------------------------------------------------
# pack / unpack
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("N,K,dtype", [(256, 512, "f16"), (12, 96, "f16"), (4, 32, "f32"), (36, 2080, "bf16"),
                                       (1024, 4096, "f16"), (64, 11008, "f16")])
def test_pack_weights_bit_exact(N, K, dtype):
    _say(f"pack N={N} K={K} {dtype}")
    W, lo, hi, part = rcp_synth.linear_layer(1, f"pack{N}x{K}", N, K)
    if dtype == "f16":
        Wd, W32 = _t(W), W.astype(np.float32)
    elif dtype == "f32":
        W32 = (W.astype(np.float32) * np.float32(1.0009765))  # values off the fp16 grid
        Wd = _t(W32)
    else:
        Wd = _t(W.astype(np.float32)).to(torch.bfloat16)
        W32 = Wd.to(torch.float32).cpu().numpy()
    packed, cb = rcp.pack_weights(Wd, _t(lo), _t(hi), _t(part))
    idx = rcp.unpack_indices(packed, N, K)
    torch.cuda.synchronize()
    ref_packed, ref_cb, ref_idx = oracle.pack_weights(W32, lo, hi, part, want_idx=True)
    assert np.array_equal(cb.cpu().numpy().view(np.uint16), ref_cb)
    assert np.array_equal(packed.cpu().numpy(), ref_packed)
    assert np.array_equal(idx.cpu().numpy(), ref_idx)


def test_pack_grid_edge_values():
    """Weights sitting exactly on thresholds, LUT values that are fp16 ties, subnormal levels."""
    N, K = 8, 64
    rng = np.random.default_rng(5)
    lo = np.array([0, -1, -3e-6, -0.3333, 0, -65000, -1e-3, -2.0], np.float32)
    hi = np.array([1, 1, 5e-6, 0.6667, 2049.0 / 1024, 65000, 1e-3, 2.0], np.float32)
    part = np.array([[0.5, 0.25, 0.25]] * 4 + [[0.25, 0.5, 0.25]] * 4, np.float32)
    W = rng.uniform(-1, 1, size=(N, K)).astype(np.float32) * (hi - lo)[:, None]
    for h in range(N):
        T, _ = oracle.ldp_grid(lo[h], hi[h], *part[h])
        W[h, :3] = T
        W[h, 3:6] = np.nextafter(T, np.float32(-np.inf))
    packed, cb = rcp.pack_weights(_t(W), _t(lo), _t(hi), _t(part))
    torch.cuda.synchronize()
    ref_packed, ref_cb = oracle.pack_weights(W, lo, hi, part)
    assert np.array_equal(cb.cpu().numpy().view(np.uint16), ref_cb)
    assert np.array_equal(packed.cpu().numpy(), ref_packed)


# ------------------------------------------------------------------------------------------
# weight-only GEMV (16- / 32-bit activations)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("blocks,lanes", [(0, 0), (2, 64), (0, 128), (3, 256)])
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("N,K", [(4, 32), (12, 96), (256, 512), (20, 2080), (1028, 4096), (72, 11008), (40, 14336),
                                 (8, 32768)])
def test_weight_only_gemv_close_to_oracle(N, K, dtype, blocks, lanes):
    """lanes = 64 / 128 / 256: one, two or four wavefronts per row group; 0: the library's choice."""
    _say(f"weight-only gemv N={N} K={K} {dtype} blocks={blocks} lanes={lanes}")
    rcp.set_option("gemv_blocks", blocks)
    rcp.set_option("gemv_lanes", lanes)
    idx = rcp_synth.random_indices(41, f"wo{N}x{K}", N, K)
    packed = oracle.pack_indices(idx)
    rng = np.random.default_rng(41)
    cb = np.sort(rng.standard_normal((N, 4)) * 0.03, axis=1).astype(np.float16).view(np.uint16)
    x16 = rcp_synth.activation(41, f"wo{K}", 1, K)
    if dtype == "f16":
        xd = _t(x16)
    elif dtype == "bf16":
        xd = _t(x16.astype(np.float32)).to(torch.bfloat16)
    else:
        xd = _t(x16.astype(np.float32) * np.float32(1.0009765))
    x64 = xd.to(torch.float64).cpu().numpy()
    ref = oracle.w2a16_gemv(packed, cb, N, K, x64)[0]
    lut = np.abs(_f16(cb))
    cond = (np.take_along_axis(lut, idx.astype(np.int64), axis=1) * np.abs(x64)).sum(axis=1)
    for out_dtype in (torch.float32, torch.float16):
        out = rcp.w2a16_gemv(_t(packed), _t(cb.view(np.float16)), N, K, xd, out_dtype=out_dtype)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64).ravel()
        half = 2.0 ** -11 * np.abs(ref) if out_dtype == torch.float16 else 0.0
        assert np.all(np.abs(got - ref) <= 1e-3 * cond + half + 1e-30)
        assert np.linalg.norm(got - ref) <= 1e-3 * np.linalg.norm(ref) + 1e-30


def test_weight_only_gemv_equals_w2a4_on_dequantised_int4_activations():
    """x = S*q (S a power of two) is exact in fp16: the weight-only kernel must then agree with the W2A4 kernel."""
    N, K = 512, 4096
    packed, cb, xq, sc = _gemv_case(43, N, K, 1)
    sc[:] = np.array([0.25], np.float16).view(np.uint16)
    q = oracle.unpack_act(xq, 1, K)
    x = (q.astype(np.float32) * 0.25).astype(np.float16)
    o4 = rcp.w2a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, _t(xq), _t(sc.view(np.float16)), 1, out_dtype=torch.float32)
    o16 = rcp.w2a16_gemv(_t(packed), _t(cb.view(np.float16)), N, K, _t(x), out_dtype=torch.float32)
    torch.cuda.synchronize()
    a, b = o4.cpu().numpy().astype(np.float64).ravel(), o16.cpu().numpy().astype(np.float64).ravel()
    assert np.linalg.norm(a - b) <= 1e-4 * np.linalg.norm(a)


# ------------------------------------------------------------------------------------------
# group-wise quantisation units (128 input channels per LUT)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("N,K,dtype", [(8, 128, "f16"), (12, 256, "f32"), (64, 4096, "f16"), (36, 4224, "bf16"),
                                       (16, 11008, "f16"), (8, 14336, "f16"), (4, 32768, "f16")])
def test_grouped_pack_bit_exact(N, K, dtype):
    _say(f"grouped pack N={N} K={K} {dtype}")
    W, lo, hi, part = rcp_synth.linear_layer_grouped(3, f"gpack{N}x{K}", N, K)
    if dtype == "f16":
        Wd, W32 = _t(W), W.astype(np.float32)
    elif dtype == "f32":
        W32 = (W.astype(np.float32) * np.float32(1.0009765))
        Wd = _t(W32)
    else:
        Wd = _t(W.astype(np.float32)).to(torch.bfloat16)
        W32 = Wd.to(torch.float32).cpu().numpy()
    packed, cb = rcp.pack_weights_grouped(Wd, _t(lo), _t(hi), _t(part))
    idx = rcp.unpack_indices_grouped(packed, N, K)
    torch.cuda.synchronize()
    ref_packed, ref_cb, ref_idx = oracle.pack_weights_grouped(W32, lo, hi, part, want_idx=True)
    assert np.array_equal(cb.cpu().numpy().view(np.uint16).ravel(), ref_cb)
    assert np.array_equal(packed.cpu().numpy(), ref_packed)
    assert np.array_equal(idx.cpu().numpy(), ref_idx)


def _grouped_gemv_case(seed, N, K):
    NG = K // 128
    idx = rcp_synth.random_indices(seed, f"ggemv{N}x{K}", N, K)
    q = rcp_synth.random_int4(seed, f"ggemv{K}", 1, K)
    rng = np.random.default_rng(seed)
    # levels in the grouped layout [N/4][NG][4 rows][4], ascending per (row, group)
    cb = np.sort(rng.standard_normal((N // 4, NG, 4, 4)) * 0.03, axis=3).astype(np.float16).view(np.uint16)
    sc = (np.abs(rng.standard_normal(1)) * 0.2 + 0.05).astype(np.float16).view(np.uint16)
    xq = ((q[:, 0::2].astype(np.uint8) & 0xF) | ((q[:, 1::2].astype(np.uint8) & 0xF) << 4)).astype(np.uint8)
    return oracle.pack_indices_grouped(idx), cb, xq, sc


def _check_grouped_gemv(packed, cb, N, K, xq, sc, out_dtype):
    NG = K // 128
    ref_O, ref_P = oracle.w2a4_gemv_grouped(packed, cb.ravel(), N, K, xq, sc)
    out, P = rcp.w2a4_gemv_grouped(_t(packed), _t(cb.view(np.float16)), N, K, _t(xq), _t(sc.view(np.float16)),
                                   out_dtype=out_dtype, want_partial_sums=True)
    torch.cuda.synchronize()
    assert np.array_equal(P.cpu().numpy(), ref_P), "per-group partial sums are not bit-exact"
    got = out.cpu().numpy().astype(np.float64).ravel()
    lut = np.abs(_f16(cb)).reshape(N // 4, NG, 4, 4).transpose(0, 2, 1, 3).reshape(N, NG, 4)
    cond = _f16(sc)[0] * (lut * np.abs(ref_P)).sum(axis=(1, 2))
    half = 2.0 ** -11 * np.abs(ref_O) if out_dtype == torch.float16 else 0.0
    assert np.all(np.abs(got - ref_O) <= 1e-3 * cond + half + 1e-30)
    assert np.linalg.norm(got - ref_O) <= 1e-3 * np.linalg.norm(ref_O) + 1e-30
    out2 = rcp.w2a4_gemv_grouped(_t(packed), _t(cb.view(np.float16)), N, K, _t(xq), _t(sc.view(np.float16)),
                                 out_dtype=out_dtype)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


@pytest.mark.parametrize("blocks", [0, 1, 5])
@pytest.mark.parametrize("N,K", [(4, 128), (8, 256), (36, 4096), (1028, 4096), (72, 11008), (40, 14336), (20, 4224),
                                 (12, 32768)])
@pytest.mark.parametrize("lanes", [32, 64])
def test_grouped_gemv_partial_sums_bit_exact_and_output_close(N, K, blocks, lanes):
    """Both forms of the kernel: a lane owns whole groups (32 lanes per four rows), two lanes share a group (64)."""
    _say(f"grouped gemv N={N} K={K} blocks={blocks} lanes={lanes}")
    rcp.set_option("gemv_blocks", blocks)
    rcp.set_option("gemv_lanes", lanes)
    packed, cb, xq, sc = _grouped_gemv_case(21, N, K)
    _check_grouped_gemv(packed, cb, N, K, xq, sc, torch.float32 if blocks else torch.float16)
    rcp.set_option("gemv_nt", 1)     # the weight loads' cache hint of large matrices, forced
    _check_grouped_gemv(packed, cb, N, K, xq, sc, torch.float32)


@pytest.mark.parametrize("rows", [16, 64])
@pytest.mark.parametrize("waves", [0, 2])
@pytest.mark.parametrize("M", [1, 2, 5, 8, 16])
@pytest.mark.parametrize("N,K", [(4, 128), (68, 256), (1028, 4096), (72, 11008), (40, 14336), (12, 32768)])
def test_grouped_gemm_several_tokens(N, K, M, waves, rows):
    """Group-wise LUTs with M tokens (matrix-core kernel with 64-row and 16-row workgroups; M = 1 takes the
    GEMV unless forced)."""
    _say(f"grouped gemm N={N} K={K} M={M} waves={waves} rows={rows}")
    rcp.set_option("gemm_waves", waves)
    rcp.set_option("gemm_rows", rows)
    if waves:
        rcp.set_option("gemv_variant", 2)   # the matrix-core kernel also for one token
    NG = K // 128
    idx = rcp_synth.random_indices(71, f"ggemm{N}x{K}", N, K)
    q = rcp_synth.random_int4(71 + M, f"ggemm{K}", M, K)
    rng = np.random.default_rng(71)
    cb = np.sort(rng.standard_normal((N // 4, NG, 4, 4)) * 0.03, axis=3).astype(np.float16).view(np.uint16)
    sc = (np.abs(rng.standard_normal(M)) * 0.2 + 0.05).astype(np.float16).view(np.uint16)
    xq = ((q[:, 0::2].astype(np.uint8) & 0xF) | ((q[:, 1::2].astype(np.uint8) & 0xF) << 4)).astype(np.uint8)
    packed = oracle.pack_indices_grouped(idx)
    ref_O, ref_P = oracle.w2a4_gemv_grouped(packed, cb.ravel(), N, K, xq, sc, M=M)
    ref_O, ref_P = ref_O.reshape(M, N), ref_P.reshape(M, N, NG, 4)
    lut = np.abs(_f16(cb)).reshape(N // 4, NG, 4, 4).transpose(0, 2, 1, 3).reshape(N, NG, 4)
    cond = _f16(sc)[:, None] * (lut[None] * np.abs(ref_P)).sum(axis=(2, 3))
    for out_dtype in (torch.float32, torch.float16):
        out, P = rcp.w2a4_gemm_grouped(_t(packed), _t(cb.view(np.float16)), N, K, _t(xq), _t(sc.view(np.float16)), M,
                                       out_dtype=out_dtype, want_partial_sums=True)
        torch.cuda.synchronize()
        assert np.array_equal(P.cpu().numpy(), ref_P), "per-group partial sums are not bit-exact"
        got = out.cpu().numpy().astype(np.float64)
        half = 2.0 ** -11 * np.abs(ref_O) if out_dtype == torch.float16 else 0.0
        assert np.all(np.abs(got - ref_O) <= 1e-3 * cond + half + 1e-30)
        assert np.linalg.norm(got - ref_O) <= 1e-3 * np.linalg.norm(ref_O) + 1e-30
        out2 = rcp.w2a4_gemm_grouped(_t(packed), _t(cb.view(np.float16)), N, K, _t(xq), _t(sc.view(np.float16)), M,
                                     out_dtype=out_dtype)
        torch.cuda.synchronize()
        assert torch.equal(out, out2)


@pytest.mark.parametrize("rows", [16, 64])
def test_grouped_gemm_extreme_activations(rows):
    """q = -8 / +7 everywhere with integer levels: exact integer outputs for all 16 tokens."""
    N, K, M = 64, 14336, 16
    rcp.set_option("gemm_rows", rows)
    NG = K // 128
    idx = rcp_synth.random_indices(73, "ggext", N, K)
    packed = oracle.pack_indices_grouped(idx)
    xq = np.empty((M, K // 2), np.uint8)
    xq[0::2] = 0x88
    xq[1::2] = 0x77
    rng = np.random.default_rng(73)
    cb = np.sort(rng.integers(-3, 4, size=(N // 4, NG, 4, 4)), axis=3).astype(np.float16).view(np.uint16)
    sc = np.full(M, 1.0, np.float16).view(np.uint16)
    ref_O, ref_P = oracle.w2a4_gemv_grouped(packed, cb.ravel(), N, K, xq, sc, M=M)
    out, P = rcp.w2a4_gemm_grouped(_t(packed), _t(cb.view(np.float16)), N, K, _t(xq), _t(sc.view(np.float16)), M,
                                   out_dtype=torch.float32, want_partial_sums=True)
    torch.cuda.synchronize()
    assert np.array_equal(P.cpu().numpy(), ref_P)
    assert np.array_equal(out.cpu().numpy().astype(np.float64), ref_O)


def test_grouped_gemv_extreme_activations_and_integer_levels():
    """q = -8 everywhere (largest magnitude sums) and integer levels: the output is an exact integer."""
    N, K = 24, 11008
    NG = K // 128
    idx = rcp_synth.random_indices(22, "gext", N, K)
    packed = oracle.pack_indices_grouped(idx)
    xq = np.full((1, K // 2), 0x88, np.uint8)
    rng = np.random.default_rng(22)
    cb = np.sort(rng.integers(-3, 4, size=(N // 4, NG, 4, 4)), axis=3).astype(np.float16).view(np.uint16)
    sc = np.array([1.0], np.float16).view(np.uint16)
    ref_O, ref_P = oracle.w2a4_gemv_grouped(packed, cb.ravel(), N, K, xq, sc)
    out, P = rcp.w2a4_gemv_grouped(_t(packed), _t(cb.view(np.float16)), N, K, _t(xq), _t(sc.view(np.float16)),
                                   out_dtype=torch.float32, want_partial_sums=True)
    torch.cuda.synchronize()
    assert np.array_equal(P.cpu().numpy(), ref_P)
    assert np.array_equal(out.cpu().numpy().astype(np.float64).ravel(), ref_O)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("N,K,ratio", [(8, 128, 1.0), (36, 4096, 1.0), (1028, 4096, 0.9), (72, 11008, 1.0), (40, 14336, 1.0),
                                       (16, 16384, 1.0), (8, 32768, 1.0)])
@pytest.mark.parametrize("lanes", [32, 64])
def test_grouped_fused_quantise_gemv_equals_the_two_calls(N, K, ratio, dtype, lanes):
    """One launch (quantiser in the prologue of the grouped GEMV) must give the bits of the two calls."""
    _say(f"grouped fused quant+gemv N={N} K={K} ratio={ratio} {dtype} lanes={lanes}")
    rcp.set_option("gemv_lanes", lanes)
    packed, cb, _, _ = _grouped_gemv_case(61, N, K)
    x16 = rcp_synth.activation(61, f"gfq{K}", 1, K)
    xd = {"f16": _t(x16), "bf16": _t(x16.astype(np.float32)).to(torch.bfloat16),
          "f32": _t(x16.astype(np.float32) * np.float32(1.0009765))}[dtype]
    pk, lv = _t(packed), _t(cb.view(np.float16))
    xq, sc = rcp.rotate_quant_act(xd, None, ratio)
    ref_out, ref_P = rcp.w2a4_gemv_grouped(pk, lv, N, K, xq, sc, out_dtype=torch.float32, want_partial_sums=True)
    xq2 = torch.zeros_like(xq)
    sc2 = torch.zeros_like(sc)
    out, P = rcp.quant_w2a4_gemv_grouped(pk, lv, N, K, xd, ratio, out_dtype=torch.float32, xq_out=xq2, scale_out=sc2,
                                         want_partial_sums=True)
    torch.cuda.synchronize()
    assert torch.equal(xq2, xq) and torch.equal(sc2.view(torch.int16), sc.view(torch.int16))
    assert torch.equal(P, ref_P)
    assert torch.equal(out, ref_out)
    # against the oracle too (x_q, S of non-rotated inputs are bit-exact)
    oxq, osc, _ = oracle.quantize_act(xd.to(torch.float32).cpu().numpy(), ratio)
    assert np.array_equal(xq2.cpu().numpy(), oxq) and np.array_equal(sc2.cpu().numpy().view(np.uint16), osc)
    if K <= 16384:
        out3 = rcp.quant_w2a4_gemv_grouped(pk, lv, N, K, xd, ratio, out_dtype=torch.float32)
        torch.cuda.synchronize()
        assert torch.equal(out3, ref_out)


@pytest.mark.parametrize("N,K", [(64, 4096), (32, 11008)])
def test_grouped_whole_path(N, K):
    """export -> quantise -> grouped GEMV against the oracle doing the same from the same inputs."""
    _say(f"grouped whole path N={N} K={K}")
    W, lo, hi, part = rcp_synth.linear_layer_grouped(4, f"gwhole{N}x{K}", N, K)
    x = rcp_synth.activation(4, f"gwhole{K}", 1, K)
    packed, cb = rcp.pack_weights_grouped(_t(W), _t(lo), _t(hi), _t(part))
    xq, sc = rcp.rotate_quant_act(_t(x))
    out, P = rcp.w2a4_gemv_grouped(packed, cb, N, K, xq, sc, out_dtype=torch.float32, want_partial_sums=True)
    torch.cuda.synchronize()
    ref_packed, ref_cb = oracle.pack_weights_grouped(W.astype(np.float32), lo, hi, part)
    ref_xq, ref_sc, _ = oracle.quantize_act(x.astype(np.float32))
    assert np.array_equal(xq.cpu().numpy(), ref_xq) and np.array_equal(sc.cpu().numpy().view(np.uint16), ref_sc)
    ref_O, ref_P = oracle.w2a4_gemv_grouped(ref_packed, ref_cb, N, K, ref_xq, ref_sc)
    assert np.array_equal(P.cpu().numpy(), ref_P)
    got = out.cpu().numpy().astype(np.float64).ravel()
    assert np.linalg.norm(got - ref_O) <= 1e-3 * np.linalg.norm(ref_O)
    # and close to the unquantised product in the sense the 2-bit grid allows
    exact = W.astype(np.float64) @ x.astype(np.float64).ravel()
    cos = float(got @ exact / (np.linalg.norm(got) * np.linalg.norm(exact)))
    assert cos > 0.7


# ------------------------------------------------------------------------------------------
# GEMV
# ------------------------------------------------------------------------------------------
def _gemv_case(seed, N, K, M):
    idx = rcp_synth.random_indices(seed, f"gemv{N}x{K}", N, K)
    q = rcp_synth.random_int4(seed, f"gemv{M}x{K}", M, K)
    rng = np.random.default_rng(seed)
    cb = np.sort(rng.standard_normal((N, 4)) * 0.03, axis=1).astype(np.float16).view(np.uint16)
    sc = (np.abs(rng.standard_normal(M)) * 0.2 + 0.05).astype(np.float16).view(np.uint16)
    xq = ((q[:, 0::2].astype(np.uint8) & 0xF) | ((q[:, 1::2].astype(np.uint8) & 0xF) << 4)).astype(np.uint8)
    return oracle.pack_indices(idx), cb, xq, sc


def _check_gemv(packed, cb, N, K, xq, sc, M, out_dtype):
    ref_O, ref_P = oracle.w2a4_gemv(packed, cb, N, K, xq, sc, M)
    out, P = rcp.w2a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, _t(xq), _t(sc.view(np.float16)), M,
                           out_dtype=out_dtype, want_partial_sums=True)
    torch.cuda.synchronize()
    assert np.array_equal(P.cpu().numpy(), ref_P), "per-level partial sums are not bit-exact"
    got = out.cpu().numpy().astype(np.float64)
    cond = _f16(sc)[:, None] * (np.abs(_f16(cb))[None, :, :] * np.abs(ref_P)).sum(axis=2)
    half = 2.0 ** -11 * np.abs(ref_O) if out_dtype == torch.float16 else 0.0
    assert np.all(np.abs(got - ref_O) <= 1e-3 * cond + half + 1e-30)
    assert np.linalg.norm(got - ref_O) <= 1e-3 * np.linalg.norm(ref_O) + 1e-30
    # the call without the verification output must give the same numbers
    out2 = rcp.w2a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, _t(xq), _t(sc.view(np.float16)), M,
                         out_dtype=out_dtype)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


@pytest.mark.parametrize("lanes", [0, 16, 32, 64, 128, 256])
@pytest.mark.parametrize("N,K", [(256, 512), (4, 32), (12, 96), (20, 2080), (1028, 4096), (72, 11008), (40, 14336),
                                 (2048, 2048)])
def test_gemv_partial_sums_bit_exact_and_output_close(N, K, lanes):
    _say(f"gemv N={N} K={K} lanes={lanes}")
    rcp.set_option("gemv_lanes", lanes)
    packed, cb, xq, sc = _gemv_case(N + K, N, K, 1)
    _check_gemv(packed, cb, N, K, xq, sc, 1, torch.float32)
    _check_gemv(packed, cb, N, K, xq, sc, 1, torch.float16)


@pytest.mark.parametrize("dtype", ["f16", "f32", "bf16"])
@pytest.mark.parametrize("N,K", [(12, 96), (1028, 4096), (72, 11008), (260, 2080), (4100, 2048)])
def test_gemv_with_non_temporal_weight_loads(N, K, dtype):
    """The form the launcher takes for matrices of 32 MB and more (32 lanes per row group, four loads per stage,
    non-temporal weight loads), forced on small ones: pre-quantised and fused calls, same results."""
    _say(f"gemv non-temporal N={N} K={K} {dtype}")
    rcp.set_option("gemv_lanes", 32)
    rcp.set_option("gemv_unroll", 4)
    rcp.set_option("gemv_nt", 1)
    rcp.set_option("gemv_oneshot", 2)
    packed, cb, xq, sc = _gemv_case(N + K + 5, N, K, 1)
    _check_gemv(packed, cb, N, K, xq, sc, 1, torch.float32 if dtype == "f32" else torch.float16)
    x16 = rcp_synth.activation(5, f"nt{K}", 1, K)
    xd = _t(x16) if dtype == "f16" else _t(x16.astype(np.float32)) if dtype == "f32" else _t(x16.astype(np.float32)).to(torch.bfloat16)
    ref_xq, ref_sc, _ = oracle.quantize_act(xd.to(torch.float32).cpu().numpy(), 1.0)
    ref_O, ref_P = oracle.w2a4_gemv(packed, cb, N, K, ref_xq, ref_sc, 1)
    out, P = rcp.quant_w2a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, xd, 1.0, out_dtype=torch.float32,
                                 want_partial_sums=True)
    torch.cuda.synchronize()
    assert np.array_equal(P.cpu().numpy().reshape(ref_P.shape), ref_P)
    rcp.set_option("gemv_nt", 2)
    out2 = rcp.quant_w2a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, xd, 1.0, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


def test_largest_row_count_the_packer_accepts():
    """N = 262140 (the packer's grid limit) at the smallest K; one more group of rows is refused."""
    N, K = 262140, 32
    idx = rcp_synth.random_indices(9, "maxN", N, K)
    rng = np.random.default_rng(9)
    W = rng.standard_normal((N, K)).astype(np.float16)
    lo = np.full(N, -1.0, np.float32)
    hi = np.full(N, 1.0, np.float32)
    part = np.tile(np.array([0.25, 0.5, 0.25], np.float32), (N, 1))
    packed, cb = rcp.pack_weights(_t(W), _t(lo), _t(hi), _t(part))
    ref_packed, ref_cb = oracle.pack_weights(W.astype(np.float32), lo, hi, part)
    torch.cuda.synchronize()
    assert np.array_equal(packed.cpu().numpy(), ref_packed) and np.array_equal(cb.cpu().numpy().view(np.uint16).ravel(), ref_cb.ravel())
    q = rcp_synth.random_int4(9, "maxN", 1, K)
    xq = ((q[:, 0::2].astype(np.uint8) & 0xF) | ((q[:, 1::2].astype(np.uint8) & 0xF) << 4)).astype(np.uint8)
    sc = np.array([0.5], np.float16).view(np.uint16)
    _check_gemv(ref_packed, ref_cb.reshape(N, 4), N, K, xq, sc, 1, torch.float32)
    with pytest.raises(rcp.RcpError):
        rcp.pack_weights(torch.zeros((N + 4, K), dtype=torch.float16, device=DEV), _t(np.zeros(N + 4, np.float32)),
                         _t(np.ones(N + 4, np.float32)), _t(np.tile(np.array([0.25, 0.5, 0.25], np.float32), (N + 4, 1))))


@pytest.mark.parametrize("lanes,unroll", [(16, 2), (32, 4), (64, 2), (256, 4)])
@pytest.mark.parametrize("blocks", [1, 3, 64])
def test_gemv_grid_stride_with_few_workgroups(blocks, lanes, unroll):
    _say(f"gemv grid-stride blocks={blocks} lanes={lanes} unroll={unroll}")
    rcp.set_option("gemv_blocks", blocks)
    rcp.set_option("gemv_lanes", lanes)
    rcp.set_option("gemv_unroll", unroll)
    N, K = 1028, 1024
    packed, cb, xq, sc = _gemv_case(3, N, K, 1)
    _check_gemv(packed, cb, N, K, xq, sc, 1, torch.float32)


def test_gemv_extreme_activations_and_integer_codebook():
    """q = -8 everywhere with index 3 everywhere drives the accumulators to their largest
    magnitude; an integer codebook makes the fp32 epilogue exact."""
    N, K = 16, 14336
    idx = np.full((N, K), 3, np.uint8)
    idx[1::2] = rcp_synth.random_indices(0, "ext", N // 2, K)
    cb = np.tile(np.array([0, 1, 2, 3], np.float16).view(np.uint16), (N, 1))
    xq = np.full((1, K // 2), 0x88, np.uint8)
    one = np.array([1.0], np.float16).view(np.uint16)
    packed = oracle.pack_indices(idx)
    ref_O, ref_P = oracle.w2a4_gemv(packed, cb, N, K, xq, one, 1)
    out, P = rcp.w2a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, _t(xq), _t(one.view(np.float16)), 1,
                           out_dtype=torch.float32, want_partial_sums=True)
    torch.cuda.synchronize()
    assert np.array_equal(P.cpu().numpy(), ref_P)
    assert np.array_equal(out.cpu().numpy().astype(np.float64), ref_O)
    assert ref_P[0, 0, 3] == -8 * K


@pytest.mark.parametrize("variant", [0, 1, 2])
@pytest.mark.parametrize("M", [2, 3, 4, 7, 8, 16])
@pytest.mark.parametrize("N,K", [(256, 512), (44, 2080), (256, 4096), (32, 11008)])
def test_small_batch_matches_oracle(N, K, M, variant):
    """variant 1: plain-ALU kernel, 2: matrix-core kernel, 0: the library's own choice."""
    _say(f"skinny gemm N={N} K={K} M={M} variant={variant}")
    rcp.set_option("gemv_variant", variant)
    packed, cb, xq, sc = _gemv_case(M * 1000 + N, N, K, M)
    _check_gemv(packed, cb, N, K, xq, sc, M, torch.float32)
    _check_gemv(packed, cb, N, K, xq, sc, M, torch.float16)


@pytest.mark.parametrize("rows", [16, 20, 44, 64])
@pytest.mark.parametrize("waves", [1, 2, 4, 8])
@pytest.mark.parametrize("N,K,M", [(4, 32, 1), (68, 96, 5), (1028, 4096, 16), (132, 14336, 9), (64, 32768, 16), (200, 160, 2),
                                   (24, 4224, 8)])
def test_matrix_core_kernel_shapes_and_workgroup_sizes(N, K, M, waves, rows):
    """Ragged N (not a multiple of the rows of a workgroup), K not a multiple of 128, fewer K steps than wavefronts,
    M = 1; 16-row workgroups and workgroups of 5, 11 and 16 groups of four rows."""
    _say(f"mfma gemm N={N} K={K} M={M} waves={waves} rows={rows}")
    rcp.set_option("gemv_variant", 2)
    rcp.set_option("gemm_waves", waves)
    rcp.set_option("gemm_rows", rows)
    packed, cb, xq, sc = _gemv_case(77 + M, N, K, M)
    for stage in (1, 2):    # one and two 128-column steps per pipeline stage
        rcp.set_option("gemm_stage", stage)
        _check_gemv(packed, cb, N, K, xq, sc, M, torch.float32)


@pytest.mark.parametrize("rows", [16, 64])
def test_matrix_core_kernel_extreme_activations(rows):
    """q = -8 everywhere and q = 7 everywhere: the largest sums the fp32 accumulators must hold exactly."""
    N, K, M = 64, 32768, 16
    rcp.set_option("gemv_variant", 2)
    rcp.set_option("gemm_rows", rows)
    idx = rcp_synth.random_indices(31, "mfma_ext", N, K)
    packed = oracle.pack_indices(idx)
    xq = np.empty((M, K // 2), np.uint8)
    xq[0::2] = 0x88
    xq[1::2] = 0x77
    rng = np.random.default_rng(31)
    cb = np.sort(rng.integers(-3, 4, size=(N, 4)), axis=1).astype(np.float16).view(np.uint16)
    sc = np.full(M, 1.0, np.float16).view(np.uint16)
    ref_O, ref_P = oracle.w2a4_gemv(packed, cb, N, K, xq, sc, M)
    out, P = rcp.w2a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, _t(xq), _t(sc.view(np.float16)), M,
                           out_dtype=torch.float32, want_partial_sums=True)
    torch.cuda.synchronize()
    assert np.array_equal(P.cpu().numpy(), ref_P)
    assert np.array_equal(out.cpu().numpy().astype(np.float64), ref_O)


def _tie_activations(kind, dtype, K):
    """One token whose scaled values sit on or next to the quantiser's rounding boundaries k + 1/2."""
    rng = np.random.default_rng(77 + K)
    if kind == "exact":
        # S = 0.25 exactly (amax 1.75); every other value is an odd multiple of S/2: all of them exact ties
        x = (0.125 * (2 * rng.integers(-7, 7, size=K) + 1)).astype(np.float32)
        x[0] = 1.75
    else:
        # an arbitrary scale; values are (k + 1/2) S rounded to the storage type, and their neighbours one step up or down
        amax = np.float32(3.3711)
        S = np.float16(amax / np.float32(7.0)).astype(np.float32)
        x = ((rng.integers(-7, 7, size=K) + 0.5) * S).astype(np.float32)
        x[0] = amax
    if dtype == "f16":
        x = x.astype(np.float16)
        if kind == "near":
            step = rng.integers(-1, 2, size=K).astype(np.int16)
            step[0] = 0
            x = (x.view(np.int16) + step).view(np.float16)
        return _t(x)
    if dtype == "bf16":
        return _t(x).to(torch.bfloat16)
    if kind == "near":
        x = np.nextafter(x, x + rng.integers(-1, 2, size=K).astype(np.float32), dtype=np.float32)
        x[0] = np.float32(3.3711)
    return _t(x)


@pytest.mark.parametrize("kind", ["exact", "near"])
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("path", ["general", "oneshot", "grouped", "w3", "act"])
@pytest.mark.parametrize("K", [4096, 11008])
def test_fused_quantisers_on_rounding_ties(path, dtype, kind, K):
    """x / S on and around the boundaries k + 1/2: the fused prologues (which resolve ties of 16-bit inputs arithmetically
    and redo 32-bit inputs with the IEEE division) must give the oracle's x_q and S bit for bit."""
    N = 1028
    _say(f"fused quantisers on ties {path} {dtype} {kind} K={K}")
    xd = _tie_activations(kind, dtype, K)
    x32 = xd.to(torch.float32).cpu().numpy().reshape(1, K)
    ref_xq, ref_sc, _ = oracle.quantize_act(x32, 1.0)
    xq = torch.zeros((1, K // 2), dtype=torch.uint8, device=DEV)
    sc = torch.zeros((1,), dtype=torch.float16, device=DEV)
    rng = np.random.default_rng(5)
    if path == "act":  # the quantiser as a launch of its own
        xq, sc = rcp.rotate_quant_act(xd.reshape(1, K))
    elif path in ("general", "oneshot"):
        rcp.set_option("gemv_oneshot", 1 if path == "oneshot" else 2)
        pk = torch.randint(0, 256, (N * K // 4,), dtype=torch.uint8, device=DEV)
        cb = _t(np.sort(rng.standard_normal((N, 4)) * 0.03, axis=1).astype(np.float16))
        rcp.quant_w2a4_gemv(pk, cb, N, K, xd, 1.0, xq_out=xq, scale_out=sc)
    elif path == "grouped":
        pk = torch.randint(0, 256, (N * K // 4,), dtype=torch.uint8, device=DEV)
        cb = _t(np.sort(rng.standard_normal((N // 4, K // 128, 4, 4)) * 0.03, axis=3).astype(np.float16))
        rcp.quant_w2a4_gemv_grouped(pk, cb, N, K, xd, 1.0, xq_out=xq, scale_out=sc)
    else:
        pk = torch.randint(0, 256, (3 * N * K // 8,), dtype=torch.uint8, device=DEV)
        cb = _t(np.sort(rng.standard_normal((N, 8)) * 0.03, axis=1).astype(np.float16))
        rcp.quant_w3a4_gemv(pk, cb, N, K, xd, 1.0, xq_out=xq, scale_out=sc)
    torch.cuda.synchronize()
    assert np.array_equal(sc.cpu().numpy().view(np.uint16), ref_sc)
    assert np.array_equal(xq.cpu().numpy(), ref_xq)


@pytest.mark.parametrize("waves", [0, 4, 8])
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("N,K,ratio", [(256, 512, 1.0), (1028, 4096, 1.0), (40, 2080, 0.9), (64, 11008, 1.0),
                                       (24, 16384, 1.0), (16, 32768, 1.0), (4, 32, 1.0), (2052, 2048, 1.0)])
def test_fused_quantise_gemv_equals_the_two_calls(N, K, ratio, dtype, waves):
    """rcp_quant_w2a4_gemv: x_q, S and P bit-exact against the oracle's quantiser + GEMV, with four and
    with eight wavefronts per workgroup."""
    _say(f"fused N={N} K={K} ratio={ratio} {dtype} waves={waves}")
    rcp.set_option("gemv_waves", waves)
    packed, cb, _, _ = _gemv_case(N * 3 + K, N, K, 1)
    x16 = rcp_synth.activation(5, f"fused{K}", 1, K)
    if dtype == "f16":
        xd = _t(x16)
    elif dtype == "bf16":
        xd = _t(x16.astype(np.float32)).to(torch.bfloat16)
    else:
        xd = _t(x16.astype(np.float32) * np.float32(0.99963))
    x32 = xd.to(torch.float32).cpu().numpy()
    xq = torch.zeros((1, K // 2), dtype=torch.uint8, device=DEV)
    sc = torch.zeros((1,), dtype=torch.float16, device=DEV)
    out, P = rcp.quant_w2a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, xd, ratio, out_dtype=torch.float32,
                                 xq_out=xq, scale_out=sc, want_partial_sums=True)
    torch.cuda.synchronize()
    ref_xq, ref_sc, _ = oracle.quantize_act(x32, ratio)
    assert np.array_equal(sc.cpu().numpy().view(np.uint16), ref_sc)
    assert np.array_equal(xq.cpu().numpy(), ref_xq)
    ref_O, ref_P = oracle.w2a4_gemv(packed, cb, N, K, ref_xq, ref_sc, 1)
    assert np.array_equal(P.cpu().numpy(), ref_P)
    got = out.cpu().numpy().astype(np.float64)
    assert np.linalg.norm(got - ref_O) <= 1e-3 * np.linalg.norm(ref_O) + 1e-30
    if K <= 16384:  # the scratch outputs are optional there, and the result must not depend on them
        out2 = rcp.quant_w2a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, xd, ratio, out_dtype=torch.float32)
        torch.cuda.synchronize()
        assert torch.equal(out, out2)


@pytest.mark.parametrize("oneshot", [1, 2])
@pytest.mark.parametrize("N,K", [(4, 1024), (1028, 1024), (72, 2080), (1028, 4096), (40, 5120), (72, 11008), (40, 14336),
                                 (24, 16384), (1100, 8192)])
def test_oneshot_gemv_partial_sums_bit_exact_and_output_close(N, K, oneshot):
    """The kernel that issues every weight load up front (forced on: 1) and the general kernel on the same
    shapes (2): ragged N, K that fills 1 .. 16 units per lane with a ragged last one."""
    _say(f"one-shot gemv N={N} K={K} oneshot={oneshot}")
    rcp.set_option("gemv_oneshot", oneshot)
    packed, cb, xq, sc = _gemv_case(N + K + 1, N, K, 1)
    _check_gemv(packed, cb, N, K, xq, sc, 1, torch.float32)
    _check_gemv(packed, cb, N, K, xq, sc, 1, torch.float16)


def test_oneshot_gemv_extreme_activations_and_integer_codebook():
    """q = -8 everywhere with index 3 everywhere: the largest accumulator magnitudes, exact integer output."""
    rcp.set_option("gemv_oneshot", 1)
    N, K = 16, 14336
    idx = np.full((N, K), 3, np.uint8)
    idx[1::2] = rcp_synth.random_indices(0, "ext1", N // 2, K)
    cb = np.tile(np.array([0, 1, 2, 3], np.float16).view(np.uint16), (N, 1))
    xq = np.full((1, K // 2), 0x88, np.uint8)
    one = np.array([1.0], np.float16).view(np.uint16)
    packed = oracle.pack_indices(idx)
    ref_O, ref_P = oracle.w2a4_gemv(packed, cb, N, K, xq, one, 1)
    out, P = rcp.w2a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, _t(xq), _t(one.view(np.float16)), 1,
                           out_dtype=torch.float32, want_partial_sums=True)
    torch.cuda.synchronize()
    assert np.array_equal(P.cpu().numpy(), ref_P)
    assert np.array_equal(out.cpu().numpy().astype(np.float64), ref_O)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("N,K,ratio", [(1028, 1024, 1.0), (1028, 4096, 1.0), (40, 2080, 0.9), (64, 11008, 1.0), (24, 16384, 1.0),
                                       (2052, 2048, 1.0)])
def test_oneshot_fused_quantise_gemv_equals_the_two_calls(N, K, ratio, dtype):
    """rcp_quant_w2a4_gemv through the one-shot kernel: x_q, S and P bit-exact against the oracle's quantiser +
    GEMV, and the output bit-identical to the general kernel's."""
    _say(f"one-shot fused N={N} K={K} ratio={ratio} {dtype}")
    packed, cb, _, _ = _gemv_case(N * 5 + K, N, K, 1)
    x16 = rcp_synth.activation(6, f"fused1{K}", 1, K)
    if dtype == "f16":
        xd = _t(x16)
    elif dtype == "bf16":
        xd = _t(x16.astype(np.float32)).to(torch.bfloat16)
    else:
        xd = _t(x16.astype(np.float32) * np.float32(0.99963))
    x32 = xd.to(torch.float32).cpu().numpy()
    res = {}
    for oneshot in (1, 2):
        rcp.set_option("gemv_oneshot", oneshot)
        xq = torch.zeros((1, K // 2), dtype=torch.uint8, device=DEV)
        sc = torch.zeros((1,), dtype=torch.float16, device=DEV)
        out, P = rcp.quant_w2a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, xd, ratio, out_dtype=torch.float32,
                                     xq_out=xq, scale_out=sc, want_partial_sums=True)
        out16 = rcp.quant_w2a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, xd, ratio, out_dtype=torch.float16)
        torch.cuda.synchronize()
        res[oneshot] = (out, P, xq, sc, out16)
    out, P, xq, sc, _ = res[1]
    ref_xq, ref_sc, _ = oracle.quantize_act(x32, ratio)
    assert np.array_equal(sc.cpu().numpy().view(np.uint16), ref_sc)
    assert np.array_equal(xq.cpu().numpy(), ref_xq)
    ref_O, ref_P = oracle.w2a4_gemv(packed, cb, N, K, ref_xq, ref_sc, 1)
    assert np.array_equal(P.cpu().numpy(), ref_P)
    got = out.cpu().numpy().astype(np.float64)
    assert np.linalg.norm(got - ref_O) <= 1e-3 * np.linalg.norm(ref_O) + 1e-30
    for a, b in zip(res[1], res[2]):
        assert torch.equal(a, b), "the one-shot kernel and the general kernel differ"


# ------------------------------------------------------------------------------------------
# activation preparation
# ------------------------------------------------------------------------------------------
def _check_act_against_rotated(y64, xq, sc, ratio):
    """Tie-band criterion: with the kernel's own scale, every code is within 1/2 (+ slack for
    the binary32 rotation) of the exactly rotated value divided by the scale."""
    M, K = y64.shape
    s = _f16(sc)
    a = np.abs(y64).max(axis=1)
    target = ratio * a / 7.0
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(s, 2.0 ** -14))) - 10)
    assert np.all(np.abs(s - target) <= 0.5 * ulp + 1e-5 * target + 1e-12), "scale is not fp16(ratio*amax/7)"
    q = oracle.unpack_act(xq, M, K).astype(np.float64)
    z = np.clip(y64 / s[:, None], -8.5, 7.5)
    slack = 2e-5 * (np.abs(z) + 1.0) * np.sqrt(np.log2(K) + 1)
    assert np.all(np.abs(q - z) <= 0.5 + slack)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("M,K,ratio", [(1, 512, 1.0), (1, 4096, 1.0), (3, 2080, 0.9), (1, 11008, 1.0), (16, 4096, 1.0),
                                       (2, 32768, 1.0), (1, 32, 1.0)])
def test_quantise_without_rotation_bit_exact(M, K, ratio, dtype):
    _say(f"quant M={M} K={K} ratio={ratio} {dtype}")
    x16 = rcp_synth.activation(2, f"q{M}x{K}", M, K)
    if dtype == "f16":
        xd = _t(x16)
    elif dtype == "bf16":
        xd = _t(x16.astype(np.float32)).to(torch.bfloat16)
    else:
        xd = _t(x16.astype(np.float32) * np.float32(1.00037))
    x32 = xd.to(torch.float32).cpu().numpy()
    xq, sc = rcp.rotate_quant_act(xd, None, ratio)
    torch.cuda.synchronize()
    ref_xq, ref_sc, _ = oracle.quantize_act(x32, ratio)
    assert np.array_equal(sc.cpu().numpy().view(np.uint16), ref_sc)
    assert np.array_equal(xq.cpu().numpy(), ref_xq)


@pytest.mark.parametrize("scale_to", [7.0, 7.0 * 0.37109375, 7.0 * 1.3330078125, 7.0 * 3.0e-3])
def test_quantise_at_rounding_boundaries(scale_to):
    """Inputs whose quotient by S sits exactly on n + 1/2 or one or two binary32 steps beside it:
    ties must go to even, neighbours to their side, exactly as the correctly rounded division says."""
    K = 4096
    s = np.float32(np.float16(scale_to / 7.0))            # the S the kernel will derive (amax = scale_to)
    half = np.arange(-8.5, 8.0, 1.0, dtype=np.float32)    # -8.5 .. 7.5
    base = (half * s).astype(np.float32)
    cand = [base]
    for k in (1, 2, 3):
        up, dn = base.copy(), base.copy()
        for _ in range(k):
            up, dn = np.nextafter(up, np.float32(np.inf)), np.nextafter(dn, np.float32(-np.inf))
        cand += [up, dn]
    vals = np.concatenate(cand)
    x = np.zeros((1, K), np.float32)
    x[0, :vals.size] = vals
    x[0, K - 1] = np.float32(scale_to)                    # fixes amax, hence S
    x[0, :vals.size] = np.clip(x[0, :vals.size], -scale_to, scale_to)
    xq, sc = rcp.rotate_quant_act(_t(x), None, 1.0)
    torch.cuda.synchronize()
    ref_xq, ref_sc, _ = oracle.quantize_act(x, 1.0)
    assert np.array_equal(sc.cpu().numpy().view(np.uint16), ref_sc)
    assert np.array_equal(xq.cpu().numpy(), ref_xq)
    packed, cb, _, _ = _gemv_case(77, 8, K, 1)
    xq2 = torch.zeros((1, K // 2), dtype=torch.uint8, device=DEV)
    rcp.quant_w2a4_gemv(_t(packed), _t(cb.view(np.float16)), 8, K, _t(x), 1.0, xq_out=xq2,
                        scale_out=torch.zeros((1,), dtype=torch.float16, device=DEV))
    torch.cuda.synchronize()
    assert np.array_equal(xq2.cpu().numpy(), ref_xq)


def test_quantise_degenerate_inputs():
    K = 4096
    x = np.zeros((3, K), np.float16)
    x[1, 77] = -12.5
    x[2, :] = 6e-8  # fp16 subnormal: the scale underflows and falls back to 1
    xq, sc = rcp.rotate_quant_act(_t(x), None, 1.0)
    torch.cuda.synchronize()
    ref_xq, ref_sc, _ = oracle.quantize_act(x.astype(np.float32), 1.0)
    assert np.array_equal(sc.cpu().numpy().view(np.uint16), ref_sc)
    assert np.array_equal(xq.cpu().numpy(), ref_xq)
    big = np.full((1, K), 3e6, np.float32)
    xq, sc = rcp.rotate_quant_act(_t(big), None, 1.0)
    torch.cuda.synchronize()
    ref_xq, ref_sc, _ = oracle.quantize_act(big, 1.0)
    assert np.array_equal(sc.cpu().numpy().view(np.uint16), ref_sc) and np.array_equal(xq.cpu().numpy(), ref_xq)


@pytest.mark.parametrize("M,n", [(1, 32), (1, 64), (2, 256), (1, 512), (1, 2048), (3, 4096), (1, 8192), (1, 16384)])
def test_hadamard_rotation_bit_exact_against_binary32_butterfly(M, n):
    _say(f"wht M={M} n={n}")
    x = rcp_synth.activation(3, f"wht{M}x{n}", M, n)
    xq, sc = rcp.rotate_quant_act(_t(x), rcp.Rotation.wht(n), 1.0)
    torch.cuda.synchronize()
    y32 = oracle.fwht_f32(x.astype(np.float32))
    ref_xq, ref_sc, _ = oracle.quantize_act(y32, 1.0)
    assert np.array_equal(sc.cpu().numpy().view(np.uint16), ref_sc)
    assert np.array_equal(xq.cpu().numpy(), ref_xq)
    if n <= 8192:  # and against the dense fp64 definition, within the tie band
        y64 = oracle.rotate(x.astype(np.float64), oracle.ROT_WHT, n_wht=n)
        _check_act_against_rotated(np.atleast_2d(y64), xq.cpu().numpy(), sc.cpu().numpy().view(np.uint16), 1.0)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
@pytest.mark.parametrize("M,n,m,ratio", [(1, 64, 172, 1.0), (1, 512, 28, 1.0), (2, 8, 12, 0.9), (1, 2, 16, 1.0),
                                         (3, 64, 172, 1.0), (1, 128, 172, 1.0), (2, 1024, 16, 0.9)])
def test_kronecker_rotation_within_tie_band(M, n, m, ratio, dtype):
    _say(f"kron M={M} n={n} m={m} {dtype}")
    K = n * m
    Q = rcp_synth.orthogonal(1, m)
    x = rcp_synth.activation(4, f"kron{M}x{K}", M, K)
    xd = _t(x) if dtype == "f16" else _t(x.astype(np.float32))
    xq, sc = rcp.rotate_quant_act(xd, rcp.Rotation.kron(n, _t(Q)), ratio)
    torch.cuda.synchronize()
    y64 = oracle.rotate(x.astype(np.float64), oracle.ROT_KRON, n_wht=n, m=m, Q=Q.astype(np.float64))
    _check_act_against_rotated(np.atleast_2d(y64), xq.cpu().numpy(), sc.cpu().numpy().view(np.uint16), ratio)


@pytest.mark.parametrize("kind,M,n,m", [("none", 2, 2080, 1), ("wht", 1, 64, 1), ("wht", 2, 4096, 1), ("wht", 1, 16384, 1),
                                        ("kron", 1, 64, 172), ("kron", 2, 512, 28), ("kron", 1, 128, 12),
                                        ("kron", 1, 1024, 8), ("kron", 1, 8, 12), ("kron", 1, 64, 7),
                                        # 64 Hadamard rows, the form with one workgroup per output column: smallest and
                                        # largest Q, uneven shares of the four wavefronts, several tokens; 32 rows
                                        # fall outside it
                                        ("kron", 3, 64, 16), ("kron", 2, 64, 20), ("kron", 1, 64, 256), ("kron", 1, 64, 12),
                                        ("kron", 16, 64, 172), ("kron", 1, 32, 256),
                                        # too many columns per wavefront for that form: one wavefront per column, token in LDS
                                        ("kron", 2, 128, 172), ("kron", 1, 512, 36), ("kron", 1, 256, 68)])
def test_rotation_only_entry_point(kind, M, n, m):
    _say(f"rotate-only {kind} M={M} n={n} m={m}")
    K = n * m
    x = rcp_synth.activation(6, f"rot{kind}{K}", M, K)
    if kind == "none":
        y = rcp.rotate_act(_t(x), None)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), x.astype(np.float32))
        return
    if kind == "wht":
        y = rcp.rotate_act(_t(x), rcp.Rotation.wht(n))
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), oracle.fwht_f32(x.astype(np.float32)))  # same binary32 butterfly
        return
    Q = rcp_synth.orthogonal(2, m)
    y = rcp.rotate_act(_t(x), rcp.Rotation.kron(n, _t(Q)))
    torch.cuda.synchronize()
    y64 = np.atleast_2d(oracle.rotate(x.astype(np.float64), oracle.ROT_KRON, n_wht=n, m=m, Q=Q.astype(np.float64)))
    scale = np.linalg.norm(x.astype(np.float64), axis=1, keepdims=True)
    assert np.all(np.abs(y.cpu().numpy().astype(np.float64) - y64) <= 2e-6 * scale)


# ------------------------------------------------------------------------------------------
# whole path
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("M,n,m,ratio", [(1, 32, 128, 1.0), (3, 8, 64, 0.9), (1, 64, 128, 1.0), (2, 2, 16, 1.0), (1, 32, 64, 1.0),
                                         (16, 32, 128, 1.0), (1, 64, 256, 1.0)])
def test_heads_rotation_bit_exact_against_binary32_butterfly(M, n, m, ratio, dtype):
    """y = (H_n (x) I_m) x with binary32 butterflies in ascending stride order per column: x_q, S and
    the rotation-only output must equal the oracle's bit for bit."""
    _say(f"heads rotation M={M} n={n} m={m} ratio={ratio} {dtype}")
    K = n * m
    x16 = rcp_synth.activation(81, f"heads{K}", M, K)
    xd = {"f16": _t(x16), "bf16": _t(x16.astype(np.float32)).to(torch.bfloat16),
          "f32": _t(x16.astype(np.float32) * np.float32(1.0009765))}[dtype]
    x32 = xd.to(torch.float32).cpu().numpy()
    rot = rcp.Rotation.heads(n, m)
    xq, sc = rcp.rotate_quant_act(xd, rot, ratio)
    y = rcp.rotate_act(xd, rot)
    torch.cuda.synchronize()
    # oracle: order-n butterflies on every column of the n x m view
    y32 = np.stack([oracle.fwht_f32(x32[t].reshape(n, m).T.copy()).T.reshape(K) for t in range(M)])
    assert np.array_equal(y.cpu().numpy(), y32)
    ref_xq, ref_sc, _ = oracle.quantize_act(y32, ratio)
    assert np.array_equal(sc.cpu().numpy().view(np.uint16), ref_sc)
    assert np.array_equal(xq.cpu().numpy(), ref_xq)
    # and the binary32 result is the dense binary64 definition within binary32 bounds
    y64 = oracle.rotate(x32.astype(np.float64), oracle.ROT_HEADS, n_wht=n, m=m)
    assert np.all(np.abs(y32 - y64) <= 16 * 2.0 ** -24 * np.abs(x32).reshape(M, n, m).sum(axis=1).max())


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("N,n,m,ratio", [(1028, 32, 128, 1.0), (64, 8, 64, 0.9), (256, 64, 128, 1.0), (16, 2, 16, 1.0),
                                         (4096, 32, 128, 1.0), (40, 64, 256, 1.0)])
def test_fused_heads_rotation_quantise_gemv_equals_the_separate_calls(N, n, m, ratio, dtype):
    """Rotation across heads + quantiser + GEMV in one launch: the bits of rcp_rotate_quant_act + rcp_w2a4_gemv."""
    _say(f"fused heads rotation N={N} n={n} m={m} ratio={ratio} {dtype}")
    K = n * m
    packed, cb, _, _ = _gemv_case(91, N, K, 1)
    x16 = rcp_synth.activation(91, f"fh{K}", 1, K)
    xd = {"f16": _t(x16), "bf16": _t(x16.astype(np.float32)).to(torch.bfloat16),
          "f32": _t(x16.astype(np.float32) * np.float32(1.0009765))}[dtype]
    pk, lv = _t(packed), _t(cb.view(np.float16))
    rot = rcp.Rotation.heads(n, m)
    xq, sc = rcp.rotate_quant_act(xd, rot, ratio)
    ref_out, ref_P = rcp.w2a4_gemv(pk, lv, N, K, xq, sc, 1, out_dtype=torch.float32, want_partial_sums=True)
    xq2, sc2 = torch.zeros_like(xq), torch.zeros_like(sc)
    out, P = rcp.rotate_quant_w2a4_gemv(pk, lv, N, K, xd, rot, ratio, out_dtype=torch.float32, xq_out=xq2, scale_out=sc2,
                                        want_partial_sums=True)
    torch.cuda.synchronize()
    assert torch.equal(xq2, xq) and torch.equal(sc2.view(torch.int16), sc.view(torch.int16))
    assert torch.equal(P, ref_P) and torch.equal(out, ref_out)
    # no rotation given: the plain fused call
    o1 = rcp.rotate_quant_w2a4_gemv(pk, lv, N, K, xd, None, ratio, out_dtype=torch.float32)
    o2 = rcp.quant_w2a4_gemv(pk, lv, N, K, xd, ratio, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2)
    if n * m == 4096:
        with pytest.raises(rcp.RcpError):
            rcp.rotate_quant_w2a4_gemv(pk, lv, N, K, xd, rcp.Rotation.wht(K), ratio)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("N,K,ratio", [(256, 512, 1.0), (64, 32, 1.0), (1028, 64, 0.9), (40, 128, 1.0), (2048, 2048, 1.0),
                                       (516, 1024, 0.9), (8192, 2048, 1.0), (12, 256, 1.0)])
def test_fused_short_hadamard_rotation_quantise_gemv(N, K, ratio, dtype):
    """The order-K Hadamard rotation (K <= 2048) inside the fused quantise+GEMV launch: x_q and S bit-exact against the
    oracle's binary32 butterfly + quantiser, P bit-exact against the oracle's GEMV, and every bit equal to the two
    separate calls."""
    _say(f"fused short WHT N={N} K={K} ratio={ratio} {dtype}")
    packed, cb, _, _ = _gemv_case(93, N, K, 1)
    x16 = rcp_synth.activation(93, f"fw{K}", 1, K)
    xd = {"f16": _t(x16), "bf16": _t(x16.astype(np.float32)).to(torch.bfloat16),
          "f32": _t(x16.astype(np.float32) * np.float32(1.0009765))}[dtype]
    x32 = xd.to(torch.float32).cpu().numpy()
    pk, lv = _t(packed), _t(cb.view(np.float16))
    rot = rcp.Rotation.wht(K)
    xq, sc = rcp.rotate_quant_act(xd, rot, ratio)
    ref_out, ref_P = rcp.w2a4_gemv(pk, lv, N, K, xq, sc, 1, out_dtype=torch.float32, want_partial_sums=True)
    xq2, sc2 = torch.zeros_like(xq), torch.zeros_like(sc)
    out, P = rcp.rotate_quant_w2a4_gemv(pk, lv, N, K, xd, rot, ratio, out_dtype=torch.float32, xq_out=xq2, scale_out=sc2,
                                        want_partial_sums=True)
    o16 = rcp.rotate_quant_w2a4_gemv(pk, lv, N, K, xd, rot, ratio, out_dtype=torch.float16)
    r16 = rcp.w2a4_gemv(pk, lv, N, K, xq, sc, 1, out_dtype=torch.float16)
    torch.cuda.synchronize()
    oxq, osc, _ = oracle.quantize_act(oracle.fwht_f32(x32), ratio)
    assert np.array_equal(xq2.cpu().numpy(), oxq) and np.array_equal(sc2.cpu().numpy().view(np.uint16), osc)
    assert torch.equal(xq2, xq) and torch.equal(sc2.view(torch.int16), sc.view(torch.int16))
    _, oP = oracle.w2a4_gemv(packed, cb, N, K, oxq, osc, 1)
    assert np.array_equal(P.cpu().numpy(), oP)
    assert torch.equal(P, ref_P) and torch.equal(out, ref_out) and torch.equal(o16, r16)


def test_long_hadamard_rotation_is_not_fused():
    pk = torch.zeros(64 * 4096 // 4, dtype=torch.uint8, device=DEV)
    lv = torch.zeros((64, 4), dtype=torch.float16, device=DEV)
    x = torch.zeros((1, 4096), dtype=torch.float16, device=DEV)
    with pytest.raises(rcp.RcpError) as e:
        rcp.rotate_quant_w2a4_gemv(pk, lv, 64, 4096, x, rcp.Rotation.wht(4096), 1.0)
    assert e.value.code == -4


def test_heads_rotation_argument_errors():
    x = torch.zeros((1, 4096), dtype=torch.float16, device=DEV)
    for n, m in ((128, 32), (32, 100), (3, 1024)):
        with pytest.raises((rcp.RcpError, AssertionError)):
            rcp.rotate_quant_act(torch.zeros((1, n * m), dtype=torch.float16, device=DEV), rcp.Rotation.heads(n, m))
    with pytest.raises(rcp.RcpError):
        rcp.rotate_quant_act(x, rcp.Rotation.heads(32, 64))       # 32 * 64 != 4096


def _rotation(rot, seed):
    if rot is None:
        return None, dict(kind=oracle.ROT_NONE)
    if rot[0] == "wht":
        return rcp.Rotation.wht(rot[1]), dict(kind=oracle.ROT_WHT, n_wht=rot[1])
    Q = rcp_synth.orthogonal(seed, rot[2])
    return rcp.Rotation.kron(rot[1], _t(Q)), dict(kind=oracle.ROT_KRON, n_wht=rot[1], m=rot[2], Q=Q.astype(np.float64))


@pytest.mark.parametrize("config,rows", [("tiny", None), ("llama32_1b", 96), ("llama2_7b", 64), ("llama3_8b", 64)])
def test_whole_path_on_config_shapes(config, rows):
    """pack -> rotate+quantise -> GEMV on the GPU; the oracle takes the same steps, except that
    its GEMV consumes the GPU's (x_q, S) so that a legal tie flip upstream cannot leak in.
    Full K always; `rows` output rows of each layer (None = all) keep the CPU side short."""
    for name, N, K, rot in rcp_synth.CONFIGS[config]:
        n = N if rows is None else rows
        _say(f"path {config}/{name} N={n} (of {N}) K={K} rot={rot}")
        W, lo, hi, part = rcp_synth.linear_layer(0, f"{config}/{name}", n, K)
        x = rcp_synth.activation(0, f"{config}/{name}", 1, K)
        grot, orot = _rotation(rot, 0)
        packed, cb = rcp.pack_weights(_t(W), _t(lo), _t(hi), _t(part))
        xq, sc = rcp.rotate_quant_act(_t(x), grot, 1.0)
        out, P = rcp.w2a4_gemv(packed, cb, n, K, xq, sc, 1, out_dtype=torch.float16, want_partial_sums=True)
        torch.cuda.synchronize()
        ref_packed, ref_cb = oracle.pack_weights(W.astype(np.float32), lo, hi, part)
        assert np.array_equal(packed.cpu().numpy(), ref_packed)
        assert np.array_equal(cb.cpu().numpy().view(np.uint16), ref_cb)
        xq_h, sc_h = xq.cpu().numpy(), sc.cpu().numpy().view(np.uint16)
        y64 = oracle.rotate(x.astype(np.float64), **orot)
        _check_act_against_rotated(np.atleast_2d(y64), xq_h, sc_h, 1.0)
        ref_O, ref_P = oracle.w2a4_gemv(ref_packed, ref_cb, n, K, xq_h, sc_h, 1)
        assert np.array_equal(P.cpu().numpy(), ref_P)
        got = out.cpu().numpy().astype(np.float64)
        assert np.linalg.norm(got - ref_O) <= 1e-3 * np.linalg.norm(ref_O)


# ------------------------------------------------------------------------------------------
# full sizes, in the launch configuration the benchmark times
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name,N,K,rotated", [("qkv", 12288, 4096, False), ("o", 4096, 4096, False),
                                              ("gate_up", 22016, 4096, False), ("down", 4096, 11008, True)])
def test_full_size_llama2_7b_launches_as_benchmarked(name, N, K, rotated):
    """The four launches of a LLaMA-2-7B layer at full size, default work distribution, the calls bench.py makes
    (rcp_rotate_act for the down input, then the fused quantise+GEMV): packed bytes, LUT, x_q / S (plain inputs) and
    all N x 4 partial sums bit-exact, every output within the bar; the oracle runs the whole matrix."""
    _say(f"full size {name} {N}x{K}")
    W, lo, hi, part = rcp_synth.linear_layer(7, f"full/{name}", N, K)
    x = rcp_synth.activation(7, f"full/{name}", 1, K)
    packed, cb = rcp.pack_weights(_t(W), _t(lo), _t(hi), _t(part))
    xq = torch.empty((1, K // 2), dtype=torch.uint8, device=DEV)
    sc = torch.empty((1,), dtype=torch.float16, device=DEV)
    if rotated:
        Q = rcp_synth.orthogonal(7, 172)
        rot = rcp.Rotation.kron(64, _t(Q))
        y = rcp.rotate_act(_t(x), rot)
        out, P = rcp.quant_w2a4_gemv(packed, cb, N, K, y, 1.0, out_dtype=torch.float16, xq_out=xq, scale_out=sc,
                                     want_partial_sums=True)
    else:
        out, P = rcp.quant_w2a4_gemv(packed, cb, N, K, _t(x), 1.0, out_dtype=torch.float16, xq_out=xq, scale_out=sc,
                                     want_partial_sums=True)
    torch.cuda.synchronize()
    ref_packed, ref_cb = oracle.pack_weights(W.astype(np.float32), lo, hi, part)
    assert np.array_equal(packed.cpu().numpy(), ref_packed)
    assert np.array_equal(cb.cpu().numpy().view(np.uint16), ref_cb)
    xq_h, sc_h = xq.cpu().numpy(), sc.cpu().numpy().view(np.uint16)
    if rotated:
        y64 = oracle.rotate(x.astype(np.float64), oracle.ROT_KRON, n_wht=64, m=172, Q=Q.astype(np.float64))
        _check_act_against_rotated(np.atleast_2d(y64), xq_h, sc_h, 1.0)
    else:
        oxq, osc, _ = oracle.quantize_act(x.astype(np.float32), 1.0)
        assert np.array_equal(xq_h, oxq) and np.array_equal(sc_h, osc)
    ref_O, ref_P = oracle.w2a4_gemv(ref_packed, ref_cb, N, K, xq_h, sc_h, 1)
    assert np.array_equal(P.cpu().numpy(), ref_P)
    got = out.cpu().numpy().astype(np.float64)
    cond = _f16(sc_h)[:, None] * (np.abs(_f16(ref_cb))[None, :, :] * np.abs(ref_P)).sum(axis=2)
    assert np.all(np.abs(got - ref_O) <= 1e-3 * cond + 2.0 ** -11 * np.abs(ref_O) + 1e-30)
    assert np.linalg.norm(got - ref_O) <= 1e-3 * np.linalg.norm(ref_O)


@pytest.mark.parametrize("config,name,N,K,rot", [
    ("llama32_1b", "q_o", 2048, 2048, None), ("llama32_1b", "gate_up", 8192, 2048, None),
    ("llama32_1b", "down", 2048, 8192, ("wht", 8192)),
    ("llama3_8b", "k_v", 1024, 4096, None), ("llama3_8b", "gate_up", 14336, 4096, None),
    ("llama3_8b", "down", 4096, 14336, ("kron", 512, 28))])
def test_full_size_llama32_1b_and_llama3_8b_layers_as_benchmarked(config, name, N, K, rot):
    """The layer sizes of the LLaMA-3.2-1B and LLaMA-3-8B configurations at full size through the calls the benchmark
    times: plain inputs -> fused quantise+GEMV; order-8192 Hadamard -> rcp_rotate_quant_act (bit-exact against the
    binary32 butterfly) then the GEMV; H_512 (x) Q_28 -> rcp_rotate_act then the fused quantise+GEMV.  Packed bytes,
    LUT and all N x 4 partial sums bit-exact against the oracle on the whole matrix, every output inside the bar."""
    _say(f"full size {config}/{name} {N}x{K} rot={rot}")
    W, lo, hi, part = rcp_synth.linear_layer(11, f"full/{config}/{name}", N, K)
    x = rcp_synth.activation(11, f"full/{config}/{name}", 1, K)
    packed, cb = rcp.pack_weights(_t(W), _t(lo), _t(hi), _t(part))
    xq = torch.empty((1, K // 2), dtype=torch.uint8, device=DEV)
    sc = torch.empty((1,), dtype=torch.float16, device=DEV)
    if rot is None:
        out, P = rcp.quant_w2a4_gemv(packed, cb, N, K, _t(x), 1.0, out_dtype=torch.float16, xq_out=xq, scale_out=sc,
                                     want_partial_sums=True)
    elif rot[0] == "wht":
        rcp.rotate_quant_act(_t(x), rcp.Rotation.wht(K), 1.0, xq_out=xq, scale_out=sc)
        out, P = rcp.w2a4_gemv(packed, cb, N, K, xq, sc, 1, out_dtype=torch.float16, want_partial_sums=True)
    else:
        Q = rcp_synth.orthogonal(11, rot[2])
        y = rcp.rotate_act(_t(x), rcp.Rotation.kron(rot[1], _t(Q)))
        out, P = rcp.quant_w2a4_gemv(packed, cb, N, K, y, 1.0, out_dtype=torch.float16, xq_out=xq, scale_out=sc,
                                     want_partial_sums=True)
    torch.cuda.synchronize()
    ref_packed, ref_cb = oracle.pack_weights(W.astype(np.float32), lo, hi, part)
    assert np.array_equal(packed.cpu().numpy(), ref_packed)
    assert np.array_equal(cb.cpu().numpy().view(np.uint16), ref_cb)
    xq_h, sc_h = xq.cpu().numpy(), sc.cpu().numpy().view(np.uint16)
    if rot is None:
        oxq, osc, _ = oracle.quantize_act(x.astype(np.float32), 1.0)
        assert np.array_equal(xq_h, oxq) and np.array_equal(sc_h, osc)
    elif rot[0] == "wht":
        oxq, osc, _ = oracle.quantize_act(oracle.fwht_f32(x.astype(np.float32)), 1.0)
        assert np.array_equal(xq_h, oxq) and np.array_equal(sc_h, osc)
    else:
        y64 = oracle.rotate(x.astype(np.float64), oracle.ROT_KRON, n_wht=rot[1], m=rot[2], Q=Q.astype(np.float64))
        _check_act_against_rotated(np.atleast_2d(y64), xq_h, sc_h, 1.0)
    ref_O, ref_P = oracle.w2a4_gemv(ref_packed, ref_cb, N, K, xq_h, sc_h, 1)
    assert np.array_equal(P.cpu().numpy(), ref_P)
    got = out.cpu().numpy().astype(np.float64)
    cond = _f16(sc_h)[:, None] * (np.abs(_f16(ref_cb))[None, :, :] * np.abs(ref_P)).sum(axis=2)
    assert np.all(np.abs(got - ref_O) <= 1e-3 * cond + 2.0 ** -11 * np.abs(ref_O) + 1e-30)
    assert np.linalg.norm(got - ref_O) <= 1e-3 * np.linalg.norm(ref_O)


@pytest.mark.parametrize("N,K,M", [(4096, 4096, 8), (4096, 4096, 16), (4096, 11008, 8), (12288, 4096, 8)])
def test_full_size_small_batch_other_layers_match_oracle(N, K, M):
    """The out-projection and the down projection of a 7B layer with several tokens (4096 rows: the matrix-core
    kernel's 16-row workgroups; 8 tokens: low and high activation parts share one B operand), and q|k|v at 8 tokens,
    at full size with the automatic choice of kernel: P bit-exact, O within the bar."""
    _say(f"full size small batch {N}x{K} M={M}")
    idx = rcp_synth.random_indices(12, f"fullsb{N}x{K}", N, K)
    packed = oracle.pack_indices(idx)
    rng = np.random.default_rng(12)
    cb = np.sort(rng.standard_normal((N, 4)) * 0.03, axis=1).astype(np.float16).view(np.uint16)
    x = rcp_synth.activation(12, f"fullsb{N}x{K}", M, K)
    xq, sc = rcp.rotate_quant_act(_t(x))
    out, P = rcp.w2a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, xq, sc, M, out_dtype=torch.float16, want_partial_sums=True)
    torch.cuda.synchronize()
    xq_h, sc_h = xq.cpu().numpy(), sc.cpu().numpy().view(np.uint16)
    oxq, osc, _ = oracle.quantize_act(x.astype(np.float32), 1.0)
    assert np.array_equal(xq_h, oxq) and np.array_equal(sc_h, osc)
    ref_O, ref_P = oracle.w2a4_gemv(packed, cb, N, K, xq_h, sc_h, M)
    assert np.array_equal(P.cpu().numpy(), ref_P)
    got = out.cpu().numpy().astype(np.float64)
    assert np.linalg.norm(got - ref_O) <= 1e-3 * np.linalg.norm(ref_O)


@pytest.mark.parametrize("M", [4, 16])
def test_full_size_small_batch_layer_matches_oracle(M):
    """gate|up of a 7B layer (22016 x 4096) with M tokens as the benchmark runs it: P bit-exact, O within the bar."""
    N, K = 22016, 4096
    _say(f"full size small batch M={M}")
    idx = rcp_synth.random_indices(8, "fullsb", N, K)
    packed = oracle.pack_indices(idx)
    rng = np.random.default_rng(8)
    cb = np.sort(rng.standard_normal((N, 4)) * 0.03, axis=1).astype(np.float16).view(np.uint16)
    x = rcp_synth.activation(8, "fullsb", M, K)
    xq, sc = rcp.rotate_quant_act(_t(x))
    out, P = rcp.w2a4_gemv(_t(packed), _t(cb.view(np.float16)), N, K, xq, sc, M, out_dtype=torch.float16, want_partial_sums=True)
    torch.cuda.synchronize()
    xq_h, sc_h = xq.cpu().numpy(), sc.cpu().numpy().view(np.uint16)
    oxq, osc, _ = oracle.quantize_act(x.astype(np.float32), 1.0)
    assert np.array_equal(xq_h, oxq) and np.array_equal(sc_h, osc)
    ref_O, ref_P = oracle.w2a4_gemv(packed, cb, N, K, xq_h, sc_h, M)
    assert np.array_equal(P.cpu().numpy(), ref_P)
    got = out.cpu().numpy().astype(np.float64)
    assert np.linalg.norm(got - ref_O) <= 1e-3 * np.linalg.norm(ref_O)


def test_large_matrix_as_benchmarked():
    """131072 x 4096 (the bench line's `large_matrix`): the non-temporal form of the one-token kernel, the fused call and
    the kernel for group-wise tables in the launch configurations that size selects, every output against the oracle.
    Any byte string is a valid packed matrix, so the weights are random bytes."""
    N, K = 131072, 4096
    NG = K // 128
    _say("large matrix 131072 x 4096")
    rng = np.random.default_rng(131)
    packed = rng.integers(0, 256, size=N * K // 4, dtype=np.uint8)
    cb = np.sort(rng.standard_normal((N, 4)) * 0.03, axis=1).astype(np.float16).view(np.uint16)
    x = rcp_synth.activation(131, "large", 1, K)
    xq_t, sc_t = rcp.rotate_quant_act(_t(x))
    torch.cuda.synchronize()
    xq, sc = xq_t.cpu().numpy(), sc_t.cpu().numpy().view(np.uint16)
    oxq, osc, _ = oracle.quantize_act(x.astype(np.float32), 1.0)
    assert np.array_equal(xq, oxq) and np.array_equal(sc, osc)
    _check_gemv(packed, cb, N, K, xq, sc, 1, torch.float32)
    pk, lut = _t(packed), _t(cb.view(np.float16))
    ref = rcp.w2a4_gemv(pk, lut, N, K, xq_t, sc_t, 1, out_dtype=torch.float32)
    fused = rcp.quant_w2a4_gemv(pk, lut, N, K, _t(x), 1.0, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(fused, ref)
    del pk, lut, ref, fused
    lv = np.sort(rng.standard_normal((N // 4, NG, 4, 4)) * 0.03, axis=3).astype(np.float16).view(np.uint16)
    _check_grouped_gemv(packed, lv, N, K, xq, sc, torch.float32)


def test_full_size_grouped_and_weight_only_as_benchmarked():
    """gate|up at full size (22016 x 4096) through the group-wise fused call and the weight-only call."""
    N, K = 22016, 4096
    NG = K // 128
    _say("full size grouped / weight-only")
    W, lo, hi, part = rcp_synth.linear_layer_grouped(9, "fullg", N, K)
    x = rcp_synth.activation(9, "fullg", 1, K)
    packed, cb = rcp.pack_weights_grouped(_t(W), _t(lo), _t(hi), _t(part))
    xq = torch.empty((1, K // 2), dtype=torch.uint8, device=DEV)
    sc = torch.empty((1,), dtype=torch.float16, device=DEV)
    out, P = rcp.quant_w2a4_gemv_grouped(packed, cb, N, K, _t(x), 1.0, out_dtype=torch.float16, xq_out=xq, scale_out=sc,
                                         want_partial_sums=True)
    torch.cuda.synchronize()
    ref_packed, ref_cb = oracle.pack_weights_grouped(W.astype(np.float32), lo, hi, part)
    assert np.array_equal(packed.cpu().numpy(), ref_packed)
    assert np.array_equal(cb.cpu().numpy().view(np.uint16).ravel(), ref_cb)
    oxq, osc, _ = oracle.quantize_act(x.astype(np.float32), 1.0)
    assert np.array_equal(xq.cpu().numpy(), oxq) and np.array_equal(sc.cpu().numpy().view(np.uint16), osc)
    ref_O, ref_P = oracle.w2a4_gemv_grouped(ref_packed, ref_cb, N, K, oxq, osc)
    assert np.array_equal(P.cpu().numpy(), ref_P)
    got = out.cpu().numpy().astype(np.float64).ravel()
    assert np.linalg.norm(got - ref_O) <= 1e-3 * np.linalg.norm(ref_O)

    # weight-only on per-channel weights of the same size
    Wc, loc, hic, partc = rcp_synth.linear_layer(9, "fullwo", N, K)
    pk, lut = rcp.pack_weights(_t(Wc), _t(loc), _t(hic), _t(partc))
    o16 = rcp.w2a16_gemv(pk, lut, N, K, _t(x), out_dtype=torch.float32)
    torch.cuda.synchronize()
    rp, rc = oracle.pack_weights(Wc.astype(np.float32), loc, hic, partc)
    assert np.array_equal(pk.cpu().numpy(), rp)
    ref = oracle.w2a16_gemv(rp, rc, N, K, x.astype(np.float64))[0]
    g16 = o16.cpu().numpy().astype(np.float64).ravel()
    assert np.linalg.norm(g16 - ref) <= 1e-3 * np.linalg.norm(ref)
