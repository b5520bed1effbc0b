"""rcp_quant_w2a4_gemv_sequence (several dependent one-token GEMVs in one launch) against the one-launch-per-matrix
calls, bit for bit, and against the oracle on a chained case.  Every launch is followed by a check of the workspace's
error word (a wait that ran out of its bound) and of the counters the launch must leave at zero."""
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


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(autouse=True)
def _auto_options():
    yield
    rcp.set_option("reset", 0)


def _random_layer(seed, shapes):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    out = []
    for N, K in shapes:
        pk = torch.randint(0, 256, (N * K // 4,), dtype=torch.uint8, device=DEV, generator=g)
        lv = (torch.randn((N, 4), device=DEV, generator=g) * 0.03).sort(dim=1).values.to(torch.float16).contiguous()
        out.append((pk, lv))
    return out


def _sync_and_check(ws, n_rot_values):
    torch.cuda.synchronize()
    assert int(ws[0].item()) == 0, "a wait inside the sequence kernel ran out of its bound"
    counters = ws[:ws.numel() - n_rot_values] if n_rot_values else ws
    assert bool((counters == 0).all().item()), "the launch left a counter or go word set"


H, I = 4096, 11008
LAYER = [(3 * H, H), (H, H), (2 * I, H), (H, I)]


def _layer_steps(w, x0, o, rot, xq=None, sc=None):
    xq = xq or [None] * 4
    sc = sc or [None] * 4
    return [rcp.GemvStep(w[0][0], w[0][1], 3 * H, H, x0, o[0], xq_out=xq[0], scale_out=sc[0]),
            rcp.GemvStep(w[1][0], w[1][1], H, H, o[0][0, :H], o[1], xq_out=xq[1], scale_out=sc[1]),
            rcp.GemvStep(w[2][0], w[2][1], 2 * I, H, o[1], o[2], xq_out=xq[2], scale_out=sc[2]),
            rcp.GemvStep(w[3][0], w[3][1], H, I, o[2][0, :I], o[3], rot=rot, xq_out=xq[3], scale_out=sc[3])]


def _layer_per_launch(w, x0, o, rot, ybuf, xq=None, sc=None):
    xq = xq or [None] * 4
    sc = sc or [None] * 4
    rcp.quant_w2a4_gemv(w[0][0], w[0][1], 3 * H, H, x0, 1.0, out=o[0], xq_out=xq[0], scale_out=sc[0])
    rcp.quant_w2a4_gemv(w[1][0], w[1][1], H, H, o[0][0, :H], 1.0, out=o[1], xq_out=xq[1], scale_out=sc[1])
    rcp.quant_w2a4_gemv(w[2][0], w[2][1], 2 * I, H, o[1], 1.0, out=o[2], xq_out=xq[2], scale_out=sc[2])
    rcp.rotate_act(o[2][:, :I], rot, y_out=ybuf)
    rcp.quant_w2a4_gemv(w[3][0], w[3][1], H, I, ybuf, 1.0, out=o[3], xq_out=xq[3], scale_out=sc[3])


@pytest.mark.parametrize("layers_per_launch", [1, 2, 4])
def test_full_size_llama2_7b_layer_chain_equals_the_per_launch_path(layers_per_launch):
    """q|k|v -> o (reads q) -> gate|up (reads o's output) -> H_64 (x) Q_172 -> down (reads the gate half), 1, 2 or 4
    layers per launch, each layer starting from its own input: outputs, x_q and S of every entry bit-identical to
    rcp_quant_w2a4_gemv / rcp_rotate_act launched one by one; repeated with new inputs on the same workspace."""
    _say(f"sequence: full-size 7B layer chain, {layers_per_launch} layer(s) per launch")
    Q = _t(rcp_synth.orthogonal(3, 172))
    rot = rcp.Rotation.kron(64, Q)
    ybuf = torch.empty((1, I), dtype=torch.float32, device=DEV)
    ws_layers = [_random_layer(50 + l, LAYER) for l in range(layers_per_launch)]
    x0s = [torch.empty((1, H), dtype=torch.float16, device=DEV) for _ in range(layers_per_launch)]
    got = [[torch.zeros((1, N), dtype=torch.float16, device=DEV) for N, _ in LAYER] for _ in range(layers_per_launch)]
    ref = [[torch.zeros((1, N), dtype=torch.float16, device=DEV) for N, _ in LAYER] for _ in range(layers_per_launch)]
    xq_g = [[torch.zeros(K // 2, dtype=torch.uint8, device=DEV) for _, K in LAYER] for _ in range(layers_per_launch)]
    sc_g = [[torch.zeros(1, dtype=torch.float16, device=DEV) for _ in LAYER] for _ in range(layers_per_launch)]
    xq_r = [[torch.zeros(K // 2, dtype=torch.uint8, device=DEV) for _, K in LAYER] for _ in range(layers_per_launch)]
    sc_r = [[torch.zeros(1, dtype=torch.float16, device=DEV) for _ in LAYER] for _ in range(layers_per_launch)]
    steps = sum((_layer_steps(ws_layers[l], x0s[l], got[l], rot, xq_g[l], sc_g[l]) for l in range(layers_per_launch)), [])
    ws = rcp.gemv_sequence_workspace(steps)
    for trial in range(3):      # new inputs every time: a stale cached value of an earlier launch would show
        for l in range(layers_per_launch):
            x0s[l].copy_(_t(rcp_synth.activation(60 + 7 * trial + l, f"seq{trial}/{l}", 1, H)))
        rcp.quant_w2a4_gemv_sequence(steps, ws)
        _sync_and_check(ws, I)
        for l in range(layers_per_launch):
            _layer_per_launch(ws_layers[l], x0s[l], ref[l], rot, ybuf, xq_r[l], sc_r[l])
        torch.cuda.synchronize()
        for l in range(layers_per_launch):
            for i in range(4):
                assert torch.equal(xq_g[l][i], xq_r[l][i]), (trial, l, i)
                assert torch.equal(sc_g[l][i].view(torch.int16), sc_r[l][i].view(torch.int16)), (trial, l, i)
                assert torch.equal(got[l][i], ref[l][i]), (trial, l, i)


@pytest.mark.parametrize("x_dtype,out_dtype", [(torch.float16, torch.float32), (torch.bfloat16, torch.float16),
                                               (torch.float32, torch.float32)])
@pytest.mark.parametrize("blocks", [0, 64, 7])
def test_small_ragged_chain_every_type_and_few_workgroups(x_dtype, out_dtype, blocks):
    """Ragged sizes (N not a multiple of 16, K not a multiple of 1024), binary32 and fp16 outputs feeding the next
    entry, bf16 / fp32 first inputs, and grids far smaller than the number of row groups."""
    _say(f"sequence: small chain {x_dtype} -> {out_dtype}, seq_blocks={blocks}")
    rcp.set_option("seq_blocks", blocks)
    shapes = [(1028, 608), (608, 1024), (96, 608)]
    w = _random_layer(9, shapes)
    x = _t(rcp_synth.activation(9, "seq_small", 1, 608)).to(x_dtype)
    o_g = [torch.zeros((1, N), dtype=out_dtype, device=DEV) for N, _ in shapes]
    o_r = [torch.zeros((1, N), dtype=out_dtype, device=DEV) for N, _ in shapes]
    steps = [rcp.GemvStep(w[0][0], w[0][1], 1028, 608, x, o_g[0], clip_ratio=0.9),
             rcp.GemvStep(w[1][0], w[1][1], 608, 1024, o_g[0][0, :1024], o_g[1]),
             rcp.GemvStep(w[2][0], w[2][1], 96, 608, o_g[1], o_g[2])]
    ws = rcp.gemv_sequence_workspace(steps)
    for _ in range(2):
        rcp.quant_w2a4_gemv_sequence(steps, ws)
        _sync_and_check(ws, 0)
    rcp.quant_w2a4_gemv(w[0][0], w[0][1], 1028, 608, x, 0.9, out=o_r[0])
    rcp.quant_w2a4_gemv(w[1][0], w[1][1], 608, 1024, o_r[0][0, :1024], 1.0, out=o_r[1])
    rcp.quant_w2a4_gemv(w[2][0], w[2][1], 96, 608, o_r[1], 1.0, out=o_r[2])
    torch.cuda.synchronize()
    for a, b in zip(o_g, o_r):
        assert torch.equal(a, b)


@pytest.mark.parametrize("n,m,x_dtype", [(512, 28, torch.float16), (64, 172, torch.float32), (128, 64, torch.bfloat16),
                                         (1024, 16, torch.float16), (256, 36, torch.float32)])
def test_rotated_entries_equal_rotate_act_then_the_fused_call(n, m, x_dtype):
    """Kronecker rotations of every Hadamard factor the sequence kernel rotates (64 ... 1024), each input type, as the
    second entry of a chain (its input is the first entry's output for fp16, a fresh tensor otherwise)."""
    _say(f"sequence: rotated entry {n} x {m}, {x_dtype}")
    K = n * m
    N0, K0 = K, 512
    w = _random_layer(11, [(N0, K0), (260, K)])
    Q = _t(rcp_synth.orthogonal(5, m))
    rot = rcp.Rotation.kron(n, Q)
    x0 = _t(rcp_synth.activation(11, "seq_rot0", 1, K0))
    o0_g = torch.zeros((1, N0), dtype=torch.float16, device=DEV)
    o0_r = torch.zeros((1, N0), dtype=torch.float16, device=DEV)
    fresh = _t(rcp_synth.activation(12, "seq_rot1", 1, K)).to(x_dtype)
    chained = x_dtype == torch.float16
    o1_g = torch.zeros((1, 260), dtype=torch.float32, device=DEV)
    xq_g = torch.zeros(K // 2, dtype=torch.uint8, device=DEV)
    sc_g = torch.zeros(1, dtype=torch.float16, device=DEV)
    steps = [rcp.GemvStep(w[0][0], w[0][1], N0, K0, x0, o0_g),
             rcp.GemvStep(w[1][0], w[1][1], 260, K, o0_g if chained else fresh, o1_g, rot=rot, xq_out=xq_g, scale_out=sc_g)]
    ws = rcp.gemv_sequence_workspace(steps)
    rcp.quant_w2a4_gemv_sequence(steps, ws)
    _sync_and_check(ws, K)
    rcp.quant_w2a4_gemv(w[0][0], w[0][1], N0, K0, x0, 1.0, out=o0_r)
    y = rcp.rotate_act(o0_r if chained else fresh, rot)
    xq_r = torch.zeros(K // 2, dtype=torch.uint8, device=DEV)
    sc_r = torch.zeros(1, dtype=torch.float16, device=DEV)
    o1_r = rcp.quant_w2a4_gemv(w[1][0], w[1][1], 260, K, y, 1.0, out_dtype=torch.float32, xq_out=xq_r, scale_out=sc_r)
    torch.cuda.synchronize()
    assert torch.equal(o0_g, o0_r)
    assert torch.equal(ws[ws.numel() - K:].view(torch.float32), y[0])      # the rotated vector itself
    assert torch.equal(xq_g, xq_r) and torch.equal(sc_g.view(torch.int16), sc_r.view(torch.int16))
    assert torch.equal(o1_g, o1_r)


def test_sequences_of_different_length_share_one_workspace():
    """A rotated 2-entry sequence and a 12-entry sequence take turns on one workspace (the rotated vector of the first
    must not land where the second keeps its counters)."""
    _say("sequence: two sequences, one workspace")
    n, m = 64, 28
    K = n * m
    w = _random_layer(31, [(K, 256), (128, K), (256, 256)])
    Q = _t(rcp_synth.orthogonal(6, m))
    rot = rcp.Rotation.kron(n, Q)
    x = _t(rcp_synth.activation(31, "share", 1, 256))
    a0 = torch.zeros((1, K), dtype=torch.float16, device=DEV)
    a1 = torch.zeros((1, 128), dtype=torch.float16, device=DEV)
    short = [rcp.GemvStep(w[0][0], w[0][1], K, 256, x, a0), rcp.GemvStep(w[1][0], w[1][1], 128, K, a0, a1, rot=rot)]
    bufs = [x] + [torch.zeros((1, 256), dtype=torch.float16, device=DEV) for _ in range(12)]
    long_ = [rcp.GemvStep(w[2][0], w[2][1], 256, 256, bufs[i], bufs[i + 1]) for i in range(12)]
    ws = rcp.gemv_sequence_workspace(short)
    assert ws.numel() >= rcp.gemv_sequence_workspace(long_).numel()
    for _ in range(3):
        rcp.quant_w2a4_gemv_sequence(short, ws)
        rcp.quant_w2a4_gemv_sequence(long_, ws)
    _sync_and_check(ws, K)
    r0 = rcp.quant_w2a4_gemv(w[0][0], w[0][1], K, 256, x, 1.0)
    r1 = rcp.quant_w2a4_gemv(w[1][0], w[1][1], 128, K, rcp.rotate_act(r0, rot), 1.0)
    cur = x
    for i in range(12):
        cur = rcp.quant_w2a4_gemv(w[2][0], w[2][1], 256, 256, cur, 1.0)
        torch.cuda.synchronize()
        assert torch.equal(cur, bufs[i + 1]), i
    assert torch.equal(r0, a0) and torch.equal(r1, a1)


def test_chain_against_the_oracle():
    """Export -> chain of two entries (the second rotated) on the GPU; the oracle takes the same steps on the CPU, its
    GEMVs consuming the GPU's (x_q, S) so that a legal tie flip of the Kronecker rotation cannot leak in."""
    _say("sequence: chain against the oracle")
    N0, K0, n, m, N1 = 64 * 28, 1024, 64, 28, 512
    K1 = n * m
    W0, lo0, hi0, p0 = rcp_synth.linear_layer(21, "seq_or0", N0, K0)
    W1, lo1, hi1, p1 = rcp_synth.linear_layer(21, "seq_or1", N1, K1)
    pk0, cb0 = rcp.pack_weights(_t(W0), _t(lo0), _t(hi0), _t(p0))
    pk1, cb1 = rcp.pack_weights(_t(W1), _t(lo1), _t(hi1), _t(p1))
    x0 = rcp_synth.activation(21, "seq_or", 1, K0)
    Q = rcp_synth.orthogonal(21, m)
    o0 = torch.zeros((1, N0), dtype=torch.float16, device=DEV)
    o1 = torch.zeros((1, N1), dtype=torch.float32, device=DEV)
    xq = [torch.zeros(K0 // 2, dtype=torch.uint8, device=DEV), torch.zeros(K1 // 2, dtype=torch.uint8, device=DEV)]
    sc = [torch.zeros(1, dtype=torch.float16, device=DEV) for _ in range(2)]
    steps = [rcp.GemvStep(pk0, cb0, N0, K0, _t(x0), o0, xq_out=xq[0], scale_out=sc[0]),
             rcp.GemvStep(pk1, cb1, N1, K1, o0, o1, rot=rcp.Rotation.kron(n, _t(Q)), xq_out=xq[1], scale_out=sc[1])]
    ws = rcp.gemv_sequence_workspace(steps)
    rcp.quant_w2a4_gemv_sequence(steps, ws)
    _sync_and_check(ws, K1)
    rp0, rc0 = oracle.pack_weights(W0.astype(np.float32), lo0, hi0, p0)
    rp1, rc1 = oracle.pack_weights(W1.astype(np.float32), lo1, hi1, p1)
    oxq, osc, _ = oracle.quantize_act(x0.astype(np.float32), 1.0)
    assert np.array_equal(xq[0].cpu().numpy().reshape(1, -1), oxq) and np.array_equal(sc[0].cpu().numpy().view(np.uint16), osc)
    O0, _ = oracle.w2a4_gemv(rp0, rc0, N0, K0, oxq, osc, 1)
    g0 = o0.cpu().numpy().astype(np.float64)
    assert np.linalg.norm(g0 - O0) <= 1e-3 * np.linalg.norm(O0)
    # the second entry's input is the GPU's own fp16 output of the first
    y64 = oracle.rotate(o0.cpu().numpy().astype(np.float64), oracle.ROT_KRON, n_wht=n, m=m, Q=Q.astype(np.float64))
    xq1, sc1 = xq[1].cpu().numpy().reshape(1, -1), sc[1].cpu().numpy().view(np.uint16)
    s = float(sc1.view(np.float16)[0])
    q = oracle.unpack_int4(xq1)[0] if hasattr(oracle, "unpack_int4") else None
    if q is None:
        b = xq1[0].astype(np.int16)
        lo_n, hi_n = b & 15, b >> 4
        q = np.stack([np.where(lo_n > 7, lo_n - 16, lo_n), np.where(hi_n > 7, hi_n - 16, hi_n)], axis=1).reshape(-1)
    assert np.all(np.abs(q - np.clip(np.atleast_2d(y64)[0] / s, -8.5, 7.5)) <= 0.5 + 1e-3)
    O1, _ = oracle.w2a4_gemv(rp1, rc1, N1, K1, xq1, sc1, 1)
    g1 = o1.cpu().numpy().astype(np.float64)
    assert np.linalg.norm(g1 - O1) <= 1e-3 * np.linalg.norm(O1)


def test_argument_errors_and_limits():
    w = _random_layer(1, [(64, 128)])
    x = torch.zeros((1, 128), dtype=torch.float16, device=DEV)
    o = torch.zeros((1, 64), dtype=torch.float16, device=DEV)
    step = rcp.GemvStep(w[0][0], w[0][1], 64, 128, x, o)
    ws = rcp.gemv_sequence_workspace([step])
    with pytest.raises(rcp.RcpError):      # too many entries
        rcp.quant_w2a4_gemv_sequence([step] * 17, torch.zeros(1 << 18, dtype=torch.int32, device=DEV))
    with pytest.raises(rcp.RcpError):      # workspace too small
        rcp.quant_w2a4_gemv_sequence([step, step], ws[:ws.numel() - 64])
    with pytest.raises(rcp.RcpError):      # a pure Hadamard rotation is not rotated inside a sequence
        rcp.quant_w2a4_gemv_sequence([rcp.GemvStep(w[0][0], w[0][1], 64, 128, x, o, rot=rcp.Rotation.wht(128))], ws)
    rcp.set_option("seq_blocks", 4096)
    with pytest.raises(rcp.RcpError) as e:  # more workgroups than can be resident at once
        rcp.quant_w2a4_gemv_sequence([step], ws)
    assert e.value.code == -4
    rcp.set_option("seq_blocks", 0)
    torch.cuda.synchronize()
    assert bool((ws == 0).all().item()) and bool((o == 0).all().item())   # nothing was launched
