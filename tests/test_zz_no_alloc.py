"""The entry point that allocates nothing (rcp_rotate_quant_act_static) against rcp_rotate_quant_act: same bits, on two
calls in a row that share the library's fixed scratch array, the second with a smaller input."""
import numpy as np
import pytest
import torch

import paper_2502_15779_amd as rcp
import rcp_synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _pair(seed, M, n, m, dtype):
    K = n * m
    x = _t(rcp_synth.activation(seed, f"static{M}x{K}", M, K))
    if dtype == torch.float32:
        x = x.float() * 1.0009765
    elif dtype == torch.bfloat16:
        x = x.float().to(torch.bfloat16)
    Q = _t(rcp_synth.orthogonal(seed, m))
    return x, rcp.Rotation.kron(n, Q), Q


def test_static_scratch_matches_the_workspace_call_twice_in_a_row():
    print("static scratch: 64x172 (4 tokens) then 64x28 (1 token)", flush=True)
    x1, rot1, _q1 = _pair(3, 4, 64, 172, torch.float16)
    x2, rot2, _q2 = _pair(4, 1, 64, 28, torch.float32)
    outs = []
    for x, rot in ((x1, rot1), (x2, rot2)):
        M, K = x.shape
        xq = torch.full((M, K // 2), 0xAB, dtype=torch.uint8, device=DEV)
        sc = torch.full((M,), 7.0, dtype=torch.float16, device=DEV)
        outs.append((xq, sc))
    # the two calls back to back on one stream: the second, smaller one finds the first one's values in the array
    rcp.rotate_quant_act_static(x1, rot1, 1.0, *outs[0])
    rcp.rotate_quant_act_static(x2, rot2, 0.9, *outs[1])
    torch.cuda.synchronize()
    ref1 = rcp.rotate_quant_act(x1, rot1, 1.0)
    ref2 = rcp.rotate_quant_act(x2, rot2, 0.9)
    torch.cuda.synchronize()
    for (xq, sc), (rxq, rsc) in zip(outs, (ref1, ref2)):
        assert torch.equal(xq, rxq)
        assert torch.equal(sc.view(torch.int16), rsc.view(torch.int16))


def test_static_scratch_other_rotations_and_the_size_limit():
    print("static scratch: plain / Hadamard inputs, largest Kronecker size, one beyond", flush=True)
    x = _t(rcp_synth.activation(5, "static_wht", 3, 4096))
    for rot in (None, rcp.Rotation.wht(4096), rcp.Rotation.heads(32, 128)):
        xq = torch.empty((3, 2048), dtype=torch.uint8, device=DEV)
        sc = torch.empty((3,), dtype=torch.float16, device=DEV)
        rcp.rotate_quant_act_static(x, rot, 1.0, xq, sc)
        rxq, rsc = rcp.rotate_quant_act(x, rot, 1.0)
        torch.cuda.synchronize()
        assert torch.equal(xq, rxq) and torch.equal(sc.view(torch.int16), rsc.view(torch.int16))
    # 16 tokens x 14336 channels: 917504 bytes of scratch, inside the 1 MiB array
    xb, rotb, _qb = _pair(6, 16, 512, 28, torch.bfloat16)
    xq = torch.empty((16, 7168), dtype=torch.uint8, device=DEV)
    sc = torch.empty((16,), dtype=torch.float16, device=DEV)
    rcp.rotate_quant_act_static(xb, rotb, 1.0, xq, sc)
    rxq, rsc = rcp.rotate_quant_act(xb, rotb, 1.0)
    torch.cuda.synchronize()
    assert torch.equal(xq, rxq) and torch.equal(sc.view(torch.int16), rsc.view(torch.int16))
    # 16 tokens x 32768 channels need 2 MiB: refused, outputs untouched
    xl, rotl, _ql = _pair(7, 16, 128, 256, torch.float16)
    xq = torch.full((16, 16384), 0x5A, dtype=torch.uint8, device=DEV)
    sc = torch.full((16,), 3.0, dtype=torch.float16, device=DEV)
    with pytest.raises(rcp.RcpError) as e:
        rcp.rotate_quant_act_static(xl, rotl, 1.0, xq, sc)
    assert e.value.code == -5
    torch.cuda.synchronize()
    assert bool((xq == 0x5A).all()) and bool((sc == 3.0).all())
