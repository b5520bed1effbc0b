"""Host-side contracts that need no GPU: the benchmark refuses more than one GPU with a message, its byte
accounting matches the tensor list of Section 4.4, and the seeded input generators are reproducible."""
import os
import subprocess
import sys

import numpy as np

import rcp_synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_byte_accounting_follows_the_tensor_list():
    sys.path.insert(0, ROOT)
    import bench
    # W_q: N*K/4 bytes, LUT: N*4 fp16, X_q: K/2 bytes, S: one fp16, O: N fp16 (Section 4.4)
    for N, K in [(4096, 4096), (11008, 4096), (4096, 11008)]:
        assert bench.gemv_bytes(N, K) == N * K // 4 + 8 * N + K // 2 + 2 + 2 * N
    names = [l[0] for l in bench.layer_launches()]
    assert names == ["qkv", "o", "gate_up", "down"]
    shapes = {l[0]: (l[1], l[2]) for l in bench.layer_launches()}
    assert shapes["qkv"] == (3 * 4096, 4096) and shapes["gate_up"] == (2 * 11008, 4096) and shapes["down"] == (4096, 11008)
    assert [l[3] for l in bench.layer_launches()] == [False, False, False, True]       # only the down input is rotated online


def test_generators_are_seeded_and_hold_no_method_arithmetic():
    a = rcp_synth.kv_vectors(3, "k", 5, 2)
    b = rcp_synth.kv_vectors(3, "k", 5, 2)
    c = rcp_synth.kv_vectors(4, "k", 5, 2)
    assert a.dtype == np.float16 and a.shape == (5, 2, 128) and np.array_equal(a, b) and not np.array_equal(a, c)
    assert not np.array_equal(rcp_synth.kv_vectors(3, "v", 5, 2), a)                   # one stream per tensor name
    q = rcp_synth.query_vectors(3, "q", 4)
    assert q.shape == (4, 128) and np.array_equal(q, rcp_synth.query_vectors(3, "q", 4))
    W1, lo1, hi1, p1 = rcp_synth.linear_layer(1, "t", 8, 64)
    W2, lo2, hi2, p2 = rcp_synth.linear_layer(1, "t", 8, 64)
    assert np.array_equal(W1, W2) and np.array_equal(lo1, lo2) and np.array_equal(p1, p2)
    assert np.all(lo1 < hi1) and np.allclose(p1.sum(axis=1), 1.0, atol=1e-6)
    src = open(os.path.join(ROOT, "rcp_synth.py")).read()
    assert "import oracle" not in src and "paper_2502_15779_amd" not in src
