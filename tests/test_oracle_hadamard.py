"""Pins for the oracle's rotation: the paper's definition of the normalised Hadamard
matrix (Appendix: Sylvester recursion, H H^T = I, first row all ones, other rows
balanced), scipy's Sylvester construction, numpy's Kronecker product."""
import numpy as np
import pytest
import scipy.linalg

import oracle
import rcp_synth


@pytest.mark.parametrize("n", [1, 2, 4, 8, 64, 512, 1024])
def test_matrix_is_the_sylvester_matrix(n):
    H = oracle.hadamard_matrix(n)
    assert np.array_equal(H, scipy.linalg.hadamard(n, dtype=np.int8))
    Hi = H.astype(np.int64)
    assert np.array_equal(Hi @ Hi.T, n * np.eye(n, dtype=np.int64))  # H'H'^T = n I, exactly
    assert np.all(H[0] == 1)
    if n > 1:
        assert np.all((H[1:] == 1).sum(axis=1) == n // 2)
    i, j = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    pop = np.array([bin(v).count("1") for v in (i & j).ravel()]).reshape(n, n)
    assert np.array_equal(H, np.where(pop % 2 == 0, 1, -1))  # closed form (-1)^popcount(i&j)


def test_matrix_8192_sampled_rows_are_orthogonal():
    n = 8192
    H = oracle.hadamard_matrix(n)
    rows = np.random.default_rng(0).choice(n, size=48, replace=False)
    G = H[rows].astype(np.int32) @ H.astype(np.int32).T
    want = np.zeros_like(G)
    want[np.arange(rows.size), rows] = n
    assert np.array_equal(G, want)


def test_rejects_non_power_of_two():
    with pytest.raises(RuntimeError):
        oracle.hadamard_matrix(12)
    with pytest.raises(RuntimeError):
        oracle.rotate(np.zeros(12), oracle.ROT_WHT, n_wht=12)


@pytest.mark.parametrize("n", [2, 32, 512, 2048])
def test_wht_rotation_properties(n):
    rng = np.random.default_rng(n)
    x = rng.standard_normal(n)
    y = oracle.rotate(x, oracle.ROT_WHT, n_wht=n)
    Hn = scipy.linalg.hadamard(n).astype(np.float64) / np.sqrt(n)
    np.testing.assert_allclose(y, Hn @ x, rtol=0, atol=1e-12 * np.sqrt(n))
    np.testing.assert_allclose(y[0], x.sum() / np.sqrt(n), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose((y * y).sum(), (x * x).sum(), rtol=1e-12)       # Parseval
    np.testing.assert_allclose(oracle.rotate(y, oracle.ROT_WHT, n_wht=n), x, atol=1e-12)  # involution
    e = np.zeros(n)
    e[n // 3] = 1.0
    np.testing.assert_allclose(oracle.rotate(e, oracle.ROT_WHT, n_wht=n), Hn[:, n // 3], atol=1e-15)


def test_rotation_none_is_identity_and_tokens_are_independent():
    x = np.random.default_rng(1).standard_normal((3, 64))
    assert np.array_equal(oracle.rotate(x, oracle.ROT_NONE), x)
    y = oracle.rotate(x, oracle.ROT_WHT, n_wht=64)
    for t in range(3):
        np.testing.assert_array_equal(y[t], oracle.rotate(x[t], oracle.ROT_WHT, n_wht=64))


@pytest.mark.parametrize("n,m", [(2, 3), (8, 5), (16, 12), (64, 28)])
def test_kronecker_matches_numpy_kron(n, m):
    Q = rcp_synth.orthogonal(3, m).astype(np.float64)
    assert not np.allclose(Q, Q.T)  # so that a transposed Q cannot pass
    x = np.random.default_rng(n * m).standard_normal(n * m)
    R = np.kron(scipy.linalg.hadamard(n) / np.sqrt(n), Q)
    y = oracle.rotate(x, oracle.ROT_KRON, n_wht=n, m=m, Q=Q)
    np.testing.assert_allclose(y, R @ x, atol=1e-12)
    np.testing.assert_allclose(R @ R.T, np.eye(n * m), atol=1e-6)  # Q is fp32-rounded
    # computational invariance: (W R^T)(R x) = W x
    W = np.random.default_rng(5).standard_normal((7, n * m))
    np.testing.assert_allclose((W @ R.T) @ y, W @ x, atol=1e-5)


@pytest.mark.parametrize("n,m", [(64, 172), (512, 28)])
def test_kronecker_full_size_matches_matrix_form(n, m):
    """K = 11008 and 14336: Y = H_n X Q^T with X the n x m row-major view of x."""
    Q = rcp_synth.orthogonal(0, m).astype(np.float64)
    x = rcp_synth.activation(0, "down", 1, n * m)[0].astype(np.float64)
    y = oracle.rotate(x, oracle.ROT_KRON, n_wht=n, m=m, Q=Q)
    Y = (scipy.linalg.hadamard(n) / np.sqrt(n)) @ x.reshape(n, m) @ Q.T
    np.testing.assert_allclose(y, Y.ravel(), atol=1e-10)
    np.testing.assert_allclose((y * y).sum(), (x * x).sum(), rtol=1e-5)


@pytest.mark.parametrize("n", [2, 16, 512, 4096, 8192])
def test_fwht_f32_agrees_with_dense_fp64(n):
    x = rcp_synth.activation(1, f"fwht{n}", 1, n)[0]
    y32 = oracle.fwht_f32(x.astype(np.float32))
    y64 = oracle.rotate(x.astype(np.float64), oracle.ROT_WHT, n_wht=n)
    # log2(n) rounding steps of relative size 2^-24 on values bounded by ||x||_2
    tol = 2.0 ** -23 * (np.log2(n) + 1) * np.linalg.norm(x.astype(np.float64))
    assert np.max(np.abs(y32.astype(np.float64) - y64)) <= tol


@pytest.mark.parametrize("n", [4, 64, 1024, 4096])
def test_fwht_f32_is_exact_on_small_integers_when_n_is_a_power_of_four(n):
    # all partial sums are integers below 2^24 and 1/sqrt(n) is a power of two
    x = np.random.default_rng(n).integers(-8, 8, size=n).astype(np.float32)
    y32 = oracle.fwht_f32(x)
    want = (scipy.linalg.hadamard(n).astype(np.int64) @ x.astype(np.int64)) / np.sqrt(n)
    assert np.array_equal(y32.astype(np.float64), want)


def test_rotation_preserves_componentwise_variance():
    """Appendix: for i.i.d. components of variance sigma^2, Var(Y_i) = sigma^2."""
    n = 4096
    x = np.random.default_rng(11).uniform(-1, 1, size=(64, n))  # variance 1/3, platykurtic
    y = oracle.fwht_f32(x.astype(np.float32)).astype(np.float64)
    assert abs(y.var() - 1.0 / 3.0) < 0.01 / 3.0
    kurt = lambda v: ((v - v.mean()) ** 4).mean() / v.var() ** 2 - 3.0
    assert kurt(x.ravel()) < -1.0          # uniform: excess kurtosis -1.2
    assert abs(kurt(y.ravel())) < 0.05     # Kurt(Y_i) = Kurt(X)/n -> ~0


# ---- Hadamard across heads: R = H_n (x) I_m (the online factor of R_2, Section 2.1) ------------
@pytest.mark.parametrize("n,m", [(2, 8), (8, 16), (32, 128), (64, 24)])
def test_heads_rotation_is_kron_of_hadamard_and_identity(n, m):
    from scipy.linalg import hadamard
    rng = np.random.default_rng(n * 1000 + m)
    x = rng.standard_normal((2, n * m))
    y = oracle.rotate(x, oracle.ROT_HEADS, n_wht=n, m=m)
    R = np.kron(hadamard(n).astype(np.float64), np.eye(m)) / np.sqrt(n)
    assert np.allclose(y, x @ R.T, rtol=1e-12, atol=1e-12)
    # the general Kronecker kind with Q = I is the same operator
    y2 = oracle.rotate(x, oracle.ROT_KRON, n_wht=n, m=m, Q=np.eye(m))
    assert np.allclose(y, y2, rtol=1e-13, atol=1e-13)
    # involution (H_n is symmetric and orthogonal after scaling) and norm preservation
    assert np.allclose(oracle.rotate(y, oracle.ROT_HEADS, n_wht=n, m=m), x, rtol=1e-12, atol=1e-12)
    assert np.allclose(np.linalg.norm(y, axis=1), np.linalg.norm(x, axis=1), rtol=1e-12)


def test_heads_rotation_special_cases():
    rng = np.random.default_rng(7)
    x = rng.standard_normal(64)
    # one channel per head: the plain transform
    assert np.allclose(oracle.rotate(x, oracle.ROT_HEADS, n_wht=64, m=1), oracle.rotate(x, oracle.ROT_WHT, n_wht=64))
    # head 0 of the output is the scaled sum of the heads, channel by channel
    X = rng.standard_normal((8, 16))
    y = oracle.rotate(X.ravel(), oracle.ROT_HEADS, n_wht=8, m=16).reshape(8, 16)
    assert np.allclose(y[0], X.sum(axis=0) / np.sqrt(8))
    # binary32 butterflies column by column stay within binary32 bounds of the definition
    y32 = oracle.fwht_f32(X.T.astype(np.float32)).T
    assert np.allclose(y32, y, rtol=0, atol=8 * 2.0 ** -24 * np.abs(X).sum(axis=0).max())
    with pytest.raises(RuntimeError):
        oracle.rotate(x, oracle.ROT_HEADS, n_wht=8, m=7)
