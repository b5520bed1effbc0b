"""Seeded synthetic inputs for the W2A4 GEMV path (numpy only).

This module is the one thing the CPU oracle's tests and the HIP path's tests
share.  It draws random tensors with the shapes and value distributions of the
workloads and holds none of the method's arithmetic (no thresholds, no packing,
no rotation, no quantisation).  The recipe:

  weights      W ~ N(0, 0.02^2) in fp32, rounded to fp16, N x K (LLaMA-shaped)
  clip range   per output row: the row's 1 % and 99 % quantiles (a stand-in for
               the learned sigma(beta)*min / sigma(gamma)*max)
  partitions   per output row: softmax of three N(0,1) logits -> (p1, p2, p3)
               (a stand-in for the learned partition fractions)
  activations  fp16 N(0,1); 1 % of the entries, chosen uniformly, multiplied by 20
  Q            m x m orthogonal: QR of a Gaussian matrix, signs fixed so that the
               diagonal of the triangular factor is positive, rounded to fp32

  3-bit grid   a stand-in for the normal-float table of the 3-bit format (which the paper
               cites and does not print): standard-normal quantiles at evenly spaced
               probabilities, four from 3 % up to the median and four above it up to 97 %,
               each side divided by its end value -> eight values in [-1, 1] with one 0
  centre frac  per output row: logistic of a N(0, 0.5^2) logit (a stand-in for the learnt
               centre point between the two clip values)

  KV vectors   head vectors of 128 values for the 4-bit cache, fp16: N(mu_h, sigma_h^2) with a
               per-head spread sigma_h = exp(N(0, 0.4^2)) and a per-head offset
               mu_h = 0.3 * sigma_h * N(0,1) (rotated keys and values are near-Gaussian; the
               offset makes the zero points differ from the mid code); queries: fp16 N(0,1)

Every tensor has its own random stream derived from (seed, tensor name).
"""
import statistics
import zlib

import numpy as np

# Layer shapes as (name, N out, K in, rotation) ; rotation is None, ("wht", n) or
# ("kron", n_wht, m).  Only inputs whose rotation cannot be fused into the
# previous weights offline are rotated online (the FFN down-projection input).
CONFIGS = {
    "tiny": [("tiny", 256, 512, ("wht", 512))],
    "llama32_1b": [
        ("qo", 2048, 2048, None),
        ("gate_up", 8192, 2048, None),
        ("down", 2048, 8192, ("wht", 8192)),
    ],
    "llama2_7b": [
        ("qkvo", 4096, 4096, None),
        ("gate_up", 11008, 4096, None),
        ("down", 4096, 11008, ("kron", 64, 172)),
    ],
    "llama3_8b": [
        ("qo", 4096, 4096, None),
        ("kv", 1024, 4096, None),
        ("gate_up", 14336, 4096, None),
        ("down", 4096, 14336, ("kron", 512, 28)),
    ],
}


def _rng(seed: int, name: str) -> np.random.Generator:
    return np.random.default_rng([int(seed), zlib.crc32(name.encode())])


def weights(seed: int, name: str, N: int, K: int) -> np.ndarray:
    """fp16 N x K, N(0, 0.02^2)."""
    w = _rng(seed, "W:" + name).standard_normal((N, K), dtype=np.float32) * np.float32(0.02)
    return w.astype(np.float16)


def clip_range(W: np.ndarray):
    """Row-wise 1 % / 99 % quantiles as float32 (lo, hi)."""
    Wf = W.astype(np.float32)
    lo = np.quantile(Wf, 0.01, axis=1).astype(np.float32)
    hi = np.quantile(Wf, 0.99, axis=1).astype(np.float32)
    return lo, hi


def partitions(seed: int, name: str, N: int) -> np.ndarray:
    """float32 [N, 3], rows on the open 2-simplex."""
    z = _rng(seed, "part:" + name).standard_normal((N, 3))
    e = np.exp(z - z.max(axis=1, keepdims=True))
    return (e / e.sum(axis=1, keepdims=True)).astype(np.float32)


def activation(seed: int, name: str, M: int, K: int) -> np.ndarray:
    """fp16 M x K, N(0,1) with 1 % of entries scaled by 20."""
    g = _rng(seed, "x:" + name)
    x = g.standard_normal((M, K), dtype=np.float32)
    outlier = g.random((M, K)) < 0.01
    x = np.where(outlier, x * np.float32(20.0), x)
    return x.astype(np.float16)


def orthogonal(seed: int, m: int) -> np.ndarray:
    """float32 m x m orthogonal matrix."""
    a = _rng(seed, f"Q:{m}").standard_normal((m, m))
    q, r = np.linalg.qr(a)
    q = q * np.sign(np.diag(r))[None, :]
    return np.ascontiguousarray(q.astype(np.float32))


def random_indices(seed: int, name: str, N: int, K: int, levels: int = 4) -> np.ndarray:
    """uint8 N x K uniform in 0..levels-1 (for tests that start from indices)."""
    return _rng(seed, "idx:" + name).integers(0, levels, size=(N, K), dtype=np.uint8)


def random_int4(seed: int, name: str, M: int, K: int) -> np.ndarray:
    """int8 M x K uniform in -8..7."""
    return _rng(seed, "q:" + name).integers(-8, 8, size=(M, K), dtype=np.int8)


def linear_layer(seed: int, name: str, N: int, K: int):
    """All offline inputs of one linear layer: (W fp16, lo, hi, part)."""
    W = weights(seed, name, N, K)
    lo, hi = clip_range(W)
    return W, lo, hi, partitions(seed, name, N)


def linear_layer_grouped(seed: int, name: str, N: int, K: int, group: int = 128):
    """Offline inputs of one linear layer quantised in groups of `group` input channels:
    (W fp16, lo [N, K/group], hi [N, K/group], part [N, K/group, 3]); 2 % / 98 % quantiles per group."""
    W = weights(seed, name, N, K)
    NG = K // group
    Wg = W.astype(np.float32).reshape(N, NG, group)
    lo = np.quantile(Wg, 0.02, axis=2).astype(np.float32)
    hi = np.quantile(Wg, 0.98, axis=2).astype(np.float32)
    part = partitions(seed, name + ":grouped", N * NG).reshape(N, NG, 3)
    return W, np.ascontiguousarray(lo), np.ascontiguousarray(hi), np.ascontiguousarray(part)


def normal_quantile_grid() -> np.ndarray:
    """float32 [8], ascending: -1, two negative values, 0, three positive values, 1."""
    nd = statistics.NormalDist()
    tail = 0.03
    neg = [nd.inv_cdf(tail + (0.5 - tail) * i / 3) for i in range(3)]
    pos = [nd.inv_cdf(0.5 + (0.5 - tail) * i / 4) for i in range(1, 5)]
    g = [v / -neg[0] for v in neg] + [0.0] + [v / pos[-1] for v in pos]
    return np.asarray(g, dtype=np.float32)


def centre_fractions(seed: int, name: str, N: int) -> np.ndarray:
    """float32 [N] in (0, 1), scattered around 1/2."""
    z = _rng(seed, "centre:" + name).standard_normal(N) * 0.5
    return (1.0 / (1.0 + np.exp(-z))).astype(np.float32)


def linear_layer_w3(seed: int, name: str, N: int, K: int):
    """Offline inputs of one 3-bit linear layer: (W fp16, lo, hi, centre fraction, grid)."""
    W = weights(seed, name, N, K)
    lo, hi = clip_range(W)
    return W, lo, hi, centre_fractions(seed, name, N), normal_quantile_grid()


def kv_vectors(seed: int, name: str, n_tokens: int, H: int, d: int = 128) -> np.ndarray:
    """n_tokens x H x d fp16 head vectors (keys or values after their rotation)."""
    g = _rng(seed, "kv:" + name)
    sigma = np.exp(0.4 * g.standard_normal(H)).astype(np.float32)
    mu = 0.3 * sigma * g.standard_normal(H).astype(np.float32)
    x = g.standard_normal((n_tokens, H, d), dtype=np.float32) * sigma[None, :, None] + mu[None, :, None]
    return x.astype(np.float16)


def query_vectors(seed: int, name: str, H: int, d: int = 128) -> np.ndarray:
    """H x d fp16 query head vectors."""
    return _rng(seed, "query:" + name).standard_normal((H, d), dtype=np.float32).astype(np.float16)
