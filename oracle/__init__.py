"""ctypes front end of the plain CPU oracle (oracle/rcp_oracle.c).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg may import this package.  It never imports the HIP
package and takes numpy (host) arrays only.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None

ROT_NONE, ROT_WHT, ROT_KRON, ROT_HEADS = 0, 1, 2, 3


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        L.rcp_ref_f64_to_f16_bits.restype = ctypes.c_uint16
        L.rcp_ref_f64_to_f16_bits.argtypes = [ctypes.c_double]
        L.rcp_ref_f16_bits_to_f64.restype = ctypes.c_double
        L.rcp_ref_f16_bits_to_f64.argtypes = [ctypes.c_uint16]
        L.rcp_ref_ldp_grid.restype = None
        L.rcp_ref_ldp_grid.argtypes = [ctypes.c_float] * 5 + [ctypes.c_void_p, ctypes.c_void_p]
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def max_threads() -> int:
    return int(lib().rcp_ref_max_threads())


def set_threads(n: int) -> None:
    lib().rcp_ref_set_threads(ctypes.c_int(n))


def f64_to_f16_bits(v: float) -> int:
    return int(lib().rcp_ref_f64_to_f16_bits(float(v)))


def f16_bits_to_f64(bits: int) -> float:
    return float(lib().rcp_ref_f16_bits_to_f64(int(bits)))


def hadamard_matrix(n: int) -> np.ndarray:
    out = np.empty((n, n), dtype=np.int8)
    _check(lib().rcp_ref_hadamard_matrix(ctypes.c_int(n), _p(out)), "hadamard_matrix")
    return out


def rotate(x, kind=ROT_NONE, n_wht=0, m=1, Q=None) -> np.ndarray:
    """y = R x in fp64 by the dense definition. x: (M, K) or (K,)."""
    x2 = _c(np.atleast_2d(x), np.float64)
    M, K = x2.shape
    y = np.empty_like(x2)
    Qc = _c(Q, np.float64) if Q is not None else None
    _check(lib().rcp_ref_rotate(_p(x2), M, K, int(kind), int(n_wht), int(m),
                                _p(Qc) if Qc is not None else None, _p(y)), "rotate")
    return y.reshape(np.shape(x))


def fwht_f32(v) -> np.ndarray:
    """Binary32 ascending-stride butterfly + scaling by (float)(1/sqrt n)."""
    out = _c(v, np.float32).copy()
    flat = out.reshape(-1, out.shape[-1])
    for row in flat:
        _check(lib().rcp_ref_fwht_f32(_p(row), int(row.shape[0])), "fwht_f32")
    return out


def ldp_grid(clip_lo, clip_hi, p1, p2, p3):
    """-> (thresholds float32[3], level bit patterns uint16[4]) for one unit."""
    T = np.empty(3, dtype=np.float32)
    Lv = np.empty(4, dtype=np.uint16)
    lib().rcp_ref_ldp_grid(float(np.float32(clip_lo)), float(np.float32(clip_hi)),
                           float(np.float32(p1)), float(np.float32(p2)), float(np.float32(p3)),
                           _p(T), _p(Lv))
    return T, Lv


def pack_weights(W, clip_lo, clip_hi, part, want_idx=False):
    """-> packed uint8[N*K/4], codebook uint16[N,4] (fp16 bits) [, idx uint8[N,K]]."""
    Wc = _c(W, np.float32)
    N, K = Wc.shape
    lo, hi, pt = _c(clip_lo, np.float32), _c(clip_hi, np.float32), _c(part, np.float32)
    assert lo.shape == (N,) and hi.shape == (N,) and pt.shape == (N, 3)
    packed = np.empty(N * K // 4, dtype=np.uint8)
    cb = np.empty((N, 4), dtype=np.uint16)
    idx = np.empty((N, K), dtype=np.uint8) if want_idx else None
    _check(lib().rcp_ref_pack_weights(_p(Wc), N, K, _p(lo), _p(hi), _p(pt), _p(packed), _p(cb),
                                      _p(idx) if want_idx else None), "pack_weights")
    return (packed, cb, idx) if want_idx else (packed, cb)


def unpack_indices(packed, N, K) -> np.ndarray:
    pk = _c(packed, np.uint8)
    assert pk.size == N * K // 4
    idx = np.empty((N, K), dtype=np.uint8)
    _check(lib().rcp_ref_unpack_indices(_p(pk), N, K, _p(idx)), "unpack_indices")
    return idx


def pack_indices(idx) -> np.ndarray:
    ic = _c(idx, np.uint8)
    N, K = ic.shape
    packed = np.empty(N * K // 4, dtype=np.uint8)
    _check(lib().rcp_ref_pack_indices(_p(ic), N, K, _p(packed)), "pack_indices")
    return packed


def quantize_act(y, clip_ratio=1.0):
    """y: (M, K) float32 -> (xq uint8[M, K/2], scale fp16 bits uint16[M], q int8[M, K])."""
    yc = _c(np.atleast_2d(y), np.float32)
    M, K = yc.shape
    xq = np.empty((M, K // 2), dtype=np.uint8)
    sc = np.empty(M, dtype=np.uint16)
    q = np.empty((M, K), dtype=np.int8)
    _check(lib().rcp_ref_quantize_act(_p(yc), M, K, ctypes.c_float(clip_ratio), _p(xq), _p(sc),
                                      _p(q)), "quantize_act")
    return xq, sc, q


def unpack_act(xq, M, K) -> np.ndarray:
    xc = _c(xq, np.uint8)
    assert xc.size == M * K // 2
    q = np.empty((M, K), dtype=np.int8)
    _check(lib().rcp_ref_unpack_act(_p(xc), M, K, _p(q)), "unpack_act")
    return q


def w2a4_gemv(packed, codebook, N, K, xq, scale_bits, M=1):
    """-> (O float64[M, N], P int32[M, N, 4])."""
    pk, cb = _c(packed, np.uint8), _c(codebook, np.uint16)
    xc, sc = _c(xq, np.uint8), _c(scale_bits, np.uint16)
    assert pk.size == N * K // 4 and cb.size == N * 4 and xc.size == M * K // 2 and sc.size == M
    out = np.empty((M, N), dtype=np.float64)
    P = np.empty((M, N, 4), dtype=np.int32)
    _check(lib().rcp_ref_w2a4_gemv(_p(pk), _p(cb), N, K, _p(xc), _p(sc), M, _p(out), _p(P)),
           "w2a4_gemv")
    return out, P


def dequant_dot(packed, codebook, N, K, xq, scale_bits, M=1) -> np.ndarray:
    pk, cb = _c(packed, np.uint8), _c(codebook, np.uint16)
    xc, sc = _c(xq, np.uint8), _c(scale_bits, np.uint16)
    out = np.empty((M, N), dtype=np.float64)
    _check(lib().rcp_ref_dequant_dot(_p(pk), _p(cb), N, K, _p(xc), _p(sc), M, _p(out)),
           "dequant_dot")
    return out


def w2a16_gemv(packed, codebook, N, K, x) -> np.ndarray:
    """Weight-only product: x (M, K) of any float type (taken exactly) -> O float64 (M, N)."""
    pk, cb = _c(packed, np.uint8), _c(codebook, np.uint16)
    xc = _c(np.atleast_2d(x), np.float64)
    M = xc.shape[0]
    assert pk.size == N * K // 4 and cb.size == 4 * N and xc.shape[1] == K
    out = np.empty((M, N), dtype=np.float64)
    _check(lib().rcp_ref_w2a16_gemv(_p(pk), _p(cb), N, K, _p(xc), M, _p(out)), "w2a16_gemv")
    return out


# ---- group-wise quantisation units (group size 128) ----------------------------------------
def grouped_lut_index(h, g, NG):
    """Half-word index of level 0 of row h, group g in the grouped LUT layout."""
    return (((h // 4) * NG + g) * 4 + (h % 4)) * 4


def pack_weights_grouped(W, clip_lo, clip_hi, part, group=128, want_idx=False):
    """W [N,K]; clip_lo/hi [N,NG]; part [N,NG,3] -> packed uint8[N*K/4], codebook uint16[N*NG*4] (grouped layout)."""
    Wc = _c(W, np.float32)
    N, K = Wc.shape
    NG = K // group
    lo, hi, pt = _c(clip_lo, np.float32), _c(clip_hi, np.float32), _c(part, np.float32)
    assert lo.shape == (N, NG) and hi.shape == (N, NG) and pt.shape == (N, NG, 3)
    packed = np.empty(N * K // 4, dtype=np.uint8)
    cb = np.empty(N * NG * 4, dtype=np.uint16)
    idx = np.empty((N, K), dtype=np.uint8) if want_idx else None
    _check(lib().rcp_ref_pack_weights_grouped(_p(Wc), N, K, group, _p(lo), _p(hi), _p(pt), _p(packed), _p(cb),
                                              _p(idx) if want_idx else None), "pack_weights_grouped")
    return (packed, cb, idx) if want_idx else (packed, cb)


def pack_indices_grouped(idx, group=128) -> np.ndarray:
    ic = _c(idx, np.uint8)
    N, K = ic.shape
    packed = np.empty(N * K // 4, dtype=np.uint8)
    _check(lib().rcp_ref_pack_indices_grouped(_p(ic), N, K, group, _p(packed)), "pack_indices_grouped")
    return packed


def unpack_indices_grouped(packed, N, K, group=128) -> np.ndarray:
    pk = _c(packed, np.uint8)
    assert pk.size == N * K // 4
    idx = np.empty((N, K), dtype=np.uint8)
    _check(lib().rcp_ref_unpack_indices_grouped(_p(pk), N, K, group, _p(idx)), "unpack_indices_grouped")
    return idx


def w2a4_gemv_grouped(packed, codebook, N, K, xq, scale_bits, group=128, M=1):
    """-> (O float64 [N] and P int32 [N, NG, 4] for M = 1; [M, N] and [M, N, NG, 4] otherwise)."""
    pk, cb = _c(packed, np.uint8), _c(codebook, np.uint16)
    xc, sc = _c(xq, np.uint8), _c(scale_bits, np.uint16)
    NG = K // group
    assert pk.size == N * K // 4 and cb.size == N * NG * 4 and xc.size == M * K // 2 and sc.size >= M
    out = np.empty((M, N), dtype=np.float64)
    P = np.empty((M, N, NG, 4), dtype=np.int32)
    _check(lib().rcp_ref_w2a4_gemv_grouped(_p(pk), _p(cb), N, K, group, _p(xc), _p(sc), M, _p(out), _p(P)),
           "w2a4_gemv_grouped")
    return (out[0], P[0]) if M == 1 else (out, P)


# ---- 3-bit variant (LDP on the asymmetric normal-float format, Section 4.3) -------------------
def w3_grid(clip_lo, clip_hi, frac, grid):
    """(thresholds float32[7], level bit patterns uint16[8]) of one quantisation unit."""
    g = _c(grid, np.float32)
    assert g.shape == (8,)
    T = np.empty(7, dtype=np.float32)
    L = np.empty(8, dtype=np.uint16)
    f = lib().rcp_ref_w3_grid
    f.restype = None
    f.argtypes = [ctypes.c_float] * 3 + [ctypes.c_void_p] * 3
    f(float(clip_lo), float(clip_hi), float(frac), _p(g), _p(T), _p(L))
    return T, L


def pack_weights_w3(W, clip_lo, clip_hi, frac, grid, want_idx=False):
    W = _c(W, np.float32)
    N, K = W.shape
    packed = np.empty(N * K // 8 * 3, dtype=np.uint8)
    codebook = np.empty((N, 8), dtype=np.uint16)
    idx = np.empty((N, K), dtype=np.uint8) if want_idx else None
    _check(lib().rcp_ref_pack_weights_w3(_p(W), N, K, _p(_c(clip_lo, np.float32)), _p(_c(clip_hi, np.float32)),
                                         _p(_c(frac, np.float32)), _p(_c(grid, np.float32)), _p(packed),
                                         _p(codebook), _p(idx) if want_idx else None), "pack_weights_w3")
    return (packed, codebook, idx) if want_idx else (packed, codebook)


def pack_indices_w3(idx) -> np.ndarray:
    idx = _c(idx, np.uint8)
    N, K = idx.shape
    packed = np.empty(N * K // 8 * 3, dtype=np.uint8)
    _check(lib().rcp_ref_pack_indices_w3(_p(idx), N, K, _p(packed)), "pack_indices_w3")
    return packed


def unpack_indices_w3(packed, N, K) -> np.ndarray:
    packed = _c(packed, np.uint8)
    idx = np.empty((N, K), dtype=np.uint8)
    _check(lib().rcp_ref_unpack_indices_w3(_p(packed), N, K, _p(idx)), "unpack_indices_w3")
    return idx


def w3a4_gemv(packed, codebook, N, K, xq, scale_bits):
    """(out float64[N], P int32[N][8]) for one token."""
    packed = _c(packed, np.uint8)
    codebook = _c(codebook, np.uint16)
    xq = _c(xq, np.uint8)
    sb = _c(np.atleast_1d(scale_bits), np.uint16)
    out = np.empty(N, dtype=np.float64)
    P = np.empty((N, 8), dtype=np.int32)
    _check(lib().rcp_ref_w3a4_gemv(_p(packed), _p(codebook), N, K, _p(xq), _p(sb), _p(out), _p(P)), "w3a4_gemv")
    return out, P


# ---- 4-bit KV cache and one-token attention over it ---------------------------------------
KV_D = 128


def kv4_new_cache(H, S_max):
    """(codes uint8[H][S_max][64], params uint8[H][S_max][4]) zero-filled."""
    return np.zeros((H, S_max, KV_D // 2), dtype=np.uint8), np.zeros((H, S_max, 4), dtype=np.uint8)


def kv4_append(x, pos, clip_ratio, codes, params, rotate=False):
    """Quantise x float32[n][H][128] into cache positions pos .. pos + n - 1 (in place); rotate: order-128
    Hadamard transform of every head vector first."""
    x = _c(x, np.float32)
    n, H, d = x.shape
    assert d == KV_D and codes.shape[0] == H and codes.flags.c_contiguous and params.flags.c_contiguous
    S_max = codes.shape[1]
    _check(lib().rcp_ref_kv4_append(_p(x), n, H, S_max, int(pos), int(bool(rotate)), ctypes.c_float(clip_ratio), _p(codes),
                                    _p(params)),
           "kv4_append")


def kv4_params(params):
    """(scale_bits uint16[H][S_max], zero int16[H][S_max]) views of the parameter bytes."""
    return params.view(np.uint16)[..., 0], params.view(np.int16)[..., 1]


def kv4_dequant(codes, params, pos, n):
    """float64[n][H][128]: the values the stored codes stand for."""
    H, S_max = codes.shape[:2]
    out = np.empty((n, H, KV_D), dtype=np.float64)
    _check(lib().rcp_ref_kv4_dequant(_p(codes), _p(params), H, S_max, int(pos), int(n), _p(out)), "kv4_dequant")
    return out


def kv4_attn_decode(q, S, k_codes, k_params, v_codes, v_params, softmax_scale):
    """float64[H_q][128]: one query token against the first S cached tokens."""
    q = _c(q, np.float64)
    H_q = q.shape[0]
    H_kv, S_max = k_codes.shape[:2]
    out = np.empty((H_q, KV_D), dtype=np.float64)
    _check(lib().rcp_ref_kv4_attn_decode(_p(q), H_q, H_kv, S_max, int(S), _p(k_codes), _p(k_params), _p(v_codes),
                                         _p(v_params), ctypes.c_double(softmax_scale), _p(out)), "kv4_attn_decode")
    return out
