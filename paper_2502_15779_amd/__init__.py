"""Python binding of librcp.so, the MI355X W2A4 GEMV path of RCP (arXiv 2502.15779).

Argument marshalling only: every function takes torch tensors that already live on the
GPU, hands their device pointers and the current HIP stream to the C ABI declared in
include/rcp.h, and returns torch tensors.  PyTorch supplies device memory and streams;
all arithmetic runs in the library's HIP kernels.  There is no CPU fallback: if the
shared library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librcp.so")

F16, F32, BF16 = 0, 1, 2
ROT_NONE, ROT_WHT, ROT_KRON, ROT_HEADS = 0, 1, 2, 3
MAX_M = 16
GROUP = 128  # input channels per quantisation unit of the *_grouped calls

_DTYPES = {torch.float16: F16, torch.float32: F32, torch.bfloat16: BF16}


class RcpError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"librcp error {code}: {message}")
        self.code = code


class _Rotation(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("n_wht", ctypes.c_int), ("m", ctypes.c_int), ("Q", ctypes.c_void_p)]


class Rotation:
    """Host-side rotation descriptor; keeps the device tensor Q alive."""

    def __init__(self, kind=ROT_NONE, n_wht=0, m=1, Q=None):
        self.kind, self.n_wht, self.m, self.Q = int(kind), int(n_wht), int(m), Q
        if Q is not None:
            assert Q.is_cuda and Q.dtype == torch.float32 and Q.is_contiguous() and Q.shape == (m, m)
        self._c = _Rotation(self.kind, self.n_wht, self.m, Q.data_ptr() if Q is not None else None)

    @staticmethod
    def none():
        return Rotation(ROT_NONE)

    @staticmethod
    def wht(n):
        return Rotation(ROT_WHT, n_wht=n)

    @staticmethod
    def heads(n_heads, head_dim):
        """Hadamard across heads: y = (H_{n_heads} (x) I_{head_dim}) x."""
        return Rotation(ROT_HEADS, n_wht=n_heads, m=head_dim)

    @staticmethod
    def kron(n_wht, Q):
        return Rotation(ROT_KRON, n_wht=n_wht, m=Q.shape[0], Q=Q)


class _GemvStep(ctypes.Structure):
    _fields_ = [("packed", ctypes.c_void_p), ("codebook", ctypes.c_void_p), ("N", ctypes.c_int), ("K", ctypes.c_int),
                ("x", ctypes.c_void_p), ("x_dtype", ctypes.c_int), ("rot", _Rotation), ("clip_ratio", ctypes.c_float),
                ("out", ctypes.c_void_p), ("out_dtype", ctypes.c_int), ("xq_out", ctypes.c_void_p),
                ("scale_out", ctypes.c_void_p)]


class GemvStep:
    """One entry of quant_w2a4_gemv_sequence; keeps its tensors alive.  x may be (a view into) the `out` of an earlier entry."""

    def __init__(self, packed, codebook, N, K, x, out, rot: Rotation = None, clip_ratio: float = 1.0, xq_out=None,
                 scale_out=None):
        if x.numel() != K or x.dtype not in _DTYPES:
            raise ValueError("x must hold K values of float16, bfloat16 or float32")
        if out.dtype not in (torch.float16, torch.float32) or out.numel() != N:
            raise ValueError("out must hold N values of float16 or float32")
        if packed.numel() * packed.element_size() < N * K // 4 or codebook.numel() < 4 * N:
            raise ValueError("packed / codebook buffers do not match N, K")
        if xq_out is not None and xq_out.numel() * xq_out.element_size() < K // 2:
            raise ValueError("xq_out too small")
        self.tensors = (packed, codebook, x, out, rot, xq_out, scale_out)
        opt = lambda t, name: _dev(t, name).value if t is not None else None
        r = rot._c if rot is not None else _Rotation(ROT_NONE, 0, 1, None)
        self.c = _GemvStep(_dev(packed, "packed").value, _dev(codebook, "codebook").value, int(N), int(K), _dev(x, "x").value,
                           _DTYPES[x.dtype], r, float(clip_ratio), _dev(out, "out").value, _DTYPES[out.dtype],
                           opt(xq_out, "xq_out"), opt(scale_out, "scale_out"))


def _step_array(steps):
    arr = (_GemvStep * len(steps))()
    for i, s in enumerate(steps):
        arr[i] = s.c
    return arr


def gemv_sequence_workspace(steps, device="cuda:0"):
    """A zeroed workspace for quant_w2a4_gemv_sequence(steps); word 0 (int32) is the error flag."""
    need = int(lib().rcp_gemv_sequence_workspace_bytes(_step_array(steps), len(steps)))
    if need == 0:
        raise RcpError(-2, lib().rcp_last_error().decode())
    return torch.zeros((need + 3) // 4, dtype=torch.int32, device=device)


def quant_w2a4_gemv_sequence(steps, workspace):
    """The entries of `steps` (GemvStep) in order in one launch; an entry may read what an earlier one wrote."""
    _check(lib().rcp_quant_w2a4_gemv_sequence(_step_array(steps), len(steps), _dev(workspace, "workspace"),
                                              workspace.numel() * workspace.element_size(), _stream()))


_lib = None


def build():
    """Compile librcp.so from csrc/ (hipcc, gfx950)."""
    global _lib
    from . import _build
    _lib = None
    return _build.build()


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RcpError(-100, f"{LIB_PATH} is missing: run __graft_entry__.build() first (no CPU fallback exists)")
        L = ctypes.CDLL(LIB_PATH)
        vp, ci, cz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        L.rcp_version.restype = ci
        L.rcp_last_error.restype = ctypes.c_char_p
        L.rcp_set_option.restype = ci
        L.rcp_set_option.argtypes = [ctypes.c_char_p, ci]
        L.rcp_packed_bytes.restype = cz
        L.rcp_packed_bytes.argtypes = [ci, ci]
        L.rcp_act_workspace_bytes.restype = cz
        L.rcp_act_workspace_bytes.argtypes = [ci, ci, ctypes.POINTER(_Rotation)]
        L.rcp_pack_weights.restype = ci
        L.rcp_pack_weights.argtypes = [vp, ci, ci, ci, vp, vp, vp, vp, vp, vp]
        L.rcp_unpack_indices.restype = ci
        L.rcp_unpack_indices.argtypes = [vp, ci, ci, vp, vp]
        L.rcp_rotate_quant_act.restype = ci
        L.rcp_rotate_quant_act.argtypes = [vp, ci, ci, ci, ctypes.POINTER(_Rotation), ctypes.c_float, vp, vp, vp, cz, vp]
        L.rcp_rotate_quant_act_static.restype = ci
        L.rcp_rotate_quant_act_static.argtypes = [vp, ci, ci, ci, ctypes.POINTER(_Rotation), ctypes.c_float, vp, vp, vp]
        L.rcp_w2a4_gemv_variant.restype = ci
        L.rcp_w2a4_gemv_variant.argtypes = [ci, ci, ci]
        L.rcp_gemv_sequence_workspace_bytes.restype = cz
        L.rcp_gemv_sequence_workspace_bytes.argtypes = [ctypes.POINTER(_GemvStep), ci]
        L.rcp_quant_w2a4_gemv_sequence.restype = ci
        L.rcp_quant_w2a4_gemv_sequence.argtypes = [ctypes.POINTER(_GemvStep), ci, vp, cz, vp]
        L.rcp_stream_read.restype = ci
        L.rcp_stream_read.argtypes = [vp, cz, vp, vp]
        L.rcp_rotate_act.restype = ci
        L.rcp_rotate_act.argtypes = [vp, ci, ci, ci, ctypes.POINTER(_Rotation), vp, vp]
        L.rcp_w2a4_gemv.restype = ci
        L.rcp_w2a4_gemv.argtypes = [vp, vp, ci, ci, vp, vp, ci, vp, ci, vp, vp]
        L.rcp_quant_w2a4_gemv.restype = ci
        L.rcp_quant_w2a4_gemv.argtypes = [vp, vp, ci, ci, vp, ci, ctypes.c_float, vp, ci, vp, vp, vp, vp]
        L.rcp_pack_weights_grouped.restype = ci
        L.rcp_pack_weights_grouped.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp]
        L.rcp_unpack_indices_grouped.restype = ci
        L.rcp_unpack_indices_grouped.argtypes = [vp, ci, ci, ci, vp, vp]
        L.rcp_w2a4_gemv_grouped.restype = ci
        L.rcp_w2a4_gemv_grouped.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp, ci, vp, vp]
        L.rcp_w2a4_gemm_grouped.restype = ci
        L.rcp_w2a4_gemm_grouped.argtypes = [vp, vp, ci, ci, ci, vp, vp, ci, vp, ci, vp, vp]
        L.rcp_quant_w2a4_gemv_grouped.restype = ci
        L.rcp_quant_w2a4_gemv_grouped.argtypes = [vp, vp, ci, ci, ci, vp, ci, ctypes.c_float, vp, ci, vp, vp, vp, vp]
        L.rcp_rotate_quant_w2a4_gemv.restype = ci
        L.rcp_rotate_quant_w2a4_gemv.argtypes = [vp, vp, ci, ci, vp, ci, ctypes.POINTER(_Rotation), ctypes.c_float, vp, ci,
                                                 vp, vp, vp, vp]
        L.rcp_w2a16_gemv.restype = ci
        L.rcp_w2a16_gemv.argtypes = [vp, vp, ci, ci, vp, ci, vp, ci, vp]
        L.rcp_pack_weights_w3.restype = ci
        L.rcp_pack_weights_w3.argtypes = [vp, ci, ci, ci, vp, vp, vp, ctypes.POINTER(ctypes.c_float), vp, vp, vp]
        L.rcp_unpack_indices_w3.restype = ci
        L.rcp_unpack_indices_w3.argtypes = [vp, ci, ci, vp, vp]
        L.rcp_w3a4_gemv.restype = ci
        L.rcp_w3a4_gemv.argtypes = [vp, vp, ci, ci, vp, vp, vp, ci, vp, vp]
        L.rcp_quant_w3a4_gemv.restype = ci
        L.rcp_quant_w3a4_gemv.argtypes = [vp, vp, ci, ci, vp, ci, ctypes.c_float, vp, ci, vp, vp, vp, vp]
        L.rcp_kv4_workspace_bytes.restype = ctypes.c_size_t
        L.rcp_kv4_workspace_bytes.argtypes = [ci, ci]
        L.rcp_kv4_append.restype = ci
        L.rcp_kv4_append.argtypes = [vp, ci, ci, ci, ci, ci, ci, ctypes.c_float, vp, vp, vp]
        ip = ctypes.POINTER(ctypes.c_int)
        L.rcp_kv4_append_batched.restype = ci
        L.rcp_kv4_append_batched.argtypes = [vp, ci, ci, ci, ci, ip, ci, ctypes.c_float, vp, vp, vp]
        L.rcp_kv4_attn_decode_batched.restype = ci
        L.rcp_kv4_attn_decode_batched.argtypes = [vp, ci, ci, ci, ci, ci, ip, vp, vp, vp, vp, ctypes.c_float, vp, ci, vp,
                                                  ctypes.c_size_t, vp]
        L.rcp_kv4_append_kv.restype = ci
        L.rcp_kv4_append_kv.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, ctypes.c_float, vp, vp, vp, vp, vp]
        L.rcp_kv4_rotate_attn_decode.restype = ci
        L.rcp_kv4_rotate_attn_decode.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, ctypes.c_float, vp, ci, vp,
                                                 ctypes.c_size_t, vp]
        L.rcp_kv4_attn_decode.restype = ci
        L.rcp_kv4_attn_decode.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, ctypes.c_float, vp, ci, vp,
                                          ctypes.c_size_t, vp]
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise RcpError(rc, lib().rcp_last_error().decode())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, what):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise ValueError(f"{what} must be a contiguous CUDA tensor")
    return ctypes.c_void_p(t.data_ptr())


def version() -> int:
    return int(lib().rcp_version())


def set_option(name: str, value: int) -> None:
    _check(lib().rcp_set_option(name.encode(), int(value)))


def packed_bytes(N: int, K: int) -> int:
    return int(lib().rcp_packed_bytes(N, K))


def act_workspace_bytes(M: int, K: int, rot: Rotation = None) -> int:
    return int(lib().rcp_act_workspace_bytes(M, K, ctypes.byref(rot._c) if rot is not None else None))


def pack_weights(W, clip_lo, clip_hi, part, packed_out=None, codebook_out=None):
    """W [N, K] (fp16 / bf16 / fp32), clip_lo / clip_hi [N] fp32, part [N, 3] fp32
    -> (packed uint8 [N*K/4], codebook fp16 [N, 4])."""
    N, K = W.shape
    nbytes = packed_bytes(N, K)
    if packed_out is None:
        packed_out = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=W.device)
    if codebook_out is None:
        codebook_out = torch.empty((N, 4), dtype=torch.float16, device=W.device)
    for t, name in ((clip_lo, "clip_lo"), (clip_hi, "clip_hi"), (part, "part")):
        if t.dtype != torch.float32:
            raise ValueError(f"{name} must be float32")
    if clip_lo.numel() != N or clip_hi.numel() != N or part.numel() != 3 * N:
        raise ValueError("clip_lo / clip_hi / part do not match N")
    if W.dtype not in _DTYPES:
        raise ValueError("W must be float16, bfloat16 or float32")
    _check(lib().rcp_pack_weights(_dev(W, "W"), _DTYPES[W.dtype], N, K, _dev(clip_lo, "clip_lo"),
                                  _dev(clip_hi, "clip_hi"), _dev(part, "part"), _dev(packed_out, "packed_out"),
                                  _dev(codebook_out, "codebook_out"), _stream()))
    return packed_out, codebook_out


def unpack_indices(packed, N, K, idx_out=None):
    if idx_out is None:
        idx_out = torch.empty((N, K), dtype=torch.uint8, device=packed.device)
    if packed.numel() * packed.element_size() < N * K // 4:
        raise ValueError("packed buffer too small")
    _check(lib().rcp_unpack_indices(_dev(packed, "packed"), N, K, _dev(idx_out, "idx_out"), _stream()))
    return idx_out


def rotate_quant_act(x, rot: Rotation = None, clip_ratio: float = 1.0, xq_out=None, scale_out=None, workspace=None):
    """x [M, K] (fp16 / bf16 / fp32) -> (xq uint8 [M, K/2], scale fp16 [M])."""
    if x.dim() == 1:
        x = x.unsqueeze(0)
    M, K = x.shape
    if x.dtype not in _DTYPES:
        raise ValueError("x must be float16, bfloat16 or float32")
    if xq_out is None:
        xq_out = torch.empty((M, max(K // 2, 1)), dtype=torch.uint8, device=x.device)
    if scale_out is None:
        scale_out = torch.empty((M,), dtype=torch.float16, device=x.device)
    need = act_workspace_bytes(M, K, rot)
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    ws_ptr = _dev(workspace, "workspace") if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().rcp_rotate_quant_act(_dev(x, "x"), _DTYPES[x.dtype], M, K,
                                      ctypes.byref(rot._c) if rot is not None else None,
                                      ctypes.c_float(clip_ratio), _dev(xq_out, "xq_out"), _dev(scale_out, "scale_out"),
                                      ws_ptr, ws_bytes, _stream()))
    return xq_out, scale_out


ACT_STATIC_SCRATCH_BYTES = 1 << 20


def rotate_quant_act_static(x, rot: Rotation, clip_ratio: float, xq_out, scale_out):
    """rotate_quant_act through the entry point that allocates nothing: the caller passes both outputs and the
    Kronecker scratch is the library's fixed device array (at most ACT_STATIC_SCRATCH_BYTES)."""
    if x.dim() == 1:
        x = x.unsqueeze(0)
    M, K = x.shape
    if x.dtype not in _DTYPES:
        raise ValueError("x must be float16, bfloat16 or float32")
    _check(lib().rcp_rotate_quant_act_static(_dev(x, "x"), _DTYPES[x.dtype], M, K,
                                             ctypes.byref(rot._c) if rot is not None else None,
                                             ctypes.c_float(clip_ratio), _dev(xq_out, "xq_out"),
                                             _dev(scale_out, "scale_out"), _stream()))
    return xq_out, scale_out


def w2a4_gemv_variant(N: int, K: int, M: int) -> int:
    """1 = vector-ALU kernel, 2 = matrix-core kernel: what w2a4_gemv runs for this shape under the current options."""
    rc = int(lib().rcp_w2a4_gemv_variant(N, K, M))
    if rc < 0:
        _check(rc)
    return rc


def w2a4_gemv(packed, codebook, N, K, xq, scale, M=1, out=None, out_dtype=torch.float16, partial_sums=None,
              want_partial_sums=False):
    """-> out [M, N] (and the int32 [M, N, 4] per-level partial sums when asked for)."""
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=packed.device)
    if out.dtype not in (torch.float16, torch.float32):
        raise ValueError("out must be float16 or float32")
    if want_partial_sums and partial_sums is None:
        partial_sums = torch.empty((M, N, 4), dtype=torch.int32, device=packed.device)
    if packed.numel() * packed.element_size() < N * K // 4 or codebook.numel() < 4 * N:
        raise ValueError("packed / codebook buffers do not match N, K")
    if xq.numel() * xq.element_size() < M * K // 2 or scale.numel() < M or out.numel() < M * N:
        raise ValueError("xq / scale / out buffers do not match M, N, K")
    if partial_sums is not None and (partial_sums.dtype != torch.int32 or partial_sums.numel() < 4 * M * N):
        raise ValueError("partial_sums must be int32 [M, N, 4]")
    _check(lib().rcp_w2a4_gemv(_dev(packed, "packed"), _dev(codebook, "codebook"), N, K, _dev(xq, "xq"),
                               _dev(scale, "scale"), M, _dev(out, "out"), _DTYPES[out.dtype],
                               _dev(partial_sums, "partial_sums") if partial_sums is not None else None, _stream()))
    return (out, partial_sums) if partial_sums is not None else out


def quant_w2a4_gemv(packed, codebook, N, K, x, clip_ratio=1.0, out=None, out_dtype=torch.float16, xq_out=None,
                    scale_out=None, partial_sums=None, want_partial_sums=False):
    """One token: quantise x (no rotation) and run the GEMV in a single launch -> out [1, N]."""
    if x.numel() != K or x.dtype not in _DTYPES:
        raise ValueError("x must hold K values of float16, bfloat16 or float32")
    if out is None:
        out = torch.empty((1, N), dtype=out_dtype, device=packed.device)
    if out.dtype not in (torch.float16, torch.float32) or out.numel() < N:
        raise ValueError("out must be float16 or float32 with N elements")
    if want_partial_sums and partial_sums is None:
        partial_sums = torch.empty((1, N, 4), dtype=torch.int32, device=packed.device)
    if packed.numel() * packed.element_size() < N * K // 4 or codebook.numel() < 4 * N:
        raise ValueError("packed / codebook buffers do not match N, K")
    if xq_out is not None and xq_out.numel() * xq_out.element_size() < K // 2:
        raise ValueError("xq_out too small")
    if partial_sums is not None and (partial_sums.dtype != torch.int32 or partial_sums.numel() < 4 * N):
        raise ValueError("partial_sums must be int32 [1, N, 4]")
    opt = lambda t, name: _dev(t, name) if t is not None else None
    _check(lib().rcp_quant_w2a4_gemv(_dev(packed, "packed"), _dev(codebook, "codebook"), N, K, _dev(x, "x"),
                                     _DTYPES[x.dtype], ctypes.c_float(clip_ratio), _dev(out, "out"), _DTYPES[out.dtype],
                                     opt(xq_out, "xq_out"), opt(scale_out, "scale_out"), opt(partial_sums, "partial_sums"),
                                     _stream()))
    return (out, partial_sums) if partial_sums is not None else out


def rotate_act(x, rot: Rotation = None, y_out=None):
    """x [M, K] -> y = R x as float32 [M, K] (rotation only)."""
    if x.dim() == 1:
        x = x.unsqueeze(0)
    M, K = x.shape
    if x.dtype not in _DTYPES:
        raise ValueError("x must be float16, bfloat16 or float32")
    if y_out is None:
        y_out = torch.empty((M, K), dtype=torch.float32, device=x.device)
    if y_out.dtype != torch.float32 or y_out.numel() < M * K:
        raise ValueError("y_out must be float32 [M, K]")
    _check(lib().rcp_rotate_act(_dev(x, "x"), _DTYPES[x.dtype], M, K,
                                ctypes.byref(rot._c) if rot is not None else None, _dev(y_out, "y_out"), _stream()))
    return y_out


def stream_read(buffer, nbytes=None, sink=None):
    """Measurement helper: stream `nbytes` of `buffer` through plain 128-bit loads."""
    total = buffer.numel() * buffer.element_size()
    nbytes = total if nbytes is None else min(int(nbytes), total)
    _check(lib().rcp_stream_read(_dev(buffer, "buffer"), nbytes, _dev(sink, "sink") if sink is not None else None, _stream()))


def pack_weights_grouped(W, clip_lo, clip_hi, part, group=GROUP, packed_out=None, codebook_out=None):
    """W [N, K], clip_lo / clip_hi [N, K/group] fp32, part [N, K/group, 3] fp32
    -> (packed uint8 [N*K/4] in the grouped layout, codebook fp16 [N/4, K/group, 4, 4])."""
    N, K = W.shape
    NG = K // group
    if packed_out is None:
        packed_out = torch.empty(max(N * K // 4, 1), dtype=torch.uint8, device=W.device)
    if codebook_out is None:
        codebook_out = torch.empty((max(N // 4, 1), max(NG, 1), 4, 4), dtype=torch.float16, device=W.device)
    for t, name in ((clip_lo, "clip_lo"), (clip_hi, "clip_hi"), (part, "part")):
        if t.dtype != torch.float32:
            raise ValueError(f"{name} must be float32")
    if clip_lo.numel() != N * NG or clip_hi.numel() != N * NG or part.numel() != 3 * N * NG:
        raise ValueError("clip_lo / clip_hi / part do not match N, K/group")
    if W.dtype not in _DTYPES:
        raise ValueError("W must be float16, bfloat16 or float32")
    if packed_out.numel() * packed_out.element_size() < N * K // 4 or codebook_out.numel() < 4 * N * NG:
        raise ValueError("packed_out / codebook_out too small")
    _check(lib().rcp_pack_weights_grouped(_dev(W, "W"), _DTYPES[W.dtype], N, K, group, _dev(clip_lo, "clip_lo"),
                                          _dev(clip_hi, "clip_hi"), _dev(part, "part"), _dev(packed_out, "packed_out"),
                                          _dev(codebook_out, "codebook_out"), _stream()))
    return packed_out, codebook_out


def unpack_indices_grouped(packed, N, K, group=GROUP, idx_out=None):
    if idx_out is None:
        idx_out = torch.empty((N, K), dtype=torch.uint8, device=packed.device)
    if packed.numel() * packed.element_size() < N * K // 4 or idx_out.numel() < N * K:
        raise ValueError("packed / idx_out buffer too small")
    _check(lib().rcp_unpack_indices_grouped(_dev(packed, "packed"), N, K, group, _dev(idx_out, "idx_out"), _stream()))
    return idx_out


def w2a4_gemv_grouped(packed, codebook, N, K, xq, scale, group=GROUP, out=None, out_dtype=torch.float16,
                      partial_sums=None, want_partial_sums=False):
    """One token -> out [1, N] (and the int32 [N, K/group, 4] per-group partial sums when asked for)."""
    NG = max(K // group, 1)
    if out is None:
        out = torch.empty((1, N), dtype=out_dtype, device=packed.device)
    if out.dtype not in (torch.float16, torch.float32) or out.numel() < N:
        raise ValueError("out must be float16 or float32 with N elements")
    if want_partial_sums and partial_sums is None:
        partial_sums = torch.empty((N, NG, 4), dtype=torch.int32, device=packed.device)
    if packed.numel() * packed.element_size() < N * K // 4 or codebook.numel() < 4 * N * NG:
        raise ValueError("packed / codebook buffers do not match N, K, group")
    if xq.numel() * xq.element_size() < K // 2 or scale.numel() < 1:
        raise ValueError("xq / scale buffers do not match K")
    if partial_sums is not None and (partial_sums.dtype != torch.int32 or partial_sums.numel() < 4 * N * NG):
        raise ValueError("partial_sums must be int32 [N, K/group, 4]")
    _check(lib().rcp_w2a4_gemv_grouped(_dev(packed, "packed"), _dev(codebook, "codebook"), N, K, group,
                                       _dev(xq, "xq"), _dev(scale, "scale"), _dev(out, "out"), _DTYPES[out.dtype],
                                       _dev(partial_sums, "partial_sums") if partial_sums is not None else None,
                                       _stream()))
    return (out, partial_sums) if partial_sums is not None else out


def w2a16_gemv(packed, codebook, N, K, x, out=None, out_dtype=torch.float16):
    """Weight-only product for one token: x holds K values (fp16 / bf16 / fp32) -> out [1, N]."""
    if x.numel() != K or x.dtype not in _DTYPES:
        raise ValueError("x must hold K values of float16, bfloat16 or float32")
    if out is None:
        out = torch.empty((1, N), dtype=out_dtype, device=packed.device)
    if out.dtype not in (torch.float16, torch.float32) or out.numel() < N:
        raise ValueError("out must be float16 or float32 with N elements")
    if packed.numel() * packed.element_size() < N * K // 4 or codebook.numel() < 4 * N:
        raise ValueError("packed / codebook buffers do not match N, K")
    _check(lib().rcp_w2a16_gemv(_dev(packed, "packed"), _dev(codebook, "codebook"), N, K, _dev(x, "x"),
                                _DTYPES[x.dtype], _dev(out, "out"), _DTYPES[out.dtype], _stream()))
    return out


def quant_w2a4_gemv_grouped(packed, codebook, N, K, x, clip_ratio=1.0, group=GROUP, out=None, out_dtype=torch.float16,
                            xq_out=None, scale_out=None, partial_sums=None, want_partial_sums=False):
    """One token, group-wise LUTs: quantise x (no rotation) and run the grouped GEMV in a single launch."""
    NG = max(K // group, 1)
    if x.numel() != K or x.dtype not in _DTYPES:
        raise ValueError("x must hold K values of float16, bfloat16 or float32")
    if out is None:
        out = torch.empty((1, N), dtype=out_dtype, device=packed.device)
    if out.dtype not in (torch.float16, torch.float32) or out.numel() < N:
        raise ValueError("out must be float16 or float32 with N elements")
    if want_partial_sums and partial_sums is None:
        partial_sums = torch.empty((N, NG, 4), dtype=torch.int32, device=packed.device)
    if packed.numel() * packed.element_size() < N * K // 4 or codebook.numel() < 4 * N * NG:
        raise ValueError("packed / codebook buffers do not match N, K, group")
    if xq_out is not None and xq_out.numel() * xq_out.element_size() < K // 2:
        raise ValueError("xq_out too small")
    if partial_sums is not None and (partial_sums.dtype != torch.int32 or partial_sums.numel() < 4 * N * NG):
        raise ValueError("partial_sums must be int32 [N, K/group, 4]")
    opt = lambda t, name: _dev(t, name) if t is not None else None
    _check(lib().rcp_quant_w2a4_gemv_grouped(_dev(packed, "packed"), _dev(codebook, "codebook"), N, K, group,
                                             _dev(x, "x"), _DTYPES[x.dtype], ctypes.c_float(clip_ratio), _dev(out, "out"),
                                             _DTYPES[out.dtype], opt(xq_out, "xq_out"), opt(scale_out, "scale_out"),
                                             opt(partial_sums, "partial_sums"), _stream()))
    return (out, partial_sums) if partial_sums is not None else out


def w2a4_gemm_grouped(packed, codebook, N, K, xq, scale, M, group=GROUP, out=None, out_dtype=torch.float16,
                      partial_sums=None, want_partial_sums=False):
    """Group-wise LUTs, M tokens -> out [M, N] (and int32 [M, N, K/group, 4] partial sums when asked for)."""
    NG = max(K // group, 1)
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=packed.device)
    if out.dtype not in (torch.float16, torch.float32) or out.numel() < M * N:
        raise ValueError("out must be float16 or float32 with M*N elements")
    if want_partial_sums and partial_sums is None:
        partial_sums = torch.empty((M, N, NG, 4), dtype=torch.int32, device=packed.device)
    if packed.numel() * packed.element_size() < N * K // 4 or codebook.numel() < 4 * N * NG:
        raise ValueError("packed / codebook buffers do not match N, K, group")
    if xq.numel() * xq.element_size() < M * K // 2 or scale.numel() < M:
        raise ValueError("xq / scale buffers do not match M, K")
    if partial_sums is not None and (partial_sums.dtype != torch.int32 or partial_sums.numel() < 4 * M * N * NG):
        raise ValueError("partial_sums must be int32 [M, N, K/group, 4]")
    _check(lib().rcp_w2a4_gemm_grouped(_dev(packed, "packed"), _dev(codebook, "codebook"), N, K, group,
                                       _dev(xq, "xq"), _dev(scale, "scale"), M, _dev(out, "out"), _DTYPES[out.dtype],
                                       _dev(partial_sums, "partial_sums") if partial_sums is not None else None,
                                       _stream()))
    return (out, partial_sums) if partial_sums is not None else out


def rotate_quant_w2a4_gemv(packed, codebook, N, K, x, rot=None, clip_ratio=1.0, out=None, out_dtype=torch.float16,
                           xq_out=None, scale_out=None, partial_sums=None, want_partial_sums=False):
    """One token: rotation (none or across heads), quantiser and GEMV in a single launch -> out [1, N]."""
    if x.numel() != K or x.dtype not in _DTYPES:
        raise ValueError("x must hold K values of float16, bfloat16 or float32")
    if out is None:
        out = torch.empty((1, N), dtype=out_dtype, device=packed.device)
    if out.dtype not in (torch.float16, torch.float32) or out.numel() < N:
        raise ValueError("out must be float16 or float32 with N elements")
    if want_partial_sums and partial_sums is None:
        partial_sums = torch.empty((1, N, 4), dtype=torch.int32, device=packed.device)
    if packed.numel() * packed.element_size() < N * K // 4 or codebook.numel() < 4 * N:
        raise ValueError("packed / codebook buffers do not match N, K")
    if xq_out is not None and xq_out.numel() * xq_out.element_size() < K // 2:
        raise ValueError("xq_out too small")
    if partial_sums is not None and (partial_sums.dtype != torch.int32 or partial_sums.numel() < 4 * N):
        raise ValueError("partial_sums must be int32 [1, N, 4]")
    opt = lambda t, name: _dev(t, name) if t is not None else None
    _check(lib().rcp_rotate_quant_w2a4_gemv(_dev(packed, "packed"), _dev(codebook, "codebook"), N, K, _dev(x, "x"),
                                            _DTYPES[x.dtype], ctypes.byref(rot._c) if rot is not None else None,
                                            ctypes.c_float(clip_ratio), _dev(out, "out"), _DTYPES[out.dtype],
                                            opt(xq_out, "xq_out"), opt(scale_out, "scale_out"),
                                            opt(partial_sums, "partial_sums"), _stream()))
    return (out, partial_sums) if partial_sums is not None else out


# ---- 3-bit variant (eight levels per output channel) ------------------------------------------
def pack_weights_w3(W, clip_lo, clip_hi, frac, grid, packed_out=None, codebook_out=None):
    """W [N, K] (fp16 / bf16 / fp32), clip_lo / clip_hi / frac [N] fp32 on the GPU, grid: eight ascending
    host floats -> (packed uint8 [3*N*K/8], codebook fp16 [N, 8])."""
    N, K = W.shape
    if packed_out is None:
        packed_out = torch.empty(max(3 * N * K // 8, 1), dtype=torch.uint8, device=W.device)
    if codebook_out is None:
        codebook_out = torch.empty((N, 8), dtype=torch.float16, device=W.device)
    for t, name in ((clip_lo, "clip_lo"), (clip_hi, "clip_hi"), (frac, "frac")):
        if t.dtype != torch.float32 or t.numel() != N:
            raise ValueError(f"{name} must be float32 with N elements")
    if W.dtype not in _DTYPES:
        raise ValueError("W must be float16, bfloat16 or float32")
    g = [float(v) for v in grid]
    if len(g) != 8:
        raise ValueError("grid must hold eight values")
    if packed_out.numel() * packed_out.element_size() < 3 * N * K // 8 or codebook_out.numel() < 8 * N:
        raise ValueError("packed_out / codebook_out buffers do not match N, K")
    _check(lib().rcp_pack_weights_w3(_dev(W, "W"), _DTYPES[W.dtype], N, K, _dev(clip_lo, "clip_lo"),
                                     _dev(clip_hi, "clip_hi"), _dev(frac, "frac"), (ctypes.c_float * 8)(*g),
                                     _dev(packed_out, "packed_out"), _dev(codebook_out, "codebook_out"), _stream()))
    return packed_out, codebook_out


def unpack_indices_w3(packed, N, K, idx_out=None):
    if idx_out is None:
        idx_out = torch.empty((N, K), dtype=torch.uint8, device=packed.device)
    if packed.numel() * packed.element_size() < 3 * N * K // 8:
        raise ValueError("packed buffer too small")
    _check(lib().rcp_unpack_indices_w3(_dev(packed, "packed"), N, K, _dev(idx_out, "idx_out"), _stream()))
    return idx_out


def w3a4_gemv(packed, codebook, N, K, xq, scale, out=None, out_dtype=torch.float16, partial_sums=None,
              want_partial_sums=False):
    """One token -> out [1, N] (and the int32 [N, 8] per-level partial sums when asked for)."""
    if out is None:
        out = torch.empty((1, N), dtype=out_dtype, device=packed.device)
    if out.dtype not in (torch.float16, torch.float32) or out.numel() < N:
        raise ValueError("out must be float16 or float32 with N elements")
    if want_partial_sums and partial_sums is None:
        partial_sums = torch.empty((N, 8), dtype=torch.int32, device=packed.device)
    if packed.numel() * packed.element_size() < 3 * N * K // 8 or codebook.numel() < 8 * N:
        raise ValueError("packed / codebook buffers do not match N, K")
    if xq.numel() * xq.element_size() < K // 2 or scale.numel() < 1:
        raise ValueError("xq / scale buffers do not match K")
    if partial_sums is not None and (partial_sums.dtype != torch.int32 or partial_sums.numel() < 8 * N):
        raise ValueError("partial_sums must be int32 [N, 8]")
    _check(lib().rcp_w3a4_gemv(_dev(packed, "packed"), _dev(codebook, "codebook"), N, K, _dev(xq, "xq"),
                               _dev(scale, "scale"), _dev(out, "out"), _DTYPES[out.dtype],
                               _dev(partial_sums, "partial_sums") if partial_sums is not None else None, _stream()))
    return (out, partial_sums) if partial_sums is not None else out


def quant_w3a4_gemv(packed, codebook, N, K, x, clip_ratio=1.0, out=None, out_dtype=torch.float16, xq_out=None,
                    scale_out=None, partial_sums=None, want_partial_sums=False):
    """One token, 3-bit weights: quantise x (no rotation) and run the eight-level GEMV in a single launch."""
    if x.numel() != K or x.dtype not in _DTYPES:
        raise ValueError("x must hold K values of float16, bfloat16 or float32")
    if out is None:
        out = torch.empty((1, N), dtype=out_dtype, device=packed.device)
    if out.dtype not in (torch.float16, torch.float32) or out.numel() < N:
        raise ValueError("out must be float16 or float32 with N elements")
    if want_partial_sums and partial_sums is None:
        partial_sums = torch.empty((N, 8), dtype=torch.int32, device=packed.device)
    if packed.numel() * packed.element_size() < 3 * N * K // 8 or codebook.numel() < 8 * N:
        raise ValueError("packed / codebook buffers do not match N, K")
    if xq_out is not None and xq_out.numel() * xq_out.element_size() < K // 2:
        raise ValueError("xq_out too small")
    if partial_sums is not None and (partial_sums.dtype != torch.int32 or partial_sums.numel() < 8 * N):
        raise ValueError("partial_sums must be int32 [N, 8]")
    opt = lambda t, name: _dev(t, name) if t is not None else None
    _check(lib().rcp_quant_w3a4_gemv(_dev(packed, "packed"), _dev(codebook, "codebook"), N, K, _dev(x, "x"),
                                     _DTYPES[x.dtype], ctypes.c_float(clip_ratio), _dev(out, "out"), _DTYPES[out.dtype],
                                     opt(xq_out, "xq_out"), opt(scale_out, "scale_out"), opt(partial_sums, "partial_sums"),
                                     _stream()))
    return (out, partial_sums) if partial_sums is not None else out


# ---- 4-bit KV cache ------------------------------------------------------------------------
KV_HEAD_DIM = 128


def kv4_new_cache(H, S_max, device):
    """(codes uint8 [H, S_max, 64], params uint8 [H, S_max, 4]) zero-filled device buffers."""
    return (torch.zeros((H, S_max, KV_HEAD_DIM // 2), dtype=torch.uint8, device=device),
            torch.zeros((H, S_max, 4), dtype=torch.uint8, device=device))


def kv4_workspace_bytes(H_q, S):
    return int(lib().rcp_kv4_workspace_bytes(H_q, S))


def kv4_append(x, pos, codes, params, clip_ratio=0.95, rotate=False):
    """Quantise x [n_tokens, H, 128] into cache positions pos .. pos + n_tokens - 1 (in place); rotate: the
    order-128 Hadamard transform of every head vector first (keys)."""
    if x.dim() != 3 or x.shape[2] != KV_HEAD_DIM or not x.is_contiguous():
        raise ValueError("x must be contiguous [n_tokens, H, 128]")
    n, H = int(x.shape[0]), int(x.shape[1])
    if codes.dtype != torch.uint8 or params.dtype != torch.uint8 or codes.dim() != 3 or codes.shape[0] != H or \
            codes.shape[2] != KV_HEAD_DIM // 2 or tuple(params.shape) != (H, codes.shape[1], 4) or \
            not codes.is_contiguous() or not params.is_contiguous():
        raise ValueError("codes must be uint8 [H, S_max, 64] and params uint8 [H, S_max, 4], contiguous")
    if n == 0:      # an empty tensor has no device pointer to hand over
        return
    _check(lib().rcp_kv4_append(_dev(x, "x"), _DTYPES[x.dtype], n, H, int(codes.shape[1]), int(pos), int(bool(rotate)),
                                ctypes.c_float(clip_ratio), _dev(codes, "codes"), _dev(params, "params"), _stream()))


def kv4_attn_decode(q, S, k_codes, k_params, v_codes, v_params, softmax_scale, out=None, out_dtype=torch.float32,
                    workspace=None):
    """One query token [H_q, 128] against the first S cached tokens -> out [H_q, 128]."""
    if q.dim() != 2 or q.shape[1] != KV_HEAD_DIM or not q.is_contiguous():
        raise ValueError("q must be contiguous [H_q, 128]")
    H_q, H_kv, S_max = int(q.shape[0]), int(k_codes.shape[0]), int(k_codes.shape[1])
    for c, p in ((k_codes, k_params), (v_codes, v_params)):
        if c.dtype != torch.uint8 or p.dtype != torch.uint8 or tuple(c.shape) != (H_kv, S_max, KV_HEAD_DIM // 2) or \
                tuple(p.shape) != (H_kv, S_max, 4) or not c.is_contiguous() or not p.is_contiguous():
            raise ValueError("cache buffers must be uint8 [H_kv, S_max, 64] / [H_kv, S_max, 4], contiguous")
    if out is None:
        out = torch.empty((H_q, KV_HEAD_DIM), dtype=out_dtype, device=q.device)
    if out.dtype not in (torch.float16, torch.float32) or out.numel() < H_q * KV_HEAD_DIM:
        raise ValueError("out must be float16 or float32 [H_q, 128]")
    if workspace is None:
        workspace = torch.empty(max(kv4_workspace_bytes(H_q, S), 16), dtype=torch.uint8, device=q.device)
    _check(lib().rcp_kv4_attn_decode(_dev(q, "q"), _DTYPES[q.dtype], H_q, H_kv, S_max, int(S), _dev(k_codes, "k_codes"),
                                     _dev(k_params, "k_params"), _dev(v_codes, "v_codes"), _dev(v_params, "v_params"),
                                     ctypes.c_float(softmax_scale), _dev(out, "out"), _DTYPES[out.dtype],
                                     _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                                     _stream()))
    return out


def kv4_append_kv(k, v, pos, k_codes, k_params, v_codes, v_params, clip_ratio=0.95, rotate_k=False):
    """The new keys and values k, v [n_tokens, H, 128] of the same tokens into both caches in one launch."""
    if k.dim() != 3 or k.shape[2] != KV_HEAD_DIM or not k.is_contiguous() or v.shape != k.shape or v.dtype != k.dtype or \
            not v.is_contiguous():
        raise ValueError("k and v must be contiguous [n_tokens, H, 128] of one dtype")
    n, H = int(k.shape[0]), int(k.shape[1])
    for codes, params in ((k_codes, k_params), (v_codes, v_params)):
        if codes.dtype != torch.uint8 or params.dtype != torch.uint8 or codes.dim() != 3 or codes.shape[0] != H or \
                codes.shape[2] != KV_HEAD_DIM // 2 or tuple(params.shape) != (H, codes.shape[1], 4) or \
                not codes.is_contiguous() or not params.is_contiguous() or codes.shape[1] != k_codes.shape[1]:
            raise ValueError("codes must be uint8 [H, S_max, 64] and params uint8 [H, S_max, 4], contiguous, one S_max")
    if n == 0:
        return
    _check(lib().rcp_kv4_append_kv(_dev(k, "k"), _dev(v, "v"), _DTYPES[k.dtype], n, H, int(k_codes.shape[1]), int(pos),
                                   int(bool(rotate_k)), ctypes.c_float(clip_ratio), _dev(k_codes, "k_codes"),
                                   _dev(k_params, "k_params"), _dev(v_codes, "v_codes"), _dev(v_params, "v_params"), _stream()))


def kv4_rotate_attn_decode(q, S, k_codes, k_params, v_codes, v_params, softmax_scale, out=None, out_dtype=torch.float32,
                           workspace=None):
    """kv4_attn_decode on the un-rotated query: the order-128 Hadamard rotation of every query head runs inside the
    attention kernel."""
    if q.dim() != 2 or q.shape[1] != KV_HEAD_DIM or not q.is_contiguous():
        raise ValueError("q must be contiguous [H_q, 128]")
    H_q, H_kv, S_max = int(q.shape[0]), int(k_codes.shape[0]), int(k_codes.shape[1])
    for c, p in ((k_codes, k_params), (v_codes, v_params)):
        if c.dtype != torch.uint8 or p.dtype != torch.uint8 or tuple(c.shape) != (H_kv, S_max, KV_HEAD_DIM // 2) or \
                tuple(p.shape) != (H_kv, S_max, 4) or not c.is_contiguous() or not p.is_contiguous():
            raise ValueError("cache buffers must be uint8 [H_kv, S_max, 64] / [H_kv, S_max, 4], contiguous")
    if out is None:
        out = torch.empty((H_q, KV_HEAD_DIM), dtype=out_dtype, device=q.device)
    if out.dtype not in (torch.float16, torch.float32) or out.numel() < H_q * KV_HEAD_DIM:
        raise ValueError("out must be float16 or float32 [H_q, 128]")
    if workspace is None:
        workspace = torch.empty(max(kv4_workspace_bytes(H_q, S), 16), dtype=torch.uint8, device=q.device)
    _check(lib().rcp_kv4_rotate_attn_decode(_dev(q, "q"), _DTYPES[q.dtype], H_q, H_kv, S_max, int(S), _dev(k_codes, "k_codes"),
                                            _dev(k_params, "k_params"), _dev(v_codes, "v_codes"), _dev(v_params, "v_params"),
                                            ctypes.c_float(softmax_scale), _dev(out, "out"), _DTYPES[out.dtype],
                                            _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                                            _stream()))
    return out


def kv4_append_batched(x, positions, codes, params, clip_ratio=0.95, rotate=False):
    """One new token for each of B sequences: x [B, H, 128] into the pooled cache codes [B*H, S_max, 64] /
    params [B*H, S_max, 4], sequence b at positions[b] (a host list of ints)."""
    if x.dim() != 3 or x.shape[2] != KV_HEAD_DIM or not x.is_contiguous():
        raise ValueError("x must be contiguous [B, H, 128]")
    B, H = int(x.shape[0]), int(x.shape[1])
    if len(positions) != B:
        raise ValueError("one position per sequence")
    if codes.dtype != torch.uint8 or params.dtype != torch.uint8 or codes.dim() != 3 or codes.shape[0] != B * H or \
            codes.shape[2] != KV_HEAD_DIM // 2 or tuple(params.shape) != (B * H, codes.shape[1], 4) or \
            not codes.is_contiguous() or not params.is_contiguous():
        raise ValueError("codes must be uint8 [B*H, S_max, 64] and params uint8 [B*H, S_max, 4], contiguous")
    pos = (ctypes.c_int * B)(*[int(p) for p in positions])
    _check(lib().rcp_kv4_append_batched(_dev(x, "x"), _DTYPES[x.dtype], B, H, int(codes.shape[1]), pos, int(bool(rotate)),
                                        ctypes.c_float(clip_ratio), _dev(codes, "codes"), _dev(params, "params"), _stream()))


def kv4_attn_decode_batched(q, lengths, k_codes, k_params, v_codes, v_params, softmax_scale, out=None,
                            out_dtype=torch.float32, workspace=None):
    """B sequences: q [B, H_q, 128], sequence b against its first lengths[b] cached tokens of the pooled cache
    [B*H_kv, S_max, ...] -> out [B, H_q, 128]."""
    if q.dim() != 3 or q.shape[2] != KV_HEAD_DIM or not q.is_contiguous():
        raise ValueError("q must be contiguous [B, H_q, 128]")
    B, H_q = int(q.shape[0]), int(q.shape[1])
    if len(lengths) != B or k_codes.shape[0] % B != 0:
        raise ValueError("one length per sequence, and a pooled cache of B * H_kv heads")
    H_kv, S_max = int(k_codes.shape[0]) // B, int(k_codes.shape[1])
    for c, p in ((k_codes, k_params), (v_codes, v_params)):
        if c.dtype != torch.uint8 or p.dtype != torch.uint8 or tuple(c.shape) != (B * H_kv, S_max, KV_HEAD_DIM // 2) or \
                tuple(p.shape) != (B * H_kv, S_max, 4) or not c.is_contiguous() or not p.is_contiguous():
            raise ValueError("cache buffers must be uint8 [B*H_kv, S_max, 64] / [B*H_kv, S_max, 4], contiguous")
    if out is None:
        out = torch.empty((B, H_q, KV_HEAD_DIM), dtype=out_dtype, device=q.device)
    if out.dtype not in (torch.float16, torch.float32) or out.numel() < B * H_q * KV_HEAD_DIM:
        raise ValueError("out must be float16 or float32 [B, H_q, 128]")
    if workspace is None:
        workspace = torch.empty(max(B * kv4_workspace_bytes(H_q, max(int(n) for n in lengths)), 16), dtype=torch.uint8,
                                device=q.device)
    lens = (ctypes.c_int * B)(*[int(n) for n in lengths])
    _check(lib().rcp_kv4_attn_decode_batched(_dev(q, "q"), _DTYPES[q.dtype], B, H_q, H_kv, S_max, lens,
                                             _dev(k_codes, "k_codes"), _dev(k_params, "k_params"), _dev(v_codes, "v_codes"),
                                             _dev(v_params, "v_params"), ctypes.c_float(softmax_scale), _dev(out, "out"),
                                             _DTYPES[out.dtype], _dev(workspace, "workspace"),
                                             workspace.numel() * workspace.element_size(), _stream()))
    return out
