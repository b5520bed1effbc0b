"""Host-only checks of the C ABI: the library loads without a GPU, exports every function that
include/rcp.h declares, and turns bad arguments into error codes before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "rcp.h")
LIB = os.path.join(ROOT, "paper_2502_15779_amd", "librcp.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    return ctypes.CDLL(LIB)


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rcp_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_function_is_exported(lib):
    names = _declared_functions()
    assert {"rcp_pack_weights", "rcp_rotate_quant_act", "rcp_w2a4_gemv", "rcp_unpack_indices",
            "rcp_packed_bytes", "rcp_act_workspace_bytes", "rcp_last_error", "rcp_version",
            "rcp_set_option", "rcp_quant_w2a4_gemv", "rcp_rotate_act", "rcp_stream_read",
            "rcp_pack_weights_grouped", "rcp_unpack_indices_grouped", "rcp_w2a4_gemv_grouped",
            "rcp_w2a16_gemv", "rcp_quant_w2a4_gemv_grouped", "rcp_w2a4_gemm_grouped",
            "rcp_rotate_quant_w2a4_gemv", "rcp_pack_weights_w3", "rcp_unpack_indices_w3", "rcp_w3a4_gemv",
            "rcp_kv4_workspace_bytes", "rcp_kv4_append", "rcp_kv4_attn_decode", "rcp_quant_w3a4_gemv",
            "rcp_kv4_append_batched", "rcp_kv4_attn_decode_batched", "rcp_kv4_append_kv",
            "rcp_kv4_rotate_attn_decode"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_size_queries(lib):
    lib.rcp_packed_bytes.restype = ctypes.c_size_t
    assert lib.rcp_packed_bytes(4096, 4096) == 4096 * 4096 // 4
    assert lib.rcp_packed_bytes(4096, 11008) == 11272192
    assert lib.rcp_packed_bytes(6, 32) == 0 and lib.rcp_packed_bytes(8, 24) == 0 and lib.rcp_packed_bytes(0, 32) == 0


class Rot(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("n_wht", ctypes.c_int), ("m", ctypes.c_int), ("Q", ctypes.c_void_p)]


def test_argument_errors_need_no_gpu(lib):
    lib.rcp_last_error.restype = ctypes.c_char_p
    vp = ctypes.c_void_p
    fake = vp(0x1000)  # aligned, never dereferenced: every call below must fail validation first
    odd = vp(0x1004)
    gemv = lib.rcp_w2a4_gemv
    gemv.argtypes = [vp, vp, ctypes.c_int, ctypes.c_int, vp, vp, ctypes.c_int, vp, ctypes.c_int, vp, vp]
    assert gemv(None, fake, 8, 32, fake, fake, 1, fake, 0, None, None) == -1
    assert b"NULL" in lib.rcp_last_error()
    assert gemv(fake, fake, 6, 32, fake, fake, 1, fake, 0, None, None) == -2
    assert gemv(fake, fake, 8, 48, fake, fake, 1, fake, 0, None, None) == -2
    assert gemv(fake, fake, 8, 32, fake, fake, 0, fake, 0, None, None) == -2
    assert gemv(fake, fake, 8, 32, fake, fake, 17, fake, 0, None, None) == -2
    assert gemv(fake, fake, 8, 32, fake, fake, 1, fake, 2, None, None) == -4
    assert gemv(odd, fake, 8, 32, fake, fake, 1, fake, 0, None, None) == -3
    pack = lib.rcp_pack_weights
    pack.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp, vp, vp, vp, vp]
    assert pack(fake, 0, 8, 32, fake, fake, None, fake, fake, None) == -1
    assert pack(fake, 7, 8, 32, fake, fake, fake, fake, fake, None) == -4
    assert pack(fake, 0, 8, 40, fake, fake, fake, fake, fake, None) == -2
    act = lib.rcp_rotate_quant_act
    act.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(Rot), ctypes.c_float, vp, vp, vp,
                    ctypes.c_size_t, vp]
    assert act(fake, 0, 1, 64, None, 1.5, fake, fake, None, 0, None) == -4      # clip ratio
    assert act(fake, 0, 1, 96, ctypes.byref(Rot(1, 96, 1, None)), 1.0, fake, fake, None, 0, None) == -2
    assert act(fake, 0, 1, 64, ctypes.byref(Rot(1, 32, 1, None)), 1.0, fake, fake, None, 0, None) == -2
    assert act(fake, 0, 1, 96, ctypes.byref(Rot(2, 32, 4, fake)), 1.0, fake, fake, None, 0, None) == -2
    assert act(fake, 0, 1, 96, ctypes.byref(Rot(2, 32, 3, None)), 1.0, fake, fake, None, 0, None) == -1
    assert act(fake, 0, 1, 96, ctypes.byref(Rot(2, 32, 3, fake)), 1.0, fake, fake, None, 0, None) == -5
    assert b"workspace" in lib.rcp_last_error()
    assert act(fake, 0, 1, 64, ctypes.byref(Rot(9, 0, 0, None)), 1.0, fake, fake, None, 0, None) == -4
    # across-heads Hadamard: heads a power of two in 2..64, head size a multiple of 8, heads * size == K
    assert act(fake, 0, 1, 4096, ctypes.byref(Rot(3, 32, 64, None)), 1.0, fake, fake, None, 0, None) == -2
    assert act(fake, 0, 1, 4096, ctypes.byref(Rot(3, 128, 32, None)), 1.0, fake, fake, None, 0, None) == -4
    assert act(fake, 0, 1, 96, ctypes.byref(Rot(3, 8, 12, None)), 1.0, fake, fake, None, 0, None) == -2
    assert act(fake, 0, 1, 96, ctypes.byref(Rot(3, 6, 16, None)), 1.0, fake, fake, None, 0, None) == -2
    ci = ctypes.c_int
    gg = lib.rcp_w2a4_gemv_grouped
    gg.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp, ci, vp, vp]
    assert gg(fake, fake, 8, 256, 128, fake, None, fake, 0, None, None) == -1
    assert gg(fake, fake, 8, 256, 64, fake, fake, fake, 0, None, None) == -4     # group size other than 128
    assert b"128" in lib.rcp_last_error()
    assert gg(fake, fake, 8, 160, 128, fake, fake, fake, 0, None, None) == -2    # K not a multiple of the group
    assert gg(fake, fake, 6, 256, 128, fake, fake, fake, 0, None, None) == -2
    assert gg(fake, fake, 8, 256, 128, odd, fake, fake, 0, None, None) == -3
    wo = lib.rcp_w2a16_gemv
    wo.argtypes = [vp, vp, ci, ci, vp, ci, vp, ci, vp]
    assert wo(fake, fake, 8, 64, None, 0, fake, 0, None) == -1
    assert wo(fake, fake, 8, 72, fake, 0, fake, 0, None) == -2
    assert wo(fake, fake, 8, 64, fake, 3, fake, 0, None) == -4
    assert wo(fake, fake, 8, 64, fake, 0, fake, 2, None) == -4
    assert wo(fake, fake, 8, 64, odd, 0, fake, 0, None) == -3
    pg = lib.rcp_pack_weights_grouped
    pg.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp]
    assert pg(fake, 0, 8, 256, 128, fake, None, fake, fake, fake, None) == -1
    assert pg(fake, 0, 8, 256, 32, fake, fake, fake, fake, fake, None) == -4
    assert pg(fake, 5, 8, 256, 128, fake, fake, fake, fake, fake, None) == -4
    ug = lib.rcp_unpack_indices_grouped
    ug.argtypes = [vp, ci, ci, ci, vp, vp]
    assert ug(fake, 8, 96, 128, fake, None) == -2
    lib.rcp_set_option.argtypes = [ctypes.c_char_p, ctypes.c_int]
    assert lib.rcp_set_option(b"gemv_lanes", 48) == -4
    assert lib.rcp_set_option(b"nonsense", 1) == -4
    assert lib.rcp_set_option(b"gemv_lanes", 0) == 0
    assert lib.rcp_set_option(b"gemm_waves", 3) == -4
    assert lib.rcp_set_option(b"gemm_waves", 8) == 0 and lib.rcp_set_option(b"gemm_waves", 0) == 0
    assert lib.rcp_set_option(b"gemv_variant", 3) == -4
    assert lib.rcp_set_option(b"kv_tokens", 96) == -4
    assert lib.rcp_set_option(b"kv_tokens", 128) == 0 and lib.rcp_set_option(b"kv_tokens", 1024) == 0
    assert lib.rcp_set_option(b"kv_tokens", 4096) == -4 and lib.rcp_set_option(b"kv_tokens", 0) == 0
    assert lib.rcp_set_option(b"gemv_nt", 3) == -4 and lib.rcp_set_option(b"gemv_nt", 1) == 0 and lib.rcp_set_option(b"gemv_nt", 0) == 0
    assert lib.rcp_set_option(b"gemm_stage", 3) == -4 and lib.rcp_set_option(b"gemm_stage", 2) == 0
    assert lib.rcp_set_option(b"gemm_stage", 0) == 0
    assert lib.rcp_set_option(b"gemm_rows", 30) == -4 and lib.rcp_set_option(b"gemm_rows", 12) == -4
    assert lib.rcp_set_option(b"gemm_rows", 68) == -4 and lib.rcp_set_option(b"gemm_rows", 44) == 0
    assert lib.rcp_set_option(b"gemm_rows", 16) == 0 and lib.rcp_set_option(b"gemm_rows", 0) == 0
    assert lib.rcp_set_option(b"gemv_waves", 2) == -4
    assert lib.rcp_set_option(b"gemv_waves", 8) == 0 and lib.rcp_set_option(b"gemv_waves", 0) == 0
    assert lib.rcp_set_option(b"gemv_oneshot", 3) == -4
    assert lib.rcp_set_option(b"gemv_oneshot", 2) == 0 and lib.rcp_set_option(b"gemv_oneshot", 0) == 0
    gmm = lib.rcp_w2a4_gemm_grouped
    gmm.argtypes = [vp, vp, ci, ci, ci, vp, vp, ci, vp, ci, vp, vp]
    assert gmm(fake, fake, 8, 256, 128, fake, fake, 0, fake, 0, None, None) == -2
    assert gmm(fake, fake, 8, 256, 128, fake, fake, 17, fake, 0, None, None) == -2
    assert gmm(fake, fake, 8, 256, 96, fake, fake, 4, fake, 0, None, None) == -4
    qg = lib.rcp_quant_w2a4_gemv_grouped
    qg.argtypes = [vp, vp, ci, ci, ci, vp, ci, ctypes.c_float, vp, ci, vp, vp, vp, vp]
    assert qg(fake, fake, 8, 256, 128, fake, 0, 0.0, fake, 0, None, None, None, None) == -4   # clip ratio
    assert qg(fake, fake, 8, 256, 128, None, 0, 1.0, fake, 0, None, None, None, None) == -1
    # 3-bit variant: the grid is a host array and is checked before anything is launched
    p3 = lib.rcp_pack_weights_w3
    f8 = ctypes.c_float * 8
    p3.argtypes = [vp, ci, ci, ci, vp, vp, vp, ctypes.POINTER(ctypes.c_float), vp, vp, vp]
    good = f8(-1, -0.5, -0.2, 0, 0.15, 0.3, 0.6, 1)
    assert p3(fake, 0, 8, 64, fake, fake, fake, None, fake, fake, None) == -1
    assert p3(fake, 0, 8, 64, fake, fake, fake, f8(-1, -0.5, -0.5, 0, 0.15, 0.3, 0.6, 1), fake, fake, None) == -4
    assert b"ascending" in lib.rcp_last_error()
    assert p3(fake, 0, 8, 64, fake, fake, fake, f8(-1, -0.5, -0.2, 0, 0.15, 0.3, 0.6, float("inf")), fake, fake, None) == -4
    assert p3(fake, 0, 8, 64, fake, fake, fake, f8(float("nan"), -0.5, -0.2, 0, 0.15, 0.3, 0.6, 1), fake, fake, None) == -4
    assert p3(fake, 0, 6, 64, fake, fake, fake, good, fake, fake, None) == -2
    assert p3(fake, 4, 8, 64, fake, fake, fake, good, fake, fake, None) == -4
    assert p3(odd, 0, 8, 64, fake, fake, fake, good, fake, fake, None) == -3
    g3 = lib.rcp_w3a4_gemv
    g3.argtypes = [vp, vp, ci, ci, vp, vp, vp, ci, vp, vp]
    assert g3(fake, fake, 8, 64, fake, None, fake, 0, None, None) == -1
    assert g3(fake, fake, 8, 48, fake, fake, fake, 0, None, None) == -2
    assert g3(fake, fake, 8, 64, fake, fake, fake, 2, None, None) == -4
    assert g3(fake, fake, 8, 64, fake, vp(0x1001), fake, 0, None, None) == -3
    q3 = lib.rcp_quant_w3a4_gemv
    q3.argtypes = [vp, vp, ci, ci, vp, ci, ctypes.c_float, vp, ci, vp, vp, vp, vp]
    assert q3(fake, fake, 8, 64, None, 0, 1.0, fake, 0, None, None, None, None) == -1
    assert q3(fake, fake, 8, 48, fake, 0, 1.0, fake, 0, None, None, None, None) == -2
    assert q3(fake, fake, 8, 64, fake, 5, 1.0, fake, 0, None, None, None, None) == -4
    assert q3(fake, fake, 8, 64, fake, 0, 0.0, fake, 0, None, None, None, None) == -4
    assert q3(fake, fake, 8, 64, fake, 0, 1.0, fake, 2, None, None, None, None) == -4
    assert q3(fake, fake, 8, 64, odd, 0, 1.0, fake, 0, None, None, None, None) == -3
    assert q3(fake, fake, 8, 64, fake, 0, 1.0, fake, 0, None, vp(0x1001), None, None) == -3
    u3 = lib.rcp_unpack_indices_w3
    u3.argtypes = [vp, ci, ci, vp, vp]
    assert u3(fake, 10, 64, fake, None) == -2
    # 4-bit KV cache
    ap = lib.rcp_kv4_append
    ap.argtypes = [vp, ci, ci, ci, ci, ci, ci, ctypes.c_float, vp, vp, vp]
    assert ap(None, 0, 1, 2, 8, 0, 0, 0.95, fake, fake, None) == -1
    assert ap(fake, 7, 1, 2, 8, 0, 0, 0.95, fake, fake, None) == -4
    assert ap(fake, 0, 3, 2, 8, 6, 0, 0.95, fake, fake, None) == -2          # runs past S_max
    assert ap(fake, 0, 1, 2, 8, -1, 0, 0.95, fake, fake, None) == -2
    assert ap(fake, 0, 1, 0, 8, 0, 0, 0.95, fake, fake, None) == -2
    assert ap(fake, 0, 1, 2, 8, 0, 0, 0.0, fake, fake, None) == -4
    assert ap(fake, 0, 1, 2, 8, 0, 0, 1.5, fake, fake, None) == -4
    assert ap(odd, 0, 1, 2, 8, 0, 1, 0.95, fake, fake, None) == -3
    akv = lib.rcp_kv4_append_kv
    akv.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, ctypes.c_float, vp, vp, vp, vp, vp]
    assert akv(fake, None, 0, 1, 2, 8, 0, 1, 0.95, fake, fake, fake, fake, None) == -1
    assert akv(fake, fake, 0, 3, 2, 8, 6, 1, 0.95, fake, fake, fake, fake, None) == -2     # runs past S_max
    assert akv(fake, fake, 5, 1, 2, 8, 0, 1, 0.95, fake, fake, fake, fake, None) == -4
    assert akv(fake, odd, 0, 1, 2, 8, 0, 1, 0.95, fake, fake, fake, fake, None) == -3
    adf = lib.rcp_kv4_rotate_attn_decode
    adf.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, ctypes.c_float, vp, ci, vp, ctypes.c_size_t, vp]
    assert adf(None, 0, 4, 4, 8, 8, fake, fake, fake, fake, 0.1, fake, 1, fake, 1 << 20, None) == -1
    assert adf(fake, 0, 4, 3, 8, 8, fake, fake, fake, fake, 0.1, fake, 1, fake, 1 << 20, None) == -2   # H_q % H_kv
    assert adf(fake, 0, 4, 4, 8, 9, fake, fake, fake, fake, 0.1, fake, 1, fake, 1 << 20, None) == -2   # S > S_max
    assert adf(fake, 0, 4, 4, 8, 8, fake, fake, fake, fake, 0.1, fake, 1, fake, 16, None) == -5        # workspace
    assert adf(odd, 0, 4, 4, 8, 8, fake, fake, fake, fake, 0.1, fake, 1, fake, 1 << 20, None) == -3
    kws = lib.rcp_kv4_workspace_bytes
    kws.restype = ctypes.c_size_t
    kws.argtypes = [ci, ci]
    assert kws(0, 10) == 0 and kws(4, 0) == 0 and kws(4, 262145) == 0
    assert kws(32, 1) == 32 * 132 * 4 and kws(32, 65) == 2 * 32 * 132 * 4
    assert kws(32, 4096) == 32 * 64 * 132 * 4                          # sized for 64 tokens per workgroup
    assert kws(1, 262144) == 4096 * 132 * 4
    at = lib.rcp_kv4_attn_decode
    at.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, ctypes.c_float, vp, ci, vp, ctypes.c_size_t, vp]
    big = 1 << 30
    assert at(fake, 0, 4, 4, 8, 8, fake, fake, fake, None, 0.1, fake, 1, fake, big, None) == -1
    assert at(fake, 0, 4, 3, 8, 8, fake, fake, fake, fake, 0.1, fake, 1, fake, big, None) == -2
    assert at(fake, 0, 4, 4, 8, 9, fake, fake, fake, fake, 0.1, fake, 1, fake, big, None) == -2
    assert at(fake, 0, 4, 4, 8, 0, fake, fake, fake, fake, 0.1, fake, 1, fake, big, None) == -2
    assert at(fake, 0, 4, 4, 8, 8, fake, fake, fake, fake, 0.1, fake, 2, fake, big, None) == -4      # bf16 output
    assert at(fake, 9, 4, 4, 8, 8, fake, fake, fake, fake, 0.1, fake, 1, fake, big, None) == -4
    assert at(fake, 0, 4, 4, 1 << 19, 1 << 19, fake, fake, fake, fake, 0.1, fake, 1, fake, big, None) == -4
    assert at(fake, 0, 4, 4, 8, 8, fake, odd, fake, fake, 0.1, fake, 1, fake, big, None) == -3
    assert at(fake, 0, 4, 4, 8, 8, fake, fake, fake, fake, 0.1, fake, 1, None, 0, None) == -5
    assert at(fake, 0, 4, 4, 8, 8, fake, fake, fake, fake, 0.1, fake, 1, fake, 4 * 132 * 4 - 1, None) == -5
    assert b"workspace" in lib.rcp_last_error()
    ip = ctypes.POINTER(ctypes.c_int)
    i3 = ctypes.c_int * 3
    apb = lib.rcp_kv4_append_batched
    apb.argtypes = [vp, ci, ci, ci, ci, ip, ci, ctypes.c_float, vp, vp, vp]
    assert apb(fake, 0, 3, 2, 8, None, 0, 0.95, fake, fake, None) == -1
    assert apb(fake, 0, 17, 2, 8, i3(0, 1, 2), 0, 0.95, fake, fake, None) == -2
    assert apb(fake, 0, 3, 2, 8, i3(0, 8, 2), 0, 0.95, fake, fake, None) == -2       # position past the end
    assert apb(fake, 0, 3, 2, 8, i3(0, -1, 2), 0, 0.95, fake, fake, None) == -2
    assert apb(fake, 0, 3, 2, 8, i3(0, 1, 2), 0, 2.0, fake, fake, None) == -4
    assert apb(fake, 0, 3, 2, 8, i3(0, 1, 2), 0, 0.95, odd, fake, None) == -3
    atb = lib.rcp_kv4_attn_decode_batched
    atb.argtypes = [vp, ci, ci, ci, ci, ci, ip, vp, vp, vp, vp, ctypes.c_float, vp, ci, vp, ctypes.c_size_t, vp]
    assert atb(fake, 0, 3, 4, 4, 8, None, fake, fake, fake, fake, 0.1, fake, 1, fake, big, None) == -1
    assert atb(fake, 0, 0, 4, 4, 8, i3(1, 2, 3), fake, fake, fake, fake, 0.1, fake, 1, fake, big, None) == -2
    assert atb(fake, 0, 3, 4, 4, 8, i3(1, 9, 3), fake, fake, fake, fake, 0.1, fake, 1, fake, big, None) == -2
    assert atb(fake, 0, 3, 4, 4, 8, i3(1, 0, 3), fake, fake, fake, fake, 0.1, fake, 1, fake, big, None) == -2
    assert atb(fake, 0, 3, 4, 3, 8, i3(1, 2, 3), fake, fake, fake, fake, 0.1, fake, 1, fake, big, None) == -2
    assert atb(fake, 0, 3, 4, 4, 8, i3(1, 2, 3), fake, fake, fake, fake, 0.1, fake, 2, fake, big, None) == -4
    assert atb(fake, 0, 3, 4, 4, 8, i3(1, 2, 3), fake, fake, fake, fake, 0.1, fake, 1, fake, 3 * 4 * 132 * 4 - 1, None) == -5
    assert atb(fake, 0, 3, 4, 4, 8, i3(1, 2, 3), fake, fake, fake, odd, 0.1, fake, 1, fake, big, None) == -3
    ws = lib.rcp_act_workspace_bytes
    ws.restype = ctypes.c_size_t
    ws.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(Rot)]
    assert ws(1, 4096, None) == 0
    assert ws(2, 11008, ctypes.byref(Rot(2, 64, 172, fake))) == 2 * 11008 * 4


def test_product_path_has_no_cpu_fallback():
    """The binding must not import the oracle, and a missing library must raise."""
    src = open(os.path.join(ROOT, "paper_2502_15779_amd", "__init__.py")).read()
    assert "import oracle" not in src and "from oracle" not in src
    for name in os.listdir(os.path.join(ROOT, "paper_2502_15779_amd", "csrc")):
        assert "oracle" not in open(os.path.join(ROOT, "paper_2502_15779_amd", "csrc", name)).read().lower()
    import paper_2502_15779_amd as rcp
    saved, rcp._lib, rcp.LIB_PATH = rcp._lib, None, rcp.LIB_PATH + ".absent"
    try:
        with pytest.raises(rcp.RcpError):
            rcp.lib()
    finally:
        rcp.LIB_PATH = rcp.LIB_PATH[: -len(".absent")]
        rcp._lib = saved


def test_documented_kernel_crossover_with_nothing_forced(lib):
    """include/rcp.h: one token on the vector ALUs, two tokens too below 8192 rows; two tokens from 8192 rows on and
    three or more tokens on the matrix cores.  Read from the library's own choice, with every option automatic."""
    lib.rcp_set_option.argtypes = [ctypes.c_char_p, ctypes.c_int]
    assert lib.rcp_set_option(b"reset", 0) == 0
    v = lib.rcp_w2a4_gemv_variant
    v.argtypes = [ctypes.c_int] * 3
    header = re.sub(r"\s*\*\s*", " ", open(HEADER).read())
    assert "two tokens too when N < 8192" in header and "three or more tokens" in header
    for N in (256, 4096, 8188):
        assert v(N, 4096, 1) == 1 and v(N, 4096, 2) == 1 and v(N, 4096, 3) == 2 and v(N, 4096, 16) == 2
    for N in (8192, 12288, 22016):
        assert v(N, 4096, 1) == 1 and v(N, 4096, 2) == 2 and v(N, 4096, 3) == 2 and v(N, 4096, 16) == 2
    assert v(6, 4096, 1) == -2 and v(8, 4096, 17) == -2
    # a forced variant is reported, and "reset" takes it back
    assert lib.rcp_set_option(b"gemv_variant", 1) == 0 and v(22016, 4096, 16) == 1
    assert lib.rcp_set_option(b"reset", 0) == 0 and v(22016, 4096, 16) == 2


def test_static_scratch_entry_point_rejects_before_touching_the_device(lib):
    lib.rcp_last_error.restype = ctypes.c_char_p
    vp = ctypes.c_void_p
    fake = vp(0x1000)
    act = lib.rcp_rotate_quant_act_static
    act.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(Rot), ctypes.c_float, vp, vp, vp]
    assert act(None, 0, 1, 64, None, 1.0, fake, fake, None) == -1
    assert act(fake, 0, 17, 64, None, 1.0, fake, fake, None) == -2
    assert act(fake, 0, 1, 64, None, 0.0, fake, fake, None) == -4
    assert act(fake, 0, 1, 96, ctypes.byref(Rot(2, 32, 4, fake)), 1.0, fake, fake, None) == -2
    # 16 tokens x 32768 channels x 4 bytes = 2 MiB of Kronecker scratch: beyond the fixed 1 MiB array
    assert act(fake, 0, 16, 32768, ctypes.byref(Rot(2, 128, 256, fake)), 1.0, fake, fake, None) == -5
    assert b"exceed" in lib.rcp_last_error()


def test_sequence_entry_point_rejects_before_touching_the_device(lib):
    vp, ci = ctypes.c_void_p, ctypes.c_int

    class Step(ctypes.Structure):
        _fields_ = [("packed", vp), ("codebook", vp), ("N", ci), ("K", ci), ("x", vp), ("x_dtype", ci), ("rot", Rot),
                    ("clip_ratio", ctypes.c_float), ("out", vp), ("out_dtype", ci), ("xq_out", vp), ("scale_out", vp)]
    seq = lib.rcp_quant_w2a4_gemv_sequence
    seq.argtypes = [ctypes.POINTER(Step), ci, vp, ctypes.c_size_t, vp]
    need = lib.rcp_gemv_sequence_workspace_bytes
    need.argtypes = [ctypes.POINTER(Step), ci]
    need.restype = ctypes.c_size_t
    fake = 0x1000
    good = Step(fake, fake, 64, 128, fake, 0, Rot(0, 0, 1, None), 1.0, fake, 0, None, None)
    arr = (Step * 2)(good, good)
    assert need(arr, 2) > 0 and need(arr, 0) == 0 and need(arr, 17) == 0
    assert seq(None, 1, vp(fake), 1 << 20, None) == -1
    assert seq(arr, 0, vp(fake), 1 << 20, None) == -2
    assert seq(arr, 2, None, 1 << 20, None) == -1
    assert seq(arr, 2, vp(fake), 16, None) == -5
    assert seq(arr, 2, vp(fake + 16), 1 << 20, None) == -3          # workspace not 256-byte aligned
    bad = (Step * 1)(Step(fake, fake, 64, 32768, fake, 0, Rot(0, 0, 1, None), 1.0, fake, 0, None, None))
    assert seq(bad, 1, vp(fake), 1 << 20, None) == -4               # K beyond the in-kernel quantiser
    bad = (Step * 1)(Step(fake, fake, 64, 128, fake, 0, Rot(1, 128, 1, None), 1.0, fake, 0, None, None))
    assert seq(bad, 1, vp(fake), 1 << 20, None) == -4               # pure Hadamard rotation
    bad = (Step * 1)(Step(fake, fake, 64, 128, fake, 0, Rot(0, 0, 1, None), 1.0, fake, 2, None, None))
    assert seq(bad, 1, vp(fake), 1 << 20, None) == -4               # bf16 output
    bad = (Step * 1)(Step(fake, fake, 62, 128, fake, 0, Rot(0, 0, 1, None), 1.0, fake, 0, None, None))
    assert seq(bad, 1, vp(fake), 1 << 20, None) == -2
