// C ABI of librcp.so: argument validation, error strings, dispatch to the launchers.
// Every rule checked here is stated in include/rcp.h.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "rcp_internal.hpp"

namespace rcp {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int check_launch(const char* what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(RCP_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return RCP_OK;
}

Options& options()
{
    static Options o = {};
    return o;
}

int num_compute_units()
{
    static thread_local int cached_dev = -1, cached_cus = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (dev != cached_dev) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        cached_dev = dev;
        cached_cus = cus;
    }
    return cached_cus;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static bool pow2(int n) { return n > 0 && (n & (n - 1)) == 0; }

static int check_shape(const char* fn, int N, int K)
{
    if (N <= 0 || N % 4 != 0) return fail(RCP_ERR_SHAPE, "%s: N=%d must be a positive multiple of 4", fn, N);
    if (K <= 0 || K % 32 != 0) return fail(RCP_ERR_SHAPE, "%s: K=%d must be a positive multiple of 32", fn, K);
    if (K > RCP_MAX_K) return fail(RCP_ERR_SHAPE, "%s: K=%d exceeds RCP_MAX_K=%d", fn, K, RCP_MAX_K);
    if (static_cast<long long>(N) * K / 4 > 0x7fffffffLL * 4)
        return fail(RCP_ERR_SHAPE, "%s: N*K too large", fn);
    return RCP_OK;
}

static int check_rotation(const char* fn, int K, const rcp_rotation* rot)
{
    if (rot == nullptr || rot->kind == RCP_ROT_NONE) return RCP_OK;
    if (rot->kind == RCP_ROT_WHT) {
        if (!pow2(rot->n_wht) || rot->n_wht != K)
            return fail(RCP_ERR_SHAPE, "%s: WHT needs n_wht == K == power of two (n_wht=%d, K=%d)", fn, rot->n_wht, K);
        if (K > RCP_MAX_WHT) return fail(RCP_ERR_UNSUPPORTED, "%s: WHT order %d exceeds RCP_MAX_WHT=%d", fn, K, RCP_MAX_WHT);
        return RCP_OK;
    }
    if (rot->kind == RCP_ROT_KRON) {
        if (!pow2(rot->n_wht) || rot->m < 1 || static_cast<long long>(rot->n_wht) * rot->m != K)
            return fail(RCP_ERR_SHAPE, "%s: KRON needs n_wht (power of two) * m == K (n_wht=%d, m=%d, K=%d)", fn,
                        rot->n_wht, rot->m, K);
        if (rot->m > RCP_MAX_KRON_M) return fail(RCP_ERR_UNSUPPORTED, "%s: m=%d exceeds RCP_MAX_KRON_M=%d", fn, rot->m, RCP_MAX_KRON_M);
        if (rot->n_wht > 1024) return fail(RCP_ERR_UNSUPPORTED, "%s: KRON Hadamard factor %d exceeds 1024", fn, rot->n_wht);
        if (rot->Q == nullptr) return fail(RCP_ERR_NULL, "%s: KRON rotation with Q == NULL", fn);
        if (!aligned16(rot->Q)) return fail(RCP_ERR_ALIGN, "%s: Q is not 16-byte aligned", fn);
        return RCP_OK;
    }
    if (rot->kind == RCP_ROT_HEADS) {
        if (!pow2(rot->n_wht) || rot->m < 1 || static_cast<long long>(rot->n_wht) * rot->m != K)
            return fail(RCP_ERR_SHAPE, "%s: HEADS needs n_wht (power of two) * m == K (n_wht=%d, m=%d, K=%d)", fn,
                        rot->n_wht, rot->m, K);
        if (rot->n_wht < 2 || rot->n_wht > 64) return fail(RCP_ERR_UNSUPPORTED, "%s: HEADS with %d heads (2 .. 64 supported)", fn, rot->n_wht);
        if (rot->m % 8 != 0) return fail(RCP_ERR_SHAPE, "%s: HEADS needs a head size that is a multiple of 8 (m=%d)", fn, rot->m);
        if (K > RCP_MAX_WHT) return fail(RCP_ERR_UNSUPPORTED, "%s: HEADS rotation of K=%d exceeds %d", fn, K, RCP_MAX_WHT);
        return RCP_OK;
    }
    return fail(RCP_ERR_UNSUPPORTED, "%s: unknown rotation kind %d", fn, rot->kind);
}

static int check_group(const char* fn, int K, int group)
{
    if (group != RCP_GROUP) return fail(RCP_ERR_UNSUPPORTED, "%s: group=%d, this build supports %d only", fn, group, RCP_GROUP);
    if (K % RCP_GROUP != 0) return fail(RCP_ERR_SHAPE, "%s: K=%d must be a multiple of the group size %d", fn, K, RCP_GROUP);
    return RCP_OK;
}

}  // namespace rcp

using namespace rcp;

extern "C" {

int rcp_version(void) { return 100; }

const char* rcp_last_error(void) { return g_err; }

size_t rcp_packed_bytes(int N, int K)
{
    if (N <= 0 || N % 4 != 0 || K <= 0 || K % 32 != 0 || K > RCP_MAX_K) return 0;
    return static_cast<size_t>(N) * static_cast<size_t>(K) / 4;
}

size_t rcp_act_workspace_bytes(int M, int K, const rcp_rotation* rot)
{
    if (M <= 0 || K <= 0) return 0;
    return act_workspace_bytes(M, K, rot);
}

int rcp_set_option(const char* name, int value)
{
    if (name == nullptr) return fail(RCP_ERR_NULL, "rcp_set_option: name is NULL");
    Options& o = options();
    if (strcmp(name, "reset") == 0) {
        o = Options{};
        return RCP_OK;
    }
    if (strcmp(name, "gemv_lanes") == 0) {
        if (value != 0 && value != 16 && value != 32 && value != 64 && value != 128 && value != 256)
            return fail(RCP_ERR_UNSUPPORTED, "rcp_set_option: gemv_lanes must be 0, 16, 32, 64, 128 or 256");
        o.gemv_lanes = value;
    } else if (strcmp(name, "gemv_unroll") == 0) {
        if (value != 0 && value != 2 && value != 4)
            return fail(RCP_ERR_UNSUPPORTED, "rcp_set_option: gemv_unroll must be 0, 2 or 4");
        o.gemv_unroll = value;
    } else if (strcmp(name, "gemv_blocks") == 0) {
        if (value < 0 || value > (1 << 20)) return fail(RCP_ERR_UNSUPPORTED, "rcp_set_option: gemv_blocks out of range");
        o.gemv_blocks = value;
    } else if (strcmp(name, "gemv_variant") == 0) {
        if (value < 0 || value > 2) return fail(RCP_ERR_UNSUPPORTED, "rcp_set_option: gemv_variant must be 0, 1 or 2");
        o.gemv_variant = value;
    } else if (strcmp(name, "gemm_waves") == 0) {
        if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8)
            return fail(RCP_ERR_UNSUPPORTED, "rcp_set_option: gemm_waves must be 0, 1, 2, 4 or 8");
        o.gemm_waves = value;
    } else if (strcmp(name, "gemv_nt") == 0) {
        if (value < 0 || value > 2) return fail(RCP_ERR_UNSUPPORTED, "rcp_set_option: gemv_nt must be 0, 1 or 2");
        o.gemv_nt = value;
    } else if (strcmp(name, "gemm_stage") == 0) {
        if (value < 0 || value > 2) return fail(RCP_ERR_UNSUPPORTED, "rcp_set_option: gemm_stage must be 0, 1 or 2");
        o.gemm_stage = value;
    } else if (strcmp(name, "gemm_rows") == 0) {
        if (value != 0 && (value < 16 || value > 64 || value % 4 != 0))
            return fail(RCP_ERR_UNSUPPORTED, "rcp_set_option: gemm_rows must be 0 or a multiple of 4 from 16 to 64");
        o.gemm_rows = value;
    } else if (strcmp(name, "kv_tokens") == 0) {
        if (value != 0 && value != 64 && value != 128 && value != 256 && value != 512 && value != 1024 && value != 2048)
            return fail(RCP_ERR_UNSUPPORTED, "rcp_set_option: kv_tokens must be 0, 64, 128, 256, 512, 1024 or 2048");
        o.kv_tokens = value;
    } else if (strcmp(name, "gemv_waves") == 0) {
        if (value != 0 && value != 4 && value != 8)
            return fail(RCP_ERR_UNSUPPORTED, "rcp_set_option: gemv_waves must be 0, 4 or 8");
        o.gemv_waves = value;
    } else if (strcmp(name, "gemv_oneshot") == 0) {
        if (value < 0 || value > 2) return fail(RCP_ERR_UNSUPPORTED, "rcp_set_option: gemv_oneshot must be 0, 1 or 2");
        o.gemv_oneshot = value;
    } else if (strcmp(name, "seq_blocks") == 0) {
        if (value < 0 || value > 4096) return fail(RCP_ERR_UNSUPPORTED, "rcp_set_option: seq_blocks out of range");
        o.seq_blocks = value;
    } else
        return fail(RCP_ERR_UNSUPPORTED, "rcp_set_option: unknown option '%s'", name);
    return RCP_OK;
}

int rcp_pack_weights(const void* W, rcp_dtype w_dtype, int N, int K, const float* clip_lo,
                     const float* clip_hi, const float* part, void* packed_out, void* codebook_out,
                     void* stream)
{
    if (!W || !clip_lo || !clip_hi || !part || !packed_out || !codebook_out)
        return fail(RCP_ERR_NULL, "rcp_pack_weights: NULL pointer argument");
    if (int rc = check_shape("rcp_pack_weights", N, K)) return rc;
    if (w_dtype != RCP_F16 && w_dtype != RCP_F32 && w_dtype != RCP_BF16)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_pack_weights: unknown dtype %d", static_cast<int>(w_dtype));
    if (!aligned16(W) || !aligned16(packed_out) || !aligned16(codebook_out) || !aligned16(clip_lo) ||
        !aligned16(clip_hi) || !aligned16(part))
        return fail(RCP_ERR_ALIGN, "rcp_pack_weights: device buffers must be 16-byte aligned");
    return launch_pack(W, w_dtype, N, K, clip_lo, clip_hi, part, packed_out, codebook_out,
                       static_cast<hipStream_t>(stream));
}

int rcp_unpack_indices(const void* packed, int N, int K, uint8_t* idx_out, void* stream)
{
    if (!packed || !idx_out) return fail(RCP_ERR_NULL, "rcp_unpack_indices: NULL pointer argument");
    if (int rc = check_shape("rcp_unpack_indices", N, K)) return rc;
    if (!aligned16(packed) || !aligned16(idx_out))
        return fail(RCP_ERR_ALIGN, "rcp_unpack_indices: device buffers must be 16-byte aligned");
    return launch_unpack(packed, N, K, idx_out, static_cast<hipStream_t>(stream));
}

int rcp_rotate_quant_act(const void* x, rcp_dtype x_dtype, int M, int K, const rcp_rotation* rot,
                         float clip_ratio, void* xq_out, void* scale_out, void* workspace,
                         size_t workspace_bytes, void* stream)
{
    if (!x || !xq_out || !scale_out) return fail(RCP_ERR_NULL, "rcp_rotate_quant_act: NULL pointer argument");
    if (M <= 0 || M > RCP_MAX_M) return fail(RCP_ERR_SHAPE, "rcp_rotate_quant_act: M=%d outside 1..%d", M, RCP_MAX_M);
    if (K <= 0 || K % 32 != 0 || K > RCP_MAX_K)
        return fail(RCP_ERR_SHAPE, "rcp_rotate_quant_act: K=%d must be a positive multiple of 32, at most %d", K, RCP_MAX_K);
    if (x_dtype != RCP_F16 && x_dtype != RCP_F32 && x_dtype != RCP_BF16)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_rotate_quant_act: unknown dtype %d", static_cast<int>(x_dtype));
    if (!(clip_ratio > 0.0f) || !(clip_ratio <= 1.0f))
        return fail(RCP_ERR_UNSUPPORTED, "rcp_rotate_quant_act: clip_ratio %g outside (0, 1]", static_cast<double>(clip_ratio));
    if (int rc = check_rotation("rcp_rotate_quant_act", K, rot)) return rc;
    if (!aligned16(x) || !aligned16(xq_out) || !aligned16(workspace))
        return fail(RCP_ERR_ALIGN, "rcp_rotate_quant_act: device buffers must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(scale_out) & 1u) != 0)
        return fail(RCP_ERR_ALIGN, "rcp_rotate_quant_act: scale_out must be 2-byte aligned");
    size_t need = act_workspace_bytes(M, K, rot);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need))
        return fail(RCP_ERR_WORKSPACE, "rcp_rotate_quant_act: workspace of %zu bytes needed, %zu given", need,
                    workspace ? workspace_bytes : static_cast<size_t>(0));
    return launch_act(x, x_dtype, M, K, rot, clip_ratio, xq_out, scale_out, workspace, workspace_bytes,
                      static_cast<hipStream_t>(stream));
}

int rcp_rotate_quant_act_static(const void* x, rcp_dtype x_dtype, int M, int K, const rcp_rotation* rot,
                                float clip_ratio, void* xq_out, void* scale_out, void* stream)
{
    if (!x || !xq_out || !scale_out) return fail(RCP_ERR_NULL, "rcp_rotate_quant_act_static: NULL pointer argument");
    if (M <= 0 || M > RCP_MAX_M) return fail(RCP_ERR_SHAPE, "rcp_rotate_quant_act_static: M=%d outside 1..%d", M, RCP_MAX_M);
    if (K <= 0 || K % 32 != 0 || K > RCP_MAX_K)
        return fail(RCP_ERR_SHAPE, "rcp_rotate_quant_act_static: K=%d must be a positive multiple of 32, at most %d", K, RCP_MAX_K);
    if (x_dtype != RCP_F16 && x_dtype != RCP_F32 && x_dtype != RCP_BF16)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_rotate_quant_act_static: unknown dtype %d", static_cast<int>(x_dtype));
    if (!(clip_ratio > 0.0f) || !(clip_ratio <= 1.0f))
        return fail(RCP_ERR_UNSUPPORTED, "rcp_rotate_quant_act_static: clip_ratio %g outside (0, 1]", static_cast<double>(clip_ratio));
    if (int rc = check_rotation("rcp_rotate_quant_act_static", K, rot)) return rc;
    if (!aligned16(x) || !aligned16(xq_out))
        return fail(RCP_ERR_ALIGN, "rcp_rotate_quant_act_static: device buffers must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(scale_out) & 1u) != 0)
        return fail(RCP_ERR_ALIGN, "rcp_rotate_quant_act_static: scale_out must be 2-byte aligned");
    return launch_act_static(x, x_dtype, M, K, rot, clip_ratio, xq_out, scale_out, static_cast<hipStream_t>(stream));
}

int rcp_stream_read(const void* buffer, size_t bytes, void* sink_or_null, void* stream)
{
    if (!buffer) return fail(RCP_ERR_NULL, "rcp_stream_read: NULL pointer argument");
    if (!aligned16(buffer) || (reinterpret_cast<uintptr_t>(sink_or_null) & 3u) != 0)
        return fail(RCP_ERR_ALIGN, "rcp_stream_read: buffer must be 16-byte and sink 4-byte aligned");
    return launch_stream_read(buffer, bytes, static_cast<uint32_t*>(sink_or_null), static_cast<hipStream_t>(stream));
}

int rcp_rotate_act(const void* x, rcp_dtype x_dtype, int M, int K, const rcp_rotation* rot, float* y_out, void* stream)
{
    if (!x || !y_out) return fail(RCP_ERR_NULL, "rcp_rotate_act: NULL pointer argument");
    if (M <= 0 || M > RCP_MAX_ROTATE_ROWS)
        return fail(RCP_ERR_SHAPE, "rcp_rotate_act: M=%d outside 1..%d", M, RCP_MAX_ROTATE_ROWS);
    if (K <= 0 || K % 32 != 0 || K > RCP_MAX_K)
        return fail(RCP_ERR_SHAPE, "rcp_rotate_act: K=%d must be a positive multiple of 32, at most %d", K, RCP_MAX_K);
    if (x_dtype != RCP_F16 && x_dtype != RCP_F32 && x_dtype != RCP_BF16)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_rotate_act: unknown dtype %d", static_cast<int>(x_dtype));
    if (int rc = check_rotation("rcp_rotate_act", K, rot)) return rc;
    if (!aligned16(x) || !aligned16(y_out)) return fail(RCP_ERR_ALIGN, "rcp_rotate_act: device buffers must be 16-byte aligned");
    return launch_rotate(x, x_dtype, M, K, rot, y_out, static_cast<hipStream_t>(stream));
}

int rcp_w2a4_gemv(const void* packed, const void* codebook, int N, int K, const void* xq,
                  const void* scale, int M, void* out, rcp_dtype out_dtype,
                  int32_t* partial_sums_or_null, void* stream)
{
    if (!packed || !codebook || !xq || !scale || !out)
        return fail(RCP_ERR_NULL, "rcp_w2a4_gemv: NULL pointer argument");
    if (int rc = check_shape("rcp_w2a4_gemv", N, K)) return rc;
    if (M <= 0 || M > RCP_MAX_M) return fail(RCP_ERR_SHAPE, "rcp_w2a4_gemv: M=%d outside 1..%d", M, RCP_MAX_M);
    if (out_dtype != RCP_F16 && out_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_w2a4_gemv: out_dtype must be RCP_F16 or RCP_F32");
    if (!aligned16(packed) || !aligned16(codebook) || !aligned16(xq) || !aligned16(out) ||
        !aligned16(partial_sums_or_null))
        return fail(RCP_ERR_ALIGN, "rcp_w2a4_gemv: device buffers must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(scale) & 1u) != 0)
        return fail(RCP_ERR_ALIGN, "rcp_w2a4_gemv: scale must be 2-byte aligned");
    return launch_gemv(packed, codebook, N, K, xq, scale, M, out, out_dtype, partial_sums_or_null,
                       static_cast<hipStream_t>(stream));
}

int rcp_w2a4_gemv_variant(int N, int K, int M)
{
    if (int rc = check_shape("rcp_w2a4_gemv_variant", N, K)) return rc;
    if (M <= 0 || M > RCP_MAX_M) return fail(RCP_ERR_SHAPE, "rcp_w2a4_gemv_variant: M=%d outside 1..%d", M, RCP_MAX_M);
    return gemv_variant(N, K, M);
}

int rcp_quant_w2a4_gemv(const void* packed, const void* codebook, int N, int K, const void* x,
                        rcp_dtype x_dtype, float clip_ratio, void* out, rcp_dtype out_dtype,
                        void* xq_out_or_null, void* scale_out_or_null, int32_t* partial_sums_or_null,
                        void* stream)
{
    if (!packed || !codebook || !x || !out) return fail(RCP_ERR_NULL, "rcp_quant_w2a4_gemv: NULL pointer argument");
    if (int rc = check_shape("rcp_quant_w2a4_gemv", N, K)) return rc;
    if (x_dtype != RCP_F16 && x_dtype != RCP_F32 && x_dtype != RCP_BF16)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_quant_w2a4_gemv: unknown dtype %d", static_cast<int>(x_dtype));
    if (out_dtype != RCP_F16 && out_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_quant_w2a4_gemv: out_dtype must be RCP_F16 or RCP_F32");
    if (!(clip_ratio > 0.0f) || !(clip_ratio <= 1.0f))
        return fail(RCP_ERR_UNSUPPORTED, "rcp_quant_w2a4_gemv: clip_ratio %g outside (0, 1]", static_cast<double>(clip_ratio));
    if (!aligned16(packed) || !aligned16(codebook) || !aligned16(x) || !aligned16(out) || !aligned16(xq_out_or_null) ||
        !aligned16(partial_sums_or_null))
        return fail(RCP_ERR_ALIGN, "rcp_quant_w2a4_gemv: device buffers must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(scale_out_or_null) & 1u) != 0)
        return fail(RCP_ERR_ALIGN, "rcp_quant_w2a4_gemv: scale_out must be 2-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (quant_gemv_supported(K))
        return launch_quant_gemv(packed, codebook, N, K, x, x_dtype, clip_ratio, out, out_dtype, xq_out_or_null,
                                 scale_out_or_null, partial_sums_or_null, 0, 0, st);
    // K too large for the in-kernel quantiser: two launches through the caller's x_q / S buffers
    if (!xq_out_or_null || !scale_out_or_null)
        return fail(RCP_ERR_WORKSPACE, "rcp_quant_w2a4_gemv: K=%d needs xq_out and scale_out as scratch", K);
    if (int rc = launch_act(x, x_dtype, 1, K, nullptr, clip_ratio, xq_out_or_null, scale_out_or_null, nullptr, 0, st)) return rc;
    return launch_gemv(packed, codebook, N, K, xq_out_or_null, scale_out_or_null, 1, out, out_dtype, partial_sums_or_null, st);
}

int rcp_rotate_quant_w2a4_gemv(const void* packed, const void* codebook, int N, int K, const void* x,
                               rcp_dtype x_dtype, const rcp_rotation* rot, float clip_ratio, void* out,
                               rcp_dtype out_dtype, void* xq_out_or_null, void* scale_out_or_null,
                               int32_t* partial_sums_or_null, void* stream)
{
    if (rot == nullptr || rot->kind == RCP_ROT_NONE)
        return rcp_quant_w2a4_gemv(packed, codebook, N, K, x, x_dtype, clip_ratio, out, out_dtype, xq_out_or_null,
                                   scale_out_or_null, partial_sums_or_null, stream);
    if (!packed || !codebook || !x || !out) return fail(RCP_ERR_NULL, "rcp_rotate_quant_w2a4_gemv: NULL pointer argument");
    if (int rc = check_shape("rcp_rotate_quant_w2a4_gemv", N, K)) return rc;
    const bool short_wht = rot->kind == RCP_ROT_WHT && wht_gemv_supported(K);
    if (rot->kind != RCP_ROT_HEADS && !short_wht)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_rotate_quant_w2a4_gemv: only RCP_ROT_NONE, RCP_ROT_HEADS and RCP_ROT_WHT with "
                                         "K <= 2048 run inside the GEMV; use rcp_rotate_act + rcp_quant_w2a4_gemv for kind %d", rot->kind);
    if (int rc = check_rotation("rcp_rotate_quant_w2a4_gemv", K, rot)) return rc;
    if (x_dtype != RCP_F16 && x_dtype != RCP_F32 && x_dtype != RCP_BF16)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_rotate_quant_w2a4_gemv: unknown dtype %d", static_cast<int>(x_dtype));
    if (out_dtype != RCP_F16 && out_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_rotate_quant_w2a4_gemv: out_dtype must be RCP_F16 or RCP_F32");
    if (!(clip_ratio > 0.0f) || !(clip_ratio <= 1.0f))
        return fail(RCP_ERR_UNSUPPORTED, "rcp_rotate_quant_w2a4_gemv: clip_ratio %g outside (0, 1]", static_cast<double>(clip_ratio));
    if (!aligned16(packed) || !aligned16(codebook) || !aligned16(x) || !aligned16(out) || !aligned16(xq_out_or_null) ||
        !aligned16(partial_sums_or_null))
        return fail(RCP_ERR_ALIGN, "rcp_rotate_quant_w2a4_gemv: device buffers must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(scale_out_or_null) & 1u) != 0)
        return fail(RCP_ERR_ALIGN, "rcp_rotate_quant_w2a4_gemv: scale_out must be 2-byte aligned");
    if (short_wht)
        return launch_wht_quant_gemv(packed, codebook, N, K, x, x_dtype, clip_ratio, out, out_dtype, xq_out_or_null,
                                     scale_out_or_null, partial_sums_or_null, static_cast<hipStream_t>(stream));
    return launch_quant_gemv(packed, codebook, N, K, x, x_dtype, clip_ratio, out, out_dtype, xq_out_or_null,
                             scale_out_or_null, partial_sums_or_null, rot->n_wht, rot->m, static_cast<hipStream_t>(stream));
}

static int check_sequence(const char* fn, const rcp_gemv_step* steps, int n)
{
    if (!steps) return fail(RCP_ERR_NULL, "%s: steps is NULL", fn);
    if (n < 1 || n > RCP_SEQ_MAX_STEPS) return fail(RCP_ERR_SHAPE, "%s: n=%d outside 1..%d", fn, n, RCP_SEQ_MAX_STEPS);
    for (int i = 0; i < n; ++i) {
        const rcp_gemv_step& s = steps[i];
        if (!s.packed || !s.codebook || !s.x || !s.out) return fail(RCP_ERR_NULL, "%s: entry %d: NULL pointer", fn, i);
        if (int rc = check_shape(fn, s.N, s.K)) return rc;
        if (s.K > 16384) return fail(RCP_ERR_UNSUPPORTED, "%s: entry %d: K=%d exceeds 16384", fn, i, s.K);
        if (s.x_dtype != RCP_F16 && s.x_dtype != RCP_F32 && s.x_dtype != RCP_BF16)
            return fail(RCP_ERR_UNSUPPORTED, "%s: entry %d: unknown x_dtype %d", fn, i, s.x_dtype);
        if (s.out_dtype != RCP_F16 && s.out_dtype != RCP_F32)
            return fail(RCP_ERR_UNSUPPORTED, "%s: entry %d: out_dtype must be RCP_F16 or RCP_F32", fn, i);
        if (!(s.clip_ratio > 0.0f) || !(s.clip_ratio <= 1.0f))
            return fail(RCP_ERR_UNSUPPORTED, "%s: entry %d: clip_ratio %g outside (0, 1]", fn, i, static_cast<double>(s.clip_ratio));
        if (s.rot.kind != RCP_ROT_NONE && s.rot.kind != RCP_ROT_KRON)
            return fail(RCP_ERR_UNSUPPORTED, "%s: entry %d: only RCP_ROT_NONE and RCP_ROT_KRON run inside a sequence", fn, i);
        if (int rc = check_rotation(fn, s.K, &s.rot)) return rc;
        if (!aligned16(s.packed) || !aligned16(s.codebook) || !aligned16(s.x) || !aligned16(s.out) || !aligned16(s.xq_out_or_null))
            return fail(RCP_ERR_ALIGN, "%s: entry %d: device buffers must be 16-byte aligned", fn, i);
        if ((reinterpret_cast<uintptr_t>(s.scale_out_or_null) & 1u) != 0)
            return fail(RCP_ERR_ALIGN, "%s: entry %d: scale_out must be 2-byte aligned", fn, i);
    }
    return RCP_OK;
}

size_t rcp_gemv_sequence_workspace_bytes(const rcp_gemv_step* steps, int n)
{
    if (check_sequence("rcp_gemv_sequence_workspace_bytes", steps, n) != RCP_OK) return 0;
    return gemv_sequence_workspace_bytes(steps, n);
}

int rcp_quant_w2a4_gemv_sequence(const rcp_gemv_step* steps, int n, void* workspace, size_t workspace_bytes, void* stream)
{
    if (int rc = check_sequence("rcp_quant_w2a4_gemv_sequence", steps, n)) return rc;
    if (!workspace) return fail(RCP_ERR_NULL, "rcp_quant_w2a4_gemv_sequence: workspace is NULL");
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
        return fail(RCP_ERR_ALIGN, "rcp_quant_w2a4_gemv_sequence: workspace must be 256-byte aligned");
    const size_t need = gemv_sequence_workspace_bytes(steps, n);
    if (workspace_bytes < need)
        return fail(RCP_ERR_WORKSPACE, "rcp_quant_w2a4_gemv_sequence: workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    return launch_gemv_sequence(steps, n, workspace, static_cast<hipStream_t>(stream));
}

int rcp_w2a16_gemv(const void* packed, const void* codebook, int N, int K, const void* x, rcp_dtype x_dtype,
                   void* out, rcp_dtype out_dtype, void* stream)
{
    if (!packed || !codebook || !x || !out) return fail(RCP_ERR_NULL, "rcp_w2a16_gemv: NULL pointer argument");
    if (int rc = check_shape("rcp_w2a16_gemv", N, K)) return rc;
    if (x_dtype != RCP_F16 && x_dtype != RCP_F32 && x_dtype != RCP_BF16)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_w2a16_gemv: unknown dtype %d", static_cast<int>(x_dtype));
    if (out_dtype != RCP_F16 && out_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_w2a16_gemv: out_dtype must be RCP_F16 or RCP_F32");
    if (!aligned16(packed) || !aligned16(codebook) || !aligned16(x) || !aligned16(out))
        return fail(RCP_ERR_ALIGN, "rcp_w2a16_gemv: device buffers must be 16-byte aligned");
    return launch_w2a16_gemv(packed, codebook, N, K, x, x_dtype, out, out_dtype, static_cast<hipStream_t>(stream));
}

int rcp_pack_weights_grouped(const void* W, rcp_dtype w_dtype, int N, int K, int group, const float* clip_lo,
                             const float* clip_hi, const float* part, void* packed_out, void* codebook_out,
                             void* stream)
{
    if (!W || !clip_lo || !clip_hi || !part || !packed_out || !codebook_out)
        return fail(RCP_ERR_NULL, "rcp_pack_weights_grouped: NULL pointer argument");
    if (int rc = check_shape("rcp_pack_weights_grouped", N, K)) return rc;
    if (int rc = check_group("rcp_pack_weights_grouped", K, group)) return rc;
    if (w_dtype != RCP_F16 && w_dtype != RCP_F32 && w_dtype != RCP_BF16)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_pack_weights_grouped: unknown dtype %d", static_cast<int>(w_dtype));
    if (!aligned16(W) || !aligned16(packed_out) || !aligned16(codebook_out) || !aligned16(clip_lo) ||
        !aligned16(clip_hi) || !aligned16(part))
        return fail(RCP_ERR_ALIGN, "rcp_pack_weights_grouped: device buffers must be 16-byte aligned");
    return launch_pack_grouped(W, w_dtype, N, K, clip_lo, clip_hi, part, packed_out, codebook_out,
                               static_cast<hipStream_t>(stream));
}

int rcp_unpack_indices_grouped(const void* packed, int N, int K, int group, uint8_t* idx_out, void* stream)
{
    if (!packed || !idx_out) return fail(RCP_ERR_NULL, "rcp_unpack_indices_grouped: NULL pointer argument");
    if (int rc = check_shape("rcp_unpack_indices_grouped", N, K)) return rc;
    if (int rc = check_group("rcp_unpack_indices_grouped", K, group)) return rc;
    if (!aligned16(packed) || !aligned16(idx_out))
        return fail(RCP_ERR_ALIGN, "rcp_unpack_indices_grouped: device buffers must be 16-byte aligned");
    return launch_unpack_grouped(packed, N, K, idx_out, static_cast<hipStream_t>(stream));
}

int rcp_w2a4_gemv_grouped(const void* packed, const void* codebook, int N, int K, int group, const void* xq,
                          const void* scale, void* out, rcp_dtype out_dtype, int32_t* partial_sums_or_null,
                          void* stream)
{
    if (!packed || !codebook || !xq || !scale || !out)
        return fail(RCP_ERR_NULL, "rcp_w2a4_gemv_grouped: NULL pointer argument");
    if (int rc = check_shape("rcp_w2a4_gemv_grouped", N, K)) return rc;
    if (int rc = check_group("rcp_w2a4_gemv_grouped", K, group)) return rc;
    if (out_dtype != RCP_F16 && out_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_w2a4_gemv_grouped: out_dtype must be RCP_F16 or RCP_F32");
    if (!aligned16(packed) || !aligned16(codebook) || !aligned16(xq) || !aligned16(out) ||
        !aligned16(partial_sums_or_null))
        return fail(RCP_ERR_ALIGN, "rcp_w2a4_gemv_grouped: device buffers must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(scale) & 1u) != 0)
        return fail(RCP_ERR_ALIGN, "rcp_w2a4_gemv_grouped: scale must be 2-byte aligned");
    return launch_gemv_grouped(packed, codebook, N, K, xq, scale, out, out_dtype, partial_sums_or_null,
                               static_cast<hipStream_t>(stream));
}

int rcp_w2a4_gemm_grouped(const void* packed, const void* codebook, int N, int K, int group, const void* xq,
                          const void* scale, int M, void* out, rcp_dtype out_dtype, int32_t* partial_sums_or_null,
                          void* stream)
{
    if (!packed || !codebook || !xq || !scale || !out)
        return fail(RCP_ERR_NULL, "rcp_w2a4_gemm_grouped: NULL pointer argument");
    if (int rc = check_shape("rcp_w2a4_gemm_grouped", N, K)) return rc;
    if (int rc = check_group("rcp_w2a4_gemm_grouped", K, group)) return rc;
    if (M <= 0 || M > RCP_MAX_M) return fail(RCP_ERR_SHAPE, "rcp_w2a4_gemm_grouped: M=%d outside 1..%d", M, RCP_MAX_M);
    if (out_dtype != RCP_F16 && out_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_w2a4_gemm_grouped: out_dtype must be RCP_F16 or RCP_F32");
    if (!aligned16(packed) || !aligned16(codebook) || !aligned16(xq) || !aligned16(out) ||
        !aligned16(partial_sums_or_null))
        return fail(RCP_ERR_ALIGN, "rcp_w2a4_gemm_grouped: device buffers must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(scale) & 1u) != 0)
        return fail(RCP_ERR_ALIGN, "rcp_w2a4_gemm_grouped: scale must be 2-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (M == 1 && options().gemv_variant != 2)
        return launch_gemv_grouped(packed, codebook, N, K, xq, scale, out, out_dtype, partial_sums_or_null, st);
    return launch_gemm_mfma_grouped(packed, codebook, N, K, xq, scale, M, out, out_dtype, partial_sums_or_null, st);
}

int rcp_quant_w2a4_gemv_grouped(const void* packed, const void* codebook, int N, int K, int group, const void* x,
                                rcp_dtype x_dtype, float clip_ratio, void* out, rcp_dtype out_dtype,
                                void* xq_out_or_null, void* scale_out_or_null, int32_t* partial_sums_or_null,
                                void* stream)
{
    if (!packed || !codebook || !x || !out)
        return fail(RCP_ERR_NULL, "rcp_quant_w2a4_gemv_grouped: NULL pointer argument");
    if (int rc = check_shape("rcp_quant_w2a4_gemv_grouped", N, K)) return rc;
    if (int rc = check_group("rcp_quant_w2a4_gemv_grouped", K, group)) return rc;
    if (x_dtype != RCP_F16 && x_dtype != RCP_F32 && x_dtype != RCP_BF16)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_quant_w2a4_gemv_grouped: unknown dtype %d", static_cast<int>(x_dtype));
    if (out_dtype != RCP_F16 && out_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_quant_w2a4_gemv_grouped: out_dtype must be RCP_F16 or RCP_F32");
    if (!(clip_ratio > 0.0f) || !(clip_ratio <= 1.0f))
        return fail(RCP_ERR_UNSUPPORTED, "rcp_quant_w2a4_gemv_grouped: clip_ratio %g outside (0, 1]", static_cast<double>(clip_ratio));
    if (!aligned16(packed) || !aligned16(codebook) || !aligned16(x) || !aligned16(out) || !aligned16(xq_out_or_null) ||
        !aligned16(partial_sums_or_null))
        return fail(RCP_ERR_ALIGN, "rcp_quant_w2a4_gemv_grouped: device buffers must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(scale_out_or_null) & 1u) != 0)
        return fail(RCP_ERR_ALIGN, "rcp_quant_w2a4_gemv_grouped: scale_out must be 2-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (quant_gemv_grouped_supported(K))
        return launch_quant_gemv_grouped(packed, codebook, N, K, x, x_dtype, clip_ratio, out, out_dtype, xq_out_or_null,
                                         scale_out_or_null, partial_sums_or_null, st);
    // K too large for the in-kernel quantiser: two launches through the caller's x_q / S buffers
    if (!xq_out_or_null || !scale_out_or_null)
        return fail(RCP_ERR_WORKSPACE, "rcp_quant_w2a4_gemv_grouped: K=%d needs xq_out and scale_out as scratch", K);
    if (int rc = launch_act(x, x_dtype, 1, K, nullptr, clip_ratio, xq_out_or_null, scale_out_or_null, nullptr, 0, st)) return rc;
    return launch_gemv_grouped(packed, codebook, N, K, xq_out_or_null, scale_out_or_null, out, out_dtype, partial_sums_or_null, st);
}

int rcp_pack_weights_w3(const void* W, rcp_dtype w_dtype, int N, int K, const float* clip_lo, const float* clip_hi,
                        const float* frac, const float* grid_host, void* packed_out, void* codebook_out, void* stream)
{
    if (!W || !clip_lo || !clip_hi || !frac || !grid_host || !packed_out || !codebook_out)
        return fail(RCP_ERR_NULL, "rcp_pack_weights_w3: NULL pointer argument");
    if (int rc = check_shape("rcp_pack_weights_w3", N, K)) return rc;
    if (w_dtype != RCP_F16 && w_dtype != RCP_F32 && w_dtype != RCP_BF16)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_pack_weights_w3: unknown dtype %d", static_cast<int>(w_dtype));
    W3Grid grid;
    for (int j = 0; j < 8; ++j) {
        grid.g[j] = grid_host[j];
        if (!(grid.g[j] - grid.g[j] == 0.0f) || (j > 0 && !(grid.g[j] > grid.g[j - 1])))
            return fail(RCP_ERR_UNSUPPORTED, "rcp_pack_weights_w3: the grid must be eight finite, strictly ascending values");
    }
    if (!aligned16(W) || !aligned16(packed_out) || !aligned16(codebook_out) || !aligned16(clip_lo) ||
        !aligned16(clip_hi) || !aligned16(frac))
        return fail(RCP_ERR_ALIGN, "rcp_pack_weights_w3: device buffers must be 16-byte aligned");
    return launch_pack_w3(W, w_dtype, N, K, clip_lo, clip_hi, frac, grid, packed_out, codebook_out,
                          static_cast<hipStream_t>(stream));
}

int rcp_unpack_indices_w3(const void* packed, int N, int K, uint8_t* idx_out, void* stream)
{
    if (!packed || !idx_out) return fail(RCP_ERR_NULL, "rcp_unpack_indices_w3: NULL pointer argument");
    if (int rc = check_shape("rcp_unpack_indices_w3", N, K)) return rc;
    if (!aligned16(packed) || !aligned16(idx_out))
        return fail(RCP_ERR_ALIGN, "rcp_unpack_indices_w3: device buffers must be 16-byte aligned");
    return launch_unpack_w3(packed, N, K, idx_out, static_cast<hipStream_t>(stream));
}

int rcp_w3a4_gemv(const void* packed, const void* codebook, int N, int K, const void* xq, const void* scale, void* out,
                  rcp_dtype out_dtype, int32_t* partial_sums_or_null, void* stream)
{
    if (!packed || !codebook || !xq || !scale || !out) return fail(RCP_ERR_NULL, "rcp_w3a4_gemv: NULL pointer argument");
    if (int rc = check_shape("rcp_w3a4_gemv", N, K)) return rc;
    if (out_dtype != RCP_F16 && out_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_w3a4_gemv: out_dtype must be RCP_F16 or RCP_F32");
    if (!aligned16(packed) || !aligned16(codebook) || !aligned16(xq) || !aligned16(out) ||
        !aligned16(partial_sums_or_null))
        return fail(RCP_ERR_ALIGN, "rcp_w3a4_gemv: device buffers must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(scale) & 1u) != 0)
        return fail(RCP_ERR_ALIGN, "rcp_w3a4_gemv: scale must be 2-byte aligned");
    return launch_w3a4_gemv(packed, codebook, N, K, xq, scale, out, out_dtype, partial_sums_or_null,
                            static_cast<hipStream_t>(stream));
}

int rcp_quant_w3a4_gemv(const void* packed, const void* codebook, int N, int K, const void* x, rcp_dtype x_dtype,
                        float clip_ratio, void* out, rcp_dtype out_dtype, void* xq_out_or_null, void* scale_out_or_null,
                        int32_t* partial_sums_or_null, void* stream)
{
    if (!packed || !codebook || !x || !out) return fail(RCP_ERR_NULL, "rcp_quant_w3a4_gemv: NULL pointer argument");
    if (int rc = check_shape("rcp_quant_w3a4_gemv", N, K)) return rc;
    if (x_dtype != RCP_F16 && x_dtype != RCP_F32 && x_dtype != RCP_BF16)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_quant_w3a4_gemv: unknown dtype %d", static_cast<int>(x_dtype));
    if (out_dtype != RCP_F16 && out_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_quant_w3a4_gemv: out_dtype must be RCP_F16 or RCP_F32");
    if (!(clip_ratio > 0.0f) || !(clip_ratio <= 1.0f))
        return fail(RCP_ERR_UNSUPPORTED, "rcp_quant_w3a4_gemv: clip_ratio %g outside (0, 1]", static_cast<double>(clip_ratio));
    if (!aligned16(packed) || !aligned16(codebook) || !aligned16(x) || !aligned16(out) || !aligned16(xq_out_or_null) ||
        !aligned16(partial_sums_or_null))
        return fail(RCP_ERR_ALIGN, "rcp_quant_w3a4_gemv: device buffers must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(scale_out_or_null) & 1u) != 0)
        return fail(RCP_ERR_ALIGN, "rcp_quant_w3a4_gemv: scale_out must be 2-byte aligned");
    return launch_quant_w3a4_gemv(packed, codebook, N, K, x, x_dtype, clip_ratio, out, out_dtype, xq_out_or_null,
                                  scale_out_or_null, partial_sums_or_null, static_cast<hipStream_t>(stream));
}

size_t rcp_kv4_workspace_bytes(int H_q, int S)
{
    if (H_q <= 0 || S <= 0 || S > RCP_KV_MAX_S) return 0;
    return kv4_workspace_bytes(H_q, S);
}

int rcp_kv4_append(const void* x, rcp_dtype x_dtype, int n_tokens, int H, int S_max, int pos, int rotate,
                   float clip_ratio, void* codes, void* params, void* stream)
{
    if (!x || !codes || !params) return fail(RCP_ERR_NULL, "rcp_kv4_append: NULL pointer argument");
    if (x_dtype != RCP_F16 && x_dtype != RCP_BF16 && x_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_kv4_append: unknown x_dtype %d", static_cast<int>(x_dtype));
    if (H <= 0 || S_max <= 0 || n_tokens < 0 || pos < 0 || static_cast<long long>(pos) + n_tokens > S_max)
        return fail(RCP_ERR_SHAPE, "rcp_kv4_append: H=%d, S_max=%d, pos=%d, n_tokens=%d do not fit", H, S_max, pos, n_tokens);
    if (static_cast<long long>(n_tokens) * H > 0x7fffffffLL / RCP_KV_HEAD_DIM)
        return fail(RCP_ERR_SHAPE, "rcp_kv4_append: n_tokens * H too large");
    if (!(clip_ratio > 0.0f) || clip_ratio > 1.0f)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_kv4_append: clip_ratio must be in (0, 1]");
    if (!aligned16(x) || !aligned16(codes) || !aligned16(params))
        return fail(RCP_ERR_ALIGN, "rcp_kv4_append: device buffers must be 16-byte aligned");
    return launch_kv4_append(x, x_dtype, n_tokens, H, S_max, pos, nullptr, rotate != 0, clip_ratio, codes, params,
                             static_cast<hipStream_t>(stream));
}

int rcp_kv4_append_kv(const void* k, const void* v, rcp_dtype x_dtype, int n_tokens, int H, int S_max, int pos, int rotate_k,
                      float clip_ratio, void* k_codes, void* k_params, void* v_codes, void* v_params, void* stream)
{
    if (!k || !v || !k_codes || !k_params || !v_codes || !v_params) return fail(RCP_ERR_NULL, "rcp_kv4_append_kv: NULL pointer argument");
    if (x_dtype != RCP_F16 && x_dtype != RCP_BF16 && x_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_kv4_append_kv: unknown x_dtype %d", static_cast<int>(x_dtype));
    if (H <= 0 || S_max <= 0 || n_tokens < 0 || pos < 0 || static_cast<long long>(pos) + n_tokens > S_max)
        return fail(RCP_ERR_SHAPE, "rcp_kv4_append_kv: H=%d, S_max=%d, pos=%d, n_tokens=%d do not fit", H, S_max, pos, n_tokens);
    if (static_cast<long long>(n_tokens) * H > 0x7fffffffLL / RCP_KV_HEAD_DIM)
        return fail(RCP_ERR_SHAPE, "rcp_kv4_append_kv: n_tokens * H too large");
    if (!(clip_ratio > 0.0f) || clip_ratio > 1.0f)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_kv4_append_kv: clip_ratio must be in (0, 1]");
    if (!aligned16(k) || !aligned16(v) || !aligned16(k_codes) || !aligned16(k_params) || !aligned16(v_codes) || !aligned16(v_params))
        return fail(RCP_ERR_ALIGN, "rcp_kv4_append_kv: device buffers must be 16-byte aligned");
    return launch_kv4_append_kv(k, v, x_dtype, n_tokens, H, S_max, pos, rotate_k != 0, clip_ratio, k_codes, k_params, v_codes, v_params,
                                static_cast<hipStream_t>(stream));
}

int rcp_kv4_append_batched(const void* x, rcp_dtype x_dtype, int B, int H, int S_max, const int* pos_host, int rotate,
                           float clip_ratio, void* codes, void* params, void* stream)
{
    if (!x || !codes || !params || !pos_host) return fail(RCP_ERR_NULL, "rcp_kv4_append_batched: NULL pointer argument");
    if (x_dtype != RCP_F16 && x_dtype != RCP_BF16 && x_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_kv4_append_batched: unknown x_dtype %d", static_cast<int>(x_dtype));
    if (B < 1 || B > RCP_MAX_M) return fail(RCP_ERR_SHAPE, "rcp_kv4_append_batched: B=%d outside 1..%d", B, RCP_MAX_M);
    if (H <= 0 || S_max <= 0 || H > 0x7fffffff / RCP_KV_HEAD_DIM / RCP_MAX_M)
        return fail(RCP_ERR_SHAPE, "rcp_kv4_append_batched: H=%d, S_max=%d out of range", H, S_max);
    for (int b = 0; b < B; ++b)
        if (pos_host[b] < 0 || pos_host[b] >= S_max)
            return fail(RCP_ERR_SHAPE, "rcp_kv4_append_batched: position %d of sequence %d outside 0..%d", pos_host[b], b, S_max - 1);
    if (!(clip_ratio > 0.0f) || clip_ratio > 1.0f)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_kv4_append_batched: clip_ratio must be in (0, 1]");
    if (!aligned16(x) || !aligned16(codes) || !aligned16(params))
        return fail(RCP_ERR_ALIGN, "rcp_kv4_append_batched: device buffers must be 16-byte aligned");
    return launch_kv4_append(x, x_dtype, B, H, S_max, 0, pos_host, rotate != 0, clip_ratio, codes, params,
                             static_cast<hipStream_t>(stream));
}

int rcp_kv4_attn_decode(const void* q, rcp_dtype q_dtype, int H_q, int H_kv, int S_max, int S, const void* k_codes,
                        const void* k_params, const void* v_codes, const void* v_params, float softmax_scale, void* out,
                        rcp_dtype out_dtype, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!q || !k_codes || !k_params || !v_codes || !v_params || !out)
        return fail(RCP_ERR_NULL, "rcp_kv4_attn_decode: NULL pointer argument");
    if (q_dtype != RCP_F16 && q_dtype != RCP_BF16 && q_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_kv4_attn_decode: unknown q_dtype %d", static_cast<int>(q_dtype));
    if (out_dtype != RCP_F16 && out_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_kv4_attn_decode: out_dtype must be RCP_F16 or RCP_F32");
    if (H_q <= 0 || H_kv <= 0 || H_q % H_kv != 0 || H_q > 65535)
        return fail(RCP_ERR_SHAPE, "rcp_kv4_attn_decode: H_q=%d must be a positive multiple of H_kv=%d", H_q, H_kv);
    if (S_max <= 0 || S < 1 || S > S_max)
        return fail(RCP_ERR_SHAPE, "rcp_kv4_attn_decode: S=%d must lie in 1 .. S_max=%d", S, S_max);
    if (S > RCP_KV_MAX_S) return fail(RCP_ERR_UNSUPPORTED, "rcp_kv4_attn_decode: S=%d exceeds RCP_KV_MAX_S=%d", S, RCP_KV_MAX_S);
    if (!aligned16(q) || !aligned16(k_codes) || !aligned16(k_params) || !aligned16(v_codes) || !aligned16(v_params) ||
        !aligned16(out) || !aligned16(workspace))
        return fail(RCP_ERR_ALIGN, "rcp_kv4_attn_decode: device buffers must be 16-byte aligned");
    const size_t need = kv4_workspace_bytes(H_q, S);
    if (workspace == nullptr || workspace_bytes < need)
        return fail(RCP_ERR_WORKSPACE, "rcp_kv4_attn_decode: workspace of %zu bytes needed, %zu given", need,
                    workspace ? workspace_bytes : static_cast<size_t>(0));
    return launch_kv4_attn(q, q_dtype, 1, H_q, H_kv, S_max, S, nullptr, k_codes, k_params, v_codes, v_params, softmax_scale,
                           out, out_dtype, workspace, static_cast<hipStream_t>(stream));
}

int rcp_kv4_rotate_attn_decode(const void* q, rcp_dtype q_dtype, int H_q, int H_kv, int S_max, int S, const void* k_codes,
                               const void* k_params, const void* v_codes, const void* v_params, float softmax_scale, void* out,
                               rcp_dtype out_dtype, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!q || !k_codes || !k_params || !v_codes || !v_params || !out)
        return fail(RCP_ERR_NULL, "rcp_kv4_rotate_attn_decode: NULL pointer argument");
    if (q_dtype != RCP_F16 && q_dtype != RCP_BF16 && q_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_kv4_rotate_attn_decode: unknown q_dtype %d", static_cast<int>(q_dtype));
    if (out_dtype != RCP_F16 && out_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_kv4_rotate_attn_decode: out_dtype must be RCP_F16 or RCP_F32");
    if (H_q <= 0 || H_kv <= 0 || H_q % H_kv != 0 || H_q > 65535)
        return fail(RCP_ERR_SHAPE, "rcp_kv4_rotate_attn_decode: H_q=%d must be a positive multiple of H_kv=%d", H_q, H_kv);
    if (S_max <= 0 || S < 1 || S > S_max)
        return fail(RCP_ERR_SHAPE, "rcp_kv4_rotate_attn_decode: S=%d must lie in 1 .. S_max=%d", S, S_max);
    if (S > RCP_KV_MAX_S) return fail(RCP_ERR_UNSUPPORTED, "rcp_kv4_rotate_attn_decode: S=%d exceeds RCP_KV_MAX_S=%d", S, RCP_KV_MAX_S);
    if (!aligned16(q) || !aligned16(k_codes) || !aligned16(k_params) || !aligned16(v_codes) || !aligned16(v_params) ||
        !aligned16(out) || !aligned16(workspace))
        return fail(RCP_ERR_ALIGN, "rcp_kv4_rotate_attn_decode: device buffers must be 16-byte aligned");
    const size_t need = kv4_workspace_bytes(H_q, S);
    if (workspace == nullptr || workspace_bytes < need)
        return fail(RCP_ERR_WORKSPACE, "rcp_kv4_rotate_attn_decode: workspace of %zu bytes needed, %zu given", need,
                    workspace ? workspace_bytes : static_cast<size_t>(0));
    return launch_kv4_attn(q, q_dtype, 1, H_q, H_kv, S_max, S, nullptr, k_codes, k_params, v_codes, v_params, softmax_scale,
                           out, out_dtype, workspace, static_cast<hipStream_t>(stream), true);
}

int rcp_kv4_attn_decode_batched(const void* q, rcp_dtype q_dtype, int B, int H_q, int H_kv, int S_max, const int* S_host,
                                const void* k_codes, const void* k_params, const void* v_codes, const void* v_params,
                                float softmax_scale, void* out, rcp_dtype out_dtype, void* workspace,
                                size_t workspace_bytes, void* stream)
{
    if (!q || !k_codes || !k_params || !v_codes || !v_params || !out || !S_host)
        return fail(RCP_ERR_NULL, "rcp_kv4_attn_decode_batched: NULL pointer argument");
    if (q_dtype != RCP_F16 && q_dtype != RCP_BF16 && q_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_kv4_attn_decode_batched: unknown q_dtype %d", static_cast<int>(q_dtype));
    if (out_dtype != RCP_F16 && out_dtype != RCP_F32)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_kv4_attn_decode_batched: out_dtype must be RCP_F16 or RCP_F32");
    if (B < 1 || B > RCP_MAX_M) return fail(RCP_ERR_SHAPE, "rcp_kv4_attn_decode_batched: B=%d outside 1..%d", B, RCP_MAX_M);
    if (H_q <= 0 || H_kv <= 0 || H_q % H_kv != 0 || H_q > 65535 / RCP_MAX_M)
        return fail(RCP_ERR_SHAPE, "rcp_kv4_attn_decode_batched: H_q=%d must be a positive multiple of H_kv=%d (at most %d)", H_q,
                    H_kv, 65535 / RCP_MAX_M);
    if (S_max <= 0) return fail(RCP_ERR_SHAPE, "rcp_kv4_attn_decode_batched: S_max=%d", S_max);
    int longest = 0;
    for (int b = 0; b < B; ++b) {
        if (S_host[b] < 1 || S_host[b] > S_max)
            return fail(RCP_ERR_SHAPE, "rcp_kv4_attn_decode_batched: length %d of sequence %d outside 1..S_max=%d", S_host[b], b, S_max);
        longest = S_host[b] > longest ? S_host[b] : longest;
    }
    if (longest > RCP_KV_MAX_S)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_kv4_attn_decode_batched: length %d exceeds RCP_KV_MAX_S=%d", longest, RCP_KV_MAX_S);
    if (!aligned16(q) || !aligned16(k_codes) || !aligned16(k_params) || !aligned16(v_codes) || !aligned16(v_params) ||
        !aligned16(out) || !aligned16(workspace))
        return fail(RCP_ERR_ALIGN, "rcp_kv4_attn_decode_batched: device buffers must be 16-byte aligned");
    const size_t need = static_cast<size_t>(B) * kv4_workspace_bytes(H_q, longest);
    if (workspace == nullptr || workspace_bytes < need)
        return fail(RCP_ERR_WORKSPACE, "rcp_kv4_attn_decode_batched: workspace of %zu bytes needed, %zu given", need,
                    workspace ? workspace_bytes : static_cast<size_t>(0));
    return launch_kv4_attn(q, q_dtype, B, H_q, H_kv, S_max, longest, S_host, k_codes, k_params, v_codes, v_params,
                           softmax_scale, out, out_dtype, workspace, static_cast<hipStream_t>(stream));
}

}  // extern "C"
