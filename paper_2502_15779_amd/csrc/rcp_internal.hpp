// Internal declarations shared by the translation units of librcp.so.
// Nothing here is part of the C ABI (that is include/rcp.h).
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "rcp.h"

namespace rcp {

// ---- error plumbing (api.hip) -------------------------------------------------
int fail(int code, const char* fmt, ...);
int check_launch(const char* what);  // hipGetLastError() -> RCP_ERR_HIP / RCP_OK

// ---- tuning knobs (api.hip), 0 = automatic --------------------------------------
struct Options {
    int gemv_lanes;      // lanes that share one group of four rows: 16 .. 256
    int gemv_unroll;     // 16-byte loads per lane and pipeline stage: 2 or 4
    int gemv_blocks;     // workgroups launched by the GEMV
    int gemv_variant;    // 0 automatic, 1 plain-ALU kernel for every M, 2 matrix-core kernel for every M
    int gemm_waves;      // wavefronts per workgroup of the matrix-core kernel: 1, 2, 4, 8
    int gemm_stage;      // K steps per pipeline stage of the matrix-core kernel: 1, 2
    int gemv_nt;         // non-temporal weight loads in the general one-token kernel: 1 = always, 2 = never
    int gemv_waves;      // wavefronts per workgroup of the fused one-token GEMV: 4 or 8
    int gemm_rows;       // output rows per workgroup of the matrix-core kernel: 16 or 64
    int kv_tokens;       // cached tokens per workgroup of the KV4 attention kernel: 64, 128 or 256
    int seq_blocks;      // workgroups of the GEMV sequence kernel
    int gemv_oneshot;    // one-token GEMV with all loads issued up front: 0 automatic, 1 whenever the shape fits, 2 never
};
Options& options();
int num_compute_units();

// ---- launchers (one per .hip file) -------------------------------------------------
int launch_pack(const void* W, rcp_dtype dt, int N, int K, const float* lo, const float* hi,
                const float* part, void* packed, void* codebook, hipStream_t st);
int launch_unpack(const void* packed, int N, int K, uint8_t* idx, hipStream_t st);
// group-wise quantisation units (128 input channels per LUT)
int launch_pack_grouped(const void* W, rcp_dtype dt, int N, int K, const float* lo, const float* hi,
                        const float* part, void* packed, void* codebook, hipStream_t st);
int launch_unpack_grouped(const void* packed, int N, int K, uint8_t* idx, hipStream_t st);
int launch_gemv_grouped(const void* packed, const void* codebook, int N, int K, const void* xq,
                        const void* scale, void* out, rcp_dtype out_dt, int32_t* P, hipStream_t st);

size_t act_workspace_bytes(int M, int K, const rcp_rotation* rot);
int launch_act(const void* x, rcp_dtype dt, int M, int K, const rcp_rotation* rot, float clip_ratio,
               void* xq, void* scale, void* ws, size_t ws_bytes, hipStream_t st);
// the same with the Kronecker scratch in the library's own fixed device array (allocates nothing)
int launch_act_static(const void* x, rcp_dtype dt, int M, int K, const rcp_rotation* rot, float clip_ratio, void* xq,
                      void* scale, hipStream_t st);

int launch_stream_read(const void* p, size_t bytes, uint32_t* sink, hipStream_t st);
int launch_rotate(const void* x, rcp_dtype dt, int M, int K, const rcp_rotation* rot, float* y, hipStream_t st);

int launch_gemv(const void* packed, const void* codebook, int N, int K, const void* xq,
                const void* scale, int M, void* out, rcp_dtype out_dt, int32_t* P, hipStream_t st);
bool quant_gemv_grouped_supported(int K);
int launch_quant_gemv_grouped(const void* packed, const void* codebook, int N, int K, const void* x, rcp_dtype x_dt,
                              float clip_ratio, void* out, rcp_dtype out_dt, void* xq_out, void* scale_out, int32_t* P,
                              hipStream_t st);
// weight-only GEMV: 16- or 32-bit activations, no activation quantiser (w2a16_gemv.hip)
int launch_w2a16_gemv(const void* packed, const void* codebook, int N, int K, const void* x, rcp_dtype x_dt,
                      void* out, rcp_dtype out_dt, hipStream_t st);
// 3-bit variant: eight levels per output row (pack.hip, w3a4_gemv.hip)
struct W3Grid {
    float g[8];
};
int launch_pack_w3(const void* W, rcp_dtype dt, int N, int K, const float* lo, const float* hi, const float* frac,
                   const W3Grid& grid, void* packed, void* codebook, hipStream_t st);
int launch_unpack_w3(const void* packed, int N, int K, uint8_t* idx, hipStream_t st);
int launch_w3a4_gemv(const void* packed, const void* codebook, int N, int K, const void* xq, const void* scale,
                     void* out, rcp_dtype out_dt, int32_t* P, hipStream_t st);
// matrix-core kernel for several tokens (gemm_mfma.hip)
int launch_quant_w3a4_gemv(const void* packed, const void* codebook, int N, int K, const void* x, rcp_dtype x_dt,
                           float clip_ratio, void* out, rcp_dtype out_dt, void* xq_out, void* scale_out, int32_t* P,
                           hipStream_t st);
size_t kv4_workspace_bytes(int H_q, int S);
int launch_kv4_append(const void* x, rcp_dtype dt, int n_tokens, int H, int S_max, int pos, const int* positions, bool rotate,
                      float clip_ratio, void* codes, void* params, hipStream_t st);
int launch_kv4_attn(const void* q, rcp_dtype q_dt, int B, int H_q, int H_kv, int S_max, int S, const int* lengths,
                    const void* k_codes, const void* k_params, const void* v_codes, const void* v_params,
                    float softmax_scale, void* out, rcp_dtype out_dt, void* workspace, hipStream_t st, bool rotate_q = false);
int launch_kv4_append_kv(const void* k, const void* v, rcp_dtype dt, int n_tokens, int H, int S_max, int pos, bool rotate_k,
                         float clip_ratio, void* k_codes, void* k_params, void* v_codes, void* v_params, hipStream_t st);
int launch_gemm_mfma(const void* packed, const void* codebook, int N, int K, const void* xq, const void* scale,
                     int M, void* out, rcp_dtype out_dt, int32_t* P, hipStream_t st);
int launch_gemm_mfma_grouped(const void* packed, const void* codebook, int N, int K, const void* xq,
                             const void* scale, int M, void* out, rcp_dtype out_dt, int32_t* P, hipStream_t st);
// fused quantise + GEMV for one token; x is the raw activation, xq_out / scale_out optional;
// rot_heads > 0: Hadamard across rot_heads heads of rot_head_dim channels applied in the prologue
int launch_quant_gemv(const void* packed, const void* codebook, int N, int K, const void* x, rcp_dtype x_dt,
                      float clip_ratio, void* out, rcp_dtype out_dt, void* xq_out, void* scale_out, int32_t* P,
                      int rot_heads, int rot_head_dim, hipStream_t st);
bool quant_gemv_supported(int K);
// the same with the order-K Hadamard rotation in the prologue (K a power of two, at most 2048)
bool wht_gemv_supported(int K);
int launch_wht_quant_gemv(const void* packed, const void* codebook, int N, int K, const void* x, rcp_dtype x_dt,
                          float clip_ratio, void* out, rcp_dtype out_dt, void* xq_out, void* scale_out, int32_t* P,
                          hipStream_t st);
// several dependent one-token GEMVs in one launch (gemv_seq.hip)
size_t gemv_sequence_workspace_bytes(const rcp_gemv_step* steps, int n);
int launch_gemv_sequence(const rcp_gemv_step* steps, int n, void* workspace, hipStream_t st);
// one-token GEMV with every load of a workgroup issued up front (gemv_oneshot.hip); x_dt < 0: quantised activations
bool gemv_oneshot_applies(int N, int K, bool fused);
int launch_gemv_oneshot(const void* packed, const void* codebook, int N, int K, const void* x, int x_dt, const void* scale,
                        float clip_ratio, void* out, rcp_dtype out_dt, int32_t* P, void* xq_out, void* scale_out, hipStream_t st);
int gemv_variant(int N, int K, int M);  // 1 vector-ALU kernel, 2 matrix-core kernel: what launch_gemv picks

// ---- small device helpers ------------------------------------------------------------
__device__ __forceinline__ float half_bits_to_float(uint16_t h)
{
    return __half2float(__ushort_as_half(h));
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b)
{
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// The binary32 value `o` (already rounded to binary32) rounded once more, to nearest even, to fp16.  The value is
// made opaque first: otherwise the compiler may merge the multiplication that produced it with the conversion
// into one instruction with a single rounding, and two kernels computing the same output could then differ in the
// last fp16 bit depending on how each was compiled.
__device__ __forceinline__ __half round_to_half(float o)
{
    asm volatile("" : "+v"(o));
    return __float2half_rn(o);
}

// Load element i of a tensor of 16- or 32-bit floats as fp32 (the widening is exact).
template <int DT>
__device__ __forceinline__ float load_as_float(const void* p, size_t i)
{
    if constexpr (DT == RCP_F32) return static_cast<const float*>(p)[i];
    else if constexpr (DT == RCP_F16) return half_bits_to_float(static_cast<const uint16_t*>(p)[i]);
    else return bf16_bits_to_float(static_cast<const uint16_t*>(p)[i]);
}

// Eight consecutive elements starting at element index i (a multiple of 8), in two steps so that a
// kernel can issue other loads between the memory access and the first use of its result:
// the raw 16 (two-byte types) or 32 bytes, then the exact widening to fp32.
template <int DT>
struct Raw8 {
    uint4 a;
    uint4 b;  // second half of eight fp32 values; unused for the two-byte types
};

template <int DT>
__device__ __forceinline__ Raw8<DT> load8_raw(const void* p, size_t i)
{
    Raw8<DT> r;
    if constexpr (DT == RCP_F32) {
        const uint4* q = reinterpret_cast<const uint4*>(static_cast<const float*>(p) + i);
        r.a = q[0];
        r.b = q[1];
    } else {
        r.a = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(p) + i);
        r.b = make_uint4(0u, 0u, 0u, 0u);
    }
    return r;
}

template <int DT>
__device__ __forceinline__ void widen8(const Raw8<DT>& r, float (&v)[8])
{
    if constexpr (DT == RCP_F32) {
        v[0] = __uint_as_float(r.a.x); v[1] = __uint_as_float(r.a.y); v[2] = __uint_as_float(r.a.z); v[3] = __uint_as_float(r.a.w);
        v[4] = __uint_as_float(r.b.x); v[5] = __uint_as_float(r.b.y); v[6] = __uint_as_float(r.b.z); v[7] = __uint_as_float(r.b.w);
    } else {
        const uint32_t w[4] = {r.a.x, r.a.y, r.a.z, r.a.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint16_t lo16 = static_cast<uint16_t>(w[e] & 0xffffu), hi16 = static_cast<uint16_t>(w[e] >> 16);
            if constexpr (DT == RCP_F16) {
                v[2 * e] = half_bits_to_float(lo16);
                v[2 * e + 1] = half_bits_to_float(hi16);
            } else {
                v[2 * e] = bf16_bits_to_float(lo16);
                v[2 * e + 1] = bf16_bits_to_float(hi16);
            }
        }
    }
}

template <int DT>
__device__ __forceinline__ void load8_as_float(const void* p, size_t i, float (&v)[8])
{
    widen8<DT>(load8_raw<DT>(p, i), v);
}

// ---- wavefront-wide reductions without LDS traffic: DPP rotations inside each row of 16
// lanes, then the four row results are read into scalar registers ----------------------------
__device__ __forceinline__ int row_sum16(int v)
{
    // rotations inside a row of 16 lanes: after ror 8, 4, 2, 1 every lane holds the row sum
    v += __builtin_amdgcn_update_dpp(0, v, 0x128, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x124, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x122, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x121, 0xf, 0xf, false);
    return v;
}

__device__ __forceinline__ int wave_sum(int v)
{
    v = row_sum16(v);
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
           __builtin_amdgcn_readlane(v, 48);
}

__device__ __forceinline__ float wave_max(float v)
{
#define RCP_ROW_MAX(ctrl) v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, 0xf, 0xf, false)))
    RCP_ROW_MAX(0x128);
    RCP_ROW_MAX(0x124);
    RCP_ROW_MAX(0x122);
    RCP_ROW_MAX(0x121);
#undef RCP_ROW_MAX
    const int b = __float_as_int(v);
    return fmaxf(fmaxf(__int_as_float(__builtin_amdgcn_readlane(b, 0)), __int_as_float(__builtin_amdgcn_readlane(b, 16))),
                 fmaxf(__int_as_float(__builtin_amdgcn_readlane(b, 32)), __int_as_float(__builtin_amdgcn_readlane(b, 48))));
}

// ---- packed-int4 dot product and two-register folds (GEMV kernels) ---------------------------
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int dot8(uint32_t a, uint32_t b, int c)
{
    return __builtin_amdgcn_sdot8(static_cast<int>(a), static_cast<int>(b), c, false);
}

// Adds the upper 32 lanes of a and b onto their lower 32: lanes 0..31 get a + a(lane^32),
// lanes 32..63 get b + b(lane^32)  (v_permlane32_swap folds two registers into one).
__device__ __forceinline__ int fold32(int a, int b)
{
    auto r = __builtin_amdgcn_permlane32_swap(static_cast<unsigned>(a), static_cast<unsigned>(b), false, false);
    return static_cast<int>(r[0]) + static_cast<int>(r[1]);
}

// Same for neighbouring 16-lane rows: even rows get a + a(row^1), odd rows b + b(row^1).
__device__ __forceinline__ int fold16(int a, int b)
{
    auto r = __builtin_amdgcn_permlane16_swap(static_cast<unsigned>(a), static_cast<unsigned>(b), false, false);
    return static_cast<int>(r[0]) + static_cast<int>(r[1]);
}

// The same folds and row sums for binary32 values.
__device__ __forceinline__ float fold32f(float a, float b)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ float fold16f(float a, float b)
{
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ float row_sum16f(float v)
{
#define RCP_ROW_ADD(ctrl) v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, 0xf, 0xf, false))
    RCP_ROW_ADD(0x128);
    RCP_ROW_ADD(0x124);
    RCP_ROW_ADD(0x122);
    RCP_ROW_ADD(0x121);
#undef RCP_ROW_ADD
    return v;
}

// One cell (4 rows x 8 columns, bit planes b0 and b1) against the matching int4 dword of MT tokens.
// acc[p][m]: plane p in {b0, b1, b0&b1}, nibble mask m in {1, 3, 7, F}
template <int MT>
__device__ __forceinline__ void cell_update(uint32_t b0, uint32_t b1, const uint32_t (&x)[MT], int (&acc)[MT][3][4])
{
    const uint32_t pl[3] = {b0, b1, b0 & b1};
#pragma unroll
    for (int p = 0; p < 3; ++p) {
        const uint32_t m1 = pl[p] & 0x11111111u, m3 = pl[p] & 0x33333333u, m7 = pl[p] & 0x77777777u;
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            acc[t][p][0] = dot8(x[t], m1, acc[t][p][0]);
            acc[t][p][1] = dot8(x[t], m3, acc[t][p][1]);
            acc[t][p][2] = dot8(x[t], m7, acc[t][p][2]);
            acc[t][p][3] = dot8(x[t], pl[p], acc[t][p][3]);
        }
    }
}

// ---- Walsh-Hadamard butterflies shared by the activation kernels and the rotating GEMV prologue ----
template <int LE>
__device__ __forceinline__ void register_stages(float (&v)[1 << LE], int first_bit)
{
#pragma unroll
    for (int b = 0; b < LE; ++b) {
        if (b < first_bit) continue;
        const int s = 1 << b;
#pragma unroll
        for (int i = 0; i < (1 << LE); ++i)
            if ((i & s) == 0) {
                const float p = v[i], q = v[i + s];
                v[i] = p + q;
                v[i + s] = p - q;
            }
    }
}

// The butterflies whose stride is a lane distance: element index bits LE .. LE + nbits - 1 are the low bits of the lane
// number (thread t owns elements t * EPT ...), so stage b exchanges with lane ^ (1 << b) -- DPP for 1, 2 and 8, a lane
// permutation for 4, the 16- and 32-lane swaps for the last two.  z <- z + partner in the lane with the bit clear,
// partner - z in the other: the additions of the plain butterfly, no LDS and no barrier.
template <int EPT>
__device__ __forceinline__ void lane_stages(float (&v)[EPT], int lane, int nbits)
{
    // stage by stage, the EPT values of a stage side by side: their exchanges are independent and overlap.
    // partner - z is written partner + (-z): the sign of z is flipped in the lanes with the stage's bit set (one XOR
    // with a per-lane mask), which leaves one addition for both halves.
    auto flip = [](float z, uint32_t sign) { return __uint_as_float(__float_as_uint(z) ^ sign); };
    // (all exchanges of a stage first, then all additions: written as two loops so that the eight chains are issued
    // interleaved instead of one after the other)
#define RCP_LANE_STAGE_DPP(BIT, CTRL)                                                                                   \
    if (nbits > BIT) {                                                                                                   \
        const uint32_t sg = static_cast<uint32_t>((lane >> BIT) & 1) << 31;                                              \
        float p[EPT];                                                                                                    \
        _Pragma("unroll") for (int e = 0; e < EPT; ++e)                                                                  \
            p[e] = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v[e]), CTRL, 0xf, 0xf, false));          \
        __builtin_amdgcn_sched_barrier(0);                                                                               \
        _Pragma("unroll") for (int e = 0; e < EPT; ++e) v[e] = p[e] + flip(v[e], sg);                                    \
    }
    RCP_LANE_STAGE_DPP(0, 0xB1)  // lane ^ 1
    RCP_LANE_STAGE_DPP(1, 0x4E)  // lane ^ 2
    if (nbits > 2) {
        const uint32_t sg = static_cast<uint32_t>((lane >> 2) & 1) << 31;
        float p[EPT];
#pragma unroll
        for (int e = 0; e < EPT; ++e) p[e] = __shfl_xor(v[e], 4, 64);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < EPT; ++e) v[e] = p[e] + flip(v[e], sg);
    }
    RCP_LANE_STAGE_DPP(3, 0x128)  // row_ror 8 = lane ^ 8
#undef RCP_LANE_STAGE_DPP
    // the swaps leave (value of the lane with the bit clear, value of the lane with it set) in every lane
#define RCP_LANE_STAGE_SWAP(BIT, SWAP)                                                                                   \
    if (nbits > BIT) {                                                                                                   \
        const uint32_t sg = static_cast<uint32_t>((lane >> BIT) & 1) << 31;                                              \
        uint32_t lo[EPT], hi[EPT];                                                                                       \
        _Pragma("unroll") for (int e = 0; e < EPT; ++e) {                                                                \
            auto r = SWAP(__float_as_uint(v[e]), __float_as_uint(v[e]), false, false);                                   \
            lo[e] = r[0];                                                                                                \
            hi[e] = r[1];                                                                                                \
        }                                                                                                                \
        __builtin_amdgcn_sched_barrier(0);                                                                               \
        _Pragma("unroll") for (int e = 0; e < EPT; ++e) v[e] = __uint_as_float(lo[e]) + __uint_as_float(hi[e] ^ sg);     \
    }
    RCP_LANE_STAGE_SWAP(4, __builtin_amdgcn_permlane16_swap)
    RCP_LANE_STAGE_SWAP(5, __builtin_amdgcn_permlane32_swap)
#undef RCP_LANE_STAGE_SWAP
}

// Where element a of the transform lives in LDS.  Every access pattern of the kernel (EPT
// consecutive elements per thread, and elements 2^lo apart per thread with neighbouring threads
// on neighbouring low bits) has some index bits fixed across the lanes of a wavefront; folding
// bits 3..5 into bits 0..2 and bits 6..7 into bits 3..4 makes each of them hit 32 different
// banks per half wavefront (without it the first and last pass are 8- to 16-way conflicted).
__device__ __forceinline__ int wht_slot(int a)
{
    return a ^ ((a >> 3) & 7) ^ (((a >> 6) & 3) << 3);
}

// ---- pieces shared by the one-launch-per-matrix GEMV and the sequence kernel ------------------
// The row (0..3 within its row group) whose sums lane `lane` ends up holding after
// reduce_rows<LW>, and whether the lane is one of those that write a result.
template <int LW>
__device__ __forceinline__ int lane_row(int lane)
{
    const int rho = lane >> 4;
    if constexpr (LW == 64) return ((rho & 1) << 1) | (rho >> 1);
    else if constexpr (LW == 32) return (rho & 1) + 2 * (lane & 1);
    else return lane & 3;
}
template <int LW>
__device__ __forceinline__ bool lane_writes(int lane)
{
    if constexpr (LW == 64) return (lane & 15) == 0;
    else if constexpr (LW == 32) return (lane & 15) < 2;
    else return (lane & 15) < 4;
}

// g[4p + r] is this lane's share of 2^r * f_r of plane p.  Sums over the LW lanes that
// share the row group and leaves in f[p] the total for row lane_row<LW>(lane).
template <int LW>
__device__ __forceinline__ void reduce_rows(const int (&g)[12], int lane, int (&f)[3])
{
    if constexpr (LW == 64) {
        int s[6];
#pragma unroll
        for (int i = 0; i < 6; ++i) s[i] = fold32(g[2 * i], g[2 * i + 1]);
#pragma unroll
        for (int p = 0; p < 3; ++p) f[p] = row_sum16(fold16(s[2 * p], s[2 * p + 1]));
    } else if constexpr (LW == 32) {
        const bool odd = lane & 1;
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            const int lo = row_sum16(fold16(g[4 * p + 0], g[4 * p + 1]));  // rows r = 0 | 1
            const int hi = row_sum16(fold16(g[4 * p + 2], g[4 * p + 3]));  // rows r = 2 | 3
            f[p] = odd ? hi : lo;
        }
    } else {
        const int j = lane & 3;
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            const int a0 = row_sum16(g[4 * p + 0]), a1 = row_sum16(g[4 * p + 1]);
            const int a2 = row_sum16(g[4 * p + 2]), a3 = row_sum16(g[4 * p + 3]);
            f[p] = (j == 0) ? a0 : (j == 1) ? a1 : (j == 2) ? a2 : a3;
        }
    }
}

// LDS: quantised activations, token t at dword t*(K/8), padded so that the reads of a
// lane whose unit lies beyond K stay inside the allocation (their weights are zero);
// then 4*MT ints of per-wavefront sums of q; then, for WS > 1, the cross-wavefront
// reduction slots int[2][4 waves][4 rows][3*MT].
__host__ __device__ constexpr int gemv_x_bytes(int K, int M, int span /* LG * UNR */)
{
    const int U = K / 16;
    const int padded_units = ((U + span - 1) / span) * span;
    return ((M - 1) * U + padded_units) * 8;
}

// ---- FP4 (E2M1) operands of the 16x16x128 matrix instruction -------------------------------
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

// eight int4 (two's complement) -> eight FP4 codes of lo = q & 3 in {0, 1, 2, 3}
__device__ __forceinline__ uint32_t fp4_lo(uint32_t x)
{
    const uint32_t n0 = x & 0x11111111u, n1 = x & 0x22222222u;
    const uint32_t both = n0 & (n1 >> 1);            // lo == 3 -> code 0101 (3.0): bit 0
    return both | (((n0 ^ both) | n1) << 1);         // lo == 1 -> 0010 (1.0), lo >= 2 -> bit 2 (2.0)
}

// eight int4 -> eight FP4 codes of hi = q >> 2 in {-2, -1, 0, 1}: 1100, 1010, 0000, 0010
__device__ __forceinline__ uint32_t fp4_hi(uint32_t x)
{
    const uint32_t n3 = x & 0x88888888u, n2 = x & 0x44444444u;
    return n3 | ((n3 >> 1) & ~n2) | (n2 >> 1);
}

// ---- the int4 quantiser (shared by the activation kernels and the fused GEMV prologue) ----
// S = fp16((ratio * a) / 7); 1 when that is zero, capped at the largest finite half.
__device__ __forceinline__ uint16_t scale_bits_from_amax(float a, float clip_ratio)
{
    const float raw = __fdiv_rn(__fmul_rn(clip_ratio, a), 7.0f);
    uint16_t b = __half_as_ushort(__float2half_rn(raw));
    if ((b & 0x7fffu) == 0) b = 0x3c00u;
    if ((b & 0x7fffu) >= 0x7c00u) b = 0x7bffu;
    return b;
}

// Eight values -> one dword of int4: nibble j = clamp(rint(y[j] / s), -8, 7), where y/s is
// the correctly rounded binary32 quotient.  t = y * (1/s) carries two roundings, the quotient
// one: for |t| <= 16.5 the two differ by less than 3e-6, so rint(t) is already the answer
// unless t sits within 1e-5 of a rounding boundary n + 1/2 (beyond 16 both clamp to the same
// end); in that rare case the eight values are redone with the IEEE division.
// The clamped integers r_j are packed four at a time in binary32, where
// sum_j (r_j + 8) * 16^j < 2^16 is exact, and the offset-binary nibbles become two's
// complement by flipping each nibble's top bit.
// The same in two pieces for callers that quantise several groups of eight and want their instruction chains
// interleaved: quantize8_fast rounds through the reciprocal without any branch and keeps, in `far`, the largest distance
// of a scaled value from its rounded value; if that ends up above 0.49999 for a lane, the caller redoes that lane's
// groups with quantize8_exact (one branch for all groups instead of one per group).  That is for binary32 inputs, where
// a value that close to a boundary is a one-in-50000 event; 16-bit inputs, where exact ties are a one-in-a-thousand
// event per value and most wavefronts would take the branch, go through quantize8_short instead.
__device__ __forceinline__ uint32_t pack8_int4(const float (&n)[8])
{
    float r[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = __builtin_amdgcn_fmed3f(n[j], -8.0f, 7.0f);
    const float lo = fmaf(r[3], 4096.0f, fmaf(r[2], 256.0f, fmaf(r[1], 16.0f, r[0] + 34952.0f)));  // + 0x8888
    const float hi = fmaf(r[7], 4096.0f, fmaf(r[6], 256.0f, fmaf(r[5], 16.0f, r[4] + 34952.0f)));
    return (static_cast<uint32_t>(lo) | (static_cast<uint32_t>(hi) << 16)) ^ 0x88888888u;
}

__device__ __forceinline__ uint32_t quantize8_fast(const float (&y)[8], float rs, float& far)
{
    float n[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float t = __fmul_rn(y[j], rs);
        n[j] = rintf(t);
        far = fmaxf(far, fabsf(t - n[j]));
    }
    return pack8_int4(n);
}

// For y that holds fp16 or bf16 numbers as they came from memory (no rotation in between): no second pass at all.  With
// at most 11 significant bits in y and in the fp16 scale, the exact quotient y/s is either exactly a half-integer k + 1/2
// or at least 2^-13 away from every one of them up to 16.5 ((2 m_y 2^e - (2k+1) m_s) / (2 m_s) with integers m < 2^11 is
// zero or at least that large).  One Newton step on the quotient, q1 = q0 + (y - q0 s) (1/s) with the residual taken
// exactly by a fused multiply-add, lands on k + 1/2 itself in the first case (the residual's share of the error of 1/s is
// far below half a unit in the last place), where rint breaks the tie to even exactly like the correctly rounded
// quotient would; in the second case q1 and the correctly rounded quotient are both within 2e-6 of the exact one and on
// the same side of every boundary.  Beyond 16.5 both clamp to the same end.
__device__ __forceinline__ uint32_t quantize8_short(const float (&y)[8], float s, float rs)
{
    float n[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float q0 = __fmul_rn(y[j], rs);
        const float q1 = __fmaf_rn(__fmaf_rn(-q0, s, y[j]), rs, q0);
        n[j] = rintf(q1);
    }
    return pack8_int4(n);
}

__device__ __forceinline__ uint32_t quantize8_exact(const float (&y)[8], float s)
{
    float n[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) n[j] = rintf(__fdiv_rn(y[j], s));
    return pack8_int4(n);
}

__device__ __forceinline__ uint32_t quantize8(const float (&y)[8], float s)
{
    const float rs = __frcp_rn(s);
    float n[8];
    float far = 0.0f;  // largest distance of a t from its rounded value (one maximum instead of eight tests)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float t = __fmul_rn(y[j], rs);
        n[j] = rintf(t);
        far = fmaxf(far, fabsf(t - n[j]));
    }
    if (__builtin_expect(far > 0.49999f, 0)) {
#pragma unroll
        for (int j = 0; j < 8; ++j) n[j] = rintf(__fdiv_rn(y[j], s));
    }
    float r[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = __builtin_amdgcn_fmed3f(n[j], -8.0f, 7.0f);
    const float lo = fmaf(r[3], 4096.0f, fmaf(r[2], 256.0f, fmaf(r[1], 16.0f, r[0] + 34952.0f)));  // + 0x8888
    const float hi = fmaf(r[7], 4096.0f, fmaf(r[6], 256.0f, fmaf(r[5], 16.0f, r[4] + 34952.0f)));
    return (static_cast<uint32_t>(lo) | (static_cast<uint32_t>(hi) << 16)) ^ 0x88888888u;
}

}  // namespace rcp
