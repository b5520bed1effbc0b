// 4-bit KV cache (Appendix table of quantisation configurations: asymmetric, groups of 128 = one
// head vector, clipping ratio 0.95; the quantiser is Eqn. 1 with N = 4) and one-token attention
// over it (Section 2.1: R3 rotates queries and keys so that the cache can be held in 4 bits).
//
// Layout of one cached tensor (keys or values) of one layer, head size 128:
//   codes   [H][S_max][64 bytes]  element j of a head vector in byte j / 2, bits 4 * (j % 2) ...
//   params  [H][S_max] dwords     bits 0..15 the binary16 step s, bits 16..31 the int16 zero point z
// Head-major, so that the tokens one head attends to are contiguous: a wavefront reads 1 KiB
// (16 tokens) per load instruction.
#include <math.h>

#include "rcp_internal.hpp"

namespace rcp {

constexpr int KV_D = 128;

// Batched calls: per-sequence lengths (attention) or positions (append) travel by value.
struct KvBatch {
    int v[RCP_MAX_M];
    int H_q, H_kv;
};

// ---------------------------------------------------------------------------------------
// append: quantise n_tokens x H head vectors into cache positions pos ...
// Sixteen lanes (one DPP row) own a head vector, eight consecutive elements each.
// ROT: the vector first goes through the normalised order-128 Hadamard transform: butterflies in
// ascending stride order (1, 2, 4 in registers, 8 .. 64 between the sixteen lanes), each output
// one IEEE add or subtract, then one multiplication by (float)(1/sqrt(128)).
// ---------------------------------------------------------------------------------------
// BATCHED: row i of x belongs to sequence i (one new token each), whose cache starts at head
// i * H of the pooled cache and whose position is batch.v[i].
template <int DT, bool ROT, bool BATCHED>
__device__ __forceinline__ void kv4_append_rows(const void* __restrict__ x, int rows, int H, int S_max, int pos, float clip_ratio,
                                                uint32_t* __restrict__ codes, uint32_t* __restrict__ params, const KvBatch& batch,
                                                int block)
{
    // every product and difference below is rounded on its own (hi_c - lo_c must not become a
    // fused multiply-add: for a constant vector it has to be exactly zero).  The pragma covers
    // the operators written in this body, hence plain * and - rather than the __f*_rn wrappers.
#pragma clang fp contract(off)
    const int row = block * 16 + (threadIdx.x >> 4);
    const int l = threadIdx.x & 15;
    const bool have = row < rows;
    const int rr = have ? row : rows - 1;  // surplus lanes repeat the last vector and store nothing
    float v[8];
    load8_as_float<DT>(x, static_cast<size_t>(rr) * KV_D + 8 * l, v);
    if constexpr (ROT) {
#pragma unroll
        for (int st = 1; st < 8; st <<= 1)
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if ((e & st) == 0) {
                    const float a = v[e], b = v[e + st];
                    v[e] = a + b;
                    v[e + st] = a - b;
                }
#pragma unroll
        for (int m = 1; m < 16; m <<= 1) {  // element stride 8 * m: the partner is lane l ^ m of the row
            const bool upper = (l & m) != 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float other = __shfl_xor(v[e], m, 16);
                v[e] = upper ? other - v[e] : v[e] + other;
            }
        }
        const float norm = 0.088388347648318440550f;  // (float)(1 / sqrt(128))
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = v[e] * norm;
    }
    float lo = v[0], hi = v[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) {
        lo = fminf(lo, v[j]);
        hi = fmaxf(hi, v[j]);
    }
#define RCP_ROW_MINMAX(ctrl)                                                                                        \
    lo = fminf(lo, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(lo), ctrl, 0xf, 0xf, false)));    \
    hi = fmaxf(hi, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(hi), ctrl, 0xf, 0xf, false)))
    RCP_ROW_MINMAX(0x128);
    RCP_ROW_MINMAX(0x124);
    RCP_ROW_MINMAX(0x122);
    RCP_ROW_MINMAX(0x121);
#undef RCP_ROW_MINMAX
    const float lo_c = clip_ratio * lo, hi_c = clip_ratio * hi;
    const float range = hi_c - lo_c;
    const float raw = __fdiv_rn(range, 15.0f);
    uint16_t sb = __half_as_ushort(__float2half_rn(raw));
    if ((sb & 0x7fffu) == 0) sb = 0x3c00u;
    if ((sb & 0x7fffu) >= 0x7c00u) sb = 0x7bffu;
    const float s = half_bits_to_float(sb);
    float zf = -rintf(__fdiv_rn(lo_c, s));
    zf = fminf(fmaxf(zf, -32768.0f), 32767.0f);
    const int z = static_cast<int>(zf);
    zf = static_cast<float>(z);
    uint32_t word = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float r = __builtin_amdgcn_fmed3f(rintf(__fdiv_rn(v[j], s)) + zf, 0.0f, 15.0f);
        word |= static_cast<uint32_t>(r) << (4 * j);
    }
    if (have) {
        const int i = row / H, h = row - i * H;
        const size_t slot = BATCHED ? static_cast<size_t>(row) * S_max + batch.v[i]
                                    : static_cast<size_t>(h) * S_max + (pos + i);
        codes[slot * 16 + l] = word;
        if (l == 0) params[slot] = static_cast<uint32_t>(sb) | (static_cast<uint32_t>(z & 0xffff) << 16);
    }
}

template <int DT, bool ROT, bool BATCHED>
__global__ __launch_bounds__(256) void kv4_append_kernel(const void* __restrict__ x, int rows, int H, int S_max, int pos,
                                                         float clip_ratio, uint32_t* __restrict__ codes,
                                                         uint32_t* __restrict__ params, KvBatch batch)
{
    kv4_append_rows<DT, ROT, BATCHED>(x, rows, H, S_max, pos, clip_ratio, codes, params, batch, blockIdx.x);
}

// The new keys and the new values of the same tokens in one launch: blockIdx.y = 0 quantises the keys (rotated when
// rotate_k is set), blockIdx.y = 1 the values (never rotated) -- the arithmetic of kv4_append_kernel on each.
template <int DT>
__global__ __launch_bounds__(256) void kv4_append_kv_kernel(const void* __restrict__ k, const void* __restrict__ v, int rows, int H,
                                                            int S_max, int pos, int rotate_k, float clip_ratio,
                                                            uint32_t* __restrict__ k_codes, uint32_t* __restrict__ k_params,
                                                            uint32_t* __restrict__ v_codes, uint32_t* __restrict__ v_params)
{
    const KvBatch none = {};
    if (blockIdx.y == 0) {
        if (rotate_k) kv4_append_rows<DT, true, false>(k, rows, H, S_max, pos, clip_ratio, k_codes, k_params, none, blockIdx.x);
        else kv4_append_rows<DT, false, false>(k, rows, H, S_max, pos, clip_ratio, k_codes, k_params, none, blockIdx.x);
    } else {
        kv4_append_rows<DT, false, false>(v, rows, H, S_max, pos, clip_ratio, v_codes, v_params, none, blockIdx.x);
    }
}

// ---------------------------------------------------------------------------------------
// one-token attention, split along the sequence.
// Workgroup (split, query head): L = 64, 128 or 256 cached tokens.  Four lanes own a token, 16 bytes (32
// elements) of its vector each; a wavefront covers 16 tokens per load, the workgroup 64.
//   pass 1  scores q . K_t (kept in registers), their maximum m
//   pass 2  p_t = exp(score_t - m), l = sum p_t, acc_j = sum_t p_t * V_tj
// and (m, l, acc) go to the workspace; kv4_combine_kernel merges the splits.
// With x_tj = s_t * (c_tj - z_t):  q . K_t = s_t * (sum_j q_j c_tj - z_t * sum_j q_j)  and
// sum_t p_t V_tj = sum_t (p_t s_t) c_tj - sum_t p_t s_t z_t, so the codes enter as plain integers.
//
// Register r = 8 d + 4 e + b of a lane stands for element 8 d + 2 b + e of its 32 (dword d of
// the 16 bytes, byte b, nibble e): the order in which the nibbles come out of two masks.
// ---------------------------------------------------------------------------------------
constexpr int KV_THREADS = 256;
constexpr int KV_MAX_L = 256;          // tokens per workgroup at most: four per lane group, all loads in flight at once
constexpr int KV_PART = KV_D + 4;      // floats per partial result: acc[128], m, l, 2 unused
constexpr float KV_LAZY = 30.0f;       // how far a score may exceed the streaming kernel's reference before it is raised
constexpr int KV_STREAM_L = 1024;      // tokens per workgroup of the streaming kernel unless the option says otherwise

// The four low nibbles and the four high nibbles of a dword as bytes.  The empty asm keeps the
// compiler from folding the mask into each later byte extraction (a 4-bit field extract plus a
// conversion per element); with the bytes opaque, (x >> 8 b) & 0xff becomes one
// v_cvt_f32_ubyte<b> per element.
__device__ __forceinline__ void nibble_bytes(uint32_t w, uint32_t& lo, uint32_t& hi)
{
    lo = w & 0x0f0f0f0fu;
    hi = (w >> 4) & 0x0f0f0f0fu;
    asm("" : "+v"(lo), "+v"(hi));
}

// Four bytes b in 0..15 -> four floats b * unit in two instructions: read as FP8 (E4M3) numbers, the codes
// 0..7 are subnormals and 8..15 the first binade, both linear in b, so v_cvt_pk_f32_fp8 converts two at a
// time; `kv_fp8_unit()` is what it gives for the byte 1 (a power of two), divided out again by the callers.
typedef float v2f __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void bytes_to_floats(uint32_t x, float (&f)[4])
{
    const v2f a = __builtin_amdgcn_cvt_pk_f32_fp8(static_cast<int>(x), false);
    const v2f b = __builtin_amdgcn_cvt_pk_f32_fp8(static_cast<int>(x), true);
    f[0] = a[0];
    f[1] = a[1];
    f[2] = b[0];
    f[3] = b[1];
}

__device__ __forceinline__ float kv_fp8_unit() { return __builtin_amdgcn_cvt_pk_f32_fp8(1, false)[0]; }

__device__ __forceinline__ int kv_elem_of_reg(int r) { return 8 * (r >> 3) + 2 * (r & 3) + ((r >> 2) & 1); }

__device__ __forceinline__ float quad_sum(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false));  // lanes 1,0,3,2
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false));  // lanes 2,3,0,1
    return v;
}

// sum over the four tokens of a row of 16 lanes (lanes 4 apart hold the same piece)
__device__ __forceinline__ float row_tokens_sum(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x124, 0xf, 0xf, false));  // row_ror 4
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x128, 0xf, 0xf, false));  // row_ror 8
    return v;
}

// The query values of a lane (32 consecutive elements of a head vector, the four lanes of a quad hold all 128) through
// the normalised order-128 Hadamard transform: butterflies in ascending stride order (1 .. 16 in registers, 32 and 64
// between the lanes of the quad), each output one IEEE add or subtract, then one multiplication by (float)(1/sqrt(128)):
// bit for bit what rcp_rotate_act gives for a row of 128.
__device__ __forceinline__ void kv_rotate_query(float (&t)[32], int piece)
{
#pragma clang fp contract(off)
#pragma unroll
    for (int st = 1; st < 32; st <<= 1)
#pragma unroll
        for (int e = 0; e < 32; ++e)
            if ((e & st) == 0) {
                const float a = t[e], b = t[e + st];
                t[e] = a + b;
                t[e + st] = a - b;
            }
#pragma unroll
    for (int e = 0; e < 32; ++e) {  // stride 32: the partner is lane piece ^ 1 of the quad
        const float other = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(t[e]), 0xB1, 0xf, 0xf, false));
        t[e] = (piece & 1) ? other - t[e] : t[e] + other;
    }
#pragma unroll
    for (int e = 0; e < 32; ++e) {  // stride 64: lane piece ^ 2
        const float other = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(t[e]), 0x4E, 0xf, 0xf, false));
        t[e] = (piece & 2) ? other - t[e] : t[e] + other;
    }
    const float norm = 0.088388347648318440550f;  // (float)(1 / sqrt(128))
#pragma unroll
    for (int e = 0; e < 32; ++e) t[e] = t[e] * norm;
}

// This lane's 32 query values in register order (r = 8 d + 4 e + b <-> element 8 d + 2 b + e) and their sum.
template <int QDT>
__device__ __forceinline__ float kv_query_registers(const Raw8<QDT> (&qraw)[4], bool rotate, int piece, float (&qr)[32])
{
    float t[32];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        float t8[8];
        widen8<QDT>(qraw[d], t8);
#pragma unroll
        for (int e = 0; e < 8; ++e) t[8 * d + e] = t8[e];
    }
    if (rotate) kv_rotate_query(t, piece);  // uniform
    float qsum = 0.0f;
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                qr[8 * d + 4 * e + b] = t[8 * d + 2 * b + e];
                qsum += qr[8 * d + 4 * e + b];
            }
    return qsum;
}

// out_hj = sum_i e^(m_i - M) acc_ij / sum_i e^(m_i - M) l_i over the splits i of one head (src: its partial results).
// `groups` x 128 (virtual) threads: thread (g, j) merges the splits i = g, g + groups, ... of column j, four at a time so
// that their loads are in flight together, against its own running maximum; the groups meet in LDS and are merged the
// same way.
constexpr int KV_CT = 1024;
struct KvMergeLds {
    float red[KV_CT / KV_D][KV_D];
    float dred[KV_CT / KV_D], mred[KV_CT / KV_D];
};

__device__ __forceinline__ void kv_merge_head(const float* __restrict__ src, int splits, int groups, void* __restrict__ out,
                                              bool out_f16, int h, KvMergeLds& lds, int nthreads)
{
    for (int vt = threadIdx.x; vt < groups * KV_D; vt += nthreads) {
        const int j = vt & (KV_D - 1), g = vt >> 7;
        float M = -INFINITY, num = 0.0f, den = 0.0f;
        for (int i0 = g; i0 < splits; i0 += 4 * groups) {
            float mi[4], li[4], ai[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = min(i0 + groups * u, splits - 1);
                mi[u] = *(src + i * KV_PART + KV_D);
                li[u] = *(src + i * KV_PART + KV_D + 1);
                ai[u] = *(src + i * KV_PART + j);
            }
            float mb = M;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i0 + groups * u < splits) mb = fmaxf(mb, mi[u]);
            const float r = __expf(M - mb);  // 0 on the first round (M = -inf, mb finite)
            num *= r;
            den *= r;
            M = mb;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float e = (i0 + groups * u < splits) ? __expf(mi[u] - M) : 0.0f;
                num = fmaf(e, ai[u], num);
                den = fmaf(e, li[u], den);
            }
        }
        lds.red[g][j] = num;  // a group without a split leaves M = -inf, num = den = 0
        if (j == 0) {
            lds.dred[g] = den;
            lds.mred[g] = M;
        }
    }
    __syncthreads();
    if (threadIdx.x < KV_D) {
        const int tid = threadIdx.x;
        float Mt = lds.mred[0];
        for (int w = 1; w < groups; ++w) Mt = fmaxf(Mt, lds.mred[w]);
        float n = 0.0f, d = 0.0f;
        for (int w = 0; w < groups; ++w) {
            const float e = __expf(lds.mred[w] - Mt);
            n = fmaf(e, lds.red[w][tid], n);
            d = fmaf(e, lds.dred[w], d);
        }
        const float r = n / d;
        if (out_f16) static_cast<__half*>(out)[h * KV_D + tid] = __float2half_rn(r);
        else static_cast<float*>(out)[h * KV_D + tid] = r;
    }
}

// BATCHED: blockIdx.z is the sequence; its length is batch.v[z], its caches start at head z * H_kv of
// the pooled buffers, its query and partial results at row z * H_q; workgroups past its end leave.
// Which (split, query head, cache head) a workgroup works on.  Workgroups go to the eight dies (each with
// its own L2) in turn by their index, so the H_q / H_kv query heads that read the same cache head over the
// same split are given indices 8 apart: they run on one die at about the same time and the cache bytes come
// from HBM once instead of once per query head.  Unit u = (split, cache head); index = u % 8 + 8 * (rep * (u / 8) + r)
// for query head r of the group.  With rep = 1 this is the plain order.  False for the padding of the grid.
__device__ __forceinline__ bool kv_place(unsigned index, int splits, int rep, int H_kv, int& split, int& h, int& hk)
{
    const unsigned die = index & 7u, t = index >> 3;
    const unsigned r = t % static_cast<unsigned>(rep), k = t / static_cast<unsigned>(rep);
    const unsigned u = 8u * k + die;
    if (u >= static_cast<unsigned>(splits) * static_cast<unsigned>(H_kv)) return false;
    split = static_cast<int>(u % static_cast<unsigned>(splits));
    hk = static_cast<int>(u / static_cast<unsigned>(splits));
    h = hk * rep + static_cast<int>(r);
    return true;
}

// QROT: the query first goes through the order-128 Hadamard transform (R3), in the prologue, while the cache loads are
// in flight.
template <int QDT, int ITERS, bool BATCHED, bool QROT = false>
__global__ __launch_bounds__(KV_THREADS) void kv4_attn_kernel(const void* __restrict__ q, int S, int S_max, int rep, int splits,
                                                              float softmax_scale, const u32x4* __restrict__ k_codes,
                                                              const uint32_t* __restrict__ k_params,
                                                              const u32x4* __restrict__ v_codes,
                                                              const uint32_t* __restrict__ v_params,
                                                              float* __restrict__ part, KvBatch batch)
{
    __shared__ float red[4][KV_D];
    __shared__ float wmax[4], lrow[4][4], zrow[4][4];
    constexpr int L = 64 * ITERS;
    int split, h, hk;
    if (!kv_place(blockIdx.x, splits, rep, batch.H_kv, split, h, hk)) return;  // padding of the grid
    const int tid = threadIdx.x, slot = tid >> 2, piece = tid & 3, wave = tid >> 6;
    const int t0 = split * L;
    if constexpr (BATCHED) {
        const int seq = blockIdx.z;
        S = batch.v[seq];
        if (t0 >= S) return;  // the whole workgroup: this sequence has fewer splits
        h += seq * batch.H_q;
        hk += seq * batch.H_kv;
    }
    const int t_end = min(S, t0 + L);
    const size_t head_base = static_cast<size_t>(hk) * S_max;

    // every load of the workgroup is issued before the first use: the query, then the keys,
    // then the values (slots past the end repeat the last token and get weight 0)
    Raw8<QDT> qraw[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) qraw[d] = load8_raw<QDT>(q, static_cast<size_t>(h) * KV_D + 32 * piece + 8 * d);
    u32x4 kw[ITERS], vw[ITERS];
    uint32_t kp[ITERS], vp[ITERS];
    bool valid[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int t = t0 + it * 64 + slot;
        valid[it] = t < t_end;
        const size_t at = head_base + (valid[it] ? t : t_end - 1);
        // the cache is read once per call: loads with the non-temporal hint (6.6 -> 6.0 us at 1024 tokens, 13.2 -> 12.5 at
        // 8192, 57 -> 51 us for 16 sequences of 4096 in the streaming kernel)
        kw[it] = __builtin_nontemporal_load(k_codes + (at * 4 + piece));
        kp[it] = __builtin_nontemporal_load(k_params + at);
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int t = t0 + it * 64 + slot;
        const size_t at = head_base + (valid[it] ? t : t_end - 1);
        vw[it] = __builtin_nontemporal_load(v_codes + (at * 4 + piece));
        vp[it] = __builtin_nontemporal_load(v_params + at);
    }

    // this lane's 32 query values in register order (the softmax scale goes onto the score)
    float qr[32];
    const float qsum = kv_query_registers<QDT>(qraw, QROT, piece, qr);

    const float unit = kv_fp8_unit(), inv_unit = 1.0f / unit;
    const float scale_by_unit = softmax_scale * inv_unit, qsum_unit = qsum * unit;

    // ---- pass 1: scores (all four lanes of a token end up holding its score) ----
    float score[ITERS];
    float top = -INFINITY;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        float dot[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t lo, hi;
            nibble_bytes(kw[it][d], lo, hi);
            float fl[4], fh[4];
            bytes_to_floats(lo, fl);
            bytes_to_floats(hi, fh);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                dot[d] = fmaf(qr[8 * d + b], fl[b], dot[d]);
                dot[d] = fmaf(qr[8 * d + 4 + b], fh[b], dot[d]);
            }
        }
        // dot = unit * sum q c: the unit (a power of two) is taken out exactly
        const float s = half_bits_to_float(static_cast<uint16_t>(kp[it] & 0xffffu)) * scale_by_unit;
        const float z = static_cast<float>(static_cast<int>(kp[it]) >> 16);
        float sc = s * (((dot[0] + dot[1]) + (dot[2] + dot[3])) - z * qsum_unit);
        sc = quad_sum(sc);
        score[it] = valid[it] ? sc : -INFINITY;
        top = fmaxf(top, score[it]);
    }
    top = wave_max(top);
    if ((tid & 63) == 0) wmax[wave] = top;
    __syncthreads();
    const float m = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));

    // ---- pass 2: weights and the value sum ----
    float acc[32];
#pragma unroll
    for (int r = 0; r < 32; ++r) acc[r] = 0.0f;
    float lsum = 0.0f, zacc = 0.0f;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const float p = __expf(score[it] - m);  // exp(-inf) = 0 for the surplus slots
        const float w0 = p * half_bits_to_float(static_cast<uint16_t>(vp[it] & 0xffffu));
        const float w = w0 * inv_unit;  // the converted codes carry the factor unit
        lsum += p;
        zacc = fmaf(w0, static_cast<float>(static_cast<int>(vp[it]) >> 16), zacc);
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t lo, hi;
            nibble_bytes(vw[it][d], lo, hi);
            float fl[4], fh[4];
            bytes_to_floats(lo, fl);
            bytes_to_floats(hi, fh);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                acc[8 * d + b] = fmaf(w, fl[b], acc[8 * d + b]);
                acc[8 * d + 4 + b] = fmaf(w, fh[b], acc[8 * d + 4 + b]);
            }
        }
    }

    // ---- the 64 tokens of a workgroup pass are summed: rows of 16 lanes by DPP, the four rows
    // by two register folds (after which a lane of row w holds registers 4 k + w), the four
    // wavefronts through LDS ----
#pragma unroll
    for (int r = 0; r < 32; ++r) acc[r] = row_tokens_sum(acc[r]);
    lsum = row_tokens_sum(lsum);
    zacc = row_tokens_sum(zacc);
    float f16v[16], f32v[8];
#pragma unroll
    for (int k = 0; k < 16; ++k) f16v[k] = fold16f(acc[2 * k], acc[2 * k + 1]);
#pragma unroll
    for (int k = 0; k < 8; ++k) f32v[k] = fold32f(f16v[2 * k], f16v[2 * k + 1]);
    const int rw = (tid >> 4) & 3;
    if ((tid & 12) == 0) {
#pragma unroll
        for (int k = 0; k < 8; ++k) red[wave][32 * piece + kv_elem_of_reg(4 * k + rw)] = f32v[k];
        if (piece == 0) {
            lrow[wave][rw] = lsum;
            zrow[wave][rw] = zacc;
        }
    }
    __syncthreads();
    float* dst = part + (static_cast<size_t>(h) * splits + split) * KV_PART;
    if (tid < KV_D) {
        float zs = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
            for (int r = 0; r < 4; ++r) zs += zrow[w][r];
        dst[tid] = ((red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid])) - zs;
    } else if (tid == KV_D) {
        float ls = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
            for (int r = 0; r < 4; ++r) ls += lrow[w][r];
        dst[KV_D] = m;
        dst[KV_D + 1] = ls;
    }
}

// ---------------------------------------------------------------------------------------
// The streaming form for long contexts and batches, where the device is refilled many times and
// a workgroup that loads, waits, computes and leaves keeps too few bytes in flight.  Workgroup =
// (split of L tokens, head [, sequence]), L = 512 ... 2048.  The split is cut into chunks of 16
// tokens; wavefront w takes chunks w, w + 4, ... and walks them on its own: no workgroup barrier
// inside the loop, the loads of its next two chunks in flight while it computes one.  Each
// wavefront keeps a reference m (uniform over the wavefront; the running maximum, raised lazily)
// and rescales its sums when a chunk raises it:  acc <- acc * e^(m_old - m_new);  p_t = e^(score_t - m_new).
// At the end the four wavefronts merge in LDS with the same rule and (m, l, acc) of the split
// goes to the workspace for kv4_combine_kernel.
// ---------------------------------------------------------------------------------------
struct KvChunk {
    u32x4 kw, vw;
    uint32_t kp, vp;
    bool valid;
};

template <int QDT, bool BATCHED, bool QROT = false>
__global__ __launch_bounds__(KV_THREADS) void kv4_attn_stream_kernel(const void* __restrict__ q, int S, int S_max, int rep,
                                                                     int splits, float softmax_scale,
                                                                     const u32x4* __restrict__ k_codes,
                                                                     const uint32_t* __restrict__ k_params,
                                                                     const u32x4* __restrict__ v_codes,
                                                                     const uint32_t* __restrict__ v_params, int L,
                                                                     float* __restrict__ part, KvBatch batch)
{
    __shared__ float red[4][KV_D];
    __shared__ float wm[4], lrow[4][4], zrow[4][4];
    int split, h, hk;
    if (!kv_place(blockIdx.x, splits, rep, batch.H_kv, split, h, hk)) return;  // padding of the grid
    const int tid = threadIdx.x, lane = tid & 63, slot = lane >> 2, piece = tid & 3;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int t0 = split * L;
    if constexpr (BATCHED) {
        const int seq = blockIdx.z;
        S = batch.v[seq];
        if (t0 >= S) return;  // the whole workgroup: this sequence has fewer splits
        h += seq * batch.H_q;
        hk += seq * batch.H_kv;
    }
    const int t_end = min(S, t0 + L);
    const size_t head_base = static_cast<size_t>(hk) * S_max;
    // chunks of this wavefront that hold at least one cached token
    const int span = t_end - t0 - 16 * wave;
    const int nchunks = span > 0 ? (span + 63) >> 6 : 0;

    auto load = [&](int c, KvChunk& r) {  // chunk c of this wavefront: tokens t0 + 16 (4 c + wave) ...; past the end: the last token, weight 0
        const int t = t0 + 16 * (4 * c + wave) + slot;
        r.valid = t < t_end;
        const size_t at = head_base + (r.valid ? t : t_end - 1);
        // read once per call: non-temporal loads, as in kv4_attn_kernel
        r.kw = __builtin_nontemporal_load(k_codes + (at * 4 + piece));
        r.kp = __builtin_nontemporal_load(k_params + at);
        r.vw = __builtin_nontemporal_load(v_codes + (at * 4 + piece));
        r.vp = __builtin_nontemporal_load(v_params + at);
    };

    Raw8<QDT> qraw[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) qraw[d] = load8_raw<QDT>(q, static_cast<size_t>(h) * KV_D + 32 * piece + 8 * d);
    KvChunk cA, cB;
    load(0, cA);
    load(1, cB);

    float qr[32];
    const float qsum = kv_query_registers<QDT>(qraw, QROT, piece, qr);
    const float unit = kv_fp8_unit(), inv_unit = 1.0f / unit;
    const float scale_by_unit = softmax_scale * inv_unit, qsum_unit = qsum * unit;

    float acc[32];
#pragma unroll
    for (int r = 0; r < 32; ++r) acc[r] = 0.0f;
    float lsum = 0.0f, zacc = 0.0f;
    float m = -INFINITY;  // uniform over the wavefront
    int chunk = 0;

    auto step = [&](KvChunk& cur) {
        float dot[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t lo, hi;
            nibble_bytes(cur.kw[d], lo, hi);
            float fl[4], fh[4];
            bytes_to_floats(lo, fl);
            bytes_to_floats(hi, fh);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                dot[d] = fmaf(qr[8 * d + b], fl[b], dot[d]);
                dot[d] = fmaf(qr[8 * d + 4 + b], fh[b], dot[d]);
            }
        }
        const float s = half_bits_to_float(static_cast<uint16_t>(cur.kp & 0xffffu)) * scale_by_unit;
        const float z = static_cast<float>(static_cast<int>(cur.kp) >> 16);
        float sc = quad_sum(s * (((dot[0] + dot[1]) + (dot[2] + dot[3])) - z * qsum_unit));
        sc = cur.valid ? sc : -INFINITY;
        // The reference m only has to keep the exponentials in range, so it is raised lazily: when some score
        // of the chunk exceeds it by more than KV_LAZY (always on the first chunk, where m = -inf; every chunk
        // that is stepped holds a cached token, so the new maximum is finite).  Weights then stay below
        // e^KV_LAZY and the sums of a split far inside the binary32 range.
        if (__builtin_amdgcn_ballot_w64(sc > m + KV_LAZY) != 0) {  // uniform
            const float m_new = fmaxf(m, wave_max(sc));
            const float alpha = __expf(m - m_new);  // 0 on the first chunk
#pragma unroll
            for (int r = 0; r < 32; ++r) acc[r] *= alpha;
            lsum *= alpha;
            zacc *= alpha;
            m = m_new;
        }
        const float p = __expf(sc - m);
        const float w0 = p * half_bits_to_float(static_cast<uint16_t>(cur.vp & 0xffffu));
        const float w = w0 * inv_unit;
        lsum += p;
        zacc = fmaf(w0, static_cast<float>(static_cast<int>(cur.vp) >> 16), zacc);
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t lo, hi;
            nibble_bytes(cur.vw[d], lo, hi);
            float fl[4], fh[4];
            bytes_to_floats(lo, fl);
            bytes_to_floats(hi, fh);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                acc[8 * d + b] = fmaf(w, fl[b], acc[8 * d + b]);
                acc[8 * d + 4 + b] = fmaf(w, fh[b], acc[8 * d + 4 + b]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        load(chunk + 2, cur);  // refill with the chunk two steps ahead (past the end: a harmless repeat of the last token)
        __builtin_amdgcn_sched_barrier(0);
        ++chunk;
    };
    // steps counted up front and run in pairs: one loop body, one exit (four chunks in flight instead of
    // two: 130 registers and no gain)
    for (int i = 0; i < nchunks / 2; ++i) {
        step(cA);
        step(cB);
    }
    if (nchunks & 1) step(cA);

    // ---- the 16 tokens of a wavefront's chunks are summed as in kv4_attn_kernel; the four wavefronts
    // merge through LDS, each weighted by e^(its m - the largest m) ----
#pragma unroll
    for (int r = 0; r < 32; ++r) acc[r] = row_tokens_sum(acc[r]);
    lsum = row_tokens_sum(lsum);
    zacc = row_tokens_sum(zacc);
    float f16v[16], f32v[8];
#pragma unroll
    for (int k = 0; k < 16; ++k) f16v[k] = fold16f(acc[2 * k], acc[2 * k + 1]);
#pragma unroll
    for (int k = 0; k < 8; ++k) f32v[k] = fold32f(f16v[2 * k], f16v[2 * k + 1]);
    const int rw = (tid >> 4) & 3;
    if ((tid & 12) == 0) {
#pragma unroll
        for (int k = 0; k < 8; ++k) red[wave][32 * piece + kv_elem_of_reg(4 * k + rw)] = f32v[k];
        if (piece == 0) {
            lrow[wave][rw] = lsum;
            zrow[wave][rw] = zacc;
        }
    }
    if (lane == 0) wm[wave] = m;
    __syncthreads();
    float* dst = part + (static_cast<size_t>(h) * splits + split) * KV_PART;
    if (tid <= KV_D) {
        const float M = fmaxf(fmaxf(wm[0], wm[1]), fmaxf(wm[2], wm[3]));  // wavefront 0 always has a token: finite
        float total = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float e = __expf(wm[w] - M);  // 0 for a wavefront without tokens
            float v;
            if (tid < KV_D) v = red[w][tid] - ((zrow[w][0] + zrow[w][1]) + (zrow[w][2] + zrow[w][3]));
            else v = (lrow[w][0] + lrow[w][1]) + (lrow[w][2] + lrow[w][3]);
            total = fmaf(e, v, total);
        }
        if (tid < KV_D) dst[tid] = total;
        else {
            dst[KV_D] = M;
            dst[KV_D + 1] = total;
        }
    }
}

// The merge of the splits as a kernel of its own: one workgroup of `groups` x 128 threads per head (kv_merge_head).
// BATCHED: blockIdx.x = sequence * H_q + head; a sequence of length batch.v[z] has written only its
// first ceil(length / L) of the `splits` slots of each head.
template <bool OUT_F16, bool BATCHED>
__global__ __launch_bounds__(KV_CT) void kv4_combine_kernel(const float* __restrict__ part, int splits, int groups,
                                                            void* __restrict__ out, int L, KvBatch batch)
{
    __shared__ KvMergeLds lds;
    const int h = blockIdx.x;
    const float* src = part + static_cast<size_t>(h) * splits * KV_PART;
    if constexpr (BATCHED) {
        // the sequence's own number of splits and thread groups, so that the merge runs in the same order
        // as in a call for this sequence alone
        splits = (batch.v[h / batch.H_q] + L - 1) / L;
        groups = min(groups, (splits + 3) / 4);
    }
    kv_merge_head(src, splits, groups, out, OUT_F16, h, lds, groups * KV_D);
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
// Tokens per workgroup are chosen in launch_kv4_attn (measured: 64 never wins, the per-workgroup
// reduction then weighs too much); the "kv_tokens" option overrides.
size_t kv4_workspace_bytes(int H_q, int S)
{
    const int splits = (S + 63) / 64;  // the most any split length needs
    return static_cast<size_t>(H_q) * splits * KV_PART * sizeof(float);
}

// positions == nullptr: n_tokens tokens of one sequence from `pos` on; otherwise one token for each of
// n_tokens sequences of a pooled cache, at positions[i]
int launch_kv4_append(const void* x, rcp_dtype dt, int n_tokens, int H, int S_max, int pos, const int* positions, bool rotate,
                      float clip_ratio, void* codes, void* params, hipStream_t st)
{
    const int rows = n_tokens * H;
    if (rows == 0) return RCP_OK;
    const unsigned grid = static_cast<unsigned>((rows + 15) / 16);
    auto* c = static_cast<uint32_t*>(codes);
    auto* p = static_cast<uint32_t*>(params);
    KvBatch batch = {};
    const bool batched = positions != nullptr;
    if (batched)
        for (int i = 0; i < n_tokens; ++i) batch.v[i] = positions[i];
    auto launch = [&](auto kernel) { kernel<<<grid, 256, 0, st>>>(x, rows, H, S_max, pos, clip_ratio, c, p, batch); };
#define RCP_KV_APPEND(DT)                                                   \
    do {                                                                    \
        if (batched) {                                                      \
            if (rotate) launch(&kv4_append_kernel<DT, true, true>);         \
            else launch(&kv4_append_kernel<DT, false, true>);               \
        } else {                                                            \
            if (rotate) launch(&kv4_append_kernel<DT, true, false>);        \
            else launch(&kv4_append_kernel<DT, false, false>);              \
        }                                                                   \
    } while (0)
    if (dt == RCP_F32) RCP_KV_APPEND(RCP_F32);
    else if (dt == RCP_F16) RCP_KV_APPEND(RCP_F16);
    else RCP_KV_APPEND(RCP_BF16);
#undef RCP_KV_APPEND
    return check_launch("rcp_kv4_append");
}

// keys and values of the same n_tokens tokens in one launch
int launch_kv4_append_kv(const void* k, const void* v, rcp_dtype dt, int n_tokens, int H, int S_max, int pos, bool rotate_k,
                         float clip_ratio, void* k_codes, void* k_params, void* v_codes, void* v_params, hipStream_t st)
{
    const int rows = n_tokens * H;
    if (rows == 0) return RCP_OK;
    const dim3 grid(static_cast<unsigned>((rows + 15) / 16), 2u);
    auto launch = [&](auto kernel) {
        kernel<<<grid, 256, 0, st>>>(k, v, rows, H, S_max, pos, rotate_k ? 1 : 0, clip_ratio, static_cast<uint32_t*>(k_codes),
                                     static_cast<uint32_t*>(k_params), static_cast<uint32_t*>(v_codes), static_cast<uint32_t*>(v_params));
    };
    if (dt == RCP_F32) launch(&kv4_append_kv_kernel<RCP_F32>);
    else if (dt == RCP_F16) launch(&kv4_append_kv_kernel<RCP_F16>);
    else launch(&kv4_append_kv_kernel<RCP_BF16>);
    return check_launch("rcp_kv4_append_kv");
}

// lengths == nullptr: one sequence of S tokens; otherwise B sequences of a pooled cache, lengths[b] tokens each
// rotate_q (single sequence only): the order-128 Hadamard rotation of the query inside the attention kernel
int launch_kv4_attn(const void* q, rcp_dtype q_dt, int B, int H_q, int H_kv, int S_max, int S, const int* lengths,
                    const void* k_codes, const void* k_params, const void* v_codes, const void* v_params,
                    float softmax_scale, void* out, rcp_dtype out_dt, void* workspace, hipStream_t st, bool rotate_q)
{
    const bool batched = lengths != nullptr;
    const bool fused = !batched && rotate_q;
    KvBatch batch = {};
    long long total = S;
    if (batched) {
        S = 0;
        total = 0;
        for (int b = 0; b < B; ++b) {
            batch.v[b] = lengths[b];
            S = lengths[b] > S ? lengths[b] : S;  // the longest sequence sizes the grid
            total += lengths[b];
        }
        batch.H_q = H_q;
        batch.H_kv = H_kv;
    }
    // 128 tokens per workgroup below 2048 x 32 (token, head) pairs, 256 below 4096 x 32, then the streaming kernel: on
    // splits of 512 tokens up to 8192 x 32 pairs, of 1024 tokens beyond (sweeps at 32 heads, one to sixteen sequences:
    // 4096 tokens 9.2 -> 8.9 us, 8192 tokens 12.4 -> 11.5, 8 x 1024 tokens 12.5 -> 11.4 against 256 per workgroup)
    int L = options().kv_tokens;
    if (L == 0) L = total * H_q < 65536 ? 128 : total * H_q < 131072 ? KV_MAX_L : total * H_q <= 262144 ? 512 : KV_STREAM_L;
    const bool stream = L > KV_MAX_L;
    const int splits = (S + L - 1) / L;
    const int rep = H_q / H_kv;
    batch.H_q = H_q;
    batch.H_kv = H_kv;
    // one index per (split, query head), padded to whole groups of 8 * rep (see kv_place)
    const unsigned units = static_cast<unsigned>(splits) * static_cast<unsigned>(H_kv);
    const dim3 grid(8u * static_cast<unsigned>(rep) * ((units + 7u) / 8u), 1u, static_cast<unsigned>(batched ? B : 1));
    auto* kc = static_cast<const u32x4*>(k_codes);
    auto* vc = static_cast<const u32x4*>(v_codes);
    auto* kp = static_cast<const uint32_t*>(k_params);
    auto* vp = static_cast<const uint32_t*>(v_params);
    auto* part = static_cast<float*>(workspace);
    auto launch = [&](auto kernel) {
        kernel<<<grid, KV_THREADS, 0, st>>>(q, S, S_max, rep, splits, softmax_scale, kc, kp, vc, vp, part, batch);
    };
#define RCP_KV_LAUNCH(QDT, ITERS)                                        \
    do {                                                                 \
        if (batched) launch(&kv4_attn_kernel<QDT, ITERS, true>);         \
        else if (fused) launch(&kv4_attn_kernel<QDT, ITERS, false, true>); \
        else launch(&kv4_attn_kernel<QDT, ITERS, false>);                \
    } while (0)
    auto launch_stream = [&](auto kernel) {
        kernel<<<grid, KV_THREADS, 0, st>>>(q, S, S_max, rep, splits, softmax_scale, kc, kp, vc, vp, L, part, batch);
    };
#define RCP_KV_DISPATCH(QDT)                                                   \
    do {                                                                       \
        if (stream) {                                                          \
            if (batched) launch_stream(&kv4_attn_stream_kernel<QDT, true>);    \
            else if (fused) launch_stream(&kv4_attn_stream_kernel<QDT, false, true>); \
            else launch_stream(&kv4_attn_stream_kernel<QDT, false>);           \
        } else if (L == 64) RCP_KV_LAUNCH(QDT, 1);                             \
        else if (L == 128) RCP_KV_LAUNCH(QDT, 2);                              \
        else RCP_KV_LAUNCH(QDT, 4);                                            \
    } while (0)
    if (q_dt == RCP_F32) RCP_KV_DISPATCH(RCP_F32);
    else if (q_dt == RCP_F16) RCP_KV_DISPATCH(RCP_F16);
    else RCP_KV_DISPATCH(RCP_BF16);
#undef RCP_KV_DISPATCH
#undef RCP_KV_LAUNCH
    int rc = check_launch("rcp_kv4_attn_decode");
    if (rc != RCP_OK) return rc;
    int groups = (splits + 3) / 4;
    if (groups > KV_CT / KV_D) groups = KV_CT / KV_D;
    const unsigned cgrid = static_cast<unsigned>(H_q) * (batched ? B : 1);
    auto combine = [&](auto kernel) { kernel<<<cgrid, groups * KV_D, 0, st>>>(part, splits, groups, out, L, batch); };
    if (batched) {
        if (out_dt == RCP_F16) combine(&kv4_combine_kernel<true, true>);
        else combine(&kv4_combine_kernel<false, true>);
    } else {
        if (out_dt == RCP_F16) combine(&kv4_combine_kernel<true, false>);
        else combine(&kv4_combine_kernel<false, false>);
    }
    return check_launch("rcp_kv4_attn_decode(combine)");
}

}  // namespace rcp
