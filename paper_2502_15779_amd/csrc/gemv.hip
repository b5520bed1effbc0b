// Non-uniform W2A4 GEMV for CDNA4 (Section 4.4 of the paper states the problem; the kernel
// design is this library's own).
//
// The product is evaluated through exact integer per-level partial sums
//     P[h][l] = sum_{k : idx[h][k] = l} q[k],   O[h] = S * sum_l LUT[h][l] * P[h][l],
// and the partial sums through the Walsh basis of the 2-bit index idx = b0 + 2*b1:
//     F0 = sum b0*q,  F1 = sum b1*q,  F3 = sum (b0 & b1)*q,  T = sum q
//     P3 = F3,  P1 = F0 - F3,  P2 = F1 - F3,  P0 = T - F0 - F1 + F3.
// The packed layout keeps b0 and b1 as bit planes with the bits of FOUR rows in each
// nibble, so one 32-bit plane word and the packed int4 activation word go straight into
// v_dot8_i32_i4: the nibble (b[r0], b[r1], b[r2], b[r3]) read as a signed int4 is
// b[r0] + 2 b[r1] + 4 b[r2] - 8 b[r3].  Four dot products with the nibble masks 1, 3, 7, F
// give a triangular system that is solved exactly for the four rows:
//     D1 = f0, D3 = f0 + 2 f1, D7 = D3 + 4 f2, DF = D7 - 8 f3.
// Per 32 weights that is 1 AND (b0 & b1) + 9 ANDs + 12 dots, and no shift, no table
// look-up and no float conversion in the loop.  The LUT is touched only in the epilogue.
//
// Work decomposition.  A group of four rows is K/16 units of 16 bytes (4 rows x 16
// columns).  LG = 64*WS lanes (WS = 1, 2 or 4 wavefronts of a 256-thread workgroup) share
// one row group: lane t takes units t, t + LG, t + 2 LG, ...  so every load instruction of
// a wavefront reads 1 KiB of consecutive bytes.  The kernel is latency bound at LLaMA
// sizes (a 4096 x 4096 matrix is 4 MiB, less than what must be in flight to fill HBM), so
// a lane issues the loads of its first row group before anything else, and the loads of
// the next row group before it reduces the current one.
#include "rcp_internal.hpp"

namespace rcp {

constexpr int GEMV_THREADS = 256;
constexpr int GEMV_WAVES = GEMV_THREADS / 64;
constexpr int GEMV_UNROLL = 4;  // 16-byte loads in flight per lane and buffer

__device__ __forceinline__ int dot8(uint32_t a, uint32_t b, int c)
{
    return __builtin_amdgcn_sdot8(static_cast<int>(a), static_cast<int>(b), c, false);
}

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
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    return v;
}

// Sum twelve per-lane values over the 64 lanes of a wavefront, scattering the results:
// afterwards every lane of 16-lane row rho holds in t[k] the total of g[4k + perm(rho)],
// perm = (0, 2, 1, 3).  Halving steps use the gfx950 lane-swap instructions: swapping the
// upper half of one register with the lower half of another and adding folds two
// registers into one.
__device__ __forceinline__ void reduce_scatter12(const int (&g)[12], int (&t)[3])
{
    int s[6];
#pragma unroll
    for (int i = 0; i < 6; ++i) {
        // lanes 0..31 <- g[2i] (own + lane^32), lanes 32..63 <- g[2i+1]
        auto r = __builtin_amdgcn_permlane32_swap(static_cast<unsigned>(g[2 * i]), static_cast<unsigned>(g[2 * i + 1]), false, false);
        s[i] = static_cast<int>(r[0]) + static_cast<int>(r[1]);
    }
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        // rows 0 and 2 <- s[2k] (own + row^1), rows 1 and 3 <- s[2k+1]
        auto r = __builtin_amdgcn_permlane16_swap(static_cast<unsigned>(s[2 * k]), static_cast<unsigned>(s[2 * k + 1]), false, false);
        t[k] = row_sum16(static_cast<int>(r[0]) + static_cast<int>(r[1]));
    }
}

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

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// LDS: quantised activations, token t at dword t*(K/8), padded so that the reads of a
// lane whose unit lies beyond K stay inside the allocation (their weights are zero);
// then 4*MT ints of per-wavefront sums of q; then, for WS > 1, the cross-wavefront
// reduction slots int[2][4 waves][4 rows][3*MT].
template <int MT>
__host__ __device__ constexpr int gemv_x_bytes(int K, int M, int lanes)
{
    const int U = K / 16;
    const int span = lanes * GEMV_UNROLL;
    const int padded_units = ((U + span - 1) / span) * span;
    return ((M - 1) * U + padded_units) * 8;
}

// Weight loads go through a buffer resource that covers exactly one row group, so a unit
// beyond K (or a whole row group beyond N) reads as zero without a branch in the loop.
template <int WS, int MT, bool OUT_F16>
__global__ __launch_bounds__(GEMV_THREADS) void gemv_kernel(const uint4* __restrict__ packed,
                                                            const uint2* __restrict__ codebook, int N, int K,
                                                            const uint4* __restrict__ xq,
                                                            const uint16_t* __restrict__ scale, int M,
                                                            void* __restrict__ out, int32_t* __restrict__ Pout, int dbg)
{
    extern __shared__ uint4 smem4[];
    constexpr int SLOTS = GEMV_WAVES / WS;  // row groups a workgroup works on at a time
    constexpr int LG = 64 * WS;             // lanes per row group
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int slot = wave / WS, wsub = wave % WS;
    const int tg = wsub * 64 + lane;  // this lane's position among the LG lanes
    const int U = K / 16, G = N / 4;
    const int xdw = K / 8;  // activation dwords per token
    const int nbatch = (G + SLOTS - 1) / SLOTS;
    const int nchunk = (U + LG * GEMV_UNROLL - 1) / (LG * GEMV_UNROLL);
    const int rho = lane >> 4;
    const int my_row = ((rho & 1) << 1) | (rho >> 1);  // perm(rho): the row this lane's sums belong to

    auto row_group = [&](int g) {
        const bool ok = g < G;
        return __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint4*>(packed + static_cast<size_t>(ok && dbg != 2 ? g : (g & 7)) * U), 0, ok ? U * 16 : 0, 0x00020000);
    };
    auto load_chunk = [&](__amdgpu_buffer_rsrc_t rg, int ch, u32x4 (&w)[GEMV_UNROLL]) {
        const int voff = (tg + ch * GEMV_UNROLL * LG) * 16;
#pragma unroll
        for (int i = 0; i < GEMV_UNROLL; ++i) w[i] = __builtin_amdgcn_raw_buffer_load_b128(rg, voff, i * LG * 16, 0);
    };

    // Memory returns loads in issue order, so the small ones the prologue needs go first:
    // the activations (first 4 KiB per token straight into registers) and the scales; then
    // the weight loads of the first row group, before any other work.
    const int per_token = xdw / 4;  // 16-byte pieces of one token's activations
    u32x4 xfirst[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint4*>(xq + static_cast<size_t>(t < M ? t : 0) * per_token), 0, t < M ? per_token * 16 : 0, 0x00020000);
        xfirst[t] = __builtin_amdgcn_raw_buffer_load_b128(xr, static_cast<int>(threadIdx.x) * 16, 0, 0);
    }
    float sc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) sc[t] = half_bits_to_float(scale[t < M ? t : 0]);

    int b = blockIdx.x;
    u32x4 wnext[GEMV_UNROLL];
    __amdgpu_buffer_rsrc_t rg_cur = row_group(b * SLOTS + slot);
    load_chunk(rg_cur, 0, wnext);
    uint2 lut_next = codebook[4 * min(b * SLOTS + slot, G - 1) + my_row];

    // stage the activations and sum them: T[t] = sum_k q[t][k], the same for every row
    const int x_bytes = gemv_x_bytes<MT>(K, M, LG);
    int* tsum = reinterpret_cast<int*>(reinterpret_cast<char*>(smem4) + x_bytes);  // [GEMV_WAVES][MT]
    int* red = tsum + GEMV_WAVES * MT;
    {
        u32x4* sx4 = reinterpret_cast<u32x4*>(smem4);
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            int s = 0;
            if (t < M) {
                // a piece beyond the token's end was read as zero and is not stored
                if (static_cast<int>(threadIdx.x) < per_token) sx4[t * per_token + threadIdx.x] = xfirst[t];
                s = dot8(xfirst[t].x, 0x11111111u, s);
                s = dot8(xfirst[t].y, 0x11111111u, s);
                s = dot8(xfirst[t].z, 0x11111111u, s);
                s = dot8(xfirst[t].w, 0x11111111u, s);
                for (int i = threadIdx.x + GEMV_THREADS; i < per_token; i += GEMV_THREADS) {  // K > 8192 only
                    const uint4 v = xq[t * per_token + i];
                    smem4[t * per_token + i] = v;
                    s = dot8(v.x, 0x11111111u, s);
                    s = dot8(v.y, 0x11111111u, s);
                    s = dot8(v.z, 0x11111111u, s);
                    s = dot8(v.w, 0x11111111u, s);
                }
            }
            s = wave_sum(s);
            if (lane == 0) tsum[wave * MT + t] = s;
        }
    }
    __syncthreads();
    const uint2* sx2 = reinterpret_cast<const uint2*>(smem4);
    int T[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) T[t] = tsum[t] + tsum[MT + t] + tsum[2 * MT + t] + tsum[3 * MT + t];

    int parity = 0;
    for (; b < nbatch; b += gridDim.x) {
        const int g = b * SLOTS + slot;
        const int gn = (b + static_cast<int>(gridDim.x)) * SLOTS + slot;  // >= G past the end: reads as zero
        const __amdgpu_buffer_rsrc_t rg_next = row_group(gn);
        const uint2 lut_raw = lut_next;
        int acc[MT][3][4];
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int p = 0; p < 3; ++p)
#pragma unroll
                for (int m = 0; m < 4; ++m) acc[t][p][m] = 0;

        for (int ch = 0; ch < nchunk; ++ch) {
            u32x4 w[GEMV_UNROLL];
#pragma unroll
            for (int i = 0; i < GEMV_UNROLL; ++i) w[i] = wnext[i];
            // keep the memory pipe busy: next chunk of this row group, else the first chunk
            // of this workgroup's next row group
            const bool last = ch + 1 == nchunk;
            load_chunk(last ? rg_next : rg_cur, last ? 0 : ch + 1, wnext);
            const uint2* xrow = sx2 + tg + ch * GEMV_UNROLL * LG;
#pragma unroll
            for (int i = 0; i < GEMV_UNROLL; ++i) {
                uint32_t xa[MT], xb[MT];
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    const uint2 xv = xrow[(MT == 1 ? 0 : min(t, M - 1)) * (xdw / 2) + i * LG];
                    xa[t] = xv.x;
                    xb[t] = xv.y;
                }
                if (dbg == 1) {
                    acc[0][0][0] ^= w[i].x ^ w[i].y ^ w[i].z ^ w[i].w ^ xa[0] ^ xb[0];
                    continue;
                }
                cell_update<MT>(w[i].x, w[i].y, xa, acc);
                cell_update<MT>(w[i].z, w[i].w, xb, acc);
            }
        }
        rg_cur = rg_next;
        lut_next = codebook[4 * min(gn, G - 1) + my_row];

        // The triangular solve is linear, so it is applied per lane before the reduction
        // (the power-of-two divisions wait until the sums are complete):
        // gsum[p] of the lanes of row rho = 2^r * f_r of plane p, r = perm(rho).
        int gsum[MT][3];
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            int g12[12];
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                g12[4 * p + 0] = acc[t][p][0];
                g12[4 * p + 1] = acc[t][p][1] - acc[t][p][0];
                g12[4 * p + 2] = acc[t][p][2] - acc[t][p][1];
                g12[4 * p + 3] = acc[t][p][2] - acc[t][p][3];
            }
            reduce_scatter12(g12, gsum[t]);
        }

        if constexpr (WS > 1) {
            // one lane per 16-lane row publishes its wavefront's sums; the first wavefront
            // of the slot adds the others.  Two buffers alternate so that one barrier per
            // row group is enough.
            int* mine = red + ((parity * GEMV_WAVES + wave) * 4 + rho) * (3 * MT);
            if ((lane & 15) == 0) {
#pragma unroll
                for (int t = 0; t < MT; ++t)
#pragma unroll
                    for (int p = 0; p < 3; ++p) mine[3 * t + p] = gsum[t][p];
            }
            __syncthreads();
            if (wsub == 0 && (lane & 15) == 0) {
#pragma unroll
                for (int ws = 1; ws < WS; ++ws) {
                    const int* other = red + ((parity * GEMV_WAVES + wave + ws) * 4 + rho) * (3 * MT);
#pragma unroll
                    for (int t = 0; t < MT; ++t)
#pragma unroll
                        for (int p = 0; p < 3; ++p) gsum[t][p] += other[3 * t + p];
                }
            }
            parity ^= 1;
        }

        if (g < G && wsub == 0 && (lane & 15) == 0) {
            const int r = my_row;
            const int h = 4 * g + r;
            const float c0 = half_bits_to_float(static_cast<uint16_t>(lut_raw.x & 0xffffu));
            const float c1 = half_bits_to_float(static_cast<uint16_t>(lut_raw.x >> 16));
            const float c2 = half_bits_to_float(static_cast<uint16_t>(lut_raw.y & 0xffffu));
            const float c3 = half_bits_to_float(static_cast<uint16_t>(lut_raw.y >> 16));
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                if (t >= M) continue;
                const int F0 = gsum[t][0] >> r, F1 = gsum[t][1] >> r, F3 = gsum[t][2] >> r;
                const int P3 = F3, P1 = F0 - F3, P2 = F1 - F3;
                const int P0 = T[t] - F0 - F1 + F3;
                float o = c0 * static_cast<float>(P0);
                o = fmaf(c1, static_cast<float>(P1), o);
                o = fmaf(c2, static_cast<float>(P2), o);
                o = fmaf(c3, static_cast<float>(P3), o);
                o *= sc[t];
                const size_t oi = static_cast<size_t>(t) * N + h;
                if constexpr (OUT_F16) static_cast<__half*>(out)[oi] = __float2half_rn(o);
                else static_cast<float*>(out)[oi] = o;
                if (Pout != nullptr)
                    reinterpret_cast<int4*>(Pout)[oi] = make_int4(P0, P1, P2, P3);
            }
        }
    }
}

template <int WS, int MT, bool OUT_F16>
static int launch_one(const void* packed, const void* codebook, int N, int K, const void* xq,
                      const void* scale, int M, void* out, int32_t* P, int blocks, size_t lds, hipStream_t st)
{
    if (lds > 65536) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemv_kernel<WS, MT, OUT_F16>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e != hipSuccess) return fail(RCP_ERR_HIP, "rcp_w2a4_gemv: LDS opt-in failed: %s", hipGetErrorString(e));
    }
    gemv_kernel<WS, MT, OUT_F16><<<blocks, GEMV_THREADS, lds, st>>>(
        static_cast<const uint4*>(packed), static_cast<const uint2*>(codebook), N, K, static_cast<const uint4*>(xq),
        static_cast<const uint16_t*>(scale), M, out, P, options().gemv_variant);
    return check_launch("rcp_w2a4_gemv");
}

template <int WS>
static int launch_ws(const void* packed, const void* codebook, int N, int K, const void* xq,
                     const void* scale, int M, void* out, rcp_dtype out_dt, int32_t* P, int blocks,
                     size_t lds_x, hipStream_t st)
{
#define RCP_GO(MT)                                                                                              \
    do {                                                                                                        \
        const size_t lds = gemv_x_bytes<MT>(K, M, 64 * WS) + GEMV_WAVES * MT * sizeof(int) +                  \
                           (WS > 1 ? 2 * GEMV_WAVES * 4 * 3 * MT * sizeof(int) : 0);                          \
        return out_dt == RCP_F16                                                                                \
                   ? launch_one<WS, MT, true>(packed, codebook, N, K, xq, scale, M, out, P, blocks, lds, st)   \
                   : launch_one<WS, MT, false>(packed, codebook, N, K, xq, scale, M, out, P, blocks, lds, st); \
    } while (0)
    if (M == 1) RCP_GO(1);
    if (M == 2) RCP_GO(2);
    if (M <= 4) RCP_GO(4);
    if (M <= 8) RCP_GO(8);
    RCP_GO(16);
#undef RCP_GO
}

int launch_gemv(const void* packed, const void* codebook, int N, int K, const void* xq,
                const void* scale, int M, void* out, rcp_dtype out_dt, int32_t* P, hipStream_t st)
{
    const size_t lds_x = static_cast<size_t>(M) * K / 2;
    if (lds_x > 150 * 1024)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_w2a4_gemv: M*K/2 = %zu bytes of activations exceed the LDS budget", lds_x);
    const Options& opt = options();
    const int G = N / 4, U = K / 16;
    const int cus = num_compute_units();

    // Wavefronts per row group.  More of them put a small matrix on more wavefronts and cut
    // the number of loads a lane has to issue one after the other; fewer save the
    // cross-wavefront reduction.  Prefer the smallest split that (a) lets a lane cover its
    // share of a row group with one batch of loads and (b) gives every SIMD a few wavefronts.
    int ws = opt.gemv_lanes / 64;
    if (ws == 0) {
        ws = 1;
        while (ws < 4 && (U > 64 * ws * GEMV_UNROLL || static_cast<long long>(G) * ws < 8LL * cus)) ws *= 2;
        while (ws > 1 && U <= 32 * ws) ws /= 2;
    }
    const int slots = GEMV_WAVES / ws;
    const int nbatch = (G + slots - 1) / slots;
    int blocks = opt.gemv_blocks;
    if (blocks == 0) {
        const int cap = cus * 8;
        blocks = nbatch < cap ? nbatch : cap;
    }
    if (blocks > nbatch) blocks = nbatch;
    if (blocks < 1) blocks = 1;
    switch (ws) {
        case 1: return launch_ws<1>(packed, codebook, N, K, xq, scale, M, out, out_dt, P, blocks, lds_x, st);
        case 2: return launch_ws<2>(packed, codebook, N, K, xq, scale, M, out, out_dt, P, blocks, lds_x, st);
        default: return launch_ws<4>(packed, codebook, N, K, xq, scale, M, out, out_dt, P, blocks, lds_x, st);
    }
}

}  // namespace rcp
