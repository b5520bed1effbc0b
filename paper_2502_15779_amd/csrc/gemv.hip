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
// give a triangular system that the epilogue solves exactly for the four rows:
//     D1 = f0, D3 = f0 + 2 f1, D7 = D3 + 4 f2, DF = D7 - 8 f3.
// Per 32 weights that is 1 AND (b0 & b1) + 9 ANDs + 12 dots, and no shift, no table
// look-up and no float conversion in the loop.  The LUT is touched only in the epilogue.
#include "rcp_internal.hpp"

namespace rcp {

constexpr int GEMV_THREADS = 256;
constexpr int GEMV_WAVES = GEMV_THREADS / 64;
constexpr int GEMV_UNROLL = 4;

__device__ __forceinline__ int dot8(uint32_t a, uint32_t b, int c)
{
    return __builtin_amdgcn_sdot8(static_cast<int>(a), static_cast<int>(b), c, false);
}

// All-reduce (sum) over aligned groups of LPG lanes of a wave64.
template <int LPG>
__device__ __forceinline__ int group_allreduce(int v)
{
    // rotations inside a row of 16 lanes: after ror 8, 4, 2, 1 every lane holds the row sum
    v += __builtin_amdgcn_update_dpp(0, v, 0x128, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x124, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x122, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x121, 0xf, 0xf, false);
    if constexpr (LPG >= 32) v += __shfl_xor(v, 16, 64);
    if constexpr (LPG >= 64) v += __shfl_xor(v, 32, 64);
    return v;
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

// Grid-stride over groups of four rows.  A wave works on 64/LPG row groups at a time; the
// LPG lanes of a slot walk the row group's 16-byte units (4 rows x 16 columns) with stride
// LPG, so each load instruction of a slot reads LPG*16 contiguous bytes.
// LDS holds the quantised activations of all tokens: token t at dword t*(K/8).
template <int LPG, int MT, bool OUT_F16>
__global__ __launch_bounds__(GEMV_THREADS) void gemv_kernel(const uint4* __restrict__ packed,
                                                            const uint2* __restrict__ codebook, int N, int K,
                                                            const uint4* __restrict__ xq,
                                                            const uint16_t* __restrict__ scale, int M,
                                                            void* __restrict__ out, int32_t* __restrict__ Pout)
{
    extern __shared__ uint4 smem4[];
    const int xdw = K / 8;  // activation dwords per token
    {
        const int n16 = M * (xdw / 4);
        for (int i = threadIdx.x; i < n16; i += GEMV_THREADS) smem4[i] = xq[i];
    }
    __syncthreads();
    const uint32_t* sx = reinterpret_cast<const uint32_t*>(smem4);
    const uint2* sx2 = reinterpret_cast<const uint2*>(smem4);

    const int lane = threadIdx.x & 63;
    // T[t] = sum_k q[t][k], the same for every row
    int T[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        int s = 0;
        if (t < M)
            for (int d = lane; d < xdw; d += 64) s = dot8(sx[t * xdw + d], 0x11111111u, s);
        T[t] = group_allreduce<64>(s);
    }

    constexpr int SLOTS = 64 / LPG;
    const int U = K / 16;
    const int G = N / 4;
    const int slot = lane / LPG, tl = lane % LPG;
    const int wave = blockIdx.x * GEMV_WAVES + (threadIdx.x >> 6);
    const int nwaves = gridDim.x * GEMV_WAVES;

    for (int gb = wave * SLOTS; gb < G; gb += nwaves * SLOTS) {
        const int g = gb + slot;
        const bool valid = g < G;
        const int gc = valid ? g : G - 1;  // keep every address in bounds; the result is dropped
        const uint4* __restrict__ row = packed + static_cast<size_t>(gc) * U;
        const int h = 4 * gc + (tl & 3);
        const uint2 lut_raw = codebook[h];  // needed by lanes tl < 4 only; issued early

        int acc[MT][3][4];
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int p = 0; p < 3; ++p)
#pragma unroll
                for (int m = 0; m < 4; ++m) acc[t][p][m] = 0;

        for (int u0 = tl; u0 < U; u0 += LPG * GEMV_UNROLL) {
            uint4 w[GEMV_UNROLL];
#pragma unroll
            for (int i = 0; i < GEMV_UNROLL; ++i) {
                const int u = u0 + i * LPG;
                w[i] = (u < U) ? row[u] : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < GEMV_UNROLL; ++i) {
                const int u = min(u0 + i * LPG, U - 1);
                uint32_t xa[MT], xb[MT];
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    const uint2 xv = (t < M) ? sx2[t * (xdw / 2) + u] : make_uint2(0, 0);
                    xa[t] = xv.x;
                    xb[t] = xv.y;
                }
                cell_update<MT>(w[i].x, w[i].y, xa, acc);
                cell_update<MT>(w[i].z, w[i].w, xb, acc);
            }
        }

#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int p = 0; p < 3; ++p)
#pragma unroll
                for (int m = 0; m < 4; ++m) acc[t][p][m] = group_allreduce<LPG>(acc[t][p][m]);

        if (valid && tl < 4) {
            const int r = tl;
            const float c0 = half_bits_to_float(static_cast<uint16_t>(lut_raw.x & 0xffffu));
            const float c1 = half_bits_to_float(static_cast<uint16_t>(lut_raw.x >> 16));
            const float c2 = half_bits_to_float(static_cast<uint16_t>(lut_raw.y & 0xffffu));
            const float c3 = half_bits_to_float(static_cast<uint16_t>(lut_raw.y >> 16));
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                if (t >= M) continue;
                int f[3];
#pragma unroll
                for (int p = 0; p < 3; ++p) {
                    const int D1 = acc[t][p][0], D3 = acc[t][p][1], D7 = acc[t][p][2], DF = acc[t][p][3];
                    f[p] = (r == 0) ? D1 : (r == 1) ? ((D3 - D1) >> 1) : (r == 2) ? ((D7 - D3) >> 2) : ((D7 - DF) >> 3);
                }
                const int P3 = f[2], P1 = f[0] - f[2], P2 = f[1] - f[2];
                const int P0 = T[t] - f[0] - f[1] + f[2];
                float o = c0 * static_cast<float>(P0);
                o = fmaf(c1, static_cast<float>(P1), o);
                o = fmaf(c2, static_cast<float>(P2), o);
                o = fmaf(c3, static_cast<float>(P3), o);
                o *= half_bits_to_float(scale[t]);
                const size_t oi = static_cast<size_t>(t) * N + h;
                if constexpr (OUT_F16) static_cast<__half*>(out)[oi] = __float2half_rn(o);
                else static_cast<float*>(out)[oi] = o;
                if (Pout != nullptr)
                    reinterpret_cast<int4*>(Pout)[oi] = make_int4(P0, P1, P2, P3);
            }
        }
    }
}

template <int LPG, int MT>
static int launch_typed(const void* packed, const void* codebook, int N, int K, const void* xq,
                        const void* scale, int M, void* out, rcp_dtype out_dt, int32_t* P, int blocks,
                        size_t lds, hipStream_t st)
{
    auto* pk = static_cast<const uint4*>(packed);
    auto* cb = static_cast<const uint2*>(codebook);
    auto* xv = static_cast<const uint4*>(xq);
    auto* sc = static_cast<const uint16_t*>(scale);
    if (out_dt == RCP_F16) {
        if (lds > 65536) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemv_kernel<LPG, MT, true>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
            if (e != hipSuccess) return fail(RCP_ERR_HIP, "rcp_w2a4_gemv: LDS opt-in failed: %s", hipGetErrorString(e));
        }
        gemv_kernel<LPG, MT, true><<<blocks, GEMV_THREADS, lds, st>>>(pk, cb, N, K, xv, sc, M, out, P);
    } else {
        if (lds > 65536) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemv_kernel<LPG, MT, false>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
            if (e != hipSuccess) return fail(RCP_ERR_HIP, "rcp_w2a4_gemv: LDS opt-in failed: %s", hipGetErrorString(e));
        }
        gemv_kernel<LPG, MT, false><<<blocks, GEMV_THREADS, lds, st>>>(pk, cb, N, K, xv, sc, M, out, P);
    }
    return check_launch("rcp_w2a4_gemv");
}

template <int LPG>
static int launch_lpg(const void* packed, const void* codebook, int N, int K, const void* xq,
                      const void* scale, int M, void* out, rcp_dtype out_dt, int32_t* P, int blocks,
                      size_t lds, hipStream_t st)
{
#define RCP_GO(MT) return launch_typed<LPG, MT>(packed, codebook, N, K, xq, scale, M, out, out_dt, P, blocks, lds, st)
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
    const size_t lds = static_cast<size_t>(M) * K / 2;
    if (lds > 160 * 1024 - 1024)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_w2a4_gemv: M*K/2 = %zu bytes of activations exceed the LDS budget", lds);
    const Options& opt = options();
    const int G = N / 4, U = K / 16;
    const int cus = num_compute_units();

    // Lanes per row group: fewer lanes mean a cheaper cross-lane reduction per row, more
    // lanes mean more waves for a small matrix.  Aim at >= 8 waves per compute unit.
    int lpg = opt.gemv_lpg;
    if (lpg == 0) {
        lpg = 16;
        while (lpg < 64 && (static_cast<long long>(G) * lpg / 64 < 8LL * cus || U / lpg > 64)) lpg *= 2;
        while (lpg > 16 && U < lpg) lpg /= 2;
    }
    const int slots = 64 / lpg;
    const int waves_needed = (G + slots - 1) / slots;
    int blocks = opt.gemv_blocks;
    if (blocks == 0) {
        const int full = (waves_needed + GEMV_WAVES - 1) / GEMV_WAVES;
        const int cap = cus * 8;  // 8 workgroups of 4 waves per compute unit
        blocks = full < cap ? full : cap;
    }
    if (blocks < 1) blocks = 1;
    switch (lpg) {
        case 16: return launch_lpg<16>(packed, codebook, N, K, xq, scale, M, out, out_dt, P, blocks, lds, st);
        case 32: return launch_lpg<32>(packed, codebook, N, K, xq, scale, M, out, out_dt, P, blocks, lds, st);
        default: return launch_lpg<64>(packed, codebook, N, K, xq, scale, M, out, out_dt, P, blocks, lds, st);
    }
}

}  // namespace rcp
