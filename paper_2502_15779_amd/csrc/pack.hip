// Offline export: LDP grid -> thresholds and LUT, 2-bit indices -> bit-plane cells
// (Section 4.3 "Partition", LUT equation of Section 4.4; layout in include/rcp.h).
#include "rcp_internal.hpp"

namespace rcp {

// IEEE double -> binary16 bit pattern, one rounding to nearest even, done on the
// integer image of the double (no intermediate binary32 step, which would round twice).
__device__ static uint16_t double_to_half_bits(double v)
{
    const uint64_t bits = static_cast<uint64_t>(__double_as_longlong(v));
    const uint16_t sign = static_cast<uint16_t>((bits >> 48) & 0x8000u);
    const int biased = static_cast<int>((bits >> 52) & 0x7ff);
    const uint64_t frac = bits & 0x000fffffffffffffull;
    if (biased == 0x7ff) return static_cast<uint16_t>(sign | (frac ? 0x7e00u : 0x7c00u));
    if (biased == 0) return sign;  // zero or a double subnormal: far below half's range
    const int e = biased - 1023;
    if (e > 15) return static_cast<uint16_t>(sign | 0x7c00u);
    const uint64_t sig = frac | (1ull << 52);  // 53-bit significand, value = sig * 2^(e-52)
    int shift;                                 // low bits of sig that do not fit
    uint32_t base;                             // result before adding the kept bits
    if (e >= -14) {
        shift = 42;
        base = static_cast<uint32_t>(e + 14) << 10;  // exponent field minus one: the hidden bit adds 1<<10
    } else {
        shift = 42 + (-14 - e);
        base = 0;
        if (shift > 54) return sign;  // below half of the smallest subnormal
    }
    const uint64_t kept = sig >> shift;
    const uint64_t rem = sig & ((1ull << shift) - 1);
    const uint64_t halfway = 1ull << (shift - 1);
    uint32_t r = base + static_cast<uint32_t>(kept);
    if (rem > halfway || (rem == halfway && (kept & 1))) r += 1;  // a carry walks into the exponent
    return static_cast<uint16_t>(sign | r);
}

struct LdpGrid {
    float T[3];
    uint16_t L[4];
};

// Thresholds and LUT of one output row, in double, in the order written in rcp.h,
// with no multiply-add fusion so that any IEEE implementation gives the same bits.
__device__ static LdpGrid ldp_grid(float lo_f, float hi_f, float p1_f, float p2_f, float p3_f)
{
    const double lo = lo_f, hi = hi_f, p1 = p1_f, p2 = p2_f, p3 = p3_f;
    const double range = __dsub_rn(hi, lo);
    const double t1 = __ddiv_rn(p1, 2.0);
    const double t2 = __dadd_rn(t1, __ddiv_rn(__dadd_rn(p1, p2), 2.0));
    const double t3 = __dadd_rn(t2, __ddiv_rn(__dadd_rn(p2, p3), 2.0));
    const double w1 = __ddiv_rn(__dadd_rn(t1, t2), 2.0);
    const double w2 = __ddiv_rn(__dadd_rn(t2, t3), 2.0);
    LdpGrid g;
    g.T[0] = __double2float_rn(__dadd_rn(lo, __dmul_rn(range, t1)));
    g.T[1] = __double2float_rn(__dadd_rn(lo, __dmul_rn(range, t2)));
    g.T[2] = __double2float_rn(__dadd_rn(lo, __dmul_rn(range, t3)));
    g.L[0] = double_to_half_bits(lo);
    g.L[1] = double_to_half_bits(__dadd_rn(lo, __dmul_rn(range, w1)));
    g.L[2] = double_to_half_bits(__dadd_rn(lo, __dmul_rn(range, w2)));
    g.L[3] = double_to_half_bits(hi);
    return g;
}

// One workgroup packs one group of four rows for a span of cells; one thread per cell
// (4 rows x 8 columns -> two 32-bit bit planes).  Thresholds of the four rows sit in LDS.
constexpr int PACK_THREADS = 256;

template <int DT>
__global__ __launch_bounds__(PACK_THREADS) void pack_kernel(const void* __restrict__ W, int N, int K,
                                                            const float* __restrict__ clip_lo,
                                                            const float* __restrict__ clip_hi,
                                                            const float* __restrict__ part,
                                                            uint2* __restrict__ packed,
                                                            uint16_t* __restrict__ codebook)
{
    __shared__ float sT[4][3];
    const int g = blockIdx.y;
    const int cells = K / 8;
    if (threadIdx.x < 4) {
        const int h = 4 * g + threadIdx.x;
        LdpGrid grid = ldp_grid(clip_lo[h], clip_hi[h], part[3 * h], part[3 * h + 1], part[3 * h + 2]);
        sT[threadIdx.x][0] = grid.T[0];
        sT[threadIdx.x][1] = grid.T[1];
        sT[threadIdx.x][2] = grid.T[2];
        if (blockIdx.x == 0) {
            uint2 lut;
            lut.x = static_cast<uint32_t>(grid.L[0]) | (static_cast<uint32_t>(grid.L[1]) << 16);
            lut.y = static_cast<uint32_t>(grid.L[2]) | (static_cast<uint32_t>(grid.L[3]) << 16);
            reinterpret_cast<uint2*>(codebook)[h] = lut;
        }
    }
    __syncthreads();
    const int o = blockIdx.x * PACK_THREADS + threadIdx.x;
    if (o >= cells) return;
    uint32_t b0 = 0, b1 = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        float w[8];
        load8_as_float<DT>(W, static_cast<size_t>(4 * g + r) * K + static_cast<size_t>(o) * 8, w);
        const float T1 = sT[r][0], T2 = sT[r][1], T3 = sT[r][2];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t idx = static_cast<uint32_t>(w[j] >= T1) + static_cast<uint32_t>(w[j] >= T2) +
                                 static_cast<uint32_t>(w[j] >= T3);
            b0 |= (idx & 1u) << (4 * j + r);
            b1 |= (idx >> 1) << (4 * j + r);
        }
    }
    packed[static_cast<size_t>(g) * cells + o] = make_uint2(b0, b1);
}

// One thread per cell: 32 index bytes out.
__global__ __launch_bounds__(PACK_THREADS) void unpack_kernel(const uint2* __restrict__ packed, int N, int K,
                                                              uint8_t* __restrict__ idx)
{
    const int g = blockIdx.y;
    const int cells = K / 8;
    const int o = blockIdx.x * PACK_THREADS + threadIdx.x;
    if (o >= cells) return;
    const uint2 c = packed[static_cast<size_t>(g) * cells + o];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        uint32_t lo4 = 0, hi4 = 0;  // eight index bytes of row r
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t v = ((c.x >> (4 * j + r)) & 1u) | (((c.y >> (4 * j + r)) & 1u) << 1);
            if (j < 4) lo4 |= v << (8 * j);
            else hi4 |= v << (8 * (j - 4));
        }
        *reinterpret_cast<uint2*>(idx + static_cast<size_t>(4 * g + r) * K + static_cast<size_t>(o) * 8) =
            make_uint2(lo4, hi4);
    }
}

int launch_pack(const void* W, rcp_dtype dt, int N, int K, const float* lo, const float* hi,
                const float* part, void* packed, void* codebook, hipStream_t st)
{
    const int cells = K / 8;
    dim3 grid((cells + PACK_THREADS - 1) / PACK_THREADS, N / 4);
    if (N / 4 > 65535) return fail(RCP_ERR_SHAPE, "rcp_pack_weights: N=%d exceeds 262140", N);
    auto* pk = static_cast<uint2*>(packed);
    auto* cb = static_cast<uint16_t*>(codebook);
    switch (dt) {
        case RCP_F16: pack_kernel<RCP_F16><<<grid, PACK_THREADS, 0, st>>>(W, N, K, lo, hi, part, pk, cb); break;
        case RCP_F32: pack_kernel<RCP_F32><<<grid, PACK_THREADS, 0, st>>>(W, N, K, lo, hi, part, pk, cb); break;
        default: pack_kernel<RCP_BF16><<<grid, PACK_THREADS, 0, st>>>(W, N, K, lo, hi, part, pk, cb); break;
    }
    return check_launch("rcp_pack_weights");
}

int launch_unpack(const void* packed, int N, int K, uint8_t* idx, hipStream_t st)
{
    if (N / 4 > 65535) return fail(RCP_ERR_SHAPE, "rcp_unpack_indices: N=%d exceeds 262140", N);
    dim3 grid((K / 8 + PACK_THREADS - 1) / PACK_THREADS, N / 4);
    unpack_kernel<<<grid, PACK_THREADS, 0, st>>>(static_cast<const uint2*>(packed), N, K, idx);
    return check_launch("rcp_unpack_indices");
}

// ---------------------------------------------------------------------------------------------
// Group-wise quantisation units (128 input channels per unit; Appendix table of quantisation
// configurations, LUT shape H x N*4 of Section 4.4).  Same cells, but the 16-byte units of a
// row group are stored lane-major (layout in include/rcp.h) so that lane g%32 of the GEMV
// finds the eight units of "its" group at a fixed stride.
// ---------------------------------------------------------------------------------------------
constexpr int GROUP = 128;

// unit position of unit i (0..7) of group g inside its row group
__device__ __forceinline__ int grouped_unit_pos(int g, int i, int NG)
{
    const int round = g >> 5;
    const int R = min(32, NG - 32 * round);
    return 256 * round + i * R + (g & 31);
}

// One workgroup: one group of four rows x 16 quantisation groups (256 cells); the first 64
// threads derive the (row, group) grids, every thread then packs one cell.
template <int DT>
__global__ __launch_bounds__(PACK_THREADS) void pack_grouped_kernel(const void* __restrict__ W, int N, int K,
                                                                    const float* __restrict__ clip_lo,
                                                                    const float* __restrict__ clip_hi,
                                                                    const float* __restrict__ part,
                                                                    uint2* __restrict__ packed,
                                                                    uint16_t* __restrict__ codebook)
{
    __shared__ float sT[16][4][3];
    const int g4 = blockIdx.y;
    const int NG = K / GROUP;
    const int cells = K / 8;
    if (threadIdx.x < 64) {
        const int r = threadIdx.x & 3, gl = threadIdx.x >> 2;
        const int g = blockIdx.x * 16 + gl;
        if (g < NG) {
            const int h = 4 * g4 + r;
            const size_t q = static_cast<size_t>(h) * NG + g;
            LdpGrid grid = ldp_grid(clip_lo[q], clip_hi[q], part[3 * q], part[3 * q + 1], part[3 * q + 2]);
            sT[gl][r][0] = grid.T[0];
            sT[gl][r][1] = grid.T[1];
            sT[gl][r][2] = grid.T[2];
            uint2 lut;
            lut.x = static_cast<uint32_t>(grid.L[0]) | (static_cast<uint32_t>(grid.L[1]) << 16);
            lut.y = static_cast<uint32_t>(grid.L[2]) | (static_cast<uint32_t>(grid.L[3]) << 16);
            // grouped LUT layout [N/4][NG][4 rows][4 levels]
            reinterpret_cast<uint2*>(codebook)[(static_cast<size_t>(g4) * NG + g) * 4 + r] = lut;
        }
    }
    __syncthreads();
    const int o = blockIdx.x * PACK_THREADS + threadIdx.x;  // logical cell: columns 8o .. 8o+7
    if (o >= cells) return;
    const int gl = threadIdx.x >> 4;  // 16 cells per quantisation group
    uint32_t b0 = 0, b1 = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        float w[8];
        load8_as_float<DT>(W, static_cast<size_t>(4 * g4 + r) * K + static_cast<size_t>(o) * 8, w);
        const float T1 = sT[gl][r][0], T2 = sT[gl][r][1], T3 = sT[gl][r][2];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t idx = static_cast<uint32_t>(w[j] >= T1) + static_cast<uint32_t>(w[j] >= T2) +
                                 static_cast<uint32_t>(w[j] >= T3);
            b0 |= (idx & 1u) << (4 * j + r);
            b1 |= (idx >> 1) << (4 * j + r);
        }
    }
    const int u = o >> 1;
    const int pos = grouped_unit_pos(u >> 3, u & 7, NG);
    packed[static_cast<size_t>(g4) * cells + 2 * pos + (o & 1)] = make_uint2(b0, b1);
}

__global__ __launch_bounds__(PACK_THREADS) void unpack_grouped_kernel(const uint2* __restrict__ packed, int N, int K,
                                                                      uint8_t* __restrict__ idx)
{
    const int g4 = blockIdx.y;
    const int cells = K / 8;
    const int o = blockIdx.x * PACK_THREADS + threadIdx.x;
    if (o >= cells) return;
    const int u = o >> 1;
    const int pos = grouped_unit_pos(u >> 3, u & 7, K / GROUP);
    const uint2 c = packed[static_cast<size_t>(g4) * cells + 2 * pos + (o & 1)];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        uint32_t lo4 = 0, hi4 = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t v = ((c.x >> (4 * j + r)) & 1u) | (((c.y >> (4 * j + r)) & 1u) << 1);
            if (j < 4) lo4 |= v << (8 * j);
            else hi4 |= v << (8 * (j - 4));
        }
        *reinterpret_cast<uint2*>(idx + static_cast<size_t>(4 * g4 + r) * K + static_cast<size_t>(o) * 8) =
            make_uint2(lo4, hi4);
    }
}

int launch_pack_grouped(const void* W, rcp_dtype dt, int N, int K, const float* lo, const float* hi,
                        const float* part, void* packed, void* codebook, hipStream_t st)
{
    if (N / 4 > 65535) return fail(RCP_ERR_SHAPE, "rcp_pack_weights_grouped: N=%d exceeds 262140", N);
    dim3 grid((K / 8 + PACK_THREADS - 1) / PACK_THREADS, N / 4);
    auto* pk = static_cast<uint2*>(packed);
    auto* cb = static_cast<uint16_t*>(codebook);
    switch (dt) {
        case RCP_F16: pack_grouped_kernel<RCP_F16><<<grid, PACK_THREADS, 0, st>>>(W, N, K, lo, hi, part, pk, cb); break;
        case RCP_F32: pack_grouped_kernel<RCP_F32><<<grid, PACK_THREADS, 0, st>>>(W, N, K, lo, hi, part, pk, cb); break;
        default: pack_grouped_kernel<RCP_BF16><<<grid, PACK_THREADS, 0, st>>>(W, N, K, lo, hi, part, pk, cb); break;
    }
    return check_launch("rcp_pack_weights_grouped");
}

int launch_unpack_grouped(const void* packed, int N, int K, uint8_t* idx, hipStream_t st)
{
    if (N / 4 > 65535) return fail(RCP_ERR_SHAPE, "rcp_unpack_indices_grouped: N=%d exceeds 262140", N);
    dim3 grid((K / 8 + PACK_THREADS - 1) / PACK_THREADS, N / 4);
    unpack_grouped_kernel<<<grid, PACK_THREADS, 0, st>>>(static_cast<const uint2*>(packed), N, K, idx);
    return check_launch("rcp_unpack_indices_grouped");
}

// ---------------------------------------------------------------------------------------------
// 3-bit variant: LDP on the asymmetric normal-float format (Section 4.3, paragraph on the NF3
// format).  Eight levels per output row from the clip values, the centre fraction and the
// format's grid; three bit planes per unit of 4 rows x 32 columns (layout in include/rcp.h).
// ---------------------------------------------------------------------------------------------
struct W3Levels {
    float T[7];
    uint16_t L[8];
};

__device__ static W3Levels w3_levels(float lo_f, float hi_f, float frac_f, const W3Grid& grid)
{
    const double lo = lo_f, hi = hi_f;
    const double c = __dadd_rn(lo, __dmul_rn(__dsub_rn(hi, lo), static_cast<double>(frac_f)));
    const double s_neg = fabs(__dsub_rn(c, lo)), s_pos = fabs(__dsub_rn(hi, c));
    double L[8];
    W3Levels out;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const double g = grid.g[j];
        L[j] = __dadd_rn(c, __dmul_rn(g < 0.0 ? s_neg : s_pos, g));
        out.L[j] = double_to_half_bits(L[j]);
    }
#pragma unroll
    for (int j = 1; j < 8; ++j) out.T[j - 1] = __double2float_rn(__ddiv_rn(__dadd_rn(L[j - 1], L[j]), 2.0));
    return out;
}

// byte offset of plane 0 of unit u inside its row group, and the distance between planes
__device__ __forceinline__ size_t w3_unit_offset(int u, int U, int& plane_stride)
{
    const int j = u >> 6;
    const int R = min(64, U - 64 * j);
    plane_stride = 16 * R;
    return static_cast<size_t>(3072) * j + 16 * (u & 63);
}

// One workgroup: one group of four rows x 256 units; one thread per unit.
template <int DT>
__global__ __launch_bounds__(PACK_THREADS) void pack_w3_kernel(const void* __restrict__ W, int N, int K,
                                                               const float* __restrict__ clip_lo,
                                                               const float* __restrict__ clip_hi,
                                                               const float* __restrict__ frac, W3Grid grid,
                                                               uint8_t* __restrict__ packed,
                                                               uint16_t* __restrict__ codebook)
{
    __shared__ float sT[4][7];
    const int g = blockIdx.y;
    const int U = K / 32;
    if (threadIdx.x < 4) {
        const int h = 4 * g + threadIdx.x;
        const W3Levels lv = w3_levels(clip_lo[h], clip_hi[h], frac[h], grid);
#pragma unroll
        for (int j = 0; j < 7; ++j) sT[threadIdx.x][j] = lv.T[j];
        if (blockIdx.x == 0) {
            uint4 lut;
            lut.x = lv.L[0] | (static_cast<uint32_t>(lv.L[1]) << 16);
            lut.y = lv.L[2] | (static_cast<uint32_t>(lv.L[3]) << 16);
            lut.z = lv.L[4] | (static_cast<uint32_t>(lv.L[5]) << 16);
            lut.w = lv.L[6] | (static_cast<uint32_t>(lv.L[7]) << 16);
            reinterpret_cast<uint4*>(codebook)[h] = lut;
        }
    }
    __syncthreads();
    const int u = blockIdx.x * PACK_THREADS + threadIdx.x;
    if (u >= U) return;
    uint32_t pl[3][4] = {};
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float w[8];
            load8_as_float<DT>(W, static_cast<size_t>(4 * g + r) * K + static_cast<size_t>(u) * 32 + 8 * c, w);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                uint32_t idx = 0;
#pragma unroll
                for (int t = 0; t < 7; ++t) idx += static_cast<uint32_t>(w[j] >= sT[r][t]);
                pl[0][c] |= (idx & 1u) << (4 * j + r);
                pl[1][c] |= ((idx >> 1) & 1u) << (4 * j + r);
                pl[2][c] |= (idx >> 2) << (4 * j + r);
            }
        }
    }
    int ps;
    uint8_t* dst = packed + static_cast<size_t>(g) * U * 48 + w3_unit_offset(u, U, ps);
#pragma unroll
    for (int p = 0; p < 3; ++p)
        *reinterpret_cast<uint4*>(dst + static_cast<size_t>(p) * ps) = make_uint4(pl[p][0], pl[p][1], pl[p][2], pl[p][3]);
}

__global__ __launch_bounds__(PACK_THREADS) void unpack_w3_kernel(const uint8_t* __restrict__ packed, int N, int K,
                                                                 uint8_t* __restrict__ idx)
{
    const int g = blockIdx.y;
    const int U = K / 32;
    const int u = blockIdx.x * PACK_THREADS + threadIdx.x;
    if (u >= U) return;
    int ps;
    const uint8_t* src = packed + static_cast<size_t>(g) * U * 48 + w3_unit_offset(u, U, ps);
    uint32_t pl[3][4];
#pragma unroll
    for (int p = 0; p < 3; ++p) {
        const uint4 v = *reinterpret_cast<const uint4*>(src + static_cast<size_t>(p) * ps);
        pl[p][0] = v.x;
        pl[p][1] = v.y;
        pl[p][2] = v.z;
        pl[p][3] = v.w;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            uint32_t lo4 = 0, hi4 = 0;  // eight index bytes of row r, columns 8c .. 8c+7 of the unit
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int b = 4 * j + r;
                const uint32_t v = ((pl[0][c] >> b) & 1u) | (((pl[1][c] >> b) & 1u) << 1) | (((pl[2][c] >> b) & 1u) << 2);
                if (j < 4) lo4 |= v << (8 * j);
                else hi4 |= v << (8 * (j - 4));
            }
            *reinterpret_cast<uint2*>(idx + static_cast<size_t>(4 * g + r) * K + static_cast<size_t>(u) * 32 + 8 * c) =
                make_uint2(lo4, hi4);
        }
    }
}

int launch_pack_w3(const void* W, rcp_dtype dt, int N, int K, const float* lo, const float* hi, const float* frac,
                   const W3Grid& grid, void* packed, void* codebook, hipStream_t st)
{
    if (N / 4 > 65535) return fail(RCP_ERR_SHAPE, "rcp_pack_weights_w3: N=%d exceeds 262140", N);
    dim3 blocks((K / 32 + PACK_THREADS - 1) / PACK_THREADS, N / 4);
    auto* pk = static_cast<uint8_t*>(packed);
    auto* cb = static_cast<uint16_t*>(codebook);
    switch (dt) {
        case RCP_F16: pack_w3_kernel<RCP_F16><<<blocks, PACK_THREADS, 0, st>>>(W, N, K, lo, hi, frac, grid, pk, cb); break;
        case RCP_F32: pack_w3_kernel<RCP_F32><<<blocks, PACK_THREADS, 0, st>>>(W, N, K, lo, hi, frac, grid, pk, cb); break;
        default: pack_w3_kernel<RCP_BF16><<<blocks, PACK_THREADS, 0, st>>>(W, N, K, lo, hi, frac, grid, pk, cb); break;
    }
    return check_launch("rcp_pack_weights_w3");
}

int launch_unpack_w3(const void* packed, int N, int K, uint8_t* idx, hipStream_t st)
{
    if (N / 4 > 65535) return fail(RCP_ERR_SHAPE, "rcp_unpack_indices_w3: N=%d exceeds 262140", N);
    dim3 blocks((K / 32 + PACK_THREADS - 1) / PACK_THREADS, N / 4);
    unpack_w3_kernel<<<blocks, PACK_THREADS, 0, st>>>(static_cast<const uint8_t*>(packed), N, K, idx);
    return check_launch("rcp_unpack_indices_w3");
}

}  // namespace rcp
