// Weight-only GEMV: O[h] = sum_k LUT[h][idx[h][k]] * x[k] with 16- or 32-bit activations (the
// W2-only decode variant measured in the paper's inference-latency section, where the
// non-uniform dequantisation is merged into a 16-bit linear layer).  One token.
//
// Without integer activations there are no per-level integer sums to form; each weight has to
// become a number.  The dequantisation is a table look-up in LDS that yields TWO weights at a
// time as a packed fp16 pair, ready for v_dot2_f32_f16 against a packed pair of activations:
//   - for row r of a cell, E_r = ((B0 >> r) & 0x1111..) | (((B1 >> r) & 0x1111..) << 1) holds
//     the eight 2-bit indices of the row, one per nibble (5 operations for 8 weights);
//     (built for two rows at once, about 12 operations per 32 weights);
//   - a byte of E_r is the index pair of two neighbouring columns, t = lo + 16*hi;
//   - the wavefront keeps, for its current group of four rows, the 4 x 16 pairs
//     (LUT[r][lo], LUT[r][hi]) at dword 4*r + t of a 64-dword table: the 64 entries fall into
//     64 different LDS banks, so the 64 lanes' look-ups never conflict (equal addresses are
//     broadcast); the two free top bits of every byte of E_r carry the wavefront's table number,
//     so a byte times four IS the LDS address;
//   - one byte-select-and-shift (SDWA), one ds_read_b32 and one dot2 per two weights.
// About 1.4 vector-ALU and 0.5 LDS operations per weight, against 0.69 for the W2A4 kernel.
// For bfloat16 / binary32 activations the pairs are multiplied with binary32 activations by
// mixed-precision FMAs instead of dot2.  Accumulation is binary32 throughout.
//
// Work decomposition and pipeline are those of the W2A4 kernel with 64 lanes per row group:
// lane t takes the 16-byte units t, t + 64, ...; the loads of the next (row group, chunk) are
// in flight while the current chunk is computed; units past K read zeros (index 0) and meet
// zero-padded activations.
#include "rcp_internal.hpp"

namespace rcp {

constexpr int WO_THREADS = 256;
constexpr int WO_WAVES = WO_THREADS / 64;
constexpr int WO_UNR = 4;          // 16-byte loads per lane and pipeline stage
constexpr int WO_TABLE_DWORDS = 64;

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

__host__ __device__ constexpr int wo_padded_units(int K)
{
    const int U = K / 16, span = 64 * WO_UNR;
    return ((U + span - 1) / span) * span;
}

// ((v >> 8*byte) & 0xff) << 2 in one instruction: a shift whose source operand selects a byte
__device__ __forceinline__ uint32_t byte_times4(uint32_t v, int byte)
{
    uint32_t d;
    const uint32_t two = 2;
    switch (byte) {
        case 0: asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(d) : "v"(two), "v"(v)); break;
        case 1: asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(d) : "v"(two), "v"(v)); break;
        case 2: asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(d) : "v"(two), "v"(v)); break;
        default: asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(d) : "v"(two), "v"(v)); break;
    }
    return d;
}

__device__ __forceinline__ uint32_t lut_half(uint2 row, int l)
{
    const uint32_t w = (l & 2) ? row.y : row.x;
    return (l & 1) ? (w >> 16) : (w & 0xffffu);
}

// XF32: activations are held in LDS as binary32 (bf16 / fp32 input), else as fp16 pairs.
template <bool XF32, int XDT, bool OUT_F16>
__global__ __launch_bounds__(WO_THREADS) void w2a16_kernel(const uint4* __restrict__ packed,
                                                           const uint2* __restrict__ codebook, int N, int K,
                                                           const void* __restrict__ x, void* __restrict__ out)
{
    extern __shared__ uint32_t wo_smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int U = K / 16, G = N / 4;
    const int nbatch = (G + WO_WAVES - 1) / WO_WAVES;
    const int nchunk = (U + 64 * WO_UNR - 1) / (64 * WO_UNR);
    const int nblk = gridDim.x;
    uint32_t* tab = wo_smem + wave * WO_TABLE_DWORDS;
    const uint32_t wave_bits = 0x40404040u * static_cast<uint32_t>(wave);
    uint32_t* sx = wo_smem + WO_WAVES * WO_TABLE_DWORDS;
    constexpr int XD = XF32 ? 16 : 8;  // dwords of activations per unit

    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint4*>(packed), 0, static_cast<int>(static_cast<unsigned>(G) * static_cast<unsigned>(U) * 16u), 0x00020000);
    const int my_units = (U % (64 * WO_UNR)) != 0 ? (U - lane + 63) / 64 : 0x7fffffff;
    auto batch_offset = [&](int bb) -> unsigned { return (static_cast<unsigned>(bb * WO_WAVES + wave) * U + lane) * 16u; };
    const unsigned batch_stride = static_cast<unsigned>(nblk) * WO_WAVES * U * 16u;
    auto load_chunk = [&](unsigned base, int ch, int bb, u32x4 (&w)[WO_UNR]) {
        const bool row_ok = bb * WO_WAVES + wave < G;
#pragma unroll
        for (int i = 0; i < WO_UNR; ++i) {
            const int it = ch * WO_UNR + i;
            const unsigned off = (it < my_units && row_ok) ? base : 0x80000000u;
            w[i] = __builtin_amdgcn_raw_buffer_load_b128(wres, static_cast<int>(off), it * 64 * 16, 0);
        }
    };
    // the four LUT rows of a row group, one per 16 table entries: lane d builds entry d
    const int ent_r = (lane >> 2) & 3, ent_lo = lane & 3, ent_hi = lane >> 4;
    auto load_lut = [&](int bb) -> uint2 { return codebook[min(4 * (bb * WO_WAVES + wave) + ent_r, N - 1)]; };
    auto build_table = [&](uint2 row) { tab[lane] = lut_half(row, ent_lo) | (lut_half(row, ent_hi) << 16); };

    int b = blockIdx.x;
    unsigned base = batch_offset(b);
    u32x4 wA[WO_UNR], wB[WO_UNR];
    load_chunk(base, 0, b, wA);
    uint2 lut_row = load_lut(b);

    // stage the activations, zero beyond K
    const int padded = wo_padded_units(K);
    if constexpr (!XF32) {
        const uint4* x4 = static_cast<const uint4*>(x);  // eight fp16 per uint4: two per unit
        uint4* s4 = reinterpret_cast<uint4*>(sx);
        for (int j = threadIdx.x; j < padded * 2; j += WO_THREADS) s4[j] = j < K / 8 ? x4[j] : make_uint4(0u, 0u, 0u, 0u);
    } else {
        float4* s4 = reinterpret_cast<float4*>(sx);
        for (int j = threadIdx.x; j < padded * 2; j += WO_THREADS) {  // eight values per step
            float v[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
            if (j < K / 8) load8_as_float<XDT>(x, static_cast<size_t>(j) * 8, v);
            s4[2 * j] = make_float4(v[0], v[1], v[2], v[3]);
            s4[2 * j + 1] = make_float4(v[4], v[5], v[6], v[7]);
        }
    }
    build_table(lut_row);
    __syncthreads();

    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    int ch = 0;

    // One cell (4 rows x 8 columns) in two phases, so that the 16 look-ups of the next cell can be
    // in flight while the products of the current one are taken.
    // Phase 1: the 16 pairs (LUT[r][idx of column 2jp], LUT[r][idx of column 2jp+1]).
    auto cell_lookup = [&](uint32_t B0, uint32_t B1, uint32_t (&pair)[4][4]) {
        // C02 / C13: per nibble the 2-bit indices of rows 0 and 2 (1 and 3) of one column; wave_bits
        // puts this wavefront's table number into the two free top bits of every byte
        const uint32_t C02 = (B0 & 0x55555555u) | ((B1 & 0x55555555u) << 1);
        const uint32_t C13 = ((B0 >> 1) & 0x55555555u) | (B1 & 0xaaaaaaaau);
        const uint32_t E[4] = {(C02 & 0x33333333u) | wave_bits, (C13 & 0x33333333u) | wave_bits,
                               ((C02 >> 2) & 0x33333333u) | wave_bits, ((C13 >> 2) & 0x33333333u) | wave_bits};
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int jp = 0; jp < 4; ++jp) {
                // byte jp of E[r] = lo | hi << 4 | wave << 6; times 4 it is the byte address of the
                // pair in this wavefront's table, up to the row's 16 bytes.  The read uses the
                // absolute LDS address: the tables start at LDS offset 0 (this kernel has no static
                // LDS, which the launcher verifies), so no base has to be added.
                const uint32_t addr = byte_times4(E[r], jp);
                pair[r][jp] = *reinterpret_cast<const __attribute__((address_space(3))) uint32_t*>(addr + 16 * r);
            }
    };
    // Phase 2: products with the cell's 8 activations.
    auto cell_dot = [&](const uint32_t (&pair)[4][4], const uint32_t* xs) {
        uint32_t xv[XF32 ? 8 : 4];
        {
            const uint4 v = *reinterpret_cast<const uint4*>(xs);  // 16-byte aligned by construction
            xv[0] = v.x; xv[1] = v.y; xv[2] = v.z; xv[3] = v.w;
            if constexpr (XF32) {
                const uint4 u = *reinterpret_cast<const uint4*>(xs + 4);
                xv[4] = u.x; xv[5] = u.y; xv[6] = u.z; xv[7] = u.w;
            }
        }
#pragma unroll
        for (int jp = 0; jp < 4; ++jp)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if constexpr (!XF32) {
                    acc[r] = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, pair[r][jp]), __builtin_bit_cast(half2_t, xv[jp]), acc[r], false);
                } else {
                    acc[r] = fmaf(half_bits_to_float(static_cast<uint16_t>(pair[r][jp] & 0xffffu)), __uint_as_float(xv[2 * jp]), acc[r]);
                    acc[r] = fmaf(half_bits_to_float(static_cast<uint16_t>(pair[r][jp] >> 16)), __uint_as_float(xv[2 * jp + 1]), acc[r]);
                }
            }
    };

    auto step = [&](u32x4 (&w)[WO_UNR], u32x4 (&wnext)[WO_UNR]) {
        const bool last = ch + 1 == nchunk;
        const int b2 = last ? b + nblk : b;
        const int ch2 = last ? 0 : ch + 1;
        const unsigned base2 = base + (last ? batch_stride : 0u);
        load_chunk(base2, ch2, b2, wnext);
        if (last) lut_row = load_lut(b2);
        // no work on `w` may move above the loads just issued
        __builtin_amdgcn_sched_barrier(0);

        const uint32_t* xrow = sx + (lane + ch * WO_UNR * 64) * XD;
        uint32_t pA[4][4], pB[4][4];
        cell_lookup(w[0].x, w[0].y, pA);
#pragma unroll
        for (int i = 0; i < WO_UNR; ++i) {
            cell_lookup(w[i].z, w[i].w, pB);
            __builtin_amdgcn_sched_barrier(0);
            cell_dot(pA, xrow + i * 64 * XD);
            if (i + 1 < WO_UNR) cell_lookup(w[i + 1].x, w[i + 1].y, pA);
            __builtin_amdgcn_sched_barrier(0);
            cell_dot(pB, xrow + i * 64 * XD + XD / 2);
        }

        if (last) {
            // row totals over the 64 lanes: 16-lane row rho ends up with output row 2*(rho&1) + (rho>>1)
            const float s01 = fold32f(acc[0], acc[1]);
            const float s23 = fold32f(acc[2], acc[3]);
            const float tot = row_sum16f(fold16f(s01, s23));
            const int rg = b * WO_WAVES + wave;
            if (rg < G && (lane & 15) == 0) {
                const int rho = lane >> 4;
                const int h = 4 * rg + (((rho & 1) << 1) | (rho >> 1));
                if constexpr (OUT_F16) static_cast<__half*>(out)[h] = __float2half_rn(tot);
                else static_cast<float*>(out)[h] = tot;
            }
            acc[0] = acc[1] = acc[2] = acc[3] = 0.0f;
            build_table(lut_row);  // for the next row group; LDS operations of a wavefront stay in order
        }
        b = b2;
        ch = ch2;
        base = base2;
    };
    while (true) {
        step(wA, wB);
        if (b >= nbatch) break;
        step(wB, wA);
        if (b >= nbatch) break;
    }
}

template <bool XF32, int XDT>
static int launch_wo(const void* packed, const void* codebook, int N, int K, const void* x, void* out, rcp_dtype out_dt,
                     hipStream_t st)
{
    const int G = N / 4;
    const int nbatch = (G + WO_WAVES - 1) / WO_WAVES;
    const int cus = num_compute_units();
    int blocks = options().gemv_blocks;
    if (blocks == 0) blocks = nbatch <= cus * 8 ? nbatch : cus * 4;
    if (blocks > nbatch) blocks = nbatch;
    if (blocks < 1) blocks = 1;
    const size_t lds = (static_cast<size_t>(WO_WAVES) * WO_TABLE_DWORDS + static_cast<size_t>(wo_padded_units(K)) * (XF32 ? 16 : 8)) * 4;
    if (lds > 160 * 1024)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_w2a16_gemv: K=%d needs %zu bytes of LDS for the activations", K, lds);
    auto launch = [&](auto kernel) -> int {
        // the look-ups address the tables by absolute LDS offset: dynamic LDS must start at 0
        hipFuncAttributes attr;
        if (hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(kernel)) != hipSuccess || attr.sharedSizeBytes != 0)
            return fail(RCP_ERR_HIP, "rcp_w2a16_gemv: kernel has static LDS, table addressing would be wrong");
        if (lds > 65536) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                               static_cast<int>(lds));
            if (e != hipSuccess) return fail(RCP_ERR_HIP, "rcp_w2a16_gemv: LDS opt-in failed: %s", hipGetErrorString(e));
        }
        kernel<<<blocks, WO_THREADS, lds, st>>>(static_cast<const uint4*>(packed), static_cast<const uint2*>(codebook), N, K, x, out);
        return check_launch("rcp_w2a16_gemv");
    };
    if (out_dt == RCP_F16) return launch(&w2a16_kernel<XF32, XDT, true>);
    return launch(&w2a16_kernel<XF32, XDT, false>);
}

int launch_w2a16_gemv(const void* packed, const void* codebook, int N, int K, const void* x, rcp_dtype x_dt,
                      void* out, rcp_dtype out_dt, hipStream_t st)
{
    if (static_cast<long long>(N) * K / 4 >= (1LL << 31))
        return fail(RCP_ERR_SHAPE, "rcp_w2a16_gemv: packed matrix of %lld bytes exceeds 2 GiB", static_cast<long long>(N) * K / 4);
    if (x_dt == RCP_F16) return launch_wo<false, RCP_F16>(packed, codebook, N, K, x, out, out_dt, st);
    if (x_dt == RCP_BF16) return launch_wo<true, RCP_BF16>(packed, codebook, N, K, x, out, out_dt, st);
    return launch_wo<true, RCP_F32>(packed, codebook, N, K, x, out, out_dt, st);
}

}  // namespace rcp
