// Weight-only GEMV: O[h] = sum_k LUT[h][idx[h][k]] * x[k] with 16- or 32-bit activations (the
// W2-only decode variant measured in the paper's inference-latency section, where the
// non-uniform dequantisation is merged into a 16-bit linear layer).  One token.
//
// Without integer activations there are no per-level integer sums to form; each weight has to
// become a number.  The dequantisation is a table look-up in LDS that yields TWO weights at a
// time as a packed fp16 pair, ready for v_dot2_f32_f16 against a packed pair of activations:
//   - for row r of a cell, E_r = ((B0 >> r) & 0x1111..) | (((B1 >> r) & 0x1111..) << 1) holds
//     the eight 2-bit indices of the row, one per nibble (5 operations for 8 weights);
//     (built for two rows at once, about 20 operations per 32 weights);
//   - a byte of E_r is made the index pair of two neighbouring columns, t = lo + 4*hi;
//   - the wavefront keeps, for its current group of four rows, the 4 x 16 pairs
//     (LUT[r][lo], LUT[r][hi]) at dword t + 16*r of a 64-dword table: the 16 entries one
//     instruction can touch (all lanes look up the same row r) lie in 16 different LDS banks, so
//     the look-ups never conflict (equal addresses are broadcast); the four free top bits of
//     every byte of E_r carry r and the wavefront's table number, so a byte times four IS the
//     LDS address;
//   - one byte-select-and-shift (SDWA), one ds_read_b32 and one dot2 per two weights.
// About 1.6 vector-ALU and 0.5 LDS operations per weight, against 0.69 for the W2A4 kernel.
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
constexpr int WO_TABLE_DWORDS = 64;

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

__host__ __device__ constexpr int wo_padded_units(int K, int span /* lanes per row group x loads per stage */)
{
    const int U = K / 16;
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
// WS wavefronts share one row group (each with a table of its own; one LDS exchange of the four
// row totals per row group): short, wide matrices would otherwise put a single wavefront on a
// SIMD, which issues an instruction only every ~7 cycles.  UNR: 16-byte loads per lane and stage.
// NT: weight loads with the non-temporal hint (launches of 4 MB and more: on a sweep of its own the kernel is level with
// and without it, inside a decode step of 32 layers the hint is worth 1.6 %, 1.094 -> 1.077 ms).
template <bool XF32, int XDT, int WS, int UNR, bool NT = false>
__global__ __launch_bounds__(WO_THREADS) void w2a16_kernel(const uint4* __restrict__ packed,
                                                           const uint2* __restrict__ codebook, int N, int K,
                                                           const void* __restrict__ x, void* __restrict__ out,
                                                           int out_f16, int nblk)
{
    constexpr int WO_UNR = UNR;
    constexpr int SLOTS = WO_WAVES / WS;  // row groups a workgroup works on at a time
    constexpr int LG = 64 * WS;           // lanes per row group
    extern __shared__ uint32_t wo_smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int U = K / 16, G = N / 4;
    const int slot = wave / WS, wsub = wave % WS;
    const int tg = wsub * 64 + lane;  // this lane's position among the LG lanes of its row group
    const int nbatch = (G + SLOTS - 1) / SLOTS;
    const int nchunk = (U + LG * WO_UNR - 1) / (LG * WO_UNR);
    // (nblk, the number of workgroups, is an argument: the launch dimensions would have to be fetched from memory)
    uint32_t* tab = wo_smem + wave * WO_TABLE_DWORDS;
    const uint32_t wave_bits = 0x40404040u * static_cast<uint32_t>(wave);
    uint32_t* sx = wo_smem + WO_WAVES * WO_TABLE_DWORDS;
    constexpr int XD = XF32 ? 16 : 8;  // dwords of activations per unit

    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint4*>(packed), 0, static_cast<int>(static_cast<unsigned>(G) * static_cast<unsigned>(U) * 16u), 0x00020000);
    const int my_units = (U % (LG * WO_UNR)) != 0 ? (U - tg + LG - 1) / LG : 0x7fffffff;
    auto batch_offset = [&](int bb) -> unsigned { return (static_cast<unsigned>(bb * SLOTS + slot) * U + tg) * 16u; };
    const unsigned batch_stride = static_cast<unsigned>(nblk) * SLOTS * U * 16u;
    auto load_chunk = [&](unsigned base, int ch, int bb, u32x4 (&w)[WO_UNR]) {
        const bool row_ok = bb * SLOTS + slot < G;
#pragma unroll
        for (int i = 0; i < WO_UNR; ++i) {
            const int it = ch * WO_UNR + i;
            const unsigned off = (it < my_units && row_ok) ? base : 0x80000000u;
            w[i] = __builtin_amdgcn_raw_buffer_load_b128(wres, static_cast<int>(off), it * LG * 16, NT ? 2 : 0);
        }
    };
    // the four LUT rows of a row group, one per 16 table entries: lane d builds entry d
    const int ent_lo = lane & 3, ent_hi = (lane >> 2) & 3, ent_r = lane >> 4;
    auto load_lut = [&](int bb) -> uint2 { return codebook[min(4 * (bb * SLOTS + slot) + ent_r, N - 1)]; };
    auto build_table = [&](uint2 row) { tab[lane] = lut_half(row, ent_lo) | (lut_half(row, ent_hi) << 16); };

    // memory answers loads in issue order: this thread's activations (up to WO_XG pieces of eight, K <= 12288; a longer
    // token's remaining pieces are fetched in the staging loop) go first, so that staging them does not have to wait
    // for the weights
    constexpr int WO_XG = 6;
    const int xpieces = min((K / 8 + WO_THREADS - 1) / WO_THREADS, WO_XG);  // pieces held in registers
    Raw8<XDT> xr[WO_XG];
#pragma unroll
    for (int i = 0; i < WO_XG; ++i) {
        if (i * WO_THREADS >= K / 8) break;  // uniform
        xr[i] = load8_raw<XDT>(x, static_cast<size_t>(min(static_cast<int>(threadIdx.x) + i * WO_THREADS, K / 8 - 1)) * 8);
    }
    int b = blockIdx.x;
    uint2 lut_row = load_lut(b);  // needed for the table before the first step: ahead of the weights too
    __builtin_amdgcn_sched_barrier(0);
    unsigned base = batch_offset(b);
    u32x4 wA[WO_UNR], wB[WO_UNR];
    load_chunk(base, 0, b, wA);
    // (a use right here keeps the compiler from moving the activation load down into the staging branch)
    asm volatile("" ::"v"(xr[0].a.x), "v"(xr[0].a.w), "v"(lut_row.x));

    // stage the activations, zero beyond K
    const int padded = wo_padded_units(K, LG * WO_UNR);
    // behind the activations: the exchange slots of the row totals (WS > 1), two sets that alternate
    float* red = reinterpret_cast<float*>(sx + padded * XD);
    int parity = 0;
    if constexpr (!XF32) {
        const uint4* x4 = static_cast<const uint4*>(x);  // eight fp16 per uint4: two per unit
        uint4* s4 = reinterpret_cast<uint4*>(sx);
        // the pieces in registers apart from the loop: behind a join with the loop's own loads the compiler would
        // wait for every load in flight, the weights included
#pragma unroll
        for (int i = 0; i < WO_XG; ++i) {
            if (i * WO_THREADS >= K / 8) break;  // uniform
            const int j = threadIdx.x + i * WO_THREADS;
            if (j < padded * 2) s4[j] = j < K / 8 ? xr[i].a : make_uint4(0u, 0u, 0u, 0u);
        }
        for (int j = threadIdx.x + xpieces * WO_THREADS; j < padded * 2; j += WO_THREADS)
            s4[j] = j < K / 8 ? x4[j] : make_uint4(0u, 0u, 0u, 0u);
    } else {
        float4* s4 = reinterpret_cast<float4*>(sx);
#pragma unroll
        for (int i = 0; i < WO_XG; ++i) {  // the pieces in registers apart from the loop, as above
            if (i * WO_THREADS >= K / 8) break;  // uniform
            const int j = threadIdx.x + i * WO_THREADS;
            if (j < padded * 2) {
                float v[8];
                widen8<XDT>(xr[i], v);
                const bool in = j < K / 8;
                s4[2 * j] = in ? make_float4(v[0], v[1], v[2], v[3]) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                s4[2 * j + 1] = in ? make_float4(v[4], v[5], v[6], v[7]) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            }
        }
        for (int j = threadIdx.x + xpieces * WO_THREADS; j < padded * 2; j += WO_THREADS) {  // eight values per step
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
        // C02 / C13: per nibble the 2-bit indices of rows 0 and 2 (1 and 3) of one column.  E[r]: per
        // byte lo | hi << 2 (the indices of two neighbouring columns) | r << 4 | wavefront << 6, which
        // times 4 is the byte address of the pair in LDS.
        const uint32_t C02 = (B0 & 0x55555555u) | ((B1 & 0x55555555u) << 1);
        const uint32_t C13 = ((B0 >> 1) & 0x55555555u) | (B1 & 0xaaaaaaaau);
        const uint32_t E[4] = {
            (C02 & 0x03030303u) | ((C02 >> 2) & 0x0c0c0c0cu) | (wave_bits | 0x00000000u),
            (C13 & 0x03030303u) | ((C13 >> 2) & 0x0c0c0c0cu) | (wave_bits | 0x10101010u),
            ((C02 >> 2) & 0x03030303u) | ((C02 >> 4) & 0x0c0c0c0cu) | (wave_bits | 0x20202020u),
            ((C13 >> 2) & 0x03030303u) | ((C13 >> 4) & 0x0c0c0c0cu) | (wave_bits | 0x30303030u)};
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int jp = 0; jp < 4; ++jp) {
                // The read uses the absolute LDS address: the tables start at LDS offset 0 (this
                // kernel has no static LDS, which the launcher verifies), so no base has to be added.
                const uint32_t addr = byte_times4(E[r], jp);
                pair[r][jp] = *reinterpret_cast<const __attribute__((address_space(3))) uint32_t*>(addr);
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

        const uint32_t* xrow = sx + (tg + ch * WO_UNR * LG) * XD;
        uint32_t pA[4][4], pB[4][4];
        cell_lookup(w[0].x, w[0].y, pA);
#pragma unroll
        for (int i = 0; i < WO_UNR; ++i) {
            cell_lookup(w[i].z, w[i].w, pB);
            __builtin_amdgcn_sched_barrier(0);
            cell_dot(pA, xrow + i * LG * XD);
            if (i + 1 < WO_UNR) cell_lookup(w[i + 1].x, w[i + 1].y, pA);
            __builtin_amdgcn_sched_barrier(0);
            cell_dot(pB, xrow + i * LG * XD + XD / 2);
        }

        if (last) {
            // row totals over the 64 lanes: 16-lane row rho ends up with output row 2*(rho&1) + (rho>>1)
            const float s01 = fold32f(acc[0], acc[1]);
            const float s23 = fold32f(acc[2], acc[3]);
            float tot = row_sum16f(fold16f(s01, s23));
            const int rho = lane >> 4;
            if constexpr (WS > 1) {
                // the wavefronts of a row group exchange their four totals; the first one adds them
                float* mine = red + (parity * WO_WAVES + wave) * 4;
                if ((lane & 15) == 0) mine[rho] = tot;
                __syncthreads();
                if (wsub == 0 && (lane & 15) == 0) {
#pragma unroll
                    for (int ws = 1; ws < WS; ++ws) tot += red[(parity * WO_WAVES + wave + ws) * 4 + rho];
                }
                parity ^= 1;
            }
            const int rg = b * SLOTS + slot;
            if (rg < G && wsub == 0 && (lane & 15) == 0) {
                const int h = 4 * rg + (((rho & 1) << 1) | (rho >> 1));
                if (out_f16) static_cast<__half*>(out)[h] = __float2half_rn(tot);
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

template <bool XF32, int XDT, int WS, int UNR, bool NT>
static int launch_wo_one(const void* packed, const void* codebook, int N, int K, const void* x, void* out, rcp_dtype out_dt,
                         hipStream_t st)
{
    constexpr int SLOTS = WO_WAVES / WS;
    const int G = N / 4;
    const int nbatch = (G + SLOTS - 1) / SLOTS;
    const int cus = num_compute_units();
    int blocks = options().gemv_blocks;
    if (blocks == 0) blocks = nbatch <= cus * 8 ? nbatch : cus * 4;
    if (blocks > nbatch) blocks = nbatch;
    if (blocks < 1) blocks = 1;
    const size_t lds = (static_cast<size_t>(WO_WAVES) * WO_TABLE_DWORDS +
                        static_cast<size_t>(wo_padded_units(K, 64 * WS * UNR)) * (XF32 ? 16 : 8) + 2 * WO_WAVES * 4) * 4;
    if (lds > 160 * 1024)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_w2a16_gemv: K=%d needs %zu bytes of LDS for the activations", K, lds);
    auto kernel = &w2a16_kernel<XF32, XDT, WS, UNR, NT>;
    // the look-ups address the tables by absolute LDS offset: dynamic LDS must start at 0 (checked once
    // per kernel variant; the answer is a property of the compiled code)
    static int lds_checked = 0;  // 1 once the variant is known to have no static LDS
    if (lds_checked == 0) {
        hipFuncAttributes attr;
        if (hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(kernel)) != hipSuccess)
            return fail(RCP_ERR_HIP, "rcp_w2a16_gemv: cannot query the kernel's attributes");
        lds_checked = attr.sharedSizeBytes == 0 ? 1 : -1;
    }
    if (lds_checked < 0)
        return fail(RCP_ERR_HIP, "rcp_w2a16_gemv: kernel has static LDS, table addressing would be wrong");
    if (lds > 65536) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           static_cast<int>(lds));
        if (e != hipSuccess) return fail(RCP_ERR_HIP, "rcp_w2a16_gemv: LDS opt-in failed: %s", hipGetErrorString(e));
    }
    kernel<<<blocks, WO_THREADS, lds, st>>>(static_cast<const uint4*>(packed), static_cast<const uint2*>(codebook), N, K, x, out,
                                            out_dt == RCP_F16 ? 1 : 0, blocks);
    return check_launch("rcp_w2a16_gemv");
}

// Shape -> (wavefronts per row group, loads per stage): enough wavefronts to give every SIMD
// several, and no more loads per stage than a lane has units.
template <bool XF32, int XDT>
static int launch_wo(const void* packed, const void* codebook, int N, int K, const void* x, void* out, rcp_dtype out_dt,
                     hipStream_t st)
{
    const int G = N / 4, U = K / 16;
    const int cus = num_compute_units();
    int ws = G <= cus * 4 ? 4 : (G <= cus * 8 ? 2 : 1);
    const int forced = options().gemv_lanes;  // 64, 128, 256 lanes per row group
    if (forced == 64) ws = 1;
    if (forced == 128) ws = 2;
    if (forced == 256) ws = 4;
    while (ws > 1 && U < 64 * ws) ws /= 2;
    // loads per stage: the largest of 4, 2, 1 that pads a lane's units by at most a tenth (padding
    // units are computed on like real ones, and the kernel is bound by instruction issue)
    const int per_lane = (U + 64 * ws - 1) / (64 * ws);
    int unr = 1;
    for (int c = 2; c <= 4; c *= 2)
        if (((per_lane + c - 1) / c) * c * 10 <= per_lane * 11) unr = c;
    // ("gemv_nt": 1 = non-temporal weight loads always, 2 = never; automatic: from 4 MB of packed weights on -- with
    // the out-projection's 4 MB left out the step takes 1.089 ms, with them in 1.077)
    const bool nt = options().gemv_nt != 0 ? options().gemv_nt == 1 : static_cast<long long>(N) * K / 4 >= (4LL << 20);
#define RCP_WO(WS, UNR)                                                                                      \
    return nt ? launch_wo_one<XF32, XDT, WS, UNR, true>(packed, codebook, N, K, x, out, out_dt, st)          \
              : launch_wo_one<XF32, XDT, WS, UNR, false>(packed, codebook, N, K, x, out, out_dt, st)
    if (ws == 1) { if (unr == 4) RCP_WO(1, 4); if (unr == 2) RCP_WO(1, 2); RCP_WO(1, 1); }
    if (ws == 2) { if (unr == 4) RCP_WO(2, 4); if (unr == 2) RCP_WO(2, 2); RCP_WO(2, 1); }
    if (unr == 4) RCP_WO(4, 4);
    if (unr == 2) RCP_WO(4, 2);
    RCP_WO(4, 1);
#undef RCP_WO
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
