// Skinny W2A4 GEMM (2 <= M <= 16 tokens) on the matrix cores (the small-batch case of Section
// 4.4's kernel; the Appendix "GEMM Kernel Design" reports that a dequantise-then-MMA design did
// not pay off on the hardware used there).  Here nothing is dequantised: the bit-plane layout
// is itself a valid FP4 operand.
//
// With several tokens the per-level partial sums
//     F_p[h][m] = sum_k b_p[h][k] * q[m][k],  p in {b0, b1, b0 & b1}
// are a dense contraction of a 0/1 matrix with a small-integer matrix.  A nibble of a plane word
// holds one column of four rows; masked down to one bit it is, read as an FP4 (E2M1) number,
//     bit 0 -> 0.5,  bit 1 -> 1.0,  bit 2 -> 2.0   (bit 3 is the sign: it is shifted to bit 2)
// so a plane word ANDed with 0x1111.., 0x2222.., 0x4444.. is the A operand of
// v_mfma_f32_16x16x128_f8f6f4 for rows r = 0, 1, 2 (and (w >> 1) & 0x4444.. for r = 3) without
// any expansion; the factors 0.5 / 1 / 2 are taken out again by the instruction's E8M0 scale of the A operand.
// The int4 activation q = 4*hi + lo, lo in {0..3}, hi in {-2..1}, is recoded into two FP4
// operands.  Up to 8 tokens they share one B operand (columns 0..7 carry lo, columns 8..15 hi of
// the same tokens, the hi columns weighted 2^2 by the per-lane E8M0 scale of the B operand); beyond
// that lo and hi are two B operands, hi weighted the same way, accumulating into the same registers.
// Every product and every sum is a small multiple of 1/2, so the fp32 accumulators are exact
// (|F_p| <= 8K < 2^24) and the per-level sums stay bit-exact.
//
// Work decomposition.  A workgroup owns 16 groups of four rows (64 output rows): lane l of a
// wavefront supplies row group l%16 and the 32 columns of K-block l/16 of a 128-column step
// (two 16-byte units), and token l%16 for the B operand.  The wavefronts of the workgroup take
// the 128-column steps of K in turn and add their accumulators into LDS at the end, where the
// epilogue (per-level sums -> LUT -> scale) runs once per (token, row).
#include "rcp_internal.hpp"

namespace rcp {

constexpr int MM_MAX_THREADS = 512;
constexpr int MM_STRIDE = 65;       // LDS row stride (ints): conflict-free for both phases
constexpr int MM_PLANE = 16 * MM_STRIDE;
constexpr int MM_SUMS = 3 * MM_PLANE + 16;          // ints that are accumulated into (zeroed first)
constexpr int MM_LDS_INTS = MM_SUMS + 2 * 64 + 16;  // + the 64 LUT rows of the block and the scales

struct MmStage {
    u32x4 wa, wb;  // two units: 4 rows x 32 columns, bit planes b0 / b1 interleaved per cell
    u32x4 xq;      // 32 int4 activations of this lane's token
};

// PACKED: M <= 8, lo and hi of token n in columns n and n + 8 of one B operand.
// NARROW: the workgroup owns 4 row groups (16 output rows) instead of 16: the 16 rows of the A
// operand are then (row group, row in the nibble) pairs, lane l supplying row group (l%16)/4 masked
// down to row l%4, so one instruction per plane covers all four rows.  Four lanes load the same
// weights and the activations are recoded once per 16 instead of once per 64 rows, but a matrix
// of 4096 rows becomes 256 workgroups instead of 64.
// MM_NS: K steps per pipeline stage.
template <bool OUT_F16, bool PACKED, bool NARROW, int MM_NS>
__global__ __launch_bounds__(MM_MAX_THREADS) void gemm_mfma_kernel(const uint4* __restrict__ packed,
                                                                   const uint2* __restrict__ codebook, int N, int K,
                                                                   const uint4* __restrict__ xq,
                                                                   const uint16_t* __restrict__ scale, int M, int W, int RG,
                                                                   void* __restrict__ out, int32_t* __restrict__ Pout)
{
    __shared__ int red[MM_LDS_INTS];  // F sums [plane][token][row of the block], T[token]; LUT rows, scales
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // (W, the wavefronts of the workgroup, is an argument: the launch dimensions would have to be fetched from memory)
    const int i = lane & 15, kb = lane >> 4;
    const int U = K / 16, G = N / 4;
    const int KS = (K + 127) >> 7;  // steps of 128 columns
    // RG row groups per workgroup (wide form: 1..16, chosen by the launcher so that the grid fills the compute units
    // evenly; lanes with i >= RG load nothing and their rows of the A operand are zero)
    const int RB = NARROW ? 16 : 4 * RG;  // output rows of the workgroup
    const int rg = NARROW ? static_cast<int>(blockIdx.x) * 4 + (i >> 2) : static_cast<int>(blockIdx.x) * RG + i;
    // NARROW: this lane's row of the nibble as a mask (the fourth row is the FP4 sign bit: shifted down first)
    const uint32_t row_mask = (i & 3) == 0 ? 0x11111111u : (i & 3) == 1 ? 0x22222222u : 0x44444444u;
    const int row_shift = (i & 3) == 3 ? 1 : 0;
    // E8M0 scale that takes the mask's value (0.5, 1, 2, 2 for rows 0..3 of a nibble) out of the products again
    const int row_scale = (i & 3) == 0 ? 0x80 : (i & 3) == 1 ? 0x7f : 0x7e;


    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint4*>(packed), 0, static_cast<int>(static_cast<unsigned>(G) * static_cast<unsigned>(U) * 16u), 0x00020000);
    // tokens beyond M start beyond the end of the resource and read as zero
    const __amdgpu_buffer_rsrc_t xres =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4*>(xq), 0, M * (K / 2), 0x00020000);
    const unsigned wbase = (rg < G && (NARROW || i < RG)) ? (static_cast<unsigned>(rg) * U + 2u * kb) * 16u : 0x80000000u;
    const int token = PACKED ? (i & 7) : i;  // the token whose activations this lane feeds into B
    const bool hi_lane = PACKED && i >= 8;
    const int col_scale = hi_lane ? 0x81 : 0x7f;  // E8M0 scale of this lane's B values: 2^2 for a hi column
    const unsigned xbase = static_cast<unsigned>(token) * (K / 2) + kb * 16u;

    auto load = [&](int step_index, MmStage& st) {
        const int s = __builtin_amdgcn_readfirstlane(step_index);  // the same for the whole wavefront: scalar offsets
        const bool ok = 8 * s + 2 * kb < U;  // false for the K tail and for steps past the end
        const unsigned wo = ok ? wbase : 0x80000000u;
        const unsigned xo = ok ? xbase : 0x80000000u;
        st.wa = __builtin_amdgcn_raw_buffer_load_b128(wres, static_cast<int>(wo), s * 128, 0);
        st.wb = __builtin_amdgcn_raw_buffer_load_b128(wres, static_cast<int>(wo), s * 128 + 16, 0);
        st.xq = __builtin_amdgcn_raw_buffer_load_b128(xres, static_cast<int>(xo), s * 64, 0);
    };

    // Two register sets of MM_NS steps each alternate: one is in flight while the other is computed.
    MmStage sA[MM_NS], sB[MM_NS];
    int s = wave;  // this wavefront's current step; the launcher guarantees wave < KS
#pragma unroll
    for (int j = 0; j < MM_NS; ++j) load(s + j * W, sA[j]);
    // what the epilogue needs from memory is fetched now and parked in LDS after the loop
    uint2 lut_pre = make_uint2(0u, 0u);
    uint32_t scale_pre = 0;
    if (tid < RB) lut_pre = codebook[min(static_cast<int>(blockIdx.x) * RB + tid, N - 1)];
    if (tid < M) scale_pre = scale[tid];
    __builtin_amdgcn_sched_barrier(0);  // the loads leave before the LDS is cleared
    for (int j = tid; j < MM_SUMS; j += 64 * W) red[j] = 0;
    __syncthreads();  // LDS is zero before anyone adds to it

    constexpr int NB = PACKED ? 1 : 2;  // B operands per A operand
    v4f acc[3][4];
#pragma unroll
    for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[p][r] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
    int tsum = 0;

    auto compute = [&](const MmStage& cur) {
        const uint32_t xw[4] = {cur.xq.x, cur.xq.y, cur.xq.z, cur.xq.w};
        v8i bop[NB];
#pragma unroll
        for (int h = 0; h < NB; ++h) bop[h] = v8i{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t lo = fp4_lo(xw[d]), hi = fp4_hi(xw[d]);
            if constexpr (PACKED) {
                bop[0][d] = static_cast<int>(hi_lane ? hi : lo);
            } else {
                bop[0][d] = static_cast<int>(lo);
                bop[1][d] = static_cast<int>(hi);
            }
            tsum = dot8(xw[d], 0x11111111u, tsum);
        }
        const uint32_t p0[4] = {cur.wa.x, cur.wa.z, cur.wb.x, cur.wb.z};
        const uint32_t p1[4] = {cur.wa.y, cur.wa.w, cur.wb.y, cur.wb.w};
        if constexpr (NARROW) {
            v8i an[3];
#pragma unroll
            for (int p = 0; p < 3; ++p) an[p] = v8i{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                an[0][d] = static_cast<int>((p0[d] >> row_shift) & row_mask);
                an[1][d] = static_cast<int>((p1[d] >> row_shift) & row_mask);
                an[2][d] = an[0][d] & an[1][d];
            }
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                if constexpr (PACKED) {
                    acc[p][0] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(an[p], bop[0], acc[p][0], 4, 4, 0, row_scale, 0, col_scale);
                } else {
                    acc[p][0] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(an[p], bop[0], acc[p][0], 4, 4, 0, row_scale, 0, 0x7f);
                    acc[p][0] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(an[p], bop[1], acc[p][0], 4, 4, 0, row_scale, 0, 0x81);
                }
            }
            return;
        }
        // plane by plane, so that only two sets of masks are alive at a time
        v8i a[3][4];
#pragma unroll
        for (int p = 0; p < 3; ++p) {
#pragma unroll
            for (int r = 0; r < 4; ++r) a[p][r] = v8i{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                if (p < 2) {
                    const uint32_t w = p == 0 ? p0[d] : p1[d];
                    a[p][0][d] = static_cast<int>(w & 0x11111111u);
                    a[p][1][d] = static_cast<int>(w & 0x22222222u);
                    a[p][2][d] = static_cast<int>(w & 0x44444444u);
                    a[p][3][d] = static_cast<int>((w >> 1) & 0x44444444u);
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) a[2][r][d] = a[0][r][d] & a[1][r][d];  // the masks of b0 & b1
                }
            }
            if constexpr (PACKED) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[p][r] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[p][r], bop[0], acc[p][r], 4, 4, 0, r == 0 ? 0x80 : r == 1 ? 0x7f : 0x7e, 0, col_scale);
            } else {
                // E8M0 scales (byte 0): the inverse of the mask's value for A, 2^0 for lo, 2^2 for hi
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[p][r] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[p][r], bop[0], acc[p][r], 4, 4, 0, r == 0 ? 0x80 : r == 1 ? 0x7f : 0x7e, 0, 0x7f);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[p][r] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[p][r], bop[1], acc[p][r], 4, 4, 0, r == 0 ? 0x80 : r == 1 ? 0x7f : 0x7e, 0, 0x81);
            }
        }
    };
    // Steps past the end of K read zeros (no traffic) and add zeros.
    auto stage = [&](const MmStage (&cur)[MM_NS], MmStage (&next)[MM_NS]) {
#pragma unroll
        for (int j = 0; j < MM_NS; ++j) load(s + (MM_NS + j) * W, next[j]);
        // nothing that needs `cur` may move above the loads just issued
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < MM_NS; ++j) compute(cur[j]);
        s += MM_NS * W;
    };
    while (true) {
        stage(sA, sB);
        if (s >= KS) break;
        stage(sB, sA);
        if (s >= KS) break;
    }
    // The last stage loaded (zeros, past the end of K) is "used" here on purpose: without a use
    // on the exit path the optimiser sinks each stage's loads below the exit test, next to their
    // use in the following stage, and the loop is no longer pipelined.
    uint32_t keep = 0;
#pragma unroll
    for (int j = 0; j < MM_NS; ++j) keep |= sA[j].wa.x | sA[j].wb.x | sA[j].xq.x | sB[j].wa.x | sB[j].wb.x | sB[j].xq.x;
    if (__builtin_expect(K < 0, 0)) red[0] = static_cast<int>(keep);  // never true

    // acc[p][r][v] = F_p (packed: its lo part, or four times its hi part) of row 4*(RG*block + 4*kb + v) + r and this
    // lane's token, an integer: the instruction's scales have taken out the mask's power of two and weighted the hi
    // columns.  The wavefronts (and, when packed, the two columns of a token) add them up in LDS (integer adds: the
    // binary32 LDS add is far slower).
    if constexpr (NARROW) {
        // acc[p][0][v]: row v of row group kb of the block
        int* dst = red + token * MM_STRIDE + 4 * kb;
#pragma unroll
        for (int p = 0; p < 3; ++p)
#pragma unroll
            for (int v = 0; v < 4; ++v) atomicAdd(dst + p * MM_PLANE + v, static_cast<int>(acc[p][0][v]));
    } else {
        int* dst = red + token * MM_STRIDE + 16 * kb;
#pragma unroll
        for (int p = 0; p < 3; ++p)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int v = 0; v < 4; ++v) atomicAdd(dst + p * MM_PLANE + 4 * v + r, static_cast<int>(acc[p][r][v]));
    }
    if (!hi_lane) atomicAdd(red + 3 * MM_PLANE + token, tsum);
    {
        if (tid < RB) {
            red[MM_SUMS + 2 * tid] = static_cast<int>(lut_pre.x);
            red[MM_SUMS + 2 * tid + 1] = static_cast<int>(lut_pre.y);
        }
        if (tid < 16) red[MM_SUMS + 128 + tid] = static_cast<int>(scale_pre);
    }
    __syncthreads();

    for (int o = tid; o < M * 64; o += 64 * W) {
        const int n = o >> 6, hh = o & 63;
        const int h = blockIdx.x * RB + hh;
        if (hh >= RB || h >= N) continue;
        const int F0 = red[n * MM_STRIDE + hh], F1 = red[MM_PLANE + n * MM_STRIDE + hh];
        const int F3 = red[2 * MM_PLANE + n * MM_STRIDE + hh];
        const int T = red[3 * MM_PLANE + n];
        const int P3 = F3, P1 = F0 - F3, P2 = F1 - F3, P0 = T - F0 - F1 + F3;
        const uint2 lut = make_uint2(static_cast<uint32_t>(red[MM_SUMS + 2 * hh]), static_cast<uint32_t>(red[MM_SUMS + 2 * hh + 1]));
        const float c0 = half_bits_to_float(static_cast<uint16_t>(lut.x & 0xffffu));
        const float c1 = half_bits_to_float(static_cast<uint16_t>(lut.x >> 16));
        const float c2 = half_bits_to_float(static_cast<uint16_t>(lut.y & 0xffffu));
        const float c3 = half_bits_to_float(static_cast<uint16_t>(lut.y >> 16));
        float val = c0 * static_cast<float>(P0);
        val = fmaf(c1, static_cast<float>(P1), val);
        val = fmaf(c2, static_cast<float>(P2), val);
        val = fmaf(c3, static_cast<float>(P3), val);
        val *= half_bits_to_float(static_cast<uint16_t>(red[MM_SUMS + 128 + n]));
        const size_t oi = static_cast<size_t>(n) * N + h;
        if constexpr (OUT_F16) static_cast<__half*>(out)[oi] = __float2half_rn(val);
        else static_cast<float*>(out)[oi] = val;
        if (Pout != nullptr) reinterpret_cast<int4*>(Pout)[oi] = make_int4(P0, P1, P2, P3);
    }
}

int launch_gemm_mfma(const void* packed, const void* codebook, int N, int K, const void* xq, const void* scale,
                     int M, void* out, rcp_dtype out_dt, int32_t* P, hipStream_t st)
{
    const int KS = (K + 127) / 128;
    // 16-row workgroups when 64-row ones would leave most compute units idle; otherwise the wide form with the fewest
    // row groups per workgroup (<= 16) that still gives a whole number of workgroups per compute unit, so that no unit
    // carries twice the work of its neighbour ("gemm_rows" = 16 forces the first form, 20, 24 .. 64 the second)
    const int cus = num_compute_units(), G = N / 4;
    bool narrow = G <= 8 * cus;  // up to 8192 rows on 256 units (sweeps: 8192 x 2048 4.0 against 4.35 us)
    int RG = 16;
    for (int per_cu = 1; per_cu <= 64; ++per_cu) {
        const int want = (G + per_cu * cus - 1) / (per_cu * cus);
        if (want <= 16) {
            RG = want;
            break;
        }
    }
    if (options().gemm_rows != 0) {
        narrow = options().gemm_rows == 16;
        if (!narrow) RG = options().gemm_rows / 4;
    }
    const int blocks = narrow ? (N + 15) / 16 : (G + RG - 1) / RG;
    // 8 wavefronts per workgroup share the K steps of a row block (sweeps: 8 with one step per
    // pipeline stage beats 4 with deeper stages on every LLaMA shape), never more than there are steps
    int waves = 8;
    if (options().gemm_waves != 0) waves = options().gemm_waves;
    while (waves > 1 && waves > KS) waves /= 2;
    auto* pk = static_cast<const uint4*>(packed);
    auto* cb = static_cast<const uint2*>(codebook);
    auto* x4 = static_cast<const uint4*>(xq);
    auto* sc = static_cast<const uint16_t*>(scale);
    const dim3 grid(blocks), block(waves * 64);
    // two steps per pipeline stage once a wavefront has eight or more steps to walk (4096 x 11008: 6.9 against 7.6 us;
    // slower on the short loops of K = 4096)
    const bool deep = options().gemm_stage != 0 ? options().gemm_stage == 2 : KS >= 8 * waves;
#define RCP_MM(F16, PK, NA)                                                                                   \
    do {                                                                                                      \
        if (deep) gemm_mfma_kernel<F16, PK, NA, 2><<<grid, block, 0, st>>>(pk, cb, N, K, x4, sc, M, waves, RG, out, P); \
        else gemm_mfma_kernel<F16, PK, NA, 1><<<grid, block, 0, st>>>(pk, cb, N, K, x4, sc, M, waves, RG, out, P);      \
    } while (0)
    const bool f16 = out_dt == RCP_F16, pkd = M <= 8;
    if (narrow) {
        if (pkd) { if (f16) RCP_MM(true, true, true); else RCP_MM(false, true, true); }
        else     { if (f16) RCP_MM(true, false, true); else RCP_MM(false, false, true); }
    } else {
        if (pkd) { if (f16) RCP_MM(true, true, false); else RCP_MM(false, true, false); }
        else     { if (f16) RCP_MM(true, false, false); else RCP_MM(false, false, false); }
    }
#undef RCP_MM
    return check_launch("rcp_w2a4_gemv");
}

}  // namespace rcp
