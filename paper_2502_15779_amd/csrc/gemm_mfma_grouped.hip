// Skinny W2A4 GEMM (several tokens) with group-wise look-up tables on the matrix cores: the
// scheme of gemm_mfma.hip (masked bit-plane words as FP4 operands of the 16x16x128 matrix
// instruction) applied to the paper's deployed weight setting, one LUT per (row, 128 input
// channels) (Appendix table of quantisation configurations; Section 4.4 for the product).
//
//     P[m][h][g][l] = sum_{k in group g : idx[h][k] = l} q[m][k]              (exact)
//     O[m][h]       = S[m] * sum_g sum_l LUT[h][g][l] * P[m][h][g][l]        (fp32)
//
// One 128-column step of the matrix instruction is exactly one quantisation group, so the
// accumulators are not carried from step to step: after the 24 instructions of a step (three
// bit planes x four rows of a nibble x lo / hi part of the int4 activation, hi weighted 2^2 and
// the 0.5 / 1 / 2 of the masks undone by the instruction's E8M0 scales) a lane holds the exact
// plane sums F_p of 16 rows for one token and adds their products with the group's levels to 16
// running fp32 outputs.  The per-group sum of q that level 0 needs comes from two more
// instructions with an all-ones A operand.
//
// Work decomposition: a workgroup owns 64 output rows, its 8 wavefronts take the groups of K in
// turn.  Lane l supplies row group l%16 and the two 16-byte units 2*(l/16), 2*(l/16)+1 of the
// group (the grouped packed layout keeps the same unit of neighbouring groups side by side, so
// the wavefronts of a workgroup, which work on neighbouring groups, share cache lines), and
// token l%16 for the B operand.  The 512 bytes of levels a step needs are fetched once per
// wavefront (16 bytes = two rows per lane); the fetching lane turns the four levels of a row
// into the coefficients of (sum of q, F_b0, F_b1, F_b0&b1),
//     O += L0*T + (L1-L0)*F0 + (L2-L0)*F1 + (L3-L2-L1+L0)*F3      (= sum_l L_l * P_l),
// once for all 16 token lanes, and passes them through a wavefront-private LDS buffer from which
// they are read back as broadcasts: four FMAs per (row, token) and group.  At the end every
// wavefront parks its 16 x 64 partial outputs in LDS and the workgroup adds them in a fixed
// order (deterministic), scales and stores.
#include "rcp_internal.hpp"

namespace rcp {

constexpr int MG_THREADS = 512;
constexpr int MG_WAVES = MG_THREADS / 64;
constexpr int MG_STRIDE = 65;  // LDS row stride in floats: conflict-free writes and reads

struct MgStage {
    u32x4 wa, wb;  // units 2*kb and 2*kb+1 of the group: 4 rows x 32 columns, planes interleaved per cell
    u32x4 xq;      // 32 int4 activations of this lane's token
    u32x4 lut;     // lanes 0..31: 16 bytes of the levels of (row group lane/2, this group)
};

// NARROW: the workgroup owns 4 row groups (16 output rows): the 16 rows of the A operand are (row group,
// row in the nibble) pairs as in gemm_mfma.hip, the mask and its E8M0 scale are per-lane values, and
// one instruction per plane and activation part covers all four rows of a nibble.
// WANTP: the per-group sums are written to Pout as well (a verification output: with its stores and branches in the
// loop the wide form needs 221 registers instead of 102, which leaves room for a single workgroup on a compute unit).
template <bool OUT_F16, bool NARROW, bool WANTP>
__global__ __launch_bounds__(MG_THREADS) void gemm_mfma_grouped_kernel(const uint4* __restrict__ packed,
                                                                       const uint4* __restrict__ codebook, int N, int K,
                                                                       const uint4* __restrict__ xq,
                                                                       const uint16_t* __restrict__ scale, int M, int W,
                                                                       void* __restrict__ out, int32_t* __restrict__ Pout)
{
    __shared__ float slab[MG_WAVES * 16 * MG_STRIDE];  // [wavefront][token][row of the block]
    __shared__ float4 coef_lds[MG_WAVES][64];          // [wavefront][row of the block]: coefficients of (T, F0, F1, F3)
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // (W, the wavefronts of the workgroup, is an argument: the launch dimensions would have to be fetched from memory)
    const int i = lane & 15, kb = lane >> 4;
    const int U = K / 16, G = N / 4, NG = K / RCP_GROUP;
    constexpr int RB = NARROW ? 16 : 64;   // output rows of the workgroup
    constexpr int RGB = RB / 4;            // its row groups
    const int rg = NARROW ? static_cast<int>(blockIdx.x) * 4 + (i >> 2) : static_cast<int>(blockIdx.x) * 16 + i;
    // NARROW: this lane's row of the nibble as a mask, the shift that brings the fourth row (the FP4 sign
    // bit) down, and the scale that undoes the mask's 0.5 / 1 / 2
    const uint32_t row_mask = (i & 3) == 0 ? 0x11111111u : (i & 3) == 1 ? 0x22222222u : 0x44444444u;
    const int row_shift = (i & 3) == 3 ? 1 : 0;
    const int row_scale = (i & 3) == 0 ? 0x80 : (i & 3) == 1 ? 0x7f : 0x7e;

    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint4*>(packed), 0, static_cast<int>(static_cast<unsigned>(G) * static_cast<unsigned>(U) * 16u), 0x00020000);
    const __amdgpu_buffer_rsrc_t cres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint4*>(codebook), 0, static_cast<int>(static_cast<unsigned>(G) * static_cast<unsigned>(NG) * 32u), 0x00020000);
    // tokens beyond M start beyond the end of the resource and read as zero
    const __amdgpu_buffer_rsrc_t xres =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4*>(xq), 0, M * (K / 2), 0x00020000);
    const unsigned row_base = rg < G ? static_cast<unsigned>(rg) * U * 16u : 0x80000000u;
    const unsigned xbase = static_cast<unsigned>(i) * (K / 2) + kb * 16u;
    // the piece of the levels this lane fetches: row group lane/2 of the block, half lane&1
    const int lut_rg = blockIdx.x * RGB + (lane >> 1);
    const unsigned lut_base = (lane < 2 * RGB && lut_rg < G) ? static_cast<unsigned>(lut_rg) * NG * 32u + (lane & 1) * 16u : 0x80000000u;

    auto load = [&](int group_index, MgStage& st) {
        const int g = __builtin_amdgcn_readfirstlane(group_index);  // uniform: scalar offsets
        const bool ok = g < NG;
        const int round = g >> 5;
        const int R = min(32, NG - 32 * round);
        const unsigned pos = 256u * round + 2u * kb * R + (g & 31);  // unit 2*kb of group g; unit 2*kb+1 is R further
        const unsigned wo = (ok && row_base != 0x80000000u) ? row_base + pos * 16u : 0x80000000u;
        st.wa = __builtin_amdgcn_raw_buffer_load_b128(wres, static_cast<int>(wo), 0, 0);
        st.wb = __builtin_amdgcn_raw_buffer_load_b128(wres, static_cast<int>(wo), ok ? R * 16 : 0, 0);
        st.xq = __builtin_amdgcn_raw_buffer_load_b128(xres, static_cast<int>(ok ? xbase : 0x80000000u), ok ? g * 64 : 0, 0);
        st.lut = __builtin_amdgcn_raw_buffer_load_b128(cres, static_cast<int>((ok && lut_base != 0x80000000u) ? lut_base : 0x80000000u),
                                                       ok ? g * 32 : 0, 0);
    };

    MgStage sA, sB;
    int g = wave;  // this wavefront's current group
    load(g, sA);

    // [v][r]: output of row 4*(4*kb + v) + r of the block for token i; NARROW: [v][0], row 4*kb + v
    float o[4][4];
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int r = 0; r < 4; ++r) o[v][r] = 0.0f;

    // E8M0 scales (byte 0 is used): 2^1, 2^0, 2^-1 undo the 0.5 / 1 / 2 of the masked nibbles;
    // 2^2 weighs the high part of the activation
    constexpr int SC_A[4] = {0x80, 0x7f, 0x7e, 0x7e};
    constexpr int SC_ONE = 0x7f, SC_HI = 0x81;

    auto compute = [&](const MgStage& cur, int gcur) {
        if (lane < 2 * RGB) {
            // two rows: 4 * (lane / 2) + 2 * (lane & 1) and the next one
            const uint32_t lw[4] = {cur.lut.x, cur.lut.y, cur.lut.z, cur.lut.w};
#pragma unroll
            for (int rr = 0; rr < 2; ++rr) {
                const float c0 = half_bits_to_float(static_cast<uint16_t>(lw[2 * rr] & 0xffffu));
                const float c1 = half_bits_to_float(static_cast<uint16_t>(lw[2 * rr] >> 16));
                const float c2 = half_bits_to_float(static_cast<uint16_t>(lw[2 * rr + 1] & 0xffffu));
                const float c3 = half_bits_to_float(static_cast<uint16_t>(lw[2 * rr + 1] >> 16));
                coef_lds[wave][2 * lane + rr] = make_float4(c0, c1 - c0, c2 - c0, ((c3 - c2) - c1) + c0);
            }
        }
        const uint32_t xw[4] = {cur.xq.x, cur.xq.y, cur.xq.z, cur.xq.w};
        v8i blo = {0, 0, 0, 0, 0, 0, 0, 0}, bhi = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            blo[d] = static_cast<int>(fp4_lo(xw[d]));
            bhi[d] = static_cast<int>(fp4_hi(xw[d]));
        }
        const v4f zero = {0.0f, 0.0f, 0.0f, 0.0f};
        // sum of q over the group, for this lane's token (the same in all four registers)
        const v8i ones = {0x22222222, 0x22222222, 0x22222222, 0x22222222, 0, 0, 0, 0};
        v4f tq = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ones, blo, zero, 4, 4, 0, SC_ONE, 0, SC_ONE);
        tq = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ones, bhi, tq, 4, 4, 0, SC_ONE, 0, SC_HI);

        const uint32_t p0[4] = {cur.wa.x, cur.wa.z, cur.wb.x, cur.wb.z};
        const uint32_t p1[4] = {cur.wa.y, cur.wa.w, cur.wb.y, cur.wb.w};
        if constexpr (NARROW) {
            v4f acc[3][1];
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
                acc[p][0] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(an[p], blo, zero, 4, 4, 0, row_scale, 0, SC_ONE);
                acc[p][0] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(an[p], bhi, acc[p][0], 4, 4, 0, row_scale, 0, SC_HI);
            }
            const bool store_pn = WANTP && i < M && gcur < NG;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float4 c = coef_lds[wave][4 * kb + v];
                const float F0 = acc[0][0][v], F1 = acc[1][0][v], F3 = acc[2][0][v];
                float val = o[v][0];
                val = fmaf(c.x, tq[v], val);
                val = fmaf(c.y, F0, val);
                val = fmaf(c.z, F1, val);
                val = fmaf(c.w, F3, val);
                o[v][0] = val;
                if constexpr (WANTP) if (store_pn) {
                    const int h = 4 * (static_cast<int>(blockIdx.x) * 4 + kb) + v;
                    if (h < N)
                        reinterpret_cast<int4*>(Pout)[(static_cast<size_t>(i) * N + h) * NG + gcur] =
                            make_int4(static_cast<int>(tq[v] - F0 - F1 + F3), static_cast<int>(F0 - F3),
                                      static_cast<int>(F1 - F3), static_cast<int>(F3));
                }
            }
            return;
        }
        // one row of the nibble at a time: its three plane operands, six instructions, and the products with the
        // coefficients of its 16 rows of the block
        const bool store_p = WANTP && i < M && gcur < NG;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            v8i a[3];
#pragma unroll
            for (int p = 0; p < 3; ++p) a[p] = v8i{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const uint32_t m = r == 0 ? 0x11111111u : r == 1 ? 0x22222222u : 0x44444444u;
                a[0][d] = static_cast<int>((p0[d] >> (r == 3 ? 1 : 0)) & m);
                a[1][d] = static_cast<int>((p1[d] >> (r == 3 ? 1 : 0)) & m);
                a[2][d] = a[0][d] & a[1][d];  // the mask of b0 & b1
            }
            v4f ar[3];
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                ar[p] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[p], blo, zero, 4, 4, 0, SC_A[r], 0, SC_ONE);
                ar[p] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[p], bhi, ar[p], 4, 4, 0, SC_A[r], 0, SC_HI);
            }
            // plane sums (exact small integers in binary32) times the coefficients of (row, group)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float4 c = coef_lds[wave][4 * (4 * kb + v) + r];
                const float F0 = ar[0][v], F1 = ar[1][v], F3 = ar[2][v];
                float val = o[v][r];
                val = fmaf(c.x, tq[v], val);
                val = fmaf(c.y, F0, val);
                val = fmaf(c.z, F1, val);
                val = fmaf(c.w, F3, val);
                o[v][r] = val;
                if constexpr (WANTP) if (store_p) {
                    const int h = 4 * (blockIdx.x * 16 + 4 * kb + v) + r;
                    if (h < N)
                        reinterpret_cast<int4*>(Pout)[(static_cast<size_t>(i) * N + h) * NG + gcur] =
                            make_int4(static_cast<int>(tq[v] - F0 - F1 + F3), static_cast<int>(F0 - F3),
                                      static_cast<int>(F1 - F3), static_cast<int>(F3));
                }
            }
            __builtin_amdgcn_sched_barrier(0);  // rows are not interleaved: one row's operands and sums live at a time
        }
    };
    // Two register sets alternate: the next group's loads are in flight while the current one is
    // computed.  Groups past the end of K read zeros and add zeros.
    auto stage = [&](const MgStage& cur, MgStage& next) {
        load(g + W, next);
        // nothing that needs `cur` may move above the loads just issued
        __builtin_amdgcn_sched_barrier(0);
        compute(cur, g);
        g += W;
    };
    while (true) {
        stage(sA, sB);
        if (g >= NG) break;
        stage(sB, sA);
        if (g >= NG) break;
    }
    // The last stage loaded (zeros) is "used" here on purpose: without a use on the exit path the
    // optimiser sinks each stage's loads below the exit test and the loop is no longer pipelined.
    const uint32_t keep = sA.wa.x | sA.wb.x | sA.xq.x | sA.lut.x | sB.wa.x | sB.wb.x | sB.xq.x | sB.lut.x;
    if (__builtin_expect(K < 0, 0)) slab[0] = __uint_as_float(keep);  // never true

    if constexpr (NARROW) {
        float* dst = slab + (wave * 16 + i) * MG_STRIDE + 4 * kb;
#pragma unroll
        for (int v = 0; v < 4; ++v) dst[v] = o[v][0];
    } else {
        float* dst = slab + (wave * 16 + i) * MG_STRIDE + 16 * kb;
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int r = 0; r < 4; ++r) dst[4 * v + r] = o[v][r];
    }
    __syncthreads();

    for (int idx = tid; idx < M * RB; idx += 64 * W) {
        const int n = idx / RB, hh = idx % RB;
        const int h = blockIdx.x * RB + hh;
        if (h >= N) continue;
        float val = 0.0f;
        for (int w = 0; w < W; ++w) val += slab[(w * 16 + n) * MG_STRIDE + hh];  // fixed order
        val *= half_bits_to_float(scale[n]);
        const size_t oi = static_cast<size_t>(n) * N + h;
        if constexpr (OUT_F16) static_cast<__half*>(out)[oi] = __float2half_rn(val);
        else static_cast<float*>(out)[oi] = val;
    }
}

int launch_gemm_mfma_grouped(const void* packed, const void* codebook, int N, int K, const void* xq,
                             const void* scale, int M, void* out, rcp_dtype out_dt, int32_t* P, hipStream_t st)
{
    if (static_cast<long long>(N) * K / 4 >= (1LL << 31))
        return fail(RCP_ERR_SHAPE, "rcp_w2a4_gemm_grouped: packed matrix of %lld bytes exceeds 2 GiB",
                    static_cast<long long>(N) * K / 4);
    // 16-row workgroups when 64-row ones would leave most compute units idle ("gemm_rows" = 16 / 64 forces a form)
    bool narrow = (N + 63) / 64 < num_compute_units() / 2;
    if (options().gemm_rows != 0) narrow = options().gemm_rows == 16;
    const int blocks = narrow ? (N + 15) / 16 : (N + 63) / 64;
    const int NG = K / RCP_GROUP;
    int waves = MG_WAVES;
    if (options().gemm_waves != 0) waves = options().gemm_waves;
    while (waves > 1 && waves > NG) waves /= 2;
    auto* pk = static_cast<const uint4*>(packed);
    auto* cb = static_cast<const uint4*>(codebook);
    auto* x4 = static_cast<const uint4*>(xq);
    auto* sc = static_cast<const uint16_t*>(scale);
#define RCP_MG(F16, NA)                                                                                                  \
    do {                                                                                                                 \
        if (P != nullptr) gemm_mfma_grouped_kernel<F16, NA, true><<<blocks, waves * 64, 0, st>>>(pk, cb, N, K, x4, sc, M, waves, out, P); \
        else gemm_mfma_grouped_kernel<F16, NA, false><<<blocks, waves * 64, 0, st>>>(pk, cb, N, K, x4, sc, M, waves, out, P);             \
    } while (0)
    if (narrow) {
        if (out_dt == RCP_F16) RCP_MG(true, true);
        else RCP_MG(false, true);
    } else {
        if (out_dt == RCP_F16) RCP_MG(true, false);
        else RCP_MG(false, false);
    }
#undef RCP_MG
    return check_launch("rcp_w2a4_gemm_grouped");
}

}  // namespace rcp
