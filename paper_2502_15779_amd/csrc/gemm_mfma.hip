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
// v_mfma_scale_f32_16x16x128_f8f6f4 for rows r = 0, 1, 2 (and (w >> 1) & 0x4444.. for r = 3)
// without any expansion; the per-lane E8M0 scale of the instruction (2^1, 2^0, 2^-1) turns the
// 0.5 / 1 / 2 back into 1.  The int4 activation q = 4*hi + lo, lo in {0..3}, hi in {-2..1}, is
// recoded into two FP4 operands (lo, and hi with scale 2^2); both accumulate into the same
// registers.  Every product and every sum is a small integer, so the fp32 accumulators hold
// the exact integer F_p (|F_p| <= 8K < 2^24) and the per-level sums stay bit-exact.
//
// Work decomposition.  A workgroup owns 16 groups of four rows (64 output rows): lane l of a
// wavefront supplies row group l%16 and the 32 columns of K-block l/16 of a 128-column step
// (two 16-byte units), and token l%16 for the B operand.  The wavefronts of the workgroup take
// the 128-column steps of K in turn and add their accumulators into LDS at the end, where the
// epilogue (per-level sums -> LUT -> scale) runs once per (token, row).
#include "rcp_internal.hpp"

namespace rcp {

constexpr int MM_MAX_THREADS = 512;
constexpr int MM_PF = 4;            // K steps in flight per wavefront
constexpr int MM_STRIDE = 65;       // LDS row stride (ints): conflict-free for both phases
constexpr int MM_PLANE = 16 * MM_STRIDE;
constexpr int MM_LDS_INTS = 3 * MM_PLANE + 16;

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

struct MmStage {
    u32x4 wa, wb;  // two units: 4 rows x 32 columns, bit planes b0 / b1 interleaved per cell
    u32x4 xq;      // 32 int4 activations of this lane's token
};

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

template <bool OUT_F16>
__global__ __launch_bounds__(MM_MAX_THREADS) void gemm_mfma_kernel(const uint4* __restrict__ packed,
                                                                   const uint2* __restrict__ codebook, int N, int K,
                                                                   const uint4* __restrict__ xq,
                                                                   const uint16_t* __restrict__ scale, int M,
                                                                   void* __restrict__ out, int32_t* __restrict__ Pout)
{
    __shared__ int red[MM_LDS_INTS];  // F sums [plane][token][row of the block], then T[token]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int W = static_cast<int>(blockDim.x) >> 6;
    const int i = lane & 15, kb = lane >> 4;
    const int U = K / 16, G = N / 4;
    const int KS = (K + 127) >> 7;  // steps of 128 columns
    const int rg = blockIdx.x * 16 + i;

    for (int j = tid; j < MM_LDS_INTS; j += blockDim.x) red[j] = 0;

    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint4*>(packed), 0, static_cast<int>(static_cast<unsigned>(G) * static_cast<unsigned>(U) * 16u), 0x00020000);
    // tokens beyond M start beyond the end of the resource and read as zero
    const __amdgpu_buffer_rsrc_t xres =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4*>(xq), 0, M * (K / 2), 0x00020000);
    const unsigned wbase = rg < G ? (static_cast<unsigned>(rg) * U + 2u * kb) * 16u : 0x80000000u;
    const unsigned xbase = static_cast<unsigned>(i) * (K / 2) + kb * 16u;

    auto load = [&](int s, MmStage& st) {
        const bool ok = 8 * s + 2 * kb < U;  // false for the K tail and for steps past the end
        const unsigned wo = ok ? wbase : 0x80000000u;
        const unsigned xo = ok ? xbase : 0x80000000u;
        st.wa = __builtin_amdgcn_raw_buffer_load_b128(wres, static_cast<int>(wo), s * 128, 0);
        st.wb = __builtin_amdgcn_raw_buffer_load_b128(wres, static_cast<int>(wo), s * 128 + 16, 0);
        st.xq = __builtin_amdgcn_raw_buffer_load_b128(xres, static_cast<int>(xo), s * 64, 0);
    };

    MmStage st[MM_PF];
#pragma unroll
    for (int j = 0; j < MM_PF; ++j) load(wave + j * W, st[j]);
    __syncthreads();  // LDS is zero before anyone adds to it

    v4f acc[3][4];
#pragma unroll
    for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[p][r] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
    int tsum = 0;

    // E8M0 scales (byte 0 is used): 2^1, 2^0, 2^-1 undo the 0.5 / 1 / 2 of the masked nibbles;
    // 2^2 weighs the high part of the activation
    constexpr int SC_A[4] = {0x80, 0x7f, 0x7e, 0x7e};
    constexpr int SC_LO = 0x7f, SC_HI = 0x81;

    for (int s0 = wave; s0 < KS; s0 += MM_PF * W) {
#pragma unroll
        for (int j = 0; j < MM_PF; ++j) {
            const int s = s0 + j * W;
            if (s < KS) {  // uniform per wavefront
            const MmStage cur = st[j];
            load(s + MM_PF * W, st[j]);

            const uint32_t xw[4] = {cur.xq.x, cur.xq.y, cur.xq.z, cur.xq.w};
            v8i blo = {0, 0, 0, 0, 0, 0, 0, 0}, bhi = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                blo[d] = static_cast<int>(fp4_lo(xw[d]));
                bhi[d] = static_cast<int>(fp4_hi(xw[d]));
                tsum = dot8(xw[d], 0x11111111u, tsum);
            }
            const uint32_t p0[4] = {cur.wa.x, cur.wa.z, cur.wb.x, cur.wb.z};
            const uint32_t p1[4] = {cur.wa.y, cur.wa.w, cur.wb.y, cur.wb.w};
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                v8i a[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) a[r] = v8i{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const uint32_t w = p == 0 ? p0[d] : p == 1 ? p1[d] : (p0[d] & p1[d]);
                    a[0][d] = static_cast<int>(w & 0x11111111u);
                    a[1][d] = static_cast<int>(w & 0x22222222u);
                    a[2][d] = static_cast<int>(w & 0x44444444u);
                    a[3][d] = static_cast<int>((w >> 1) & 0x44444444u);
                }
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[p][r] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[r], blo, acc[p][r], 4, 4, 0, SC_A[r], 0, SC_LO);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[p][r] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[r], bhi, acc[p][r], 4, 4, 0, SC_A[r], 0, SC_HI);
            }
            }
        }
    }

    // acc[p][r][v] = F_p of row 4*(16*block + 4*kb + v) + r and token i: add over the wavefronts
    {
        int* dst = red + i * MM_STRIDE + 16 * kb;
#pragma unroll
        for (int p = 0; p < 3; ++p)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    atomicAdd(dst + p * MM_PLANE + 4 * v + r, static_cast<int>(acc[p][r][v]));
        atomicAdd(red + 3 * MM_PLANE + i, tsum);
    }
    __syncthreads();

    for (int o = tid; o < M * 64; o += blockDim.x) {
        const int n = o >> 6, hh = o & 63;
        const int h = blockIdx.x * 64 + hh;
        if (h >= N) continue;
        const int F0 = red[n * MM_STRIDE + hh], F1 = red[MM_PLANE + n * MM_STRIDE + hh];
        const int F3 = red[2 * MM_PLANE + n * MM_STRIDE + hh];
        const int T = red[3 * MM_PLANE + n];
        const int P3 = F3, P1 = F0 - F3, P2 = F1 - F3, P0 = T - F0 - F1 + F3;
        const uint2 lut = codebook[h];
        const float c0 = half_bits_to_float(static_cast<uint16_t>(lut.x & 0xffffu));
        const float c1 = half_bits_to_float(static_cast<uint16_t>(lut.x >> 16));
        const float c2 = half_bits_to_float(static_cast<uint16_t>(lut.y & 0xffffu));
        const float c3 = half_bits_to_float(static_cast<uint16_t>(lut.y >> 16));
        float val = c0 * static_cast<float>(P0);
        val = fmaf(c1, static_cast<float>(P1), val);
        val = fmaf(c2, static_cast<float>(P2), val);
        val = fmaf(c3, static_cast<float>(P3), val);
        val *= half_bits_to_float(scale[n]);
        const size_t oi = static_cast<size_t>(n) * N + h;
        if constexpr (OUT_F16) static_cast<__half*>(out)[oi] = __float2half_rn(val);
        else static_cast<float*>(out)[oi] = val;
        if (Pout != nullptr) reinterpret_cast<int4*>(Pout)[oi] = make_int4(P0, P1, P2, P3);
    }
}

int launch_gemm_mfma(const void* packed, const void* codebook, int N, int K, const void* xq, const void* scale,
                     int M, void* out, rcp_dtype out_dt, int32_t* P, hipStream_t st)
{
    const int blocks = (N + 63) / 64;
    const int KS = (K + 127) / 128;
    // enough wavefronts to occupy the chip: 4 or 8 per workgroup, never more than there are K steps
    int waves = blocks * 4 >= 4 * num_compute_units() ? 4 : 8;
    if (options().gemm_waves != 0) waves = options().gemm_waves;
    while (waves > 1 && waves > KS) waves /= 2;
    auto* pk = static_cast<const uint4*>(packed);
    auto* cb = static_cast<const uint2*>(codebook);
    auto* x4 = static_cast<const uint4*>(xq);
    auto* sc = static_cast<const uint16_t*>(scale);
    if (out_dt == RCP_F16)
        gemm_mfma_kernel<true><<<blocks, waves * 64, 0, st>>>(pk, cb, N, K, x4, sc, M, out, P);
    else
        gemm_mfma_kernel<false><<<blocks, waves * 64, 0, st>>>(pk, cb, N, K, x4, sc, M, out, P);
    return check_launch("rcp_w2a4_gemv");
}

}  // namespace rcp
