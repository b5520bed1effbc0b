// One-token W2A4 GEMV (Section 4.4), the form for matrices that give a wavefront a single row group:
// every weight load of the workgroup is issued at the very start of the kernel, before the activations are
// staged, so that the whole matrix is in flight at once and no wavefront waits for a second round trip to
// memory.  (The general kernel of gemv.hip keeps two stages of loads in flight and asks for the next one only
// when a stage has been consumed; with more than two stages per row group its later ones start a full memory
// latency late.  With several row groups per wavefront the general kernel stays ahead: a compute unit's memory
// pipeline takes loads in issue order, so a wavefront that has asked for everything up front cannot start its
// prologue until the pipeline has accepted all of it, and the activation loads of the compute unit's second
// workgroup queue behind the first one's weights -- measured with per-wavefront timestamps.)
//
// Arithmetic, data layout, reduction and epilogue are those of gemv_kernel: exact integer per-level sums
// through the Walsh basis of the 2-bit index, four rows per nibble, v_dot8_i32_i4, lane-swap reduction, one
// binary32 epilogue per row.  The results are bit-identical to gemv_kernel's (integer sums are exact and the
// epilogue is the same sequence of binary32 operations).
//
// Work decomposition: one wavefront per row group; lane t takes units t, t + 64, ..., at most UPL of them
// (64 * UPL >= K / 16); workgroup b of four wavefronts takes row groups 4b .. 4b + 3.
#include <math.h>

#include "rcp_internal.hpp"

namespace rcp {

constexpr int ONE_XG = 8;     // groups of eight raw activations a thread can hold in the fused quantiser: K <= 16384
constexpr int ONE_WAVES = 4;  // wavefronts (= row groups) per workgroup

// XDT < 0: x_in holds the quantised activations (K/2 bytes) and `scale` their scale.
// XDT = RCP_F16 / RCP_F32 / RCP_BF16: x_in is the raw activation; the workgroup quantises it itself exactly as
// quant_kernel would, and the first workgroup publishes x_q and S when xq_out / scale_out are given.
// The first 56 bytes of arguments reach the wavefront in scalar registers at launch.
// NT: the weight loads carry the non-temporal hint (see the launcher).
template <int UPL, int XDT, bool NT = false>
__global__ __launch_bounds__(ONE_WAVES * 64) void gemv_oneshot_kernel(const uint4* __restrict__ packed,
                                                                      const uint2* __restrict__ codebook, int N, int K,
                                                                      const void* __restrict__ x_in,
                                                                      const uint16_t* __restrict__ scale, int out_f16,
                                                                      float clip_ratio, void* __restrict__ out,
                                                                      int32_t* __restrict__ Pout, uint32_t* __restrict__ xq_out,
                                                                      uint16_t* __restrict__ scale_out)
{
    constexpr int NW = ONE_WAVES;
    constexpr int TH = NW * 64;
    constexpr int XT = XDT >= 0 ? XDT : 0;
    extern __shared__ uint4 smem4[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int U = K / 16, G = N / 4;
    const int xdw = K / 8;
    const int units = (U + 63) / 64;  // units per lane (the last one may be ragged)
    const int my_row = lane_row<64>(lane);
    const int my_units = (U - lane + 63) / 64;
    const int g = static_cast<int>(blockIdx.x) * NW + wave;  // this wavefront's row group

    // one resource over the whole matrix: an offset past its end reads zeros without touching memory
    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint4*>(packed), 0, static_cast<int>(static_cast<unsigned>(G) * static_cast<unsigned>(U) * 16u), 0x00020000);

    // ---- 1. the activations (memory answers in issue order: what the prologue needs goes first)
    const int per_token = xdw / 4;
    u32x4 xfirst[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};  // quantised activations: up to 32 bytes per thread
    uint16_t scb = 0;
    Raw8<XT> xraw8[XDT >= 0 ? ONE_XG : 1];
    if constexpr (XDT < 0) {
        const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(x_in), 0, per_token * 16, 0x00020000);
        xfirst[0] = __builtin_amdgcn_raw_buffer_load_b128(xr, static_cast<int>(threadIdx.x) * 16, 0, 0);
        if (per_token > TH)  // uniform
            xfirst[1] = __builtin_amdgcn_raw_buffer_load_b128(xr, (static_cast<int>(threadIdx.x) + TH) * 16, 0, 0);
        scb = scale[0];
    } else {
#pragma unroll
        for (int i = 0; i < ONE_XG; ++i) {
            if (i * TH >= xdw) break;  // uniform
            const int u8 = min(static_cast<int>(threadIdx.x) + i * TH, xdw - 1);  // clamped: duplicates are harmless
            xraw8[i] = load8_raw<XT>(x_in, static_cast<size_t>(u8) * 8);
        }
    }
    // ---- 2. the LUT row (ahead of the weights: memory answers in order, and it is needed last)
    const uint2 lut = codebook[min(4 * g + my_row, N - 1)];
    __builtin_amdgcn_sched_barrier(0);
    // ---- 3. every weight load of this wavefront
    u32x4 w[UPL];
    {
        const unsigned base = (static_cast<unsigned>(g) * U + lane) * 16u;  // beyond the matrix for a row group >= G
#pragma unroll
        for (int i = 0; i < UPL; ++i) {
            const unsigned off = i < my_units ? base : 0x80000000u;
            w[i] = __builtin_amdgcn_raw_buffer_load_b128(wres, static_cast<int>(off), i * 64 * 16, NT ? 2 : 0);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    // the arguments that did not arrive in registers are fetched here, while the loads are in flight
    asm volatile("" ::"s"(out), "s"(Pout), "s"(xq_out), "s"(scale_out));

    // ---- 4. stage the activations in LDS and sum them: T = sum_k q[k]
    constexpr int x_bytes = UPL * 64 * 8;  // padded: a lane whose unit lies beyond K reads garbage times zero weights
    int* tsum = reinterpret_cast<int*>(reinterpret_cast<char*>(smem4) + x_bytes);  // [NW]
    float sc;
    if constexpr (XDT < 0) {
        sc = half_bits_to_float(scb);
        u32x4* sx4 = reinterpret_cast<u32x4*>(smem4);
        int s = 0;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if (h * TH >= per_token) break;  // uniform
            // a piece beyond the end was read as zero and is not stored
            if (static_cast<int>(threadIdx.x) + h * TH < per_token) sx4[threadIdx.x + h * TH] = xfirst[h];
            s = dot8(xfirst[h].x, 0x11111111u, s);
            s = dot8(xfirst[h].y, 0x11111111u, s);
            s = dot8(xfirst[h].z, 0x11111111u, s);
            s = dot8(xfirst[h].w, 0x11111111u, s);
        }
        s = wave_sum(s);
        if (lane == 0) tsum[wave] = s;
    } else {
        float xr8[ONE_XG][8];
#pragma unroll
        for (int i = 0; i < ONE_XG; ++i) {
            if (i * TH >= xdw) break;
            widen8<XT>(xraw8[i], xr8[i]);
        }
        float a = 0.0f;
#pragma unroll
        for (int i = 0; i < ONE_XG; ++i) {
            if (i * TH >= xdw) break;
#pragma unroll
            for (int j = 0; j < 8; ++j) a = fmaxf(a, fabsf(xr8[i][j]));
        }
        a = wave_max(a);
        float* amax_slots = reinterpret_cast<float*>(tsum + NW);
        if (lane == 0) amax_slots[wave] = a;
        __syncthreads();
        a = fmaxf(fmaxf(amax_slots[0], amax_slots[1]), fmaxf(amax_slots[2], amax_slots[3]));
        const uint16_t sb = scale_bits_from_amax(a, clip_ratio);
        sc = half_bits_to_float(sb);
        uint32_t* sx1 = reinterpret_cast<uint32_t*>(smem4);
        const bool publish = blockIdx.x == 0 && xq_out != nullptr;
        int s = 0;
        // all groups of eight are rounded first, without branches, so that their instruction chains interleave
        // (a thread past the end of the token works on a duplicate of the last group and stores nothing)
        uint32_t qd[ONE_XG];
        const float rs = __frcp_rn(sc);
        // fp16 / bf16 values straight from memory take the form of the quantiser that needs no second pass
        constexpr bool SHORT_IN = (XT == RCP_F16 || XT == RCP_BF16);
        float far = 0.0f;
#pragma unroll
        for (int i = 0; i < ONE_XG; ++i) {
            if (i * TH >= xdw) break;
            qd[i] = SHORT_IN ? quantize8_short(xr8[i], sc, rs) : quantize8_fast(xr8[i], rs, far);
        }
        if (!SHORT_IN && __builtin_expect(far > 0.49999f, 0)) {
#pragma unroll
            for (int i = 0; i < ONE_XG; ++i) {
                if (i * TH >= xdw) break;
                qd[i] = quantize8_exact(xr8[i], sc);
            }
        }
#pragma unroll
        for (int i = 0; i < ONE_XG; ++i) {
            if (i * TH >= xdw) break;
            const int u8 = threadIdx.x + i * TH;
            if (u8 < xdw) {
                sx1[u8] = qd[i];
                s = dot8(qd[i], 0x11111111u, s);
            }
        }
        if (publish) {
#pragma unroll
            for (int i = 0; i < ONE_XG; ++i) {
                if (i * TH >= xdw) break;
                const int u8 = threadIdx.x + i * TH;
                if (u8 < xdw) xq_out[u8] = qd[i];
            }
        }
        if (blockIdx.x == 0 && threadIdx.x == 0 && scale_out != nullptr) scale_out[0] = sb;
        s = wave_sum(s);
        if (lane == 0) tsum[wave] = s;
    }
    __syncthreads();
    const int T = tsum[0] + tsum[1] + tsum[2] + tsum[3];

    // ---- 5. the dot products, in the order the loads were issued
    const uint2* sx2 = reinterpret_cast<const uint2*>(smem4);
    int acc[1][3][4];
#pragma unroll
    for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int m = 0; m < 4; ++m) acc[0][p][m] = 0;
#pragma unroll
    for (int i = 0; i < UPL; ++i) {
        if (i < units) {  // uniform
            const uint2 xv = sx2[lane + i * 64];
            const uint32_t xa[1] = {xv.x}, xb[1] = {xv.y};
            cell_update<1>(w[i].x, w[i].y, xa, acc);
            cell_update<1>(w[i].z, w[i].w, xb, acc);
        }
    }
    // the triangular solve is linear: applied per lane before the reduction
    int g12[12], fsum[3];
#pragma unroll
    for (int p = 0; p < 3; ++p) {
        g12[4 * p + 0] = acc[0][p][0];
        g12[4 * p + 1] = acc[0][p][1] - acc[0][p][0];
        g12[4 * p + 2] = acc[0][p][2] - acc[0][p][1];
        g12[4 * p + 3] = acc[0][p][2] - acc[0][p][3];
    }
    reduce_rows<64>(g12, lane, fsum);
    if (g < G && lane_writes<64>(lane)) {
        const int r = my_row;
        const int h = 4 * g + r;
        const float c0 = half_bits_to_float(static_cast<uint16_t>(lut.x & 0xffffu));
        const float c1 = half_bits_to_float(static_cast<uint16_t>(lut.x >> 16));
        const float c2 = half_bits_to_float(static_cast<uint16_t>(lut.y & 0xffffu));
        const float c3 = half_bits_to_float(static_cast<uint16_t>(lut.y >> 16));
        const int F0 = fsum[0] >> r, F1 = fsum[1] >> r, F3 = fsum[2] >> r;
        const int P3 = F3, P1 = F0 - F3, P2 = F1 - F3;
        const int P0 = T - F0 - F1 + F3;
        float o = c0 * static_cast<float>(P0);
        o = fmaf(c1, static_cast<float>(P1), o);
        o = fmaf(c2, static_cast<float>(P2), o);
        o = fmaf(c3, static_cast<float>(P3), o);
        o *= sc;
        if (out_f16) static_cast<__half*>(out)[h] = round_to_half(o);
        else static_cast<float*>(out)[h] = o;
        if (Pout != nullptr) reinterpret_cast<int4*>(Pout)[h] = make_int4(P0, P1, P2, P3);
    }
}

// Units per lane of the instantiated forms; 0 when the row is too long (K > 16384).
static int oneshot_upl(int K)
{
    const int units = (K / 16 + 63) / 64;
    for (int c : {2, 4, 8, 12, 16})
        if (units <= c) return c;
    return 0;
}

// One row group per wavefront, at least one workgroup per compute unit and at most two; with the quantiser in the
// prologue only up to K = 8192 (beyond that the quantiser of the 256 threads outlasts the loads either way and the
// general kernel's smaller register footprint wins: 4096 x 14336 binary32 6.4 vs 6.9 us).
bool gemv_oneshot_applies(int N, int K, bool fused)
{
    const Options& opt = options();
    if (opt.gemv_oneshot == 2 || opt.gemv_lanes != 0 || opt.gemv_blocks != 0 || opt.gemv_unroll != 0) return false;
    if (K / 16 < 64 || oneshot_upl(K) == 0) return false;
    if (opt.gemv_oneshot == 1) return true;
    const int nbatch = (N / 4 + ONE_WAVES - 1) / ONE_WAVES;
    const int cus = num_compute_units();
    if (nbatch < cus) return false;
    // activations quantised beforehand: any number of workgroups per compute unit once a row group is four loads or more
    // per lane -- the queue of short workgroups keeps the loads coming to the end (sweeps: 14336 x 4096 5.1 -> 4.8 us,
    // 22016 x 4096 6.2 -> 6.0, 28672 x 4096 7.5 -> 6.9, 16384 x 4096 5.5 -> 5.0, 12288 x 8192 6.6 -> 6.2; K = 2048 level) --
    // up to the size from which the general kernel's non-temporal form takes over
    if (!fused && K >= 4096 && static_cast<long long>(N) * K / 4 < (32LL << 20)) return true;
    // otherwise at most two workgroups per unit: with the quantiser in the prologue every further workgroup repeats it
    if (nbatch > 2 * cus) return false;
    return !fused || K <= 8192;
}

template <int UPL, int XDT>
static int launch_oneshot_one(const void* packed, const void* codebook, int N, int K, const void* x, const void* scale,
                              float clip_ratio, void* out, rcp_dtype out_dt, int32_t* P, void* xq_out, void* scale_out, hipStream_t st)
{
    const size_t lds = static_cast<size_t>(UPL) * 64 * 8 + 2 * ONE_WAVES * sizeof(int);
    const int blocks = (N / 4 + ONE_WAVES - 1) / ONE_WAVES;
    auto launch = [&](auto kernel) {
        kernel<<<blocks, ONE_WAVES * 64, lds, st>>>(
            static_cast<const uint4*>(packed), static_cast<const uint2*>(codebook), N, K, x, static_cast<const uint16_t*>(scale),
            out_dt == RCP_F16 ? 1 : 0, clip_ratio, out, P, static_cast<uint32_t*>(xq_out), static_cast<uint16_t*>(scale_out));
    };
    // Non-temporal weight loads from 8 MB of packed weights on, as in the general kernel ("gemv_nt": 1 = always,
    // 2 = never): judged inside a decode step, not on a sweep of this kernel.
    const bool nt = options().gemv_nt != 0 ? options().gemv_nt == 1 : static_cast<long long>(N) * K / 4 >= (8LL << 20);
    if (nt) launch(&gemv_oneshot_kernel<UPL, XDT, true>);
    else launch(&gemv_oneshot_kernel<UPL, XDT, false>);
    return check_launch("rcp_w2a4_gemv");
}

template <int XDT>
static int launch_oneshot_upl(const void* packed, const void* codebook, int N, int K, const void* x, const void* scale,
                              float clip_ratio, void* out, rcp_dtype out_dt, int32_t* P, void* xq_out, void* scale_out, hipStream_t st)
{
    switch (oneshot_upl(K)) {
        case 2: return launch_oneshot_one<2, XDT>(packed, codebook, N, K, x, scale, clip_ratio, out, out_dt, P, xq_out, scale_out, st);
        case 4: return launch_oneshot_one<4, XDT>(packed, codebook, N, K, x, scale, clip_ratio, out, out_dt, P, xq_out, scale_out, st);
        case 8: return launch_oneshot_one<8, XDT>(packed, codebook, N, K, x, scale, clip_ratio, out, out_dt, P, xq_out, scale_out, st);
        case 12: return launch_oneshot_one<12, XDT>(packed, codebook, N, K, x, scale, clip_ratio, out, out_dt, P, xq_out, scale_out, st);
        case 16: return launch_oneshot_one<16, XDT>(packed, codebook, N, K, x, scale, clip_ratio, out, out_dt, P, xq_out, scale_out, st);
        default: return fail(RCP_ERR_UNSUPPORTED, "rcp_w2a4_gemv: K = %d is outside the one-shot kernel", K);
    }
}

// x_dt < 0: x holds quantised activations and `scale` their scale; otherwise x is the raw activation of that type.
int launch_gemv_oneshot(const void* packed, const void* codebook, int N, int K, const void* x, int x_dt, const void* scale,
                        float clip_ratio, void* out, rcp_dtype out_dt, int32_t* P, void* xq_out, void* scale_out, hipStream_t st)
{
    if (x_dt < 0) return launch_oneshot_upl<-1>(packed, codebook, N, K, x, scale, clip_ratio, out, out_dt, P, xq_out, scale_out, st);
    if (x_dt == RCP_F16) return launch_oneshot_upl<RCP_F16>(packed, codebook, N, K, x, scale, clip_ratio, out, out_dt, P, xq_out, scale_out, st);
    if (x_dt == RCP_F32) return launch_oneshot_upl<RCP_F32>(packed, codebook, N, K, x, scale, clip_ratio, out, out_dt, P, xq_out, scale_out, st);
    return launch_oneshot_upl<RCP_BF16>(packed, codebook, N, K, x, scale, clip_ratio, out, out_dt, P, xq_out, scale_out, st);
}

}  // namespace rcp
