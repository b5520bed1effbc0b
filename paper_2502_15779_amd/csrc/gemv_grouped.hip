// W2A4 GEMV with group-wise look-up tables: every (output row, 128 input channels) has its own
// four levels (Appendix table of quantisation configurations: weight group size 128; Section
// 4.4: the LUT has N*4 entries per row for N groups per channel).  One token.
//
//     P[h][g][l] = sum_{k in group g : idx[h][k] = l} q[k]            (int32, exact)
//     O[h]       = S * sum_g sum_l LUT[h][g][l] * P[h][g][l]          (fp32)
//
// The integer part is the bit-plane / v_dot8 scheme of gemv.hip.  What changes is where a
// sum may cross lanes: levels differ from group to group, so a lane keeps a whole group to
// itself, turns its twelve dot-product accumulators into the per-level sums of the four rows,
// multiplies them with the group's levels and adds the four fp32 results to running row
// totals.  Only those four floats per lane are reduced across lanes, once per row group.
//
// Work decomposition.  32 lanes share one group of four rows, so a wavefront works on two row
// groups and a workgroup on eight.  Lane l takes the groups l, l + 32, l + 64, ... ("rounds").
// The grouped packed layout stores unit i (0..7) of the R groups of a round at unit position
// 256*round + i*R + l, so the eight 16-byte loads of a lane are each contiguous across the
// lanes; the quantised activations are staged into LDS in the same order.  The loop over
// (row-group batch, round) is software pipelined exactly like the per-channel kernel: the
// eight weight loads and the 32 bytes of levels of the next step are in flight while the
// current step is computed.
#include "rcp_internal.hpp"

namespace rcp {

constexpr int GG_THREADS = 256;
constexpr int GG_GROUP = 128;   // input channels per quantisation unit
constexpr int GG_UNITS = 8;     // 16-byte units per (row group, quantisation group)

template <int UPL>
struct GroupStep {
    u32x4 w[UPL];   // this lane's units of its group: 4 rows x 16 columns each
    u32x4 lut[2];   // levels of rows 0,1 | rows 2,3 (four fp16 each)
};

// LDS: activations in grouped unit order (one uint2 per unit, padded by 32 so that idle lanes
// of a short round read inside the allocation), then the sums of q per half group.
__host__ __device__ constexpr size_t gemv_grouped_lds_bytes(int K)
{
    return static_cast<size_t>(K / 16 + 32) * 8 + static_cast<size_t>(K / GG_GROUP) * 8;
}

// XDT < 0: `xq` / `scale` are the quantised activations.  XDT = RCP_F16 / RCP_F32 / RCP_BF16:
// `xraw` is the raw activation (K <= 16384) and every workgroup quantises it itself with the
// arithmetic of quant_kernel (amax, S = fp16(ratio*amax/7), q = rint(x/S)); the first
// workgroup also writes x_q and S to xq_out / scale_out when those are given.
constexpr int GG_XU = 4;  // 16-value units of raw activations per thread: K <= 16384

// (The first 56 bytes of arguments reach the wavefront in scalar registers at launch: everything the
// prologue needs at once is among them.)
// NT: weight loads with the non-temporal hint (22016 x 4096 8.15 -> 7.95 us, 4096 x 11008 6.84 -> 6.67; the 5 MB of
// 4096 x 4096 are 11 % slower with it on a sweep of their own, but inside the decode step, where weights that bypass the
// caches leave the activations and tables in them, the hint on that launch too is worth 1.2 % of the step: on from 4 MB).
// LG: lanes per group of four rows.  32: a lane owns whole quantisation groups.  64 (matrices with too few rows to give
// every compute unit a workgroup otherwise): two lanes share a group, four units each -- the sum over levels is linear
// in the per-level sums, so each lane multiplies the sums over its own 64 columns by the group's levels and nothing but
// the four fp32 row totals ever crosses lanes (the per-group sums are put together only for the optional P output).
// WANTP: the per-group sums go to Pout as well (a verification output; its stores and exchanges stay out of the loop of
// the production instantiation).
template <bool OUT_F16, int XDT, bool NT = false, int LG = 32, bool WANTP = false>
__global__ __launch_bounds__(GG_THREADS) void gemv_grouped_kernel(const uint4* __restrict__ packed,
                                                                  const uint4* __restrict__ codebook, int N, int K,
                                                                  const void* __restrict__ xraw,
                                                                  const uint4* __restrict__ xq,
                                                                  const uint16_t* __restrict__ scale, float clip_ratio,
                                                                  int nblk,
                                                                  void* __restrict__ out, int32_t* __restrict__ Pout,
                                                                  uint32_t* __restrict__ xq_out,
                                                                  uint16_t* __restrict__ scale_out)
{
    extern __shared__ uint2 sx2[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int SPL = LG / 32;            // lanes that share a quantisation group
    constexpr int UPL = GG_UNITS / SPL;     // 16-byte units per lane and group
    constexpr int GG_SLOTS = GG_THREADS / LG;  // row groups a workgroup works on at a time
    const int ln = lane & 31;
    const int half = SPL == 2 ? lane >> 5 : 0;  // which units of the group this lane owns
    const int slot = SPL == 2 ? wave : wave * 2 + (lane >> 5);
    const int U = K / 16, G = N / 4, NG = K / GG_GROUP;
    const int nround = (NG + 31) >> 5;
    const int nbatch = (G + GG_SLOTS - 1) / GG_SLOTS;
    // (nblk, the number of workgroups, is an argument: the launch dimensions would have to be fetched from memory)
    int* tgs = reinterpret_cast<int*>(sx2 + U + 32);

    // Buffer resources: an offset past the end is answered with zeros, so neither idle lanes
    // nor row groups beyond N need a branch.
    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint4*>(packed), 0, static_cast<int>(static_cast<unsigned>(G) * static_cast<unsigned>(U) * 16u), 0x00020000);
    const __amdgpu_buffer_rsrc_t cres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint4*>(codebook), 0, static_cast<int>(static_cast<unsigned>(G) * static_cast<unsigned>(NG) * 32u), 0x00020000);
    const __amdgpu_buffer_rsrc_t xres =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4*>(xq), 0, K / 2, 0x00020000);

    auto load_step = [&](int b, int rd, GroupStep<UPL>& s) {
        const int rg = b * GG_SLOTS + slot;
        const int R = min(32, NG - 32 * rd);
        const bool valid = ln < R && rg < G;
        const unsigned woff = valid ? (static_cast<unsigned>(rg) * U + 256u * rd + half * UPL * R + ln) * 16u : 0x80000000u;
#pragma unroll
        for (int i = 0; i < UPL; ++i)
            s.w[i] = __builtin_amdgcn_raw_buffer_load_b128(wres, static_cast<int>(woff), i * R * 16, NT ? 2 : 0);
        const unsigned coff = valid ? (static_cast<unsigned>(rg) * NG + 32u * rd + ln) * 32u : 0x80000000u;
        s.lut[0] = __builtin_amdgcn_raw_buffer_load_b128(cres, static_cast<int>(coff), 0, 0);
        s.lut[1] = __builtin_amdgcn_raw_buffer_load_b128(cres, static_cast<int>(coff), 16, 0);
    };

    // The pipeline runs two steps ahead: (b, rd) is the step being computed, (b1, rd1) and (b2, rd2)
    // the next two (the following round of 32 groups, else the first round of this workgroup's next
    // batch); the loads of the first two steps are issued before the activations are staged.
    int b = blockIdx.x, rd = 0;
    auto advance = [&](int& bb, int& rr) {
        if (rr + 1 == nround) {
            rr = 0;
            bb += nblk;
        } else
            ++rr;
    };
    int b1 = b, rd1 = rd;
    advance(b1, rd1);
    int b2 = b1, rd2 = rd1;
    advance(b2, rd2);
    GroupStep<UPL> sA, sB;
    float S;
    if constexpr (XDT < 0) {
        // Small loads first (memory answers in issue order): this thread's group of activations
        // (64 bytes; NG <= 256 threads take part) and the scale, then the first weight step.
        u32x4 xg[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            xg[i] = __builtin_amdgcn_raw_buffer_load_b128(xres, static_cast<int>(threadIdx.x) * 64, i * 16, 0);
        const uint16_t sbits = scale[0];
        // the activation loads stay in front of the weight loads (memory answers in issue order, and the
        // staging must not have to wait for weights)
        __builtin_amdgcn_sched_barrier(0);
        S = half_bits_to_float(sbits);
        load_step(b, rd, sA);
        load_step(b1, rd1, sB);
        asm volatile("" ::"s"(out), "s"(Pout));  // fetch the late arguments while the loads are in flight

        if (static_cast<int>(threadIdx.x) < NG) {
            const int g = threadIdx.x;
            const int r0 = g >> 5;
            const int R = min(32, NG - 32 * r0);
            uint2* dst = sx2 + 256 * r0 + (g & 31);
            int t[2] = {0, 0};  // units 0..3 | units 4..7
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                dst[(2 * i) * R] = make_uint2(xg[i].x, xg[i].y);
                dst[(2 * i + 1) * R] = make_uint2(xg[i].z, xg[i].w);
                int& ti = t[i >> 1];
                ti = dot8(xg[i].x, 0x11111111u, ti);
                ti = dot8(xg[i].y, 0x11111111u, ti);
                ti = dot8(xg[i].z, 0x11111111u, ti);
                ti = dot8(xg[i].w, 0x11111111u, ti);
            }
            if constexpr (SPL == 2) {
                tgs[2 * g] = t[0];
                tgs[2 * g + 1] = t[1];
            } else
                tgs[g] = t[0] + t[1];
        }
        __syncthreads();
    } else {
        // Fused quantiser.  Thread t takes the 16-value units t, t + 256, ...; they stay in registers, as they came
        // from memory, between the two passes (maximum, then quantisation).
        __shared__ float amax_slots[GG_THREADS / 64];
        constexpr int XT = XDT >= 0 ? XDT : 0;
        float a = 0.0f;
        // the activations are requested first (memory answers in issue order), the weights of the
        // first two steps right behind them, and only then is anything waited for
        Raw8<XT> xr[GG_XU][2];
#pragma unroll
        for (int i = 0; i < GG_XU; ++i) {
            if (i * GG_THREADS >= U) break;  // uniform
            const int u = min(static_cast<int>(threadIdx.x) + i * GG_THREADS, U - 1);  // clamped: duplicates are harmless
            xr[i][0] = load8_raw<XT>(xraw, static_cast<size_t>(u) * 16);
            xr[i][1] = load8_raw<XT>(xraw, static_cast<size_t>(u) * 16 + 8);
        }
        load_step(b, rd, sA);
        load_step(b1, rd1, sB);
        asm volatile("" ::"s"(out), "s"(Pout), "s"(xq_out), "s"(scale_out), "s"(clip_ratio));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < GG_XU; ++i) {
            if (i * GG_THREADS >= U) break;
            float v[2][8];
            widen8<XT>(xr[i][0], v[0]);
            widen8<XT>(xr[i][1], v[1]);
#pragma unroll
            for (int j = 0; j < 8; ++j) a = fmaxf(a, fmaxf(fabsf(v[0][j]), fabsf(v[1][j])));
        }
        for (int g = threadIdx.x; g < NG * SPL; g += GG_THREADS) tgs[g] = 0;
        a = wave_max(a);
        if (lane == 0) amax_slots[wave] = a;
        __syncthreads();
        a = fmaxf(fmaxf(amax_slots[0], amax_slots[1]), fmaxf(amax_slots[2], amax_slots[3]));
        const uint16_t sb = scale_bits_from_amax(a, clip_ratio);
        S = half_bits_to_float(sb);
        const bool publish = blockIdx.x == 0 && xq_out != nullptr;
        // all units are rounded first, without branches, so that their instruction chains interleave (a thread past the
        // end of the token works on a duplicate of the last unit and stores nothing)
        uint2 qv[GG_XU];
        const float rs = __frcp_rn(S);
        // fp16 / bf16 values straight from memory take the form of the quantiser that needs no second pass
        constexpr bool SHORT_IN = (XT == RCP_F16 || XT == RCP_BF16);
        float far = 0.0f;
#pragma unroll
        for (int i = 0; i < GG_XU; ++i) {
            if (i * GG_THREADS >= U) break;
            float v[2][8];
            widen8<XT>(xr[i][0], v[0]);
            widen8<XT>(xr[i][1], v[1]);
            qv[i] = SHORT_IN ? make_uint2(quantize8_short(v[0], S, rs), quantize8_short(v[1], S, rs))
                             : make_uint2(quantize8_fast(v[0], rs, far), quantize8_fast(v[1], rs, far));
        }
        if (!SHORT_IN && __builtin_expect(far > 0.49999f, 0)) {
#pragma unroll
            for (int i = 0; i < GG_XU; ++i) {
                if (i * GG_THREADS >= U) break;
                float v[2][8];
                widen8<XT>(xr[i][0], v[0]);
                widen8<XT>(xr[i][1], v[1]);
                qv[i] = make_uint2(quantize8_exact(v[0], S), quantize8_exact(v[1], S));
            }
        }
#pragma unroll
        for (int i = 0; i < GG_XU; ++i) {
            if (i * GG_THREADS >= U) break;
            const int u = threadIdx.x + i * GG_THREADS;
            if (u < U) {
                const int g = u >> 3, r0 = g >> 5;
                const int R = min(32, NG - 32 * r0);
                sx2[256 * r0 + (u & 7) * R + (g & 31)] = qv[i];
                atomicAdd(&tgs[SPL == 2 ? 2 * g + ((u & 7) >> 2) : g], dot8(qv[i].y, 0x11111111u, dot8(qv[i].x, 0x11111111u, 0)));
            }
        }
        if (publish) {
#pragma unroll
            for (int i = 0; i < GG_XU; ++i) {
                if (i * GG_THREADS >= U) break;
                const int u = threadIdx.x + i * GG_THREADS;
                if (u < U) reinterpret_cast<uint2*>(xq_out)[u] = qv[i];
            }
        }
        if (blockIdx.x == 0 && threadIdx.x == 0 && scale_out != nullptr) scale_out[0] = sb;
        __syncthreads();
    }

    float o[4] = {0.0f, 0.0f, 0.0f, 0.0f};

    // One pipeline step: compute the current step from `cur` (the loads of the following step are in
    // flight in the other register set), then refill `cur` with the step two ahead.
    auto step = [&](GroupStep<UPL>& cur) {
        const bool last = rd + 1 == nround;

        const int R = min(32, NG - 32 * rd);
        const uint2* xp = sx2 + 256 * rd + half * UPL * R + ln;
        int acc[1][3][4];
#pragma unroll
        for (int p = 0; p < 3; ++p)
#pragma unroll
            for (int m = 0; m < 4; ++m) acc[0][p][m] = 0;
#pragma unroll
        for (int i = 0; i < UPL; ++i) {
            const uint2 xv = xp[i * R];
            const uint32_t xa[1] = {xv.x}, xb[1] = {xv.y};
            cell_update<1>(cur.w[i].x, cur.w[i].y, xa, acc);
            cell_update<1>(cur.w[i].z, cur.w[i].w, xb, acc);
        }
        const bool valid = ln < R;
        const int g = 32 * rd + ln;
        const int Tg = valid ? tgs[SPL == 2 ? 2 * g + half : g] : 0;
        const int rg = b * GG_SLOTS + slot;
        const uint32_t lw[8] = {cur.lut[0].x, cur.lut[0].y, cur.lut[0].z, cur.lut[0].w,
                                cur.lut[1].x, cur.lut[1].y, cur.lut[1].z, cur.lut[1].w};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            // the triangular system of the four nibble masks, solved for row r of each plane
            int F[3];
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                const int v = r == 0 ? acc[0][p][0]
                            : r == 1 ? acc[0][p][1] - acc[0][p][0]
                            : r == 2 ? acc[0][p][2] - acc[0][p][1]
                                     : acc[0][p][2] - acc[0][p][3];
                F[p] = v >> r;
            }
            const int P3 = F[2], P1 = F[0] - F[2], P2 = F[1] - F[2];
            const int P0 = Tg - F[0] - F[1] + F[2];
            const float c0 = half_bits_to_float(static_cast<uint16_t>(lw[2 * r] & 0xffffu));
            const float c1 = half_bits_to_float(static_cast<uint16_t>(lw[2 * r] >> 16));
            const float c2 = half_bits_to_float(static_cast<uint16_t>(lw[2 * r + 1] & 0xffffu));
            const float c3 = half_bits_to_float(static_cast<uint16_t>(lw[2 * r + 1] >> 16));
            float v = o[r];
            v = fmaf(c0, static_cast<float>(P0), v);
            v = fmaf(c1, static_cast<float>(P1), v);
            v = fmaf(c2, static_cast<float>(P2), v);
            v = fmaf(c3, static_cast<float>(P3), v);
            o[r] = v;
            if constexpr (WANTP) {
                int4 Pg = make_int4(P0, P1, P2, P3);
                if constexpr (SPL == 2) {  // the group's sums: this lane's 64 columns plus the other lane's
                    Pg.x += __shfl_xor(P0, 32, 64);
                    Pg.y += __shfl_xor(P1, 32, 64);
                    Pg.z += __shfl_xor(P2, 32, 64);
                    Pg.w += __shfl_xor(P3, 32, 64);
                }
                if (valid && rg < G && half == 0) reinterpret_cast<int4*>(Pout)[static_cast<size_t>(4 * rg + r) * NG + g] = Pg;
            }
        }

        // `cur` is consumed: refill it, before the row totals below
        __builtin_amdgcn_sched_barrier(0);
        load_step(b2, rd2, cur);
        __builtin_amdgcn_sched_barrier(0);

        if (last) {
            // row totals over the lanes of the row group: even 16-lane rows end up with
            // rows 0 and 2, odd ones with rows 1 and 3
            float s01 = row_sum16f(fold16f(o[0], o[1]));
            float s23 = row_sum16f(fold16f(o[2], o[3]));
            if constexpr (SPL == 2) {
                s01 += __shfl_xor(s01, 32, 64);
                s23 += __shfl_xor(s23, 32, 64);
            }
            if (rg < G && (lane & 15) == 0 && half == 0) {
                const int odd = (lane >> 4) & 1;
                const int h = 4 * rg + odd;
                const float v0 = s01 * S, v1 = s23 * S;
                if constexpr (OUT_F16) {
                    static_cast<__half*>(out)[h] = __float2half_rn(v0);
                    static_cast<__half*>(out)[h + 2] = __float2half_rn(v1);
                } else {
                    static_cast<float*>(out)[h] = v0;
                    static_cast<float*>(out)[h + 2] = v1;
                }
            }
            o[0] = o[1] = o[2] = o[3] = 0.0f;
        }
        b = b1;
        rd = rd1;
        b1 = b2;
        rd1 = rd2;
        advance(b2, rd2);
    };
    // steps counted up front and run in pairs: one loop body, one exit (with an exit after either
    // step the merged exit branches make the wait-count analysis stall on all loads in flight)
    const int my_batches = (nbatch - static_cast<int>(blockIdx.x) + nblk - 1) / nblk;
    const int nsteps = my_batches * nround;
    for (int i = 0; i < nsteps / 2; ++i) {
        step(sA);
        step(sB);
    }
    if (nsteps & 1) step(sA);
}

struct GroupedArgs {
    const void *packed, *codebook;
    int N, K;
    const void *xq, *scale;
    void* out;
    rcp_dtype out_dt;
    int32_t* P;
    const void* xraw;  // fused quantiser when non-null
    rcp_dtype x_dt;
    float clip_ratio;
    void *xq_out, *scale_out;
};

template <bool OUT_F16, int XDT, bool NT, int LG = 32>
static int launch_grouped_nt(const GroupedArgs& a, int blocks, size_t lds, hipStream_t st)
{
    auto launch = [&](auto kernel) {
        kernel<<<blocks, GG_THREADS, lds, st>>>(
            static_cast<const uint4*>(a.packed), static_cast<const uint4*>(a.codebook), a.N, a.K, a.xraw,
            static_cast<const uint4*>(a.xq), static_cast<const uint16_t*>(a.scale), a.clip_ratio, blocks, a.out, a.P,
            static_cast<uint32_t*>(a.xq_out), static_cast<uint16_t*>(a.scale_out));
    };
    if (a.P != nullptr) launch(&gemv_grouped_kernel<OUT_F16, XDT, NT, LG, true>);
    else launch(&gemv_grouped_kernel<OUT_F16, XDT, NT, LG, false>);
    return check_launch("rcp_w2a4_gemv_grouped");
}

template <bool OUT_F16, int XDT>
static int launch_grouped_one(const GroupedArgs& a, int blocks, size_t lds, bool two_lanes, hipStream_t st)
{
    if (two_lanes) {
        const bool nt2 = options().gemv_nt != 0 ? options().gemv_nt == 1 : static_cast<long long>(a.N) * a.K / 4 >= (4LL << 20);
        return nt2 ? launch_grouped_nt<OUT_F16, XDT, true, 64>(a, blocks, lds, st)
                   : launch_grouped_nt<OUT_F16, XDT, false, 64>(a, blocks, lds, st);
    }
    // ("gemv_nt": 1 = non-temporal weight loads always, 2 = never; automatic: from 4 MB of packed weights on)
    const bool nt = options().gemv_nt != 0 ? options().gemv_nt == 1 : static_cast<long long>(a.N) * a.K / 4 >= (4LL << 20);
    return nt ? launch_grouped_nt<OUT_F16, XDT, true>(a, blocks, lds, st) : launch_grouped_nt<OUT_F16, XDT, false>(a, blocks, lds, st);
}

static int dispatch_grouped(const GroupedArgs& a, hipStream_t st)
{
    if (static_cast<long long>(a.N) * a.K / 4 >= (1LL << 31))
        return fail(RCP_ERR_SHAPE, "rcp_w2a4_gemv_grouped: packed matrix of %lld bytes exceeds 2 GiB",
                    static_cast<long long>(a.N) * a.K / 4);
    const int G = a.N / 4;
    const int cus = num_compute_units();
    // two lanes per quantisation group, four row groups per workgroup: twice the wavefronts for the same loads
    // (sweeps: 4096 x 4096 3.97 -> 3.48 us, 4096 x 11008 6.43 -> 5.20, 12288 x 4096 5.81 -> 5.24, 22016 x 4096
    // 7.98 -> 7.68 with activations quantised beforehand); "gemv_lanes" = 32 asks for the other form
    const bool two_lanes = options().gemv_lanes != 32;
    const int slots = two_lanes ? 4 : 8;
    const int nbatch = (G + slots - 1) / slots;
    int blocks = options().gemv_blocks;
    // one workgroup per compute unit walks its batches with the loads of the next two in flight (sweeps with two lanes
    // per group, fused: 12288 x 4096 5.7 us with 512 or 768 workgroups, 5.3 with 256; 22016 x 4096 8.2 -> 7.95;
    // 14336 x 4096 6.9 -> 6.1; counts between one and two per unit are worst)
    // (a matrix with 24 and more batches per unit, 131072 x 4096, streams a tenth faster from eight workgroups per unit)
    if (blocks == 0) blocks = two_lanes ? (nbatch >= cus * 24 ? cus * 8 : cus) : (nbatch <= cus * 8 ? nbatch : cus * 4);
    // every workgroup quantises x itself: fewer, longer-lived workgroups
    if (options().gemv_blocks == 0 && a.xraw != nullptr && blocks > cus * 2) blocks = cus * 2;
    if (blocks > nbatch) blocks = nbatch;
    if (blocks < 1) blocks = 1;
    const size_t lds = gemv_grouped_lds_bytes(a.K);
#define RCP_GG(XDT) \
    return a.out_dt == RCP_F16 ? launch_grouped_one<true, XDT>(a, blocks, lds, two_lanes, st) \
                               : launch_grouped_one<false, XDT>(a, blocks, lds, two_lanes, st)
    if (a.xraw == nullptr) RCP_GG(-1);
    if (a.x_dt == RCP_F16) RCP_GG(RCP_F16);
    if (a.x_dt == RCP_F32) RCP_GG(RCP_F32);
    RCP_GG(RCP_BF16);
#undef RCP_GG
}

int launch_gemv_grouped(const void* packed, const void* codebook, int N, int K, const void* xq,
                        const void* scale, void* out, rcp_dtype out_dt, int32_t* P, hipStream_t st)
{
    const GroupedArgs a = {packed, codebook, N, K, xq, scale, out, out_dt, P, nullptr, RCP_F16, 1.0f, nullptr, nullptr};
    return dispatch_grouped(a, st);
}

bool quant_gemv_grouped_supported(int K) { return K / 16 <= GG_XU * GG_THREADS; }

int launch_quant_gemv_grouped(const void* packed, const void* codebook, int N, int K, const void* x, rcp_dtype x_dt,
                              float clip_ratio, void* out, rcp_dtype out_dt, void* xq_out, void* scale_out, int32_t* P,
                              hipStream_t st)
{
    const GroupedArgs a = {packed, codebook, N, K, nullptr, nullptr, out, out_dt, P, x, x_dt, clip_ratio, xq_out, scale_out};
    return dispatch_grouped(a, st);
}

}  // namespace rcp
