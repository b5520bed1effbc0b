// Non-uniform W3A4 GEMV for CDNA4: the GEMV of Section 4.4 with the eight-level LUT of the
// 3-bit variant (Section 4.3, paragraph on the asymmetric normal-float 3-bit format).  The
// kernel design is this library's own and extends the 2-bit kernel's scheme.
//
// The product goes through exact integer per-level partial sums
//     P[h][l] = sum_{k : idx[h][k] = l} q[k],   O[h] = S * sum_l LUT[h][l] * P[h][l],
// and the partial sums through the monomials of the index bits idx = b0 + 2 b1 + 4 b2:
//     F_s = sum_k q[k] * prod_{i in s} b_i[k]   for the seven non-empty subsets s,  F_0 = T = sum q,
//     P_l = sum_{s >= l} (-1)^{|s| - |l|} F_s   (subset inversion: three rounds of subtractions).
// The packed layout keeps each bit plane with the bits of FOUR rows in a nibble, so a plane
// word (or the AND of plane words) and the packed int4 activation word go straight into
// v_dot8_i32_i4; the nibble masks 1, 3, 7, F give a triangular system solved exactly for the
// four rows, as in the 2-bit kernel.  Per 32 weights: 4 ANDs for the products, 21 for the
// masks, 28 dot instructions; no shift, no table look-up and no float conversion in the loop.
//
// Work decomposition: one wavefront per group of four rows; its 64 lanes take the 64 units
// (4 rows x 32 columns, three 16-byte plane pieces) of a block side by side, so each plane is
// read as one contiguous kilobyte.  The loads of the next block (or of the wavefront's next
// row group) are in flight while the current one is computed.
#include "rcp_internal.hpp"

namespace rcp {

constexpr int W3_THREADS = 256;
constexpr int W3_WAVES = W3_THREADS / 64;

struct W3Planes {
    u32x4 p[3];
};

// acc[s-1][m]: monomial s = 1..7 (bit i of s: plane i is a factor), nibble mask m in {1, 3, 7, F}
__device__ __forceinline__ void w3_unit_update(const W3Planes& w, const u32x4& x, int (&acc)[7][4])
{
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const uint32_t b0 = w.p[0][c], b1 = w.p[1][c], b2 = w.p[2][c];
        const uint32_t b01 = b0 & b1;
        const uint32_t pl[7] = {b0, b1, b01, b2, b0 & b2, b1 & b2, b01 & b2};
#pragma unroll
        for (int s = 0; s < 7; ++s) {
            acc[s][0] = dot8(x[c], pl[s] & 0x11111111u, acc[s][0]);
            acc[s][1] = dot8(x[c], pl[s] & 0x33333333u, acc[s][1]);
            acc[s][2] = dot8(x[c], pl[s] & 0x77777777u, acc[s][2]);
            acc[s][3] = dot8(x[c], pl[s], acc[s][3]);
        }
    }
}

// WS wavefronts share one row group: wavefront w of them takes the blocks w, w + WS, ... and the
// monomial sums meet in LDS.  A workgroup therefore works on W3_WAVES / WS row groups at a time.
//
// XDT < 0: `x_in` / `scale` are the quantised activations of one token.  XDT = RCP_F16 / RCP_F32 /
// RCP_BF16: `x_in` is the token itself; every workgroup quantises it in its prologue (thread t takes
// the 16-value units t, t + 256, ...; maximum, then the shared int4 quantiser), which is bit-identical
// to the separate quantiser launch, and workgroup 0 also writes x_q and S to `xq_out` / `scale_out`
// when those are given.
constexpr int W3_XR = 3;  // 16-value units per thread requested ahead of the weights (all of them up to K = 12288)

// NT: weight loads with the non-temporal hint (matrices of 16 MB and more, one wavefront per row group: 22016 x 4096
// 10.2 -> 10.0 us, 12288 x 4096 6.6 -> 6.5 us; the 6 MB of 4096 x 4096 are 6 % slower with it).
template <bool OUT_F16, int WS, int XDT, bool NT = false>
__global__ __launch_bounds__(W3_THREADS) void w3a4_gemv_kernel(const uint8_t* __restrict__ packed,
                                                               const uint4* __restrict__ codebook, int N, int K,
                                                               const void* __restrict__ x_in,
                                                               const uint16_t* __restrict__ scale, float clip_ratio,
                                                               int nblocks, void* __restrict__ out,
                                                               int32_t* __restrict__ Pout, uint2* __restrict__ xq_out,
                                                               uint16_t* __restrict__ scale_out)
{
    const uint4* xq = static_cast<const uint4*>(x_in);
    // x: 64 * nblk pieces of 16 bytes (zero beyond K); W3_WAVES sums of q; for WS > 1 the exchange
    // slots int[2 parities][W3_WAVES][4 rows][8]
    extern __shared__ uint4 smem4[];
    constexpr int SLOTS = W3_WAVES / WS;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wsub = wave % WS, slot = wave / WS;
    const int U = K / 32, G = N / 4;
    const int nblk = (U + 63) >> 6;  // the launcher guarantees nblk >= WS: every wavefront has a block
    const int nbatch = (G + SLOTS - 1) / SLOTS;
    const unsigned group_bytes = static_cast<unsigned>(U) * 48u;
    // One buffer resource over the whole matrix: a row group beyond N lands past its end and
    // reads zeros.  A lane beyond the last unit of a row group reads bytes of another plane or
    // row group; its activations in LDS are zero, so it adds nothing.
    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(packed), 0, static_cast<int>(static_cast<unsigned>(G) * group_bytes), 0x00020000);
    auto load_block = [&](int gi, int j, W3Planes& w) {
        const int R = min(64, U - 64 * j);
        // the whole offset goes into the vector operand: only that one is range-checked; a row group
        // past the end gets an offset beyond any matrix (they are below 2 GiB)
        const unsigned base = gi < G ? static_cast<unsigned>(gi) * group_bytes + 3072u * j + 16u * lane : 0x80000000u;
#pragma unroll
        for (int p = 0; p < 3; ++p)
            w.p[p] = __builtin_amdgcn_raw_buffer_load_b128(wres, static_cast<int>(base + 16u * R * p), 0, NT ? 2 : 0);
    };

    // The pipeline runs two steps ahead: (b, j) is the block being computed, (b1, j1) and (b2, j2)
    // the next two; a wavefront goes to its following block of the row group, else to its first
    // block in the workgroup's next batch.  The loads of the first two steps are issued here,
    // before the activations are staged; row groups past the end read zeros.
    int b = blockIdx.x;  // this workgroup's current batch of SLOTS row groups
    int j = wsub;
    const int bstride = nblocks;  // an argument: the launch dimensions would have to be fetched from memory
    auto advance = [&](int& bb, int& jj) {
        jj += WS;
        if (jj >= nblk) {
            jj = wsub;
            bb += bstride;
        }
    };
    int b1 = b, j1 = j;
    advance(b1, j1);
    int b2 = b1, j2 = j1;
    advance(b2, j2);
    const int xpieces = 64 * nblk;  // pieces of 16 bytes in LDS (zero beyond K)
    int* tsum = reinterpret_cast<int*>(smem4 + 64 * nblk);
    int* red = tsum + W3_WAVES;
    W3Planes wA, wB;
    const int my_row = (((lane >> 4) & 1) << 1) | (lane >> 5);  // the row this lane holds after the folds
    uint4 lut;
    uint16_t sbits;
    if constexpr (XDT < 0) {
        // memory answers loads in issue order: this thread's first piece of the activations goes first, so that
        // staging them does not have to wait for the weights
        sbits = scale[0];
        uint4 xfirst = make_uint4(0u, 0u, 0u, 0u);
        if (static_cast<int>(threadIdx.x) < U) xfirst = xq[threadIdx.x];
        __builtin_amdgcn_sched_barrier(0);
        load_block(b * SLOTS + slot, j, wA);
        load_block(b1 * SLOTS + slot, j1, wB);
        lut = codebook[min(4 * (b * SLOTS + slot) + my_row, N - 1)];

        int s = 0;
        // the first piece apart from the loop: behind a join with the loop's own loads the compiler would
        // wait for every load in flight, the weights included
        if (static_cast<int>(threadIdx.x) < xpieces) {
            smem4[threadIdx.x] = xfirst;
            s = dot8(xfirst.x, 0x11111111u, s);
            s = dot8(xfirst.y, 0x11111111u, s);
            s = dot8(xfirst.z, 0x11111111u, s);
            s = dot8(xfirst.w, 0x11111111u, s);
        }
        for (int i = threadIdx.x + W3_THREADS; i < xpieces; i += W3_THREADS) {  // K > 8192 only
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (i < U) v = xq[i];
            smem4[i] = v;
            s = dot8(v.x, 0x11111111u, s);
            s = dot8(v.y, 0x11111111u, s);
            s = dot8(v.z, 0x11111111u, s);
            s = dot8(v.w, 0x11111111u, s);
        }
        s = wave_sum(s);
        if (lane == 0) tsum[wave] = s;
    } else {
        // Fused quantiser: the raw activations are requested first, the weights of the first two steps
        // right behind them, and only then is anything waited for.  A thread's units stay in registers, as they came
        // from memory, between the two passes (re-reading them from cache for the second pass cost about a microsecond
        // on K = 11008); only beyond 12288 values are the remaining ones read again.
        __shared__ float amax_slots[W3_WAVES];
        constexpr int XT = XDT >= 0 ? XDT : 0;
        const int U16 = K / 16;  // 16-value units (uint2 of x_q); K is a multiple of 32
        Raw8<XT> xr[W3_XR][2];
#pragma unroll
        for (int i = 0; i < W3_XR; ++i) {
            if (i * W3_THREADS >= U16) break;  // uniform
            const int u = min(static_cast<int>(threadIdx.x) + i * W3_THREADS, U16 - 1);  // clamped: duplicates are harmless
            xr[i][0] = load8_raw<XT>(x_in, static_cast<size_t>(u) * 16);
            xr[i][1] = load8_raw<XT>(x_in, static_cast<size_t>(u) * 16 + 8);
        }
        load_block(b * SLOTS + slot, j, wA);
        load_block(b1 * SLOTS + slot, j1, wB);
        lut = codebook[min(4 * (b * SLOTS + slot) + my_row, N - 1)];
        asm volatile("" ::"s"(out), "s"(Pout), "s"(xq_out), "s"(scale_out));  // fetch the late arguments now
        __builtin_amdgcn_sched_barrier(0);
        float a = 0.0f;
#pragma unroll
        for (int i = 0; i < W3_XR; ++i) {
            if (i * W3_THREADS >= U16) break;
            float v[2][8];
            widen8<XT>(xr[i][0], v[0]);
            widen8<XT>(xr[i][1], v[1]);
#pragma unroll
            for (int e = 0; e < 8; ++e) a = fmaxf(a, fmaxf(fabsf(v[0][e]), fabsf(v[1][e])));
        }
        for (int u = threadIdx.x + W3_XR * W3_THREADS; u < U16; u += W3_THREADS) {  // K > 12288 only
            float v[2][8];
            load8_as_float<XT>(x_in, static_cast<size_t>(u) * 16, v[0]);
            load8_as_float<XT>(x_in, static_cast<size_t>(u) * 16 + 8, v[1]);
#pragma unroll
            for (int e = 0; e < 8; ++e) a = fmaxf(a, fmaxf(fabsf(v[0][e]), fabsf(v[1][e])));
        }
        a = wave_max(a);
        if (lane == 0) amax_slots[wave] = a;
        __syncthreads();
        a = fmaxf(fmaxf(amax_slots[0], amax_slots[1]), fmaxf(amax_slots[2], amax_slots[3]));
        sbits = scale_bits_from_amax(a, clip_ratio);
        const float S = half_bits_to_float(sbits);
        const bool publish = blockIdx.x == 0 && xq_out != nullptr;
        uint2* sx2 = reinterpret_cast<uint2*>(smem4);
        int s = 0;
        // the units in registers are rounded first, without branches, so that their instruction chains interleave (a
        // thread past the end of the token works on a duplicate of the last unit and stores zeros)
        uint2 qr[W3_XR];
        const float rs = __frcp_rn(S);
        // fp16 / bf16 values straight from memory take the form of the quantiser that needs no second pass
        constexpr bool SHORT_IN = (XT == RCP_F16 || XT == RCP_BF16);
        float far = 0.0f;
#pragma unroll
        for (int i = 0; i < W3_XR; ++i) {
            if (i * W3_THREADS >= U16) break;  // uniform
            float v[2][8];
            widen8<XT>(xr[i][0], v[0]);
            widen8<XT>(xr[i][1], v[1]);
            qr[i] = SHORT_IN ? make_uint2(quantize8_short(v[0], S, rs), quantize8_short(v[1], S, rs))
                             : make_uint2(quantize8_fast(v[0], rs, far), quantize8_fast(v[1], rs, far));
        }
        if (!SHORT_IN && __builtin_expect(far > 0.49999f, 0)) {
#pragma unroll
            for (int i = 0; i < W3_XR; ++i) {
                if (i * W3_THREADS >= U16) break;
                float v[2][8];
                widen8<XT>(xr[i][0], v[0]);
                widen8<XT>(xr[i][1], v[1]);
                qr[i] = make_uint2(quantize8_exact(v[0], S), quantize8_exact(v[1], S));
            }
        }
#pragma unroll
        for (int i = 0; i < W3_XR; ++i) {  // the padding up to whole blocks is zeroed too
            if (i * W3_THREADS >= 2 * xpieces) break;  // uniform
            const int u = threadIdx.x + i * W3_THREADS;
            if (u < 2 * xpieces) {
                uint2 qv = make_uint2(0u, 0u);
                if (u < U16) {
                    qv = qr[i];
                    s = dot8(qv.y, 0x11111111u, dot8(qv.x, 0x11111111u, s));
                    if (publish) xq_out[u] = qv;
                }
                sx2[u] = qv;
            }
        }
        for (int u = threadIdx.x + W3_XR * W3_THREADS; u < 2 * xpieces; u += W3_THREADS) {  // K > 12288 only
            uint2 qv = make_uint2(0u, 0u);
            if (u < U16) {
                float v[2][8];
                load8_as_float<XT>(x_in, static_cast<size_t>(u) * 16, v[0]);
                load8_as_float<XT>(x_in, static_cast<size_t>(u) * 16 + 8, v[1]);
                qv = make_uint2(quantize8(v[0], S), quantize8(v[1], S));
                s = dot8(qv.y, 0x11111111u, dot8(qv.x, 0x11111111u, s));
                if (publish) xq_out[u] = qv;
            }
            sx2[u] = qv;
        }
        if (blockIdx.x == 0 && threadIdx.x == 0 && scale_out != nullptr) scale_out[0] = sbits;
        s = wave_sum(s);
        if (lane == 0) tsum[wave] = s;
    }
    __syncthreads();
    const int T = tsum[0] + tsum[1] + tsum[2] + tsum[3];

    int acc[7][4];
#pragma unroll
    for (int s = 0; s < 7; ++s)
#pragma unroll
        for (int m = 0; m < 4; ++m) acc[s][m] = 0;
    int parity = 0;

    // one pipeline step: compute the current block from `cur` (the loads of the following block are
    // in flight in the other register set), then refill `cur` with the block two steps ahead
    auto step = [&](W3Planes& cur) {
        const bool last = j + WS >= nblk;  // uniform
        const int bn = b1;
        const uint4 xv = smem4[64 * j + lane];
        const u32x4 x = {xv.x, xv.y, xv.z, xv.w};
        w3_unit_update(cur, x, acc);
        __builtin_amdgcn_sched_barrier(0);
        load_block(b2 * SLOTS + slot, j2, cur);
        __builtin_amdgcn_sched_barrier(0);
        if (last) {  // this wavefront's share of the row group is finished
            // this lane's share of 2^r f_r, then the sum over the wavefront; lanes 0, 16, 32, 48
            // end up with the seven monomial sums of rows 0, 2, 1, 3
            int F[8];
            F[0] = T;
#pragma unroll
            for (int s = 0; s < 7; ++s) {
                const int g0 = acc[s][0], g1 = acc[s][1] - acc[s][0], g2 = acc[s][2] - acc[s][1], g3 = acc[s][2] - acc[s][3];
                const int lo = fold32(g0, g1), hi = fold32(g2, g3);
                F[s + 1] = row_sum16(fold16(lo, hi)) >> my_row;
#pragma unroll
                for (int m = 0; m < 4; ++m) acc[s][m] = 0;
            }
            if constexpr (WS > 1) {
                int* mine = red + ((parity * W3_WAVES + wave) * 4 + my_row) * 8;
                if ((lane & 15) == 0 && wsub != 0) {
                    reinterpret_cast<int4*>(mine)[0] = make_int4(0, F[1], F[2], F[3]);
                    reinterpret_cast<int4*>(mine)[1] = make_int4(F[4], F[5], F[6], F[7]);
                }
                __syncthreads();  // every wavefront of the workgroup finishes a batch the same number of times
                if ((lane & 15) == 0 && wsub == 0) {
#pragma unroll
                    for (int w = 1; w < WS; ++w) {
                        const int4 a = reinterpret_cast<const int4*>(mine + w * 32)[0];
                        const int4 c = reinterpret_cast<const int4*>(mine + w * 32)[1];
                        F[1] += a.y; F[2] += a.z; F[3] += a.w;
                        F[4] += c.x; F[5] += c.y; F[6] += c.z; F[7] += c.w;
                    }
                }
                parity ^= 1;
            }
            const int gi = b * SLOTS + slot;
            if ((lane & 15) == 0 && wsub == 0 && gi < G) {
#pragma unroll
                for (int bit = 1; bit < 8; bit <<= 1)
#pragma unroll
                    for (int l = 0; l < 8; ++l)
                        if ((l & bit) == 0) F[l] -= F[l | bit];
                const int h = 4 * gi + my_row;
                const uint32_t lw[4] = {lut.x, lut.y, lut.z, lut.w};
                float o = 0.0f;
#pragma unroll
                for (int l = 0; l < 8; ++l) {
                    const float c = half_bits_to_float(static_cast<uint16_t>(l & 1 ? lw[l >> 1] >> 16 : lw[l >> 1] & 0xffffu));
                    o = l == 0 ? c * static_cast<float>(F[0]) : fmaf(c, static_cast<float>(F[l]), o);
                }
                o *= half_bits_to_float(sbits);
                if constexpr (OUT_F16) static_cast<__half*>(out)[h] = __float2half_rn(o);
                else static_cast<float*>(out)[h] = o;
                if (Pout != nullptr) {
                    reinterpret_cast<int4*>(Pout)[2 * h] = make_int4(F[0], F[1], F[2], F[3]);
                    reinterpret_cast<int4*>(Pout)[2 * h + 1] = make_int4(F[4], F[5], F[6], F[7]);
                }
            }
            if (bn < nbatch) lut = codebook[min(4 * (bn * SLOTS + slot) + my_row, N - 1)];
        }
        b = b1;
        j = j1;
        b1 = b2;
        j1 = j2;
        advance(b2, j2);
    };
    // steps counted up front and run in pairs: one loop body, one exit (with an exit after either
    // step the merged exit branches make the wait-count analysis stall on all loads in flight)
    const int my_batches = (nbatch - static_cast<int>(blockIdx.x) + nblocks - 1) / nblocks;
    const int nsteps = my_batches * ((nblk - wsub + WS - 1) / WS);
    for (int i = 0; i < nsteps / 2; ++i) {
        step(wA);
        step(wB);
    }
    if (nsteps & 1) step(wA);
}

struct W3Args {
    const void* packed;
    const void* codebook;
    int N, K;
    const void* x;          // quantised activations (x_dt < 0) or the raw token
    const void* scale;      // S of the quantised activations, unused otherwise
    int x_dt;               // -1 or an rcp_dtype
    float clip_ratio;
    void* out;
    rcp_dtype out_dt;
    int32_t* P;
    void* xq_out;
    void* scale_out;
};

template <int WS, int XDT>
static int launch_w3_ws(const W3Args& a, hipStream_t st)
{
    const int G = a.N / 4, U = a.K / 32;
    const int nblk = (U + 63) / 64;
    const size_t lds = static_cast<size_t>(nblk) * 64 * 16 + W3_WAVES * sizeof(int) +
                       (WS > 1 ? 2 * W3_WAVES * 4 * 8 * sizeof(int) : 0);
    const int cus = num_compute_units();
    constexpr int SLOTS = W3_WAVES / WS;
    const int nbatch = (G + SLOTS - 1) / SLOTS;
    int blocks = options().gemv_blocks;
    // sweeps: two workgroups per compute unit on LLaMA-sized layers; a matrix with 16 and more batches per unit streams
    // 5 - 7 % faster from eight (65536 x 4096 24.4 -> 23.1 us, 131072 x 4096 46.5 -> 43.1)
    if (blocks == 0) blocks = nbatch >= cus * 16 ? cus * 8 : (nbatch <= cus * 2 ? nbatch : cus * 2);
    if (blocks > nbatch) blocks = nbatch;
    auto launch = [&](auto kernel) {
        kernel<<<blocks, W3_THREADS, lds, st>>>(static_cast<const uint8_t*>(a.packed), static_cast<const uint4*>(a.codebook), a.N,
                                                a.K, a.x, static_cast<const uint16_t*>(a.scale), a.clip_ratio, blocks, a.out, a.P,
                                                static_cast<uint2*>(a.xq_out), static_cast<uint16_t*>(a.scale_out));
    };
    // ("gemv_nt": 1 = non-temporal weight loads whenever one wavefront serves a row group, 2 = never)
    const bool nt = WS == 1 && (options().gemv_nt != 0 ? options().gemv_nt == 1
                                                       : static_cast<long long>(a.N) * a.K / 8 * 3 >= (16LL << 20));
    if constexpr (WS == 1) {
        if (nt) {
            if (a.out_dt == RCP_F16) launch(&w3a4_gemv_kernel<true, WS, XDT, true>);
            else launch(&w3a4_gemv_kernel<false, WS, XDT, true>);
            return check_launch(XDT < 0 ? "rcp_w3a4_gemv" : "rcp_quant_w3a4_gemv");
        }
    }
    if (a.out_dt == RCP_F16) launch(&w3a4_gemv_kernel<true, WS, XDT>);
    else launch(&w3a4_gemv_kernel<false, WS, XDT>);
    return check_launch(XDT < 0 ? "rcp_w3a4_gemv" : "rcp_quant_w3a4_gemv");
}

template <int XDT>
static int launch_w3_any(const W3Args& a, hipStream_t st)
{
    const int nblk = (a.K / 32 + 63) / 64;
    // wavefronts per row group: one, unless the "gemv_lanes" option (64, 128, 256) asks for 1, 2 or 4
    // (sweeps at LLaMA-2-7B sizes: with the two-steps-ahead pipeline a second wavefront per row group
    // never pays for its exchange through LDS); never more than the row group has blocks
    int ws = options().gemv_lanes >= 64 ? options().gemv_lanes / 64 : 1;
    while (ws > 1 && ws > nblk) ws /= 2;
    switch (ws) {
        case 1: return launch_w3_ws<1, XDT>(a, st);
        case 2: return launch_w3_ws<2, XDT>(a, st);
        default: return launch_w3_ws<4, XDT>(a, st);
    }
}

int launch_w3a4_gemv(const void* packed, const void* codebook, int N, int K, const void* xq, const void* scale,
                     void* out, rcp_dtype out_dt, int32_t* P, hipStream_t st)
{
    if (static_cast<long long>(N) * K / 8 * 3 >= (1LL << 31))
        return fail(RCP_ERR_SHAPE, "rcp_w3a4_gemv: packed matrix of %lld bytes exceeds 2 GiB", static_cast<long long>(N) * K / 8 * 3);
    const W3Args a = {packed, codebook, N, K, xq, scale, -1, 1.0f, out, out_dt, P, nullptr, nullptr};
    return launch_w3_any<-1>(a, st);
}

int launch_quant_w3a4_gemv(const void* packed, const void* codebook, int N, int K, const void* x, rcp_dtype x_dt,
                           float clip_ratio, void* out, rcp_dtype out_dt, void* xq_out, void* scale_out, int32_t* P,
                           hipStream_t st)
{
    if (static_cast<long long>(N) * K / 8 * 3 >= (1LL << 31))
        return fail(RCP_ERR_SHAPE, "rcp_quant_w3a4_gemv: packed matrix of %lld bytes exceeds 2 GiB",
                    static_cast<long long>(N) * K / 8 * 3);
    const W3Args a = {packed, codebook, N, K, x, nullptr, static_cast<int>(x_dt), clip_ratio, out, out_dt, P, xq_out, scale_out};
    if (x_dt == RCP_F16) return launch_w3_any<RCP_F16>(a, st);
    if (x_dt == RCP_F32) return launch_w3_any<RCP_F32>(a, st);
    return launch_w3_any<RCP_BF16>(a, st);
}

}  // namespace rcp
