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
// give a triangular system that is solved exactly for the four rows:
//     D1 = f0, D3 = f0 + 2 f1, D7 = D3 + 4 f2, DF = D7 - 8 f3.
// Per 32 weights that is 1 AND (b0 & b1) + 9 ANDs + 12 dots, and no shift, no table
// look-up and no float conversion in the loop.  The LUT is touched only in the epilogue.
//
// Work decomposition.  A group of four rows is K/16 units of 16 bytes (4 rows x 16
// columns).  LG = LW*WS lanes share one row group: LW = 16, 32 or 64 lanes of a wavefront
// (a wavefront then works on 64/LW row groups side by side), and for LW = 64 optionally
// WS = 2 or 4 wavefronts of the 256-thread workgroup.  Lane t of the LG takes units
// t, t + LG, t + 2 LG, ...  Few lanes per row group make the cross-lane reduction cheap
// (it is paid once per row group) and suit tall matrices; many lanes put a small matrix on
// enough wavefronts.  The kernel is latency bound at LLaMA sizes, so the loop is software
// pipelined over (row group, chunk of UNR units) two steps ahead: a register set is refilled
// as soon as its chunk is consumed, so the loads of the next step are in flight while the
// current one is computed and reduced, and the loads of the first two steps are issued
// before the activations are staged.
#include <math.h>

#include "rcp_internal.hpp"

namespace rcp {

constexpr int GEMV_THREADS = 256;
constexpr int GEMV_WAVES = GEMV_THREADS / 64;

// XDT < 0: `xq` / `scale` are the quantised activations.  XDT = RCP_F16 / RCP_F32 / RCP_BF16
// (one token only): `xraw` is the raw activation of that type and the workgroup quantises it
// itself, exactly as quant_kernel would (amax, S = fp16(ratio*amax/7), q = rint(x/S)); the
// first workgroup also writes x_q and S to xq_out / scale_out when those are given.
// XDT = 4 + type: before quantising, the workgroup also applies the Hadamard rotation across
// heads, y = (H_n (x) I_m) x (rot_n heads of rot_m channels), with the butterflies and the final
// scaling of heads_wht_kernel, i.e. bit-identical to rcp_rotate_quant_act with RCP_ROT_HEADS.
// XDT = 8 + type: the order-K Hadamard rotation itself, K <= 2048 (a thread holds eight consecutive
// values, as in wht_quant_kernel): the same butterflies in the same passes, bit-identical to
// rcp_rotate_quant_act with RCP_ROT_WHT.  For such short inputs the transform costs a workgroup less than
// the launch of a rotation kernel costs the chain.
constexpr int GEMV_XG = 8;  // groups of eight raw activations a thread can hold: K <= 16384

// Order-NH Hadamard transform down the columns of the NH x m matrix in LDS (ascending stride, one
// IEEE add / sub per butterfly, one multiply by `norm` at the end): a thread takes whole columns.
template <int NH>
__device__ __forceinline__ void heads_columns(float* sy, int m, float norm)
{
    for (int j = threadIdx.x; j < m; j += GEMV_THREADS) {
        float v[NH];
#pragma unroll
        for (int i = 0; i < NH; ++i) v[i] = sy[i * m + j];
#pragma unroll
        for (int st = 1; st < NH; st <<= 1)
#pragma unroll
            for (int i = 0; i < NH; ++i)
                if ((i & st) == 0) {
                    const float p = v[i], q = v[i + st];
                    v[i] = p + q;
                    v[i + st] = p - q;
                }
#pragma unroll
        for (int i = 0; i < NH; ++i) sy[i * m + j] = __fmul_rn(v[i], norm);
    }
}

// The first 56 bytes of arguments reach the wavefront in scalar registers at launch; everything the
// prologue needs at once (matrix, shape, activations, the rotation) is among them.
// NT: the weight loads carry the non-temporal hint -- a matrix is read once and need not displace anything in the
// caches (134 MB: 25.8 -> 24.2 us; on a sweep of their own matrices of 4 - 22 MB are level or slower with it, inside a
// decode step the hint on launches of 8 MB and more is worth 3 % of the step: see the launcher).
template <int LW, int WS, int UNR, int MT, bool OUT_F16, int XDT, int NW, bool NT = false>
__global__ __launch_bounds__(NW * 64) void gemv_kernel(const uint4* __restrict__ packed,
                                                            const uint2* __restrict__ codebook, int N, int K,
                                                            const void* __restrict__ x_in,
                                                            const uint16_t* __restrict__ scale, int M, float clip_ratio,
                                                            int nblk, int rot,
                                                            void* __restrict__ out, int32_t* __restrict__ Pout,
                                                            uint32_t* __restrict__ xq_out, uint16_t* __restrict__ scale_out)
{
    static_assert(WS == 1 || LW == 64, "several wavefronts per row group only with whole wavefronts");
    // `rot` is the last argument that arrives in registers: heads | channels per head << 8 for the rotation across heads,
    // log2 K for the order-K rotation; the factor 1/sqrt(n) of a power of two n is put together from its exponent
    // ((float)(1/sqrt 2) times a power of two: what the host's (float)(1.0 / sqrt((double)n)) gives)
    auto inv_sqrt_pow2 = [](int k) {
        return __uint_as_float(((k & 1) ? 0x3F3504F3u : 0x3F800000u) - (static_cast<uint32_t>(k >> 1) << 23));
    };
    const int rot_n = XDT >= 8 ? 0 : (rot & 0xff);
    const int rot_m = XDT >= 8 ? rot : (rot >> 8);
    const float rot_norm = XDT >= 8 ? inv_sqrt_pow2(rot) : (XDT >= 4 ? inv_sqrt_pow2(__ffs(rot_n) - 1) : 1.0f);
    static_assert(NW == 4 || (NW == 8 && XDT >= 0 && XDT < 4), "eight wavefronts: the fused quantiser without rotation");
    constexpr int TH = NW * 64;  // threads of the workgroup
    // one pointer for the activations: quantised (XDT < 0) or raw; the number of workgroups comes as an
    // argument (nblk) because the launch dimensions would have to be fetched from memory first
    const uint4* __restrict__ xq = static_cast<const uint4*>(x_in);
    const void* __restrict__ xraw = x_in;
    static_assert(XDT < 0 || MT == 1, "the fused quantiser handles one token");
    constexpr bool ROT = XDT >= 4 && XDT < 8;   // Hadamard across heads in the prologue
    constexpr bool ROTW = XDT >= 8;             // order-K Hadamard rotation in the prologue (K <= 2048)
    constexpr int XT = XDT >= 0 ? (XDT & 3) : 0;  // storage type of the raw activation
    extern __shared__ uint4 smem4[];
    constexpr int SW = 64 / LW;                     // row groups side by side in a wavefront
    constexpr int SLOTS = (NW / WS) * SW;   // row groups a workgroup works on at a time
    constexpr int LG = LW * WS;                     // lanes per row group
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wsub = wave % WS;
    const int slot = (wave / WS) * SW + lane / LW;
    const int tg = wsub * 64 + lane % LW;  // this lane's position among the LG lanes
    const int U = K / 16, G = N / 4;
    const int xdw = K / 8;  // activation dwords per token
    const int nbatch = (G + SLOTS - 1) / SLOTS;
    const int nchunk = (U + LG * UNR - 1) / (LG * UNR);
    const int my_row = lane_row<LW>(lane);

    // One buffer resource over the whole matrix; a unit beyond K or a row group beyond N
    // gets an offset past the end, which the hardware answers with zeros: no branch and no
    // select on the data in the loop.
    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint4*>(packed), 0, static_cast<int>(static_cast<unsigned>(G) * static_cast<unsigned>(U) * 16u), 0x00020000);
    // Lane t owns units t, t + LG, ... of a row group: my_units of them.  When K fills every
    // chunk exactly no lane ever runs past K and the test below is always true.
    const int my_units = (U % (LG * UNR)) != 0 ? (U - tg + LG - 1) / LG : 0x7fffffff;
    // Byte offset of this lane's first unit in a batch, and its step from one batch of this
    // workgroup to the next.  A row group beyond N lands beyond the end of the resource (the
    // overshoot is less than the matrix size, which is below 2 GiB, so nothing wraps).
    auto batch_offset = [&](int bb) -> unsigned {
        return (static_cast<unsigned>(bb * SLOTS + slot) * U + tg) * 16u;
    };
    const unsigned batch_stride = static_cast<unsigned>(nblk) * SLOTS * U * 16u;
    auto load_chunk = [&](unsigned base, int ch, bool valid, u32x4 (&w)[UNR]) {
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            const int it = ch * UNR + i;
            const unsigned off = (valid && it < my_units) ? base : 0x80000000u;
            w[i] = __builtin_amdgcn_raw_buffer_load_b128(wres, static_cast<int>(off), it * LG * 16, NT ? 2 : 0);
        }
    };

    // Memory returns loads in issue order, so the small ones the prologue needs go first:
    // the activations (first 4 KiB per token straight into registers) and the scales; then
    // the weight loads of the first step, before any other work.
    const int per_token = xdw / 4;  // 16-byte pieces of one token's activations
    u32x4 xfirst[MT];
    float sc[MT];
    float xr8[XDT >= 0 ? GEMV_XG : 1][8];  // raw activations of the fused path, widened to fp32 ...
    Raw8<XT> xraw8[XDT >= 0 ? GEMV_XG : 1];  // ... and as they come from memory
    if constexpr (XDT < 0) {
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const bool have = MT == 1 || t < M;  // (one token: no test, so that the load is not moved into a branch)
            const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<uint4*>(xq + static_cast<size_t>(have ? t : 0) * per_token), 0, have ? per_token * 16 : 0, 0x00020000);
            xfirst[t] = __builtin_amdgcn_raw_buffer_load_b128(xr, static_cast<int>(threadIdx.x) * 16, 0, 0);
        }
        uint16_t scb[MT];
#pragma unroll
        for (int t = 0; t < MT; ++t) scb[t] = scale[(MT == 1 || t < M) ? t : 0];
        // the activation loads stay in front of the weight loads issued below (memory answers in order,
        // and the staging must not have to wait for the weights)
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < MT; ++t) sc[t] = half_bits_to_float(scb[t]);
    } else {
#pragma unroll
        for (int i = 0; i < GEMV_XG; ++i) {
            if (i * TH >= xdw) break;  // uniform: whole blocks of 256 groups
            const int u8 = min(static_cast<int>(threadIdx.x) + i * TH, xdw - 1);  // clamped: duplicates are harmless
            xraw8[i] = load8_raw<XT>(xraw, static_cast<size_t>(u8) * 8);
        }
    }

    // The pipeline runs two steps ahead: (b, ch) is the chunk being computed, (b1, ch1) and
    // (b2, ch2) the next two; a step goes to the following chunk of its batch, else to the first
    // chunk of this workgroup's next batch.  The loads of the first two steps are issued here,
    // before the activations are staged; past the last batch loads are given the offset that
    // reads zeros.
    int b = blockIdx.x;  // this workgroup's current batch of SLOTS row groups
    int ch = 0;
    unsigned base = batch_offset(b);
    auto advance = [&](int& bb, int& cc, unsigned& bs) {
        if (cc + 1 == nchunk) {
            bb += nblk;
            cc = 0;
            bs += batch_stride;
        } else
            ++cc;
    };
    int b1 = b, ch1 = 0;
    unsigned base1 = base;
    advance(b1, ch1, base1);
    int b2 = b1, ch2 = ch1;
    unsigned base2 = base1;
    advance(b2, ch2, base2);
    u32x4 wA[UNR], wB[UNR];  // the two pipeline stages alternate between these
    load_chunk(base, 0, b < nbatch, wA);
    load_chunk(base1, ch1, b1 < nbatch, wB);
    int lut_row = min(4 * (b * SLOTS + slot) + my_row, N - 1);  // clamped: lanes past N read a valid row
    uint2 lut_cur = codebook[lut_row];
    // the arguments that did not arrive in registers are fetched while the loads above are in flight,
    // not where the quantiser or the epilogue first needs them
    asm volatile("" ::"s"(out), "s"(Pout), "s"(xq_out), "s"(scale_out));
    if constexpr (XDT >= 0) {
        // only now touch the activations: waiting for them any earlier would hold back the weight loads
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < GEMV_XG; ++i) {
            if (i * TH >= xdw) break;
            widen8<XT>(xraw8[i], xr8[i]);
        }
    }

    // stage the activations and sum them: T[t] = sum_k q[t][k], the same for every row
    const int x_bytes = gemv_x_bytes(K, M, LG * UNR);
    int* tsum = reinterpret_cast<int*>(reinterpret_cast<char*>(smem4) + x_bytes);  // [NW][MT]
    int* red = tsum + NW * MT + NW;  // NW slots in between serve the fused quantiser's maximum
    if constexpr (XDT < 0) {
        u32x4* sx4 = reinterpret_cast<u32x4*>(smem4);
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            int s = 0;
            if (MT == 1 || t < M) {
                // a piece beyond the token's end was read as zero and is not stored
                if (static_cast<int>(threadIdx.x) < per_token) sx4[t * per_token + threadIdx.x] = xfirst[t];
                s = dot8(xfirst[t].x, 0x11111111u, s);
                s = dot8(xfirst[t].y, 0x11111111u, s);
                s = dot8(xfirst[t].z, 0x11111111u, s);
                s = dot8(xfirst[t].w, 0x11111111u, s);
                for (int i = threadIdx.x + TH; i < per_token; i += TH) {  // K > 8192 only
                    const uint4 v = xq[t * per_token + i];
                    smem4[t * per_token + i] = v;
                    s = dot8(v.x, 0x11111111u, s);
                    s = dot8(v.y, 0x11111111u, s);
                    s = dot8(v.z, 0x11111111u, s);
                    s = dot8(v.w, 0x11111111u, s);
                }
            }
            s = wave_sum(s);
            if (lane == 0) tsum[wave * MT + t] = s;
        }
    } else {
        if constexpr (ROT) {
            // y = (H_n (x) I_m) x through LDS: every thread parks its values, then takes whole columns
            // (the rot_n values x[i*m + j]) through the butterflies in ascending stride order
            float* sy = reinterpret_cast<float*>(red + (WS > 1 ? 2 * NW * 4 * 3 * MT : 0));
#pragma unroll
            for (int i = 0; i < GEMV_XG; ++i) {
                if (i * TH >= xdw) break;
                const int u8 = threadIdx.x + i * TH;
                if (u8 < xdw) {
                    reinterpret_cast<float4*>(sy)[2 * u8] = make_float4(xr8[i][0], xr8[i][1], xr8[i][2], xr8[i][3]);
                    reinterpret_cast<float4*>(sy)[2 * u8 + 1] = make_float4(xr8[i][4], xr8[i][5], xr8[i][6], xr8[i][7]);
                }
            }
            __syncthreads();
            switch (rot_n) {  // uniform; the head count must be a compile-time constant for the registers
                case 2: heads_columns<2>(sy, rot_m, rot_norm); break;
                case 4: heads_columns<4>(sy, rot_m, rot_norm); break;
                case 8: heads_columns<8>(sy, rot_m, rot_norm); break;
                case 16: heads_columns<16>(sy, rot_m, rot_norm); break;
                case 32: heads_columns<32>(sy, rot_m, rot_norm); break;
                default: heads_columns<64>(sy, rot_m, rot_norm); break;
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < GEMV_XG; ++i) {
                if (i * TH >= xdw) break;
                const int u8 = min(static_cast<int>(threadIdx.x) + i * TH, xdw - 1);
                const float4 lo4 = reinterpret_cast<const float4*>(sy)[2 * u8], hi4 = reinterpret_cast<const float4*>(sy)[2 * u8 + 1];
                xr8[i][0] = lo4.x; xr8[i][1] = lo4.y; xr8[i][2] = lo4.z; xr8[i][3] = lo4.w;
                xr8[i][4] = hi4.x; xr8[i][5] = hi4.y; xr8[i][6] = hi4.z; xr8[i][7] = hi4.w;
            }
        }
        if constexpr (ROTW) {
            // y = H_K x: this thread's eight consecutive values take the strides 1, 2, 4 in registers, the next six
            // strides run between lanes, every later pass gathers through LDS the eight values whose indices differ in
            // the next three bits
            // (rot_n = K, rot_m = log2 K)
            float* sy = reinterpret_cast<float*>(red + (WS > 1 ? 2 * NW * 4 * 3 * MT : 0));
            const int tid = threadIdx.x;
            const int log2n = rot_m;
            const bool active = tid < xdw;
            if (active) register_stages<3>(xr8[0], 0);
            // the next (up to six) index bits are the lane number: those strides run between lanes (threads without
            // data only ever meet each other there)
            const int nlane = min(6, log2n - 3);
            lane_stages<8>(xr8[0], lane, nlane);
            int done = 3 + nlane;
            const bool more = done < log2n;  // uniform: strides beyond a wavefront go through LDS
            if (more && active) {
#pragma unroll
                for (int e = 0; e < 8; ++e) sy[wht_slot(tid * 8 + e)] = xr8[0][e];
            }
            while (done < log2n) {  // uniform
                const int lo = (done <= log2n - 3) ? done : (log2n - 3);
                const int low = tid & ((1 << lo) - 1), high = tid >> lo;
                const int base = (high << (lo + 3)) | low;
                __syncthreads();
                if (active) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) xr8[0][e] = sy[wht_slot(base | (e << lo))];
                    register_stages<3>(xr8[0], done - lo);
#pragma unroll
                    for (int e = 0; e < 8; ++e) sy[wht_slot(base | (e << lo))] = xr8[0][e];
                }
                done = lo + 3;
            }
            if (more) __syncthreads();
#pragma unroll
            for (int e = 0; e < 8; ++e) xr8[0][e] = active ? __fmul_rn(more ? sy[wht_slot(tid * 8 + e)] : xr8[0][e], rot_norm) : 0.0f;
        }
        // per-token symmetric int4 quantiser, the same arithmetic as quant_kernel
        float a = 0.0f;
#pragma unroll
        for (int i = 0; i < GEMV_XG; ++i) {
            if (i * TH >= xdw) break;
#pragma unroll
            for (int j = 0; j < 8; ++j) a = fmaxf(a, fabsf(xr8[i][j]));
        }
        a = wave_max(a);
        float* amax_slots = reinterpret_cast<float*>(tsum + NW * MT);  // NW floats after the sums
        if (lane == 0) amax_slots[wave] = a;
        __syncthreads();
        a = fmaxf(fmaxf(amax_slots[0], amax_slots[1]), fmaxf(amax_slots[2], amax_slots[3]));
        if constexpr (NW == 8)
            a = fmaxf(a, fmaxf(fmaxf(amax_slots[4], amax_slots[5]), fmaxf(amax_slots[6], amax_slots[7])));
        const uint16_t sb = scale_bits_from_amax(a, clip_ratio);
        const float sq = half_bits_to_float(sb);
        sc[0] = sq;
        uint32_t* sx1 = reinterpret_cast<uint32_t*>(smem4);
        const bool publish = blockIdx.x == 0 && xq_out != nullptr;
        int s = 0;
        // all groups of eight are rounded first, without branches, so that their instruction chains interleave
        // (a thread past the end of the token works on a duplicate of the last group and stores nothing)
        uint32_t qd[GEMV_XG];
        const float rs = __frcp_rn(sq);
        // fp16 / bf16 values straight from memory take the form of the quantiser that needs no second pass
        constexpr bool SHORT_IN = (XT == RCP_F16 || XT == RCP_BF16) && !ROT && !ROTW;
        float far = 0.0f;
#pragma unroll
        for (int i = 0; i < GEMV_XG; ++i) {
            if (i * TH >= xdw) break;
            qd[i] = SHORT_IN ? quantize8_short(xr8[i], sq, rs) : quantize8_fast(xr8[i], rs, far);
        }
        if (!SHORT_IN && __builtin_expect(far > 0.49999f, 0)) {
#pragma unroll
            for (int i = 0; i < GEMV_XG; ++i) {
                if (i * TH >= xdw) break;
                qd[i] = quantize8_exact(xr8[i], sq);
            }
        }
#pragma unroll
        for (int i = 0; i < GEMV_XG; ++i) {
            if (i * TH >= xdw) break;
            const int u8 = threadIdx.x + i * TH;
            if (u8 < xdw) {
                sx1[u8] = qd[i];
                s = dot8(qd[i], 0x11111111u, s);
            }
        }
        if (publish) {
#pragma unroll
            for (int i = 0; i < GEMV_XG; ++i) {
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
    const uint2* sx2 = reinterpret_cast<const uint2*>(smem4);
    int T[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        T[t] = tsum[t] + tsum[MT + t] + tsum[2 * MT + t] + tsum[3 * MT + t];
        if constexpr (NW == 8) T[t] += tsum[4 * MT + t] + tsum[5 * MT + t] + tsum[6 * MT + t] + tsum[7 * MT + t];
    }

    int acc[MT][3][4];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int p = 0; p < 3; ++p)
#pragma unroll
            for (int m = 0; m < 4; ++m) acc[t][p][m] = 0;

    int parity = 0;
    // One pipeline step: compute the current chunk from `w` (the loads of the following chunk are
    // in flight in the other register set), then start the loads of the chunk two steps ahead
    // into `w`.
    auto step = [&](u32x4 (&w)[UNR]) {
        const bool last = ch + 1 == nchunk;

        const uint2* xrow = sx2 + tg + ch * UNR * LG;
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            uint32_t xa[MT], xb[MT];
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                const uint2 xv = xrow[(MT == 1 ? 0 : min(t, M - 1)) * (xdw / 2) + i * LG];
                xa[t] = xv.x;
                xb[t] = xv.y;
            }
            cell_update<MT>(w[i].x, w[i].y, xa, acc);
            cell_update<MT>(w[i].z, w[i].w, xb, acc);
        }
        // `w` is consumed: refill it, before the reduction and the epilogue below
        __builtin_amdgcn_sched_barrier(0);
        load_chunk(base2, ch2, b2 < nbatch, w);
        __builtin_amdgcn_sched_barrier(0);

        if (last) {
            // The triangular solve is linear, so it is applied per lane before the reduction
            // (the power-of-two divisions wait until the sums are complete).
            const int g = b * SLOTS + slot;
            int fsum[MT][3];
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                int g12[12];
#pragma unroll
                for (int p = 0; p < 3; ++p) {
                    g12[4 * p + 0] = acc[t][p][0];
                    g12[4 * p + 1] = acc[t][p][1] - acc[t][p][0];
                    g12[4 * p + 2] = acc[t][p][2] - acc[t][p][1];
                    g12[4 * p + 3] = acc[t][p][2] - acc[t][p][3];
#pragma unroll
                    for (int m = 0; m < 4; ++m) acc[t][p][m] = 0;
                }
                reduce_rows<LW>(g12, lane, fsum[t]);
            }

            if constexpr (WS > 1) {
                // one lane per 16-lane row publishes its wavefront's sums; the first
                // wavefront of the slot adds the others.  Two buffers alternate so that one
                // barrier per batch is enough.
                const int rho = lane >> 4;
                int* mine = red + ((parity * NW + wave) * 4 + rho) * (3 * MT);
                if ((lane & 15) == 0) {
#pragma unroll
                    for (int t = 0; t < MT; ++t)
#pragma unroll
                        for (int p = 0; p < 3; ++p) mine[3 * t + p] = fsum[t][p];
                }
                __syncthreads();
                if (wsub == 0 && (lane & 15) == 0) {
#pragma unroll
                    for (int ws = 1; ws < WS; ++ws) {
                        const int* other = red + ((parity * NW + wave + ws) * 4 + rho) * (3 * MT);
#pragma unroll
                        for (int t = 0; t < MT; ++t)
#pragma unroll
                            for (int p = 0; p < 3; ++p) fsum[t][p] += other[3 * t + p];
                    }
                }
                parity ^= 1;
            }

            if (g < G && wsub == 0 && lane_writes<LW>(lane)) {
                const int r = my_row;
                const int h = 4 * g + r;
                const float c0 = half_bits_to_float(static_cast<uint16_t>(lut_cur.x & 0xffffu));
                const float c1 = half_bits_to_float(static_cast<uint16_t>(lut_cur.x >> 16));
                const float c2 = half_bits_to_float(static_cast<uint16_t>(lut_cur.y & 0xffffu));
                const float c3 = half_bits_to_float(static_cast<uint16_t>(lut_cur.y >> 16));
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    if (t >= M) continue;
                    const int F0 = fsum[t][0] >> r, F1 = fsum[t][1] >> r, F3 = fsum[t][2] >> r;
                    const int P3 = F3, P1 = F0 - F3, P2 = F1 - F3;
                    const int P0 = T[t] - F0 - F1 + F3;
                    float o = c0 * static_cast<float>(P0);
                    o = fmaf(c1, static_cast<float>(P1), o);
                    o = fmaf(c2, static_cast<float>(P2), o);
                    o = fmaf(c3, static_cast<float>(P3), o);
                    o *= sc[t];
                    const size_t oi = static_cast<size_t>(t) * N + h;
                    if constexpr (OUT_F16) static_cast<__half*>(out)[oi] = round_to_half(o);
                    else static_cast<float*>(out)[oi] = o;
                    if (Pout != nullptr)
                        reinterpret_cast<int4*>(Pout)[oi] = make_int4(P0, P1, P2, P3);
                }
            }
            // LUT of this lane's row in the next batch; its previous value has just been used
            lut_row = min(lut_row + 4 * nblk * SLOTS, N - 1);
            lut_cur = codebook[lut_row];
        }
        b = b1;
        ch = ch1;
        base = base1;
        b1 = b2;
        ch1 = ch2;
        base1 = base2;
        advance(b2, ch2, base2);
    };
    // The steps of this workgroup are counted up front and run in pairs, so that the loop has one
    // body (wA, then wB) and one exit.  With an exit after either step the two exit branches are
    // merged with the back edge, the wait-count analysis then sees a path "refill of wA just
    // issued -> top of the loop" and makes every other step wait for all loads in flight, which
    // undoes the prefetching.
    const int my_batches = (nbatch - static_cast<int>(blockIdx.x) + nblk - 1) / nblk;
    const int nsteps = my_batches * nchunk;
    for (int i = 0; i < nsteps / 2; ++i) {
        step(wA);
        step(wB);
    }
    if (nsteps & 1) step(wA);
}

constexpr int GEMM_MFMA_MIN_M = 2;  // one token always stays on the plain-ALU kernel

struct GemvPlan {
    int lw, ws, unr, blocks;
};

struct GemvArgs {
    const void *packed, *codebook;
    int N, K;
    const void *xq, *scale;
    int M;
    void* out;
    rcp_dtype out_dt;
    int32_t* P;
    // fused quantiser (xraw != nullptr): raw activation of one token
    const void* xraw;
    rcp_dtype x_dt;
    float clip_ratio;
    void *xq_out, *scale_out;
    int rot_n, rot_m;  // Hadamard across rot_n heads of rot_m channels in the prologue (0: none)
    bool rot_wht;      // instead: the order-K Hadamard rotation (rot_n = K, rot_m = log2 K)
};

template <int LW, int WS, int UNR, int MT, bool OUT_F16, int XDT, int NW = GEMV_WAVES, bool NT = false>
static int launch_one(const GemvArgs& a, int blocks, hipStream_t st)
{
    const size_t lds = gemv_x_bytes(a.K, a.M, LW * WS * UNR) + (NW * MT + NW) * sizeof(int) +
                       (WS > 1 ? 2 * NW * 4 * 3 * MT * sizeof(int) : 0) +
                       (XDT >= 4 ? static_cast<size_t>(a.K) * sizeof(float) + 16 : 0);
    if (lds > 160 * 1024)
        return fail(RCP_ERR_UNSUPPORTED, "rcp_w2a4_gemv: M*K/2 = %d bytes of activations exceed the LDS budget", a.M * (a.K / 2));
    auto kernel = &gemv_kernel<LW, WS, UNR, MT, OUT_F16, XDT, NW, NT>;
    if (lds > 65536) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e != hipSuccess) return fail(RCP_ERR_HIP, "rcp_w2a4_gemv: LDS opt-in failed: %s", hipGetErrorString(e));
    }
    kernel<<<blocks, NW * 64, lds, st>>>(
        static_cast<const uint4*>(a.packed), static_cast<const uint2*>(a.codebook), a.N, a.K,
        a.xraw != nullptr ? a.xraw : a.xq, static_cast<const uint16_t*>(a.scale), a.M, a.clip_ratio, blocks,
        a.rot_n > 0 ? (a.rot_wht ? a.rot_m : (a.rot_n | (a.rot_m << 8))) : 0, a.out, a.P,
        static_cast<uint32_t*>(a.xq_out), static_cast<uint16_t*>(a.scale_out));
    return check_launch("rcp_w2a4_gemv");
}

// The fused one-token call on eight wavefronts, two per row group: for matrices with so few rows that
// every compute unit gets a single workgroup, the quantiser and the dot products of that workgroup
// then run on two wavefronts per SIMD.
template <int UNR>
static int launch_wide(const GemvArgs& a, int blocks, hipStream_t st)
{
#define RCP_GO8(XDT)                                                                       \
    return a.out_dt == RCP_F16 ? launch_one<64, 2, UNR, 1, true, XDT, 8>(a, blocks, st)    \
                               : launch_one<64, 2, UNR, 1, false, XDT, 8>(a, blocks, st)
    if (a.x_dt == RCP_F16) RCP_GO8(RCP_F16);
    if (a.x_dt == RCP_F32) RCP_GO8(RCP_F32);
    RCP_GO8(RCP_BF16);
#undef RCP_GO8
}

// One token, one wavefront or half a wavefront per row group, 8 MB of packed weights and more: the non-temporal form.
template <int LW, int UNR>
static int launch_nt(const GemvArgs& a, int blocks, hipStream_t st)
{
#define RCP_GO_NT(XDT)                                                                                        \
    return a.out_dt == RCP_F16 ? launch_one<LW, 1, UNR, 1, true, XDT, GEMV_WAVES, true>(a, blocks, st)        \
                               : launch_one<LW, 1, UNR, 1, false, XDT, GEMV_WAVES, true>(a, blocks, st)
    if (a.xraw == nullptr) RCP_GO_NT(-1);
    if (a.x_dt == RCP_F16) RCP_GO_NT(RCP_F16);
    if (a.x_dt == RCP_F32) RCP_GO_NT(RCP_F32);
    RCP_GO_NT(RCP_BF16);
#undef RCP_GO_NT
}

template <int LW, int WS, int UNR>
static int launch_mt(const GemvArgs& a, int blocks, hipStream_t st)
{
#define RCP_GO(MT, XDT)                                                                   \
    return a.out_dt == RCP_F16 ? launch_one<LW, WS, UNR, MT, true, XDT>(a, blocks, st)    \
                               : launch_one<LW, WS, UNR, MT, false, XDT>(a, blocks, st)
    if (a.xraw != nullptr) {
        if constexpr (WS == 1) {  // the order-K rotation works on thread numbers only: any lanes per row group
            if (a.rot_n > 0 && a.rot_wht) {
                if (a.x_dt == RCP_F16) RCP_GO(1, 8 + RCP_F16);
                if (a.x_dt == RCP_F32) RCP_GO(1, 8 + RCP_F32);
                RCP_GO(1, 8 + RCP_BF16);
            }
        }
        if constexpr (LW == 64 && WS == 1) {  // the rotation across heads exists for one wavefront per row group only
            if (a.rot_n > 0) {
                if (a.x_dt == RCP_F16) RCP_GO(1, 4 + RCP_F16);
                if (a.x_dt == RCP_F32) RCP_GO(1, 4 + RCP_F32);
                RCP_GO(1, 4 + RCP_BF16);
            }
        }
        if (a.x_dt == RCP_F16) RCP_GO(1, RCP_F16);
        if (a.x_dt == RCP_F32) RCP_GO(1, RCP_F32);
        RCP_GO(1, RCP_BF16);
    }
    if (a.M == 1) RCP_GO(1, -1);
    if (a.M == 2) RCP_GO(2, -1);
    if (a.M <= 4) RCP_GO(4, -1);
    if (a.M <= 8) RCP_GO(8, -1);
    RCP_GO(16, -1);
#undef RCP_GO
}

// Shape -> (lanes per row group, loads in flight, workgroups).
static GemvPlan plan_gemv(int N, int K, int M, bool fused)
{
    const Options& opt = options();
    const int G = N / 4, U = K / 16;
    const int cus = num_compute_units();
    GemvPlan p;
    int lanes = opt.gemv_lanes;
    if (lanes == 0) {
        // one wavefront per row group; more only when there are fewer row groups than
        // compute units (sweeps: the cross-wavefront step costs more than it gains otherwise)
        lanes = 64;
        if (G < cus) lanes = 128;
        if (2 * G < cus) lanes = 256;
        // Several tokens multiply the per-row-group reduction and epilogue: tall matrices then
        // do better with fewer lanes per row group, which pay them once for 2 or 4 row groups
        // (sweeps on 12288 x 4096 and 22016 x 4096 at M = 4, 8, 16).
        // (from 16 row groups per compute unit on the same holds for one token: 22016 x 4096 fused
        // 7.2 -> 6.75 us, while 12288 x 4096 with 12 per unit is better off with whole wavefronts)
        if (G >= 16 * cus) lanes = 32;
        else if (M > 8 && G >= 8 * cus) lanes = 16;
        while (lanes > 16 && U < lanes) lanes /= 2;  // never more lanes than a row group has units
    }
    p.lw = lanes < 64 ? lanes : 64;
    p.ws = lanes < 64 ? 1 : lanes / 64;
    p.unr = (opt.gemv_unroll == 2 || opt.gemv_unroll == 4) ? opt.gemv_unroll : (U > lanes * 4 ? 4 : 2);
    if (M > 2) p.unr = 2;  // the token dimension multiplies the accumulators; keep registers in check
    // fused quantiser on a matrix that gives every workgroup a single batch whose row group is exactly four loads
    // per lane (4096 x 4096): all loads at once, one step (sweep: 3.69 -> 3.47 us; with activations quantised
    // beforehand two steps of two stay ahead, 2.88 vs 2.99 us, and taller matrices lose 10-15 %)
    if (fused && opt.gemv_unroll == 0 && M == 1 && U == lanes * 4 && lanes == 64 && (G + 3) / 4 <= cus) p.unr = 4;
    const int slots = (GEMV_WAVES / p.ws) * (64 / p.lw);
    const int nbatch = (G + slots - 1) / slots;
    int blocks = opt.gemv_blocks;
    if (blocks == 0) blocks = nbatch <= cus * 8 ? nbatch : cus * 4;
    // every workgroup stages the activations (and quantises them itself when fused): fewer, longer-lived
    // workgroups -- two per compute unit (sweeps: 12288 x 4096 4.99 -> 4.84 us, 22016 x 4096 7.5 -> 6.8 us un-fused)
    (void)fused;
    if (opt.gemv_blocks == 0 && blocks > cus * 2) blocks = cus * 2;
    if (blocks > nbatch) blocks = nbatch;
    if (blocks < 1) blocks = 1;
    p.blocks = blocks;
    return p;
}

// Measured crossover on LLaMA-sized layers: 3 tokens, or 2 when the matrix is tall enough to fill the
// chip with 64-row blocks; below that many rows the matrix-core kernel runs with 16-row blocks and is
// level with the plain-ALU kernel at 2 tokens.
int gemv_variant(int N, int /*K*/, int M)
{
    const int forced = options().gemv_variant;
    if (forced == 1 || forced == 2) return forced;
    const bool many = M > GEMM_MFMA_MIN_M || (M == GEMM_MFMA_MIN_M && N >= 8192);
    return many ? 2 : 1;
}

static int dispatch_gemv(const GemvArgs& a, hipStream_t st)
{
    if (static_cast<long long>(a.N) * a.K / 4 >= (1LL << 31))
        return fail(RCP_ERR_SHAPE, "rcp_w2a4_gemv: packed matrix of %lld bytes exceeds 2 GiB", static_cast<long long>(a.N) * a.K / 4);
    // several tokens: the contraction goes to the matrix cores (the fused quantiser is one token only)
    if (a.xraw == nullptr && gemv_variant(a.N, a.K, a.M) == 2)
        return launch_gemm_mfma(a.packed, a.codebook, a.N, a.K, a.xq, a.scale, a.M, a.out, a.out_dt, a.P, st);
    // one token, no rotation in the prologue, one row group per wavefront: every load issued up front
    if (a.M == 1 && a.rot_n == 0 && options().gemv_variant != 2 && options().gemv_waves != 8 &&
        gemv_oneshot_applies(a.N, a.K, a.xraw != nullptr))
        return launch_gemv_oneshot(a.packed, a.codebook, a.N, a.K, a.xraw != nullptr ? a.xraw : a.xq,
                                   a.xraw != nullptr ? static_cast<int>(a.x_dt) : -1, a.scale, a.clip_ratio, a.out, a.out_dt, a.P,
                                   a.xq_out, a.scale_out, st);
    GemvPlan p = plan_gemv(a.N, a.K, a.M, a.xraw != nullptr);
    if (a.rot_n > 0 && (!a.rot_wht || p.ws > 1)) {  // rotating prologue: one wavefront per row group at most
        p.lw = 64;
        p.ws = 1;
        const int nbatch = (a.N / 4 + GEMV_WAVES - 1) / GEMV_WAVES;
        if (p.blocks > nbatch) p.blocks = nbatch;
    }
    // one token, fused quantiser, no rotation, a single workgroup per compute unit and a long input
    // (the quantiser's share grows with K): eight wavefronts.  Sweeps: 4096 x 11008 gains 9 %,
    // 4096 x 4096 nothing, matrices with more workgroups than compute units lose.
    // ("gemv_waves" = 8 forces this form, 4 forbids it)
    const int want_waves = options().gemv_waves;
    const bool wide_ok = a.xraw != nullptr && a.rot_n == 0 && a.K / 16 >= 128 && options().gemv_lanes == 0;
    // (with fp32 activations the two forms are within 2 % of each other: left on four wavefronts)
    const bool wide_pays = (a.N / 4 + 3) / 4 <= num_compute_units() && a.K >= 8192 && a.x_dt != RCP_F32;
    if (wide_ok && (want_waves == 8 || (want_waves == 0 && wide_pays))) {
        const int nbatch = (a.N / 4 + 3) / 4;  // four row groups per workgroup, as with four wavefronts
        int blocks = options().gemv_blocks;
        if (blocks == 0 || blocks > nbatch) blocks = nbatch;
        if (blocks > 2 * num_compute_units() && options().gemv_blocks == 0) blocks = 2 * num_compute_units();
        return options().gemv_unroll == 4 ? launch_wide<4>(a, blocks, st) : launch_wide<2>(a, blocks, st);
    }
    // Non-temporal weight loads ("gemv_nt": 1 = whenever a form below runs, 2 = never).  Measured by itself a launch on
    // 4 - 22 MB is within 2 % with and without the hint; inside the decode step, where 1.6 GB of weights pass between two
    // uses of anything, the hint on the q|k|v, gate|up and down launches is worth 3 % of the step (0.743 -> 0.720 ms):
    // weights that are read once no longer push the activations, tables and Q out of the caches.  The 4 MB of the
    // out-projection are better off without it (0.720 against 0.722 ms), hence the threshold.
    const bool nt = options().gemv_nt != 0 ? options().gemv_nt == 1
                                           : static_cast<long long>(a.N) * a.K / 4 >= (8LL << 20);
    if (nt && a.M == 1 && a.rot_n == 0 && p.ws == 1) {
        if (p.lw == 32 && p.unr == 4) return launch_nt<32, 4>(a, p.blocks, st);
        if (p.lw == 64) return p.unr == 4 ? launch_nt<64, 4>(a, p.blocks, st) : launch_nt<64, 2>(a, p.blocks, st);
    }
    if (p.unr == 2) {
        switch (p.lw * p.ws) {
            case 16: return launch_mt<16, 1, 2>(a, p.blocks, st);
            case 32: return launch_mt<32, 1, 2>(a, p.blocks, st);
            case 64: return launch_mt<64, 1, 2>(a, p.blocks, st);
            case 128: return launch_mt<64, 2, 2>(a, p.blocks, st);
            default: return launch_mt<64, 4, 2>(a, p.blocks, st);
        }
    }
    switch (p.lw * p.ws) {
        case 16: return launch_mt<16, 1, 4>(a, p.blocks, st);
        case 32: return launch_mt<32, 1, 4>(a, p.blocks, st);
        case 64: return launch_mt<64, 1, 4>(a, p.blocks, st);
        case 128: return launch_mt<64, 2, 4>(a, p.blocks, st);
        default: return launch_mt<64, 4, 4>(a, p.blocks, st);
    }
}

int launch_gemv(const void* packed, const void* codebook, int N, int K, const void* xq,
                const void* scale, int M, void* out, rcp_dtype out_dt, int32_t* P, hipStream_t st)
{
    const GemvArgs a = {packed, codebook, N, K, xq, scale, M, out, out_dt, P, nullptr, RCP_F16, 1.0f, nullptr, nullptr, 0, 0, false};
    return dispatch_gemv(a, st);
}

bool quant_gemv_supported(int K) { return K / 8 <= GEMV_XG * GEMV_THREADS; }

int launch_quant_gemv(const void* packed, const void* codebook, int N, int K, const void* x, rcp_dtype x_dt,
                      float clip_ratio, void* out, rcp_dtype out_dt, void* xq_out, void* scale_out, int32_t* P,
                      int rot_heads, int rot_head_dim, hipStream_t st)
{
    const GemvArgs a = {packed, codebook, N, K, nullptr, nullptr, 1, out, out_dt, P, x, x_dt, clip_ratio, xq_out, scale_out,
                        rot_heads, rot_head_dim, false};
    return dispatch_gemv(a, st);
}

bool wht_gemv_supported(int K) { return K >= 32 && K <= 2048 && (K & (K - 1)) == 0; }

int launch_wht_quant_gemv(const void* packed, const void* codebook, int N, int K, const void* x, rcp_dtype x_dt,
                          float clip_ratio, void* out, rcp_dtype out_dt, void* xq_out, void* scale_out, int32_t* P,
                          hipStream_t st)
{
    int log2n = 0;
    while ((1 << log2n) < K) ++log2n;
    const GemvArgs a = {packed, codebook, N, K, nullptr, nullptr, 1, out, out_dt, P, x, x_dt, clip_ratio, xq_out, scale_out,
                        K, log2n, true};
    return dispatch_gemv(a, st);
}

}  // namespace rcp
