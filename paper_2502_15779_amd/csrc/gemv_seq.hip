// A sequence of dependent one-token W2A4 GEMVs in ONE launch (Section 4.4 states the GEMV; its
// "latency hiding" idea -- have the next weights in flight while something else is being waited for --
// is applied here one level up, across the dependency between consecutive linear layers of a decoder).
//
// Entry i computes exactly what rcp_rotate_act (Kronecker rotations only) followed by
// rcp_quant_w2a4_gemv computes, and may read the output of any earlier entry: every workgroup
// finishes entry i, publishes its rows, and all workgroups meet before any of them reads the
// activation of entry i + 1.  What does not depend on that meeting -- the packed weights and the
// LUT rows of entry i + 1, more than 99.9 % of its bytes -- is requested BEFORE the workgroup
// waits, so the HBM stream of the next matrix overlaps the meeting and the quantiser.
//
// Meeting ("hop") between workgroups of different dies, without fences (an L2 write-back per workgroup
// costs tens of microseconds on this 8-die part):
//   * results that other workgroups read inside the launch are written with device-scope stores
//     (write-through to the point where all dies see them) and read with device-scope loads (never served
//     from a compute unit's own cache).  Such loads are issued wide and coalesced only -- the rotation stages
//     its input in LDS first, its strided reads straight from memory cost 4 us more -- and a device-scope
//     acquire fence followed by ordinary loads is no alternative: measured, the fence's cache invalidation
//     in every wavefront takes 15-20 us per meeting;
//   * a workgroup waits until its stores are acknowledged (s_waitcnt vmcnt(0) in every thread, then a
//     workgroup barrier), then its first thread adds 1 to one of 16 arrival counters (a single
//     counter serialises 512 read-modify-writes on one address: 6.6 us measured; 16 + 1: 1.8 us);
//     the last arrival of a counter adds 1 to the top counter, the last arrival there writes the "go"
//     word, which every workgroup polls (bounded);
//   * counters and go words are left at zero by the launch itself (the last arrival clears its counter,
//     the go word of a hop is cleared by the last arrival of the following hop, when every workgroup has
//     passed it), so a workspace zeroed once serves every later launch without a memset.
// No workgroup waits for anything but "all workgroups arrived at hop h", and arriving at hop h needs
// only hops < h: with all workgroups resident at once (checked against the occupancy on the host) every
// wait ends.  Every poll loop is bounded all the same; a loop that runs out sets the error word of the
// workspace, after which all waits fall through and the launch drains with undefined outputs.
#include <math.h>
#include <string.h>

#include <type_traits>

#include "rcp_internal.hpp"

namespace rcp {

constexpr int SEQ_THREADS = 256;
constexpr int SEQ_WAVES = SEQ_THREADS / 64;
constexpr int SEQ_SUB = 16;                          // arrival counters below the top counter
constexpr int SEQ_HOP_DWORDS = 32 * (SEQ_SUB + 2);   // top counter, SEQ_SUB counters, go word: a 128-byte line each
constexpr int SEQ_HEADER_BYTES = 256;                // word 0: error flag
constexpr int SEQ_SPIN_LIMIT = 1 << 21;              // polls of about 0.2 us each before a wait gives up
constexpr int SEQ_XG = 8;                            // groups of eight raw activations a thread holds: K <= 16384
constexpr int SEQ_AUX_DEVICE = 16;                   // buffer cache policy bit sc1: device scope

struct SeqStep {
    const uint4* packed;
    const uint2* codebook;
    const void* x;
    void* out;
    const float* Q;
    uint32_t* xq_out;
    uint16_t* scale_out;
    int N, K;
    int x_dt;      // rcp_dtype of x
    int out_f16;   // 1: fp16 output, 0: binary32
    int rot_n;     // Hadamard factor of a Kronecker rotation, 0: no rotation
    int rot_m;     // order of Q
    float clip_ratio;
    int unr;       // 16-byte weight loads per lane and pipeline stage: 2 or 4
};

struct SeqArgs {
    int n;
    int nwg;
    int lds_x_bytes;  // LDS bytes reserved for the staged activations (largest entry)
    int max_rpl;      // largest (Hadamard factor / 64) of the rotated entries
    SeqStep s[RCP_SEQ_MAX_STEPS];
};

__device__ __forceinline__ uint32_t ld_dev(const uint32_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_dev(uint32_t* p, uint32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ uint32_t add_dev(uint32_t* p) { return __hip_atomic_fetch_add(p, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// First thread of a workgroup whose stores are acknowledged: count the arrival.  The last arrival of all
// clears the go word of the previous hop (nobody polls it any more) and, unless this is the closing hop of
// the launch, opens this one.
__device__ __forceinline__ void hop_arrive(uint32_t* hop, uint32_t* prev_go, bool open, int nwg)
{
    const int nsub = nwg < SEQ_SUB ? nwg : SEQ_SUB;
    const int sub = static_cast<int>(blockIdx.x) % nsub;
    const int members = (nwg - sub + nsub - 1) / nsub;
    uint32_t* c = hop + 32 * (1 + sub);
    if (add_dev(c) == static_cast<uint32_t>(members - 1)) {
        st_dev(c, 0u);
        if (add_dev(hop) == static_cast<uint32_t>(nsub - 1)) {
            st_dev(hop, 0u);
            if (prev_go != nullptr) st_dev(prev_go, 0u);
            if (open) st_dev(hop + 32 * (SEQ_SUB + 1), 1u);
        }
    }
}

// First thread of a workgroup: wait until the hop is open (bounded).
__device__ __forceinline__ void hop_wait(const uint32_t* go, uint32_t* err)
{
    int spins = 0;
    while (ld_dev(go) == 0u) {
        ++spins;
        if ((spins & 63) == 0 && (spins > SEQ_SPIN_LIMIT || ld_dev(err) != 0u)) {
            st_dev(err, 1u);
            break;
        }
        __builtin_amdgcn_s_sleep(1);
    }
}

// Eight consecutive raw activations through a buffer resource with device-scope loads.
template <int DT>
__device__ __forceinline__ Raw8<DT> load8_raw_dev(__amdgpu_buffer_rsrc_t res, int group)
{
    Raw8<DT> r;
    if constexpr (DT == RCP_F32) {
        const u32x4 a = __builtin_amdgcn_raw_buffer_load_b128(res, group * 32, 0, SEQ_AUX_DEVICE);
        const u32x4 b = __builtin_amdgcn_raw_buffer_load_b128(res, group * 32 + 16, 0, SEQ_AUX_DEVICE);
        r.a = make_uint4(a.x, a.y, a.z, a.w);
        r.b = make_uint4(b.x, b.y, b.z, b.w);
    } else {
        const u32x4 a = __builtin_amdgcn_raw_buffer_load_b128(res, group * 16, 0, SEQ_AUX_DEVICE);
        r.a = make_uint4(a.x, a.y, a.z, a.w);
        r.b = make_uint4(0u, 0u, 0u, 0u);
    }
    return r;
}

// Column jcol of Y = H_n X Q^T (n = 64 * RPL rows, m columns), the arithmetic of the stand-alone rotation
// kernel of the same shape: lane l owns rows l*RPL .. l*RPL + RPL - 1, the four wavefronts split the sum
// over j, the partial sums meet in LDS in a fixed order, the first wavefront runs the order-n Hadamard
// transform (ascending stride) and stores the column.  x is read and y written at device scope.
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
constexpr int SEQ_KRON_MAXQ = 16;

template <bool X32, int RPL>
__device__ __forceinline__ void kron_column(const uint32_t* sxraw /* LDS: the K raw input values */, bool bf16, int m,
                                            const float* sq /* LDS: row jcol of Q */, float norm, float* y, int jcol,
                                            float* part /* [4][64*RPL] */)
{
    constexpr int QW = SEQ_KRON_MAXQ / RPL;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int K = 64 * RPL * m, quads = m / 4;
    const int q0 = wave * quads / 4, q1 = (wave + 1) * quads / 4;
    const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(y, 0, K * 4, 0x00020000);

    u32x4 raw[RPL][QW];
#pragma unroll
    for (int t = 0; t < QW; ++t) {
#pragma unroll
        for (int e = 0; e < RPL; ++e) {
            raw[e][t] = u32x4{0u, 0u, 0u, 0u};
            if (q0 + t < q1) {  // uniform
                const int elem = (lane * RPL + e) * m + 4 * (q0 + t);
                if constexpr (X32) {
                    raw[e][t] = *reinterpret_cast<const u32x4*>(sxraw + elem);
                } else {
                    const u32x2 r = *reinterpret_cast<const u32x2*>(sxraw + elem / 2);
                    raw[e][t].x = r.x;
                    raw[e][t].y = r.y;
                }
            }
        }
    }
    float acc[RPL];
#pragma unroll
    for (int e = 0; e < RPL; ++e) acc[e] = 0.0f;
#pragma unroll
    for (int t = 0; t < QW; ++t) {
        if (q0 + t < q1) {
            const float4 q4 = reinterpret_cast<const float4*>(sq)[q0 + t];  // one address for the wavefront: LDS broadcast
#pragma unroll
            for (int e = 0; e < RPL; ++e) {
                float x0, x1, x2, x3;
                if constexpr (X32) {
                    x0 = __uint_as_float(raw[e][t].x); x1 = __uint_as_float(raw[e][t].y);
                    x2 = __uint_as_float(raw[e][t].z); x3 = __uint_as_float(raw[e][t].w);
                } else {
                    const uint32_t a = raw[e][t].x, b = raw[e][t].y;
                    if (bf16) {  // uniform
                        x0 = bf16_bits_to_float(static_cast<uint16_t>(a & 0xffffu)); x1 = bf16_bits_to_float(static_cast<uint16_t>(a >> 16));
                        x2 = bf16_bits_to_float(static_cast<uint16_t>(b & 0xffffu)); x3 = bf16_bits_to_float(static_cast<uint16_t>(b >> 16));
                    } else {
                        x0 = half_bits_to_float(static_cast<uint16_t>(a & 0xffffu)); x1 = half_bits_to_float(static_cast<uint16_t>(a >> 16));
                        x2 = half_bits_to_float(static_cast<uint16_t>(b & 0xffffu)); x3 = half_bits_to_float(static_cast<uint16_t>(b >> 16));
                    }
                }
                acc[e] = fmaf(x0, q4.x, acc[e]);
                acc[e] = fmaf(x1, q4.y, acc[e]);
                acc[e] = fmaf(x2, q4.z, acc[e]);
                acc[e] = fmaf(x3, q4.w, acc[e]);
            }
        }
    }
#pragma unroll
    for (int e = 0; e < RPL; ++e) part[wave * 64 * RPL + e * 64 + lane] = acc[e];
    __syncthreads();
    if (wave == 0) {
        float z[RPL];
#pragma unroll
        for (int e = 0; e < RPL; ++e)
            z[e] = ((part[e * 64 + lane] + part[64 * RPL + e * 64 + lane]) + part[2 * 64 * RPL + e * 64 + lane]) +
                   part[3 * 64 * RPL + e * 64 + lane];
#pragma unroll
        for (int st = 1; st < RPL; st <<= 1)
#pragma unroll
            for (int e = 0; e < RPL; ++e)
                if ((e & st) == 0) {
                    const float a = z[e], b = z[e + st];
                    z[e] = a + b;
                    z[e + st] = a - b;
                }
#pragma unroll
        for (int e = 0; e < RPL; ++e) {
            float v = z[e];
            const float p1 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false));  // lane ^ 1
            v = (lane & 1) ? p1 - v : v + p1;
            const float p2 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false));  // lane ^ 2
            v = (lane & 2) ? p2 - v : v + p2;
            const float p4 = __shfl_xor(v, 4, 64);
            v = (lane & 4) ? p4 - v : v + p4;
            const float p8 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x128, 0xf, 0xf, false));  // lane ^ 8
            v = (lane & 8) ? p8 - v : v + p8;
            auto r16 = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
            v = (lane & 16) ? __uint_as_float(r16[0]) - __uint_as_float(r16[1]) : __uint_as_float(r16[0]) + __uint_as_float(r16[1]);
            auto r32 = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
            v = (lane & 32) ? __uint_as_float(r32[0]) - __uint_as_float(r32[1]) : __uint_as_float(r32[0]) + __uint_as_float(r32[1]);
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v * norm), yres, ((lane * RPL + e) * m + jcol) * 4, 0, SEQ_AUX_DEVICE);
        }
    }
    __syncthreads();  // `part` is free again
}

// Column `workgroup` of the rotated vector (the host makes sure there are at least as many workgroups as columns).
// A workgroup with a column first copies the whole raw input into LDS with wide device-scope loads (the lanes' own
// reads are strided by m); `after_issue` runs when those loads have been issued -- loads return in issue order, so
// whatever it requests arrives after the input.  Row `workgroup` of Q is already in LDS (`sq`).
template <bool X32, typename F>
__device__ __forceinline__ void kron_columns(const SeqStep& st, float norm, float* y, uint32_t* sxraw, const float* sq,
                                             float* part, F&& after_issue)
{
    const bool bf16 = st.x_dt == RCP_BF16;
    if (static_cast<int>(blockIdx.x) >= st.rot_m) {  // uniform per workgroup
        after_issue();
        return;
    }
    const int bytes = st.K * (X32 ? 4 : 2);
    const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(st.x), 0, bytes, 0x00020000);
    // all loads first (at most 64 KiB: 16 pieces of 16 bytes per thread), then the LDS stores
    constexpr int MAXP = 16;
    u32x4 piece[MAXP];
#pragma unroll
    for (int i = 0; i < MAXP; ++i)
        if (i * SEQ_THREADS * 16 < bytes)  // uniform
            piece[i] = __builtin_amdgcn_raw_buffer_load_b128(xres, (static_cast<int>(threadIdx.x) + i * SEQ_THREADS) * 16, 0, SEQ_AUX_DEVICE);
    __builtin_amdgcn_sched_barrier(0);
    after_issue();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < MAXP; ++i) {
        const int p = threadIdx.x + i * SEQ_THREADS;
        if (i * SEQ_THREADS * 16 < bytes && p * 16 < bytes) *reinterpret_cast<u32x4*>(sxraw + 4 * p) = piece[i];
    }
    __syncthreads();
    const int jcol = blockIdx.x;
    switch (st.rot_n / 64) {
        case 1: kron_column<X32, 1>(sxraw, bf16, st.rot_m, sq, norm, y, jcol, part); break;
        case 2: kron_column<X32, 2>(sxraw, bf16, st.rot_m, sq, norm, y, jcol, part); break;
        case 4: kron_column<X32, 4>(sxraw, bf16, st.rot_m, sq, norm, y, jcol, part); break;
        case 8: kron_column<X32, 8>(sxraw, bf16, st.rot_m, sq, norm, y, jcol, part); break;
        default: kron_column<X32, 16>(sxraw, bf16, st.rot_m, sq, norm, y, jcol, part); break;
    }
}

// Per-token symmetric int4 quantiser of the fused one-token GEMV, reading the K raw values at device scope:
// amax over the workgroup, S = fp16(ratio * amax / 7), q = rint(x / S); x_q to LDS (plain order), its sum returned
// through tsum[wave].  `xsrc` holds K values of type DT.  `after_issue` runs once the loads are on their way.
template <int DT, typename F>
__device__ __forceinline__ float stage_quantised(const void* xsrc, int K, float clip_ratio, uint32_t* sx1, int* tsum,
                                                 float* amax_slots, uint32_t* xq_out, uint16_t* scale_out, F&& after_issue)
{
    constexpr int TH = SEQ_THREADS;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int xdw = K / 8;
    const __amdgpu_buffer_rsrc_t xres =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(xsrc), 0, K * (DT == RCP_F32 ? 4 : 2), 0x00020000);
    Raw8<DT> xraw8[SEQ_XG];
    float xr8[SEQ_XG][8];
#pragma unroll
    for (int i = 0; i < SEQ_XG; ++i) {
        if (i * TH >= xdw) break;  // uniform
        const int u8 = min(static_cast<int>(threadIdx.x) + i * TH, xdw - 1);  // clamped: duplicates are harmless
        xraw8[i] = load8_raw_dev<DT>(xres, u8);
    }
    // loads return in issue order: what `after_issue` requests (the second stage of weights) arrives after the activations
    __builtin_amdgcn_sched_barrier(0);
    after_issue();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < SEQ_XG; ++i) {
        if (i * TH >= xdw) break;
        widen8<DT>(xraw8[i], xr8[i]);
    }
    float a = 0.0f;
#pragma unroll
    for (int i = 0; i < SEQ_XG; ++i) {
        if (i * TH >= xdw) break;
#pragma unroll
        for (int j = 0; j < 8; ++j) a = fmaxf(a, fabsf(xr8[i][j]));
    }
    a = wave_max(a);
    if (lane == 0) amax_slots[wave] = a;
    __syncthreads();
    a = fmaxf(fmaxf(amax_slots[0], amax_slots[1]), fmaxf(amax_slots[2], amax_slots[3]));
    const uint16_t sb = scale_bits_from_amax(a, clip_ratio);
    const float sq = half_bits_to_float(sb);
    const bool publish = blockIdx.x == 0 && xq_out != nullptr;
    int s = 0;
#pragma unroll
    for (int i = 0; i < SEQ_XG; ++i) {
        if (i * TH >= xdw) break;
        const int u8 = threadIdx.x + i * TH;
        if (u8 < xdw) {
            const uint32_t qd = quantize8(xr8[i], sq);
            sx1[u8] = qd;
            if (publish) xq_out[u8] = qd;
            s = dot8(qd, 0x11111111u, s);
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0 && scale_out != nullptr) scale_out[0] = sb;
    s = wave_sum(s);
    if (lane == 0) tsum[wave] = s;
    return sq;
}

// Profiling hook (built only with -DRCP_SEQ_TRACE): the first thread of every workgroup records the 100 MHz
// clock at eight points of every entry into trace[workgroup][entry][8].
#ifdef RCP_SEQ_TRACE
static unsigned long long* g_seq_trace = nullptr;
#define SEQ_MARK(k)                                                                                              \
    do {                                                                                                         \
        if (trace != nullptr && threadIdx.x == 0)                                                                \
            trace[(static_cast<size_t>(blockIdx.x) * RCP_SEQ_MAX_STEPS + si) * 12 + (k)] = __builtin_amdgcn_s_memrealtime(); \
    } while (0)
#define SEQ_TRACE_PARAM , unsigned long long* trace
#else
#define SEQ_MARK(k) do { } while (0)
#define SEQ_TRACE_PARAM
#endif

__global__ __launch_bounds__(SEQ_THREADS) void gemv_sequence_kernel(const SeqArgs args, uint32_t* __restrict__ ws, float* __restrict__ ybuf SEQ_TRACE_PARAM)
{
    extern __shared__ uint4 smem4[];
    constexpr int SLOTS = SEQ_WAVES;  // row groups a workgroup works on at a time (one wavefront each)
    constexpr int LG = 64;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int slot = wave;
    const int my_row = lane_row<64>(lane);
    const int nwg = args.nwg;
    uint32_t* err = ws;
    uint32_t* hops = ws + SEQ_HEADER_BYTES / 4;
    int* tsum = reinterpret_cast<int*>(reinterpret_cast<char*>(smem4) + args.lds_x_bytes);  // [4]
    float* amax_slots = reinterpret_cast<float*>(tsum + SEQ_WAVES);                           // [4]
    float* part = amax_slots + SEQ_WAVES;                                                     // rotation: [4][64 * RPL]
    float* sq = part + 4 * 64 * args.max_rpl;                                                 // rotation: this workgroup's row of Q
    uint32_t* sxraw = reinterpret_cast<uint32_t*>(sq + RCP_MAX_KRON_M);                       // rotation: raw input, K values
    uint32_t* sx1 = reinterpret_cast<uint32_t*>(smem4);
    const uint2* sx2 = reinterpret_cast<const uint2*>(smem4);

    uint32_t* prev_go = nullptr;  // go word of the last hop this launch has used so far
    bool waiting = false;         // a hop has been arrived at and not yet waited for

    for (int si = 0; si < args.n; ++si) {
        const SeqStep& st = args.s[si];
        const int N = st.N, K = st.K;
        const int U = K / 16, G = N / 4;
        const int nbatch = (G + SLOTS - 1) / SLOTS;
        const int my_batches = static_cast<int>(blockIdx.x) < nbatch ? (nbatch - static_cast<int>(blockIdx.x) + nwg - 1) / nwg : 0;
        const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint4*>(st.packed), 0, static_cast<int>(static_cast<unsigned>(G) * static_cast<unsigned>(U) * 16u), 0x00020000);
        const __amdgpu_buffer_rsrc_t ores =
            __builtin_amdgcn_make_buffer_rsrc(st.out, 0, N * (st.out_f16 ? 2 : 4), 0x00020000);
        uint32_t* hop_rot = hops + static_cast<size_t>(2 * si) * SEQ_HOP_DWORDS;
        uint32_t* hop_end = hops + static_cast<size_t>(2 * si + 1) * SEQ_HOP_DWORDS;

        auto body = [&](auto unr_c) {
            constexpr int UNR = decltype(unr_c)::value;
            const int nchunk = (U + LG * UNR - 1) / (LG * UNR);
            const int my_units = (U % (LG * UNR)) != 0 ? (U - lane + LG - 1) / LG : 0x7fffffff;
            auto batch_offset = [&](int bb) -> unsigned { return (static_cast<unsigned>(bb * SLOTS + slot) * U + lane) * 16u; };
            const unsigned batch_stride = static_cast<unsigned>(nwg) * SLOTS * U * 16u;
            auto load_chunk = [&](unsigned base, int ch, bool valid, u32x4 (&w)[UNR]) {
#pragma unroll
                for (int i = 0; i < UNR; ++i) {
                    const int it = ch * UNR + i;
                    const unsigned off = (valid && it < my_units) ? base : 0x80000000u;
                    w[i] = __builtin_amdgcn_raw_buffer_load_b128(wres, static_cast<int>(off), it * LG * 16, 0);
                }
            };
            int b = blockIdx.x, ch = 0;
            unsigned base = batch_offset(b);
            auto advance = [&](int& bb, int& cc, unsigned& bs) {
                if (cc + 1 == nchunk) {
                    bb += nwg;
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
            // ---- nothing below depends on an earlier entry: the weights of the first step, the LUT row, the row of Q.
            // The second step's weights follow the activation loads (loads return in issue order: everything
            // requested here delays the activations that are requested after the wait).
            u32x4 wA[UNR], wB[UNR];
            load_chunk(base, 0, b < nbatch, wA);
            int lut_row = min(4 * (b * SLOTS + slot) + my_row, N - 1);
            uint2 lut_cur = st.codebook[lut_row];
            auto issue_second = [&]() { load_chunk(base1, ch1, b1 < nbatch, wB); };
            auto nothing = []() {};
            if (st.rot_n > 0 && static_cast<int>(blockIdx.x) < st.rot_m && static_cast<int>(threadIdx.x) < st.rot_m / 4)
                reinterpret_cast<float4*>(sq)[threadIdx.x] =
                    reinterpret_cast<const float4*>(st.Q + static_cast<size_t>(blockIdx.x) * st.rot_m)[threadIdx.x];
            __builtin_amdgcn_sched_barrier(0);
            SEQ_MARK(1);

            // ---- the meeting with the earlier entries
            if (waiting) {
                if (threadIdx.x == 0) hop_wait(prev_go, err);
                __syncthreads();
                waiting = false;
            }
            SEQ_MARK(2);
            const void* xsrc = st.x;
            int x_dt = st.x_dt;
            if (st.rot_n > 0) {
                const float norm = static_cast<float>(1.0 / sqrt(static_cast<double>(st.rot_n)));
                if (st.x_dt == RCP_F32) kron_columns<true>(st, norm, ybuf, sxraw, sq, part, issue_second);
                else kron_columns<false>(st, norm, ybuf, sxraw, sq, part, issue_second);
                SEQ_MARK(9);
                __builtin_amdgcn_s_waitcnt(0);  // this thread's stores of y are acknowledged
                __syncthreads();
                SEQ_MARK(10);
                if (threadIdx.x == 0) {
                    hop_arrive(hop_rot, prev_go, true, nwg);
                    hop_wait(hop_rot + 32 * (SEQ_SUB + 1), err);
                }
                SEQ_MARK(11);
                prev_go = hop_rot + 32 * (SEQ_SUB + 1);
                __syncthreads();
                xsrc = ybuf;
                x_dt = RCP_F32;
            }
            SEQ_MARK(3);

            if (my_batches > 0) {
                float sc;
                if (st.rot_n > 0) sc = stage_quantised<RCP_F32>(xsrc, K, st.clip_ratio, sx1, tsum, amax_slots, st.xq_out, st.scale_out, nothing);
                else if (x_dt == RCP_F16) sc = stage_quantised<RCP_F16>(xsrc, K, st.clip_ratio, sx1, tsum, amax_slots, st.xq_out, st.scale_out, issue_second);
                else if (x_dt == RCP_F32) sc = stage_quantised<RCP_F32>(xsrc, K, st.clip_ratio, sx1, tsum, amax_slots, st.xq_out, st.scale_out, issue_second);
                else sc = stage_quantised<RCP_BF16>(xsrc, K, st.clip_ratio, sx1, tsum, amax_slots, st.xq_out, st.scale_out, issue_second);
                __syncthreads();
                SEQ_MARK(4);
                const int T = tsum[0] + tsum[1] + tsum[2] + tsum[3];

                int acc[1][3][4];
#pragma unroll
                for (int p = 0; p < 3; ++p)
#pragma unroll
                    for (int m = 0; m < 4; ++m) acc[0][p][m] = 0;

                auto step = [&](u32x4 (&w)[UNR]) {
                    const bool last = ch + 1 == nchunk;
                    const uint2* xrow = sx2 + lane + ch * UNR * LG;
#pragma unroll
                    for (int i = 0; i < UNR; ++i) {
                        const uint2 xv = xrow[i * LG];
                        const uint32_t xa[1] = {xv.x}, xb[1] = {xv.y};
                        cell_update<1>(w[i].x, w[i].y, xa, acc);
                        cell_update<1>(w[i].z, w[i].w, xb, acc);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    load_chunk(base2, ch2, b2 < nbatch, w);
                    __builtin_amdgcn_sched_barrier(0);
                    if (last) {
                        const int g = b * SLOTS + slot;
                        int g12[12], fsum[3];
#pragma unroll
                        for (int p = 0; p < 3; ++p) {
                            g12[4 * p + 0] = acc[0][p][0];
                            g12[4 * p + 1] = acc[0][p][1] - acc[0][p][0];
                            g12[4 * p + 2] = acc[0][p][2] - acc[0][p][1];
                            g12[4 * p + 3] = acc[0][p][2] - acc[0][p][3];
#pragma unroll
                            for (int m = 0; m < 4; ++m) acc[0][p][m] = 0;
                        }
                        reduce_rows<64>(g12, lane, fsum);
                        if (g < G && lane_writes<64>(lane)) {
                            const int r = my_row;
                            const int h = 4 * g + r;
                            const float c0 = half_bits_to_float(static_cast<uint16_t>(lut_cur.x & 0xffffu));
                            const float c1 = half_bits_to_float(static_cast<uint16_t>(lut_cur.x >> 16));
                            const float c2 = half_bits_to_float(static_cast<uint16_t>(lut_cur.y & 0xffffu));
                            const float c3 = half_bits_to_float(static_cast<uint16_t>(lut_cur.y >> 16));
                            const int F0 = fsum[0] >> r, F1 = fsum[1] >> r, F3 = fsum[2] >> r;
                            const int P3 = F3, P1 = F0 - F3, P2 = F1 - F3;
                            const int P0 = T - F0 - F1 + F3;
                            float o = c0 * static_cast<float>(P0);
                            o = fmaf(c1, static_cast<float>(P1), o);
                            o = fmaf(c2, static_cast<float>(P2), o);
                            o = fmaf(c3, static_cast<float>(P3), o);
                            o *= sc;
                            // device scope: a later entry of this launch may read the value from another die
                            if (st.out_f16)
                                __builtin_amdgcn_raw_buffer_store_b16(__half_as_ushort(round_to_half(o)), ores, h * 2, 0, SEQ_AUX_DEVICE);
                            else
                                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(o), ores, h * 4, 0, SEQ_AUX_DEVICE);
                        }
                        lut_row = min(lut_row + 4 * nwg * SLOTS, N - 1);
                        lut_cur = st.codebook[lut_row];
                    }
                    b = b1;
                    ch = ch1;
                    base = base1;
                    b1 = b2;
                    ch1 = ch2;
                    base1 = base2;
                    advance(b2, ch2, base2);
                };
                const int nsteps = my_batches * nchunk;
                for (int i = 0; i < nsteps / 2; ++i) {
                    step(wA);
                    step(wB);
                }
                if (nsteps & 1) step(wA);
            }
            // keep the first loads alive on the path without work, so that they are issued before the wait either way
            asm volatile("" ::"v"(wA[0].x), "v"(lut_cur.x));
        };
        SEQ_MARK(0);
        if (st.unr == 4) body(std::integral_constant<int, 4>{});
        else body(std::integral_constant<int, 2>{});
        SEQ_MARK(5);

        // ---- publish: stores acknowledged in every thread, then one arrival per workgroup
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        SEQ_MARK(6);
        const bool closing = si + 1 == args.n;
        if (threadIdx.x == 0) hop_arrive(hop_end, prev_go, !closing, nwg);
        SEQ_MARK(7);
        prev_go = hop_end + 32 * (SEQ_SUB + 1);
        waiting = !closing;
    }
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
// The layout of a workspace does not depend on the number of entries (header, the hops of the longest sequence, then
// the rotated vector), so that calls with different sequences may share one workspace.
static size_t seq_hop_area_bytes()
{
    const size_t bytes = SEQ_HEADER_BYTES + static_cast<size_t>(2 * RCP_SEQ_MAX_STEPS + 1) * SEQ_HOP_DWORDS * 4;
    return (bytes + 255) & ~static_cast<size_t>(255);
}

static bool kron_fits(int n, int m)
{
    return m % 4 == 0 && m >= 8 && n >= 64 && n <= 1024 && (n / 64) * ((m / 4 + 3) / 4) <= SEQ_KRON_MAXQ;
}

size_t gemv_sequence_workspace_bytes(const rcp_gemv_step* steps, int n)
{
    size_t max_rot = 0;
    for (int i = 0; i < n; ++i)
        if (steps[i].rot.kind == RCP_ROT_KRON && static_cast<size_t>(steps[i].K) > max_rot) max_rot = steps[i].K;
    return seq_hop_area_bytes() + max_rot * sizeof(float);
}

int launch_gemv_sequence(const rcp_gemv_step* steps, int n, void* workspace, hipStream_t st)
{
    SeqArgs a;
    memset(&a, 0, sizeof(a));
    a.n = n;
    int lds_x = 0, max_rpl = 0;
    size_t raw_bytes = 0;  // LDS copy of the raw input of the largest rotated entry
    for (int i = 0; i < n; ++i) {
        const rcp_gemv_step& s = steps[i];
        SeqStep& d = a.s[i];
        d.packed = static_cast<const uint4*>(s.packed);
        d.codebook = static_cast<const uint2*>(s.codebook);
        d.x = s.x;
        d.out = s.out;
        d.xq_out = static_cast<uint32_t*>(s.xq_out_or_null);
        d.scale_out = static_cast<uint16_t*>(s.scale_out_or_null);
        d.N = s.N;
        d.K = s.K;
        d.x_dt = s.x_dtype;
        d.out_f16 = s.out_dtype == RCP_F16 ? 1 : 0;
        d.clip_ratio = s.clip_ratio;
        d.rot_n = 0;
        d.rot_m = 0;
        d.Q = nullptr;
        if (s.rot.kind == RCP_ROT_KRON) {
            if (!kron_fits(s.rot.n_wht, s.rot.m))
                return fail(RCP_ERR_UNSUPPORTED, "rcp_quant_w2a4_gemv_sequence: entry %d: Kronecker rotation %d x %d is outside the "
                                                 "sizes the sequence kernel rotates (Hadamard factor 64..1024, m a multiple of 4)", i,
                            s.rot.n_wht, s.rot.m);
            d.rot_n = s.rot.n_wht;
            d.rot_m = s.rot.m;
            d.Q = s.rot.Q;
            if (s.rot.n_wht / 64 > max_rpl) max_rpl = s.rot.n_wht / 64;
            const size_t rb = static_cast<size_t>(s.K) * (s.x_dtype == RCP_F32 ? 4 : 2);
            if (rb > raw_bytes) raw_bytes = rb;
        }
        const int U = s.K / 16;
        d.unr = U > 64 * 4 ? 4 : 2;
        const int xb = gemv_x_bytes(s.K, 1, 64 * d.unr);
        if (xb > lds_x) lds_x = xb;
    }
    a.lds_x_bytes = (lds_x + 15) & ~15;
    a.max_rpl = max_rpl;
    const size_t lds = static_cast<size_t>(a.lds_x_bytes) + 2 * SEQ_WAVES * sizeof(int) +
                       static_cast<size_t>(4) * 64 * max_rpl * sizeof(float) + (max_rpl > 0 ? RCP_MAX_KRON_M * sizeof(float) : 0) +
                       ((raw_bytes + 15) & ~static_cast<size_t>(15));
    if (lds > 80 * 1024) return fail(RCP_ERR_UNSUPPORTED, "rcp_quant_w2a4_gemv_sequence: %zu bytes of LDS needed (limit 80 KiB)", lds);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemv_sequence_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e != hipSuccess) return fail(RCP_ERR_HIP, "rcp_quant_w2a4_gemv_sequence: LDS opt-in failed: %s", hipGetErrorString(e));
    }

    // every workgroup must be resident at once: the grid never exceeds what the occupancy calculation guarantees
    // (the query depends on the device and on the LDS size only; 80 KiB, the most a launch may ask for, covers all)
    static thread_local int cached_dev = -1, cached_max = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return fail(RCP_ERR_HIP, "rcp_quant_w2a4_gemv_sequence: hipGetDevice failed");
    if (dev != cached_dev) {
        int per_cu = 0;
        hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gemv_sequence_kernel, SEQ_THREADS, 80 * 1024);
        if (e != hipSuccess) return fail(RCP_ERR_HIP, "rcp_quant_w2a4_gemv_sequence: occupancy query failed: %s", hipGetErrorString(e));
        cached_max = per_cu * num_compute_units();
        cached_dev = dev;
    }
    const int cus = num_compute_units();
    int want = options().seq_blocks > 0 ? options().seq_blocks : 2 * cus;
    if (want > cached_max) {
        if (options().seq_blocks > 0 || cached_max < cus)
            return fail(RCP_ERR_UNSUPPORTED, "rcp_quant_w2a4_gemv_sequence: %d workgroups cannot be resident at once (limit %d)", want, cached_max);
        want = cached_max;
    }
    a.nwg = want;
    for (int i = 0; i < n; ++i)
        if (a.s[i].rot_m > a.nwg)
            return fail(RCP_ERR_UNSUPPORTED, "rcp_quant_w2a4_gemv_sequence: entry %d: %d rotation columns need as many workgroups (%d)", i,
                        a.s[i].rot_m, a.nwg);
    uint32_t* ws = static_cast<uint32_t*>(workspace);
    float* ybuf = reinterpret_cast<float*>(static_cast<char*>(workspace) + seq_hop_area_bytes());
#ifdef RCP_SEQ_TRACE
    gemv_sequence_kernel<<<a.nwg, SEQ_THREADS, lds, st>>>(a, ws, ybuf, g_seq_trace);
#else
    gemv_sequence_kernel<<<a.nwg, SEQ_THREADS, lds, st>>>(a, ws, ybuf);
#endif
    return check_launch("rcp_quant_w2a4_gemv_sequence");
}

}  // namespace rcp

#ifdef RCP_SEQ_TRACE
extern "C" void rcp_seq_trace_buffer(void* device_buffer) { rcp::g_seq_trace = static_cast<unsigned long long*>(device_buffer); }
#endif
