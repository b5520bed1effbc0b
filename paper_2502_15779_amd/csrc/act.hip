// Online activation preparation: rotation (Appendix definition of the normalised Hadamard
// matrix; Section 2.1 for the online rotations) and per-token symmetric int4 quantisation
// (Appendix table of quantisation configurations).  All arithmetic is binary32.
//
// The Walsh-Hadamard butterflies run in ascending stride order (1, 2, 4, ...), every
// butterfly output being one IEEE add or subtract of two outputs of the previous stage,
// followed by one multiplication by (float)(1/sqrt(n)).  The result therefore does not
// depend on how the stages are spread over registers, lanes and LDS.
#include <math.h>

#include <mutex>

#include "rcp_internal.hpp"

namespace rcp {

// ---------------------------------------------------------------------------------------
// shared pieces
// ---------------------------------------------------------------------------------------
// Maximum over the workgroup; every thread gets the result.  `red` holds 16 floats.
// `nw` is the number of wavefronts of the workgroup (an argument: the launch dimensions would
// have to be fetched from memory first).
__device__ __forceinline__ float block_max(float v, float* red, int nw)
{
    v = wave_max(v);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float r = red[0];
    for (int w = 1; w < nw; ++w) r = fmaxf(r, red[w]);
    return r;
}

// ---------------------------------------------------------------------------------------
// no rotation (or an fp32 vector that is already rotated): amax, scale, quantise
// One workgroup per token; a thread owns ITERS groups of eight consecutive elements.
// ---------------------------------------------------------------------------------------
template <int DT, int ITERS>
__global__ __launch_bounds__(1024) void quant_kernel(const void* __restrict__ x, int K, float clip_ratio, int threads,
                                                     uint32_t* __restrict__ xq, uint16_t* __restrict__ scale)
{
    __shared__ float red[16];
    const int token = blockIdx.x;
    const int units = K / 8;
    float v[ITERS][8];
    float a = 0.0f;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int u = threadIdx.x + it * threads;
        if (u < units) {
            load8_as_float<DT>(x, static_cast<size_t>(token) * K + static_cast<size_t>(u) * 8, v[it]);
#pragma unroll
            for (int j = 0; j < 8; ++j) a = fmaxf(a, fabsf(v[it][j]));
        }
    }
    a = block_max(a, red, threads >> 6);
    const uint16_t sb = scale_bits_from_amax(a, clip_ratio);
    const float s = half_bits_to_float(sb);
    const float rs = __frcp_rn(s);
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int u = threadIdx.x + it * threads;
        // (16-bit inputs: the form of the quantiser that lands exactly on rounding ties and never needs a division)
        if (u < units)
            xq[static_cast<size_t>(token) * units + u] = DT == RCP_F32 ? quantize8(v[it], s) : quantize8_short(v[it], s, rs);
    }
    if (threadIdx.x == 0) scale[token] = sb;
}

// ---------------------------------------------------------------------------------------
// Walsh-Hadamard rotation of order n = K (a power of two) fused with the quantiser.
// One workgroup of n / EPT threads per token, EPT = 2^LE elements per thread.
// Pass 0 does the strides 1 .. EPT/2 in registers on EPT consecutive elements; every
// later pass gathers, through LDS, the EPT elements whose indices differ in the next LE
// index bits and does those strides in registers.
// ---------------------------------------------------------------------------------------
template <int DT, int LE, bool QUANT>
__global__ __launch_bounds__(1024) void wht_quant_kernel(const void* __restrict__ x, int n, int log2n, float norm,
                                                         float clip_ratio, int waves, uint32_t* __restrict__ xq,
                                                         uint16_t* __restrict__ scale, float* __restrict__ y_out)
{
    constexpr int EPT = 1 << LE;
    extern __shared__ float sy[];  // n floats
    __shared__ float red[16];
    const int token = blockIdx.x;
    const int tid = threadIdx.x;
    // n / EPT threads carry data; the launch rounds up to a whole wave and the surplus
    // threads only take part in barriers and in the maximum (with 0)
    const bool active = tid < n / EPT;
    float v[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) v[e] = 0.0f;
    if (active) {
#pragma unroll
        for (int c = 0; c < EPT / 8; ++c) {
            float t8[8];
            load8_as_float<DT>(x, static_cast<size_t>(token) * n + static_cast<size_t>(tid) * EPT + 8 * c, t8);
#pragma unroll
            for (int j = 0; j < 8; ++j) v[8 * c + j] = t8[j];
        }
        register_stages<LE>(v, 0);
    }
    // the next (up to six) index bits are the lane number: those strides run between lanes, without LDS
    const int nlane = min(6, log2n - LE);
    lane_stages<EPT>(v, tid & 63, nlane);  // threads without data hold zeros and only ever meet each other
    int done = LE + nlane;  // index bits whose stage is finished
    const bool more = done < log2n;  // uniform: strides beyond a wavefront go through LDS
    if (more && active) {
#pragma unroll
        for (int e = 0; e < EPT; ++e) sy[wht_slot(tid * EPT + e)] = v[e];
    }
    while (done < log2n) {
        // the LE register bits sit at index bits [lo, lo + LE); the last pass may overlap
        // bits that are already done and then skips their stages
        const int lo = (done <= log2n - LE) ? done : (log2n - LE);
        const int low = tid & ((1 << lo) - 1), high = tid >> lo;
        const int base = (high << (lo + LE)) | low;
        __syncthreads();
        if (active) {
#pragma unroll
            for (int e = 0; e < EPT; ++e) v[e] = sy[wht_slot(base | (e << lo))];
            register_stages<LE>(v, done - lo);
            // a thread writes back exactly the slots it read, so no barrier is needed here
#pragma unroll
            for (int e = 0; e < EPT; ++e) sy[wht_slot(base | (e << lo))] = v[e];
        }
        done = lo + LE;
    }
    if (more) __syncthreads();

    float a = 0.0f;
    if (active) {
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            v[e] = __fmul_rn(more ? sy[wht_slot(tid * EPT + e)] : v[e], norm);
            a = fmaxf(a, fabsf(v[e]));
        }
    }
    if constexpr (!QUANT) {  // rotation only: y in binary32
        if (active) {
#pragma unroll
            for (int c = 0; c < EPT / 4; ++c)
                reinterpret_cast<float4*>(y_out + static_cast<size_t>(token) * n + static_cast<size_t>(tid) * EPT)[c] =
                    make_float4(v[4 * c], v[4 * c + 1], v[4 * c + 2], v[4 * c + 3]);
        }
        return;
    }
    a = block_max(a, red, waves);
    const uint16_t sb = scale_bits_from_amax(a, clip_ratio);
    const float s = half_bits_to_float(sb);
    if (active) {
#pragma unroll
        for (int c = 0; c < EPT / 8; ++c) {
            float t8[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) t8[j] = v[8 * c + j];
            xq[static_cast<size_t>(token) * (n / 8) + static_cast<size_t>(tid) * (EPT / 8) + c] = quantize8(t8, s);
        }
    }
    if (tid == 0) scale[token] = sb;
}

// ---------------------------------------------------------------------------------------
// Kronecker rotation y = (H_n (x) Q) x, K = n*m: with X the n x m row-major view of x,
// Y = H_n X Q^T.  Workgroup (jblock, token) computes KRON_JB columns of Y: first
// Z[i][jj] = sum_j X[i][j] * Q[j0+jj][j] for all n rows, then the order-n Hadamard
// transform down each column, and writes fp32 y to the workspace.
// ---------------------------------------------------------------------------------------
constexpr int KRON_JB = 4;
constexpr int KRON_THREADS = 256;

template <int DT> struct XStore;
template <> struct XStore<RCP_F32> {
    using type = float;
    __device__ static float widen(float v) { return v; }
};
template <> struct XStore<RCP_F16> {
    using type = uint16_t;
    __device__ static float widen(uint16_t v) { return half_bits_to_float(v); }
};
template <> struct XStore<RCP_BF16> {
    using type = uint16_t;
    __device__ static float widen(uint16_t v) { return bf16_bits_to_float(v); }
};

template <int DT>
__global__ __launch_bounds__(KRON_THREADS) void kron_rotate_kernel(const void* __restrict__ x, int n, int m,
                                                                   const float* __restrict__ Q, float norm,
                                                                   float* __restrict__ y)
{
    extern __shared__ float smem[];
    const int K = n * m;
    using XT = typename XStore<DT>::type;
    float* sQ = smem;                             // KRON_JB * m floats
    float* sZ = sQ + KRON_JB * m;                 // n * KRON_JB floats
    XT* sX = reinterpret_cast<XT*>(sZ + n * KRON_JB);  // K elements in the input's storage type
    const int token = blockIdx.y;
    const int j0 = blockIdx.x * KRON_JB;
    const int jb = min(KRON_JB, m - j0);
    const int tid = threadIdx.x;

    {
        constexpr int PER16 = 16 / static_cast<int>(sizeof(XT));  // elements per 16-byte copy
        const uint4* src = reinterpret_cast<const uint4*>(static_cast<const XT*>(x) + static_cast<size_t>(token) * K);
        uint4* dst = reinterpret_cast<uint4*>(sX);
        for (int u = tid; u < K / PER16; u += KRON_THREADS) dst[u] = src[u];
    }
    for (int i = tid; i < KRON_JB * m; i += KRON_THREADS) {
        const int jj = i / m, j = i % m;
        sQ[i] = (jj < jb) ? Q[static_cast<size_t>(j0 + jj) * m + j] : 0.0f;
    }
    __syncthreads();

    for (int idx = tid; idx < n * KRON_JB; idx += KRON_THREADS) {
        const int i = idx / KRON_JB, jj = idx % KRON_JB;
        const XT* xr = sX + i * m;
        const float* qr = sQ + jj * m;
        float acc = 0.0f;
        for (int j = 0; j < m; ++j) acc = fmaf(XStore<DT>::widen(xr[j]), qr[j], acc);
        sZ[idx] = acc;
    }
    // Hadamard transform over i (stride KRON_JB in sZ), one stage per barrier
    for (int s = 1; s < n; s <<= 1) {
        __syncthreads();
        for (int p = tid; p < (n / 2) * KRON_JB; p += KRON_THREADS) {
            const int pi = p / KRON_JB, jj = p % KRON_JB;
            const int i = ((pi & ~(s - 1)) << 1) | (pi & (s - 1));  // index with bit s clear
            const float a = sZ[i * KRON_JB + jj], b = sZ[(i + s) * KRON_JB + jj];
            sZ[i * KRON_JB + jj] = a + b;
            sZ[(i + s) * KRON_JB + jj] = a - b;
        }
    }
    __syncthreads();
    for (int idx = tid; idx < n * KRON_JB; idx += KRON_THREADS) {
        const int i = idx / KRON_JB, jj = idx % KRON_JB;
        if (jj < jb) y[static_cast<size_t>(token) * K + static_cast<size_t>(i) * m + j0 + jj] = sZ[idx] * norm;
    }
}

// Faster form for n = 64 * RPL (64 .. 1024): one wavefront per column j' of Y.  Lane l owns
// rows i = l*RPL + e of that column: it forms Z[i][j'] = sum_j X[i][j] Q[j'][j] from LDS
// (Q row shared by the wavefront, X rows read four elements at a time), then the Hadamard
// transform over i runs in registers (strides below RPL) and across lanes (the rest), with no
// barrier after the staging one.
template <int DT, int RPL>
__global__ __launch_bounds__(KRON_THREADS) void kron_wave_kernel(const void* __restrict__ x, int n, int m,
                                                                 const float* __restrict__ Q, float norm,
                                                                 float* __restrict__ y)
{
    extern __shared__ float smem[];
    const int K = n * m;
    using XT = typename XStore<DT>::type;
    float* sQ = smem;                                   // 4 rows of Q, m floats each
    XT* sX = reinterpret_cast<XT*>(sQ + 4 * m);         // K elements in the input's storage type (m % 4 == 0)
    const int token = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int jcol = blockIdx.x * 4 + wave;
    {
        constexpr int PER16 = 16 / static_cast<int>(sizeof(XT));
        const uint4* src = reinterpret_cast<const uint4*>(static_cast<const XT*>(x) + static_cast<size_t>(token) * K);
        uint4* dst = reinterpret_cast<uint4*>(sX);
        for (int u = tid; u < K / PER16; u += KRON_THREADS) dst[u] = src[u];
    }
    for (int i = tid; i < 4 * m; i += KRON_THREADS) {
        const int jj = i / m, j = i % m;
        sQ[i] = (blockIdx.x * 4 + jj < m) ? Q[static_cast<size_t>(blockIdx.x * 4 + jj) * m + j] : 0.0f;
    }
    __syncthreads();

    float z[RPL];
    const float4* qr = reinterpret_cast<const float4*>(sQ + wave * m);
#pragma unroll
    for (int e = 0; e < RPL; ++e) {
        const XT* xr = sX + static_cast<size_t>(lane * RPL + e) * m;
        float acc = 0.0f;
#pragma unroll 8
        for (int j4 = 0; j4 < m / 4; ++j4) {
            const float4 q4 = qr[j4];
            float x0, x1, x2, x3;
            if constexpr (sizeof(XT) == 4) {
                const float4 x4 = reinterpret_cast<const float4*>(xr)[j4];
                x0 = x4.x; x1 = x4.y; x2 = x4.z; x3 = x4.w;
            } else {
                const uint2 raw = reinterpret_cast<const uint2*>(xr)[j4];
                x0 = XStore<DT>::widen(static_cast<uint16_t>(raw.x & 0xffffu));
                x1 = XStore<DT>::widen(static_cast<uint16_t>(raw.x >> 16));
                x2 = XStore<DT>::widen(static_cast<uint16_t>(raw.y & 0xffffu));
                x3 = XStore<DT>::widen(static_cast<uint16_t>(raw.y >> 16));
            }
            acc = fmaf(x0, q4.x, acc);
            acc = fmaf(x1, q4.y, acc);
            acc = fmaf(x2, q4.z, acc);
            acc = fmaf(x3, q4.w, acc);
        }
        z[e] = acc;
    }
    // Hadamard transform over the row index i = lane*RPL + e
#pragma unroll
    for (int s = 1; s < RPL; s <<= 1)
#pragma unroll
        for (int e = 0; e < RPL; ++e)
            if ((e & s) == 0) {
                const float a = z[e], b = z[e + s];
                z[e] = a + b;
                z[e + s] = a - b;
            }
#pragma unroll
    for (int s = 1; s < 64; s <<= 1)
#pragma unroll
        for (int e = 0; e < RPL; ++e) {
            const float p = __shfl_xor(z[e], s, 64);
            z[e] = (lane & s) ? (p - z[e]) : (z[e] + p);
        }
    if (jcol < m) {
#pragma unroll
        for (int e = 0; e < RPL; ++e)
            y[static_cast<size_t>(token) * K + static_cast<size_t>(lane * RPL + e) * m + jcol] = z[e] * norm;
    }
}

// Form that spreads the work over the whole chip (n = 64 * RPL): one workgroup per column j' of Y (and
// token), its four wavefronts split the sum over j.  Lane l owns rows l*RPL .. l*RPL + RPL-1: it reads
// its own stretches of X[i][.] straight from memory (the whole token stays in cache; no staging in
// LDS, no barrier before the arithmetic), the row of Q comes through scalar loads.  The four partial
// sums meet in LDS in a fixed order, then the first wavefront runs the order-n Hadamard transform in
// registers (strides below RPL) and across its lanes (lane-swap and DPP exchanges) and stores the column.
constexpr int KRON_SPLIT_MAXQ = 16;  // (rows per lane) x (groups of four columns per wavefront) kept in registers

template <int DT, int RPL>
__global__ __launch_bounds__(KRON_THREADS) void kron_split_kernel(const void* __restrict__ x, int m,
                                                                  const float* __restrict__ Q, float norm,
                                                                  float* __restrict__ y)
{
    __shared__ float part[4][64 * RPL];
    constexpr int QW = KRON_SPLIT_MAXQ / RPL;  // groups of four columns a wavefront can take
    using XT = typename XStore<DT>::type;
    const int token = blockIdx.y, jcol = blockIdx.x;
    // the grid is rounded up to a multiple of eight workgroups, one per die in turn (whole workgroups leave here;
    // step 0.744 -> 0.741 ms)
    if (jcol >= m) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int K = 64 * RPL * m, quads = m / 4;
    const int q0 = wave * quads / 4, q1 = (wave + 1) * quads / 4;  // this wavefront's groups of four columns
    const XT* xr = static_cast<const XT*>(x) + static_cast<size_t>(token) * K + static_cast<size_t>(lane) * RPL * m;
    const float* qrow = Q + static_cast<size_t>(jcol) * m;

    // all loads first, then the arithmetic
    float4 raw[RPL][QW];
#pragma unroll
    for (int t = 0; t < QW; ++t) {
#pragma unroll
        for (int e = 0; e < RPL; ++e) {
            raw[e][t] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (q0 + t < q1) {  // uniform
                if constexpr (sizeof(XT) == 4) {
                    raw[e][t] = reinterpret_cast<const float4*>(xr + static_cast<size_t>(e) * m)[q0 + t];
                } else {
                    const uint2 r = reinterpret_cast<const uint2*>(xr + static_cast<size_t>(e) * m)[q0 + t];
                    raw[e][t].x = __uint_as_float(r.x);
                    raw[e][t].y = __uint_as_float(r.y);
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
            const float4 q4 = reinterpret_cast<const float4*>(qrow)[q0 + t];  // uniform address: scalar load
#pragma unroll
            for (int e = 0; e < RPL; ++e) {
                float x0, x1, x2, x3;
                if constexpr (sizeof(XT) == 4) {
                    x0 = raw[e][t].x; x1 = raw[e][t].y; x2 = raw[e][t].z; x3 = raw[e][t].w;
                } else {
                    const uint32_t a = __float_as_uint(raw[e][t].x), b = __float_as_uint(raw[e][t].y);
                    x0 = XStore<DT>::widen(static_cast<uint16_t>(a & 0xffffu));
                    x1 = XStore<DT>::widen(static_cast<uint16_t>(a >> 16));
                    x2 = XStore<DT>::widen(static_cast<uint16_t>(b & 0xffffu));
                    x3 = XStore<DT>::widen(static_cast<uint16_t>(b >> 16));
                }
                acc[e] = fmaf(x0, q4.x, acc[e]);
                acc[e] = fmaf(x1, q4.y, acc[e]);
                acc[e] = fmaf(x2, q4.z, acc[e]);
                acc[e] = fmaf(x3, q4.w, acc[e]);
            }
        }
    }
#pragma unroll
    for (int e = 0; e < RPL; ++e) part[wave][e * 64 + lane] = acc[e];
    __syncthreads();
    if (wave != 0) return;
    float z[RPL];
#pragma unroll
    for (int e = 0; e < RPL; ++e)
        z[e] = ((part[0][e * 64 + lane] + part[1][e * 64 + lane]) + part[2][e * 64 + lane]) + part[3][e * 64 + lane];
    // Hadamard transform over the row index i = lane*RPL + e, ascending stride: first inside the lane ...
#pragma unroll
    for (int st = 1; st < RPL; st <<= 1)
#pragma unroll
        for (int e = 0; e < RPL; ++e)
            if ((e & st) == 0) {
                const float a = z[e], b = z[e + st];
                z[e] = a + b;
                z[e + st] = a - b;
            }
    // ... then across lanes: z <- z + p in the lane with the stride bit clear, p - z in its partner
#pragma unroll
    for (int e = 0; e < RPL; ++e) {
        float v = z[e];
        const float p1 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false));  // lane ^ 1
        v = (lane & 1) ? p1 - v : v + p1;
        const float p2 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false));  // lane ^ 2
        v = (lane & 2) ? p2 - v : v + p2;
        const float p4 = __shfl_xor(v, 4, 64);
        v = (lane & 4) ? p4 - v : v + p4;
        const float p8 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x128, 0xf, 0xf, false));  // row_ror 8 = lane ^ 8
        v = (lane & 8) ? p8 - v : v + p8;
        // the swaps leave (value of the lane with the bit clear, value of the lane with it set) in every lane
        auto r16 = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        v = (lane & 16) ? __uint_as_float(r16[0]) - __uint_as_float(r16[1]) : __uint_as_float(r16[0]) + __uint_as_float(r16[1]);
        auto r32 = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        v = (lane & 32) ? __uint_as_float(r32[0]) - __uint_as_float(r32[1]) : __uint_as_float(r32[0]) + __uint_as_float(r32[1]);
        y[static_cast<size_t>(token) * K + static_cast<size_t>(lane * RPL + e) * m + jcol] = v * norm;
    }
}

template <int DT, int RPL>
static int launch_kron_split(const void* x, int M, const rcp_rotation* rot, float* y, float norm, hipStream_t st)
{
    dim3 grid((rot->m + 7) / 8 * 8, M);
    kron_split_kernel<DT, RPL><<<grid, KRON_THREADS, 0, st>>>(x, rot->m, rot->Q, norm, y);
    return check_launch("rcp_rotate_quant_act(kron)");
}

// ---------------------------------------------------------------------------------------
// Hadamard rotation across heads: y = (H_n (x) I_m) x, x viewed as n heads of m channels
// (the online rotation of the self-attention output in front of the out-projection; Section 2.1:
// R_2 is split into a per-head factor that is folded into the V projection and this
// across-heads factor).  One workgroup per token: the token is widened into LDS, a thread takes
// whole columns j (the n values x[i*m + j]), transforms them in registers in ascending stride
// order -- the same butterflies as the order-n transform of a contiguous vector -- and the
// quantiser tail is that of the other kernels.
// ---------------------------------------------------------------------------------------
constexpr int HEADS_THREADS = 256;

template <int DT, int NH, bool QUANT>
__global__ __launch_bounds__(HEADS_THREADS) void heads_wht_kernel(const void* __restrict__ x, int m, float norm,
                                                                  float clip_ratio, uint32_t* __restrict__ xq,
                                                                  uint16_t* __restrict__ scale, float* __restrict__ y_out)
{
    extern __shared__ float sy[];  // K floats
    __shared__ float red[16];
    const int token = blockIdx.x;
    const int K = NH * m;
    for (int u = threadIdx.x; u < K / 8; u += HEADS_THREADS) {
        float t8[8];
        load8_as_float<DT>(x, static_cast<size_t>(token) * K + static_cast<size_t>(u) * 8, t8);
        reinterpret_cast<float4*>(sy)[2 * u] = make_float4(t8[0], t8[1], t8[2], t8[3]);
        reinterpret_cast<float4*>(sy)[2 * u + 1] = make_float4(t8[4], t8[5], t8[6], t8[7]);
    }
    __syncthreads();
    for (int j = threadIdx.x; j < m; j += HEADS_THREADS) {
        float v[NH];
#pragma unroll
        for (int i = 0; i < NH; ++i) v[i] = sy[i * m + j];
#pragma unroll
        for (int s = 1; s < NH; s <<= 1)
#pragma unroll
            for (int i = 0; i < NH; ++i)
                if ((i & s) == 0) {
                    const float p = v[i], q = v[i + s];
                    v[i] = p + q;
                    v[i + s] = p - q;
                }
#pragma unroll
        for (int i = 0; i < NH; ++i) sy[i * m + j] = __fmul_rn(v[i], norm);
    }
    __syncthreads();
    if constexpr (!QUANT) {
        for (int u = threadIdx.x; u < K / 4; u += HEADS_THREADS)
            reinterpret_cast<float4*>(y_out + static_cast<size_t>(token) * K)[u] = reinterpret_cast<const float4*>(sy)[u];
        return;
    }
    float a = 0.0f;
    for (int u = threadIdx.x; u < K; u += HEADS_THREADS) a = fmaxf(a, fabsf(sy[u]));
    a = block_max(a, red, HEADS_THREADS / 64);
    const uint16_t sb = scale_bits_from_amax(a, clip_ratio);
    const float sc = half_bits_to_float(sb);
    for (int u = threadIdx.x; u < K / 8; u += HEADS_THREADS) {
        const float4 lo4 = reinterpret_cast<const float4*>(sy)[2 * u], hi4 = reinterpret_cast<const float4*>(sy)[2 * u + 1];
        const float t8[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
        xq[static_cast<size_t>(token) * (K / 8) + u] = quantize8(t8, sc);
    }
    if (threadIdx.x == 0) scale[token] = sb;
}

// x -> binary32 copy (rotation "none" of the rotation-only entry point)
template <int DT>
__global__ __launch_bounds__(256) void widen_kernel(const void* __restrict__ x, size_t groups, float* __restrict__ y)
{
    const size_t g = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
    if (g >= groups) return;
    float v[8];
    load8_as_float<DT>(x, g * 8, v);
    reinterpret_cast<float4*>(y)[2 * g] = make_float4(v[0], v[1], v[2], v[3]);
    reinterpret_cast<float4*>(y)[2 * g + 1] = make_float4(v[4], v[5], v[6], v[7]);
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
size_t act_workspace_bytes(int M, int K, const rcp_rotation* rot)
{
    if (rot != nullptr && rot->kind == RCP_ROT_KRON) return static_cast<size_t>(M) * K * sizeof(float);
    return 0;
}

template <int DT>
static int launch_quant(const void* x, int M, int K, float clip_ratio, void* xq, void* scale, hipStream_t st)
{
    const int units = K / 8;
    int threads = ((units + 63) / 64) * 64;
    if (threads > 1024) threads = 1024;
    const int iters = (units + threads - 1) / threads;
    auto* q = static_cast<uint32_t*>(xq);
    auto* s = static_cast<uint16_t*>(scale);
    if (iters == 1) quant_kernel<DT, 1><<<M, threads, 0, st>>>(x, K, clip_ratio, threads, q, s);
    else if (iters == 2) quant_kernel<DT, 2><<<M, threads, 0, st>>>(x, K, clip_ratio, threads, q, s);
    else if (iters <= 4) quant_kernel<DT, 4><<<M, threads, 0, st>>>(x, K, clip_ratio, threads, q, s);
    else return fail(RCP_ERR_UNSUPPORTED, "rcp_rotate_quant_act: K=%d too large for the quantiser", K);
    return check_launch("rcp_rotate_quant_act(quantise)");
}

template <int DT, bool QUANT>
static int launch_wht(const void* x, int M, int n, float clip_ratio, void* xq, void* scale, float* y, hipStream_t st)
{
    int log2n = 0;
    while ((1 << log2n) < n) ++log2n;
    const float norm = static_cast<float>(1.0 / sqrt(static_cast<double>(n)));
    auto* q = static_cast<uint32_t*>(xq);
    auto* s = static_cast<uint16_t*>(scale);
    const size_t lds = static_cast<size_t>(n) * sizeof(float);
    // 8 elements per thread below 8192 points, 16 from there on (one LDS pass less after the lane stages: 8192 points
    // 5.15 -> 4.87 us; at 4096 and 2048 points 16 per thread are 20-30 % slower)
    if (n < 8192) {
        const int threads = ((n / 8 + 63) / 64) * 64;
        wht_quant_kernel<DT, 3, QUANT><<<M, threads, lds, st>>>(x, n, log2n, norm, clip_ratio, threads / 64, q, s, y);
    } else {
        if (lds + 64 > 65536) {  // 64 KiB of dynamic LDS plus the static reduction slots: above the default limit
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&wht_quant_kernel<DT, 4, QUANT>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
            if (e != hipSuccess) return fail(RCP_ERR_HIP, "rcp_rotate_quant_act: LDS opt-in failed: %s", hipGetErrorString(e));
        }
        const int threads = ((n / 16 + 63) / 64) * 64;
        wht_quant_kernel<DT, 4, QUANT><<<M, threads, lds, st>>>(x, n, log2n, norm, clip_ratio, threads / 64, q, s, y);
    }
    return check_launch("rcp_rotate_quant_act(wht)");
}

template <int DT, int RPL>
static int launch_kron_wave(const void* x, int M, int K, const rcp_rotation* rot, float* y, float norm, hipStream_t st)
{
    const int n = rot->n_wht, m = rot->m;
    const size_t lds = static_cast<size_t>(4) * m * sizeof(float) + static_cast<size_t>(K) * sizeof(typename XStore<DT>::type);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&kron_wave_kernel<DT, RPL>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e != hipSuccess) return fail(RCP_ERR_HIP, "rcp_rotate_quant_act: LDS opt-in failed: %s", hipGetErrorString(e));
    }
    dim3 grid((m + 3) / 4, M);
    kron_wave_kernel<DT, RPL><<<grid, KRON_THREADS, lds, st>>>(x, n, m, rot->Q, norm, y);
    return check_launch("rcp_rotate_quant_act(kron)");
}

template <int DT>
static int launch_kron(const void* x, int M, int K, const rcp_rotation* rot, float* y, hipStream_t st)
{
    const int n = rot->n_wht, m = rot->m;
    const float norm = static_cast<float>(1.0 / sqrt(static_cast<double>(n)));
    const size_t xbytes = static_cast<size_t>(K) * sizeof(typename XStore<DT>::type);
    // one workgroup per output column when a wavefront's share of the columns fits in registers:
    // (n/64) rows per lane x ceil(m/16) groups of four columns <= KRON_SPLIT_MAXQ
    if (m % 4 == 0 && m >= 8 && n >= 64 && n <= 1024 && (n / 64) * ((m / 4 + 3) / 4) <= KRON_SPLIT_MAXQ) {
        switch (n / 64) {
            case 1: return launch_kron_split<DT, 1>(x, M, rot, y, norm, st);
            case 2: return launch_kron_split<DT, 2>(x, M, rot, y, norm, st);
            case 4: return launch_kron_split<DT, 4>(x, M, rot, y, norm, st);
            case 8: return launch_kron_split<DT, 8>(x, M, rot, y, norm, st);
            default: return launch_kron_split<DT, 16>(x, M, rot, y, norm, st);
        }
    }
    if (m % 4 == 0 && n >= 64 && n <= 1024 && xbytes + 16 * m <= 160 * 1024) {
        switch (n / 64) {
            case 1: return launch_kron_wave<DT, 1>(x, M, K, rot, y, norm, st);
            case 2: return launch_kron_wave<DT, 2>(x, M, K, rot, y, norm, st);
            case 4: return launch_kron_wave<DT, 4>(x, M, K, rot, y, norm, st);
            case 8: return launch_kron_wave<DT, 8>(x, M, K, rot, y, norm, st);
            default: return launch_kron_wave<DT, 16>(x, M, K, rot, y, norm, st);
        }
    }
    const size_t lds = (static_cast<size_t>(KRON_JB) * m + static_cast<size_t>(n) * KRON_JB) * sizeof(float) + xbytes;
    if (lds > 160 * 1024) return fail(RCP_ERR_UNSUPPORTED, "rcp_rotate_quant_act: K=%d too large for the Kronecker kernel", K);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&kron_rotate_kernel<DT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e != hipSuccess) return fail(RCP_ERR_HIP, "rcp_rotate_quant_act: LDS opt-in failed: %s", hipGetErrorString(e));
    }
    dim3 grid((m + KRON_JB - 1) / KRON_JB, M);
    kron_rotate_kernel<DT><<<grid, KRON_THREADS, lds, st>>>(x, n, m, rot->Q, norm, y);
    return check_launch("rcp_rotate_quant_act(kron)");
}

template <int DT, bool QUANT>
static int launch_heads(const void* x, int M, int K, const rcp_rotation* rot, float clip_ratio, void* xq, void* scale,
                        float* y, hipStream_t st)
{
    const int n = rot->n_wht, m = rot->m;
    const float norm = static_cast<float>(1.0 / sqrt(static_cast<double>(n)));
    const size_t lds = static_cast<size_t>(K) * sizeof(float);
    auto* q = static_cast<uint32_t*>(xq);
    auto* s = static_cast<uint16_t*>(scale);
#define RCP_HEADS(NH)                                                                                              \
    case NH: {                                                                                                     \
        auto kernel = &heads_wht_kernel<DT, NH, QUANT>;                                                            \
        if (lds + 64 > 65536) {                                                                                    \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),                              \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)); \
            if (e != hipSuccess)                                                                                   \
                return fail(RCP_ERR_HIP, "rcp_rotate_quant_act: LDS opt-in failed: %s", hipGetErrorString(e));     \
        }                                                                                                          \
        kernel<<<M, HEADS_THREADS, lds, st>>>(x, m, norm, clip_ratio, q, s, y);                                    \
        break;                                                                                                     \
    }
    switch (n) {
        RCP_HEADS(2)
        RCP_HEADS(4)
        RCP_HEADS(8)
        RCP_HEADS(16)
        RCP_HEADS(32)
        RCP_HEADS(64)
        default: return fail(RCP_ERR_UNSUPPORTED, "rcp_rotate_quant_act: %d heads not supported (2 .. 64)", n);
    }
#undef RCP_HEADS
    return check_launch("rcp_rotate_quant_act(heads)");
}

template <int DT>
static int launch_act_typed(const void* x, int M, int K, const rcp_rotation* rot, float clip_ratio, void* xq,
                            void* scale, void* ws, hipStream_t st)
{
    const int kind = rot ? rot->kind : RCP_ROT_NONE;
    if (kind == RCP_ROT_NONE) return launch_quant<DT>(x, M, K, clip_ratio, xq, scale, st);
    if (kind == RCP_ROT_WHT) return launch_wht<DT, true>(x, M, K, clip_ratio, xq, scale, nullptr, st);
    if (kind == RCP_ROT_HEADS) return launch_heads<DT, true>(x, M, K, rot, clip_ratio, xq, scale, nullptr, st);
    if (int rc = launch_kron<DT>(x, M, K, rot, static_cast<float*>(ws), st)) return rc;
    return launch_quant<RCP_F32>(ws, M, K, clip_ratio, xq, scale, st);
}

int launch_act(const void* x, rcp_dtype dt, int M, int K, const rcp_rotation* rot, float clip_ratio,
               void* xq, void* scale, void* ws, size_t /*ws_bytes*/, hipStream_t st)
{
    switch (dt) {
        case RCP_F16: return launch_act_typed<RCP_F16>(x, M, K, rot, clip_ratio, xq, scale, ws, st);
        case RCP_F32: return launch_act_typed<RCP_F32>(x, M, K, rot, clip_ratio, xq, scale, ws, st);
        default: return launch_act_typed<RCP_BF16>(x, M, K, rot, clip_ratio, xq, scale, ws, st);
    }
}

// ---------------------------------------------------------------------------------------
// The rotated activations of a Kronecker rotation without a caller's workspace: callers that cannot
// allocate (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc) get the
// M x K binary32 values between the rotation kernel and the quantiser placed in a fixed array in device
// memory.  Every GPU the library runs on holds its own copy of the array until the process ends; the
// array's name is only a host-side handle, so the device address is looked up once per device and that
// pointer is what the kernels receive.  The rotation kernels write all M*K values before the quantiser
// reads them, so nothing has to be cleared between calls; two calls that overlap on one GPU (different
// streams) would share the array and race.
// ---------------------------------------------------------------------------------------
constexpr size_t ACT_SCRATCH_BYTES = RCP_ACT_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[ACT_SCRATCH_BYTES];

static int static_scratch(void** ptr)
{
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static void* addr[MAX_DEVICES] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(RCP_ERR_HIP, "rcp_rotate_quant_act_static: hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(RCP_ERR_UNSUPPORTED, "rcp_rotate_quant_act_static: device %d outside 0..%d", dev, MAX_DEVICES - 1);
    std::lock_guard<std::mutex> lock(mu);
    if (addr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // this device's copy (the current device)
        if (e != hipSuccess || p == nullptr)
            return fail(RCP_ERR_HIP, "rcp_rotate_quant_act_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        addr[dev] = p;
    }
    *ptr = addr[dev];
    return RCP_OK;
}

int launch_act_static(const void* x, rcp_dtype dt, int M, int K, const rcp_rotation* rot, float clip_ratio, void* xq,
                      void* scale, hipStream_t st)
{
    const size_t need = act_workspace_bytes(M, K, rot);
    if (need > ACT_SCRATCH_BYTES)
        return fail(RCP_ERR_WORKSPACE, "rcp_rotate_quant_act_static: M*K*4 = %zu bytes exceed the fixed scratch of %zu bytes; "
                                       "use rcp_rotate_quant_act with a workspace", need, ACT_SCRATCH_BYTES);
    void* ws = nullptr;
    if (int rc = static_scratch(&ws)) return rc;
    return launch_act(x, dt, M, K, rot, clip_ratio, xq, scale, ws, ACT_SCRATCH_BYTES, st);
}

template <int DT>
static int launch_rotate_typed(const void* x, int M, int K, const rcp_rotation* rot, float* y, hipStream_t st)
{
    const int kind = rot ? rot->kind : RCP_ROT_NONE;
    if (kind == RCP_ROT_WHT) return launch_wht<DT, false>(x, M, K, 1.0f, nullptr, nullptr, y, st);
    if (kind == RCP_ROT_KRON) return launch_kron<DT>(x, M, K, rot, y, st);
    if (kind == RCP_ROT_HEADS) return launch_heads<DT, false>(x, M, K, rot, 1.0f, nullptr, nullptr, y, st);
    const size_t groups = static_cast<size_t>(M) * K / 8;
    widen_kernel<DT><<<static_cast<unsigned>((groups + 255) / 256), 256, 0, st>>>(x, groups, y);
    return check_launch("rcp_rotate_act");
}

int launch_rotate(const void* x, rcp_dtype dt, int M, int K, const rcp_rotation* rot, float* y, hipStream_t st)
{
    switch (dt) {
        case RCP_F16: return launch_rotate_typed<RCP_F16>(x, M, K, rot, y, st);
        case RCP_F32: return launch_rotate_typed<RCP_F32>(x, M, K, rot, y, st);
        default: return launch_rotate_typed<RCP_BF16>(x, M, K, rot, y, st);
    }
}

}  // namespace rcp
