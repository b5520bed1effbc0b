// Online activation preparation: rotation (Appendix definition of the normalised Hadamard
// matrix; Section 2.1 for the online rotations) and per-token symmetric int4 quantisation
// (Appendix table of quantisation configurations).  All arithmetic is binary32.
//
// The Walsh-Hadamard butterflies run in ascending stride order (1, 2, 4, ...), every
// butterfly output being one IEEE add or subtract of two outputs of the previous stage,
// followed by one multiplication by (float)(1/sqrt(n)).  The result therefore does not
// depend on how the stages are spread over registers, lanes and LDS.
#include <math.h>

#include "rcp_internal.hpp"

namespace rcp {

// ---------------------------------------------------------------------------------------
// shared pieces
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v = fmaxf(v, __shfl_xor(v, d, 64));
    return v;
}

// Maximum over the workgroup; every thread gets the result.  `red` holds 16 floats.
__device__ __forceinline__ float block_max(float v, float* red)
{
    v = wave_max(v);
    const int wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
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
__global__ __launch_bounds__(1024) void quant_kernel(const void* __restrict__ x, int K, float clip_ratio,
                                                     uint32_t* __restrict__ xq, uint16_t* __restrict__ scale)
{
    __shared__ float red[16];
    const int token = blockIdx.x;
    const int units = K / 8;
    float v[ITERS][8];
    float a = 0.0f;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int u = threadIdx.x + it * blockDim.x;
        if (u < units) {
            load8_as_float<DT>(x, static_cast<size_t>(token) * K + static_cast<size_t>(u) * 8, v[it]);
#pragma unroll
            for (int j = 0; j < 8; ++j) a = fmaxf(a, fabsf(v[it][j]));
        }
    }
    a = block_max(a, red);
    const uint16_t sb = scale_bits_from_amax(a, clip_ratio);
    const float s = half_bits_to_float(sb);
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int u = threadIdx.x + it * blockDim.x;
        if (u < units) xq[static_cast<size_t>(token) * units + u] = quantize8(v[it], s);
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
template <int LE>
__device__ __forceinline__ void register_stages(float (&v)[1 << LE], int first_bit)
{
#pragma unroll
    for (int b = 0; b < LE; ++b) {
        if (b < first_bit) continue;
        const int s = 1 << b;
#pragma unroll
        for (int i = 0; i < (1 << LE); ++i)
            if ((i & s) == 0) {
                const float p = v[i], q = v[i + s];
                v[i] = p + q;
                v[i + s] = p - q;
            }
    }
}

template <int DT, int LE>
__global__ __launch_bounds__(1024) void wht_quant_kernel(const void* __restrict__ x, int n, int log2n, float norm,
                                                         float clip_ratio, uint32_t* __restrict__ xq,
                                                         uint16_t* __restrict__ scale)
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
#pragma unroll
        for (int e = 0; e < EPT; ++e) sy[tid * EPT + e] = v[e];
    }

    int done = LE;  // index bits whose stage is finished
    while (done < log2n) {
        // the LE register bits sit at index bits [lo, lo + LE); the last pass may overlap
        // bits that are already done and then skips their stages
        const int lo = (done <= log2n - LE) ? done : (log2n - LE);
        const int low = tid & ((1 << lo) - 1), high = tid >> lo;
        const int base = (high << (lo + LE)) | low;
        __syncthreads();
        if (active) {
#pragma unroll
            for (int e = 0; e < EPT; ++e) v[e] = sy[base | (e << lo)];
            register_stages<LE>(v, done - lo);
            // a thread writes back exactly the slots it read, so no barrier is needed here
#pragma unroll
            for (int e = 0; e < EPT; ++e) sy[base | (e << lo)] = v[e];
        }
        done = lo + LE;
    }
    __syncthreads();

    float a = 0.0f;
    if (active) {
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            v[e] = __fmul_rn(sy[tid * EPT + e], norm);
            a = fmaxf(a, fabsf(v[e]));
        }
    }
    a = block_max(a, red);
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
    if (iters == 1) quant_kernel<DT, 1><<<M, threads, 0, st>>>(x, K, clip_ratio, q, s);
    else if (iters == 2) quant_kernel<DT, 2><<<M, threads, 0, st>>>(x, K, clip_ratio, q, s);
    else if (iters <= 4) quant_kernel<DT, 4><<<M, threads, 0, st>>>(x, K, clip_ratio, q, s);
    else return fail(RCP_ERR_UNSUPPORTED, "rcp_rotate_quant_act: K=%d too large for the quantiser", K);
    return check_launch("rcp_rotate_quant_act(quantise)");
}

template <int DT>
static int launch_wht(const void* x, int M, int n, float clip_ratio, void* xq, void* scale, hipStream_t st)
{
    int log2n = 0;
    while ((1 << log2n) < n) ++log2n;
    const float norm = static_cast<float>(1.0 / sqrt(static_cast<double>(n)));
    auto* q = static_cast<uint32_t*>(xq);
    auto* s = static_cast<uint16_t*>(scale);
    const size_t lds = static_cast<size_t>(n) * sizeof(float);
    if (n <= 8192) {
        const int threads = ((n / 8 + 63) / 64) * 64;
        wht_quant_kernel<DT, 3><<<M, threads, lds, st>>>(x, n, log2n, norm, clip_ratio, q, s);
    } else {
        // 64 KiB of dynamic LDS plus the static reduction slots: above the default limit
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&wht_quant_kernel<DT, 4>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e != hipSuccess) return fail(RCP_ERR_HIP, "rcp_rotate_quant_act: LDS opt-in failed: %s", hipGetErrorString(e));
        wht_quant_kernel<DT, 4><<<M, n / 16, lds, st>>>(x, n, log2n, norm, clip_ratio, q, s);
    }
    return check_launch("rcp_rotate_quant_act(wht)");
}

template <int DT>
static int launch_kron(const void* x, int M, int K, const rcp_rotation* rot, float* y, hipStream_t st)
{
    const int n = rot->n_wht, m = rot->m;
    const size_t lds = (static_cast<size_t>(KRON_JB) * m + static_cast<size_t>(n) * KRON_JB) * sizeof(float) +
                       static_cast<size_t>(K) * sizeof(typename XStore<DT>::type);
    if (lds > 160 * 1024) return fail(RCP_ERR_UNSUPPORTED, "rcp_rotate_quant_act: K=%d too large for the Kronecker kernel", K);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&kron_rotate_kernel<DT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e != hipSuccess) return fail(RCP_ERR_HIP, "rcp_rotate_quant_act: LDS opt-in failed: %s", hipGetErrorString(e));
    }
    const float norm = static_cast<float>(1.0 / sqrt(static_cast<double>(n)));
    dim3 grid((m + KRON_JB - 1) / KRON_JB, M);
    kron_rotate_kernel<DT><<<grid, KRON_THREADS, lds, st>>>(x, n, m, rot->Q, norm, y);
    return check_launch("rcp_rotate_quant_act(kron)");
}

template <int DT>
static int launch_act_typed(const void* x, int M, int K, const rcp_rotation* rot, float clip_ratio, void* xq,
                            void* scale, void* ws, hipStream_t st)
{
    const int kind = rot ? rot->kind : RCP_ROT_NONE;
    if (kind == RCP_ROT_NONE) return launch_quant<DT>(x, M, K, clip_ratio, xq, scale, st);
    if (kind == RCP_ROT_WHT) return launch_wht<DT>(x, M, K, clip_ratio, xq, scale, st);
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

}  // namespace rcp
