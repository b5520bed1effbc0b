// Measurement helper: a plain streaming read of a buffer, the practical ceiling that a
// bandwidth-bound kernel of the same size can be compared with on the machine at hand.
#include "rcp_internal.hpp"

namespace rcp {

constexpr int READ_THREADS = 256;

// Every thread issues its 128-bit loads two at a time and folds them into one word; the
// store never happens for real data patterns but keeps the loads alive.
__global__ __launch_bounds__(READ_THREADS) void stream_read_kernel(const uint4* __restrict__ p, size_t n16,
                                                                   uint32_t* __restrict__ sink)
{
    const size_t tid = static_cast<size_t>(blockIdx.x) * READ_THREADS + threadIdx.x;
    const size_t stride = static_cast<size_t>(gridDim.x) * READ_THREADS;
    uint32_t acc = 0;
    for (size_t i = tid; i < n16; i += 2 * stride) {
        const uint4 a = p[i];
        const size_t j = i + stride;
        const uint4 b = j < n16 ? p[j] : make_uint4(0, 0, 0, 0);
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w;
    }
    if (acc == 0x9e3779b9u && sink != nullptr) sink[0] = acc;
}

int launch_stream_read(const void* p, size_t bytes, uint32_t* sink, hipStream_t st)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return RCP_OK;
    const int cus = num_compute_units();
    size_t blocks = (n16 + 2 * READ_THREADS - 1) / (2 * READ_THREADS);  // two loads per thread
    const size_t cap = static_cast<size_t>(cus) * 16;
    if (blocks > cap) blocks = cap;
    stream_read_kernel<<<static_cast<unsigned>(blocks), READ_THREADS, 0, st>>>(static_cast<const uint4*>(p), n16, sink);
    return check_launch("rcp_stream_read");
}

}  // namespace rcp
