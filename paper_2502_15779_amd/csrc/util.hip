// Measurement helper: a plain streaming read of a buffer, the practical ceiling that a
// bandwidth-bound kernel of the same size can be compared with on the machine at hand.
#include "rcp_internal.hpp"

namespace rcp {

constexpr int READ_THREADS = 256;

// One 128-bit load per thread and iteration with the non-temporal hint, up to 64 workgroups per compute unit: the
// fastest of the plain read kernels tried on this machine (two or four loads per thread in flight, with and without the
// hint, 4 to 64 workgroups per unit: 4.8 - 5.6 us on 22 MiB and 22.0 - 25.8 us on 128 MiB, this form the fastest on
// both).  The store never happens for real data patterns but keeps the loads alive.
__global__ __launch_bounds__(READ_THREADS) void stream_read_kernel(const uint4* __restrict__ p, size_t n16,
                                                                   uint32_t* __restrict__ sink)
{
    const size_t tid = static_cast<size_t>(blockIdx.x) * READ_THREADS + threadIdx.x;
    const size_t stride = static_cast<size_t>(gridDim.x) * READ_THREADS;
    uint32_t acc = 0;
    for (size_t i = tid; i < n16; i += stride) {
        const u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p) + i);
        acc ^= a[0] ^ a[1] ^ a[2] ^ a[3];
    }
    if (acc == 0x9e3779b9u && sink != nullptr) sink[0] = acc;
}

int launch_stream_read(const void* p, size_t bytes, uint32_t* sink, hipStream_t st)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return RCP_OK;
    const int cus = num_compute_units();
    size_t blocks = (n16 + READ_THREADS - 1) / READ_THREADS;
    const size_t cap = static_cast<size_t>(cus) * 64;
    if (blocks > cap) blocks = cap;
    stream_read_kernel<<<static_cast<unsigned>(blocks), READ_THREADS, 0, st>>>(static_cast<const uint4*>(p), n16, sink);
    return check_launch("rcp_stream_read");
}

}  // namespace rcp
