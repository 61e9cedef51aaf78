// A read-only streaming probe: what a kernel that does nothing but read reaches on this device.  The
// decode and gather kernels are bound by memory traffic; the benchmark quotes their rate next to this one
// (measured in the same run, on a buffer of the same size) as well as next to the published peak.
#include "common.h"
#include "internal.h"

namespace vlc {
namespace {

// Each block reads one contiguous share of the buffer, 16 bytes per lane and U loads per lane in flight.
template <int U>
__global__ __launch_bounds__(256) void read_stream_kernel(const uint4* __restrict__ src, size_t n16, uint32_t* sink) {
    const size_t per_block = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t b0 = (size_t)blockIdx.x * per_block;
    const size_t b1 = b0 + per_block < n16 ? b0 + per_block : n16;
    uint32_t acc = 0;
    for (size_t i = b0 + threadIdx.x; i < b1; i += 256 * U) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t j = i + (size_t)u * 256;
            v[u] = j < b1 ? src[j] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x12345678u) *sink = acc;        // keeps the loads alive; practically never taken
}

}  // namespace

hipError_t launch_read_stream(const void* buf, size_t bytes, uint32_t* sink, int blocks, hipStream_t st) {
    read_stream_kernel<8><<<blocks, 256, 0, st>>>(reinterpret_cast<const uint4*>(buf), bytes / 16, sink);
    return hipGetLastError();
}

}  // namespace vlc
