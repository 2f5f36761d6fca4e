// Measurement hook: a plain streaming read of device memory, the ceiling that the bandwidth-bound expert
// kernels are compared with (same 128-bit streamed loads, no arithmetic but an XOR).
#include "common.hpp"
#include "kernels.hpp"

namespace moemix {

// Every wavefront owns a contiguous span and reads it 8 KB at a time (eight 128-bit loads per lane in flight).
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4_t* __restrict__ src, size_t n16,
                                                           uint32_t* __restrict__ sink) {
    constexpr int UNR = 8;
    const int lane = threadIdx.x & 63;
    const size_t n_waves = (size_t)gridDim.x * 4, gw = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const size_t per = n16 / n_waves / (64 * UNR) * (64 * UNR);      // 16-byte pieces per wavefront
    const uint4_t* p = src + gw * per;
    uint4_t acc = {0u, 0u, 0u, 0u};
    for (size_t i = 0; i + 64 * UNR <= per; i += 64 * UNR) {
        uint4_t v[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) v[u] = __builtin_nontemporal_load(p + i + u * 64 + lane);
#pragma unroll
        for (int u = 0; u < UNR; ++u) acc ^= v[u];
    }
    // the pieces left over by the division into equal spans
    for (size_t i = n_waves * per + gw * 64 + lane; i < n16; i += n_waves * 64) acc ^= __builtin_nontemporal_load(src + i);
    const uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    if (x == 0x9E3779B9u) *sink = x;     // keeps the loads alive; practically never taken
}

void launch_stream_read(const void* src, size_t bytes, uint32_t* sink, int blocks, hipStream_t st) {
    TraceScope trace(kKernelStreamRead, st);
    stream_read_kernel<<<blocks, 256, 0, st>>>((const uint4_t*)src, bytes / 16, sink);
}

}  // namespace moemix
