// A plain read-only streaming kernel: the HBM read ceiling that the attention kernel's
// bandwidth is set against (besides the published peak).  Every wave reads a contiguous
// share of the buffer with 16-byte non-temporal loads, eight in flight per lane, and folds
// what it read into one word that is stored only if it matches an unlikely pattern (so the
// loads cannot be dropped).
#include "ems_device.h"
#include "ems_kernels.h"

namespace ems {

constexpr int kProbeThreads = 256;
constexpr int kProbeUnroll = 8;

__global__ __launch_bounds__(kProbeThreads) void stream_read_kernel(const u32x4* src, uint64_t lines,
                                                                    uint32_t* sink) {
    const uint64_t waves = (uint64_t)gridDim.x * (kProbeThreads / kWave);
    const uint64_t wave = (uint64_t)blockIdx.x * (kProbeThreads / kWave) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const uint64_t per = (lines + waves - 1) / waves;
    uint64_t line = wave * per;
    const uint64_t end = line + per < lines ? line + per : lines;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; line + kProbeUnroll <= end; line += kProbeUnroll) {
        u32x4 v[kProbeUnroll];
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) v[u] = __builtin_nontemporal_load(src + (line + u) * kWave + lane);
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) acc ^= v[u];
    }
    for (; line < end; ++line) acc ^= __builtin_nontemporal_load(src + line * kWave + lane);
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x5eed1e55u) sink[0] = 1u;
}

hipError_t launch_stream_read(const void* buf, uint64_t bytes, uint32_t* sink, int blocks, hipStream_t stream) {
    const uint64_t lines = bytes / (kWave * sizeof(u32x4));      // whole 1 KiB lines only
    hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(kProbeThreads), 0, stream,
                       static_cast<const u32x4*>(buf), lines, sink);
    return hipGetLastError();
}

}  // namespace ems
