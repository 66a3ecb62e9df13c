// A plain read-only streaming kernel: the HBM read ceiling that the attention kernel's
// bandwidth is set against (besides the published peak).  Every wave reads a contiguous
// share of the buffer with 16-byte non-temporal loads in two alternating batches of four
// 1 KiB lines, the next batch issued before the current one is folded, so that loads are in
// flight at all times (a loop that drains its loads at the end of every iteration measured
// 6.7 TB/s where this one reaches 7.1); what was read is folded into one word that is stored
// only if it matches an unlikely pattern (so the loads cannot be dropped).
#include "ems_device.h"
#include "ems_kernels.h"

namespace ems {

constexpr int kProbeThreads = 256;
constexpr int kProbeBatch = 4;

__global__ __launch_bounds__(kProbeThreads) void stream_read_kernel(const u32x4* src, uint64_t lines,
                                                                    uint32_t* sink) {
    const uint64_t waves = (uint64_t)gridDim.x * (kProbeThreads / kWave);
    const uint64_t wave = (uint64_t)blockIdx.x * (kProbeThreads / kWave) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const uint64_t per = (lines + waves - 1) / waves;
    uint64_t line = wave * per;
    const uint64_t end = line + per < lines ? line + per : lines;
    u32x4 acc = {0u, 0u, 0u, 0u};
    u32x4 a[kProbeBatch], b[kProbeBatch];
    auto issue = [&](u32x4* v, uint64_t at) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kProbeBatch; ++u) v[u] = __builtin_nontemporal_load(src + (at + u) * kWave + lane);
    };
    auto fold = [&](const u32x4* v) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kProbeBatch; ++u) acc ^= v[u];
    };
    if (line + kProbeBatch <= end) {
        issue(a, line);
        line += kProbeBatch;
        // batches a and b alternate; the one just issued stays in flight while the other is folded
        for (; line + 2 * kProbeBatch <= end; line += 2 * kProbeBatch) {
            issue(b, line);
            fold(a);
            issue(a, line + kProbeBatch);
            fold(b);
        }
        fold(a);
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
