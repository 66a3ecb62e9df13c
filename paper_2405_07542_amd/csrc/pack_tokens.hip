// "Unpad input tokens" on the device (EMS-SD Appendix D, Alg. 1): the input tokens of all
// samples are concatenated into one sequence and the number of tokens of each sample is
// kept.  The per-sample lists arrive as a padded [B, k_max] array plus the counts; the
// kernel writes the running sum of the counts (cu_seqlens, the form every other call of
// the library takes) and the packed ids, sample after sample, no padding.
//
// One block: block-wide exclusive scan of the counts (wave shuffles + LDS), then one wave
// per sample copies that sample's ids.
#include "ems_device.h"
#include "ems_kernels.h"

namespace ems {

constexpr int kPackThreads = 1024;

__global__ __launch_bounds__(kPackThreads) void pack_tokens_kernel(PackParams p) {
    __shared__ int32_t wave_tot[kPackThreads / kWave];
    __shared__ int32_t carry_s;
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    if (tid == 0) carry_s = 0;
    __syncthreads();
    // exclusive scan, kPackThreads samples a pass; counts are clamped to [0, k_max]
    for (int base = 0; base < p.B; base += kPackThreads) {
        const int i = base + tid;
        const int mine = i < p.B ? min(max(p.token_nums[i], 0), p.k_max) : 0;
        int incl = mine;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const int u = __shfl_up(incl, off);
            if (lane >= off) incl += u;
        }
        if (lane == kWave - 1) wave_tot[wid] = incl;
        __syncthreads();
        int before = carry_s;
        for (int w = 0; w < wid; ++w) before += wave_tot[w];
        if (i < p.B) p.cu[i] = before + incl - mine;
        __syncthreads();
        if (tid == kPackThreads - 1) carry_s = before + incl;
        __syncthreads();
    }
    if (tid == 0) p.cu[p.B] = carry_s;
    __threadfence_block();
    __syncthreads();
    for (int i = wid; i < p.B; i += kPackThreads / kWave) {
        const int k = min(max(p.token_nums[i], 0), p.k_max);
        const int dst = p.cu[i];
        for (int j = lane; j < k; j += kWave) p.packed_ids[dst + j] = p.padded_ids[(int64_t)i * p.k_max + j];
    }
}

hipError_t launch_pack_tokens(const PackParams& p, hipStream_t stream) {
    hipLaunchKernelGGL(pack_tokens_kernel, dim3(1), dim3(kPackThreads), 0, stream, p);
    return hipGetLastError();
}

}  // namespace ems
