// KV-cache append (EMS-SD Sec. 3.2 "Unpad KV cache"): after verification each
// sample's cache grows by exactly its own accepted count; the accepted rows are
// copied from the packed new K/V to the sample's own write location, so no
// padding row is ever written and every cache stays contiguous.
//
// Grid (B, 2 * n_layers, s): s blocks (4 for small launches, else 1) share the accepted
// rows of one sample for one layer's K or V; 16-byte loads and stores, four loads in
// flight per thread.  The per-sample lengths are
// written by the same launch, except when kv_len_out aliases kv_len: then a
// second, tiny launch advances them after every block has read the old ones.
// The same kernel serves the gathered append of tree-structured verification: the rows
// of an accepted root-to-leaf path are not contiguous, so each destination row names
// its packed source row.
#include "kv_append_rows.h"

namespace ems {

constexpr int kAppendThreads = 256;
constexpr int kAppendSplit = 4;        // blocks per (sample, layer, K|V) when the launch would otherwise be small

__global__ __launch_bounds__(kAppendThreads) void kv_append_kernel(AppendParams p) {
    const int i = blockIdx.x;
    const bool gather = p.rows != nullptr;
    const int acc = gather ? p.rows_cu[i + 1] - p.rows_cu[i] : p.accepted[i];
    append_sample_rows(p, i, acc, blockIdx.y, blockIdx.z, gridDim.z);
}

// Padded ("vanilla") ablation, Sec. 3.1: every sample appends the same tau_max rows at the
// aligned row l_pad; rows at or beyond the sample's own accepted count are padding and are
// only marked as such in the key mask -- their K/V is still written, as the vanilla method does.
__global__ __launch_bounds__(kAppendThreads) void padded_kv_append_kernel(PaddedAppendParams p) {
    const int i = blockIdx.x;
    const int acc = p.accepted[i];
    if (blockIdx.y == 0)
        for (int j = threadIdx.x; j < p.tau_max; j += kAppendThreads)
            p.key_mask[(int64_t)i * p.cap + p.l_pad + j] = j < acc ? 1 : 0;
    const AppendLayer& ly = p.layer[blockIdx.y >> 1];
    const bool is_v = blockIdx.y & 1;
    const int vph = p.vec_per_head;
    const int row_vecs = p.H * vph;
    const char* src = (is_v ? ly.v_new : ly.k_new) + (int64_t)i * p.k_max * row_vecs * 16;
    char* dst = (is_v ? ly.v_cache : ly.k_cache) + ((int64_t)i * p.cap + p.l_pad) * ly.row_stride_b;
    for (int v = threadIdx.x; v < row_vecs; v += kAppendThreads) {
        const int h = v / vph;
        const int c = v - h * vph;
        const int64_t doff = (int64_t)h * ly.head_stride_b + c * 16;
        for (int j = 0; j < p.tau_max; ++j) {
            const u32x4 w = *reinterpret_cast<const u32x4*>(src + ((int64_t)j * row_vecs + v) * 16);
            *reinterpret_cast<u32x4*>(dst + j * ly.row_stride_b + doff) = w;
        }
    }
}

__global__ void advance_kv_len_kernel(const int32_t* kv_len, const int32_t* accepted,
                                      const int32_t* rows_cu, int32_t* kv_len_out, int B) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < B) kv_len_out[i] = kv_len[i] + (accepted != nullptr ? accepted[i] : rows_cu[i + 1] - rows_cu[i]);
}

hipError_t launch_kv_append(const AppendParams& p, hipStream_t stream) {
    // a one-layer append of a small batch has too few (sample, layer, K|V) units to fill the chip:
    // split each over several blocks; many layers bring enough blocks by themselves
    const int split = (int64_t)p.B * 2 * p.n_layers < 2048 ? kAppendSplit : 1;
    hipLaunchKernelGGL(kv_append_kernel, dim3(p.B, 2 * p.n_layers, split), dim3(kAppendThreads), 0,
                       stream, p);
    return hipGetLastError();
}

hipError_t launch_padded_kv_append(const PaddedAppendParams& p, hipStream_t stream) {
    hipLaunchKernelGGL(padded_kv_append_kernel, dim3(p.B, 2 * p.n_layers), dim3(kAppendThreads), 0,
                       stream, p);
    return hipGetLastError();
}

hipError_t launch_advance_kv_len(const int32_t* kv_len, const int32_t* accepted, const int32_t* rows_cu,
                                 int32_t* kv_len_out, int B, hipStream_t stream) {
    hipLaunchKernelGGL(advance_kv_len_kernel, dim3((B + 255) / 256), dim3(256), 0, stream, kv_len,
                       accepted, rows_cu, kv_len_out, B);
    return hipGetLastError();
}

}  // namespace ems
