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
#include "ems_device.h"
#include "ems_kernels.h"

namespace ems {

constexpr int kAppendThreads = 256;
constexpr int kAppendSplit = 4;        // blocks per (sample, layer, K|V) when the launch would otherwise be small

__global__ __launch_bounds__(kAppendThreads) void kv_append_kernel(AppendParams p) {
    const int i = blockIdx.x;
    const bool gather = p.rows != nullptr;
    const int rows0 = gather ? p.rows_cu[i] : 0;
    const int acc = gather ? p.rows_cu[i + 1] - rows0 : p.accepted[i];
    const int len = p.kv_len[i];
    // the lengths ride along unless they are updated in place (then a later launch does it,
    // because other blocks still read kv_len[i])
    if (p.kv_len_out != nullptr && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0)
        p.kv_len_out[i] = len + acc;
    // never more than the sample brought (accepted[i] <= k_i is the caller's contract)
    const int cu_i = gather ? 0 : p.cu[i];
    const int a = gather ? acc : min(acc, p.cu[i + 1] - cu_i);
    if (a <= 0) return;
    const AppendLayer& ly = p.layer[blockIdx.y >> 1];
    const bool is_v = blockIdx.y & 1;
    const int vph = p.vec_per_head;
    const int row_vecs = p.H * vph;
    const char* src = (is_v ? ly.v_new : ly.k_new) + (int64_t)cu_i * row_vecs * 16;
    char* dst = (is_v ? ly.v_cache : ly.k_cache) + ((int64_t)p.kv_start[i] + len) * ly.row_stride_b;
    if (gridDim.z == 1) {
        // many layers in one launch: plenty of blocks; each thread owns a column of 16-byte
        // pieces and walks down the rows
        for (int v = threadIdx.x; v < row_vecs; v += kAppendThreads) {
            const int h = v / vph;
            const int c = v - h * vph;
            const int64_t doff = (int64_t)h * ly.head_stride_b + c * 16;
            for (int j = 0; j < a; ++j) {
                // gathered append (an accepted tree path): the j-th row of the path, wherever it sits
                const int r = gather ? p.rows[rows0 + j] : j;
                if (gather && (unsigned)r >= (unsigned)p.T) continue;      // not a packed row: nothing to copy
                const u32x4 w = *reinterpret_cast<const u32x4*>(src + ((int64_t)r * row_vecs + v) * 16);
                *reinterpret_cast<u32x4*>(dst + j * ly.row_stride_b + doff) = w;
            }
        }
        return;
    }
    // A small launch (one layer, modest B): the a x row_vecs 16-byte pieces of this (sample,
    // layer, K|V) are dealt round-robin to the threads of its gridDim.z blocks; a thread loads
    // four pieces before it stores them, so that four reads are in flight instead of one.
    const int total = a * row_vecs;
    const int stride = kAppendThreads * (int)gridDim.z;
    auto locate = [&](int idx, const char*& s_ptr, char*& d_ptr) -> bool {
        const int j = idx / row_vecs;
        const int v = idx - j * row_vecs;
        const int h = v / vph;
        const int c = v - h * vph;
        const int r = gather ? p.rows[rows0 + j] : j;
        s_ptr = src + ((int64_t)r * row_vecs + v) * 16;
        d_ptr = dst + (int64_t)j * ly.row_stride_b + (int64_t)h * ly.head_stride_b + c * 16;
        return !gather || (unsigned)r < (unsigned)p.T;
    };
    for (int idx0 = blockIdx.z * kAppendThreads + threadIdx.x; idx0 < total; idx0 += 4 * stride) {
        u32x4 w[4];
        char* d[4];
        bool ok[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = idx0 + u * stride;
            const char* sp = nullptr;
            d[u] = nullptr;
            ok[u] = idx < total && locate(idx, sp, d[u]);
            if (ok[u]) w[u] = *reinterpret_cast<const u32x4*>(sp);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (ok[u]) *reinterpret_cast<u32x4*>(d[u]) = w[u];
    }
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
