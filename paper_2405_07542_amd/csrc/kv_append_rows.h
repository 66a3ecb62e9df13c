// The copy of one sample's accepted rows for one layer's K or V (EMS-SD Sec. 3.2 "Unpad KV
// cache"), shared by the append kernel and by the kernel that finds the accepted counts and
// appends in one launch.
#pragma once
#include "ems_device.h"
#include "ems_kernels.h"

namespace ems {

// Block (y = 2 * layer + (V ? 1 : 0), z of nz) of sample i, which appends `acc` rows (its first acc
// packed rows, or the acc rows its row list names).  Any block size.
__device__ __forceinline__ void append_sample_rows(const AppendParams& p, int i, int acc, int y, int z, int nz) {
    const bool gather = p.rows != nullptr;
    const int rows0 = gather ? p.rows_cu[i] : 0;
    const int len = p.kv_len[i];
    const int nthreads = (int)blockDim.x;
    // the lengths ride along unless they are updated in place (then a later launch does it,
    // because other blocks still read kv_len[i])
    if (p.kv_len_out != nullptr && y == 0 && z == 0 && threadIdx.x == 0)
        p.kv_len_out[i] = len + acc;
    // never more than the sample brought (accepted[i] <= k_i is the caller's contract)
    const int cu_i = gather ? 0 : p.cu[i];
    const int a = gather ? acc : min(acc, p.cu[i + 1] - cu_i);
    if (a <= 0) return;
    const AppendLayer& ly = p.layer[y >> 1];
    const bool is_v = y & 1;
    const int vph = p.vec_per_head;
    const int row_vecs = p.H * vph;
    const char* src = (is_v ? ly.v_new : ly.k_new) + (int64_t)cu_i * row_vecs * 16;
    char* dst = (is_v ? ly.v_cache : ly.k_cache) + ((int64_t)p.kv_start[i] + len) * ly.row_stride_b;
    if (nz == 1 && nthreads <= 256) {
        // many layers in one launch: plenty of blocks; each thread owns a column of 16-byte
        // pieces and walks down the rows
        for (int v = threadIdx.x; v < row_vecs; v += nthreads) {
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
    // A small launch (one layer, modest B), or a large block: the a x row_vecs 16-byte pieces of
    // this (sample, layer, K|V) are dealt round-robin to the threads of its nz blocks; a thread
    // loads four pieces before it stores them, so that four reads are in flight instead of one.
    const int total = a * row_vecs;
    const int stride = nthreads * nz;
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
    for (int idx0 = z * nthreads + threadIdx.x; idx0 < total; idx0 += 4 * stride) {
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

}  // namespace ems
