// Greedy acceptance (EMS-SD Appendix A): greedy target token = arg-max of the
// target distribution for each packed row; acceptance length of a sample = 1 +
// the number of leading drafts equal to the target token of the row before
// them; then the running sum of the lengths and the packed accepted tokens.
//
// Two launches on the caller's stream:
//   1. argmax_partial_kernel  grid (slices, T): each block scans one slice of one
//      logits row with 16-byte loads and keeps (value, lowest index);
//   2. accept_scan_kernel     one block: finishes the arg-max per row, 16 lanes per
//      sample compare drafts with targets (ballot + count of leading matches),
//      block-wide exclusive scan of the lengths, packed copy of accepted tokens.
// Comparisons are on exactly widened values, so results are bit-exact; ties go
// to the lowest index at every merge level.
// With a parent array (token trees) step 2 walks from each sample's row 0 to the child
// that carries the target's token instead of counting leading matches, and also
// reports which packed rows form the accepted path.
// accept_append_kernel is step 2 and the append of the accepted rows (Sec. 3.2 "Unpad KV cache")
// in one launch: one workgroup is the scan block above, the others each find their own sample's
// accepted count from the same partials and copy that many rows, so that no workgroup waits for
// another.  The step around the attention call is bound by launches, not by bytes.
#include "ems_device.h"
#include "ems_kernels.h"
#include "kv_append_rows.h"

namespace ems {

__device__ __forceinline__ void take_better(float& v, int32_t& idx, float ov, int32_t oi) {
    if (ov > v || (ov == v && oi < idx)) {
        v = ov;
        idx = oi;
    }
}

struct F32 {};   // logits may also be fp32 (K/V never are)

// Elements of a 16-byte vector and how to read element e of it / element c of a row.
template <typename ET> struct Logit {
    static constexpr int per_vec = 8;
    typedef uint16_t elem_t;
    static __device__ __forceinline__ float of_vec(const u32x4 w, int e) {
        return widen(ET{}, (uint16_t)(w[e >> 1] >> ((e & 1) * 16)));
    }
    static __device__ __forceinline__ float of_elem(uint16_t bits) { return widen(ET{}, bits); }
};
template <> struct Logit<F32> {
    static constexpr int per_vec = 4;
    typedef float elem_t;
    static __device__ __forceinline__ float of_vec(const u32x4 w, int e) { return __uint_as_float(w[e]); }
    static __device__ __forceinline__ float of_elem(float x) { return x; }
};

template <typename ET>
__global__ __launch_bounds__(kArgmaxThreads) void argmax_partial_kernel(AcceptParams p) {
    typedef Logit<ET> LT;
    constexpr int PV = LT::per_vec;
    const int row = blockIdx.y, sl = blockIdx.x;
    const int tid = threadIdx.x;
    const int c0 = sl * p.slice_len;
    const int c1 = min(p.V, c0 + p.slice_len);
    const typename LT::elem_t* base = reinterpret_cast<const typename LT::elem_t*>(p.logits) + (int64_t)row * p.V;
    // -inf / "no index yet": a row slice that holds nothing above -inf resolves to its first
    // column below (all its elements are then equal), without a dependent load up front
    float best = -INFINITY;
    int32_t arg = 0x7fffffff;
    if ((p.V % PV) == 0) {
        // 16-byte non-temporal loads (the logits are read once)
        const uint64_t rowaddr = (uint64_t)base;
        auto scan8 = [&](const u32x4 w, int v) {
#pragma unroll
            for (int e = 0; e < PV; ++e) {
                const float y = LT::of_vec(w, e);
                if (y > best) {            // strict: the earlier index of this thread stays
                    best = y;
                    arg = v * PV + e;
                }
            }
        };
        const int v1 = c1 / PV;            // (slices are multiples of 8 columns; V is a multiple of PV here)
        // four loads in flight per thread; a thread whose last group is short re-reads the
        // slice's last vector instead (scanning an element twice changes nothing)
        for (int v = c0 / PV + tid; v < v1; v += 4 * kArgmaxThreads) {
            int vv[4];
            u32x4 w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                vv[u] = min(v + u * kArgmaxThreads, v1 - 1);
                w[u] = gload_stream<u32x4>(rowaddr, (uint32_t)vv[u] * 16u);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) scan8(w[u], vv[u]);
        }
    } else {
        for (int c = c0 + tid; c < c1; c += kArgmaxThreads) {
            const float y = LT::of_elem(base[c]);
            if (y > best) {
                best = y;
                arg = c;
            }
        }
    }
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1)
        take_better(best, arg, __shfl_xor(best, off), __shfl_xor(arg, off));
    __shared__ float sv[kArgmaxThreads / kWave];
    __shared__ int32_t si[kArgmaxThreads / kWave];
    if ((tid & 63) == 0) {
        sv[tid >> 6] = best;
        si[tid >> 6] = arg;
    }
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int w = 1; w < kArgmaxThreads / kWave; ++w) take_better(best, arg, sv[w], si[w]);
        if (best == -INFINITY) arg = c0;       // nothing above -inf in this slice: all equal, first wins
        ArgmaxPartial out;
        out.value = best;
        out.index = arg;
        p.partial[(int64_t)row * p.slices + sl] = out;
    }
}


// Acceptance along a token tree, one wave per sample (k <= 64 rows, lane j = row j): from row
// 0, step to the lowest-indexed child of the current row whose token equals the target's
// token after that row; stop when no child matches.  `emit(step, row)` is called once per
// accepted row, in path order.  Children have larger indices than their parents, so the
// walk moves strictly upward and ends after at most k steps whatever parent[] holds.
template <typename Emit>
__device__ __forceinline__ int tree_walk(const AcceptParams& p, int base, int k, int lane, Emit emit) {
    if (k <= 0) return 0;
    const bool in = lane < k;
    const int pj = in ? p.parent[base + lane] : -2;
    const int idj = in ? p.input_ids[base + lane] : 0;
    const int xj = in ? p.target_ids[base + lane] : 0;
    int u = 0, a = 0;
    for (;;) {
        emit(a, u);
        ++a;
        const int xu = __shfl(xj, u);
        const uint64_t m = __builtin_amdgcn_ballot_w64(in && lane > u && pj == u && idj == xu);
        if (m == 0 || a >= k) break;
        u = __builtin_ctzll(m);
    }
    return a;
}

// LDS of the scan block: the accepted counts of all samples, and -- when they fit (rows_in_lds) --
// cu_seqlens and the target and input ids of all rows, so that after the first pass over the
// partials nothing is read from global memory twice or in a dependent chain.
constexpr int kMaxSlices = 16;

__device__ __forceinline__ void accept_scan_block(const AcceptParams& p, int32_t* accept_lds) {
    __shared__ int32_t wave_tot[kAcceptThreads / kWave];
    int32_t* const acc_s = accept_lds;                         // [B]
    int32_t* const cu_s = acc_s + p.B;                         // [B + 1]   (rows_in_lds)
    int32_t* const tgt_s = cu_s + p.B + 1;                     // [T]       (rows_in_lds)
    int32_t* const ids_s = tgt_s + p.T;                        // [T]       (rows_in_lds)
    const bool in_lds = p.rows_in_lds != 0;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wid = tid >> 6;

    if (in_lds)
        for (int i = tid; i <= p.B; i += kAcceptThreads) cu_s[i] = p.cu[i];
    for (int r = tid; r < p.T; r += kAcceptThreads) {
        int32_t arg;
        if (p.logits != nullptr) {
            // all slices of the row are asked for at once (a loop over a run-time count would
            // wait for each load before asking for the next)
            const ArgmaxPartial* part = p.partial + (int64_t)r * p.slices;
            ArgmaxPartial got[kMaxSlices];
#pragma unroll
            for (int s = 0; s < kMaxSlices; ++s)
                if (s < p.slices) got[s] = part[s];
            float best = got[0].value;
            arg = got[0].index;
#pragma unroll
            for (int s = 1; s < kMaxSlices; ++s)
                if (s < p.slices) take_better(best, arg, got[s].value, got[s].index);
            p.target_ids[r] = arg;
        } else {
            arg = p.target_ids[r];
        }
        if (in_lds) {
            tgt_s[r] = arg;
            ids_s[r] = p.input_ids[r];
        }
    }
    if (p.logits != nullptr) __threadfence_block();      // (the tree walk and the fallback read target_ids back from memory)
    __syncthreads();
    auto cu_at = [&](int i) { return in_lds ? cu_s[i] : p.cu[i]; };
    auto tgt_at = [&](int r) { return in_lds ? tgt_s[r] : p.target_ids[r]; };
    auto ids_at = [&](int r) { return in_lds ? ids_s[r] : p.input_ids[r]; };

    const bool tree = p.parent != nullptr;
    if (tree) {
        // token trees: one wave per sample walks from the root
        for (int i = wid; i < p.B; i += kAcceptThreads / kWave) {
            const int base = p.cu[i];
            const int k = p.cu[i + 1] - base;
            const int a = tree_walk(p, base, min(k, kWave), lane, [](int, int) {});
            if (lane == 0) {
                acc_s[i] = a;
                p.accepted[i] = a;
            }
        }
    } else {
        // 16 lanes per sample (64 samples per pass of the block): count the leading drafts that
        // match the target's tokens, 16 rows at a time.  The loop is wave-uniform; a group that
        // has found its first mismatch idles until the other three groups of its wave have too.
        const int sub = lane >> 4, l16 = lane & 15;
        for (int i0 = 0; i0 < p.B; i0 += kAcceptThreads / 16) {
            const int i = i0 + (tid >> 4);
            const bool live = i < p.B;
            const int base = live ? cu_at(i) : 0;
            const int k = live ? cu_at(i + 1) - base : 0;
            int m = 0;
            bool done = k <= 1;
            for (int c0 = 0;; c0 += 16) {
                const int j = c0 + l16;
                const bool match = !done && j < k - 1 && tgt_at(base + j) == ids_at(base + j + 1);
                const uint32_t mine = (uint32_t)(__builtin_amdgcn_ballot_w64(match) >> (16 * sub)) & 0xffffu;
                if (!done) {
                    const uint32_t miss = ~mine & 0xffffu;      // a row past the last draft counts as a miss
                    if (miss != 0) {
                        m += __builtin_ctz(miss);
                        done = true;
                    } else {
                        m += 16;
                    }
                }
                if (__builtin_amdgcn_ballot_w64(!done) == 0) break;
            }
            if (live && l16 == 0) {
                const int a = k > 0 ? m + 1 : 0;
                acc_s[i] = a;
                p.accepted[i] = a;
            }
        }
    }
    __syncthreads();

    // exclusive scan of accepted[] over the block: each thread owns a run of samples
    const int chunk = (p.B + kAcceptThreads - 1) / kAcceptThreads;
    const int first = tid * chunk;
    int mine = 0;
    for (int c = 0; c < chunk; ++c)
        if (first + c < p.B) mine += acc_s[first + c];
    int incl = mine;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int u = __shfl_up(incl, off);
        if (lane >= off) incl += u;
    }
    if (lane == kWave - 1) wave_tot[wid] = incl;
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wid; ++w) before += wave_tot[w];
    int run = before + incl - mine;            // exclusive prefix of this thread's first sample
    for (int c = 0; c < chunk; ++c) {
        const int i = first + c;
        if (i >= p.B) break;
        const int a = acc_s[i];
        p.accepted_cu[i] = run;
        if (tree) {
            acc_s[i] = run;                     // the walk below needs the sample's offset
        } else if (p.out_tokens != nullptr) {
            const int base = cu_at(i);
            for (int j = 0; j < a; ++j) p.out_tokens[run + j] = tgt_at(base + j);
        }
        run += a;
        if (i == p.B - 1) p.accepted_cu[p.B] = run;
    }
    if (!tree || (p.out_tokens == nullptr && p.accepted_rows == nullptr)) return;
    __syncthreads();
    // token trees: the accepted rows are not a prefix of the sample's rows; walk again, now
    // that every sample knows where its share of the packed outputs begins
    for (int i = wid; i < p.B; i += kAcceptThreads / kWave) {
        const int base = p.cu[i];
        const int k = p.cu[i + 1] - base;
        const int off = acc_s[i];
        tree_walk(p, base, min(k, kWave), lane, [&](int step, int row) {
            if (lane == 0) {
                if (p.out_tokens != nullptr) p.out_tokens[off + step] = p.target_ids[base + row];
                if (p.accepted_rows != nullptr) p.accepted_rows[off + step] = base + row;
            }
        });
    }
}

__global__ __launch_bounds__(kAcceptThreads) void accept_scan_kernel(AcceptParams p) {
    extern __shared__ int32_t accept_lds[];
    accept_scan_block(p, accept_lds);
}

// The accepted count of sample i, found by a whole block of kAcceptThreads threads from the same
// inputs and by the same rule as accept_scan_block, so that both give the same number: 64 rows a
// pass, 16 threads per row finish its arg-max over the slices (or one reads target_ids), the
// first wave counts the leading matches.
__device__ __forceinline__ int block_acceptance(const AcceptParams& p, int i) {
    __shared__ int32_t match_s[kWave];
    __shared__ int32_t lead_s;
    const int tid = threadIdx.x;
    const int base = p.cu[i];
    const int k = p.cu[i + 1] - base;
    if (k <= 0) return 0;
    int m = 0;
    for (int c0 = 0; c0 < k - 1; c0 += kWave) {          // rows c0 .. c0 + 63 against the drafts after them
        const int j = c0 + (tid >> 4);
        const int s = tid & 15;
        int32_t arg = 0x7fffffff;
        if (j < k - 1) {
            if (p.logits != nullptr) {
                float best = -INFINITY;
                if (s < p.slices) {
                    const ArgmaxPartial got = p.partial[(int64_t)(base + j) * p.slices + s];
                    best = got.value;
                    arg = got.index;
                }
                // (a slice that does not exist holds (-inf, max index): it never wins, since every real
                // slice reports an index below V even when all its values are -inf)
#pragma unroll
                for (int off = 8; off >= 1; off >>= 1) {
                    const float ov = __shfl_xor(best, off);
                    const int32_t oi = __shfl_xor(arg, off);
                    take_better(best, arg, ov, oi);
                }
            } else {
                arg = p.target_ids[base + j];
            }
        }
        if (s == 0) match_s[tid >> 4] = (j < k - 1 && arg == p.input_ids[base + j + 1]) ? 1 : 0;
        __syncthreads();
        if (tid < kWave) {
            const uint64_t miss = ~__builtin_amdgcn_ballot_w64(match_s[tid] != 0);   // (a row past the last draft is a miss)
            if (tid == 0) lead_s = miss != 0 ? __builtin_ctzll(miss) : kWave;
        }
        __syncthreads();
        const int lead = lead_s;
        m += lead;
        if (lead < kWave) break;                          // (block-uniform)
    }
    return m + 1;
}

// Acceptance and append in one launch (Appendix A, then Sec. 3.2 "Unpad KV cache"): block
// (B, 0, 0) is the scan block of accept_scan_kernel and writes every output of the acceptance;
// block (i, y, 0) with i < B finds sample i's accepted count by itself (it cannot wait for the
// scan block) and appends that many rows of layer y / 2's K or V.  The blocks (B, y > 0) have
// nothing to do.
__global__ __launch_bounds__(kAcceptThreads) void accept_append_kernel(AcceptParams pa, AppendParams pp) {
    extern __shared__ int32_t accept_lds[];
    if (blockIdx.x == (unsigned)pa.B) {
        if (blockIdx.y == 0) accept_scan_block(pa, accept_lds);
        return;
    }
    const int i = blockIdx.x;
    const int acc = block_acceptance(pa, i);
    append_sample_rows(pp, i, acc, blockIdx.y, 0, 1);
}

static hipError_t launch_argmax_partial(const AcceptParams& p, hipStream_t stream) {
    if (p.logits != nullptr && p.T > 0) {
        dim3 grid(p.slices, p.T);
        if (p.logits_dtype == 1)
            hipLaunchKernelGGL(argmax_partial_kernel<BF16>, grid, dim3(kArgmaxThreads), 0, stream, p);
        else if (p.logits_dtype == 2)
            hipLaunchKernelGGL(argmax_partial_kernel<F32>, grid, dim3(kArgmaxThreads), 0, stream, p);
        else
            hipLaunchKernelGGL(argmax_partial_kernel<F16>, grid, dim3(kArgmaxThreads), 0, stream, p);
        return hipGetLastError();
    }
    return hipSuccess;
}

// LDS of the scan block: the small form (accepted counts only) or, when it fits in `limit`
// bytes, the large one (rows_in_lds)
static size_t scan_lds_bytes(AcceptParams& q, size_t limit) {
    const size_t small = sizeof(int32_t) * (size_t)q.B;
    const size_t large = sizeof(int32_t) * ((size_t)2 * q.B + 1 + (size_t)2 * q.T);
    q.rows_in_lds = large <= limit ? 1 : 0;
    return q.rows_in_lds ? large : small;
}

hipError_t launch_greedy_accept(const AcceptParams& p, hipStream_t stream) {
    hipError_t e = launch_argmax_partial(p, stream);
    if (e != hipSuccess) return e;
    AcceptParams q = p;
    const size_t lds = scan_lds_bytes(q, 60 * 1024);      // (a kernel may use 64 KiB of LDS without asking for more)
    hipLaunchKernelGGL(accept_scan_kernel, dim3(1), dim3(kAcceptThreads), lds, stream, q);
    return hipGetLastError();
}

hipError_t launch_accept_append(const AcceptParams& pa, const AppendParams& pp, hipStream_t stream) {
    hipError_t e = launch_argmax_partial(pa, stream);
    if (e != hipSuccess) return e;
    AcceptParams q = pa;
    // every block of the launch gets the scan block's LDS: keep it small when there are many
    // appending blocks, so that it does not limit how many of them a CU holds
    const size_t lds = scan_lds_bytes(q, (int64_t)pp.B * 2 * pp.n_layers > 1024 ? 8 * 1024 : 60 * 1024);
    hipLaunchKernelGGL(accept_append_kernel, dim3(pa.B + 1, 2 * pp.n_layers, 1), dim3(kAcceptThreads), lds, stream, q, pp);
    return hipGetLastError();
}

}  // namespace ems
