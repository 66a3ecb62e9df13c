// Host-visible declarations of the kernel launchers of libems (internal).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ems {

constexpr int kPartialPad = 4;          // floats after the D accumulators: [max, sum, -, -]
constexpr int kMaxLayersPerLaunch = 32;
constexpr int kArgmaxThreads = 256;
constexpr int kAcceptThreads = 1024;

struct AttnParams {
    const char* q;
    const char* k_new;
    const char* v_new;
    const char* k_cache;
    const char* v_cache;
    int64_t row_stride_b;      // bytes
    int64_t head_stride_b;     // bytes
    const int32_t* cu;
    const int32_t* kv_start;
    const int32_t* kv_len;
    const int32_t* parent;     // [T] or nullptr: token trees -- row j of a sample continues row parent[j] < j of
                               // the same sample (-1 for row 0) and sees, among the new rows, itself and its ancestors
    void* out;
    int32_t* ws_header;        // workspace header: the B+1 tile prefix sums, for the merge kernel
    float* ws;                 // 2 * num_waves partial slots of 16 (wide kernel: 32) x (D + kPartialPad) floats
    int out_f32;
    int B, H;
    int num_waves;
    float scale_log2;          // scale * log2(e)
    int write_through;         // also store the new rows' K/V at cache rows kv_len + j (paper order)
    int multi;                 // samples may bring more than 16 rows (up to 64): the wide kernel; 2 = the wave
                               // keeps all 64 rows of a pair (four blocks, two parked in LDS), 1 = pairs of 32 rows
    int wg_fold;               // the matrix-core kernels: partials shared inside a workgroup are merged
                               // in LDS, only a workgroup's first wave (and a pair's first) writes a slot
                               // (set by the host for all but very short walks; ignored by the others)
    // padded ("vanilla") ablation only: every sample has k_max rows and an aligned cache of
    // l_pad rows at row i*cap, with a byte mask [B, cap] of real (1) and padding (0) keys
    const uint8_t* key_mask;
    const int32_t* k_valid;    // [B] real rows among the k_max
    int k_max, l_pad;
    int64_t cap;
};

constexpr int kMaxLdsBytes = 160 * 1024;   // LDS a workgroup may use on gfx950
// LDS at the start of a 16-row attention workgroup: the B+1 tile prefix sums and, for batches of up
// to kIndexStashMaxB samples, a copy of cu_seqlens, kv_len and kv_start (3B+1 words), so that a
// wave's step from one sample to the next reads no global memory.
constexpr int kIndexStashMaxB = 2048;
constexpr size_t attn_prefix_lds_bytes(int B) { return (((size_t)(B + 1) * 4) + 15) & ~(size_t)15; }
// (no_stash: the padded ablation, which has no such arrays, and the vector-ALU formulation, which
// needs the room)
constexpr size_t attn_stash_lds_bytes(int B, bool no_stash) {
    return (no_stash || B > kIndexStashMaxB) ? 0 : ((((size_t)(3 * B + 1) * 4) + 15) & ~(size_t)15);
}
constexpr size_t attn_index_lds_bytes(int B, bool no_stash) { return attn_prefix_lds_bytes(B) + attn_stash_lds_bytes(B, no_stash); }
// LDS bytes per workgroup of the vector-ALU formulation (prefix sums + wave-private state), D in {64, 128}
size_t valu_attention_lds_bytes(int B, int D);

// ev_start / ev_stop (may be null) are recorded right before and right after the main
// attention kernel, i.e. they exclude the partial-merge kernel.
// valu: contractions on the vector ALU instead of the matrix cores (unpadded layout only).
hipError_t launch_verify_attention(const AttnParams& p, int blocks, int D, bool bf16, bool padded,
                                   bool valu, hipStream_t stream, hipEvent_t ev_start,
                                   hipEvent_t ev_stop);

// The same for samples of up to 64 rows (p.multi = 1: pairs of up to 32 rows, two blocks of 16 per
// wave, partial slots of 32 rows; p.multi = 2: pairs of up to 64 rows, partial slots of 64 rows).
// wide_rows64_fits: whether LDS can hold p.multi = 2 at this batch size.
bool wide_rows64_fits(int B, int D);
// The staged kernel (17..64 rows, head dims 80 and 128): tile streams per workgroup, the LDS a
// launch needs (all ones for other head dims), and the launch of its main kernel (p.num_waves
// counts streams there).
constexpr int kStagedStreams = 2;
size_t staged_attention_lds_bytes(int B, int D);
hipError_t launch_verify_attention_staged(const AttnParams& p, int blocks, int D, bool bf16, hipStream_t stream);
hipError_t launch_verify_attention_wide(const AttnParams& p, int blocks, int D, bool bf16,
                                        hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop);

struct ArgmaxPartial {
    float value;
    int32_t index;
};

struct AcceptParams {
    const void* logits;        // [T, V] or nullptr
    int logits_dtype;          // 0 = fp16, 1 = bf16, 2 = fp32
    int V;
    int rows_in_lds;           // set by the launcher: the scan block keeps cu_seqlens and all rows' ids in LDS
    int slices;                // row slices of the first pass (at most 16)
    int slice_len;             // columns per slice (multiple of 8)
    ArgmaxPartial* partial;    // [T, slices]
    int32_t* target_ids;
    const int32_t* input_ids;
    const int32_t* cu;
    int B, T;
    int32_t* accepted;
    int32_t* accepted_cu;
    int32_t* out_tokens;       // may be nullptr
    // token trees (parent != nullptr): acceptance walks from row 0 to the child that carries the
    // target's token; accepted_rows receives the packed row index of every row of the accepted path
    const int32_t* parent;
    int32_t* accepted_rows;    // may be nullptr
};

hipError_t launch_greedy_accept(const AcceptParams& p, hipStream_t stream);

struct AppendLayer {
    const char* k_new;
    const char* v_new;
    char* k_cache;
    char* v_cache;
    int64_t row_stride_b;
    int64_t head_stride_b;
};

struct AppendParams {
    AppendLayer layer[kMaxLayersPerLaunch];
    int n_layers;
    const int32_t* cu;
    const int32_t* accepted;
    // gathered append (rows != nullptr): sample i appends packed rows rows[rows_cu[i] .. rows_cu[i+1])
    // instead of its first accepted[i] rows; cu and accepted are then unused
    const int32_t* rows;
    const int32_t* rows_cu;
    int T;                     // packed rows in k_new / v_new (gathered row indices are checked against it)
    const int32_t* kv_start;
    const int32_t* kv_len;
    int32_t* kv_len_out;       // written by this launch when non-null (must not alias kv_len)
    int B, H;
    int vec_per_head;          // D * 2 / 16
};

struct PaddedAppendParams {
    AppendLayer layer[kMaxLayersPerLaunch];
    int n_layers;
    uint8_t* key_mask;         // [B, cap]
    const int32_t* accepted;
    int B, H;
    int vec_per_head;
    int k_max, l_pad, tau_max;
    int64_t cap;
};

hipError_t launch_kv_append(const AppendParams& p, hipStream_t stream);
// ems_greedy_accept's launches with the append folded into the second one (tree == nullptr,
// pp.rows == nullptr, pp.kv_len_out not aliasing pp.kv_len, pp.accepted unused)
hipError_t launch_accept_append(const AcceptParams& pa, const AppendParams& pp, hipStream_t stream);
hipError_t launch_padded_kv_append(const PaddedAppendParams& p, hipStream_t stream);
// kv_len_out[i] = kv_len[i] + accepted[i], or + (rows_cu[i+1] - rows_cu[i]) when accepted is null
hipError_t launch_advance_kv_len(const int32_t* kv_len, const int32_t* accepted, const int32_t* rows_cu,
                                 int32_t* kv_len_out, int B, hipStream_t stream);

struct PackParams {
    const int32_t* padded_ids;   // [B, k_max]
    const int32_t* token_nums;   // [B]
    int32_t* cu;                 // [B + 1] out
    int32_t* packed_ids;         // [>= sum of counts] out
    int B, k_max;
};
hipError_t launch_pack_tokens(const PackParams& p, hipStream_t stream);

// Read-only streaming probe over `bytes` of device memory (whole 1 KiB lines); sink: one word.
hipError_t launch_stream_read(const void* buf, uint64_t bytes, uint32_t* sink, int blocks, hipStream_t stream);

}  // namespace ems
