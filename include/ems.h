/*
 * ems.h -- C ABI of libems: the unpadded (ragged) verification step of batched
 * speculative decoding on one MI355X (gfx950), after EMS-SD (arXiv 2405.07542).
 *
 * One verification step of a batch of B samples:
 *   1. ems_verify_attention  packed multi-token attention; each sample reads its
 *                            own contiguous KV cache through a per-sample start
 *                            location (Sec. 3.2 "Unpad KV cache") and its own new
 *                            tokens causally; the inputs of all samples are
 *                            concatenated without padding (Sec. 3.2 "Unpad input
 *                            tokens", Appendix D Alg. 1 and Alg. 2)
 *   2. ems_greedy_accept     greedy target tokens and per-sample acceptance length
 *                            (Appendix A), plus the running sum of the lengths
 *   3. ems_kv_append         only the accepted tokens' K/V enter each cache, at the
 *                            sample's own location, which advances by its own
 *                            accepted count (Sec. 3.2, Fig. 2 / Table 1)
 * plus the padded "vanilla" method of Sec. 3.1 as an ablation in the same library, the
 * paper-order variant of steps 1 and 3 (write-through, then advance), the same three steps
 * for token trees (ems_tree_*), ems_pack_tokens (Alg. 1) and two debug validators.  The
 * measurement aids of the same library (kernel timing, read-ceiling probe, the vector-ALU
 * formulation switch, device memory figures) are declared in ems_measure.h.
 *
 * Conventions shared by every entry point
 *   - Pointers named *device* point to GPU memory owned by the caller; pointers
 *     named *host* are ordinary host memory read during the call only.
 *   - The library never allocates or frees device memory and never synchronises
 *     (the two debug validators do wait, as they say).  Work is
 *     enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = the default
 *     stream) and the call returns at once.  Device arrays must stay alive until
 *     that work is done.  A sequence of calls can be captured into a HIP graph; make
 *     the same calls once eagerly first (some kernels raise their LDS limit, a host-side
 *     setting, at their first launch on a device).
 *   - Packed tensors q, k_new, v_new, out are [T, H, D], d fastest, no padding
 *     rows; sample i owns rows cu_seqlens[i] .. cu_seqlens[i+1]-1 (k_i rows).
 *     Row 0 of a sample is its last emitted token (whose K/V is not cached yet),
 *     rows 1.. are its draft tokens: "k predicted tokens" in the paper's words
 *     means k_i = k + 1 rows here.
 *   - 16-bit element types only (ems_dtype) for q/k/v (logits may also be fp32);
 *     device pointers to such tensors must be 16-byte aligned.
 *   - Scalar and pointer arguments are validated on the host before anything is
 *     launched; the contents of device arrays (monotone cu_seqlens, regions that
 *     do not overlap, kv_len[i] + k_i within the region) are the caller's
 *     contract and are NOT checked (ems_validate_inputs does, synchronously).
 *   - Every function returns an ems_status; ems_last_error_string() gives a
 *     thread-local description of the last failure.
 *   - Thread safety: the entry points of this header keep no mutable state between calls
 *     beyond per-device facts cached on first use (compute-unit count, a kernel's LDS limit;
 *     both race-free), so they may be called from several threads at once, each on its own
 *     stream, workspace and outputs.
 */
#ifndef EMS_H
#define EMS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EMS_API __attribute__((visibility("default")))

typedef enum {
    EMS_OK = 0,
    EMS_ERR_INVALID_ARG = 1, /* bad scalar, NULL or misaligned pointer */
    EMS_ERR_UNSUPPORTED = 2, /* legal request outside what the kernels cover */
    EMS_ERR_WORKSPACE = 3,   /* workspace missing or too small */
    EMS_ERR_HIP = 4          /* a HIP runtime call failed */
} ems_status;

typedef enum { EMS_F16 = 0, EMS_BF16 = 1, EMS_F32 = 2 /* attention outputs and logits only */ } ems_dtype;

#define EMS_MAX_QUERY_ROWS 64   /* largest k_i (rows per sample per step) */
#define EMS_ROWS_PER_GROUP 16   /* with max_k up to this, the attention calls use the 16-row kernel; above
                                   it a wider one that holds 32 or all 64 rows of a (sample, head) pair */
#define EMS_MAX_LAYERS_PER_CALL 32

/*
 * Strided view of a KV-cache arena of `rows` token rows shared by all samples.
 * Element (row r, head h, dim d) is at  r*row_stride + h*head_stride + d  (in
 * elements); the D elements of one (row, head) are contiguous.  Covers
 * token-major [R,H,D] (row_stride = H*D, head_stride = D) and head-major
 * [H,R,D] (row_stride = D, head_stride = R*D).  Sample i's cache is the run of
 * rows kv_start[i] .. kv_start[i]+kv_len[i]-1: its start location is its own
 * (Sec. 3.2), so caches of different lengths sit side by side without padding.
 */
typedef struct {
    void* k;             /* device */
    void* v;             /* device */
    int64_t row_stride;  /* elements; multiple of 8 */
    int64_t head_stride; /* elements; multiple of 8 */
    int64_t rows;        /* R */
} ems_kv_cache;

/* Bytes of device workspace the attention calls (ems_verify_attention, its write-through,
 * tree and padded forms) need for these bounds on the current device (split-KV partial
 * results: two slots per wave, one workgroup per compute unit; sized for 256 units when no
 * device is present).  Never 0.  Host-side only: no device memory is touched and nothing is
 * enqueued.  ems_attention_workspace_bytes is the same function under the name that says
 * which call it sizes (ems_greedy_accept has a workspace of its own,
 * ems_accept_workspace_bytes, whose size depends on V, not on these arguments). */
EMS_API size_t ems_workspace_bytes(int B, int T, int H, int D, int max_kv_len);
EMS_API size_t ems_attention_workspace_bytes(int B, int T, int H, int D, int max_kv_len);

/*
 * Packed multi-token attention over per-sample caches (Sec. 3.2; Fig. 3).
 * For sample i, head h, row j < k_i, with L = kv_len[i]:
 *     keys/values n < L   : cache rows kv_start[i] + n
 *     keys/values n >= L  : k_new / v_new rows cu_seqlens[i] + (n - L)
 *     out[cu_seqlens[i]+j, h, :] = softmax_n( scale * <q_j, key_n> , n <= L + j ) . value_n
 * i.e. every cached row plus the sample's own new rows up to and including row j.
 * The cache is only read; k_new/v_new are read from the packed tensors.
 * fp32 accumulation; `out` is rounded once to out_dtype (dtype, or EMS_F32).
 *
 *   q,k_new,v_new,out : device [T,H,D]       cu_seqlens : device int32 [B+1]
 *   kv_start, kv_len  : device int32 [B]     cache      : host struct, device arenas
 *   max_k      >= every k_i   (<= EMS_MAX_QUERY_ROWS).  It also selects the kernel: up to
 *                 EMS_ROWS_PER_GROUP, one that holds 16 rows per (sample, head) and streams
 *                 the sample's cache once per step; up to 32, one that holds 32 rows; up to
 *                 64, one that holds all 64 (half of them parked in LDS) and still streams
 *                 the cache once -- unless the batch is so large (B above ~5000 at D = 128)
 *                 that LDS has no room for that, in which case rows 0..31 and 32..63 of a
 *                 sample stream the cache once each.  A sample with more rows than max_k
 *                 breaks the contract (rows beyond 16, resp. 64, are left unwritten).
 *   max_kv_len >= every kv_len[i]            (host-known upper bounds)
 * Samples with k_i = 0 contribute nothing; kv_len[i] = 0 is legal; T = 0 is a no-op.
 * Errors: B<1, T<0, H<1, max_k<0, max_kv_len<0, NULL/misaligned pointer,
 * non-finite scale -> INVALID_ARG; D not in {64,80,128}, max_k > 64, B > 8192
 * -> UNSUPPORTED (the padded ablation and EMS_ATTN_VALU: D in {64,128} and max_k <= 16
 * only); workspace -> WORKSPACE; launch failure -> HIP.
 */
EMS_API ems_status ems_verify_attention(
    const void* q, const void* k_new, const void* v_new,
    const ems_kv_cache* cache,
    const int32_t* cu_seqlens, const int32_t* kv_start, const int32_t* kv_len,
    void* out, ems_dtype out_dtype,
    int B, int T, int H, int D, int max_k, int max_kv_len,
    float scale, ems_dtype dtype,
    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Paper-order variant of the step (Sec. 3.2, "Unpad KV cache": the K/V of every input token
 * is written at its sample's own position before attention runs; after verification the
 * sample's location advances by its accepted count).
 * ems_verify_attention_write_through computes exactly what ems_verify_attention computes and
 * ALSO stores all k_i new rows' K/V into the cache at rows kv_start[i]+kv_len[i]+j, j < k_i
 * (those rows must lie inside the sample's region and outside every other sample's).
 * ems_kv_advance then replaces ems_kv_append: kv_len_out[i] = kv_len[i] + accepted[i]
 * (kv_len_out may alias kv_len).  Rows at or beyond the new length hold the rejected
 * drafts' K/V and are don't-care: the next step overwrites them.  The result on rows
 * [0, kv_len+accepted) is bit-identical to verify + append.
 */
EMS_API ems_status ems_verify_attention_write_through(
    const void* q, const void* k_new, const void* v_new,
    const ems_kv_cache* cache,
    const int32_t* cu_seqlens, const int32_t* kv_start, const int32_t* kv_len,
    void* out, ems_dtype out_dtype,
    int B, int T, int H, int D, int max_k, int max_kv_len,
    float scale, ems_dtype dtype,
    void* workspace, size_t workspace_bytes, void* hip_stream);
EMS_API ems_status ems_kv_advance(
    const int32_t* kv_len, const int32_t* accepted, int32_t* kv_len_out, int B, void* hip_stream);

/*
 * ems_verify_attention for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * errors as ems_verify_attention, minus the workspace: the split-KV partials go to a buffer
 * of EMS_NOALLOC_SCRATCH_BYTES that is part of the library's own device image (each GPU the
 * library runs on holds its copy from the first call on that GPU until the process ends).
 * The call allocates and frees nothing.
 *   Limits: max_k <= EMS_ROWS_PER_GROUP (the 16-row kernel) and a launch whose partials fit
 *   the buffer (any B <= 8192 at D <= 128 on a GPU of up to 256 compute units); beyond
 *   either -> EMS_ERR_UNSUPPORTED with the sizes in the message.
 *   Every call on a GPU shares that GPU's buffer: calls that overlap in time on one GPU
 *   (two streams, two threads) race on it and give wrong results; calls ordered on one stream
 *   or otherwise serialised are safe, and a call needs nothing from the call before it (the
 *   buffer holds no state that must be cleared).
 */
#define EMS_NOALLOC_SCRATCH_BYTES (18u << 20)
EMS_API ems_status ems_verify_attention_noalloc(
    const void* q, const void* k_new, const void* v_new,
    const ems_kv_cache* cache,
    const int32_t* cu_seqlens, const int32_t* kv_start, const int32_t* kv_len,
    void* out, ems_dtype out_dtype,
    int B, int T, int H, int D, int max_k, int max_kv_len,
    float scale, ems_dtype dtype, void* hip_stream);

/*
 * "Unpad input tokens" (Appendix D, Alg. 1): concatenate the input tokens of all samples and
 * keep each sample's count.  The per-sample lists are given as a padded array:
 *   padded_ids  device int32 [B, k_max]: sample i's tokens in its first token_nums[i] slots
 *   token_nums  device int32 [B]: tokens of each sample (values outside [0, k_max] are clamped)
 *   cu_seqlens  device int32 [B+1] out: running sum of the counts, cu_seqlens[B] = total T
 *   packed_ids  device int32 [capacity] out: sample after sample, no padding; the caller sizes
 *               it for the largest possible total (B * k_max always suffices)
 * Errors: B < 1 or B > 8192, k_max < 0, NULL pointer -> INVALID_ARG / UNSUPPORTED.
 * The total is known on the device only; the other calls take T from the host, so a caller
 * that does not know it reads cu_seqlens[B] back or passes capacity-sized tensors.
 */
EMS_API ems_status ems_pack_tokens(
    const int32_t* padded_ids, const int32_t* token_nums, int B, int k_max,
    int32_t* cu_seqlens, int32_t* packed_ids, void* hip_stream);

/* Bytes of device workspace ems_greedy_accept needs for up to T rows (0 when logits ==
 * NULL is intended, i.e. V == 0); the figure for T also covers every smaller T. */
EMS_API size_t ems_accept_workspace_bytes(int T, int V);

/*
 * Greedy acceptance (Appendix A: greedy token = arg-max of the target's
 * distribution; acceptance length = 1 + number of leading drafts that equal the
 * target's token for the row before them; Sec. 3.1: between 1 and k+1 tokens).
 *
 *   logits      device [T,V] of `dtype` (EMS_F16, EMS_BF16 or EMS_F32), or NULL.  When
 *               given, target_ids[r] is WRITTEN with the lowest index attaining the row
 *               maximum (+0 and -0 are equal; inputs must not hold NaN).  When NULL,
 *               target_ids is READ.
 *   input_ids   device int32 [T]: packed input tokens (row 0 of a sample = last
 *               emitted token, rows 1.. = drafts)
 *   accepted    device int32 [B] out: m_i + 1 where m_i = number of leading j in
 *               [0, k_i-2] with target_ids[cu+j] == input_ids[cu+j+1]; 0 if k_i = 0
 *   accepted_cu device int32 [B+1] out: exclusive running sum, [B] = total
 *   out_tokens  device int32 [T] or NULL: the accepted target tokens packed sample
 *               after sample; the first accepted_cu[B] entries are written
 * Errors: B<1 or B>8192, T<0, V<0, NULL required pointer -> INVALID_ARG /
 * UNSUPPORTED; workspace too small (only with logits) -> WORKSPACE.
 */
EMS_API ems_status ems_greedy_accept(
    const void* logits, ems_dtype dtype, int V,
    int32_t* target_ids, const int32_t* input_ids,
    const int32_t* cu_seqlens, int B, int T,
    int32_t* accepted, int32_t* accepted_cu, int32_t* out_tokens,
    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * KV-cache append (Sec. 3.2 "Unpad KV cache"): for every layer, sample i and
 * j < accepted[i]:  cache row kv_start[i]+kv_len[i]+j  <-  new row cu_seqlens[i]+j
 * (K and V, bit copies).  Then kv_len_out[i] = kv_len[i] + accepted[i]: the
 * sample's write location advances by its own accepted count.  No other byte of
 * any arena is written, so every cache stays contiguous and free of padding.
 *
 *   k_new_layers, v_new_layers : host arrays [n_layers] of device [T,H,D] pointers
 *   caches                     : host array [n_layers]
 *   kv_len_out                 : device int32 [B], may alias kv_len, NULL to skip
 * Errors: n_layers<1, B<1, T<0, H<1, D<8 or D%8 != 0, NULL/misaligned -> INVALID_ARG.
 * More than EMS_MAX_LAYERS_PER_CALL layers are processed in several launches.
 */
EMS_API ems_status ems_kv_append(
    const void* const* k_new_layers, const void* const* v_new_layers,
    const ems_kv_cache* caches, int n_layers,
    const int32_t* cu_seqlens, const int32_t* accepted,
    const int32_t* kv_start, const int32_t* kv_len, int32_t* kv_len_out,
    int B, int T, int H, int D, ems_dtype dtype, void* hip_stream);

/*
 * ems_greedy_accept and then ems_kv_append of the counts it found (Appendix A, then Sec. 3.2
 * "Unpad KV cache"), as one call: the arguments are those of the two calls, in their order
 * (logits_dtype describes the logits, dtype the K/V tensors), every output is what the two calls
 * give, bit for bit, and no other byte is written.  Why it exists: the step around the
 * attention call is launch-bound, and here the kernel that finds the counts also copies the
 * rows (each copying workgroup derives its sample's count itself), one launch less.  Where one
 * launch cannot do both -- kv_len_out aliasing kv_len, more than EMS_MAX_LAYERS_PER_CALL layers,
 * T == 0 -- the two calls simply run one after the other.
 * Errors: those of ems_greedy_accept and ems_kv_append; nothing is enqueued when one is
 * returned.
 */
EMS_API ems_status ems_greedy_accept_append(
    const void* logits, ems_dtype logits_dtype, int V,
    int32_t* target_ids, const int32_t* input_ids,
    const int32_t* cu_seqlens, int B, int T,
    int32_t* accepted, int32_t* accepted_cu, int32_t* out_tokens,
    void* workspace, size_t workspace_bytes,
    const void* const* k_new_layers, const void* const* v_new_layers,
    const ems_kv_cache* caches, int n_layers,
    const int32_t* kv_start, const int32_t* kv_len, int32_t* kv_len_out,
    int H, int D, ems_dtype dtype, void* hip_stream);

/*
 * Ablation: the padded "vanilla" method of Sec. 3.1, same kernels, same library.
 * Inputs are padded to k_max rows per sample ([B, k_max, H, D]; rows j >= k_valid[i] are
 * padding); the caches are aligned: sample i owns arena rows i*cap .. i*cap + l_pad - 1,
 * of which key_mask[i*cap + n] = 0 marks padding keys (they are read and masked, which is
 * the vanilla method's extra memory traffic).  Real rows give the same result as
 * ems_verify_attention on the unpadded data; padding rows are computed like the real ones
 * and hold don't-care values.  Every sample needs k_valid[i] >= 1.
 *   key_mask : device uint8 [B, cap], 4-byte aligned; cap a multiple of 32, >= l_pad
 *   workspace: ems_attention_workspace_bytes(B, B*k_max, H, D, l_pad)
 * ems_padded_kv_append writes tau_max (host value, <= k_max) rows for EVERY sample at the
 * aligned row l_pad -- its accepted rows, then padding rows -- and sets key_mask there to
 * (j < accepted[i]); the caller's aligned length becomes l_pad + tau_max.
 */
EMS_API ems_status ems_padded_verify_attention(
    const void* q_pad, const void* k_new_pad, const void* v_new_pad,
    const ems_kv_cache* cache, int64_t cap, const uint8_t* key_mask, const int32_t* k_valid,
    void* out_pad, ems_dtype out_dtype,
    int B, int k_max, int l_pad, int H, int D, float scale, ems_dtype dtype,
    void* workspace, size_t workspace_bytes, void* hip_stream);
EMS_API ems_status ems_padded_kv_append(
    const void* const* k_new_pad_layers, const void* const* v_new_pad_layers,
    const ems_kv_cache* caches, int n_layers, int64_t cap, uint8_t* key_mask,
    const int32_t* accepted, int B, int k_max, int l_pad, int tau_max,
    int H, int D, ems_dtype dtype, void* hip_stream);

/*
 * Debug aid: copies the index arrays to the host (synchronises the stream) and
 * checks the contract the other calls assume: cu_seqlens[0]=0, non-decreasing,
 * cu_seqlens[B]=T, k_i <= max_k, 0 <= kv_len[i] <= max_kv_len, kv_start[i] >= 0,
 * kv_start[i]+kv_len[i]+k_i <= rows, and regions [kv_start, kv_start+kv_len+k_i)
 * of different samples do not overlap.  Returns INVALID_ARG with a message naming
 * the first violation.
 */
EMS_API ems_status ems_validate_inputs(
    const int32_t* cu_seqlens, const int32_t* kv_start, const int32_t* kv_len,
    int B, int T, int max_k, int max_kv_len, int64_t rows, void* hip_stream);

/*
 * Tree-structured verification.  The paper names tree decoding as the next thing to combine
 * with the multi-sample method (Limitations, item 4; Sec. 2 "Dynamic Tree decoding") and
 * gives no algorithm; these three calls are the usual definition, per sample, on the same
 * packed / per-sample-cache layout.
 *
 *   parent   device int32 [T]: the k_i new rows of sample i form a token tree; row 0 (the
 *            last emitted token) is the root, parent[cu_seqlens[i]] = -1, and row j > 0
 *            continues row parent[cu_seqlens[i]+j] of the same sample, 0 <= parent < j.
 *            A chain (parent = j-1) is ordinary speculative decoding.  An entry outside
 *            [0, j) is treated as "no parent" by the attention call and matches no row in
 *            the accept call; k_i <= EMS_MAX_QUERY_ROWS as everywhere.
 *
 * ems_tree_verify_attention: as ems_verify_attention (same arguments, workspace and errors),
 *   except that among the new rows row j sees itself and its ancestors only (every cached row
 *   is still visible).  Not available with EMS_ATTN_VALU (UNSUPPORTED).
 * ems_tree_accept: as ems_greedy_accept (same arguments, workspace and errors), except that
 *   acceptance walks the tree: from row 0, step to the lowest-indexed child of the current row
 *   whose input token equals the target's token after the current row; stop when no child
 *   matches.  accepted[i] = rows on that path (>= 1; 0 if k_i = 0); out_tokens = the target's
 *   tokens after the rows of the path; accepted_rows (device int32 [T] or NULL) = the packed
 *   row index of every row of the path, both packed sample after sample at accepted_cu.
 * ems_kv_append_rows: as ems_kv_append, for rows that are not a prefix: cache row
 *   kv_start[i]+kv_len[i]+j receives packed row accepted_rows[accepted_cu[i]+j] of every layer,
 *   j < accepted_cu[i+1]-accepted_cu[i]; kv_len_out[i] = kv_len[i] + that count (may alias
 *   kv_len, may be NULL).  An index outside [0, T) copies nothing.
 */
/* Debug validator for a parent array (synchronises hip_stream, copies both arrays to the host):
 * INVALID_ARG naming the first row whose parent is not -1 (row 0) or in [0, j) (row j). */
EMS_API ems_status ems_validate_tree(
    const int32_t* cu_seqlens, const int32_t* parent, int B, int T, void* hip_stream);
EMS_API ems_status ems_tree_verify_attention(
    const void* q, const void* k_new, const void* v_new,
    const ems_kv_cache* cache,
    const int32_t* cu_seqlens, const int32_t* parent,
    const int32_t* kv_start, const int32_t* kv_len,
    void* out, ems_dtype out_dtype,
    int B, int T, int H, int D, int max_k, int max_kv_len,
    float scale, ems_dtype dtype,
    void* workspace, size_t workspace_bytes, void* hip_stream);
EMS_API ems_status ems_tree_accept(
    const void* logits, ems_dtype dtype, int V,
    int32_t* target_ids, const int32_t* input_ids, const int32_t* parent,
    const int32_t* cu_seqlens, int B, int T,
    int32_t* accepted, int32_t* accepted_cu, int32_t* out_tokens, int32_t* accepted_rows,
    void* workspace, size_t workspace_bytes, void* hip_stream);
EMS_API ems_status ems_kv_append_rows(
    const void* const* k_new_layers, const void* const* v_new_layers,
    const ems_kv_cache* caches, int n_layers,
    const int32_t* accepted_rows, const int32_t* accepted_cu,
    const int32_t* kv_start, const int32_t* kv_len, int32_t* kv_len_out,
    int B, int T, int H, int D, ems_dtype dtype, void* hip_stream);

/* Thread-local text for the last non-OK status returned on this thread. */
EMS_API const char* ems_last_error_string(void);

/* Library version, "major.minor". */
EMS_API const char* ems_version(void);

#ifdef __cplusplus
}
#endif
#endif /* EMS_H */
